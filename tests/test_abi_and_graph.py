"""CPU-side checks: the C-ABI library loads and exports what include/fleet.h declares,
the accounting closed forms reproduce the paper's printed tables, and the host task-graph
builder equals an independent re-derivation written here (plain integers, bit-exact)."""
import json
import os
import re

import numpy as np
import pytest

import paper_2604_15379_amd as F
import synth_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
GOLD = json.load(open(os.path.join(ROOT, "tests", "golden", "paper_tables.json")))


# ------------------------------------------------------------------ ABI
def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "fleet.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fleet_[a-z0-9_]+)\s*\(", hdr))
    assert declared == set(F.EXPORTS), declared ^ set(F.EXPORTS)
    lib = F.load_library()
    for name in declared:
        assert getattr(lib, name) is not None
    assert F.fleet_strerror(0) == "ok" and "timed out" in F.fleet_strerror(-4)


def test_graph_build_rejects_bad_shapes():
    sh = si.reduced_shape().asdict()
    for bad in ({"head_dim": 64}, {"hidden": 1000}, {"n_q_heads": 7}, {"max_batch": 129},
                {"vocab": 1001}, {"n_layers": 0}):
        with pytest.raises(F.FleetError):
            F.fleet_graph_build({**sh, **bad}, 1)
    with pytest.raises(F.FleetError):
        F.fleet_graph_build(sh, 2)           # batch above max_batch
    with pytest.raises(F.FleetError):
        F.fleet_graph_build(sh, 1, tile_m=24)


def test_shapes_beyond_32bit_offsets_are_rejected():
    """The kernels address a weight matrix and one (sequence, kv head) stream of the cache with
    32-bit byte offsets: a matrix of 2 GiB or more, or max_seq * 256 >= 2^31, is refused."""
    q = si.qwen3_8b_shape(1, 1025, n_layers=1).asdict()
    F.fleet_graph_build(q, 1)                                     # the real shape passes
    for bad in ({"vocab": 262144},                                # 262144 * 4096 * 2 = 2^31
                {"ffn": 131072},                                  # gate|up: 2 * 131072 * 4096 * 2 = 2^31
                {"max_seq": 1 << 23},                             # 2^23 * 256 = 2^31
                {"max_batch": 128, "n_kv_heads": 16}):            # more (sequence, kv head) pairs than counters
        with pytest.raises(F.FleetError):
            F.fleet_graph_build({**q, **bad}, 1)
    F.fleet_graph_build({**q, "vocab": 262144 - 16}, 1)
    F.fleet_graph_build({**q, "max_batch": 128}, 128)


def test_closed_forms_survive_zero_divisors():
    """Nothing in the ABI ends the process: a zero divisor gives -1 (0.0 for the hit model), and
    tile_m = 0 means the whole-batch tile as it does in the shape."""
    assert F.fleet_weight_bytes_per_xcd(4096, 4096, 0) == -1
    assert F.fleet_l2_window_bytes(4096, 0, 64, 256) == -1
    assert F.fleet_l2_window_bytes(4096, 8, 0, 256) == -1
    assert F.fleet_l2_hit_model(64, 16, 0) == 0.0
    assert F.fleet_l2_hit_model(0, 16, 32) == 0.0
    assert F.fleet_l2_hit_model(64, 0, 32) == 0.0                 # one 64-row tile: nothing to share
    assert F.fleet_l2_hit_model(128, 0, 32) == pytest.approx(0.5)  # two 64-row tiles
    assert F.fleet_effective_intensity(8, 1.0) == 0.0


def test_fma_switch_follows_the_environment_of_the_builder(monkeypatch):
    """FLEET_FMA_MAX_BATCH is read once per owner of a graph set (here: per fleet_graph_build
    call) and handed to the builder; FLEET_FLAG_PACKED_ONLY forces the MFMA path for every batch."""
    sh = si.reduced_shape(max_batch=8).asdict()
    path = lambda b, flags=0: F.parse_graph(F.fleet_graph_build(sh, b, flags=flags))["header"]["path"]
    assert [path(b) for b in (1, 2, 3, 8)] == [0, 1, 1, 1]
    monkeypatch.setenv("FLEET_FMA_MAX_BATCH", "8")
    assert [path(b) for b in (1, 2, 3, 8)] == [0, 0, 0, 0]
    assert [path(b, F.FLAG_PACKED_ONLY) for b in (1, 8)] == [1, 1]
    monkeypatch.setenv("FLEET_FMA_MAX_BATCH", "0")
    assert [path(b) for b in (1, 2)] == [1, 1]


def test_marks_let_a_step_end_before_the_lm_head():
    """Per XCD the queue marks are: ingest, every layer, final stage, LM head, end; the slice
    between the last two holds exactly the LM-head tasks (a step without logits stops there)."""
    sh = si.reduced_shape(max_batch=4, n_layers=3, vocab=512)
    g = F.parse_graph(F.fleet_graph_build(sh.asdict(), 4))
    assert g["marks"].shape == (8, 3 + 4)
    lm_op = [i for i, o in enumerate(g["ops"]) if o[13] == WK["LM"]][0]
    for x in range(8):
        q = g["qents"][g["qoff"][x]:g["qoff"][x + 1]]
        tail = q[g["marks"][x, -2]:g["marks"][x, -1]]
        assert len(tail) >= 1 and all(g["tasks"][e[0], 0] == lm_op for e in tail)
        assert all(g["tasks"][e[0], 0] != lm_op for e in q[:g["marks"][x, -2]])


# ------------------------------------------------------------------ paper tables
def test_weight_size_table():
    t = GOLD["weight_sizes"]
    tile = t["tile"]
    tot = tot_x = 0
    for r in t["rows"]:
        assert F.fleet_weight_bytes(r["K"], r["N"]) == r["weight_MiB"] << 20
        assert F.fleet_weight_bytes_per_xcd(r["K"], r["N"], 8) == r["per_xcd_MiB"] << 20
        assert F.fleet_l2_window_bytes(r["N"], 8, tile["T_N"], tile["T_K"]) == r["l2_window_KiB"] << 10
        tot += F.fleet_weight_bytes(r["K"], r["N"])
        tot_x += F.fleet_weight_bytes_per_xcd(r["K"], r["N"], 8)
    assert tot == t["all_per_layer_MiB"] << 20 and tot_x == t["all_per_xcd_MiB"] << 20


def test_l2_hit_model_and_effective_intensity():
    m = GOLD["l2_hit_model"]
    for c in m["cases"]:
        assert F.fleet_l2_hit_model(c["batch"], m["T_M"], 32) == pytest.approx(c["hit"])
    assert F.fleet_l2_hit_model(64, 16, 2) == pytest.approx(0.5)      # R capped by the workers
    for c in GOLD["effective_intensity"]["cases"]:
        assert F.fleet_effective_intensity(c["batch"], c["hit_percent"] / 100) == \
            pytest.approx(c["ai_eff"], rel=5e-3)


def test_step_bytes_accounting():
    sh = si.qwen3_8b_shape(1, 1025).asdict()
    per_layer = 368 << 20
    lm = 151936 * 4096 * 2
    kv = 36 * 2 * 8 * 128 * 2 * 1025
    assert F.fleet_step_bytes(sh, 1, [1024]) == 36 * per_layer + lm + kv
    sh64 = si.qwen3_8b_shape(64, 4097).asdict()
    assert F.fleet_step_bytes(sh64, 64, [4096] * 64) == 36 * per_layer + lm + 64 * 36 * 4096 * 4097


# ------------------------------------------------------------------ graph re-derivation
BUF = dict(NONE=0, X=1, N=2, QKV=3, ATT=4, H=5, PART=6, HIDDEN_IN=7, TOKENS=8, KC=9, VC=10, POS=11,
           HIDDEN_OUT=12, LOGITS=13, GEMM_X=14, GEMM_Y=15, GPART=16, GU32=17, TOKENS_OUT=18, PT=19, SS=20)
WK = dict(NONE=0, QKV=1, O=2, GU=3, DOWN=4, LM=5, LN1=6, LN2=7, FINAL=8, EMBED=9)
INGEST, RMSNORM, GEMM, ATTN, SWIGLU, FINAL = 0, 1, 2, 3, 4, 5
LDS_X_BYTES = 96 * 1024      # activations the FMA path may keep in LDS


FMA_MAX = 1   # largest batch on the FMA GEMV path (FLEET_FMA_MAX_BATCH unset)


def expected_graph(sh: si.Shape, batch, n_xcd, n_workers, sched, tile_m, flags=0):
    """Independent derivation of the serialized graph (same word layout)."""
    H, hd, nq, nkv, Fd = sh.hidden, sh.head_dim, sh.n_q_heads, sh.n_kv_heads, sh.ffn
    fma = batch <= FMA_MAX
    ur = 8 if fma else 16
    tm = batch if fma else (tile_m or min(64, -(-batch // 16) * 16))
    mt = -(-batch // tm)
    S = 1
    while S * 2 <= 32 and batch * nkv * S * 2 <= n_workers and S * 2 * 100 <= sh.max_seq:
        S *= 2
    ops, tasks, events, queues, marks, xready = [], [], [], [[] for _ in range(n_xcd)], [], []
    stage = [0]

    def op(body, layer, epi, path, K, N, unit_rows, n_units, m_tiles, tile, inb, outb, aux, wk, aux2=0):
        ops.append([body, layer, epi, path, K, N, unit_rows, n_units, m_tiles, tile, inb, outb, aux, wk,
                    batch, aux2])
        return len(ops) - 1

    def task(o, scope, xcd, a, wait, sig):
        tasks.append([o, scope, xcd, *a, wait, sig, stage[0]] + [0] * 6)
        return len(tasks) - 1

    def cu_stage(o, items, wait, min_per_xcd=1, from_top=False):
        ev = len(events)
        if sched == 1 or len(items) <= min_per_xcd * n_xcd:   # tasks run anywhere, or few per XCD: every
            events.append([len(items), 0, 0, len(items)])   # task signals the device counter
        else:               # grouped per XCD: one device-level signal per XCD with tasks (kind 2)
            owners = sorted({key % n_xcd for key, a in items})
            events.append([len(owners), 2, sum(1 << x for x in owners), len(items)])
        if sched == 1:
            first = len(tasks)
            for key, a in items:
                task(o, 1, -1, a, wait, ev)
            for x in range(n_xcd):
                queues[x].append([first, len(items), 2, stage[0]])
        else:
            for x in range(n_xcd):
                mine = [a for key, a in items if key % n_xcd == x]
                if mine:
                    queues[x].append([len(tasks), len(mine), 3 if from_top else 1, stage[0]])   # 3: dealt from the highest rank down
                    for a in mine:
                        task(o, 1, x, a, wait, ev)
        stage[0] += 1
        return ev

    def msplit(m_tiles):
        """M-split applies on the MFMA path when the m-tiles (>= 2) divide the XCD count."""
        return sched == 2 and not fma and m_tiles >= 2 and n_xcd % m_tiles == 0

    def plan(U, K, nb):
        """MFMA tile plan: units per tile G and k-slices KS keeping one XCD's workers equally
        busy with tall tiles (a tile of G units is charged G + 2); ties go to more units per
        tile, then to fewer slices.  Packed into aux2."""
        if fma:
            return 0
        blocks = 1 if tm <= 16 else 2 if tm <= 32 else 4
        gmax = max(1, (6 if blocks >= 4 or nb == 2 else 8) // nb)
        split_ok = not (flags & 32) and U * mt <= 4096
        wpx = max(1, n_workers // n_xcd)
        # small weight shares stay in registers whole (bit 21): one m-tile, not gate|up, K up to
        # 4096, at most 2 units per worker; G = units per worker, one k-slice
        g_res = -(-(-(-U // n_xcd)) // wpx)
        if not (flags & 128) and nb == 1 and mt == 1 and K <= 4096 and g_res <= 2:
            return g_res << 12 | 1 << 16 | 1 << 21
        if msplit(mt):      # n_xcd / mt XCDs share one m-tile and split the units
            xpm = n_xcd // mt
            ux, tiles_m = -(-U // xpm), 1
        else:
            ux, tiles_m = -(-U // n_xcd), mt
        # cost of the busiest worker, in ns: a tile streams at the rate its bytes in flight allow
        # (depth - 1 rounds of G * nb blocks of 8 KB over 3.8 us, 2.5 us where m-tiles share the
        # weights), capped per CU (30 / 45 KB/us) and by the XCD's share of the memory (700 KB/us);
        # 0.1 us per round and 16-row block; 1 us per tile, 3 us + 0.2 us per slice per split-K tile
        depth = 3 if blocks >= 4 or (blocks == 2 and nb == 1) else 4
        shared = tiles_m > 1
        best = None
        for G in range(1, min(gmax, max(1, ux)) + 1):
            for KS in (1, 2, 4, 8):
                if KS > 1 and (not split_ok or K % (KS * 256)):
                    continue
                tiles = -(-ux // G) * KS * tiles_m
                kc = K // KS
                rate = (depth - 1) * G * nb * 8 * 1000 // 2500
                rate = max(1, min(rate, 45 if shared else 30, 700 * min(tiles_m, wpx) // min(tiles, wpx)))
                tile_ns = G * nb * kc // 32 * 1000 // rate + -(-kc // 256) * blocks * 100 + (3000 + 400 * KS if KS > 1 else 1000)
                cost = -(-tiles // wpx) * tile_ns
                if tiles % wpx:
                    cost += cost // 10      # idle or unequally loaded workers
                if best is None or (cost, -G, KS) < best[0]:
                    best = ((cost, -G, KS), G, KS)
        return best[1] << 12 | best[2] << 16

    def gemm_stage(o, wait, skip=None):
        U, m_tiles = ops[o][7], ops[o][8]
        ev = len(events)
        if sched == 1:
            cu = max(1, U // n_workers) if fma else max(1, ops[o][15] >> 12 & 15)
            ksn = 1 if fma else max(1, ops[o][15] >> 16 & 15)
            ng = -(-U // cu)
            events.append([ng * m_tiles * ksn, 0, 0, ng * m_tiles * ksn])
            first = len(tasks)
            for m in range(m_tiles):
                for ks in range(ksn):
                    for g in range(ng):
                        task(o, 1, -1, [g * cu, min(cu, U - g * cu), m, ks], wait, ev)
            for x in range(n_xcd):
                queues[x].append([first, ng * m_tiles * ksn, 2, stage[0]])
        elif msplit(m_tiles):
            xpm = n_xcd // m_tiles
            bounds = [U * part // xpm for part in range(xpm + 1)]
            owners = [x for x in range(n_xcd) if bounds[x % xpm + 1] > bounds[x % xpm]]
            events.append([len(owners), 1, sum(1 << x for x in owners), len(owners)])
            for x in owners:
                part = x % xpm
                t = task(o, 2, x, [bounds[part], bounds[part + 1] - bounds[part], 0, x // xpm + 1], wait, ev)
                queues[x].append([t, 1, 0, stage[0]])
        else:
            bounds = [U * x // n_xcd for x in range(n_xcd + 1)]
            owners = [x for x in range(n_xcd) if bounds[x + 1] > bounds[x]]
            events.append([len(owners), 1, sum(1 << x for x in owners), len(owners)])
            for x in owners:
                t = task(o, 2, x, [bounds[x], bounds[x + 1] - bounds[x], skip[x] if skip else 0, 0], wait, ev)
                queues[x].append([t, 1, 0, stage[0]])
        stage[0] += 1
        return ev

    def mark():
        marks.append([len(q) for q in queues])

    rows = [(b, [b, 0, 0, 0]) for b in range(batch)]
    path = 0 if fma else 1
    NQKV, QD = (nq + 2 * nkv) * hd, nq * hd
    mark()
    ev = cu_stage(op(INGEST, -1, 0, 0, H, H, 0, 0, 1, batch, BUF["HIDDEN_IN"], BUF["X"], 0, WK["EMBED"]), rows, -1)
    xready.append(ev)
    # FMA path: RMSNorm fused into the consuming GEMV (activation mode 2, gain kind in the
    # low byte of aux2); activations that fit LDS are copied there (mode 1), else mode 0
    fuse = fma and not (flags & 4) and batch * H * 2 <= LDS_X_BYTES
    # MFMA path, tiles of 16 rows: fused too (bit 22 of aux2; the GEMM reads the fp32 residual
    # rows); taller tiles keep the norm stages
    fuse_mfma = (not fma) and not (flags & 4) and tm <= 16 and H % 64 == 0 and H <= 32768
    FUSED = 1 << 22

    PRE = 3 << 10     # weight blocks the FMA path requests before its wait (bits 10..11)

    def xm(K):
        return ((1 if fma and batch * K * 2 <= LDS_X_BYTES else 0) << 8) | PRE

    # FMA path, cooperative: the ranks that run an XCD's attention tasks take no O-projection
    # units when they are at most half of the XCD's workers
    o_skip = [0] * n_xcd
    if sched != 1:
        for x in range(n_xcd):
            n_att = S * sum(1 for p in range(batch * nkv) if p % n_xcd == x)
            o_skip[x] = n_att if 2 * n_att <= n_workers // n_xcd else 0

    for l in range(sh.n_layers):
        mark()
        if fuse:
            o_qkv = op(GEMM, l, 0, path, H, NQKV, ur, NQKV // ur, mt, tm, BUF["X"], BUF["QKV"], 0, WK["QKV"],
                       WK["LN1"] | 2 << 8 | PRE)
        elif fuse_mfma:
            o_qkv = op(GEMM, l, 0, path, H, NQKV, ur, NQKV // ur, mt, tm, BUF["X"], BUF["QKV"], 0, WK["QKV"],
                       WK["LN1"] | PRE | FUSED | plan(NQKV // ur, H, 1))
        else:
            ev = cu_stage(op(RMSNORM, l, 0, 0, H, H, 0, 0, 1, batch, BUF["X"], BUF["N"], 0, WK["LN1"]), rows, ev, 1,
                          batch <= 4 * n_xcd)     # few norm tasks per XCD: on its highest ranks
            o_qkv = op(GEMM, l, 0, path, H, NQKV, ur, NQKV // ur, mt, tm, BUF["N"], BUF["QKV"], 0, WK["QKV"],
                       xm(H) | plan(NQKV // ur, H, 1))
        # FMA path: attention workers (at most a quarter of every XCD's workers) sit out QKV too
        qkv_skip = fma and sched != 1 and all(0 < k and 4 * k <= n_workers // n_xcd for k in o_skip)
        ev = gemm_stage(o_qkv, ev, o_skip if qkv_skip else None)
        att_items = [(p, [p // nkv, p % nkv, s, S]) for p in range(batch * nkv) for s in range(S)]
        ev = cu_stage(op(ATTN, l, 0, 0, hd, QD, 0, 0, 1, batch, BUF["QKV"], BUF["ATT"], S, WK["NONE"]), att_items, ev, 32)
        # FMA path, cooperative: the O projection carries the gate/up matrix as second pointer
        # (low byte of aux2) and its gate rows (aux): idle workers warm the L2 with it
        # -- only where attention keeps at most a quarter of every XCD's workers busy
        warm = fma and sched != 1 and all(0 < k and 4 * k <= n_workers // n_xcd for k in o_skip)
        ev = gemm_stage(op(GEMM, l, 1, path, QD, H, ur, H // ur, mt, tm, BUF["ATT"], BUF["X"], Fd if warm else 0,
                           WK["O"], (WK["GU"] if warm else 0) | xm(QD) | plan(H // ur, QD, 1)), ev,
                        o_skip if fma else None)
        # flag 256 (unfused SiLU): a plain GEMM over all 2 * ffn rows stores fp32 sums and a stage
        # of CU-tasks, one per sequence, applies SiLU(gate) x up
        unfused = bool(flags & 256)
        epi, gn, gaux, gnb = (0, 2 * Fd, 0, 1) if unfused else (2, Fd, Fd, 2)
        gout = BUF["GU32"] if unfused else BUF["H"]
        if fuse:
            o_gu = op(GEMM, l, epi, path, H, gn, ur, gn // ur, mt, tm, BUF["X"], gout, gaux, WK["GU"],
                      WK["LN2"] | 2 << 8 | PRE)
        elif fuse_mfma:
            o_gu = op(GEMM, l, epi, path, H, gn, ur, gn // ur, mt, tm, BUF["X"], gout, gaux, WK["GU"],
                      WK["LN2"] | PRE | FUSED | plan(gn // ur, H, gnb))
        else:
            ev = cu_stage(op(RMSNORM, l, 0, 0, H, H, 0, 0, 1, batch, BUF["X"], BUF["N"], 0, WK["LN2"]), rows, ev)
            o_gu = op(GEMM, l, epi, path, H, gn, ur, gn // ur, mt, tm, BUF["N"], gout, gaux, WK["GU"],
                      xm(H) | plan(gn // ur, H, gnb))
        ev = gemm_stage(o_gu, ev)
        if unfused:
            ev = cu_stage(op(SWIGLU, l, 2, 0, Fd, Fd, 0, 0, 1, batch, BUF["GU32"], BUF["H"], Fd, WK["NONE"]), rows, ev)
        ev = gemm_stage(op(GEMM, l, 1, path, Fd, H, ur, H // ur, mt, tm, BUF["H"], BUF["X"], 0, WK["DOWN"],
                           xm(Fd) | plan(H // ur, Fd, 1)), ev)
        xready.append(ev)
    mark()
    ev = cu_stage(op(FINAL, -1, 0, 0, H, H, 0, 0, 1, batch, BUF["X"], BUF["N"], 1 if sh.vocab else 0, WK["FINAL"]),
                  rows, ev)
    mark()      # a step without logits ends here
    if sh.vocab:
        gemm_stage(op(GEMM, -1, 0, path, H, sh.vocab, ur, sh.vocab // ur, mt, tm, BUF["N"], BUF["LOGITS"], 0,
                      WK["LM"], xm(H) | plan(sh.vocab // ur, H, 1)), ev)
    mark()
    qoff = np.cumsum([0] + [len(q) for q in queues])
    return dict(ops=np.array(ops, np.int32), tasks=np.array(tasks, np.int32),
                events=np.array(events, np.int32), qoff=qoff.astype(np.int32),
                qents=np.array([e for q in queues for e in q], np.int32),
                marks=np.array(marks, np.int32).T, xready=np.array(xready, np.int32),
                S=S, tile_m=tm, m_tiles=mt)


CASES = [
    (si.reduced_shape(max_batch=64, n_layers=2, vocab=2064), [1, 2, 5, 8, 9, 33, 64], 8, 256),
    (si.qwen3_8b_shape(64, 4097, n_layers=3), [1, 2, 8, 32, 64], 8, 256),
    (si.qwen3_8b_shape(128, 513, n_layers=1), [65, 100, 128], 8, 256),   # two 64-row m-tiles
    (si.reduced_shape(max_batch=4), [1, 3], 4, 120),          # another chiplet count / CU count
]


@pytest.mark.parametrize("sched,tile_m,flags", [(0, 0, 0), (0, 16, 0), (1, 0, 0), (1, 16, 0), (0, 0, 4), (1, 0, 4),
                                                 (2, 16, 0), (2, 32, 0), (0, 16, 32), (1, 0, 32), (0, 0, 128), (1, 0, 128),
                                                 (0, 0, 256), (1, 16, 256)])
def test_builder_equals_independent_derivation(sched, tile_m, flags):
    for sh, batches, n_xcd, n_workers in CASES:
        for b in batches:
            got = F.parse_graph(F.fleet_graph_build(sh.asdict(), b, n_xcd, n_workers, sched, tile_m, flags))
            exp = expected_graph(sh, b, n_xcd, n_workers, sched, tile_m, flags)
            for k in ("ops", "tasks", "events", "qoff", "qents", "marks", "xready"):
                assert np.array_equal(got[k], exp[k]), (k, b, sched, tile_m)
            h = got["header"]
            assert (h["n_splits"], h["tile_m"], h["m_tiles"], h["batch"], h["sched"]) == \
                (exp["S"], exp["tile_m"], exp["m_tiles"], b, sched)


# ------------------------------------------------------------------ graph properties
def _producers(g):
    prod = {}
    for i, t in enumerate(g["tasks"]):
        prod.setdefault(int(t[8]), []).append(i)
    return prod


@pytest.mark.parametrize("sched", [0, 1, 2])
@pytest.mark.parametrize("batch", [1, 8, 32, 64])
def test_graph_invariants(batch, sched):
    sh = si.qwen3_8b_shape(64, 4097, n_layers=2)
    g = F.parse_graph(F.fleet_graph_build(sh.asdict(), batch, 8, 256, sched, 16))
    tasks, events, ops = g["tasks"], g["events"], g["ops"]
    prod = _producers(g)
    # thresholds: one device-level signal per chiplet for two-level events, per task otherwise
    for e, ev in enumerate(events):
        assert ev[3] == len(prod[e])
        if ev[1] == 0:
            assert ev[0] == len(prod[e])
        else:
            assert bin(int(ev[2])).count("1") == ev[0]
            assert sorted({int(tasks[t][2]) for t in prod[e]}) == [x for x in range(8) if ev[2] >> x & 1]
            assert all(int(tasks[t][1]) == (2 if ev[1] == 1 else 1) for t in prod[e])
    # every task is reachable from exactly one queue position (chiplet / XCD groups) or from
    # the same position of every queue (device-wide groups)
    seen = np.zeros(len(tasks), int)
    for x in range(8):
        for q in g["qents"][g["qoff"][x]:g["qoff"][x + 1]]:
            first, cnt, dist = int(q[0]), int(q[1]), int(q[2])
            if dist == 2:
                seen[first:first + cnt] += 1
            else:
                seen[first:first + cnt] += 8
                assert all(tasks[t][2] == x for t in range(first, first + cnt))
    assert (seen == 8).all()
    # queues list stages in dependency order: a task's wait event is signalled only by tasks
    # of an earlier stage, and stages never decrease along a queue
    for t in tasks:
        if t[7] >= 0:
            assert all(tasks[p][9] < t[9] for p in prod[int(t[7])])
    for x in range(8):
        st = g["qents"][g["qoff"][x]:g["qoff"][x + 1], 3]
        assert (np.diff(st) > 0).all()
    # GEMM device-tasks tile the output exactly once per k-slice of the operator's plan
    for o, op in enumerate(ops):
        if op[0] != GEMM:
            continue
        ksn = max(1, op[15] >> 16 & 15) if op[3] == 1 else 1
        cover = np.zeros((op[7], op[8], ksn), int)
        for t in tasks[tasks[:, 0] == o]:
            if t[1] == 2 and t[6] > 0:
                cover[t[3]:t[3] + t[4], t[6] - 1, :] += 1   # M-split: one m-tile of the task's units
            elif t[1] == 2:
                cover[t[3]:t[3] + t[4], :, :] += 1      # a chiplet-task walks all its tiles
            else:
                cover[t[3]:t[3] + t[4], t[5], t[6]] += 1
                assert op[3] == 0 or t[4] <= max(1, op[15] >> 12 & 15)
        assert (cover == 1).all()
        if ksn > 1:
            assert op[4] % (ksn * 256) == 0 and op[7] * op[8] <= 4096
        assert op[8] == -(-batch // op[9]) and op[5] == op[6] * op[7]


def test_paper_task_counts_and_partition_pointers():
    """Fleet's graph at bs=1: one CU-task per norm and eight chiplet-tasks per GEMM; the
    partition of chiplet k starts k*(N/8) rows into the weight matrix."""
    sh = si.qwen3_8b_shape(1, 1025, n_layers=1)
    g = F.parse_graph(F.fleet_graph_build(sh.asdict(), 1, 8, 256, 0, 0, F.FLAG_SEPARATE_NORM))
    tasks, ops = g["tasks"], g["ops"]
    want = GOLD["tasks_per_op_bs1"]
    by_wk = {int(op[13]): i for i, op in enumerate(ops)}
    for name, wk in (("qkv", WK["QKV"]), ("o_proj", WK["O"]), ("gate_up", WK["GU"]), ("down", WK["DOWN"])):
        mine = tasks[tasks[:, 0] == by_wk[wk]]
        assert len(mine) == want[name] and (mine[:, 1] == 2).all()
        op = ops[by_wk[wk]]
        rows_per_xcd = op[5] // GOLD["partition_pointer_rule"]["n_xcd"]
        for k, t in enumerate(mine):
            assert t[2] == k and t[3] * op[6] == k * rows_per_xcd and t[4] * op[6] == rows_per_xcd
    for wk in (WK["LN1"], WK["LN2"]):
        assert (tasks[:, 0] == by_wk[wk]).sum() == want["rmsnorm"]
    # m_tiles of the paper's 16-row tiles: 1 up to batch 16, 2 at 32, 4 at 64
    sh64 = si.qwen3_8b_shape(64, 4097, n_layers=1)
    for c in GOLD["l2_hit_model"]["cases"]:
        if c["batch"] > 8:
            h = F.parse_graph(F.fleet_graph_build(sh64.asdict(), c["batch"], 8, 256, 0, 16))["header"]
            assert h["m_tiles"] == c["m_tiles"]


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other --gpus value ends with a message and exit code 2,
    before anything touches a device."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert res.returncode == 2
    assert "one GPU" in (res.stdout + res.stderr)
