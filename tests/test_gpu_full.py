"""Full-size GPU parity: the 36-layer Qwen3-8B-shaped decode step in the launch
configuration bench.py times (batch 1, KV 1024), and the batch 8 / 32 / 64 configurations
on sampled sequences (rows of a decode step are independent, so the oracle computes rows
{0, B/2, B-1} from compact copies of their caches).

The 2e-2 x RMS bar is applied layer by layer with teacher forcing: every layer is started
from the oracle's residual stream entering that layer (the oracle's own result moves by
more than the bar over 36 layers when only its fp32 summation order is changed, so no two
valid implementations can meet it free-running; the free-running result is checked against
that measured envelope instead)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2604_15379_amd as F
import synth_inputs as si
from gpu_common import TOL, assert_close, rms

pytestmark = pytest.mark.gpu

L = 36
# Free-running over 36 layers the kernel may differ from the oracle by as much as the oracle
# differs from itself when only its fp32 summation order is reversed, times this factor
# (measured ratios on MI355X: 0.8 to 1.2 over all the configurations below).
ENVELOPE_FACTOR = 1.5


@pytest.fixture(scope="module")
def weights():
    shape = si.qwen3_8b_shape(max_batch=1, max_seq=2, n_layers=L)
    g = si.Gen(2, "cuda")
    w = si.make_weights(shape, g)
    print("weights on device; copying to host for the oracle", flush=True)
    return w, si.weights_to_host(w)


def _case(weights, batch, kv_lo, kv_hi, seed, rows):
    w, wh = weights
    shape = si.qwen3_8b_shape(max_batch=batch, max_seq=kv_hi + 1, n_layers=L)
    g = si.Gen(seed, "cuda")
    hidden = si.make_hidden(shape, batch, g)
    kc, vc = si.make_kv_cache(shape, g)
    pos = g.randint(kv_lo, kv_hi, batch) if kv_lo < kv_hi else torch.full((batch,), kv_hi, device="cuda", dtype=torch.int32)
    rows = sorted(set(rows))
    # compact oracle inputs for the sampled rows
    sh_o = si.Shape(**{**shape.asdict(), "max_batch": len(rows)})
    idx = torch.tensor(rows, device="cuda")
    kc_h = si.to_host_u16(kc.index_select(1, idx))
    vc_h = si.to_host_u16(vc.index_select(1, idx))
    hid_h = si.to_host_u16(hidden.index_select(0, idx))
    pos_h = pos.index_select(0, idx).cpu().numpy().astype(np.int32)
    return dict(shape=shape, w=w, wh=wh, hidden=hidden, kc=kc, vc=vc, pos=pos, rows=rows, sh_o=sh_o,
                kc_h=kc_h, vc_h=vc_h, hid_h=hid_h, pos_h=pos_h, batch=batch)


def _oracle(c, flags=0):
    k, v = c["kc_h"].copy(), c["vc_h"].copy()
    ho, lg, tr = oracle.decode_step(c["sh_o"].asdict(), c["wh"], len(c["rows"]), c["pos_h"], k, v,
                                    hidden_in=c["hid_h"], want_trace=True, flags=flags)
    return ho, lg, tr, k, v


def _gpu_free_running(c, sched, tile_m, flags=0):
    sh, B = c["shape"], c["batch"]
    f = F.fleet_create(sh.asdict(), c["w"], sched, tile_m, flags)
    try:
        kc, vc = c["kc"].clone(), c["vc"].clone()
        hout = torch.full((B, sh.hidden), float("nan"), device="cuda")
        logits = torch.full((B, sh.vocab), float("nan"), device="cuda")
        F.fleet_decode_step(f, B, c["hidden"], None, kc, vc, c["pos"], hout, logits,
                            torch.cuda.current_stream().cuda_stream)
        st = F.fleet_last_status(f)
        assert st["code"] == 0, st
        return hout, logits, kc, vc
    finally:
        F.fleet_destroy(f)


def _gpu_teacher_forced(c, tr, lg_ref, sched, tile_m, flags=0):
    """Run every layer from the oracle's input to that layer (sampled rows; the other rows
    chain the GPU's own output).  Returns the worst max|err|/RMS over layers."""
    sh, B, rows = c["shape"], c["batch"], c["rows"]
    idx = torch.tensor(rows, device="cuda")
    f = F.fleet_create(sh.asdict(), c["w"], sched, tile_m, flags)
    worst = 0.0
    try:
        kc, vc = c["kc"].clone(), c["vc"].clone()
        x = c["hidden"].float()
        xo = torch.empty_like(x)
        logits = torch.full((B, sh.vocab), float("nan"), device="cuda")
        stream = torch.cuda.current_stream().cuda_stream
        for l in range(L):
            x.index_copy_(0, idx, torch.tensor(tr[l], device="cuda"))
            F.fleet_decode_layers(f, B, l, l + 1, x, kc, vc, c["pos"], xo, logits if l == L - 1 else None, stream)
            got = xo.index_select(0, idx).cpu().numpy()
            st = F.fleet_last_status(f)
            assert st["code"] == 0, (l, st)
            worst = max(worst, assert_close(got, tr[l + 1], f"layer {l} output (teacher-forced)"))
            x, xo = xo, x
        lg = logits.index_select(0, idx).cpu().numpy()
        worst = max(worst, assert_close(lg, lg_ref, "logits (last layer teacher-forced)"))
    finally:
        F.fleet_destroy(f)
    return worst, kc, vc


def _check(c, sched, tile_m, flags=0, free_running=True):
    ho, lg, tr, k_ref, v_ref = _oracle(c)
    worst, kc, vc = _gpu_teacher_forced(c, tr, lg, sched, tile_m, flags)
    print(f"  teacher-forced worst max|err|/RMS over {L} layers + logits: {worst:.3e} (bar {TOL})", flush=True)
    # new cache entries of the sampled rows: within the residual stream's tolerance
    idx = torch.tensor(c["rows"], device="cuda")
    for got_t, ref, nm in ((kc, k_ref, "k"), (vc, v_ref, "v")):
        got = si.to_host_u16(got_t.index_select(1, idx))
        for i in range(len(c["rows"])):
            p = int(c["pos_h"][i])
            g = si.bf16_bits_to_f32(got[:, i, :, p]).astype(np.float64)
            r = si.bf16_bits_to_f32(ref[:, i, :, p]).astype(np.float64)
            assert np.abs(g - r).max() <= TOL * rms(r) + 2.0 ** -7 * np.abs(r).max(), f"new {nm} entries"
            untouched = np.ones(got.shape[3], bool)
            untouched[p] = False
            assert np.array_equal(got[:, i, :, untouched], c["kc_h" if nm == "k" else "vc_h"][:, i, :, untouched])
    if free_running:
        ho_r, lg_r, _, _, _ = _oracle(c, oracle.REVERSE_K)
        env_h = np.abs(ho_r - ho).max() / rms(ho)
        env_l = np.abs(lg_r - lg).max() / rms(lg)
        hout, logits, _, _ = _gpu_free_running(c, sched, tile_m, flags)
        eh = np.abs(hout.index_select(0, idx).cpu().numpy() - ho).max() / rms(ho)
        el = np.abs(logits.index_select(0, idx).cpu().numpy() - lg).max() / rms(lg)
        print(f"  free-running max|err|/RMS: hidden {eh:.3e} logits {el:.3e}; oracle vs its own reversed "
              f"summation order: hidden {env_h:.3e} logits {env_l:.3e}", flush=True)
        print(f"  ratio to the envelope: hidden {eh / env_h:.2f} logits {el / env_l:.2f}", flush=True)
        assert eh <= max(ENVELOPE_FACTOR * env_h, TOL) and el <= max(ENVELOPE_FACTOR * env_l, TOL)
        return hout, logits
    return None, None


def test_batch1_kv1024_bench_configuration(weights):
    c = _case(weights, 1, 1024, 1024, seed=2, rows=[0])
    _check(c, 0, 0)


@pytest.mark.parametrize("batch", [8, 32])
def test_batch8_32_ragged_kv(weights, batch):
    c = _case(weights, batch, 1024, 2048, seed=3, rows=[0, batch // 2, batch - 1])
    print(f"batch {batch}: positions of sampled rows {c['pos_h'].tolist()}", flush=True)
    _check(c, 0, 0)


def test_batch64_kv4096_cooperative_and_unaware(weights):
    c = _case(weights, 64, 4096, 4096, seed=4, rows=[0, 32, 63])
    h0, l0 = _check(c, F.SCHED_COOPERATIVE, 16)
    h1, l1 = _check(c, F.SCHED_UNAWARE, 16)
    # same tiles, same in-tile reduction order, two task-to-worker maps: identical bits
    assert torch.equal(h0, h1) and torch.equal(l0, l1)
    _check(c, F.SCHED_COOPERATIVE, 0, free_running=False)


@pytest.mark.parametrize("batch,sched,tile_m,fma_max", [
    (32, F.SCHED_UNAWARE, 0, None),      # chiplet-unaware schedule with the whole-batch tile
    (32, F.SCHED_MSPLIT, 16, None),      # M-split over 16-row tiles
    (2, F.SCHED_COOPERATIVE, 0, 2),      # FMA GEMV kernel with two batch rows
    (2, F.SCHED_COOPERATIVE, 0, None),   # MFMA kernel, two rows of a 16-row block
    (16, F.SCHED_COOPERATIVE, 0, None),  # MFMA kernel, one full 16-row block
    (8, F.SCHED_COOPERATIVE, 0, 8),      # FMA GEMV kernel with eight batch rows
    (4, F.SCHED_COOPERATIVE, 0, 8),      # FMA GEMV kernel with four batch rows
])
def test_other_schedules_and_kernel_flavours_at_full_depth(weights, monkeypatch, batch, sched, tile_m, fma_max):
    """Teacher-forced 36-layer comparison with the oracle (2e-2 x RMS per layer and on the
    logits) for the schedule / kernel-flavour combinations the other tests of this file do not
    reach: every persistent-kernel variant meets the oracle at the full model size."""
    if fma_max is not None:
        monkeypatch.setenv("FLEET_FMA_MAX_BATCH", str(fma_max))
    rows = sorted({0, batch // 2, batch - 1})
    c = _case(weights, batch, 1024, 2048, seed=3, rows=rows)
    print(f"batch {batch} sched {sched} tile_m {tile_m} fma_max {fma_max}: positions {c['pos_h'].tolist()}", flush=True)
    _check(c, sched, tile_m, free_running=False)


def test_timeout_aborts_a_full_size_step(weights, monkeypatch):
    """With a time limit of half a microsecond against a 36-layer batch-32 step (its stages last
    tens of microseconds) some dependency wait runs out: the step aborts on the device, every
    worker leaves, the status says FLEET_ETIMEOUT with the event that was waited for, and the
    same fleet geometry runs normally again afterwards."""
    monkeypatch.setenv("FLEET_TIMEOUT_MS", "0.0005")
    c = _case(weights, 32, 2048, 2048, seed=3, rows=[0])
    sh = c["shape"]
    f = F.fleet_create(sh.asdict(), c["w"], 0, 0, 0)
    monkeypatch.delenv("FLEET_TIMEOUT_MS")
    try:
        hout = torch.zeros((32, sh.hidden), device="cuda")
        logits = torch.zeros((32, sh.vocab), device="cuda")
        F.fleet_decode_step(f, 32, c["hidden"], None, c["kc"], c["vc"], c["pos"], hout, logits,
                            torch.cuda.current_stream().cuda_stream)
        st = F.fleet_last_status(f)
        print("status with a 0.5 us limit:", st, flush=True)
        assert st["code"] == -4 and st["event"] >= 0 and st["observed"] < st["needed"]
    finally:
        F.fleet_destroy(f)
    f = F.fleet_create(sh.asdict(), c["w"], 0, 0, 0)
    try:
        F.fleet_decode_step(f, 32, c["hidden"], None, c["kc"], c["vc"], c["pos"], hout, logits,
                            torch.cuda.current_stream().cuda_stream)
        assert F.fleet_last_status(f)["code"] == 0 and torch.isfinite(logits).all()
    finally:
        F.fleet_destroy(f)


@pytest.mark.parametrize("batch,kv_lo,kv_hi,reps,sched,tile_m", [
    (8, 1024, 2048, 200, 0, 0), (32, 1024, 2048, 120, 0, 0), (2, 1024, 2048, 200, 0, 0),
    (8, 1024, 2048, 100, F.SCHED_UNAWARE, 0), (32, 1024, 2048, 80, F.SCHED_MSPLIT, 16)])
def test_repeated_steps_give_identical_bits(weights, batch, kv_lo, kv_hi, reps, sched, tile_m):
    """The step is deterministic by construction (fixed reduction orders, last-arriver merges in
    index order): repeating it on the same inputs must give the same bits every time.  A
    hand-off between XCDs that sometimes delivers a stale activation row shows up here as a row
    that differs in a few steps out of a hundred, while staying inside the parity tolerance."""
    c = _case(weights, batch, kv_lo, kv_hi, seed=3, rows=[0])
    sh, B = c["shape"], batch
    f = F.fleet_create(sh.asdict(), c["w"], sched, tile_m, 0)
    try:
        kc, vc = c["kc"].clone(), c["vc"].clone()
        stream = torch.cuda.current_stream().cuda_stream
        first = None
        for r in range(reps):
            hout = torch.full((B, sh.hidden), float("nan"), device="cuda")
            logits = torch.full((B, sh.vocab), float("nan"), device="cuda")
            F.fleet_decode_step(f, B, c["hidden"], None, kc, vc, c["pos"], hout, logits, stream)
            torch.cuda.synchronize()
            assert F.fleet_last_status(f)["code"] == 0
            if first is None:
                first = (hout, logits)
                continue
            same_h = torch.equal(hout.view(torch.int32), first[0].view(torch.int32))
            same_l = torch.equal(logits.view(torch.int32), first[1].view(torch.int32))
            if not (same_h and same_l):
                rows = torch.nonzero((hout - first[0]).abs().amax(1)).flatten().tolist()
                raise AssertionError(f"step {r} differs from step 0 in batch rows {rows}")
    finally:
        F.fleet_destroy(f)


@pytest.mark.parametrize("batch", [1, 8])
def test_repeated_multi_step_launches_give_identical_bits(weights, batch):
    """Several greedy steps in one launch (the kernel walks its queues once per step, the
    counters keep growing, the next token and position come from the device): the same
    launch repeated from the same state gives the same tokens, logits and cache entries."""
    n_tokens, reps = 8, 25
    w, wh = weights
    shape = si.qwen3_8b_shape(max_batch=batch, max_seq=1100, n_layers=L)
    g = si.Gen(5, "cuda")
    kc0, vc0 = si.make_kv_cache(shape, g)
    embed = g.normal_bf16((shape.vocab, shape.hidden), 1.0)
    tok0 = g.randint(0, shape.vocab - 1, batch)
    pos0 = g.randint(900, 1000, batch)
    f = F.fleet_create(shape.asdict(), {**w, "embed": embed}, 0, 0, 0)
    try:
        first = None
        for r in range(reps):
            kc, vc = kc0.clone(), vc0.clone()
            tok, pos = tok0.clone(), pos0.clone()
            out = torch.full((n_tokens, batch), -1, device="cuda", dtype=torch.int32)
            hout = torch.zeros((batch, shape.hidden), device="cuda")
            logits = torch.zeros((batch, shape.vocab), device="cuda")
            F.fleet_decode_tokens(f, batch, tok, kc, vc, pos, n_tokens, out, hout, logits)
            torch.cuda.synchronize()
            assert F.fleet_last_status(f)["code"] == 0
            new_k = torch.stack([kc[:, b, :, int(pos0[b]):int(pos0[b]) + n_tokens] for b in range(batch)])
            cur = (out.clone(), logits.view(torch.int32).clone(), hout.view(torch.int32).clone(), new_k.view(torch.int16).clone())
            if first is None:
                first = cur
                assert (out >= 0).all() and torch.equal(pos, pos0 + n_tokens)
                continue
            for nm, a, b_ in zip(("tokens", "logits", "hidden", "new keys"), cur, first):
                assert torch.equal(a, b_), f"launch {r}: {nm} differ from launch 0"
    finally:
        F.fleet_destroy(f)
