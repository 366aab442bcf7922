#!/usr/bin/env python3
"""Benchmark of the decode-step megakernel on one MI355X.

A "step" is one pass of the whole hot path: one decode step of the 36-layer
Qwen3-8B-shaped stack (ingest, per layer RMSNorm / QKV / attention / O / RMSNorm /
gate-up + SwiGLU / down, final norm, LM head) as one launch of the persistent kernel,
on seeded synthetic weights and KV cache already resident in HBM.

Prints ONE JSON line: decode-step latency in microseconds (lower is better), with a
`roofline` object (algorithmic HBM bytes of one step / measured kernel time, against
8 TB/s) and a `cpu_baseline` object (the CPU oracle timed on a bounded sample).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0

# HBM bytes per launch of the persistent kernel (reads + writes) from the rocprofv3
# FETCH_SIZE and WRITE_SIZE passes summarised in
# profiles/fleet_persistent_kernel_counters_qwen3_8b_b1_to_b64.md, after scaling by what the
# same counters read for a plain copy of known size.  Key: (batch, kv, kv_min, sched, tile_m, flags)
# at 36 layers and seed 2; any other workload reports null unless --traffic-bytes is given.
MEASURED_TRAFFIC = {
    (1, 1024, 0, 0, 0, 0): 15450548864,
    (1, 1024, 0, 1, 0, 0): 15431806304,
    (1, 1024, 0, 0, 0, 64): 16205908416,
    (1, 1024, 0, 0, 0, 256): 16262395008,
    (8, 2048, 1024, 0, 0, 0): 17331194048,
    (8, 2048, 1024, 0, 0, 4): 17343882048,
    (8, 2048, 1024, 1, 0, 0): 17487087456,
    (32, 2048, 1024, 0, 0, 0): 23608298240,
    (32, 2048, 1024, 0, 16, 0): 24150736448,
    (32, 2048, 1024, 1, 16, 0): 32720066496,
    (32, 2048, 1024, 2, 16, 0): 38613665792,
    (64, 4096, 0, 0, 0, 0): 55967937472,
    (64, 4096, 0, 0, 16, 0): 57076790528,
    (64, 4096, 0, 1, 16, 0): 81750251392,
    (64, 4096, 0, 2, 16, 0): 100455350080,
    (64, 4096, 0, 0, 16, 32): 56763077056,
    (64, 4096, 0, 0, 16, 2048): 57070389632,
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=1)
    ap.add_argument("--kv", type=int, default=1024, help="valid KV slots per sequence before the step")
    ap.add_argument("--kv-min", type=int, default=0, help="if > 0, per-sequence lengths uniform in [kv-min, kv]")
    ap.add_argument("--layers", type=int, default=36)
    ap.add_argument("--sched", type=int, default=0, help="0 cooperative (XCD), 1 chiplet-unaware, 2 M-split")
    ap.add_argument("--tile-m", type=int, default=0)
    ap.add_argument("--flags", type=int, default=0)
    ap.add_argument("--seed", type=int, default=2)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-sweep", dest="sweep", action="store_false",
                    help="skip the extra workloads (batch 8 / 32 / 64) reported under 'sweep'")
    ap.add_argument("--gemm-sweep", action="store_true",
                    help="isolated skinny-GEMM sweep at the Qwen3-8B shapes (one JSON line per case)")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MiB",
                    help="run only a plain copy of this many MiB (counter calibration under rocprofv3)")
    ap.add_argument("--tokens-per-launch", type=int, default=0, metavar="T",
                    help="time T greedy decode steps per launch of the persistent kernel (fleet_decode_tokens) "
                         "instead of one step per launch; one JSON line")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per step from rocprofv3 counters (reported as roofline.traffic)")
    return ap.parse_args()


def cpu_baseline(shape, w_dev, hidden_dev, batch, kv, seed):
    """Time the CPU oracle on a bounded sample of the same workload: the first
    `n_sample` layers plus the LM head, one sequence; report the full-step time
    obtained by scaling the per-layer part to all layers."""
    import numpy as np
    import oracle
    import synth_inputs as si
    n_sample = min(4, shape.n_layers)
    sh = si.Shape(**{**shape.asdict(), "n_layers": n_sample, "max_batch": 1, "max_seq": kv + 1})
    wh = {k: [si.to_host_u16(a) for a in w_dev[k][:n_sample]] for k in si.PER_LAYER}
    wh["final_norm"] = si.to_host_u16(w_dev["final_norm"])
    wh["lm_head"] = si.to_host_u16(w_dev["lm_head"])
    g = si.Gen(seed + 1000)
    kc, vc = si.make_kv_cache(sh, g)
    kc, vc = si.to_host_u16(kc), si.to_host_u16(vc)
    hid = si.to_host_u16(hidden_dev[:1])
    pos = np.array([kv], np.int32)
    x0 = si.bf16_bits_to_f32(hid)
    t0 = time.perf_counter()
    x1, _ = oracle.decode_layers(sh.asdict(), wh, 1, 0, n_sample, x0, pos, kc, vc)
    t_layers = time.perf_counter() - t0
    t0 = time.perf_counter()
    n = oracle.rmsnorm(x1, wh["final_norm"], sh.rms_eps)
    oracle.linear(n, wh["lm_head"])
    t_head = time.perf_counter() - t0
    full = (t_layers / n_sample * shape.n_layers + t_head) * batch
    return {"value": full * 1e6, "unit": "us", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"{n_sample} of {shape.n_layers} layers + LM head, 1 of {batch} sequences, KV {kv}: "
                      f"{t_layers:.3f} s + {t_head:.3f} s, scaled to all layers and sequences"}


def gemm_sweep(a):
    """y = x W^T as back-to-back device-tasks of the persistent kernel; every rep reads a
    different weight copy (more than 512 MB in rotation, so the 256 MB last-level cache
    cannot serve the weights) and the launch is timed with HIP events by the library."""
    import torch
    import paper_2604_15379_amd as F
    import synth_inputs as si
    g = si.Gen(1, "cuda")
    for (K, N) in ((4096, 6144), (4096, 4096), (4096, 24576), (12288, 4096)):
        n_copies = max(2, -(-(640 << 20) // (K * N * 2)))
        ws = [g.normal_bf16((N, K), 0.02) for _ in range(n_copies)]
        for B in (1, 8, 32, 64):
            x = g.normal_bf16((B, K), 1.0)
            y = torch.empty((B, N), device="cuda", dtype=torch.float32)
            reps = 4 * n_copies
            F.fleet_gemm(B, K, N, x, ws, y, a.sched, a.tile_m, a.flags, reps)          # warm-up
            ms = min(F.fleet_gemm(B, K, N, x, ws, y, a.sched, a.tile_m, a.flags, reps) for _ in range(3))
            bytes_per_rep = K * N * 2 + B * (K * 2 + N * 4)
            print(json.dumps({"gemm": [B, K, N], "us_per_gemm": ms * 1e3 / reps, "reps": reps,
                              "GBps": bytes_per_rep * reps / (ms * 1e-3) / 1e9,
                              "frac_of_8TBps": bytes_per_rep * reps / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                              "sched_mode": a.sched, "tile_m": a.tile_m, "flags": a.flags}), flush=True)
        del ws


def tokens_per_launch(a):
    """T greedy steps in one launch (the kernel stays resident over the tokens) against the
    same T steps launched one by one from the host; positions start at --kv and advance."""
    import numpy as np
    import torch
    import paper_2604_15379_amd as F
    import synth_inputs as si
    B, T = a.batch, a.tokens_per_launch
    shape = si.qwen3_8b_shape(max_batch=B, max_seq=a.kv + T + 1, n_layers=a.layers)
    g = si.Gen(a.seed, "cuda")
    w = si.make_weights(shape, g, with_embed=True)
    kc, vc = si.make_kv_cache(shape, g)
    tok0 = g.randint(0, shape.vocab - 1, B).to(torch.int32)
    hout = torch.empty((B, shape.hidden), device="cuda", dtype=torch.float32)
    logits = torch.empty((B, shape.vocab), device="cuda", dtype=torch.float32)
    out = torch.empty((T, B), device="cuda", dtype=torch.int32)
    f = F.fleet_create(shape.asdict(), w, a.sched, a.tile_m, a.flags)
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

    def one_launch():
        tok, pos = tok0.clone(), torch.full((B,), a.kv, device="cuda", dtype=torch.int32)
        torch.cuda.synchronize()
        e0.record()
        F.fleet_decode_tokens(f, B, tok, kc, vc, pos, T, out, hout, logits, stream)
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    def host_loop():
        tok, pos = tok0.clone(), torch.full((B,), a.kv, device="cuda", dtype=torch.int32)
        torch.cuda.synchronize()
        e0.record()
        for _ in range(T):   # the host chooses the token (device-side argmax, no host sync)
            F.fleet_decode_step(f, B, None, tok, kc, vc, pos, hout, logits, stream)
            tok = logits.argmax(dim=1).to(torch.int32)
            pos += 1
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1)

    one_launch(); host_loop()
    ms_launch = min(one_launch() for _ in range(max(1, a.steps // T)))
    st = F.fleet_last_status(f)
    if st["code"] != 0:
        raise SystemExit(f"decode failed: {st}")
    ms_host = min(host_loop() for _ in range(max(1, a.steps // T)))
    F.fleet_destroy(f)
    print(json.dumps({"metric": "decode_step_latency_us", "value": ms_launch * 1e3 / T, "unit": "us", "n_gpus": 1,
                      "config": {"workload": f"Qwen3-8B-shaped greedy decoding, {a.layers} layers + LM head, batch {B}, "
                                             f"KV {a.kv}.., {T} steps per launch of the persistent kernel",
                                 "batch": B, "tokens_per_launch": T},
                      "one_step_per_launch_us": ms_host * 1e3 / T, "tokens_per_s": B * T / (ms_launch * 1e-3)}))


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: the decode step runs on a single MI355X and nothing in this "
              "build shards across GPUs; run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch
    import paper_2604_15379_amd as F
    import synth_inputs as si

    torch.cuda.set_device(0)
    if a.calibrate_copy > 0:
        n = a.calibrate_copy << 20
        src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(a.steps):
            F.fleet_copy(dst, src, n, torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(src, dst)
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": a.steps}))
        return
    if a.gemm_sweep:
        gemm_sweep(a)
        return
    if a.tokens_per_launch > 0:
        tokens_per_launch(a)
        return
    g = si.Gen(a.seed, "cuda")
    w = si.make_weights(si.qwen3_8b_shape(max_batch=1, max_seq=2, n_layers=a.layers), g)

    def time_config(batch, kv, kv_min, sched, tile_m, flags, steps, warmup):
        """One workload: seeded inputs resident in HBM, `warmup` untimed steps, `steps` timed ones
        between two events on the launch stream."""
        shape = si.qwen3_8b_shape(max_batch=batch, max_seq=kv + 1, n_layers=a.layers)
        gi = si.Gen(a.seed + 7919 * batch, "cuda")
        hidden = si.make_hidden(shape, batch, gi)
        kc, vc = si.make_kv_cache(shape, gi)
        pos_host = gi.randint(kv_min, kv, batch).cpu().numpy().astype(np.int32) if kv_min > 0 else np.full(batch, kv, np.int32)
        pos = torch.tensor(pos_host, device="cuda")
        hout = torch.empty((batch, shape.hidden), device="cuda", dtype=torch.float32)
        logits = torch.empty((batch, shape.vocab), device="cuda", dtype=torch.float32)
        f = F.fleet_create(shape.asdict(), w, sched, tile_m, flags)
        stream = torch.cuda.current_stream().cuda_stream
        try:
            for _ in range(warmup):
                F.fleet_decode_step(f, batch, hidden, None, kc, vc, pos, hout, logits, stream)
            torch.cuda.synchronize()
            st = F.fleet_last_status(f)
            if st["code"] != 0:
                raise SystemExit(f"decode step failed: {st}")
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                F.fleet_decode_step(f, batch, hidden, None, kc, vc, pos, hout, logits, stream)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1) / steps
            st = F.fleet_last_status(f)
            if st["code"] != 0 or not torch.isfinite(logits).all():
                raise SystemExit(f"decode step failed: {st}")
        finally:
            F.fleet_destroy(f)
        step_bytes = F.fleet_step_bytes(shape.asdict(), batch, pos_host)
        return dict(ms=ms, step_bytes=step_bytes, gbps=step_bytes / (ms * 1e-3) / 1e9, shape=shape, hidden=hidden,
                    workers=st["workers"])

    B = a.batch
    r = time_config(B, a.kv, a.kv_min, a.sched, a.tile_m, a.flags, a.steps, a.warmup)
    ms, step_bytes, gbps, shape = r["ms"], r["step_bytes"], r["gbps"], r["shape"]
    traffic = a.traffic_bytes
    traffic_source = "--traffic-bytes" if traffic is not None else None
    if traffic is None and a.layers == 36 and a.seed == 2:
        traffic = MEASURED_TRAFFIC.get((B, a.kv, a.kv_min, a.sched, a.tile_m, a.flags))
        if traffic is not None:
            traffic_source = ("constant from the rocprofv3 FETCH_SIZE / WRITE_SIZE passes in profiles/ "
                              "(not measured in this run)")
    out = {
        "metric": "decode_step_latency_us", "value": ms * 1e3, "unit": "us", "n_gpus": 1,
        "steps": a.steps, "warmup": a.warmup, "ms_per_step": ms, "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"Qwen3-8B-shaped decode step, {a.layers} layers + LM head, batch {B}, "
                               f"KV {a.kv_min or a.kv}..{a.kv} per sequence, random bf16 weights (seed {a.seed})",
                   "batch": B, "kv_len": a.kv, "sched_mode": ["cooperative", "unaware", "m-split"][a.sched],
                   "tile_m": a.tile_m, "flags": a.flags, "tokens_per_s": B / (ms * 1e-3)},
        "roofline": {"bound": "hbm", "achieved": gbps, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": gbps / HBM_PEAK_GBPS, "traffic": traffic, "traffic_source": traffic_source,
                     "algorithmic_bytes": step_bytes,
                     "kernel": "fleet_persistent_kernel (one launch per step)"},
        "l2_hit_model": F.fleet_l2_hit_model(B, a.tile_m, 32) if B > 2 else 0.0,
        "workers_per_xcd": r["workers"],
    }
    if a.sweep:
        # the other workloads of the metric (batch 8 / 32 with ragged KV 1024..2048, batch 64 with KV
        # 4096, cooperative against chiplet-unaware at the paper's 16-row tiles), fewer steps each
        out["sweep"] = []
        for (b, kv, kv_min, sched, tile_m, steps) in ((8, 2048, 1024, 0, 0, 10), (32, 2048, 1024, 0, 0, 10),
                                                      (64, 4096, 0, 0, 0, 5), (64, 4096, 0, 0, 16, 5),
                                                      (64, 4096, 0, 1, 16, 5)):
            t = time_config(b, kv, kv_min, sched, tile_m, 0, steps, 2)
            out["sweep"].append({"batch": b, "kv": kv, "kv_min": kv_min or kv,
                                 "sched": ["cooperative", "unaware", "m-split"][sched], "tile_m": tile_m,
                                 "ms_per_step": t["ms"], "algorithmic_bytes": t["step_bytes"],
                                 "GBps": t["gbps"], "frac": t["gbps"] / HBM_PEAK_GBPS, "steps": steps,
                                 # profiled constant (see MEASURED_TRAFFIC), not measured in this run
                                 "traffic": MEASURED_TRAFFIC.get((b, kv, kv_min, sched, tile_m, 0))
                                 if a.layers == 36 and a.seed == 2 else None})
    if not a.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(shape, w, r["hidden"], B, a.kv, a.seed)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
