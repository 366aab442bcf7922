"""The entry point that allocates nothing (fleet_decode_step_static: the step's working memory
lives in a static device array of the library) against fleet_decode_step, through the C ABI:
two calls in a row, the second with a smaller input, each compared with the result of the
existing entry point on the same inputs (same kernels, same graph: identical bits, and within
the parity bar of the oracle), plus the refusal of a step that does not fit the array."""
import numpy as np
import pytest
import torch

import paper_2604_15379_amd as F
import synth_inputs as si
from gpu_common import Model, assert_close

pytestmark = pytest.mark.gpu


def _both(f, m, entry):
    sh, B = m.shape, m.batch
    kc, vc = m.kc.clone(), m.vc.clone()
    hout = torch.full((B, sh.hidden), float("nan"), device="cuda", dtype=torch.float32)
    logits = torch.full((B, sh.vocab), float("nan"), device="cuda", dtype=torch.float32)
    entry(f, B, m.hidden, None, kc, vc, m.pos, hout, logits, torch.cuda.current_stream().cuda_stream)
    st = F.fleet_last_status(f)
    assert st["code"] == 0, st
    return hout, logits, kc, vc


def test_static_workspace_step_equals_the_allocating_one():
    sh = si.reduced_shape(max_batch=6, max_seq=200, n_layers=2, vocab=1024)
    big = Model(sh, seed=61, batch=6, positions=[0, 199, 5, 77, 128, 64])      # MFMA kernels, split-K partials
    small = Model(sh, seed=61, batch=2, positions=[150, 3])                    # FMA kernels, fewer rows
    f = F.fleet_create(sh.asdict(), big.w, 0, 0, 0)
    try:
        torch.cuda.synchronize()
        free0 = torch.cuda.mem_get_info()[0]
        for m in (big, small):                      # two calls in a row, the second smaller
            print(f"static-workspace step, batch {m.batch}", flush=True)
            got = _both(f, m, F.fleet_decode_step_static)
            assert torch.cuda.mem_get_info()[0] >= free0 - (64 << 20)   # only this test's own clones
            ref = _both(f, m, F.fleet_decode_step)
            for nm, a, b in zip(("hidden_out", "logits", "k_cache", "v_cache"), got, ref):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"{nm} differs (batch {m.batch})"
            (ho, lg), _, _ = m.run_oracle()
            assert_close(got[0].cpu().numpy(), ho, "hidden_out vs oracle")
            assert_close(got[1].cpu().numpy(), lg, "logits vs oracle")
    finally:
        F.fleet_destroy(f)


def test_static_workspace_refuses_what_does_not_fit():
    """A step whose working memory exceeds the array is refused on the host with its own error
    code before anything is launched; the allocating entry point still serves it."""
    sh = si.reduced_shape(max_batch=128, max_seq=40, n_layers=1, vocab=512)
    m = Model(sh, seed=62, batch=128, positions=np.arange(128) % 40)
    f = F.fleet_create(sh.asdict(), m.w, 0, 0, 0)
    try:
        hout = torch.zeros((128, sh.hidden), device="cuda", dtype=torch.float32)
        logits = torch.zeros((128, sh.vocab), device="cuda", dtype=torch.float32)
        with pytest.raises(F.FleetError) as e:
            F.fleet_decode_step_static(f, 128, m.hidden, None, m.kc.clone(), m.vc.clone(), m.pos, hout, logits)
        assert e.value.code == -7 and "static workspace" in str(e.value)
        F.fleet_decode_step(f, 128, m.hidden, None, m.kc.clone(), m.vc.clone(), m.pos, hout, logits)
        assert F.fleet_last_status(f)["code"] == 0
    finally:
        F.fleet_destroy(f)
