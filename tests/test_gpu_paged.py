"""GPU parity of the decode step over a paged KV cache: the pages of every sequence are
scattered over a pool; the result must equal the oracle on the contiguous cache, and the new
key/value must land in the right slot of the right page."""
import numpy as np
import pytest
import torch

import paper_2604_15379_amd as F
import synth_inputs as si
from gpu_common import Model, assert_close, check_new_kv

pytestmark = pytest.mark.gpu


def _to_pool(cache, table, page_size, n_pages):
    """cache [L][B][G][S][128] -> pool [L][n_pages][G][page_size][128] following table [B][P]."""
    L, B, G, S, D = cache.shape
    pool = torch.zeros((L, n_pages, G, page_size, D), dtype=cache.dtype, device=cache.device)
    for b in range(B):
        for i, pg in enumerate(table[b]):
            lo, hi = i * page_size, min((i + 1) * page_size, S)
            if lo < S:
                pool[:, pg, :, :hi - lo] = cache[:, b, :, lo:hi]
    return pool


def _from_pool(pool, table, page_size, S):
    L, _, G, _, D = pool.shape
    B = len(table)
    cache = torch.zeros((L, B, G, S, D), dtype=pool.dtype, device=pool.device)
    for b in range(B):
        for i, pg in enumerate(table[b]):
            lo, hi = i * page_size, min((i + 1) * page_size, S)
            if lo < S:
                cache[:, b, :, lo:hi] = pool[:, pg, :, :hi - lo]
    return cache


@pytest.mark.parametrize("batch,page_size,sched", [(1, 64, 0), (2, 64, 0), (5, 64, 0), (5, 128, 1), (20, 64, 0), (40, 256, 0)])
def test_paged_cache_equals_contiguous(batch, page_size, sched):
    print(f"paged batch={batch} page_size={page_size} sched={sched}", flush=True)
    max_seq = 300
    sh = si.reduced_shape(max_batch=batch, max_seq=max_seq, n_layers=2, vocab=1024)
    rng = np.random.default_rng(100 + batch)
    pos = rng.integers(0, max_seq, batch).astype(np.int32)
    pos[0] = 0
    if batch > 1:
        pos[1] = max_seq - 1
    m = Model(sh, seed=50 + batch, batch=batch, positions=pos)
    (ho, lg), k_ref, v_ref = m.run_oracle()
    per_seq = -(-max_seq // page_size)
    n_pages = batch * per_seq + 7
    table = rng.permutation(n_pages)[:batch * per_seq].reshape(batch, per_seq).astype(np.int32)
    kp, vp = _to_pool(m.kc, table, page_size, n_pages), _to_pool(m.vc, table, page_size, n_pages)
    tab_d = torch.tensor(table, device="cuda")
    hout = torch.full((batch, sh.hidden), float("nan"), device="cuda", dtype=torch.float32)
    logits = torch.full((batch, sh.vocab), float("nan"), device="cuda", dtype=torch.float32)
    f = F.fleet_create(sh.asdict(), m.w, sched, 0, 0)
    F.fleet_decode_step_paged(f, batch, m.hidden, None, kp, vp, tab_d, page_size, n_pages, per_seq, m.pos, hout, logits)
    st = F.fleet_last_status(f)
    F.fleet_destroy(f)
    assert st["code"] == 0, st
    assert_close(hout.cpu().numpy(), ho, "hidden_out")
    assert_close(logits.cpu().numpy(), lg, "logits")
    k_gpu = si.to_host_u16(_from_pool(kp, table, page_size, max_seq))
    v_gpu = si.to_host_u16(_from_pool(vp, table, page_size, max_seq))
    check_new_kv(m, k_gpu, v_gpu, k_ref, v_ref)


def test_bad_page_index_is_reported():
    """A page index outside the pool ends the step with FLEET_EINVAL; bad arguments are refused."""
    sh = si.reduced_shape(max_batch=2, max_seq=128, n_layers=1, vocab=512)
    m = Model(sh, seed=61, batch=2, positions=[70, 5])
    n_pages, ps = 8, 64
    table = np.array([[0, 99], [2, 3]], np.int32)        # 99 is not a page of the pool
    kp = torch.zeros((1, n_pages, sh.n_kv_heads, ps, 128), device="cuda", dtype=torch.bfloat16)
    vp = torch.zeros_like(kp)
    hout = torch.zeros((2, sh.hidden), device="cuda", dtype=torch.float32)
    logits = torch.zeros((2, sh.vocab), device="cuda", dtype=torch.float32)
    f = F.fleet_create(sh.asdict(), m.w, 0, 0, 0)
    with pytest.raises(F.FleetError):
        F.fleet_decode_step_paged(f, 2, m.hidden, None, kp, vp, torch.tensor(table, device="cuda"), 48, n_pages, 2,
                                  m.pos, hout, logits)      # page size not a power of two
    F.fleet_decode_step_paged(f, 2, m.hidden, None, kp, vp, torch.tensor(table, device="cuda"), ps, n_pages, 2,
                              m.pos, hout, logits)
    st = F.fleet_last_status(f)
    F.fleet_destroy(f)
    print("status:", st, flush=True)
    assert st["code"] == -1
