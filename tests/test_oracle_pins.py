"""Pins for the CPU oracle: every function of oracle/fleet_oracle.c is checked
against something other than itself -- closed forms, invariants, fp64 brute
force in Python loops, and library routines (numpy / torch.nn.functional)."""
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import oracle
import synth_inputs as si


def bf(x):
    """bf16 bits of fp32 values through torch's converter (independent of the oracle)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return si.to_host_u16(t)


def unbf(u):
    return si.bf16_bits_to_f32(np.asarray(u, dtype=np.uint16))


# --------------------------------------------------------------------------- bf16
def test_bf16_rne_ties_and_library():
    # exact ties: 1 + 2^-8 lies halfway between 0x3F80 and 0x3F81 -> even (0x3F80);
    # 1 + 3*2^-8 lies halfway between 0x3F81 and 0x3F82 -> even (0x3F82)
    assert int(oracle.f2bf(np.float32([1.0 + 2.0** -8]))[0]) == 0x3F80
    assert int(oracle.f2bf(np.float32([1.0 + 3 * 2.0 ** -8]))[0]) == 0x3F82
    assert int(oracle.f2bf(np.float32([1.0 + 2.0 ** -8 + 2.0 ** -20]))[0]) == 0x3F81
    assert int(oracle.f2bf(np.float32([-2.5]))[0]) == 0xC020
    rng = np.random.default_rng(0)
    x = (rng.standard_normal(4000) * np.exp(rng.uniform(-20, 20, 4000))).astype(np.float32)
    assert np.array_equal(oracle.f2bf(x), bf(x))
    assert oracle.lib().oracle_bf2f(0x3FC0) == 1.5


# --------------------------------------------------------------------------- linear
def test_linear_brute_force_fp64_tiny():
    rng = np.random.default_rng(1)
    B, K, N = 3, 5, 7
    x = unbf(bf(rng.standard_normal((B, K))))
    wb = bf(rng.standard_normal((N, K)))
    w = unbf(wb)
    ref = np.zeros((B, N))
    for b in range(B):
        for n in range(N):
            s = 0.0
            for k in range(K):
                s += float(x[b, k]) * float(w[n, k])
            ref[b, n] = s
    for flags in (0, oracle.HI, oracle.REVERSE_K):
        y = oracle.linear(x, wb, flags)
        assert y.shape == (B, N)
        np.testing.assert_allclose(y, ref, rtol=0, atol=2e-6)


def test_linear_matches_numpy_fp64_and_orientation():
    rng = np.random.default_rng(2)
    B, K, N = 4, 96, 40      # non-square: a transposed operand cannot pass
    x = unbf(bf(rng.standard_normal((B, K))))
    wb = bf(rng.standard_normal((N, K)) * 0.02)
    ref = x.astype(np.float64) @ unbf(wb).astype(np.float64).T
    np.testing.assert_allclose(oracle.linear(x, wb), ref, rtol=0, atol=1e-5)
    np.testing.assert_allclose(oracle.linear(x, wb, oracle.HI), ref, rtol=0, atol=1e-7)


def test_linear_identity_and_zero():
    rng = np.random.default_rng(3)
    x = unbf(bf(rng.standard_normal((2, 16))))
    assert np.array_equal(oracle.linear(x, bf(np.eye(16))), x)
    assert np.array_equal(oracle.linear(x, bf(np.zeros((8, 16)))), np.zeros((2, 8), np.float32))
    # a single 1 at W[n=2, k=5] picks x[:, 5] into column 2
    w = np.zeros((4, 16), np.float32)
    w[2, 5] = 1.0
    y = oracle.linear(x, bf(w))
    assert np.array_equal(y[:, 2], x[:, 5]) and not y[:, [0, 1, 3]].any()


# --------------------------------------------------------------------------- rmsnorm
def test_rmsnorm_unit_rms_and_scale_invariance():
    rng = np.random.default_rng(4)
    n = 256
    x = rng.standard_normal((3, n)).astype(np.float32) * 3.0
    g = bf(1 + 0.02 * rng.standard_normal(n))
    y = oracle.rmsnorm(x, g, 1e-6, oracle.HI)
    rms = np.sqrt(np.mean((y / unbf(g)) ** 2, axis=-1))
    np.testing.assert_allclose(rms, 1.0, atol=1e-5)
    y2 = oracle.rmsnorm(x * 7.0, g, 1e-6, oracle.HI)
    np.testing.assert_allclose(y2, y, rtol=2e-6, atol=1e-7)
    # rounded mode returns bf16-representable values within half an ulp of hi mode
    yr = oracle.rmsnorm(x, g, 1e-6)
    assert np.array_equal(unbf(bf(yr)), yr)
    assert np.all(np.abs(yr - y) <= np.abs(y) * 2.0 ** -8 + 1e-7)


def test_rmsnorm_eps_inside_root_and_library():
    # x = a everywhere: out = a / sqrt(a^2 + eps) * g ; with a^2 == eps -> g / sqrt(2)
    a = np.float32(1e-3)
    g = bf(np.ones(8))
    y = oracle.rmsnorm(np.full((1, 8), a, np.float32), g, 1e-6, oracle.HI)
    np.testing.assert_allclose(y, 1 / math.sqrt(2), rtol=1e-5)
    assert not oracle.rmsnorm(np.zeros((1, 8), np.float32), g, 1e-6).any()
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 64)).astype(np.float32)
    gg = 1 + 0.02 * rng.standard_normal(64)
    ref = F.rms_norm(torch.tensor(x, dtype=torch.float64), (64,),
                     torch.tensor(unbf(bf(gg)), dtype=torch.float64), 1e-6).numpy()
    np.testing.assert_allclose(oracle.rmsnorm(x, bf(gg), 1e-6, oracle.HI), ref, atol=2e-7)
    np.testing.assert_allclose(oracle.rmsnorm(x, bf(gg), 1e-6), ref, rtol=2.0 ** -8, atol=1e-6)


# --------------------------------------------------------------------------- rope
def _ones_gain(hd):
    return bf(np.ones(hd))


def test_rope_preserves_norm_and_pos0_is_identity():
    rng = np.random.default_rng(6)
    hd = 128
    t = rng.standard_normal(hd).astype(np.float32)
    base = oracle.head_norm_rope(t, _ones_gain(hd), 1e-6, 1e6, 0, oracle.HI)
    # position 0: rotation is the identity, what is left is the per-head RMSNorm
    np.testing.assert_allclose(base, t / np.sqrt(np.mean(t.astype(np.float64) ** 2) + 1e-6),
                               rtol=1e-6)
    for pos in (1, 17, 1024, 4096):
        r = oracle.head_norm_rope(t, _ones_gain(hd), 1e-6, 1e6, pos, oracle.HI)
        np.testing.assert_allclose(np.linalg.norm(r), np.linalg.norm(base), rtol=1e-6)
        r32 = oracle.head_norm_rope(t, _ones_gain(hd), 1e-6, 1e6, pos)
        np.testing.assert_allclose(r32, r, atol=2e-6)


def test_rope_half_split_pairing_and_angles():
    hd = 4
    # unit energy in element 0 only (norm leaves direction alone: rms -> sqrt(hd) scale)
    t = np.array([1, 0, 0, 0], np.float32)
    r = oracle.head_norm_rope(t, _ones_gain(hd), 0.0, 10000.0, 1, oracle.HI)
    s = math.sqrt(hd)
    # pair (0, 2) rotates by angle 1 * theta^0 = 1 rad; elements 1 and 3 stay 0
    np.testing.assert_allclose(r, [s * math.cos(1), 0, s * math.sin(1), 0], atol=1e-6)
    t = np.array([0, 1, 0, 0], np.float32)
    r = oracle.head_norm_rope(t, _ones_gain(hd), 0.0, 10000.0, 3, oracle.HI)
    # pair (1, 3): angle = 3 * 10000^(-2*1/4) = 3 * 0.01
    np.testing.assert_allclose(r, [0, s * math.cos(0.03), 0, s * math.sin(0.03)], atol=1e-6)


def test_rope_complex_formulation_and_relative_property():
    rng = np.random.default_rng(7)
    hd, theta = 128, 1e6
    q = rng.standard_normal(hd).astype(np.float32)
    k = rng.standard_normal(hd).astype(np.float32)
    ones = _ones_gain(hd)

    def via_complex(t, pos):
        # textbook: pair (i, i + hd/2) is the complex number t_i + j t_{i+hd/2},
        # multiplied by exp(j * pos * theta^(-2i/hd))
        tn = t.astype(np.float64) / np.sqrt(np.mean(t.astype(np.float64) ** 2) + 1e-6)
        z = torch.complex(torch.tensor(tn[: hd // 2]), torch.tensor(tn[hd // 2:]))
        ang = pos * torch.pow(torch.tensor(theta, dtype=torch.float64),
                              -torch.arange(0, hd, 2, dtype=torch.float64) / hd)
        z = z * torch.polar(torch.ones_like(ang), ang)
        return np.concatenate([z.real.numpy(), z.imag.numpy()])

    for pos in (5, 1000):
        np.testing.assert_allclose(oracle.head_norm_rope(q, ones, 1e-6, theta, pos, oracle.HI),
                                   via_complex(q, pos), atol=1e-6)
    d = []
    for p, pp in ((10, 3), (110, 103), (1010, 1003)):
        a = oracle.head_norm_rope(q, ones, 1e-6, theta, p, oracle.HI).astype(np.float64)
        b = oracle.head_norm_rope(k, ones, 1e-6, theta, pp, oracle.HI).astype(np.float64)
        d.append(a @ b)
    np.testing.assert_allclose(d, d[0], rtol=0, atol=2e-4)


def test_head_norm_uses_gain():
    rng = np.random.default_rng(8)
    hd = 128
    t = rng.standard_normal(hd).astype(np.float32)
    g = 1 + 0.02 * rng.standard_normal(hd)
    a = oracle.head_norm_rope(t, bf(g), 1e-6, 1e6, 0, oracle.HI)
    b = oracle.head_norm_rope(t, _ones_gain(hd), 1e-6, 1e6, 0, oracle.HI)
    np.testing.assert_allclose(a, b * unbf(bf(g)), rtol=1e-6)


# --------------------------------------------------------------------------- attention
def test_softmax_rows_sum_to_one_and_shift_invariance():
    rng = np.random.default_rng(9)
    s = rng.standard_normal(777).astype(np.float32) * 5
    p = oracle.softmax(s)
    assert abs(float(p.astype(np.float64).sum()) - 1.0) < 1e-5
    assert np.all(p >= 0)
    np.testing.assert_allclose(oracle.softmax(s + 100.0), p, rtol=2e-4, atol=1e-9)
    np.testing.assert_allclose(p, torch.softmax(torch.tensor(s, dtype=torch.float64), 0).numpy(),
                               rtol=1e-5)


def test_attention_special_cases():
    rng = np.random.default_rng(10)
    hd = 128
    q = unbf(bf(rng.standard_normal(hd)))
    K = bf(rng.standard_normal((9, hd)))
    V = bf(rng.standard_normal((9, hd)))
    # one key: the output is V[0] exactly
    assert np.array_equal(oracle.attend_head(q, K[:1], V[:1]), unbf(V[0]))
    # identical keys: uniform weights -> mean of V
    Ks = np.repeat(K[:1], 9, axis=0)
    np.testing.assert_allclose(oracle.attend_head(q, Ks, V), unbf(V).mean(0), atol=1e-6)
    # scale 1/sqrt(hd): two keys, q.k0 = hd * a, k1 = 0 -> weights softmax([a*sqrt(hd), 0])
    qq = np.full(hd, 0.5, np.float32)
    kk = np.zeros((2, hd), np.float32)
    kk[0] = 0.25
    w0 = 1 / (1 + math.exp(-(0.5 * 0.25 * hd) / math.sqrt(hd)))
    vv = np.zeros((2, hd), np.float32)
    vv[0], vv[1] = 1.0, -1.0
    np.testing.assert_allclose(oracle.attend_head(qq, bf(kk), bf(vv)), w0 - (1 - w0), atol=1e-6)


def test_attention_matches_library_sdpa_fp64():
    rng = np.random.default_rng(11)
    hd, n = 128, 333
    q = unbf(bf(rng.standard_normal(hd)))
    K, V = bf(rng.standard_normal((n, hd))), bf(rng.standard_normal((n, hd)))
    ref = F.scaled_dot_product_attention(
        torch.tensor(q, dtype=torch.float64)[None, None, None],
        torch.tensor(unbf(K), dtype=torch.float64)[None, None],
        torch.tensor(unbf(V), dtype=torch.float64)[None, None])[0, 0, 0].numpy()
    np.testing.assert_allclose(oracle.attend_head(q, K, V, oracle.HI), ref, atol=1e-7)
    np.testing.assert_allclose(oracle.attend_head(q, K, V), ref, atol=5e-6)


def test_split_kv_merge_equals_unsplit():
    # a log-sum-exp merge of per-chunk partial results must reproduce the unsplit
    # output: this is the property the split-KV GPU path relies on.
    rng = np.random.default_rng(12)
    hd, n = 128, 200
    q = unbf(bf(rng.standard_normal(hd)))
    K, V = bf(rng.standard_normal((n, hd))), bf(rng.standard_normal((n, hd)))
    full = oracle.attend_head(q, K, V, oracle.HI).astype(np.float64)
    kf = unbf(K).astype(np.float64)
    parts = []
    for lo, hi in ((0, 64), (64, 128), (128, 200)):
        o = oracle.attend_head(q, K[lo:hi], V[lo:hi], oracle.HI).astype(np.float64)
        s = kf[lo:hi] @ q.astype(np.float64) / math.sqrt(hd)
        m = s.max()
        parts.append((m, np.exp(s - m).sum(), o))
    M = max(p[0] for p in parts)
    num = sum(np.exp(m - M) * l * o for m, l, o in parts)
    den = sum(np.exp(m - M) * l for m, l, o in parts)
    np.testing.assert_allclose(num / den, full, atol=1e-6)


# --------------------------------------------------------------------------- swiglu
def test_swiglu_values():
    ffn = 4
    gu = np.zeros((1, 2 * ffn), np.float32)
    gu[0, :ffn] = [0.0, 1.0, 30.0, -30.0]
    gu[0, ffn:] = [5.0, 2.0, 0.5, 3.0]
    h = oracle.swiglu(gu, ffn, oracle.HI)[0]
    assert h[0] == 0.0
    np.testing.assert_allclose(h[1], 2.0 * 0.7310585786300049, rtol=1e-6)
    np.testing.assert_allclose(h[2], 15.0, rtol=1e-6)       # silu(z) -> z for large z
    assert abs(h[3]) < 1e-10                                 # silu(z) -> 0 for very negative z
    rng = np.random.default_rng(13)
    gu = rng.standard_normal((3, 2 * 32)).astype(np.float32) * 2
    ref = (F.silu(torch.tensor(gu[:, :32], dtype=torch.float64)) *
           torch.tensor(gu[:, 32:], dtype=torch.float64)).numpy()
    np.testing.assert_allclose(oracle.swiglu(gu, 32, oracle.HI), ref, atol=1e-6)
    r = oracle.swiglu(gu, 32)
    assert np.array_equal(unbf(bf(r)), r)
    np.testing.assert_allclose(r, ref, rtol=2.0 ** -8, atol=1e-6)


# --------------------------------------------------------------------------- whole step
def _tiny(seed=20, n_layers=2, B=3, vocab=64):
    sh = si.Shape(n_layers=n_layers, hidden=64, n_q_heads=4, n_kv_heads=2, head_dim=16,
                  ffn=96, vocab=vocab, max_batch=B, max_seq=12)
    g = si.Gen(seed)
    w = si.make_weights(sh, g, with_embed=True)
    # larger matrix std than the recipe so that every branch matters in a 64-wide model
    for k in ("wqkv", "wo", "wgu", "wdown"):
        w[k] = [g.normal_bf16(tuple(a.shape), 0.2) for a in w[k]]
    hid = si.make_hidden(sh, B, g)
    kc, vc = si.make_kv_cache(sh, g)
    pos = np.array([5, 0, 11][:B], np.int32)
    return sh, w, hid, kc, vc, pos


def _torch_step(sh, w, hid, kc, vc, pos):
    """The decode step composed from torch library routines in fp64."""
    f64 = lambda t: t.to(torch.float64)
    B = hid.shape[0]
    hd, nq, nkv = sh.head_dim, sh.n_q_heads, sh.n_kv_heads
    kc, vc = f64(kc).clone(), f64(vc).clone()
    x = f64(hid)
    inv = torch.pow(torch.tensor(sh.rope_theta, dtype=torch.float64),
                    -torch.arange(0, hd, 2, dtype=torch.float64) / hd)

    def rope(t, p):            # t [..., hd]
        z = torch.complex(t[..., : hd // 2], t[..., hd // 2:]) * \
            torch.polar(torch.ones_like(inv), p * inv)
        return torch.cat([z.real, z.imag], -1)

    for l in range(sh.n_layers):
        n = F.rms_norm(x, (sh.hidden,), f64(w["ln1"][l]), sh.rms_eps)
        qkv = F.linear(n, f64(w["wqkv"][l]))
        att = torch.zeros(B, nq * hd, dtype=torch.float64)
        for b in range(B):
            p = int(pos[b])
            q = qkv[b, : nq * hd].view(nq, hd)
            k = qkv[b, nq * hd: (nq + nkv) * hd].view(nkv, hd)
            v = qkv[b, (nq + nkv) * hd:].view(nkv, hd)
            q = rope(F.rms_norm(q, (hd,), f64(w["q_norm"][l]), sh.rms_eps), p)
            k = rope(F.rms_norm(k, (hd,), f64(w["k_norm"][l]), sh.rms_eps), p)
            # the cache stores bf16: the new token's k, v are rounded on the way in
            kc[l, b, :, p] = k.to(torch.bfloat16).to(torch.float64)
            vc[l, b, :, p] = v.to(torch.bfloat16).to(torch.float64)
            o = F.scaled_dot_product_attention(q[None, :, None, :], kc[l, b, :, : p + 1][None],
                                               vc[l, b, :, : p + 1][None], enable_gqa=True)
            att[b] = o.reshape(-1)
        x = x + F.linear(att, f64(w["wo"][l]))
        n = F.rms_norm(x, (sh.hidden,), f64(w["ln2"][l]), sh.rms_eps)
        gu = F.linear(n, f64(w["wgu"][l]))
        x = x + F.linear(F.silu(gu[:, : sh.ffn]) * gu[:, sh.ffn:], f64(w["wdown"][l]))
    logits = F.linear(F.rms_norm(x, (sh.hidden,), f64(w["final_norm"]), sh.rms_eps),
                      f64(w["lm_head"]))
    return x.numpy(), logits.numpy(), kc.numpy(), vc.numpy()


def _run_oracle(sh, w, hid, kc, vc, pos, flags=0, B=None, tokens=None):
    wh = si.weights_to_host(w)
    k, v = si.to_host_u16(kc).copy(), si.to_host_u16(vc).copy()
    B = hid.shape[0] if B is None else B
    ho, lg = oracle.decode_step(sh.asdict(), wh, B, pos, k, v,
                                hidden_in=None if tokens is not None else si.to_host_u16(hid),
                                tokens=tokens, flags=flags)
    return ho, lg, k, v


def test_decode_step_matches_torch_library_composition():
    sh, w, hid, kc, vc, pos = _tiny()
    rx, rl, rk, rv = _torch_step(sh, w, hid, kc, vc, pos)
    ho, lg, k, v = _run_oracle(sh, w, hid, kc, vc, pos, oracle.HI)
    np.testing.assert_allclose(ho, rx, atol=5e-5 * np.abs(rx).max())
    np.testing.assert_allclose(lg, rl, atol=5e-5 * np.abs(rl).max())
    # the cache holds bf16(k), bf16(v) of the new token at slot pos, all else untouched
    np.testing.assert_allclose(unbf(k), rk, rtol=2.0 ** -7, atol=1e-6)
    np.testing.assert_allclose(unbf(v), rv, rtol=2.0 ** -7, atol=1e-6)
    k0, v0 = si.to_host_u16(kc), si.to_host_u16(vc)
    changed = np.zeros(k.shape[:4], bool)
    for b in range(len(pos)):
        changed[:, b, :, pos[b]] = True
    assert np.array_equal(k[~changed], k0[~changed]) and np.array_equal(v[~changed], v0[~changed])
    assert (k[changed] != k0[changed]).any()
    # the rounded (bf16 intermediates, fp32 accumulation) mode stays close to it
    ho2, lg2, _, _ = _run_oracle(sh, w, hid, kc, vc, pos, 0)
    # (bf16 rounding of the intermediates: a few 2^-9-relative errors per layer)
    assert np.abs(ho2 - rx).max() <= 5e-2 * np.sqrt(np.mean(rx ** 2))
    assert np.abs(lg2 - rl).max() <= 5e-2 * np.sqrt(np.mean(rl ** 2))
    ho3, lg3, _, _ = _run_oracle(sh, w, hid, kc, vc, pos, oracle.REVERSE_K)
    assert np.abs(ho3 - ho2).max() <= 2e-2 * np.sqrt(np.mean(rx ** 2))


def _torch_step_rounded(sh, w, hid, kc, vc, pos, drop=None):
    """The fp64 torch composition with values rounded to bf16 wherever a tensor crosses an
    operator boundary (paper section 2.2, the operators of a layer): the three norm outputs, q and
    k after head norm and rotation, v, the attention output, the SwiGLU product.  drop names
    one of those points to leave unrounded."""
    f64 = lambda t: t.to(torch.float64)
    rb = lambda t: t.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    R = lambda name, t: t if drop == name else rb(t)
    B = hid.shape[0]
    hd, nq, nkv = sh.head_dim, sh.n_q_heads, sh.n_kv_heads
    kc, vc = f64(kc).clone(), f64(vc).clone()
    x = f64(hid)
    inv = torch.pow(torch.tensor(sh.rope_theta, dtype=torch.float64),
                    -torch.arange(0, hd, 2, dtype=torch.float64) / hd)

    def rope(t, p):
        z = torch.complex(t[..., : hd // 2], t[..., hd // 2:]) * \
            torch.polar(torch.ones_like(inv), p * inv)
        return torch.cat([z.real, z.imag], -1)

    for l in range(sh.n_layers):
        n = R("ln1", F.rms_norm(x, (sh.hidden,), f64(w["ln1"][l]), sh.rms_eps))
        qkv = F.linear(n, f64(w["wqkv"][l]))
        att = torch.zeros(B, nq * hd, dtype=torch.float64)
        for b in range(B):
            p = int(pos[b])
            q = qkv[b, : nq * hd].view(nq, hd)
            k = qkv[b, nq * hd: (nq + nkv) * hd].view(nkv, hd)
            v = qkv[b, (nq + nkv) * hd:].view(nkv, hd)
            q = R("q", rope(F.rms_norm(q, (hd,), f64(w["q_norm"][l]), sh.rms_eps), p))
            kc[l, b, :, p] = rb(rope(F.rms_norm(k, (hd,), f64(w["k_norm"][l]), sh.rms_eps), p))
            vc[l, b, :, p] = rb(v)
            o = F.scaled_dot_product_attention(q[None, :, None, :], kc[l, b, :, : p + 1][None],
                                               vc[l, b, :, : p + 1][None], enable_gqa=True)
            att[b] = o.reshape(-1)
        x = x + F.linear(R("att", att), f64(w["wo"][l]))
        n = R("ln2", F.rms_norm(x, (sh.hidden,), f64(w["ln2"][l]), sh.rms_eps))
        gu = F.linear(n, f64(w["wgu"][l]))
        x = x + F.linear(R("swiglu", F.silu(gu[:, : sh.ffn]) * gu[:, sh.ffn:]), f64(w["wdown"][l]))
    nf = R("final", F.rms_norm(x, (sh.hidden,), f64(w["final_norm"]), sh.rms_eps))
    return x.numpy(), F.linear(nf, f64(w["lm_head"])).numpy(), kc.numpy(), vc.numpy()


@pytest.mark.parametrize("seed", [20, 21])
def test_rounding_points_of_the_decode_step(seed):
    """Where the oracle rounds to bf16 (its header: every tensor that crosses an operator
    boundary) is pinned against the fp64 composition rounded at the same points: the two agree
    to fp32 accumulation error and the new cache entries of every layer are the same bits, while
    leaving out any single rounding point moves the result a thousand times further."""
    sh, w, hid, kc, vc, pos = _tiny(seed=seed, n_layers=3)
    ho, lg, k, v = _run_oracle(sh, w, hid, kc, vc, pos, 0)
    changed = np.zeros(k.shape[:4], bool)
    for b in range(len(pos)):
        changed[:, b, :, pos[b]] = True
    rms = lambda a: np.sqrt(np.mean(a ** 2))
    rx, rl, rk, rv = _torch_step_rounded(sh, w, hid, kc, vc, pos)
    assert np.abs(ho - rx).max() <= 1e-5 * rms(rx)
    assert np.abs(lg - rl).max() <= 1e-5 * rms(rl)
    assert np.mean(unbf(k)[changed] == rk[changed]) >= 0.99
    assert np.mean(unbf(v)[changed] == rv[changed]) >= 0.99
    for drop in ("ln1", "q", "att", "ln2", "swiglu", "final"):
        dx, dl, _, _ = _torch_step_rounded(sh, w, hid, kc, vc, pos, drop)
        assert np.abs(lg - dl).max() >= 1e-3 * rms(rl), drop
        if drop != "final":
            assert np.abs(ho - dx).max() >= 1e-3 * rms(rx), drop


def test_rows_are_independent_bit_exact():
    sh, w, hid, kc, vc, pos = _tiny(B=3)
    ho, lg, k, v = _run_oracle(sh, w, hid, kc, vc, pos)
    for b in range(3):
        sh1 = si.Shape(**{**sh.asdict(), "max_batch": 1})
        ho1, lg1, k1, v1 = _run_oracle(sh1, w, hid[b:b + 1], kc[:, b:b + 1].contiguous(),
                                       vc[:, b:b + 1].contiguous(), pos[b:b + 1])
        assert np.array_equal(ho1[0], ho[b]) and np.array_equal(lg1[0], lg[b])
        assert np.array_equal(k1[:, 0], k[:, b]) and np.array_equal(v1[:, 0], v[:, b])


def test_gqa_head_mapping_and_causal_window():
    sh, w, hid, kc, vc, pos = _tiny(n_layers=1, B=1)
    sh = si.Shape(**{**sh.asdict(), "max_batch": 1})
    kc, vc, hid, pos = kc[:, :1].contiguous(), vc[:, :1].contiguous(), hid[:1], pos[:1]
    p = int(pos[0])
    # with W_o = "pick q-head h's output into the first head_dim columns" the step's
    # hidden_out exposes one head; perturbing the other KV head must not change it
    hd, nq = sh.head_dim, sh.n_q_heads
    for h, other_g in ((0, 1), (1, 1), (2, 0), (3, 0)):   # 4 q heads, 2 kv heads: g = h // 2
        wo = torch.zeros(sh.hidden, nq * hd)
        wo[:hd, h * hd:(h + 1) * hd] = torch.eye(hd)
        w2 = dict(w)
        w2["wo"] = [wo.to(torch.bfloat16)]
        w2["wdown"] = [torch.zeros_like(w["wdown"][0])]
        base, _, _, _ = _run_oracle(sh, w2, hid, kc, vc, pos)
        vc2 = vc.clone()
        vc2[0, 0, other_g, :p] += 1.0
        pert, _, _, _ = _run_oracle(sh, w2, hid, kc, vc2, pos)
        assert np.array_equal(base, pert)
        vc3 = vc.clone()
        vc3[0, 0, 1 - other_g, :p] += 1.0
        assert not np.array_equal(base, _run_oracle(sh, w2, hid, kc, vc3, pos)[0])
        # slots above pos are never read; slot pos-1 is
        vc4 = vc.clone()
        vc4[0, 0, :, p + 1:] += 9.0
        assert np.array_equal(base, _run_oracle(sh, w2, hid, kc, vc4, pos)[0])


def test_zero_output_weights_pass_residual_through():
    sh, w, hid, kc, vc, pos = _tiny(n_layers=2, B=2)
    w2 = dict(w)
    w2["wo"] = [torch.zeros_like(a) for a in w["wo"]]
    w2["wdown"] = [torch.zeros_like(a) for a in w["wdown"]]
    ho, _, _, _ = _run_oracle(sh, w2, hid, kc, vc, pos[:2], B=2)
    assert np.array_equal(ho, unbf(si.to_host_u16(hid))[:2])


def test_embedding_gather_path():
    sh, w, hid, kc, vc, pos = _tiny(B=2)
    tok = np.array([7, 63], np.int32)
    a = _run_oracle(sh, w, hid, kc, vc, pos[:2], B=2, tokens=tok)
    b = _run_oracle(sh, w, w["embed"][tok.tolist()].contiguous(), kc, vc, pos[:2], B=2)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_rejects_bad_arguments():
    sh, w, hid, kc, vc, pos = _tiny(B=2)
    with pytest.raises(ValueError):
        _run_oracle(sh, w, hid, kc, vc, np.array([0, sh.max_seq], np.int32), B=2)


def test_layer_range_chaining_reproduces_whole_step():
    sh, w, hid, kc, vc, pos = _tiny(n_layers=3, B=2)
    wh = si.weights_to_host(w)
    k, v = si.to_host_u16(kc).copy(), si.to_host_u16(vc).copy()
    ho, lg, tr = oracle.decode_step(sh.asdict(), wh, 2, pos[:2], k, v,
                                    hidden_in=si.to_host_u16(hid)[:2], want_trace=True)
    assert np.array_equal(tr[0], unbf(si.to_host_u16(hid))[:2]) and np.array_equal(tr[-1], ho)
    k2, v2 = si.to_host_u16(kc).copy(), si.to_host_u16(vc).copy()
    x = tr[0]
    for l in range(3):
        x, lg2 = oracle.decode_layers(sh.asdict(), wh, 2, l, l + 1, x, pos[:2], k2, v2,
                                      want_logits=True)
        assert np.array_equal(x, tr[l + 1])
    assert np.array_equal(lg2, lg) and np.array_equal(k2, k) and np.array_equal(v2, v)
