"""CPU oracle of the Fleet decode step -- TEST INFRASTRUCTURE ONLY.

Thin ctypes binding over ``fleet_oracle.c`` (plain C, fp32 accumulation over
bf16-rounded inputs).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product
package never does.  All arrays are host numpy arrays; bf16 tensors travel as
``uint16`` bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "fleet_oracle.c")
_LIB = os.path.join(_DIR, "libfleet_oracle.so")

HI = 1          # double accumulation, no intermediate bf16 rounding
REVERSE_K = 2   # GEMM reductions summed from the last index down


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Shape(C.Structure):
    _fields_ = [(n, C.c_int32) for n in
                ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn",
                 "vocab", "max_batch", "max_seq")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)]


_PP = C.POINTER(C.c_void_p)


class _Weights(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, _PP) for n in ("ln1", "wqkv", "q_norm", "k_norm", "wo", "ln2",
                                   "wgu", "wdown")] + \
               [("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        _lib = C.CDLL(_LIB)
        _lib.oracle_bf2f.restype = C.c_float
        _lib.oracle_bf2f.argtypes = [C.c_uint16]
        _lib.oracle_f2bf.restype = C.c_uint16
        _lib.oracle_f2bf.argtypes = [C.c_float]
        _lib.oracle_num_threads.restype = C.c_int
        _lib.oracle_decode_step.restype = C.c_int
        _lib.oracle_decode_layers.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def _p(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def f2bf(x) -> np.ndarray:
    """fp32 -> bf16 bits, element by element through the oracle's rounding."""
    x = _f32(x)
    out = np.empty(x.shape, np.uint16)
    L = lib()
    fx, fo = x.reshape(-1), out.reshape(-1)
    for i in range(fx.size):
        fo[i] = L.oracle_f2bf(float(fx[i]))
    return out


def rmsnorm(x, gain_bf16, eps, flags=0):
    x = _f32(x)
    rows, n = x.reshape(-1, x.shape[-1]).shape
    g = _u16(gain_bf16)
    out = np.empty_like(x)
    lib().oracle_rmsnorm(_p(x), _p(g), C.c_int(rows), C.c_int(n), C.c_float(eps),
                         C.c_int(flags), _p(out))
    return out


def linear(x, w_bf16, flags=0):
    """y[b, n] = sum_k x[b, k] * W[n, k]; x fp32 [B, K], W bf16 bits [N, K]."""
    x = _f32(x)
    w = _u16(w_bf16)
    B, K = x.shape
    N, K2 = w.shape
    assert K == K2
    y = np.empty((B, N), np.float32)
    lib().oracle_linear(_p(x), _p(w), C.c_int(B), C.c_int(K), C.c_int(N),
                        C.c_int(flags), _p(y))
    return y


def head_norm_rope(t, gain_bf16, eps, theta, pos, flags=0):
    t = _f32(t).copy()
    g = _u16(gain_bf16)
    lib().oracle_head_norm_rope(_p(t), _p(g), C.c_int(t.shape[-1]), C.c_float(eps),
                                C.c_float(theta), C.c_int(pos), C.c_int(flags))
    return t


def attend_head(q, k_bf16, v_bf16, flags=0):
    q = _f32(q)
    k, v = _u16(k_bf16), _u16(v_bf16)
    n_keys, hd = k.shape
    out = np.empty(hd, np.float32)
    lib().oracle_attend_head(_p(q), _p(k), _p(v), C.c_int(n_keys), C.c_int(hd),
                             C.c_int(flags), _p(out))
    return out


def softmax(s):
    s = _f32(s).copy()
    lib().oracle_softmax(_p(s), C.c_int(s.size))
    return s


def swiglu(gu, ffn, flags=0):
    gu = _f32(gu)
    B = gu.shape[0]
    h = np.empty((B, ffn), np.float32)
    lib().oracle_swiglu(_p(gu), C.c_int(B), C.c_int(ffn), C.c_int(flags), _p(h))
    return h


def _ptr_array(arrs):
    arr = (C.c_void_p * len(arrs))()
    for i, a in enumerate(arrs):
        arr[i] = a.ctypes.data
    return arr


def _marshal(shape, weights, k_cache, v_cache, positions):
    sh = _Shape(**{k: shape[k] for k, _ in _Shape._fields_})
    keep = []
    w = _Weights()
    for name in ("ln1", "wqkv", "q_norm", "k_norm", "wo", "ln2", "wgu", "wdown"):
        arrs = [_u16(a) for a in weights[name]]
        assert len(arrs) == shape["n_layers"]
        pa = _ptr_array(arrs)
        keep += [arrs, pa]
        setattr(w, name, C.cast(pa, _PP))
    for name in ("embed", "final_norm", "lm_head"):
        a = weights.get(name)
        if a is not None:
            a = _u16(a)
            keep.append(a)
            setattr(w, name, a.ctypes.data)
    positions = np.ascontiguousarray(positions, dtype=np.int32)
    assert k_cache.dtype == np.uint16 and k_cache.flags.c_contiguous
    assert v_cache.dtype == np.uint16 and v_cache.flags.c_contiguous
    exp_shape = (shape["n_layers"], shape["max_batch"], shape["n_kv_heads"],
                 shape["max_seq"], shape["head_dim"])
    assert tuple(k_cache.shape) == exp_shape and tuple(v_cache.shape) == exp_shape
    return sh, w, positions, keep


def decode_step(shape: dict, weights: dict, batch: int, positions, k_cache, v_cache,
                hidden_in=None, tokens=None, want_logits=True, want_trace=False, flags=0):
    """One decode step.  ``weights`` maps names to uint16 arrays (per-layer names
    to lists of arrays).  ``k_cache``/``v_cache`` are uint16 arrays of shape
    [n_layers, max_batch, n_kv, max_seq, head_dim], updated in place.
    Returns (hidden_out fp32 [B, hidden], logits fp32 [B, vocab] or None), plus the
    residual stream at every layer boundary [n_layers+1, B, hidden] if want_trace."""
    sh, w, positions, keep = _marshal(shape, weights, k_cache, v_cache, positions)
    hin = None if hidden_in is None else _u16(hidden_in)
    tok = None if tokens is None else np.ascontiguousarray(tokens, dtype=np.int32)
    hout = np.empty((batch, shape["hidden"]), np.float32)
    trace = np.empty((shape["n_layers"] + 1, batch, shape["hidden"]), np.float32) \
        if want_trace else None
    logits = None
    if want_logits and shape["vocab"] > 0:
        logits = np.empty((batch, shape["vocab"]), np.float32)
    rc = lib().oracle_decode_step(C.byref(sh), C.byref(w), C.c_int(batch), _p(hin), _p(tok),
                                  _p(k_cache), _p(v_cache), _p(positions), _p(hout),
                                  _p(trace), _p(logits), C.c_int(flags))
    if rc != 0:
        raise ValueError(f"oracle_decode_step rejected its arguments (rc={rc})")
    return (hout, logits, trace) if want_trace else (hout, logits)


def decode_layers(shape: dict, weights: dict, batch: int, layer_begin: int, layer_end: int,
                  x_in, positions, k_cache, v_cache, want_logits=False, flags=0):
    """Layers [layer_begin, layer_end) on an fp32 residual stream x_in [B, hidden].
    Returns (x_out, logits or None)."""
    sh, w, positions, keep = _marshal(shape, weights, k_cache, v_cache, positions)
    x_in = _f32(x_in)
    assert x_in.shape == (batch, shape["hidden"])
    xout = np.empty_like(x_in)
    logits = None
    if want_logits and shape["vocab"] > 0 and layer_end == shape["n_layers"]:
        logits = np.empty((batch, shape["vocab"]), np.float32)
    rc = lib().oracle_decode_layers(C.byref(sh), C.byref(w), C.c_int(batch),
                                    C.c_int(layer_begin), C.c_int(layer_end), _p(x_in),
                                    _p(k_cache), _p(v_cache), _p(positions), _p(xout), None,
                                    _p(logits), C.c_int(flags))
    if rc != 0:
        raise ValueError(f"oracle_decode_layers rejected its arguments (rc={rc})")
    return xout, logits
