"""ctypes binding over libfleet.so: argument marshalling only.

Function names mirror the C ABI of ``include/fleet.h``.  Device buffers may be
passed as torch tensors (their ``data_ptr()`` is taken) or as integer addresses.
The library is loaded from the package directory; if it has not been built the
import of the first symbol raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libfleet.so")

SCHED_COOPERATIVE, SCHED_UNAWARE, SCHED_MSPLIT = 0, 1, 2
FLAG_TRACE, FLAG_SINGLE_LEVEL, FLAG_SEPARATE_NORM, FLAG_CHAINED, FLAG_TIMING = 1, 2, 4, 8, 16
FLAG_NO_SPLITK, FLAG_NO_STREAM, FLAG_NO_RESIDENT, FLAG_UNFUSED_SILU = 32, 64, 128, 256
FLAG_PACKED_ONLY, FLAG_NT_STORES = 1024, 2048
STATIC_SCRATCH_BYTES = 32 << 20

EXPORTS = (
    "fleet_create", "fleet_decode_step", "fleet_decode_step_paged", "fleet_decode_layers",
    "fleet_decode_tokens", "fleet_destroy", "fleet_decode_step_static",
    "fleet_gemm",
    "fleet_graph_build", "fleet_graph_dump", "fleet_trace_read", "fleet_last_status",
    "fleet_device_probe", "fleet_copy", "fleet_weight_bytes", "fleet_weight_bytes_per_xcd",
    "fleet_l2_window_bytes", "fleet_l2_hit_model", "fleet_effective_intensity",
    "fleet_step_bytes", "fleet_strerror",
)


class FleetError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {fleet_strerror(code)} (code {code})")


class ShapeStruct(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads",
                                         "head_dim", "ffn", "vocab", "max_batch", "max_seq")] + \
               [("rms_eps", C.c_float), ("rope_theta", C.c_float)] + \
               [(n, C.c_int32) for n in ("sched_mode", "tile_m", "flags")]


_PP = C.POINTER(C.c_void_p)


class WeightsStruct(C.Structure):
    _fields_ = [("embed", C.c_void_p)] + \
               [(n, _PP) for n in ("ln1", "wqkv", "q_norm", "k_norm", "wo", "ln2", "wgu", "wdown")] + \
               [("final_norm", C.c_void_p), ("lm_head", C.c_void_p)]


class StatusStruct(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("code", "hip_error", "task", "event", "observed",
                                         "needed", "n_xcd")] + [("workers", C.c_int32 * 8)]


_lib = None


def load_library():
    """dlopen libfleet.so (built by ``paper_2604_15379_amd.build.build()``)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: run __graft_entry__.build() "
                          "(python -c 'import __graft_entry__ as g; g.build()') first")
    lib = C.CDLL(_LIB_PATH)
    lib.fleet_strerror.restype = C.c_char_p
    lib.fleet_strerror.argtypes = [C.c_int]
    for n in ("fleet_weight_bytes", "fleet_weight_bytes_per_xcd", "fleet_l2_window_bytes",
              "fleet_step_bytes"):
        getattr(lib, n).restype = C.c_int64
    lib.fleet_weight_bytes.argtypes = [C.c_int32, C.c_int32]
    lib.fleet_weight_bytes_per_xcd.argtypes = [C.c_int32] * 3
    lib.fleet_l2_window_bytes.argtypes = [C.c_int32] * 4
    lib.fleet_l2_hit_model.restype = C.c_double
    lib.fleet_l2_hit_model.argtypes = [C.c_int32] * 3
    lib.fleet_effective_intensity.restype = C.c_double
    lib.fleet_effective_intensity.argtypes = [C.c_int32, C.c_double]
    _lib = lib
    return lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _shape_struct(shape: dict, sched_mode=0, tile_m=0, flags=0) -> ShapeStruct:
    d = dict(shape)
    d.setdefault("sched_mode", sched_mode)
    d.setdefault("tile_m", tile_m)
    d.setdefault("flags", flags)
    return ShapeStruct(**{k: d[k] for k, _ in ShapeStruct._fields_})


def fleet_strerror(code: int) -> str:
    return load_library().fleet_strerror(int(code)).decode()


class Fleet:
    """Handle returned by fleet_create (keeps the weight tensors alive)."""

    def __init__(self, handle, shape, keep):
        self.handle, self.shape, self._keep = handle, shape, keep


def fleet_create(shape: dict, weights: dict, sched_mode=0, tile_m=0, flags=0) -> Fleet:
    lib = load_library()
    sh = _shape_struct(shape, sched_mode, tile_m, flags)
    w = WeightsStruct()
    keep = [weights]
    for name in ("ln1", "wqkv", "q_norm", "k_norm", "wo", "ln2", "wgu", "wdown"):
        arr = (C.c_void_p * sh.n_layers)(*[t.data_ptr() for t in weights[name]])
        keep.append(arr)
        setattr(w, name, C.cast(arr, _PP))
    for name in ("embed", "final_norm", "lm_head"):
        t = weights.get(name)
        if t is not None:
            setattr(w, name, t.data_ptr())
    out = C.c_void_p()
    rc = lib.fleet_create(C.byref(sh), C.byref(w), C.byref(out))
    if rc != 0:
        raise FleetError(rc, "fleet_create")
    return Fleet(out, sh, keep)


def fleet_decode_step(f: Fleet, batch: int, hidden_in, tokens, k_cache, v_cache, positions,
                      hidden_out, logits, stream=0) -> None:
    rc = load_library().fleet_decode_step(f.handle, C.c_int32(batch), _ptr(hidden_in), _ptr(tokens),
                                          _ptr(k_cache), _ptr(v_cache), _ptr(positions),
                                          _ptr(hidden_out), _ptr(logits), C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_decode_step")


def fleet_decode_step_static(f: Fleet, batch: int, hidden_in, tokens, k_cache, v_cache, positions,
                             hidden_out, logits, stream=0) -> None:
    rc = load_library().fleet_decode_step_static(f.handle, C.c_int32(batch), _ptr(hidden_in), _ptr(tokens),
                                                 _ptr(k_cache), _ptr(v_cache), _ptr(positions),
                                                 _ptr(hidden_out), _ptr(logits), C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_decode_step_static")


def fleet_decode_layers(f: Fleet, batch: int, layer_begin: int, layer_end: int, x_in, k_cache,
                        v_cache, positions, x_out, logits=None, stream=0) -> None:
    rc = load_library().fleet_decode_layers(f.handle, C.c_int32(batch), C.c_int32(layer_begin),
                                            C.c_int32(layer_end), _ptr(x_in), _ptr(k_cache),
                                            _ptr(v_cache), _ptr(positions), _ptr(x_out),
                                            _ptr(logits), C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_decode_layers")


def fleet_decode_step_paged(f: Fleet, batch: int, hidden_in, tokens, k_pool, v_pool, page_table,
                            page_size: int, n_pages: int, table_stride: int, positions, hidden_out,
                            logits=None, stream=0) -> None:
    rc = load_library().fleet_decode_step_paged(
        f.handle, C.c_int32(batch), _ptr(hidden_in), _ptr(tokens), _ptr(k_pool), _ptr(v_pool),
        _ptr(page_table), C.c_int32(page_size), C.c_int32(n_pages), C.c_int32(table_stride),
        _ptr(positions), _ptr(hidden_out), _ptr(logits), C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_decode_step_paged")


def fleet_decode_tokens(f: Fleet, batch: int, tokens, k_cache, v_cache, positions, n_tokens: int,
                        tokens_out, hidden_out, logits, stream=0) -> None:
    rc = load_library().fleet_decode_tokens(f.handle, C.c_int32(batch), _ptr(tokens), _ptr(k_cache),
                                            _ptr(v_cache), _ptr(positions), C.c_int32(n_tokens),
                                            _ptr(tokens_out), _ptr(hidden_out), _ptr(logits),
                                            C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_decode_tokens")


def fleet_destroy(f: Fleet) -> None:
    if f is not None and f.handle:
        load_library().fleet_destroy(f.handle)
        f.handle = None


def fleet_gemm(B: int, K: int, N: int, x, w_copies, y, sched_mode=0, tile_m=0, flags=0, reps=1,
               stream=0) -> float:
    """Returns the kernel time in milliseconds."""
    arr = (C.c_void_p * len(w_copies))(*[t if isinstance(t, int) else t.data_ptr() for t in w_copies])
    ms = C.c_float(0)
    rc = load_library().fleet_gemm(C.c_int32(B), C.c_int32(K), C.c_int32(N), _ptr(x),
                                   C.cast(arr, _PP), C.c_int32(len(w_copies)), _ptr(y),
                                   C.c_int32(sched_mode), C.c_int32(tile_m), C.c_int32(flags),
                                   C.c_int32(reps), C.c_void_p(stream), C.byref(ms))
    if rc != 0:
        raise FleetError(rc, "fleet_gemm")
    return float(ms.value)


def _sized_call(fn, *args) -> np.ndarray:
    n = C.c_size_t(0)
    rc = fn(*args, None, C.byref(n))
    if rc != 0:
        raise FleetError(rc, fn.__name__)
    buf = np.empty(n.value // 4, np.int32)
    rc = fn(*args, buf.ctypes.data_as(C.c_void_p), C.byref(n))
    if rc != 0:
        raise FleetError(rc, fn.__name__)
    return buf[: n.value // 4]


def fleet_graph_build(shape: dict, batch: int, n_xcd: int = 8, n_workers: int = 256,
                      sched_mode=0, tile_m=0, flags=0) -> np.ndarray:
    sh = _shape_struct(shape, sched_mode, tile_m, flags)
    return _sized_call(load_library().fleet_graph_build, C.byref(sh), C.c_int32(batch),
                       C.c_int32(n_xcd), C.c_int32(n_workers))


def fleet_graph_dump(f: Fleet, batch: int) -> np.ndarray:
    return _sized_call(load_library().fleet_graph_dump, f.handle, C.c_int32(batch))


def fleet_trace_read(f: Fleet) -> np.ndarray:
    """[n_records, 8] int32: task, worker, xcd, t_enter, ticket0, ticket1, t0, t1."""
    return _sized_call(load_library().fleet_trace_read, f.handle).reshape(-1, 8)


def fleet_last_status(f: Fleet) -> dict:
    st = StatusStruct()
    rc = load_library().fleet_last_status(f.handle, C.byref(st))
    if rc != 0:
        raise FleetError(rc, "fleet_last_status")
    d = {k: getattr(st, k) for k, _ in StatusStruct._fields_ if k != "workers"}
    d["workers"] = list(st.workers)
    return d


def fleet_device_probe(n_blocks: int) -> np.ndarray:
    out = np.empty(n_blocks, np.int32)
    rc = load_library().fleet_device_probe(C.c_int32(n_blocks), out.ctypes.data_as(C.c_void_p))
    if rc != 0:
        raise FleetError(rc, "fleet_device_probe")
    return out


def fleet_copy(dst, src, nbytes: int, stream=0) -> None:
    rc = load_library().fleet_copy(_ptr(dst), _ptr(src), C.c_size_t(nbytes), C.c_void_p(stream))
    if rc != 0:
        raise FleetError(rc, "fleet_copy")


def fleet_weight_bytes(K, N):
    return int(load_library().fleet_weight_bytes(K, N))


def fleet_weight_bytes_per_xcd(K, N, n_xcd=8):
    return int(load_library().fleet_weight_bytes_per_xcd(K, N, n_xcd))


def fleet_l2_window_bytes(N, n_xcd=8, tile_n=64, tile_k=256):
    return int(load_library().fleet_l2_window_bytes(N, n_xcd, tile_n, tile_k))


def fleet_l2_hit_model(batch, tile_m=16, workers_per_xcd=32):
    return float(load_library().fleet_l2_hit_model(batch, tile_m, workers_per_xcd))


def fleet_effective_intensity(batch, l2_hit):
    return float(load_library().fleet_effective_intensity(batch, l2_hit))


def fleet_step_bytes(shape: dict, batch: int, positions) -> int:
    sh = _shape_struct(shape)
    pos = np.ascontiguousarray(positions, dtype=np.int32)
    return int(load_library().fleet_step_bytes(C.byref(sh), C.c_int32(batch),
                                               pos.ctypes.data_as(C.c_void_p)))


# ---------------------------------------------------------------- graph words -> dict
HEADER_WORDS, OP_WORDS, TASK_WORDS, EVENT_WORDS, QENT_WORDS = 32, 16, 16, 4, 4
H_NAMES = ("magic", "version", "n_ops", "n_tasks", "n_events", "n_xcd", "n_qent", "n_layers",
           "batch", "sched", "tile_m", "path", "n_splits", "n_workers", "m_tiles", "total_words")
O_NAMES = ("body", "layer", "epi", "path", "K", "N", "unit_rows", "n_units", "m_tiles", "tile_m",
           "in_buf", "out_buf", "aux", "wkind", "batch", "aux2")
T_NAMES = ("op", "scope", "xcd", "a0", "a1", "a2", "a3", "wait_event", "signal_event", "stage")


def parse_graph(words: np.ndarray) -> dict:
    """Split the serialized int32 words of a task graph into named arrays."""
    w = np.asarray(words, np.int32)
    h = {n: int(w[i]) for i, n in enumerate(H_NAMES)}
    assert h["magic"] == 0x464C5447 and h["total_words"] == w.size, "not a graph dump"
    o = HEADER_WORDS
    ops = w[o:o + h["n_ops"] * OP_WORDS].reshape(-1, OP_WORDS); o += ops.size
    tasks = w[o:o + h["n_tasks"] * TASK_WORDS].reshape(-1, TASK_WORDS); o += tasks.size
    events = w[o:o + h["n_events"] * EVENT_WORDS].reshape(-1, EVENT_WORDS); o += events.size
    qoff = w[o:o + h["n_xcd"] + 1]; o += qoff.size
    qents = w[o:o + h["n_qent"] * QENT_WORDS].reshape(-1, QENT_WORDS); o += qents.size
    n_marks = h["n_layers"] + 4
    marks = w[o:o + h["n_xcd"] * n_marks].reshape(h["n_xcd"], n_marks); o += marks.size
    xready = w[o:]
    return dict(header=h, ops=ops, tasks=tasks, events=events, qoff=qoff, qents=qents,
                marks=marks, xready=xready)
