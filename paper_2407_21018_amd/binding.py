"""ctypes binding of libthk.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors on the GPU (or raw integer device addresses); PyTorch
supplies device memory and the HIP stream, nothing else.  There is no fallback:
if the library is missing, loading raises.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libthk.so")

THK_F32, THK_BF16 = 0, 1
THK_OP_SCORE, THK_OP_DECODE, THK_OP_PRUNE, THK_OP_SCORE_VALUE, THK_OP_PRUNE_VALUE = 0, 1, 2, 3, 4


class ThkError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {thk_status_string(status)} (status {int(status)})")


class thk_shape(ctypes.Structure):
    _fields_ = [("L", ctypes.c_int32), ("B", ctypes.c_int32), ("N_q", ctypes.c_int32),
                ("N_kv", ctypes.c_int32), ("D", ctypes.c_int32), ("S", ctypes.c_int64),
                ("S_obs", ctypes.c_int32), ("T", ctypes.c_int32), ("ld_keep", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("n_split", ctypes.c_int32), ("S_recent", ctypes.c_int32),
                ("S_cap", ctypes.c_int64)]


_lib = None


def lib_path():
    return _LIB_PATH


def load():
    """Load libthk.so; raises if it has not been built (no CPU fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(f"{_LIB_PATH} is missing: build it with __graft_entry__.build()")
    # PyTorch's wheel carries its own copy of the HIP runtime.  Loading torch first makes libthk
    # bind to that same copy; loaded the other way round the process ends up with two runtimes
    # and the second one finds no device.
    import torch  # noqa: F401
    L = ctypes.CDLL(_LIB_PATH)
    sp, vp, i32 = ctypes.POINTER(thk_shape), ctypes.c_void_p, ctypes.c_int32
    L.thk_version.restype = i32
    L.thk_version.argtypes = []
    L.thk_reload_env.restype = None
    L.thk_reload_env.argtypes = []
    L.thk_status_string.restype = ctypes.c_char_p
    L.thk_status_string.argtypes = [ctypes.c_int]
    L.thk_last_hip_error.restype = ctypes.c_char_p
    L.thk_last_hip_error.argtypes = []
    L.thk_keep_count.restype = i32
    L.thk_keep_count.argtypes = [i32, ctypes.c_double]
    L.thk_workspace_bytes.restype = ctypes.c_size_t
    L.thk_workspace_bytes.argtypes = [sp, i32]
    L.thk_default_split.restype = i32
    L.thk_default_split.argtypes = [sp, i32]
    L.thk_prune_is_fused.restype = i32
    L.thk_prune_is_fused.argtypes = [sp]
    L.thk_prune_launches.restype = i32
    L.thk_prune_launches.argtypes = [sp]
    L.thk_decode_on_matrix_cores.restype = i32
    L.thk_decode_on_matrix_cores.argtypes = [sp, i32, i32]
    L.thk_score.restype = ctypes.c_int
    L.thk_score.argtypes = [sp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.thk_score_value.restype = ctypes.c_int
    L.thk_score_value.argtypes = [sp, vp, vp, vp, i32, vp, vp, ctypes.c_size_t, vp]
    L.thk_prune_value.restype = ctypes.c_int
    L.thk_prune_value.argtypes = [sp, vp, vp, vp, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.thk_score_magnitude.restype = ctypes.c_int
    L.thk_score_magnitude.argtypes = [sp, vp, i32, vp, vp, ctypes.c_size_t, vp]
    L.thk_select_topk.restype = ctypes.c_int
    L.thk_select_topk.argtypes = [sp, vp, vp, vp]
    L.thk_compact_keys.restype = ctypes.c_int
    L.thk_compact_keys.argtypes = [sp, vp, vp, vp, vp]
    L.thk_prune.restype = ctypes.c_int
    L.thk_prune.argtypes = [sp, vp, vp, vp, vp, vp, vp, ctypes.c_size_t, vp]
    L.thk_decode_attn.restype = ctypes.c_int
    L.thk_decode_attn.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp, ctypes.c_size_t, vp]
    L.thk_decode_attn_static.restype = ctypes.c_int
    L.thk_decode_attn_static.argtypes = [sp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    i64 = ctypes.c_int64
    L.thk_decode_attn_kv.restype = ctypes.c_int
    L.thk_decode_attn_kv.argtypes = [sp, vp, vp, vp, vp, vp, i32, i32, vp, vp, i32, i32, vp, vp,
                                     ctypes.c_size_t, vp]
    L.thk_compact_rows.restype = ctypes.c_int
    L.thk_compact_rows.argtypes = [sp, vp, i64, i64, vp, vp, i64, i64, vp]
    L.thk_copy_rows.restype = ctypes.c_int
    L.thk_copy_rows.argtypes = [sp, vp, i64, i64, vp, i64, i64, i64, vp]
    L.thk_cache_append.restype = ctypes.c_int
    L.thk_cache_append.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp]
    L.thk_tail_flush.restype = ctypes.c_int
    L.thk_tail_flush.argtypes = [sp, vp, vp, vp, vp, vp, i32, i32, i32, vp]
    L.thk_bench_stream.restype = ctypes.c_int
    L.thk_bench_stream.argtypes = [i32, vp, vp, ctypes.c_int64, i32, vp]
    L.thk_profile_next.restype = None
    L.thk_profile_next.argtypes = [vp, vp]
    L.thk_tail_append.restype = ctypes.c_int
    L.thk_tail_append.argtypes = [sp, vp, vp, vp, vp, i32, i32, vp]
    _lib = L
    return L


def make_shape(L, B, N_q, N_kv, D, S, S_obs, T, ld_keep=0, dtype=THK_BF16, n_split=0, S_recent=0, S_cap=0):
    return thk_shape(L, B, N_q, N_kv, D, S, S_obs, T, ld_keep, dtype, n_split, S_recent, S_cap)


def _ptr(x):
    """Device address of a torch tensor (or pass an int / None through)."""
    if x is None:
        return None
    if isinstance(x, int):
        return ctypes.c_void_p(x)
    return ctypes.c_void_p(x.data_ptr())


def _nbytes(ws):
    if ws is None:
        return 0
    if isinstance(ws, tuple):
        return ws[1]
    return ws.numel() * ws.element_size()


def _ws(ws):
    return _ptr(ws[0] if isinstance(ws, tuple) else ws)


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _need(x, n, name, where):
    """Host-side guard: a tensor handed to a kernel must hold at least the n elements
    the shape implies (a short tensor would make the kernel read or write out of bounds)."""
    if x is None or isinstance(x, int):
        return
    if x.numel() < n:
        raise ValueError(f"{where}: {name} holds {x.numel()} elements, the shape needs {n}")
    if not x.is_contiguous():
        raise ValueError(f"{where}: {name} must be contiguous")


def _dims(s):
    U = s.L * s.B * s.N_kv
    H = s.L * s.B * s.N_q
    return U, H, (s.ld_keep or s.T)


def _cache_rows(s, used):
    return s.S_cap or used


def thk_last_hip_error():
    return load().thk_last_hip_error().decode()


def _check(st, where):
    if st == 6:
        raise ThkError(st, f"{where} [{thk_last_hip_error()}]")
    if st != 0:
        raise ThkError(st, where)


def thk_version():
    return int(load().thk_version())


def thk_reload_env():
    """Make the library read its THK_* environment switches again (it reads them once per process)."""
    load().thk_reload_env()


def thk_status_string(st):
    return load().thk_status_string(int(st)).decode()


def thk_keep_count(D, lam):
    return int(load().thk_keep_count(D, lam))


def thk_workspace_bytes(shape, op):
    return int(load().thk_workspace_bytes(ctypes.byref(shape), op))


def thk_default_split(shape, op):
    return int(load().thk_default_split(ctypes.byref(shape), op))


def thk_prune_is_fused(shape):
    return int(load().thk_prune_is_fused(ctypes.byref(shape)))


def thk_prune_launches(shape):
    return int(load().thk_prune_launches(ctypes.byref(shape)))


def thk_decode_on_matrix_cores(shape, T_v=0, ld_v=0):
    return int(load().thk_decode_on_matrix_cores(ctypes.byref(shape), T_v, ld_v))


def thk_score(shape, q_obs, k, score, ws, stream=None):
    U, H, _ = _dims(shape)
    _need(q_obs, H * shape.S_obs * shape.D, "q_obs", "thk_score")
    _need(k, U * shape.S * shape.D, "k", "thk_score")
    _need(score, U * shape.D, "score", "thk_score")
    _check(load().thk_score(ctypes.byref(shape), _ptr(q_obs), _ptr(k), _ptr(score), _ws(ws),
                            _nbytes(ws), _stream(stream)), "thk_score")


def thk_score_value(shape, q_obs, k, v, causal, score_v, ws, stream=None):
    U, H, _ = _dims(shape)
    _need(q_obs, H * shape.S_obs * shape.D, "q_obs", "thk_score_value")
    _need(k, U * shape.S * shape.D, "k", "thk_score_value")
    _need(v, U * shape.S * shape.D, "v", "thk_score_value")
    _need(score_v, U * shape.D, "score_v", "thk_score_value")
    _check(load().thk_score_value(ctypes.byref(shape), _ptr(q_obs), _ptr(k), _ptr(v), int(causal),
                                  _ptr(score_v), _ws(ws), _nbytes(ws), _stream(stream)),
           "thk_score_value")


def thk_prune_value(shape, q_obs, k, v, causal, score_v, idx_v, v_pruned, ws, stream=None):
    U, H, ld = _dims(shape)
    w = "thk_prune_value"
    _need(q_obs, H * shape.S_obs * shape.D, "q_obs", w)
    _need(k, U * shape.S * shape.D, "k", w)
    _need(v, U * shape.S * shape.D, "v", w)
    _need(score_v, U * shape.D, "score_v", w)
    _need(idx_v, U * shape.T, "idx_v", w)
    _need(v_pruned, U * _cache_rows(shape, shape.S - shape.S_recent) * ld, "v_pruned", w)
    _check(load().thk_prune_value(ctypes.byref(shape), _ptr(q_obs), _ptr(k), _ptr(v), int(causal),
                                  _ptr(score_v), _ptr(idx_v), _ptr(v_pruned), _ws(ws), _nbytes(ws),
                                  _stream(stream)), w)


def thk_score_magnitude(shape, k, p, score, ws, stream=None):
    U, _, _ = _dims(shape)
    _need(k, U * shape.S * shape.D, "k", "thk_score_magnitude")
    _need(score, U * shape.D, "score", "thk_score_magnitude")
    _check(load().thk_score_magnitude(ctypes.byref(shape), _ptr(k), p, _ptr(score), _ws(ws),
                                      _nbytes(ws), _stream(stream)), "thk_score_magnitude")


def thk_select_topk(shape, score, idx, stream=None):
    U, _, _ = _dims(shape)
    _need(score, U * shape.D, "score", "thk_select_topk")
    _need(idx, U * shape.T, "idx", "thk_select_topk")
    _check(load().thk_select_topk(ctypes.byref(shape), _ptr(score), _ptr(idx), _stream(stream)),
           "thk_select_topk")


def thk_compact_keys(shape, k, idx, k_pruned, stream=None):
    U, _, ld = _dims(shape)
    _need(k, U * shape.S * shape.D, "k", "thk_compact_keys")
    _need(idx, U * shape.T, "idx", "thk_compact_keys")
    _need(k_pruned, U * _cache_rows(shape, shape.S - shape.S_recent) * ld, "k_pruned", "thk_compact_keys")
    _check(load().thk_compact_keys(ctypes.byref(shape), _ptr(k), _ptr(idx), _ptr(k_pruned),
                                   _stream(stream)), "thk_compact_keys")


def thk_prune(shape, q_obs, k, score, idx, k_pruned, ws, stream=None):
    U, H, ld = _dims(shape)
    _need(q_obs, H * shape.S_obs * shape.D, "q_obs", "thk_prune")
    _need(k, U * shape.S * shape.D, "k", "thk_prune")
    _need(score, U * shape.D, "score", "thk_prune")
    _need(idx, U * shape.T, "idx", "thk_prune")
    _need(k_pruned, U * _cache_rows(shape, shape.S - shape.S_recent) * ld, "k_pruned", "thk_prune")
    _check(load().thk_prune(ctypes.byref(shape), _ptr(q_obs), _ptr(k), _ptr(score), _ptr(idx),
                            _ptr(k_pruned), _ws(ws), _nbytes(ws), _stream(stream)), "thk_prune")


def thk_decode_attn(shape, q, k_pruned, idx, v, k_tail, v_tail, s_tail, s_tail_cap, out, ws,
                    stream=None):
    U, H, ld = _dims(shape)
    w = "thk_decode_attn"
    _need(q, H * shape.D, "q", w)
    _need(out, H * shape.D, "out", w)
    rows = _cache_rows(shape, shape.S)
    _need(k_pruned, U * rows * ld, "k_pruned", w)
    _need(idx, U * shape.T, "idx", w)
    _need(v, U * rows * shape.D, "v", w)
    if s_tail > 0:
        _need(k_tail, U * s_tail_cap * shape.D, "k_tail", w)
        _need(v_tail, U * s_tail_cap * shape.D, "v_tail", w)
    _check(load().thk_decode_attn(ctypes.byref(shape), _ptr(q), _ptr(k_pruned), _ptr(idx), _ptr(v),
                                  _ptr(k_tail), _ptr(v_tail), s_tail, s_tail_cap, _ptr(out),
                                  _ws(ws), _nbytes(ws), _stream(stream)), "thk_decode_attn")


def thk_decode_attn_static(shape, q, k_pruned, idx, v, k_tail, v_tail, s_tail, s_tail_cap, out, stream=None):
    U, H, ld = _dims(shape)
    w = "thk_decode_attn_static"
    _need(q, H * shape.D, "q", w)
    _need(out, H * shape.D, "out", w)
    rows = _cache_rows(shape, shape.S)
    _need(k_pruned, U * rows * ld, "k_pruned", w)
    _need(idx, U * shape.T, "idx", w)
    _need(v, U * rows * shape.D, "v", w)
    if s_tail > 0:
        _need(k_tail, U * s_tail_cap * shape.D, "k_tail", w)
        _need(v_tail, U * s_tail_cap * shape.D, "v_tail", w)
    _check(load().thk_decode_attn_static(ctypes.byref(shape), _ptr(q), _ptr(k_pruned), _ptr(idx), _ptr(v),
                                         _ptr(k_tail), _ptr(v_tail), s_tail, s_tail_cap, _ptr(out),
                                         _stream(stream)), w)


def thk_decode_attn_kv(shape, q, k_pruned, idx, v_pruned, idx_v, T_v, ld_v, k_tail, v_tail, s_tail,
                       s_tail_cap, out, ws, stream=None):
    U, H, ld = _dims(shape)
    w = "thk_decode_attn_kv"
    _need(q, H * shape.D, "q", w)
    _need(out, H * shape.D, "out", w)
    rows = _cache_rows(shape, shape.S)
    _need(k_pruned, U * rows * ld, "k_pruned", w)
    _need(idx, U * shape.T, "idx", w)
    _need(v_pruned, U * rows * max(ld_v, 0), "v_pruned", w)
    _need(idx_v, U * max(T_v, 0), "idx_v", w)
    if s_tail > 0:
        _need(k_tail, U * s_tail_cap * shape.D, "k_tail", w)
        _need(v_tail, U * s_tail_cap * shape.D, "v_tail", w)
    _check(load().thk_decode_attn_kv(ctypes.byref(shape), _ptr(q), _ptr(k_pruned), _ptr(idx),
                                     _ptr(v_pruned), _ptr(idx_v), T_v, ld_v, _ptr(k_tail), _ptr(v_tail),
                                     s_tail, s_tail_cap, _ptr(out), _ws(ws), _nbytes(ws),
                                     _stream(stream)), w)


def thk_tail_append(shape, k_new, v_new, k_tail, v_tail, s_tail, s_tail_cap, stream=None):
    U, _, _ = _dims(shape)
    _need(k_new, U * shape.D, "k_new", "thk_tail_append")
    _need(v_new, U * shape.D, "v_new", "thk_tail_append")
    _need(k_tail, U * s_tail_cap * shape.D, "k_tail", "thk_tail_append")
    _need(v_tail, U * s_tail_cap * shape.D, "v_tail", "thk_tail_append")
    _check(load().thk_tail_append(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(k_tail),
                                  _ptr(v_tail), s_tail, s_tail_cap, _stream(stream)),
           "thk_tail_append")


def thk_compact_rows(shape, src, src_unit_rows, src_row0, idx, k_pruned, dst_row0, n_rows, stream=None):
    U, _, ld = _dims(shape)
    _need(src, U * src_unit_rows * shape.D, "src", "thk_compact_rows")
    _need(idx, U * shape.T, "idx", "thk_compact_rows")
    _need(k_pruned, U * _cache_rows(shape, shape.S) * ld, "k_pruned", "thk_compact_rows")
    _check(load().thk_compact_rows(ctypes.byref(shape), _ptr(src), src_unit_rows, src_row0, _ptr(idx),
                                   _ptr(k_pruned), dst_row0, n_rows, _stream(stream)), "thk_compact_rows")


def thk_copy_rows(shape, src, src_unit_rows, src_row0, dst, dst_unit_rows, dst_row0, n_rows, stream=None):
    U, _, _ = _dims(shape)
    _need(src, U * src_unit_rows * shape.D, "src", "thk_copy_rows")
    _need(dst, U * dst_unit_rows * shape.D, "dst", "thk_copy_rows")
    _check(load().thk_copy_rows(ctypes.byref(shape), _ptr(src), src_unit_rows, src_row0, _ptr(dst),
                                dst_unit_rows, dst_row0, n_rows, _stream(stream)), "thk_copy_rows")


def thk_cache_append(shape, k_new, v_new, k_tail, v, s_tail, s_tail_cap, stream=None):
    U, _, _ = _dims(shape)
    _need(k_new, U * shape.D, "k_new", "thk_cache_append")
    _need(v_new, U * shape.D, "v_new", "thk_cache_append")
    _need(k_tail, U * s_tail_cap * shape.D, "k_tail", "thk_cache_append")
    _need(v, U * _cache_rows(shape, shape.S) * shape.D, "v", "thk_cache_append")
    _check(load().thk_cache_append(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(k_tail), _ptr(v),
                                   s_tail, s_tail_cap, _stream(stream)), "thk_cache_append")


def thk_tail_flush(shape, idx, k_pruned, k_tail, v, v_tail, s_tail, s_tail_cap, n_flush, stream=None):
    U, _, ld = _dims(shape)
    rows = _cache_rows(shape, shape.S)
    _need(idx, U * shape.T, "idx", "thk_tail_flush")
    _need(k_pruned, U * rows * ld, "k_pruned", "thk_tail_flush")
    _need(k_tail, U * s_tail_cap * shape.D, "k_tail", "thk_tail_flush")
    _need(v, U * rows * shape.D, "v", "thk_tail_flush")
    _need(v_tail, U * s_tail_cap * shape.D, "v_tail", "thk_tail_flush")
    _check(load().thk_tail_flush(ctypes.byref(shape), _ptr(idx), _ptr(k_pruned), _ptr(k_tail), _ptr(v),
                                 _ptr(v_tail), s_tail, s_tail_cap, n_flush, _stream(stream)), "thk_tail_flush")


THK_STREAM_READ, THK_STREAM_COPY, THK_STREAM_WRITE = 0, 1, 2


def thk_bench_stream(mode, src, dst, n_blocks, w, stream=None):
    """Plain read / copy / write stream for benchmarks: n_blocks blocks of 128 KiB of src and
    w * 4 KiB of dst each (src or dst may be None where the mode does not use it)."""
    if src is not None:
        _need(src, n_blocks * 131072 // src.element_size(), "src", "thk_bench_stream")
    if dst is not None and mode != THK_STREAM_READ:
        _need(dst, n_blocks * w * 4096 // dst.element_size(), "dst", "thk_bench_stream")
    _check(load().thk_bench_stream(mode, _ptr(src), _ptr(dst), n_blocks, w, _stream(stream)), "thk_bench_stream")


def thk_profile_next(ev_start, ev_stop):
    """ev_start / ev_stop: torch.cuda.Event(enable_timing=True) that have been recorded once
    (torch creates the HIP event lazily), raw hipEvent_t integers, or None to cancel."""
    def h(e):
        if e is None or isinstance(e, int):
            return e
        return e.cuda_event
    load().thk_profile_next(ctypes.c_void_p(h(ev_start)) if ev_start is not None else None,
                            ctypes.c_void_p(h(ev_stop)) if ev_stop is not None else None)
