"""ctypes front end of the CPU fp64 oracle (thk_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg; never by the product package.  Arrays are numpy;
bf16 tensors travel as uint16 arrays with dtype="bf16".
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "thk_oracle.c")
_LIB = os.path.join(_HERE, "libthk_oracle.so")

_DT = {"f32": 0, "bf16": 1, "f64": 2}
_NP = {"f32": np.float32, "bf16": np.uint16, "f64": np.float64}


def build(force=False):
    """Compile thk_oracle.c with gcc (OpenMP over independent units)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off",
             "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        i32, i64, vp, dbl = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p, ctypes.c_double
        L.thko_max_threads.restype = ctypes.c_int
        L.thko_keep_count.restype = i32
        L.thko_keep_count.argtypes = [i32, dbl]
        L.thko_kv_cache_bytes.restype = dbl
        L.thko_kv_cache_bytes.argtypes = [dbl] * 6
        L.thko_score.restype = None
        L.thko_score.argtypes = [ctypes.c_int, i32, i32, i32, i32, i32, i64, i32, vp, vp, vp]
        L.thko_score_bruteforce.restype = None
        L.thko_score_bruteforce.argtypes = L.thko_score.argtypes
        L.thko_score_magnitude.restype = None
        L.thko_score_magnitude.argtypes = [ctypes.c_int, i64, i32, i64, i32, vp, vp]
        L.thko_select_topk.restype = None
        L.thko_select_topk.argtypes = [i64, i32, i32, vp, vp]
        L.thko_compact_keys.restype = None
        L.thko_compact_keys.argtypes = [ctypes.c_int, i64, i64, i32, i32, i32, vp, vp, vp]
        L.thko_decode_attn.restype = None
        L.thko_decode_attn.argtypes = [ctypes.c_int, i32, i32, i32, i32, i64, i32, i32,
                                       vp, vp, vp, vp, vp, vp, i32, i32, vp]
        L.thko_score_value.restype = None
        L.thko_score_value.argtypes = [ctypes.c_int, i32, i32, i32, i32, i32, i64, i32, i32,
                                       vp, vp, vp, vp]
        L.thko_decode_attn_kv.restype = None
        L.thko_decode_attn_kv.argtypes = [ctypes.c_int, i32, i32, i32, i32, i64, i32, i32, i32, i32,
                                          vp, vp, vp, vp, vp, vp, vp, i32, i32, vp]
        L.thko_objective.restype = dbl
        L.thko_objective.argtypes = [i32, i64, i32, vp, vp, vp]
        _lib = L
    return _lib


def _arr(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != _NP[dtype]:
        raise TypeError(f"expected {_NP[dtype]} array for dtype {dtype}, got {a.dtype}")
    return a


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def max_threads():
    return int(lib().thko_max_threads())


def keep_count(D, lam):
    return int(lib().thko_keep_count(D, lam))


def kv_cache_bytes(B, S, L, N, D, bytes_per_elem):
    return float(lib().thko_kv_cache_bytes(B, S, L, N, D, bytes_per_elem))


def score(q_obs, k, dtype, brute=False):
    """q_obs [L,B,N_q,S_obs,D], k [L,B,N_kv,S,D] -> score float64 [L,B,N_kv,D]."""
    q_obs, k = _arr(q_obs, dtype), _arr(k, dtype)
    L, B, N_q, S_obs, D = q_obs.shape
    L2, B2, N_kv, S, D2 = k.shape
    assert (L, B, D) == (L2, B2, D2) and N_q % N_kv == 0 and 1 <= S_obs <= S
    out = np.empty((L, B, N_kv, D), np.float64)
    fn = lib().thko_score_bruteforce if brute else lib().thko_score
    fn(_DT[dtype], L, B, N_q, N_kv, D, S, S_obs, _p(q_obs), _p(k), _p(out))
    return out


def score_magnitude(k, dtype, p):
    """k [..., S, D] -> ||K[:,c]||_p per unit, float64 [..., D]."""
    k = _arr(k, dtype)
    S, D = k.shape[-2:]
    U = int(np.prod(k.shape[:-2], dtype=np.int64))
    out = np.empty(k.shape[:-2] + (D,), np.float64)
    lib().thko_score_magnitude(_DT[dtype], U, D, S, p, _p(k), _p(out))
    return out


def select_topk(score_, T):
    """score [..., D] float64 -> idx int16 [..., T], ascending channel order."""
    sc = _arr(np.asarray(score_, np.float64), "f64")
    D = sc.shape[-1]
    assert 1 <= T <= D
    U = int(np.prod(sc.shape[:-1], dtype=np.int64))
    idx = np.empty(sc.shape[:-1] + (T,), np.int16)
    lib().thko_select_topk(U, D, T, _p(sc), _p(idx))
    return idx


def compact_keys(k, idx, dtype, ld_keep=0, out=None):
    """k [..., S, D], idx [..., T] -> K_pruned [..., S, ld_keep] (ld_keep=0 => T)."""
    k = _arr(k, dtype)
    idx = np.ascontiguousarray(idx, np.int16)
    S, D = k.shape[-2:]
    T = idx.shape[-1]
    ld = ld_keep or T
    assert ld >= T and idx.shape[:-1] == k.shape[:-2]
    U = int(np.prod(k.shape[:-2], dtype=np.int64))
    if out is None:
        out = np.zeros(k.shape[:-2] + (S, ld), _NP[dtype])
    lib().thko_compact_keys(_DT[dtype], U, S, D, T, ld, _p(k), _p(idx), _p(out))
    return out


def decode_attn(q, k_pruned, idx, v, dtype, k_tail=None, v_tail=None, s_tail=0):
    """q [B,N_q,D], k_pruned [B,N_kv,S,ld], idx [B,N_kv,T], v [B,N_kv,S,D],
    tails [B,N_kv,cap,D] -> out float64 [B,N_q,D]."""
    q, k_pruned, v = _arr(q, dtype), _arr(k_pruned, dtype), _arr(v, dtype)
    idx = np.ascontiguousarray(idx, np.int16)
    B, N_q, D = q.shape
    B2, N_kv, S, ld = k_pruned.shape
    T = idx.shape[-1]
    assert v.shape == (B, N_kv, S, D) and B2 == B and ld >= T and N_q % N_kv == 0
    cap = 0
    if s_tail > 0:
        k_tail, v_tail = _arr(k_tail, dtype), _arr(v_tail, dtype)
        cap = k_tail.shape[2]
        assert k_tail.shape == (B, N_kv, cap, D) == v_tail.shape and s_tail <= cap
    out = np.empty((B, N_q, D), np.float64)
    lib().thko_decode_attn(_DT[dtype], B, N_q, N_kv, D, S, T, ld, _p(q), _p(k_pruned), _p(idx),
                           _p(v), _p(k_tail) if s_tail else None,
                           _p(v_tail) if s_tail else None, s_tail, cap, _p(out))
    return out


def score_value(q_obs, k, v, dtype, causal=False):
    """q_obs [L,B,N_q,S_obs,D], k and v [L,B,N_kv,S,D] -> value-channel score
    float64 [L,B,N_kv,D] (column norms of softmax(Q_obs K^T / sqrt(D)) V, summed over
    the query heads of a group)."""
    q_obs, k, v = _arr(q_obs, dtype), _arr(k, dtype), _arr(v, dtype)
    L, B, N_q, S_obs, D = q_obs.shape
    L2, B2, N_kv, S, D2 = k.shape
    assert (L, B, D) == (L2, B2, D2) and N_q % N_kv == 0 and 1 <= S_obs <= S
    assert v.shape == k.shape
    out = np.empty((L, B, N_kv, D), np.float64)
    lib().thko_score_value(_DT[dtype], L, B, N_q, N_kv, D, S, S_obs, int(bool(causal)),
                           _p(q_obs), _p(k), _p(v), _p(out))
    return out


def decode_attn_kv(q, k_pruned, idx, v_pruned, idx_v, dtype, k_tail=None, v_tail=None, s_tail=0):
    """As decode_attn with a channel-pruned value cache: v_pruned [B,N_kv,S,ld_v],
    idx_v [B,N_kv,T_v]; the tail keeps full-width rows.  out float64 [B,N_q,D]."""
    q, k_pruned, v_pruned = _arr(q, dtype), _arr(k_pruned, dtype), _arr(v_pruned, dtype)
    idx = np.ascontiguousarray(idx, np.int16)
    idx_v = np.ascontiguousarray(idx_v, np.int16)
    B, N_q, D = q.shape
    B2, N_kv, S, ld = k_pruned.shape
    T, T_v, ld_v = idx.shape[-1], idx_v.shape[-1], v_pruned.shape[-1]
    assert v_pruned.shape[:3] == (B, N_kv, S) and B2 == B and ld >= T and ld_v >= T_v
    assert N_q % N_kv == 0 and idx_v.shape[:2] == (B, N_kv)
    cap = 0
    if s_tail > 0:
        k_tail, v_tail = _arr(k_tail, dtype), _arr(v_tail, dtype)
        cap = k_tail.shape[2]
        assert k_tail.shape == (B, N_kv, cap, D) == v_tail.shape and s_tail <= cap
    out = np.empty((B, N_q, D), np.float64)
    lib().thko_decode_attn_kv(_DT[dtype], B, N_q, N_kv, D, S, T, ld, T_v, ld_v, _p(q),
                              _p(k_pruned), _p(idx), _p(v_pruned), _p(idx_v),
                              _p(k_tail) if s_tail else None, _p(v_tail) if s_tail else None,
                              s_tail, cap, _p(out))
    return out


def objective(Q, K, keep):
    """|| Q K^T - Q diag(keep) K^T ||_F for one head; Q [S_q,D], K [S_k,D] float64."""
    Q, K = _arr(np.asarray(Q, np.float64), "f64"), _arr(np.asarray(K, np.float64), "f64")
    keep = np.ascontiguousarray(keep, np.uint8)
    return float(lib().thko_objective(Q.shape[0], K.shape[0], Q.shape[1], _p(Q), _p(K), _p(keep)))


def bf16_bits(x):
    """Round a float32 numpy array to bf16 (round-to-nearest-even) -> uint16 bits."""
    x = np.ascontiguousarray(x, np.float32)
    b = x.view(np.uint32)
    rounded = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_to_f64(bits):
    """Widen uint16 bf16 bit patterns exactly to float64."""
    return (np.ascontiguousarray(bits, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
