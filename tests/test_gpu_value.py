"""GPU parity of the value-cache path (Appendix "Value Cache Pruning"): value-channel score
on the matrix cores, selection and compaction of value channels, against the CPU fp64 oracle.

Tolerance of the score: 1e-5 relative, per channel, for both element types.  Logits and
softmax run in fp32; with bf16 tensors each probability enters the product with V as two bf16
terms (hi + lo, |p - hi - lo| <= 2^-18 p), so nothing is lost against fp32 arithmetic, and the
row sum takes the fp32 probabilities.  What is left is the fp32 accumulation over the keys
(measured: 1e-7 typical, up to 5e-6 on short windows where a channel's few outputs nearly
cancel).  The index set is compared with the ORACLE's own ranking: the two may differ only in
channels whose oracle score lies within TIE_V_TOL (relative) of the oracle's T-th largest.
"""
import numpy as np
import pytest
import torch

import paper_2407_21018_amd as thk
from oracle import oracle as O
from paper_2407_21018_amd.synth import as_numpy
from helpers import DT, TDT, gpu_compact, gpu_select, ws_tensor

pytestmark = pytest.mark.gpu
D = 128
SCORE_V_TOL = 1e-5   # relative, per channel, fp32 and bf16 tensors alike
TIE_V_TOL = 1e-5     # oracle scores closer than this (relative) to the T-th largest may swap


def _randn(shape, dtype, seed, sigma=0.0):
    g = torch.Generator(device="cuda"); g.manual_seed(seed)
    x = torch.randn(*shape, generator=g, device="cuda")
    if sigma:
        x = x * torch.exp(sigma * torch.randn(shape[-1], generator=g, device="cuda"))
    return x.to(TDT[dtype])


def gpu_score_value(shape, q_obs, k, v, causal):
    U = shape.L * shape.B * shape.N_kv
    score = torch.full((U, shape.D), float("nan"), dtype=torch.float32, device=k.device)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_SCORE_VALUE))
    thk.thk_score_value(shape, q_obs, k, v, causal, score, ws)
    torch.cuda.synchronize()
    return score


def check_score(got, want, v_np_f64, G, S_obs, tag, dtype="bf16"):
    """got, want [U, D] (want > 0 for any non-zero value column)."""
    assert np.all(np.isfinite(got))
    rel = np.abs(got - want) / np.maximum(want, 1e-300)
    print(f"{tag} {dtype}: max rel {rel.max():.3e} median rel {np.median(rel):.3e}", flush=True)
    assert rel.max() <= SCORE_V_TOL


def check_idx_against_oracle_ranking(gpu_idx, ora_score, T_v):
    """gpu_idx [U, T_v] against Top_T of the oracle's own scores [U, D]: ascending, valid, and
    different only in channels that tie with the threshold score within TIE_V_TOL."""
    ora_idx = O.select_topk(ora_score, T_v)
    n_diff = 0
    for u in range(ora_score.shape[0]):
        g = gpu_idx[u].tolist()
        assert g == sorted(set(g)) and len(g) == T_v and 0 <= g[0] and g[-1] < D, f"unit {u}: invalid list"
        thr = np.sort(ora_score[u])[::-1][T_v - 1]
        for c in set(g) ^ set(ora_idx[u].tolist()):
            n_diff += 1
            assert abs(ora_score[u, c] - thr) <= TIE_V_TOL * thr, (u, c, ora_score[u, c], thr)
    return n_diff


CASES = [
    # G, S_obs, S, n_split, causal, sigma
    (1, 32, 1037, 0, 0, 0.5),
    (1, 32, 1037, 0, 1, 0.5),
    (4, 32, 1037, 3, 1, 0.5),
    (2, 32, 600, 2, 0, 1.0),
    (4, 64, 777, 0, 1, 0.5),     # 8 query tiles: two blocks per unit
    (3, 16, 300, 0, 1, 0.0),     # heads share a query tile; last tile partly empty
    (1, 8, 129, 1, 1, 0.0),
    (1, 32, 32, 1, 1, 0.0),      # the window is the whole sequence
    (1, 1, 1, 1, 0, 0.0),        # one key, one query
    (2, 5, 40, 0, 1, 0.0),
    (4, 32, 4100, 0, 0, 1.0),
    (1, 32, 4100, 8, 1, 1.0),
    (16, 32, 500, 3, 1, 0.5),    # 16 query tiles: four blocks per (unit, piece), placed 8 workgroups apart
    (5, 64, 900, 5, 0, 0.5),     # 10 tiles: three blocks, the last half empty; pieces not a multiple of 8
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("G,S_obs,S,n_split,causal,sigma", CASES)
def test_value_score_matches_oracle(G, S_obs, S, n_split, causal, sigma, dtype):
    L, B, N_kv = 1, 2, 2
    seed = 1000 + 7 * S + G
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, seed, sigma)
    k = _randn((L, B, N_kv, S, D), dtype, seed + 1, sigma)
    v = _randn((L, B, N_kv, S, D), dtype, seed + 2)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, 64, 0, DT[dtype], n_split)
    print(f"value score {dtype} G={G} S_obs={S_obs} S={S} n_split={n_split} causal={causal}", flush=True)
    got = gpu_score_value(shape, q_obs, k, v, causal).cpu().numpy().astype(np.float64)
    want = O.score_value(as_numpy(q_obs), as_numpy(k), as_numpy(v), dtype, causal=bool(causal))
    v64 = v.cpu().to(torch.float64).numpy().reshape(-1, S, D)
    check_score(got, want.reshape(-1, D), v64, G, S_obs, f"G={G} S_obs={S_obs} S={S}", dtype)


def test_value_score_split_count_changes_only_rounding():
    """Any cut of the key axis gives the same score up to fp32 merge rounding."""
    L, B, N_kv, G, S, S_obs = 1, 1, 2, 2, 3000, 32
    q_obs = _randn((L, B, N_kv * G, S_obs, D), "bf16", 5, 0.5)
    k = _randn((L, B, N_kv, S, D), "bf16", 6, 0.5)
    v = _randn((L, B, N_kv, S, D), "bf16", 7)
    ref = None
    for n in (1, 2, 5, 24):
        shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, 64, 0, thk.THK_BF16, n)
        got = gpu_score_value(shape, q_obs, k, v, 1).cpu().numpy().astype(np.float64)
        if ref is None:
            ref = got
        # a different cut changes the order of the fp32 sums: same tolerance class as against the oracle
        assert (np.abs(got - ref) / ref).max() <= 2 * SCORE_V_TOL


def test_value_prune_select_and_compact():
    """score_v -> Top_T -> compaction of V.  The selection is taken in the kernel's precision
    on both sides (the oracle selects from the float scores the GPU produced) and must agree
    exactly; the compacted values are a bit copy."""
    L, B, N_kv, G, S, S_obs, T_v = 1, 2, 2, 4, 900, 32, 77
    q_obs = _randn((L, B, N_kv * G, S_obs, D), "bf16", 21, 0.5)
    k = _randn((L, B, N_kv, S, D), "bf16", 22, 0.5)
    # give the value channels unequal magnitudes so that the ranking is not all near-ties
    v = _randn((L, B, N_kv, S, D), "bf16", 23, 0.7)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T_v, 0, thk.THK_BF16, 0)
    score = gpu_score_value(shape, q_obs, k, v, 1)
    idx = gpu_select(shape, score)
    want_idx = O.select_topk(score.cpu().numpy().astype(np.float64), T_v)
    np.testing.assert_array_equal(idx.cpu().numpy(), want_idx)
    vp = gpu_compact(shape, v, idx)
    want_vp = O.compact_keys(as_numpy(v).reshape(-1, S, D), want_idx, "bf16")
    np.testing.assert_array_equal(as_numpy(vp), want_vp)
    # ... and the list agrees with the ORACLE's own ranking up to exact-tolerance ties
    ora = O.score_value(as_numpy(q_obs), as_numpy(k), as_numpy(v), "bf16", causal=True).reshape(-1, D)
    check_idx_against_oracle_ranking(idx.cpu().numpy(), ora, T_v)


def test_value_score_argument_errors():
    A = torch.zeros(1 << 16, dtype=torch.uint8, device="cuda")
    s = thk.make_shape(1, 1, 1, 1, D, 64, 32, 64, 0, thk.THK_BF16, 0)
    def st(*a):
        try:
            thk.thk_score_value(*a)
        except thk.ThkError as e:
            return e.status
        return 0
    big = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    assert st(s, big, big, big, 2, big, big) == 2                      # causal flag out of range
    assert st(s, big, big[1:], big, 0, big, big) == 4                  # misaligned pointer
    assert st(s, big, big, big, 0, big, A[:16]) == 5                   # workspace too small
    s2 = thk.make_shape(1, 1, 1, 1, D, 16, 32, 64, 0, thk.THK_BF16, 0)
    assert st(s2, big, big, big, 0, big, big) == 2                     # S_obs > S


# ------------------------------------------------ decode over pruned K and V ----
def _rand_idx(U, T, seed):
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    idx = torch.stack([torch.randperm(D, generator=g)[:T].sort().values for _ in range(U)])
    return idx.to(torch.int16).cuda()


DECODE_CASES = [
    # dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split
    ("bf16", 1, 1037, 76, 76, 76, 0, 0, 0),
    ("bf16", 1, 1037, 76, 51, 52, 5, 16, 3),
    ("bf16", 4, 2100, 64, 64, 64, 17, 32, 0),
    ("bf16", 2, 600, 51, 89, 92, 0, 0, 1),      # wide value rows
    ("bf16", 4, 333, 128, 128, 128, 3, 8, 2),   # nothing removed: the widest rows
    ("bf16", 1, 45, 64, 1, 4, 2, 4, 1),         # a single kept value channel
    ("bf16", 8, 777, 38, 102, 104, 1, 1, 0),
    # bf16 with four query heads per KV head and T, ld_v multiples of 4: the matrix-core kernel
    ("bf16", 4, 1037, 76, 51, 52, 5, 16, 3),
    ("bf16", 4, 97, 64, 3, 4, 0, 0, 1),
    ("bf16", 4, 500, 76, 100, 104, 0, 0, 0),
    ("bf16", 4, 31, 64, 64, 64, 0, 0, 1),       # one ragged tile
    ("bf16", 8, 1300, 64, 76, 76, 33, 64, 2),
    ("bf16", 8, 300, 128, 100, 128, 2, 4, 0),   # eight heads per block, the widest staging class
    ("bf16", 16, 900, 76, 51, 52, 0, 0, 3),
    ("bf16", 3, 700, 64, 40, 40, 4, 8, 0),      # partly filled head groups
    ("bf16", 7, 500, 76, 90, 92, 0, 0, 2),
    ("bf16", 5, 400, 51, 64, 64, 3, 4, 0),      # ... on the general kernel (T not a multiple of 4)
    ("f32", 3, 300, 64, 32, 32, 0, 0, 1),
    ("f32", 1, 1037, 64, 64, 64, 0, 0, 0),
    ("f32", 4, 900, 76, 51, 52, 9, 16, 4),
    ("f32", 2, 333, 51, 128, 128, 0, 0, 1),
    ("f32", 1, 5, 3, 7, 8, 0, 0, 1),
]


@pytest.mark.parametrize("dtype,G,S,T,T_v,ld_v,s_tail,cap,n_split", DECODE_CASES)
def test_decode_attn_kv_matches_oracle(dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split, decode_merge):
    from helpers import ATTN_TOL, attn_rel_err
    L, B, N_kv = 1, 2, 2
    U = L * B * N_kv
    seed = 50 + S + T_v
    q = _randn((L * B * N_kv * G, D), dtype, seed, 0.5)
    kp = _randn((U, S, T), dtype, seed + 1, 0.5)
    vp = _randn((U, S, ld_v), dtype, seed + 2)
    if ld_v > T_v:
        vp[:, :, T_v:] = float("nan")          # the padding of a value row must never be used
    idx, idx_v = _rand_idx(U, T, seed + 3), _rand_idx(U, T_v, seed + 4)
    kt = _randn((U, max(cap, 1), D), dtype, seed + 5, 0.5)
    vt = _randn((U, max(cap, 1), D), dtype, seed + 6)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, 1, T, 0, DT[dtype], n_split)
    out = torch.full((U * G, D), float("nan"), dtype=TDT[dtype], device="cuda")
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
    print(f"decode kv {dtype} G={G} S={S} T={T} T_v={T_v} ld_v={ld_v} tail={s_tail} split={n_split}", flush=True)
    thk.thk_decode_attn_kv(shape, q, kp, idx, vp, idx_v, T_v, ld_v, kt if s_tail else None,
                           vt if s_tail else None, s_tail, cap, out, ws)
    torch.cuda.synchronize()
    vp_np = as_numpy(vp[:, :, :T_v].contiguous()).reshape(B, N_kv, S, T_v)
    want = O.decode_attn_kv(as_numpy(q).reshape(B, N_kv * G, D), as_numpy(kp).reshape(B, N_kv, S, T),
                            as_numpy(idx).reshape(B, N_kv, T), vp_np, as_numpy(idx_v).reshape(B, N_kv, T_v),
                            dtype, as_numpy(kt).reshape(B, N_kv, -1, D) if s_tail else None,
                            as_numpy(vt).reshape(B, N_kv, -1, D) if s_tail else None, s_tail)
    err = attn_rel_err(out, want.reshape(-1, D))
    print(f"   max rel err {err.max():.3e}", flush=True)
    assert err.max() <= ATTN_TOL[dtype]
    if s_tail == 0:   # removed channels are exactly zero
        o = out.float().cpu().numpy().reshape(U, G, D)
        keep = np.zeros((U, D), bool)
        np.put_along_axis(keep, idx_v.cpu().numpy().astype(np.int64), True, axis=1)
        assert np.all(o[~np.broadcast_to(keep[:, None, :], o.shape)] == 0.0)


@pytest.mark.parametrize("dtype,G,S,T,T_v,ld_v,s_tail,cap,n_split",
                         [c for c in DECODE_CASES if c[0] == "bf16" and c[1] >= 3 and c[3] % 4 == 0])
def test_decode_attn_kv_general_kernel_on_grouped_heads(dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split, thk_env,
                                                        decode_merge):
    """THK_DECODE_MFMA=0: the shapes the matrix-core kernel serves, on the general kernel."""
    thk_env.setenv("THK_DECODE_MFMA", "0")
    test_decode_attn_kv_matches_oracle(dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split, decode_merge)


def test_decode_attn_kv_with_identity_value_index_equals_key_only_decode():
    """T_v = D, idx_v = 0..D-1: the same arithmetic order is not promised, the same result to
    the attention tolerance is."""
    from helpers import ATTN_TOL, gpu_decode
    L, B, N_kv, G, S, T = 1, 2, 2, 4, 1500, 64
    U = L * B * N_kv
    q = _randn((U * G, D), "bf16", 91, 0.5)
    kp = _randn((U, S, T), "bf16", 92, 0.5)
    v = _randn((U, S, D), "bf16", 93)
    idx = _rand_idx(U, T, 94)
    ident = torch.arange(D, dtype=torch.int16, device="cuda").repeat(U, 1).contiguous()
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, 1, T, 0, thk.THK_BF16, 0)
    ref = gpu_decode(shape, q, kp, idx, v).float()
    out = torch.empty_like(q)
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
    thk.thk_decode_attn_kv(shape, q, kp, idx, v, ident, D, D, None, None, 0, 0, out, ws)
    torch.cuda.synchronize()
    rel = (out.float() - ref).abs().amax(1) / ref.abs().amax(1)
    assert rel.max().item() <= ATTN_TOL["bf16"]


def test_decode_attn_kv_argument_errors():
    big = torch.zeros(1 << 20, dtype=torch.uint8, device="cuda")
    s = thk.make_shape(1, 1, 1, 1, D, 64, 1, 64, 0, thk.THK_BF16, 1)
    def st(*a):
        try:
            thk.thk_decode_attn_kv(*a)
        except thk.ThkError as e:
            return e.status
        return 0
    assert st(s, big, big, big, big, big, 0, 0, None, None, 0, 0, big, big) == 2      # T_v < 1
    assert st(s, big, big, big, big, big, 65, 64, None, None, 0, 0, big, big) == 2    # ld_v < T_v
    assert st(s, big, big, big, big, big, 63, 63, None, None, 0, 0, big, big) == 3    # ld_v % 4 != 0
    assert st(s, big, big, big, big, None, 64, 64, None, None, 0, 0, big, big) == 1   # idx_v missing
    assert st(s, big, big, big, big, big, 64, 64, big, None, 2, 4, big, big) == 1     # tail without v_tail


# ------------------------------- thk_prune_value: the two forms of the compaction step ----
@pytest.mark.parametrize("spin", [None, "0"], ids=["wait", "give-up"])
@pytest.mark.parametrize("dtype,G,S,T_v,ld_v,S_recent", [
    ("bf16", 1, 1500, 76, 76, 0),
    ("bf16", 2, 4100, 51, 52, 32),      # padded rows, the last 32 rows stay with the caller
    ("f32", 1, 700, 64, 64, 0),
    ("bf16", 1, 1037, 1, 4, 0),         # one kept channel, odd length
    ("bf16", 1, 40000, 100, 104, 0),    # 79 row blocks per unit: the sums travel in two levels
])
def test_value_prune_compaction_in_bursts(dtype, G, S, T_v, ld_v, S_recent, spin, thk_env):
    """Long thk_prune_value calls compact V through the one-pass prune kernels with the index
    list given (their hand-off only groups a unit's stores).  Forced here on small calls, with
    the blocks waiting for each other and with every wait given up at once (the repair launch
    then compacts from the given list): scores, list and compacted values must equal those of
    the plain compaction kernel bit for bit, and the oracle's compaction."""
    L, B, N_kv, S_obs = 1, 2, 2, 32
    U = L * B * N_kv
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, 401, 0.5)
    k = _randn((L, B, N_kv, S, D), dtype, 402, 0.5)
    v = _randn((L, B, N_kv, S, D), dtype, 403, 0.7)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T_v, ld_v, DT[dtype], 0, S_recent)
    got = {}
    if spin is not None:
        thk_env.setenv("THK_PRUNE_SPIN_LIMIT", spin)
    for form in ("flat", "burst"):
        thk_env.setenv("THK_VALUE_COMPACT", form)
        score_v = torch.empty(U, D, dtype=torch.float32, device="cuda")
        idx_v = torch.full((U, T_v), -1, dtype=torch.int16, device="cuda")
        vp = torch.full((U, S - S_recent, ld_v), float("nan"), dtype=TDT[dtype], device="cuda")
        ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_PRUNE_VALUE))
        print(f"prune_value {form} {dtype} G={G} S={S} T_v={T_v} ld_v={ld_v} S_recent={S_recent} spin={spin}",
              flush=True)
        thk.thk_prune_value(shape, q_obs, k, v, 1, score_v, idx_v, vp, ws)
        torch.cuda.synchronize()
        got[form] = (score_v.cpu(), idx_v.cpu(), vp.cpu())
    assert torch.equal(got["flat"][0], got["burst"][0])
    assert torch.equal(got["flat"][1], got["burst"][1])
    assert torch.equal(got["flat"][2].view(torch.uint8), got["burst"][2].view(torch.uint8))
    want_vp = O.compact_keys(as_numpy(v).reshape(U, S, D)[:, :S - S_recent], got["burst"][1].numpy(), dtype)
    np.testing.assert_array_equal(as_numpy(got["burst"][2][:, :, :T_v].contiguous()), want_vp)
    if ld_v > T_v:
        assert (got["burst"][2][:, :, T_v:] == 0).all()   # the padding of the rows written is zero


# -------------------------------------------- the whole path: prune K, prune V, decode ----
@pytest.mark.parametrize("dtype,G,S,lam_k,lam_v,causal", [("bf16", 1, 1500, 0.4, 0.4, 1), ("bf16", 4, 2300, 0.5, 0.3, 1),
                                                         ("f32", 2, 700, 0.5, 0.5, 0)])
def test_prune_keys_and_values_then_decode(dtype, G, S, lam_k, lam_v, causal):
    """End of prefill: thk_prune for the keys, thk_prune_value for the values; then one decode
    step over both pruned caches with a short un-pruned tail.  Every stage is checked against the
    oracle fed with the GPU's own upstream results (so one tie-swap cannot cascade)."""
    from helpers import ATTN_TOL, attn_rel_err, gpu_prune
    L, B, N_kv, S_obs, cap, s_tail = 1, 2, 2, 32, 8, 3
    U = L * B * N_kv
    T, T_v = thk.thk_keep_count(D, lam_k), thk.thk_keep_count(D, lam_v)
    ld_v = (T_v + 3) // 4 * 4
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, 301, 0.5)
    k = _randn((L, B, N_kv, S, D), dtype, 302, 0.5)
    v = _randn((L, B, N_kv, S, D), dtype, 303, 0.7)
    shape_k = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, 0, DT[dtype], 0)
    _, idx, kp = gpu_prune(shape_k, q_obs, k)
    shape_v = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T_v, ld_v, DT[dtype], 0)
    score_v = torch.empty(U, D, dtype=torch.float32, device="cuda")
    idx_v = torch.full((U, T_v), -1, dtype=torch.int16, device="cuda")
    vp = torch.zeros(U, S, ld_v, dtype=TDT[dtype], device="cuda")
    ws = ws_tensor(thk.thk_workspace_bytes(shape_v, thk.THK_OP_PRUNE_VALUE))
    thk.thk_prune_value(shape_v, q_obs, k, v, causal, score_v, idx_v, vp, ws)
    torch.cuda.synchronize()
    # stage checks
    want_sc = O.score_value(as_numpy(q_obs), as_numpy(k), as_numpy(v), dtype, causal=bool(causal)).reshape(U, D)
    check_score(score_v.cpu().numpy().astype(np.float64), want_sc,
                v.cpu().to(torch.float64).numpy().reshape(U, S, D), G, S_obs, "pipeline", dtype)
    want_idx_v = O.select_topk(score_v.cpu().numpy().astype(np.float64), T_v)
    np.testing.assert_array_equal(idx_v.cpu().numpy(), want_idx_v)
    want_vp = O.compact_keys(as_numpy(v).reshape(U, S, D), want_idx_v, dtype)
    np.testing.assert_array_equal(as_numpy(vp[:, :, :T_v].contiguous()), want_vp)
    # the same call with the score left in the workspace gives the same index list
    idx_v2 = torch.full_like(idx_v, -1)
    thk.thk_prune_value(shape_v, q_obs, k, v, causal, None, idx_v2, vp, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx_v, idx_v2)
    # decode
    q = _randn((U * G, D), dtype, 304, 0.5)
    kt = _randn((U, cap, D), dtype, 305, 0.5)
    vt = _randn((U, cap, D), dtype, 306)
    shape_d = thk.make_shape(L, B, N_kv * G, N_kv, D, S, 1, T, 0, DT[dtype], 0)
    out = torch.empty(U * G, D, dtype=TDT[dtype], device="cuda")
    wsd = ws_tensor(thk.thk_workspace_bytes(shape_d, thk.THK_OP_DECODE))
    thk.thk_decode_attn_kv(shape_d, q, kp, idx, vp, idx_v, T_v, ld_v, kt, vt, s_tail, cap, out, wsd)
    torch.cuda.synchronize()
    want = O.decode_attn_kv(as_numpy(q).reshape(B, N_kv * G, D), as_numpy(kp).reshape(B, N_kv, S, T),
                            as_numpy(idx).reshape(B, N_kv, T), want_vp.reshape(B, N_kv, S, T_v),
                            want_idx_v.reshape(B, N_kv, T_v), dtype, as_numpy(kt).reshape(B, N_kv, cap, D),
                            as_numpy(vt).reshape(B, N_kv, cap, D), s_tail)
    assert attn_rel_err(out, want.reshape(-1, D)).max() <= ATTN_TOL[dtype]
