"""Seeded sweeps over shapes nobody picked by hand: decode attention (with and without
channel-pruned values) and the one-call prune against the CPU oracle.  The kernels are chosen
per shape (element type, query heads per KV head, row lengths and pitches, staging class,
split count), so a sweep walks through combinations the hand-written cases leave out."""
import numpy as np
import pytest
import torch

import paper_2407_21018_amd as thk
from oracle import oracle as O
from paper_2407_21018_amd.synth import as_numpy
from helpers import ATTN_TOL, DT, SCORE_TOL, TDT, attn_rel_err, check_idx_with_tie_rule, gpu_prune, oracle_prune, ws_tensor
from test_gpu_parity import _decode_case, _randn

pytestmark = pytest.mark.gpu
D = 128


def _decode_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        G = int(rng.choice([1, 2, 3, 4, 4, 5, 6, 7, 8, 8, 9, 12, 16]))
        T = int(rng.choice([int(rng.integers(1, 129)), 4 * int(rng.integers(1, 33))]))
        ld = 0 if rng.random() < 0.6 else min(128, T + int(rng.choice([1, 2, 4, 6, 8])))
        S = int(rng.choice([int(rng.integers(1, 70)), int(rng.integers(70, 1200)), int(rng.integers(1200, 3000))]))
        n_split = int(rng.choice([0, 0, 1, 2, 3, 5, 8]))
        cap = int(rng.choice([0, 1, 4, 16, 64]))
        s_tail = int(rng.integers(0, cap + 1)) if cap else 0
        sigma = float(rng.choice([0.0, 1.0, 1.0, 2.0]))
        # sigma = 2 on both the query and the keys puts logits in the thousands; fp32 cases draw
        # it too: the kernel forms logits of fp32 inputs in fp64 and subtracts the running maximum
        # before rounding, so the 1e-4 bar holds at any logit size
        out.append((dtype, 1, int(rng.integers(1, 3)), G, S, T, ld, n_split, s_tail, cap, sigma, 9000 + i))
    return out


@pytest.mark.parametrize("case", _decode_shapes(40, 20240721), ids=lambda c: "-".join(map(str, c[:10])))
def test_decode_random_shapes(case, decode_merge):
    dtype, B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, seed = case
    print(f"decode case {case}", flush=True)
    err, _ = _decode_case(dtype, B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, seed)
    assert err.max() <= ATTN_TOL[dtype], case


def _f32_heavy_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        G = int(rng.choice([1, 1, 2, 4, 5, 8]))
        T = int(rng.choice([int(rng.integers(8, 129)), 64, 76, 128]))
        ld = 0 if rng.random() < 0.7 else min(128, T + int(rng.choice([1, 4])))
        S = int(rng.choice([int(rng.integers(2, 70)), int(rng.integers(70, 1500)), int(rng.integers(1500, 6000))]))
        cap = int(rng.choice([0, 16, 64]))
        s_tail = int(rng.integers(0, cap + 1)) if cap else 0
        out.append(("f32", 1, int(rng.integers(1, 4)), G, S, T, ld, int(rng.choice([0, 1, 3, 8])), s_tail, cap, 2.0,
                    15000 + i))
    return out


@pytest.mark.parametrize("case", _f32_heavy_shapes(32, 20240726), ids=lambda c: "-".join(map(str, c[:10])))
def test_decode_f32_heavy_tailed_logits(case, decode_merge):
    """fp32 inputs with channel scales of sigma = 2 on BOTH the query and the keys: logits reach
    the thousands, where a logit held in fp32 is only accurate to ~1e-4 in absolute terms and a
    softmax that hangs between two keys shows it.  The kernel forms these logits in fp64 and
    rounds z - max, so the fp32 bar holds at any logit size."""
    test_decode_random_shapes(case, decode_merge)


def _rand_idx(U, T, seed):
    g = torch.Generator(device="cpu"); g.manual_seed(seed)
    idx = torch.stack([torch.sort(torch.randperm(D, generator=g)[:T]).values for _ in range(U)])
    return idx.to(torch.int16).cuda()


def _decode_kv_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "bf16" if rng.random() < 0.8 else "f32"
        G = int(rng.choice([1, 2, 3, 4, 4, 5, 7, 8, 8, 12, 16]))
        T = int(rng.choice([int(rng.integers(1, 129)), 4 * int(rng.integers(1, 33))]))
        T_v = int(rng.integers(1, 129))
        ld_v = min(128, 4 * ((T_v + 3) // 4) + 4 * int(rng.integers(0, 3)))
        S = int(rng.choice([int(rng.integers(1, 70)), int(rng.integers(70, 2500))]))
        n_split = int(rng.choice([0, 1, 2, 3]))
        cap = int(rng.choice([0, 4, 16, 64]))
        s_tail = int(rng.integers(0, cap + 1)) if cap else 0
        out.append((dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split, 9500 + i))
    return out


@pytest.mark.parametrize("case", _decode_kv_shapes(24, 20240722), ids=lambda c: "-".join(map(str, c[:9])))
def test_decode_kv_random_shapes(case, decode_merge):
    dtype, G, S, T, T_v, ld_v, s_tail, cap, n_split, seed = case
    print(f"decode kv case {case}", flush=True)
    B, N_kv = 1, 2
    U = B * N_kv
    q = _randn((U * G, D), dtype, seed, 0.5)
    kp = _randn((U, S, T), dtype, seed + 1, 0.5)
    vp = _randn((U, S, ld_v), dtype, seed + 2, 0)
    if ld_v > T_v:
        vp[:, :, T_v:] = float("nan")          # the padding of a value row must never be used
    idx, idx_v = _rand_idx(U, T, seed + 3), _rand_idx(U, T_v, seed + 4)
    kt = _randn((U, max(cap, 1), D), dtype, seed + 5, 0.5)
    vt = _randn((U, max(cap, 1), D), dtype, seed + 6, 0)
    shape = thk.make_shape(1, B, N_kv * G, N_kv, D, S, 1, T, 0, DT[dtype], n_split)
    out = torch.full((U * G, D), float("nan"), dtype=TDT[dtype], device="cuda")
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_DECODE))
    thk.thk_decode_attn_kv(shape, q, kp, idx, vp, idx_v, T_v, ld_v, kt if s_tail else None,
                           vt if s_tail else None, s_tail, cap, out, ws)
    torch.cuda.synchronize()
    vp_np = as_numpy(vp[:, :, :T_v].contiguous()).reshape(B, N_kv, S, T_v)
    want = O.decode_attn_kv(as_numpy(q).reshape(B, N_kv * G, D), as_numpy(kp).reshape(B, N_kv, S, T),
                            as_numpy(idx).reshape(B, N_kv, T), vp_np, as_numpy(idx_v).reshape(B, N_kv, T_v),
                            dtype, as_numpy(kt).reshape(B, N_kv, -1, D) if s_tail else None,
                            as_numpy(vt).reshape(B, N_kv, -1, D) if s_tail else None, s_tail)
    err = attn_rel_err(out, want.reshape(-1, D))
    assert err.max() <= ATTN_TOL[dtype], case


def _prune_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        G = int(rng.choice([1, 1, 2, 4, 8]))
        S = int(rng.choice([int(rng.integers(1, 200)), int(rng.integers(200, 5000)), 64 * int(rng.integers(1, 80))]))
        S_obs = int(min(S, rng.choice([1, 8, 32, 64])))
        T = int(rng.choice([int(rng.integers(1, 129)), 51, 64, 76]))
        block_rows = rng.choice(["", "32", "64", "128", "256", "512"])
        ld = 0 if rng.random() < 0.6 else min(128, T + int(rng.choice([1, 2, 4, 8, 12])))
        out.append((dtype, G, S, S_obs, T, ld, str(block_rows), 9800 + i))
    return out


@pytest.mark.parametrize("case", _prune_shapes(32, 20240723), ids=lambda c: "-".join(map(str, c[:7])))
def test_prune_random_shapes(case, thk_env, prune_launch):
    dtype, G, S, S_obs, T, ld, block_rows, seed = case
    print(f"prune case {case}", flush=True)
    if block_rows:
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", block_rows)
    L, B, N_kv = 1, 2, 3
    U = L * B * N_kv
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, seed, 1.0)
    k = _randn((L, B, N_kv, S, D), dtype, seed + 1, 1.0)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, ld, DT[dtype], 0)
    score, idx, kp = gpu_prune(shape, q_obs, k)
    o_sc, o_idx, _ = oracle_prune(q_obs, k, dtype, T, ld)
    o_sc = o_sc.reshape(U, D)
    rel = np.abs(score.cpu().numpy().astype(np.float64) - o_sc) / o_sc
    assert rel.max() <= SCORE_TOL, case
    check_idx_with_tie_rule(idx.cpu().numpy(), o_idx, o_sc, T)
    # compaction is judged with the list the call returned: bit-exact gather
    want = O.compact_keys(as_numpy(k).reshape(U, S, D), idx.cpu().numpy(), dtype, ld)
    np.testing.assert_array_equal(as_numpy(kp), want)   # padding columns stay zero on both sides


def _long_shapes(n, seed):
    """Longer sequences: units of 6 to 550 blocks (one and two levels of sums, launches of several
    rounds of resident blocks with the graded start), decode pieces of thousands of rows."""
    rng = np.random.default_rng(seed)
    prune, decode = [], []
    for i in range(n):
        dtype = "bf16" if rng.random() < 0.7 else "f32"
        S = int(rng.integers(3000, 70000))
        T = int(rng.choice([int(rng.integers(1, 129)), 51, 64, 76]))
        ld = 0 if rng.random() < 0.7 else min(128, T + int(rng.choice([1, 4, 8])))
        br = str(rng.choice(["", "", "", "128", "256", "512"]))
        if dtype == "f32" and br == "512":
            br = ""
        prune.append((dtype, int(rng.choice([1, 2, 4])), S, int(rng.choice([1, 32, 64])), T, ld, br, 12000 + i))
        G = int(rng.choice([1, 2, 3, 4, 5, 8, 16]))
        cap = int(rng.choice([0, 16, 64]))
        s_tail = int(rng.integers(0, cap + 1)) if cap else 0
        sigma = float(rng.choice([0.0, 1.0, 2.0]))
        decode.append((dtype, 1, int(rng.integers(1, 4)), G, int(rng.integers(3000, 60000)), T, ld,
                       int(rng.choice([0, 0, 0, 1, 3, 7, 100])), s_tail, cap, sigma,
                       13000 + i))
    return prune, decode


@pytest.mark.parametrize("case", _long_shapes(10, 20240725)[0], ids=lambda c: "-".join(map(str, c[:7])))
def test_prune_random_long_sequences(case, thk_env, prune_launch):
    test_prune_random_shapes(case, thk_env, prune_launch)


@pytest.mark.parametrize("case", _long_shapes(10, 20240725)[1], ids=lambda c: "-".join(map(str, c[:10])))
def test_decode_random_long_sequences(case, decode_merge):
    test_decode_random_shapes(case, decode_merge)


def _value_shapes(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        dtype = "bf16" if rng.random() < 0.75 else "f32"
        G = int(rng.choice([1, 1, 2, 3, 4, 8]))
        # at least 8 query rows per channel norm: with one or two rows the score is a bare signed sum
        # and the median criterion of the bf16 check (made for norms over many rows) does not apply
        S = int(rng.choice([int(rng.integers(8, 200)), int(rng.integers(200, 3000))]))
        S_obs = int(min(S, rng.choice([8, 16, 32, 64])))
        n_split = int(rng.choice([0, 0, 1, 2, 4]))
        causal = int(rng.integers(0, 2))
        sigma = float(rng.choice([0.0, 0.5, 1.0]))
        out.append((dtype, G, S_obs, S, n_split, causal, sigma))
    return out


@pytest.mark.parametrize("case", _value_shapes(20, 20240724), ids=lambda c: "-".join(map(str, c)))
def test_value_score_random_shapes(case):
    from test_gpu_value import test_value_score_matches_oracle
    dtype, G, S_obs, S, n_split, causal, sigma = case
    test_value_score_matches_oracle(G, S_obs, S, n_split, causal, sigma, dtype)
