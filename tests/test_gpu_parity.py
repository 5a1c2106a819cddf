"""GPU parity: every C-ABI entry point against the CPU fp64 oracle, element by
element, on seeded inputs that span several tiles and a ragged tail."""
import itertools

import numpy as np
import pytest
import torch

import paper_2407_21018_amd as thk
from oracle import oracle as O
from paper_2407_21018_amd.synth import as_numpy
from helpers import (ATTN_TOL, DT, SCORE_TOL, TDT, attn_rel_err, check_idx_with_tie_rule, gpu_compact,
                     gpu_decode, gpu_prune, gpu_score, gpu_select, oracle_prune, ws_tensor)

pytestmark = pytest.mark.gpu
D = 128


def _randn(shape, dtype, seed, scale_sigma=1.0, dev="cuda"):
    g = torch.Generator(device=dev); g.manual_seed(seed)
    x = torch.randn(*shape, generator=g, device=dev)
    if scale_sigma:
        sc = torch.exp(scale_sigma * torch.randn(shape[-1], generator=g, device=dev))
        x = x * sc
    return x.to(TDT[dtype])


# ----------------------------------------------------------------- score ----
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("G,n_split,S", [(1, 0, 1037), (4, 3, 1037), (2, 7, 600), (1, 1, 64), (1, 0, 5), (4, 64, 4100)])
def test_score_matches_oracle(dtype, G, n_split, S):
    L, B, N_kv, S_obs = 2, 2, 2, min(32, S)
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, 11)
    k = _randn((L, B, N_kv, S, D), dtype, 12)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, 64, 0, DT[dtype], n_split)
    got = gpu_score(shape, q_obs, k).cpu().numpy().astype(np.float64).reshape(L, B, N_kv, D)
    want = O.score(as_numpy(q_obs), as_numpy(k), dtype)
    rel = np.abs(got - want) / want
    print(f"score {dtype} G={G} split={n_split} S={S}: max rel err {rel.max():.3e}")
    assert rel.max() <= SCORE_TOL


MAGNITUDE_CASES = [
    # dtype, L, B, N_kv, S, n_split, sigma
    ("bf16", 1, 2, 3, 777, 0, 1.0),
    ("f32", 1, 2, 3, 777, 0, 1.0),
    ("bf16", 4, 2, 8, 4100, 0, 1.5),     # a layer stack in one call, several splits, ragged pieces
    ("f32", 3, 1, 5, 2049, 7, 2.0),
    ("bf16", 1, 1, 1, 5, 1, 0.0),        # shorter than one row group
    ("f32", 2, 1, 2, 33000, 0, 1.0),     # long units: fp32 chains folded into fp64 many times
]


@pytest.mark.parametrize("p", [1, 2])
@pytest.mark.parametrize("dtype,L,B,N_kv,S,n_split,sigma", MAGNITUDE_CASES)
def test_magnitude_score_matches_oracle(dtype, L, B, N_kv, S, n_split, sigma, p):
    """Eq. 1: M[n, d] = ||K[n, :, d]||_p, p = 1, 2, and the Top_T taken from it."""
    k = _randn((L, B, N_kv, S, D), dtype, 13 + S, sigma)
    shape = thk.make_shape(L, B, N_kv, N_kv, D, S, 1, 64, 0, DT[dtype], n_split)
    U = L * B * N_kv
    score = torch.empty(U, D, dtype=torch.float32, device="cuda")
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_SCORE))
    thk.thk_score_magnitude(shape, k, p, score, ws)
    torch.cuda.synchronize()
    want = O.score_magnitude(as_numpy(k), dtype, p).reshape(U, D)
    rel = np.abs(score.cpu().numpy().astype(np.float64) - want) / want
    assert rel.max() <= SCORE_TOL
    # I = Top_T(M, T): the list from the GPU's scores against the oracle's, up to exact-tolerance ties
    idx = gpu_select(shape, score).cpu().numpy()
    check_idx_with_tie_rule(idx, O.select_topk(want, 64), want, 64)


# ---------------------------------------------------------------- select ----
@pytest.mark.parametrize("T", [1, 2, 51, 63, 64, 65, 76, 127, 128])
def test_select_bit_exact_on_same_scores(T):
    """Both sides decide on the same fp32 scores: no tolerance."""
    U = 70
    g = torch.Generator(device="cuda"); g.manual_seed(100 + T)
    score = torch.randn(U, D, generator=g, device="cuda").abs()
    score[3] = score[3].round(decimals=1)      # many exact ties
    score[4] = 0.0                             # all equal
    score[5, ::2] = score[5, 1::2]             # duplicated pairs
    score[6] = torch.arange(D, device="cuda").float()        # ascending
    score[7] = torch.arange(D, 0, -1, device="cuda").float()  # descending
    shape = thk.make_shape(1, 1, U, U, D, 1, 1, T, 0, thk.THK_F32, 0)
    got = gpu_select(shape, score).cpu().numpy()
    want = O.select_topk(score.cpu().numpy().astype(np.float64), T)
    np.testing.assert_array_equal(got, want)


# --------------------------------------------------------------- compact ----
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("S,T,ld", [(1024, 64, 0), (1056, 76, 0), (2048 + 32, 51, 0), (1037, 51, 0), (1037, 76, 80),
                                     (520, 128, 0), (16, 1, 0), (3, 7, 0), (4096, 89, 0), (8, 51, 0),
                                     # padded rows, pitches that are and are not multiples of 16 bytes
                                     (300, 51, 56), (300, 51, 53), (64, 7, 8), (555, 100, 128), (33, 3, 8), (700, 89, 92)])
def test_compact_bit_exact(dtype, S, T, ld):
    L, B, N_kv = 1, 2, 3
    k = _randn((L, B, N_kv, S, D), dtype, 21)
    g = torch.Generator(device="cpu"); g.manual_seed(S + T)
    score = torch.rand(L * B * N_kv, D, generator=g).numpy().astype(np.float64)
    idx_np = O.select_topk(score, T)
    idx = torch.from_numpy(idx_np).cuda()
    shape = thk.make_shape(L, B, N_kv, N_kv, D, S, 1, T, ld, DT[dtype], 0)
    kp = gpu_compact(shape, k, idx, fill=7)            # every element of every row is written:
    want = O.compact_keys(as_numpy(k).reshape(L * B * N_kv, S, D), idx_np, dtype, ld)
    np.testing.assert_array_equal(as_numpy(kp), want)   # the padding columns as zeros


# ---------------------------------------------------------------- decode ----
def _decode_case(dtype, B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, seed):
    N_q = N_kv * G
    q = _randn((1, B, N_q, D), dtype, seed, sigma)
    k = _randn((1, B, N_kv, S, D), dtype, seed + 1, sigma)
    v = _randn((1, B, N_kv, S, D), dtype, seed + 2, 0)
    kt = _randn((1, B, N_kv, max(cap, 1), D), dtype, seed + 3, sigma)
    vt = _randn((1, B, N_kv, max(cap, 1), D), dtype, seed + 4, 0)
    g = torch.Generator(device="cpu"); g.manual_seed(seed + 5)
    idx_np = O.select_topk(torch.rand(B * N_kv, D, generator=g).numpy().astype(np.float64), T)
    idx = torch.from_numpy(idx_np).cuda()
    shape = thk.make_shape(1, B, N_q, N_kv, D, S, 1, T, ld, DT[dtype], n_split)
    kp = gpu_compact(shape, k, idx)
    out = gpu_decode(shape, q, kp, idx, v, kt if s_tail else None, vt if s_tail else None, s_tail, cap)
    U = B * N_kv
    ref = O.decode_attn(as_numpy(q)[0], as_numpy(kp).reshape(B, N_kv, S, -1), idx_np.reshape(B, N_kv, T),
                        as_numpy(v)[0], dtype, as_numpy(kt)[0] if s_tail else None,
                        as_numpy(vt)[0] if s_tail else None, s_tail)
    err = attn_rel_err(out, ref.reshape(B * N_q, D))
    return err, out


DECODE_CASES = [
    # B N_kv G   S    T   ld split tail cap sigma
    (2, 2, 1, 1037, 64, 0, 0, 0, 0, 1.0),
    (2, 2, 1, 1037, 76, 0, 0, 0, 0, 1.0),
    (2, 2, 1, 1037, 51, 0, 0, 0, 0, 1.0),
    (1, 2, 4, 1037, 64, 0, 3, 0, 0, 1.0),
    (1, 2, 4, 2048, 76, 0, 0, 17, 64, 1.0),
    (1, 1, 8, 1500, 51, 0, 2, 64, 64, 1.0),
    (1, 1, 3, 700, 64, 0, 0, 1, 4, 1.0),
    (1, 2, 2, 900, 89, 0, 7, 5, 16, 1.0),
    (1, 2, 1, 1, 64, 0, 0, 0, 0, 1.0),
    (1, 2, 1, 1, 64, 0, 0, 1, 1, 1.0),
    (1, 2, 1, 63, 128, 0, 0, 0, 0, 1.0),
    (1, 2, 1, 65, 1, 0, 0, 0, 0, 1.0),
    (1, 2, 1, 300, 7, 0, 2, 3, 8, 1.0),
    (1, 2, 1, 1037, 76, 80, 0, 0, 0, 1.0),
    (1, 2, 1, 1037, 51, 56, 4, 9, 16, 1.0),
    (2, 3, 1, 4096, 76, 0, 0, 0, 0, 0.0),      # diffuse softmax: V accumulation dominates
    (1, 2, 4, 8192, 64, 0, 64, 0, 0, 0.0),
    (1, 2, 1, 5000, 64, 0, 0, 33, 64, 2.0),    # heavy-tailed scales: near one-hot softmax
    # four query heads per KV head: bf16 takes the matrix-core kernel when T and ld are multiples of 4
    (1, 2, 4, 1037, 76, 80, 0, 0, 0, 1.0),     # padded rows
    (1, 1, 4, 333, 128, 0, 2, 7, 16, 1.0),     # nothing pruned: the wide staging class
    (1, 2, 4, 100, 4, 0, 0, 0, 0, 1.0),        # one chunk per row
    (1, 2, 4, 97, 8, 12, 0, 16, 16, 1.0),
    (1, 1, 8, 2100, 64, 0, 5, 33, 64, 0.0),    # two groups of four heads
    (1, 2, 4, 1, 64, 0, 0, 0, 0, 1.0),
    (1, 2, 4, 1, 64, 0, 0, 1, 1, 1.0),
    (1, 2, 4, 500, 64, 66, 0, 3, 8, 1.0),      # pitch not a multiple of 4: the general kernel
    (1, 1, 4, 4096, 76, 0, 0, 64, 64, 2.0),
    (1, 1, 4, 200, 124, 0, 0, 2, 4, 1.0),      # 248-byte rows: 8-byte aligned only
    (1, 1, 4, 200, 124, 128, 2, 0, 0, 1.0),    # the widest padded rows: pitch D
    (1, 2, 4, 555, 64, 128, 0, 5, 8, 0.0),     # kept channels at the front of full-width rows
    # eight query heads per KV head share one block (and every key / value byte)
    (1, 1, 16, 700, 76, 0, 0, 3, 8, 1.0),      # two blocks of eight heads
    (1, 2, 12, 400, 64, 0, 0, 0, 0, 1.0),      # 12 heads: three blocks of four
    (1, 1, 8, 333, 124, 128, 2, 5, 16, 1.0),   # the widest staging class
    (2, 2, 8, 4133, 76, 0, 0, 40, 64, 0.0),
    # head counts that do not fill the blocks' slots: the last block of a unit leaves some empty
    (1, 2, 3, 900, 64, 0, 2, 5, 16, 1.0),      # bf16: 3 of 4 matrix-core slots; f32: 3 of 4 general slots
    (1, 2, 5, 1300, 76, 0, 0, 0, 0, 1.0),      # 5 of 8
    (1, 1, 7, 650, 128, 0, 3, 17, 32, 0.0),    # 7 of 8, the wide staging class
    (1, 1, 9, 500, 64, 0, 0, 0, 0, 1.0),       # 8 + 1
    (1, 2, 6, 800, 51, 0, 2, 9, 16, 1.0),      # T not a multiple of 4: general kernel, 4 + 2
    (1, 2, 5, 300, 51, 56, 0, 0, 0, 1.0),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("case", DECODE_CASES, ids=lambda c: "-".join(map(str, c)))
def test_decode_matches_oracle(dtype, case, decode_merge):
    B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma = case
    err, _ = _decode_case(dtype, B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, 1000 + S + T)
    print(f"decode {dtype} {case}: max rel err {err.max():.3e}")
    assert err.max() <= ATTN_TOL[dtype]


@pytest.mark.parametrize("case", [c for c in DECODE_CASES if c[2] >= 3], ids=lambda c: "-".join(map(str, c)))
def test_decode_general_kernel_on_grouped_heads(case, thk_env, decode_merge):
    """THK_DECODE_MFMA=0 keeps bf16 shapes with three or more query heads per KV head on the general kernel."""
    thk_env.setenv("THK_DECODE_MFMA", "0")
    B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma = case
    err, out0 = _decode_case("bf16", B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, 1000 + S + T)
    assert err.max() <= ATTN_TOL["bf16"]
    thk_env.setenv("THK_DECODE_MFMA", "1")
    err1, out1 = _decode_case("bf16", B, N_kv, G, S, T, ld, n_split, s_tail, cap, sigma, 1000 + S + T)
    print(f"decode bf16 {case}: max rel err general {err.max():.3e}, matrix cores {err1.max():.3e}")
    assert err1.max() <= ATTN_TOL["bf16"]


@pytest.mark.parametrize("G,T,ld", [(4, 51, 52), (8, 89, 92), (3, 1, 4), (5, 38, 40), (8, 127, 128)])
def test_decode_ignores_whatever_sits_in_the_row_padding(G, T, ld):
    """Rows of T kept channels padded to a multiple of 4 elements run on the matrix-core kernel, which
    reads whole 4-element chunks: what the padding holds (here NaN) must not reach the logits."""
    B, N_kv, S, s_tail, cap = 1, 2, 1234, 7, 16
    N_q = N_kv * G
    q = _randn((1, B, N_q, D), "bf16", 31, 1.0)
    k = _randn((1, B, N_kv, S, D), "bf16", 32, 1.0)
    v = _randn((1, B, N_kv, S, D), "bf16", 33, 0)
    kt = _randn((1, B, N_kv, cap, D), "bf16", 34, 1.0)
    vt = _randn((1, B, N_kv, cap, D), "bf16", 35, 0)
    g = torch.Generator(device="cpu"); g.manual_seed(36)
    idx_np = O.select_topk(torch.rand(B * N_kv, D, generator=g).numpy().astype(np.float64), T)
    idx = torch.from_numpy(idx_np).cuda()
    shape = thk.make_shape(1, B, N_q, N_kv, D, S, 1, T, ld, thk.THK_BF16, 0)
    assert thk.thk_decode_on_matrix_cores(shape) == 1
    kp = gpu_compact(shape, k, idx)
    kp[:, :, T:] = float("nan")
    out = gpu_decode(shape, q, kp, idx, v, kt, vt, s_tail, cap)
    ref = O.decode_attn(as_numpy(q)[0], as_numpy(kp).reshape(B, N_kv, S, -1), idx_np.reshape(B, N_kv, T),
                        as_numpy(v)[0], "bf16", as_numpy(kt)[0], as_numpy(vt)[0], s_tail)
    err = attn_rel_err(out, ref.reshape(B * N_q, D))
    assert np.isfinite(out.float().cpu().numpy()).all()
    assert err.max() <= ATTN_TOL["bf16"]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_decode_split_invariance_and_determinism(dtype, decode_merge):
    outs = {}
    for n_split in (1, 2, 7, 64):
        err, out = _decode_case(dtype, 1, 2, 4, 8192 + 100, 64, 0, n_split, 11, 16, 1.0, 77)
        assert err.max() <= ATTN_TOL[dtype]
        _, out2 = _decode_case(dtype, 1, 2, 4, 8192 + 100, 64, 0, n_split, 11, 16, 1.0, 77)
        assert torch.equal(out, out2), "two runs must be bit-identical (no atomics)"
        outs[n_split] = out.float()
    ref = outs[1]
    for n_split, o in outs.items():
        rel = ((o - ref).abs().amax(-1) / ref.abs().amax(-1)).max().item()
        assert rel <= ATTN_TOL[dtype], f"n_split={n_split} deviates by {rel}"


@pytest.mark.parametrize("dtype,G,S,tail", [("bf16", 1, 1000, 0), ("bf16", 4, 70000, 9), ("f32", 2, 300, 3)])
def test_decode_with_the_largest_split_count(dtype, G, S, tail):
    """n_split = 4096, the most the interface takes: nearly every piece is empty (64 rows per piece
    at least, so S = 70000 fills 1094 of them and S = 300 five); empty pieces must carry a weight
    of zero into the merge, and the tail tiles go to pieces that have no pruned rows at all."""
    err, out = _decode_case(dtype, 1, 2, G, S, 64, 0, 4096, tail, 16, 1.0, 123)
    assert np.isfinite(out.float().cpu().numpy()).all()
    assert err.max() <= ATTN_TOL[dtype]
    _, out1 = _decode_case(dtype, 1, 2, G, S, 64, 0, 1, tail, 16, 1.0, 123)
    rel = ((out.float() - out1.float()).abs().amax(-1) / out1.float().abs().amax(-1)).max().item()
    assert rel <= ATTN_TOL[dtype]


# ----------------------------------------------------------------- prune ----
PRUNE_CASES = [("bf16", 1, 2048, 76, 1.5), ("bf16", 4, 4096 + 64, 64, 1.0), ("f32", 1, 1037, 64, 1.0),
               ("bf16", 1, 1024, 51, 2.0), ("f32", 2, 2048, 64, 1.0), ("bf16", 1, 40, 64, 1.0)]


@pytest.mark.parametrize("levels", [1, 2])
def test_prune_fused_repeated_calls_on_one_workspace(levels, thk_env, prune_launch):
    """The one-launch form hands sums and index lists from block to block through the
    workspace (one level: the last block's list to the blocks that wait; two levels: the group
    vectors to every block of the unit).  Calls that alternate between two inputs on the SAME
    workspace leave the other input's words behind each time: a block that picked up stale
    words (or words that had not fully arrived) would compact the wrong channels.  Checked
    on the GPU against a plain gather with the index list the call returned, and against the
    oracle's list for the first call of each input."""
    thk_env.setenv("THK_PRUNE_PATH", "fused")
    if levels == 1:
        L, B, N, S, S_obs, T = 4, 4, 16, 4096, 32, 76
    else:                                          # 102 blocks of 128 rows per unit
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", "128")
        L, B, N, S, S_obs, T = 1, 3, 4, 13008, 32, 64
    U = L * B * N
    shape = thk.make_shape(L, B, N, N, D, S, S_obs, T, 0, thk.THK_BF16, 0)
    assert thk.thk_prune_is_fused(shape) == 2      # the form that keeps the rows on chip
    inputs = [(_randn((L, B, N, S_obs, D), "bf16", 71 + i, 1.0), _randn((L, B, N, S, D), "bf16", 81 + i, 1.0))
              for i in range(2)]
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_PRUNE))
    ws.fill_(0xA5)
    score = torch.empty(U, D, dtype=torch.float32, device="cuda")
    idx = torch.empty(U, T, dtype=torch.int16, device="cuda")
    kp = torch.empty(U, S, T, dtype=torch.bfloat16, device="cuda")
    first_idx = {}
    for rep in range(8):
        q_obs, k = inputs[rep % 2]
        kp.fill_(-7.0)
        thk.thk_prune(shape, q_obs, k, score, idx, kp, ws)
        torch.cuda.synchronize()
        want = torch.gather(k.reshape(U, S, D), 2, idx.to(torch.int64)[:, None, :].expand(U, S, T))
        assert torch.equal(kp.view(torch.int16), want.view(torch.int16)), f"call {rep}"
        if rep < 2:
            first_idx[rep] = idx.clone()
            o_sc = O.score(as_numpy(q_obs), as_numpy(k), "bf16").reshape(U, D)
            check_idx_with_tie_rule(idx.cpu().numpy(), O.select_topk(o_sc, T), o_sc, T)
        else:
            assert torch.equal(idx, first_idx[rep % 2]), f"call {rep}"
    assert not torch.equal(first_idx[0], first_idx[1])


@pytest.mark.parametrize("levels", [1, 2])
@pytest.mark.parametrize("delay_us", [30, 200])
def test_prune_single_launch_with_a_late_prologue(levels, delay_us, thk_env):
    """The single-launch prune initialises its hand-off state inside the launch: a prologue block
    per unit clears it and then tags the unit's arrival counters with the call's nonce; a row
    block that arrives earlier finds a foreign tag, waits for the right one and arrives again.
    Here the prologue is held back from the host (THK_PRUNE_PROLOGUE_DELAY_US) so that EVERY row
    block arrives first -- on a workspace full of garbage, on the state the previous call left,
    and with the wait for the index list switched off as well (spin limit 0: the blocks give up
    and the unit's finisher compacts their rows).  Every kernel exits normally; results as ever."""
    thk_env.setenv("THK_PRUNE_LAUNCH", "solo")
    thk_env.setenv("THK_PRUNE_PROLOGUE_DELAY_US", str(delay_us))
    if levels == 1:
        L, B, N, G, S, S_obs, T = 2, 2, 4, 2, 3000, 32, 76
    else:                                          # 102 blocks of 128 rows per unit: two levels of sums
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", "128")
        L, B, N, G, S, S_obs, T = 1, 2, 2, 1, 13008, 32, 64
    U = L * B * N
    shape = thk.make_shape(L, B, N * G, N, D, S, S_obs, T, 0, thk.THK_BF16, 0)
    assert thk.thk_prune_launches(shape) == 1
    ws = ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_PRUNE))
    score = torch.empty(U, D, dtype=torch.float32, device="cuda")
    idx = torch.empty(U, T, dtype=torch.int16, device="cuda")
    kp = torch.empty(U, S, T, dtype=torch.bfloat16, device="cuda")
    for rep, (fill, spin) in enumerate([(0xA5, None), (None, None), (0xFF, "0"), (None, "0"), (0x00, None)]):
        if fill is not None:
            ws.fill_(fill)
        if spin is not None:
            thk_env.setenv("THK_PRUNE_SPIN_LIMIT", spin)
        q_obs = _randn((L, B, N * G, S_obs, D), "bf16", 171 + rep, 1.0)
        k = _randn((L, B, N, S, D), "bf16", 181 + rep, 1.0)
        kp.fill_(-7.0)
        thk.thk_prune(shape, q_obs, k, score, idx, kp, ws)
        torch.cuda.synchronize()
        o_sc, o_idx, _ = oracle_prune(q_obs, k, "bf16", T)
        rel = np.abs(score.cpu().numpy().astype(np.float64) - o_sc.reshape(U, D)) / o_sc.reshape(U, D)
        assert rel.max() <= SCORE_TOL, f"call {rep}"
        check_idx_with_tie_rule(idx.cpu().numpy(), o_idx, o_sc, T)
        want = O.compact_keys(as_numpy(k).reshape(U, S, D), idx.cpu().numpy(), "bf16")
        np.testing.assert_array_equal(as_numpy(kp), want, err_msg=f"call {rep}")


@pytest.mark.parametrize("dtype,G,S,T,ld,block_rows", [("bf16", 1, 4096, 76, 80, ""), ("bf16", 4, 3001, 51, 56, "128"),
                                                       ("f32", 1, 1037, 51, 52, ""), ("bf16", 1, 2048, 76, 88, "64"),
                                                       ("bf16", 2, 777, 100, 104, "32"), ("bf16", 1, 1500, 76, 77, "")])
def test_prune_into_padded_rows(dtype, G, S, T, ld, block_rows, thk_env, prune_launch):
    """K_pruned rows with padding behind them, whatever the pitch: the one-launch prune serves them
    and the padding columns are written as zeros."""
    if block_rows:
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", block_rows)
    L, B, N_kv, S_obs = 1, 2, 3, 32
    U = L * B * N_kv
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, 61, 1.0)
    k = _randn((L, B, N_kv, S, D), dtype, 62, 1.0)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, ld, DT[dtype], 0)
    assert thk.thk_prune_is_fused(shape) != 0
    score = torch.empty(U, D, dtype=torch.float32, device="cuda")
    idx = torch.empty(U, T, dtype=torch.int16, device="cuda")
    kp = torch.full((U, S, ld), 7, dtype=k.dtype, device="cuda")
    thk.thk_prune(shape, q_obs, k, score, idx, kp, ws_tensor(thk.thk_workspace_bytes(shape, thk.THK_OP_PRUNE)))
    torch.cuda.synchronize()
    o_sc, o_idx, _ = oracle_prune(q_obs, k, dtype, T, ld)
    check_idx_with_tie_rule(idx.cpu().numpy(), o_idx, o_sc.reshape(U, D), T)
    want = O.compact_keys(as_numpy(k).reshape(U, S, D), idx.cpu().numpy(), dtype, ld)   # zeros in the padding
    np.testing.assert_array_equal(as_numpy(kp), want)


@pytest.mark.parametrize("spin_limit", [None, 0])
@pytest.mark.parametrize("block_rows,S", [(128, 13008), (64, 13008), (128, 40016)])
def test_prune_two_level_arrival(block_rows, S, spin_limit, thk_env, prune_launch):
    """Units of more than 64 row blocks: the blocks arrive group by group, the last block of a
    group publishes the group's sums, and every block makes the index list from the group sums
    (102 blocks of 128 rows held on chip; 204 blocks of 64 rows read twice).  With the wait
    switched off from the host, blocks that find a group vector missing leave their rows, and
    possibly the caller's copy of the list, to the repair kernel."""
    thk_env.setenv("THK_PRUNE_PATH", "fused")
    thk_env.setenv("THK_PRUNE_BLOCK_ROWS", str(block_rows))
    if spin_limit is not None:
        thk_env.setenv("THK_PRUNE_SPIN_LIMIT", str(spin_limit))
    L, B, N_kv, G, S_obs, T = 1, 2, 2, 2, 32, 64       # S = 40016: 313 blocks per unit, groups of 20
    q_obs = _randn((L, B, N_kv * G, S_obs, D), "bf16", 41, 1.0)
    k = _randn((L, B, N_kv, S, D), "bf16", 42, 1.0)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, 0, thk.THK_BF16, 0)
    assert thk.thk_prune_is_fused(shape) == (2 if block_rows == 128 else 1)
    score, idx, kp = gpu_prune(shape, q_obs, k)
    o_sc, o_idx, o_kp = oracle_prune(q_obs, k, "bf16", T)
    U = L * B * N_kv
    rel = np.abs(score.cpu().numpy().astype(np.float64) - o_sc.reshape(U, D)) / o_sc.reshape(U, D)
    assert rel.max() <= SCORE_TOL
    check_idx_with_tie_rule(idx.cpu().numpy(), o_idx, o_sc, T)
    np.testing.assert_array_equal(as_numpy(kp), O.compact_keys(as_numpy(k).reshape(U, S, D), idx.cpu().numpy(), "bf16"))


@pytest.mark.parametrize("path", ["fused", "fused-small-blocks", "fused-no-wait", "hold-128", "hold-256", "hold-512",
                                  "hold-256-no-wait", "reread-256", "staged", "staged-groups"])
@pytest.mark.parametrize("dtype,G,S,T,sigma", PRUNE_CASES)
def test_prune_pipeline_matches_oracle(dtype, G, S, T, sigma, path, thk_env, prune_launch):
    """thk_prune in its one-launch form (default row blocks, 32-row blocks, and with
    the wait for the index list switched off from the host so that the repair
    kernel does every compaction) and in its staged form (one group, many groups)."""
    if prune_launch == "solo" and not (path.startswith("hold") or path in ("fused", "fused-no-wait")):
        pytest.skip("the single-launch form exists only where the rows are held on chip")
    if path.startswith("fused") or path.startswith("hold"):
        thk_env.setenv("THK_PRUNE_PATH", "fused")
    if path.startswith("hold"):      # row blocks that stay in registers between score and compaction
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", path.split("-")[1])
    if path == "hold-256-no-wait":
        thk_env.setenv("THK_PRUNE_SPIN_LIMIT", "0")
    if path == "reread-256":         # the same blocking with the rows read twice
        thk_env.setenv("THK_PRUNE_PATH", "reread")
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", "256")
    if path == "fused-small-blocks":
        thk_env.setenv("THK_PRUNE_BLOCK_ROWS", "32")
    if path == "fused-no-wait":
        thk_env.setenv("THK_PRUNE_SPIN_LIMIT", "0")
    if path.startswith("staged"):
        thk_env.setenv("THK_PRUNE_PATH", "staged")
    if path == "staged-groups":
        thk_env.setenv("THK_PRUNE_GROUP_MIB", "1")     # several groups, some starting mid-batch
    L, B, N_kv, S_obs = 2, 2, 3, min(32, S)
    q_obs = _randn((L, B, N_kv * G, S_obs, D), dtype, 31, sigma)
    k = _randn((L, B, N_kv, S, D), dtype, 32, sigma)
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, 0, DT[dtype], 0)
    score, idx, kp = gpu_prune(shape, q_obs, k)
    o_sc, o_idx, o_kp = oracle_prune(q_obs, k, dtype, T)
    U = L * B * N_kv
    rel = np.abs(score.cpu().numpy().astype(np.float64) - o_sc.reshape(U, D)) / o_sc.reshape(U, D)
    assert rel.max() <= SCORE_TOL
    differing = check_idx_with_tie_rule(idx.cpu().numpy(), o_idx, o_sc, T)
    kp_np, o_kp = as_numpy(kp), o_kp.reshape(U, S, T)
    same = [u for u in range(U) if u not in differing]
    np.testing.assert_array_equal(kp_np[same], o_kp[same])
    # the compacted keys are exactly the gather with the index list the call itself produced
    np.testing.assert_array_equal(kp_np, O.compact_keys(as_numpy(k).reshape(U, S, D), idx.cpu().numpy(), dtype))
    # the separate entry points: same bits as the staged call; the one-launch form sums the
    # partial column sums in another order, so its scores may differ in the last float bit
    sc2 = gpu_score(shape, q_obs, k)
    idx2 = gpu_select(shape, sc2)
    kp2 = gpu_compact(shape, k, idx2)
    if path.startswith("staged"):
        assert torch.equal(sc2, score) and torch.equal(idx2, idx) and torch.equal(kp2, kp)
    else:
        assert ((sc2 - score).abs() <= 2.4e-7 * score.abs()).all()
    # a second call on the same workspace gives the same bits (counters are reset per call)
    score_b, idx_b, kp_b = gpu_prune(shape, q_obs, k)
    assert torch.equal(score_b, score) and torch.equal(idx_b, idx) and torch.equal(kp_b, kp)


@pytest.mark.parametrize("pattern", ["pairs", "all-equal", "blocks-of-16", "half-zero"])
@pytest.mark.parametrize("T", [1, 2, 51, 64, 65, 127, 128])
def test_prune_breaks_exact_ties_by_channel_number(pattern, T, prune_launch):
    """Channels that are copies of each other score the same to the last bit (on the GPU and in the
    oracle alike), so Top_T has to fall back on its tie rule -- the lower channel number wins
    (Sec. 3.2's Top_T is silent on ties; the stable order is this build's reading).  The whole
    prune call must then give exactly the oracle's list: with pairs of copies, with 16 copies
    of each of 8 columns (the T-th place falls inside a run of equal scores for most T), and with
    128 equal channels (the list is 0 .. T-1); and with 64 channels that are zero everywhere
    (scores of exactly 0, the smallest key there is: for T > 64 the list ends with the lowest zeros)."""
    L, B, N_kv, G, S, S_obs = 1, 2, 3, 2, 777, 32
    src = {"pairs": torch.arange(D) // 2 * 2, "all-equal": torch.zeros(D, dtype=torch.long),
           "blocks-of-16": torch.arange(D) % 8, "half-zero": torch.arange(D)}[pattern].cuda()
    q_obs = _randn((L, B, N_kv * G, S_obs, D), "bf16", 41)[..., src].contiguous()
    k = _randn((L, B, N_kv, S, D), "bf16", 42)[..., src].contiguous()
    if pattern == "half-zero":      # every third and every fourth channel all zero: 64 scores of exactly +0
        k[..., (torch.arange(D) % 4 >= 2).cuda()] = 0
    shape = thk.make_shape(L, B, N_kv * G, N_kv, D, S, S_obs, T, 0, thk.THK_BF16, 0)
    score, idx, kp = gpu_prune(shape, q_obs, k)
    o_sc, o_idx, o_kp = oracle_prune(q_obs, k, "bf16", T)
    U = L * B * N_kv
    sc = score.cpu().numpy()
    assert (sc == sc[:, src.cpu().numpy()]).all(), "copies of a channel must score the same bits"
    np.testing.assert_array_equal(idx.cpu().numpy(), o_idx.reshape(U, T))
    np.testing.assert_array_equal(as_numpy(kp), o_kp.reshape(U, S, T))


def test_tail_append():
    L, B, N_kv, cap = 1, 3, 5, 8
    shape = thk.make_shape(L, B, N_kv, N_kv, D, 16, 1, 64, 0, thk.THK_BF16, 0)
    kt = torch.zeros(L * B * N_kv, cap, D, dtype=torch.bfloat16, device="cuda"); vt = torch.zeros_like(kt)
    news = []
    for j in range(cap):
        kn = _randn((L * B * N_kv, D), "bf16", 50 + j); vn = _randn((L * B * N_kv, D), "bf16", 90 + j)
        thk.thk_tail_append(shape, kn, vn, kt, vt, j, cap)
        news.append((kn, vn))
    torch.cuda.synchronize()
    for j, (kn, vn) in enumerate(news):
        assert torch.equal(kt[:, j], kn) and torch.equal(vt[:, j], vn)
    with pytest.raises(thk.ThkError):
        thk.thk_tail_append(shape, news[0][0], news[0][1], kt, vt, cap, cap)


def test_device_is_the_one_the_kernels_are_written_for():
    """gfx950: 256 compute units, 64-wide wavefronts, 160 KB of LDS per workgroup at most."""
    p = torch.cuda.get_device_properties(0)
    assert p.gcnArchName.startswith("gfx950")
    assert p.multi_processor_count == 256 and p.warp_size == 64
    assert p.shared_memory_per_block == 160 * 1024
    assert p.total_memory >= 256 * 2**30
