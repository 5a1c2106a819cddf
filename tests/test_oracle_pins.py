"""Pins of the CPU fp64 oracle against what the paper and the mathematics fix.

None of these checks re-types an oracle formula: each compares an oracle
routine with an explicit matrix computation done by a numpy/scipy library
routine, a closed form, an invariant, or a value from the paper.
"""
import itertools
import os

import numpy as np
import pytest
import scipy.special

from oracle import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
rng = np.random.default_rng(20240721)


def _rand(shape, dtype):
    x = rng.standard_normal(shape)
    if dtype == "f64":
        return x, x
    if dtype == "f32":
        x32 = x.astype(np.float32)
        return x32, x32.astype(np.float64)
    bits = O.bf16_bits(x.astype(np.float32))
    return bits, O.bf16_to_f64(bits)


# ---------------------------------------------------------------- score ----
@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
@pytest.mark.parametrize("G", [1, 2, 4])
def test_score_is_frobenius_norm_of_explicit_rank1_matrix(dtype, G):
    """Sec. 3.2: Score[j] = ||Q[-S_obs:, j] K[:, j]^T||_F, summed over the G
    query heads of a KV head.  numpy builds each S_obs x S matrix and takes
    its Frobenius norm with the library routine."""
    L, B, N_kv, S, S_obs, D = 2, 2, 2, 13, 3, 6
    q_raw, q = _rand((L, B, N_kv * G, S_obs, D), dtype)
    k_raw, k = _rand((L, B, N_kv, S, D), dtype)
    want = np.zeros((L, B, N_kv, D))
    for l, b, h, c in itertools.product(range(L), range(B), range(N_kv), range(D)):
        for g in range(G):
            M = np.outer(q[l, b, h * G + g, :, c], k[l, b, h, :, c])
            want[l, b, h, c] += np.linalg.norm(M, "fro")
    got = O.score(q_raw, k_raw, dtype)
    brute = O.score(q_raw, k_raw, dtype, brute=True)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    np.testing.assert_allclose(brute, want, rtol=1e-12)


def test_score_closed_form_constant_columns():
    """Columns constant in the token axis: ||a 1||*||b 1|| = |a b| sqrt(S_obs S), times G."""
    L, B, N_kv, G, S, S_obs, D = 1, 1, 2, 2, 40, 5, 8
    a = rng.standard_normal(D)
    b = rng.standard_normal(D)
    q = np.broadcast_to(a, (L, B, N_kv * G, S_obs, D)).copy()
    k = np.broadcast_to(b, (L, B, N_kv, S, D)).copy()
    got = O.score(q, k, "f64")
    want = G * np.abs(a * b) * np.sqrt(S_obs * S)
    np.testing.assert_allclose(got, np.broadcast_to(want, got.shape), rtol=1e-13)


def test_score_equivariances():
    L, B, N_kv, G, S, S_obs, D = 1, 2, 2, 2, 17, 4, 8
    q = rng.standard_normal((L, B, N_kv * G, S_obs, D))
    k = rng.standard_normal((L, B, N_kv, S, D))
    base = O.score(q, k, "f64")
    # scaling one key channel scales its score by |alpha| and no other
    k2 = k.copy(); k2[..., 3] *= -2.5
    s2 = O.score(q, k2, "f64")
    np.testing.assert_allclose(s2[..., 3], 2.5 * base[..., 3], rtol=1e-13)
    np.testing.assert_allclose(np.delete(s2, 3, -1), np.delete(base, 3, -1), rtol=0)
    # channel permutation permutes scores
    perm = rng.permutation(D)
    np.testing.assert_allclose(O.score(q[..., perm], k[..., perm], "f64"), base[..., perm], rtol=0)
    # key-row permutation and sign flips leave scores unchanged
    rows = rng.permutation(S)
    signs = rng.choice([-1.0, 1.0], size=(S, 1))
    np.testing.assert_allclose(O.score(q, k[..., rows, :] * signs, "f64"), base, rtol=1e-13)
    # the observation window is the whole of Q_obs: dropping a query row changes the score
    assert not np.allclose(O.score(q[..., 1:, :], k, "f64"), base)
    # units are independent: changing unit (0,1,1) leaves every other unit alone
    k3 = k.copy(); k3[0, 1, 1] *= 3.0
    s3 = O.score(q, k3, "f64")
    np.testing.assert_allclose(s3[0, 1, 1], 3 * base[0, 1, 1], rtol=1e-13)
    np.testing.assert_array_equal(s3[0, 0], base[0, 0]); np.testing.assert_array_equal(s3[0, 1, 0], base[0, 1, 0])


def test_score_gqa_is_sum_of_per_head_norms_not_stacked_norm():
    """Convention of this build for grouped-query attention (the paper's
    formula is per head): per-head Frobenius norms are added."""
    q = np.zeros((1, 1, 2, 1, 2)); k = np.ones((1, 1, 1, 1, 2))
    q[0, 0, 0, 0, 0] = 3.0; q[0, 0, 1, 0, 0] = 4.0
    got = O.score(q, k, "f64")
    assert got[0, 0, 0, 0] == 7.0 and got[0, 0, 0, 1] == 0.0  # stacked norm would give 5


@pytest.mark.parametrize("p", [1, 2])
def test_magnitude_score_matches_numpy_norm(p):
    """Eq. 1: M[n,d] = ||K[n,:,d]||_p."""
    k = rng.standard_normal((3, 2, 19, 8))
    np.testing.assert_allclose(O.score_magnitude(k, "f64", p),
                               np.linalg.norm(k, ord=p, axis=-2), rtol=1e-13)


# --------------------------------------------------------------- select ----
def _argsort_topk(score, T):
    order = np.argsort(-score, axis=-1, kind="stable")[..., :T]
    return np.sort(order, axis=-1).astype(np.int16)


@pytest.mark.parametrize("T", [1, 5, 51, 64, 76, 127, 128])
def test_select_matches_stable_argsort(T):
    sc = np.abs(rng.standard_normal((3, 4, 128)))
    np.testing.assert_array_equal(O.select_topk(sc, T), _argsort_topk(sc, T))


def test_select_ties_go_to_lower_index():
    sc = np.zeros((1, 128))
    sc[0, [7, 19, 100]] = 2.0          # three-way tie at the top
    sc[0, [3, 50]] = 1.0               # two-way tie below
    np.testing.assert_array_equal(O.select_topk(sc, 2)[0], [7, 19])
    np.testing.assert_array_equal(O.select_topk(sc, 4)[0], [3, 7, 19, 100])
    # zero-score channels are ordinary ties: lowest indices fill the remainder
    np.testing.assert_array_equal(O.select_topk(sc, 8)[0], [0, 1, 2, 3, 7, 19, 50, 100])
    np.testing.assert_array_equal(O.select_topk(sc, 8), _argsort_topk(sc, 8))
    # duplicated channels
    sc = np.tile(np.abs(rng.standard_normal(64)), 2)[None]
    np.testing.assert_array_equal(O.select_topk(sc, 64), _argsort_topk(sc, 64))
    np.testing.assert_array_equal(O.select_topk(sc, 128)[0], np.arange(128))
    assert O.select_topk(sc, 1)[0, 0] == int(np.argmax(sc[0]))


def test_keep_count_floor():
    """T = floor((1 - lambda) D) (Sec. 3.1; Eq. 2 constraint)."""
    assert [O.keep_count(128, l) for l in (0.0, 0.3, 0.4, 0.5, 0.6, 0.75)] == [128, 89, 76, 64, 51, 32]
    assert O.keep_count(10, 0.3) == 7 and O.keep_count(8, 0.99) == 0
    assert O.keep_count(128, 1.0) == -1 and O.keep_count(128, -0.1) == -1


# -------------------------------------------------------------- compact ----
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_compact_is_numpy_take(dtype):
    k_raw, _ = _rand((2, 3, 11, 16), dtype)
    sc = np.abs(rng.standard_normal((2, 3, 16)))
    idx = O.select_topk(sc, 6)
    got = O.compact_keys(k_raw, idx, dtype)
    want = np.take_along_axis(k_raw, np.broadcast_to(idx[..., None, :].astype(np.int64), (2, 3, 11, 6)), axis=-1)
    np.testing.assert_array_equal(got, want)
    padded = O.compact_keys(k_raw, idx, dtype, ld_keep=8)
    np.testing.assert_array_equal(padded[..., :6], want)
    assert not padded[..., 6:].any()


# ---------------------------------------------- selection <-> objective ----
def _objective_numpy(Q, K, keep):
    S = np.diag(keep.astype(np.float64))
    return np.linalg.norm(Q @ K.T - Q @ S @ K.T, "fro")


def test_objective_routine_matches_numpy():
    Q = rng.standard_normal((4, 8)); K = rng.standard_normal((9, 8))
    keep = rng.integers(0, 2, 8).astype(np.uint8)
    assert O.objective(Q, K, keep) == pytest.approx(_objective_numpy(Q, K, keep), rel=1e-12)
    assert O.objective(Q, K, np.ones(8, np.uint8)) == 0.0


def test_objective_bounded_by_pruned_scores():
    """Eq. 2: the residual Q K^T - Q S K^T is the sum of the pruned channels'
    rank-1 terms, so its norm is at most the sum of their scores."""
    D, S, S_obs = 8, 12, 3
    for T in range(1, D):
        Q = rng.standard_normal((S_obs, D)) * np.exp(rng.standard_normal(D))
        K = rng.standard_normal((S, D)) * np.exp(rng.standard_normal(D))
        sc = O.score(Q[None, None, None], K[None, None, None], "f64")[0, 0, 0]
        idx = O.select_topk(sc[None], T)[0]
        keep = np.zeros(D, np.uint8); keep[idx] = 1
        err = _objective_numpy(Q, K, keep)
        assert err <= sc[keep == 0].sum() * (1 + 1e-12)
        # greedy keeps the largest scores: no pruned channel outranks a kept one
        assert sc[keep == 0].max() <= sc[keep == 1].min()


def test_single_pruned_channel_is_exact_and_optimal():
    """With T = D-1 one rank-1 term is dropped, so the objective equals that
    channel's score and Top_T reaches the true minimum of Eq. 2."""
    D, S, S_obs = 8, 10, 4
    Q = rng.standard_normal((S_obs, D)); K = rng.standard_normal((S, D))
    sc = O.score(Q[None, None, None], K[None, None, None], "f64")[0, 0, 0]
    idx = O.select_topk(sc[None], D - 1)[0]
    keep = np.zeros(D, np.uint8); keep[idx] = 1
    errs = []
    for j in range(D):
        kj = np.ones(D, np.uint8); kj[j] = 0
        errs.append(_objective_numpy(Q, K, kj))
    np.testing.assert_allclose(errs, sc, rtol=1e-12)
    assert _objective_numpy(Q, K, keep) == pytest.approx(min(errs), rel=1e-12)
    assert int(np.argmin(errs)) == int(np.flatnonzero(keep == 0)[0])


# --------------------------------------------------------------- decode ----
def _textbook(q, K, V):
    """softmax(q K^T / sqrt(D)) V for one head, numpy + scipy softmax."""
    D = q.shape[-1]
    return scipy.special.softmax(K @ q / np.sqrt(D)) @ V


def _setup(dtype, B=2, N_kv=2, G=2, S=37, D=16, T=7, cap=5, scale=1.0):
    q_raw, q = _rand((B, N_kv * G, D), dtype)
    k_raw, k = _rand((B, N_kv, S, D), dtype)
    v_raw, v = _rand((B, N_kv, S, D), dtype)
    kt_raw, kt = _rand((B, N_kv, cap, D), dtype)
    vt_raw, vt = _rand((B, N_kv, cap, D), dtype)
    sc = np.abs(rng.standard_normal((B, N_kv, D)))
    idx = O.select_topk(sc, T)
    return dict(q=(q_raw, q), k=(k_raw, k), v=(v_raw, v), kt=(kt_raw, kt), vt=(vt_raw, vt), idx=idx)


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
def test_decode_unpruned_equals_textbook_attention(dtype):
    """T = D (lambda = 0): plain softmax(q K^T / sqrt(D)) V."""
    B, N_kv, G, S, D = 2, 2, 2, 37, 16
    d = _setup(dtype, B, N_kv, G, S, D, T=D)
    np.testing.assert_array_equal(d["idx"], np.broadcast_to(np.arange(D), (B, N_kv, D)))
    kp = O.compact_keys(d["k"][0], d["idx"], dtype)
    got = O.decode_attn(d["q"][0], kp, d["idx"], d["v"][0], dtype)
    for b, n in itertools.product(range(B), range(N_kv * G)):
        want = _textbook(d["q"][1][b, n], d["k"][1][b, n // G], d["v"][1][b, n // G])
        np.testing.assert_allclose(got[b, n], want, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("dtype", ["f64", "bf16"])
@pytest.mark.parametrize("s_tail", [0, 1, 5])
def test_decode_pruned_two_segment_equals_textbook_on_masked_keys(dtype, s_tail):
    """Sec. 3.3: pruned query x pruned keys, full query x unpruned keys,
    logits concatenated.  Equivalent: textbook attention, full D and divisor
    sqrt(D), over [K * mask ; K_tail] and [V ; V_tail]."""
    B, N_kv, G, S, D, T = 2, 2, 2, 37, 16, 7
    d = _setup(dtype, B, N_kv, G, S, D, T)
    kp = O.compact_keys(d["k"][0], d["idx"], dtype)
    got = O.decode_attn(d["q"][0], kp, d["idx"], d["v"][0], dtype,
                        d["kt"][0], d["vt"][0], s_tail)
    for b, n in itertools.product(range(B), range(N_kv * G)):
        h = n // G
        mask = np.zeros(D); mask[d["idx"][b, h]] = 1.0
        K = np.concatenate([d["k"][1][b, h] * mask, d["kt"][1][b, h, :s_tail]])
        V = np.concatenate([d["v"][1][b, h], d["vt"][1][b, h, :s_tail]])
        np.testing.assert_allclose(got[b, n], _textbook(d["q"][1][b, n], K, V), rtol=1e-11, atol=1e-13)
    if s_tail:
        # the tail really enters: dropping it changes the output
        no_tail = O.decode_attn(d["q"][0], kp, d["idx"], d["v"][0], dtype)
        assert not np.allclose(no_tail, got)


def test_decode_closed_forms():
    B, N_kv, G, S, D, T = 1, 1, 1, 9, 8, 4
    idx = np.array([[[0, 2, 5, 7]]], np.int16)
    q = rng.standard_normal((B, 1, D)); v = rng.standard_normal((B, 1, S, D))
    # identical keys: uniform weights, output = mean of V rows
    k = np.broadcast_to(rng.standard_normal(D), (B, 1, S, D)).copy()
    out = O.decode_attn(q, O.compact_keys(k, idx, "f64"), idx, v, "f64")
    np.testing.assert_allclose(out[0, 0], v[0, 0].mean(0), rtol=1e-13)
    # one key: output is its value row
    out = O.decode_attn(q, O.compact_keys(k[:, :, :1], idx, "f64"), idx, v[:, :, :1], "f64")
    np.testing.assert_allclose(out[0, 0], v[0, 0, 0], rtol=1e-15)
    # two keys, logits a*x/sqrt(D) and 0: weights are a logistic function.
    # The divisor is sqrt of the ORIGINAL D (8), not of the kept count (4).
    a, x = 1.7, 2.3
    q2 = np.zeros((1, 1, D)); q2[0, 0, 2] = a; q2[0, 0, 1] = 50.0   # channel 1 is pruned: ignored
    k2 = np.zeros((1, 1, 2, D)); k2[0, 0, 0, 2] = x; k2[0, 0, 0, 1] = 9.0
    v2 = rng.standard_normal((1, 1, 2, D))
    w = 1.0 / (1.0 + np.exp(-a * x / np.sqrt(8.0)))
    out = O.decode_attn(q2, O.compact_keys(k2, idx, "f64"), idx, v2, "f64")
    np.testing.assert_allclose(out[0, 0], w * v2[0, 0, 0] + (1 - w) * v2[0, 0, 1], rtol=1e-13)
    # the tail segment uses the FULL query: channel 1 now counts
    kt = np.zeros((1, 1, 3, D)); kt[0, 0, 0, 1] = 0.01; vt = rng.standard_normal((1, 1, 3, D))
    z = np.array([a * x, 0.0, 50.0 * 0.01]) / np.sqrt(8.0)
    wts = np.exp(z) / np.exp(z).sum()
    out = O.decode_attn(q2, O.compact_keys(k2, idx, "f64"), idx, v2, "f64", kt, vt, 1)
    np.testing.assert_allclose(out[0, 0], wts[0] * v2[0, 0, 0] + wts[1] * v2[0, 0, 1] + wts[2] * vt[0, 0, 0], rtol=1e-13)


def test_decode_large_logits_do_not_overflow():
    D = 8; idx = np.arange(D, dtype=np.int16)[None, None]
    q = np.full((1, 1, D), 300.0); k = np.zeros((1, 1, 3, D)); k[0, 0, 1] = 300.0
    v = rng.standard_normal((1, 1, 3, D))
    out = O.decode_attn(q, k, idx, v, "f64")
    np.testing.assert_allclose(out[0, 0], v[0, 0, 1], rtol=1e-13)


# ----------------------------------------------------------- accounting ----
def test_kv_size_example_of_the_paper():
    with open(os.path.join(GOLDEN, "kv_size_example.txt")) as f:
        row = [l.split() for l in f if l.strip() and not l.startswith("#")][0]
    B, S, L, N, D, e, stated = map(float, row)
    nbytes = O.kv_cache_bytes(B, S, L, N, D, e)
    assert nbytes == 2 * 13 * 2048 * 32 * 32 * 128 * 2
    assert round(nbytes / 2**30) == stated


def test_table7_memory_column():
    """Memory(M) of Table 7: 32 layers x 32 heads x 128 channels x 2 bytes per
    cached K or V token; ThinK prunes 40% of the key channels of all but the
    32 most recent tokens."""
    per_token_kv = O.kv_cache_bytes(1, 1, 32, 32, 128, 2) / 2**20     # K + V, MiB
    assert per_token_kv == 0.5
    with open(os.path.join(GOLDEN, "table7_memory.txt")) as f:
        rows = [list(map(float, l.split())) for l in f if l.strip() and not l.startswith("#")]
    for kv, think_m, vkv, vanilla_m in rows:
        assert vkv * per_token_kv == pytest.approx(vanilla_m, abs=0.05)
        k_tokens_equiv = (kv - 32) * (1 - 0.4) + 32
        assert (k_tokens_equiv + kv) * per_token_kv / 2 == pytest.approx(think_m, abs=0.05)


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Every oracle routine on buffers of exactly the stated sizes (three element types, edge
    shapes), built with gcc -fsanitize=address,undefined: any out-of-bounds access or undefined
    arithmetic aborts the program (tests/c/oracle_sanitize_check.c)."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    exe = tmp_path / "oracle_sanitize_check"
    subprocess.check_call(["gcc", "-O1", "-g", "-std=c11", "-fopenmp", "-ffp-contract=off",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
                           "-o", str(exe), os.path.join(root, "tests", "c", "oracle_sanitize_check.c"),
                           os.path.join(root, "oracle", "thk_oracle.c"), "-lm"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=300)
    assert out.returncode == 0 and "oracle sanitize check ok" in out.stdout, out.stdout + out.stderr
