"""Pins of the oracle's value-cache routines (Appendix "Value Cache Pruning").

As in test_oracle_pins.py nothing here re-types the oracle's loops: library
attention (torch scaled_dot_product_attention in fp64, scipy softmax + numpy
matmul), closed forms, invariances and reductions to the already pinned
key-only decode routine.
"""
import numpy as np
import pytest
import scipy.special
import torch

from oracle import oracle as O

rng = np.random.default_rng(20240722)


def _rand(shape, dtype, scale=1.0):
    x = rng.standard_normal(shape) * scale
    if dtype == "f64":
        return x, x
    if dtype == "f32":
        x32 = x.astype(np.float32)
        return x32, x32.astype(np.float64)
    bits = O.bf16_bits(x.astype(np.float32))
    return bits, O.bf16_to_f64(bits)


def _library_score(q, k, v, G, causal):
    """Column norms of library attention output, summed over the heads of a group."""
    L, B, N_q, S_obs, D = q.shape
    S = k.shape[3]
    qt, kt, vt = (torch.from_numpy(np.ascontiguousarray(a)) for a in (q, k, v))
    kt = kt.repeat_interleave(G, dim=2)
    vt = vt.repeat_interleave(G, dim=2)
    mask = None
    if causal:
        # window row i is the token at position S - S_obs + i
        mask = torch.ones(S_obs, S, dtype=torch.bool).tril(diagonal=S - S_obs)
    o = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=mask)
    per_head = torch.linalg.vector_norm(o, dim=3)            # [L,B,N_q,D]
    return per_head.reshape(L, B, N_q // G, G, D).sum(3).numpy()


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
@pytest.mark.parametrize("G", [1, 2, 4])
@pytest.mark.parametrize("causal", [False, True])
def test_value_score_is_column_norm_of_library_attention(dtype, G, causal):
    """Score_v[j] = ||softmax(Q_obs K^T / sqrt(D)) V[:, j]||: torch's fp64 attention
    gives the S_obs x D product, torch.linalg gives the norms."""
    L, B, N_kv, S, S_obs, D = 2, 2, 2, 19, 5, 8
    q_raw, q = _rand((L, B, N_kv * G, S_obs, D), dtype, 1.5)
    k_raw, k = _rand((L, B, N_kv, S, D), dtype, 1.5)
    v_raw, v = _rand((L, B, N_kv, S, D), dtype)
    got = O.score_value(q_raw, k_raw, v_raw, dtype, causal=causal)
    want = _library_score(q, k, v, G, causal)
    np.testing.assert_allclose(got, want, rtol=1e-11)


def test_value_score_scipy_softmax_matmul_single_head():
    """The same quantity from scipy.special.softmax and a numpy matmul."""
    S, S_obs, D = 33, 4, 16
    q = rng.standard_normal((S_obs, D))
    k = rng.standard_normal((S, D))
    v = rng.standard_normal((S, D))
    A = scipy.special.softmax(q @ k.T / np.sqrt(D), axis=1)
    want = np.linalg.norm(A @ v, axis=0)
    got = O.score_value(q[None, None, None], k[None, None, None], v[None, None, None], "f64")
    np.testing.assert_allclose(got[0, 0, 0], want, rtol=1e-12)


def test_value_score_uniform_attention_closed_form():
    """K = 0 makes every softmax row uniform: each window row of A V is the
    column mean of V, so Score_v[j] = G sqrt(S_obs) |mean_s V[s, j]|.  With the
    causal mask row i averages the first S - S_obs + i + 1 rows instead."""
    L, B, N_kv, G, S, S_obs, D = 1, 2, 2, 2, 11, 3, 6
    q = rng.standard_normal((L, B, N_kv * G, S_obs, D))
    k = np.zeros((L, B, N_kv, S, D))
    v = rng.standard_normal((L, B, N_kv, S, D))
    got = O.score_value(q, k, v, "f64")
    want = G * np.sqrt(S_obs) * np.abs(v.mean(axis=3))
    np.testing.assert_allclose(got, want, rtol=1e-12)
    got_c = O.score_value(q, k, v, "f64", causal=True)
    prefix_means = np.stack([v[:, :, :, :S - S_obs + i + 1].mean(axis=3) for i in range(S_obs)], 3)
    want_c = G * np.sqrt((prefix_means ** 2).sum(3))
    np.testing.assert_allclose(got_c, want_c, rtol=1e-12)


def test_value_score_single_key_and_one_hot_attention():
    """S = S_obs = 1: A is the 1 x 1 matrix [1], Score_v[j] = |V[0, j]|.  A key
    aligned with every query and scaled up makes the softmax one-hot on that key:
    the score tends to sqrt(S_obs) |V[p, j]|."""
    S_obs, D = 4, 8
    q = rng.standard_normal((1, 1, 1, S_obs, D))
    v1 = rng.standard_normal((1, 1, 1, 1, D))
    got = O.score_value(q[:, :, :, :1], rng.standard_normal((1, 1, 1, 1, D)), v1, "f64")
    np.testing.assert_allclose(got[0, 0, 0], np.abs(v1[0, 0, 0, 0]), rtol=1e-13)
    S, p = 9, 3
    qpos = np.abs(q) + 0.5                       # all-positive queries
    k = np.zeros((1, 1, 1, S, D))
    k[0, 0, 0, p] = 400.0                        # logit of key p dwarfs the zeros
    v = rng.standard_normal((1, 1, 1, S, D))
    got = O.score_value(qpos, k, v, "f64")
    np.testing.assert_allclose(got[0, 0, 0], np.sqrt(S_obs) * np.abs(v[0, 0, 0, p]), rtol=1e-9)


def test_value_score_causal_mask_hides_exactly_the_later_keys():
    """With the mask, window row i must not see key S - S_obs + i + 1 or later, and must
    see key S - S_obs + i.  A one-hot key at position p = S - S_obs + r (inside the
    window) is visible to rows r.. only; rows before r see uniform zeros-logits over
    their prefix.  Compare with the closed form of that mixture."""
    S, S_obs, D, r = 12, 4, 6, 2
    p = S - S_obs + r
    q = np.abs(rng.standard_normal((1, 1, 1, S_obs, D))) + 0.5
    k = np.zeros((1, 1, 1, S, D))
    k[0, 0, 0, p] = 500.0
    v = rng.standard_normal((1, 1, 1, S, D))
    got = O.score_value(q, k, v, "f64", causal=True)[0, 0, 0]
    rows = []
    for i in range(S_obs):
        if i >= r:
            rows.append(v[0, 0, 0, p])
        else:
            rows.append(v[0, 0, 0, :S - S_obs + i + 1].mean(axis=0))
    want = np.sqrt((np.stack(rows) ** 2).sum(0))
    np.testing.assert_allclose(got, want, rtol=1e-9)
    # S_obs = 1: the only window row is the last token and sees everything
    a = O.score_value(q[:, :, :, -1:], k, v, "f64", causal=True)
    b = O.score_value(q[:, :, :, -1:], k, v, "f64", causal=False)
    np.testing.assert_allclose(a, b, rtol=1e-14)


def test_value_score_invariances():
    """(a) adding one vector to every key shifts each logit row by a constant: softmax and
    score unchanged; (b) permuting (key, value) rows together changes nothing without the
    mask; (c) scaling value column j by a scales Score_v[j] by |a|; (d) G identical query
    heads give G times the single-head score; (e) a far-away logit offset does not
    overflow (row maximum is subtracted)."""
    L, B, N_kv, S, S_obs, D = 1, 1, 2, 17, 4, 8
    q = rng.standard_normal((L, B, N_kv, S_obs, D))
    k = rng.standard_normal((L, B, N_kv, S, D))
    v = rng.standard_normal((L, B, N_kv, S, D))
    base = O.score_value(q, k, v, "f64")
    delta = rng.standard_normal(D)
    np.testing.assert_allclose(O.score_value(q, k + delta, v, "f64"), base, rtol=1e-10)
    perm = rng.permutation(S)
    np.testing.assert_allclose(O.score_value(q, k[:, :, :, perm], v[:, :, :, perm], "f64"), base,
                               rtol=1e-12)
    a = rng.standard_normal(D) * 3
    np.testing.assert_allclose(O.score_value(q, k, v * a, "f64"), base * np.abs(a), rtol=1e-12)
    q3 = np.repeat(q, 3, axis=2)
    np.testing.assert_allclose(O.score_value(q3, k, v, "f64"), 3 * base, rtol=1e-12)
    big = O.score_value(q * 300, k * 300, v, "f64")
    assert np.all(np.isfinite(big))
    assert np.all(big <= np.sqrt(S_obs) * np.abs(v).max(axis=3) * (1 + 1e-12))


def test_value_score_bound_by_largest_entry():
    """Each row of A is a probability vector, so |A V[:, j]|_i <= max_s |V[s, j]| and the
    score is at most G sqrt(S_obs) max_s |V[s, j]|; it is at least the norm of the
    smallest-magnitude convex combination only when V[:, j] keeps one sign."""
    L, B, N_kv, G, S, S_obs, D = 1, 1, 1, 2, 23, 6, 5
    q = rng.standard_normal((L, B, N_kv * G, S_obs, D))
    k = rng.standard_normal((L, B, N_kv, S, D))
    v = np.abs(rng.standard_normal((L, B, N_kv, S, D))) + 0.1
    got = O.score_value(q, k, v, "f64")
    assert np.all(got <= G * np.sqrt(S_obs) * v.max(axis=3) + 1e-12)
    assert np.all(got >= G * np.sqrt(S_obs) * v.min(axis=3) - 1e-12)


# ------------------------------------------------- decode with pruned V ----
def _decode_case(dtype, G, s_tail):
    B, N_kv, S, D, T, T_v, cap = 2, 2, 21, 16, 9, 11, 5
    q_raw, _ = _rand((B, N_kv * G, D), dtype)
    k_raw, _ = _rand((B, N_kv, S, D), dtype)
    v_raw, _ = _rand((B, N_kv, S, D), dtype)
    kt_raw, _ = _rand((B, N_kv, cap, D), dtype)
    vt_raw, _ = _rand((B, N_kv, cap, D), dtype)
    idx = np.sort(np.stack([rng.permutation(D)[:T] for _ in range(B * N_kv)]), 1)
    idx_v = np.sort(np.stack([rng.permutation(D)[:T_v] for _ in range(B * N_kv)]), 1)
    idx = idx.reshape(B, N_kv, T).astype(np.int16)
    idx_v = idx_v.reshape(B, N_kv, T_v).astype(np.int16)
    return q_raw, k_raw, v_raw, kt_raw, vt_raw, idx, idx_v, s_tail


@pytest.mark.parametrize("dtype", ["f64", "f32", "bf16"])
@pytest.mark.parametrize("G", [1, 2])
@pytest.mark.parametrize("s_tail", [0, 3])
def test_decode_kv_equals_key_only_decode_on_channel_masked_values(dtype, G, s_tail):
    """Dropping value channels is multiplying V by a 0/1 diagonal: the routine must give
    what the (separately pinned) key-only decode gives on values whose removed channels
    are set to zero in the pruned segment, the tail left whole."""
    q, k, v, kt, vt, idx, idx_v, s_tail = _decode_case(dtype, G, s_tail)
    kp = np.take_along_axis(k, idx[:, :, None, :].astype(np.int64), axis=3)
    vp = np.take_along_axis(v, idx_v[:, :, None, :].astype(np.int64), axis=3)
    keep = np.zeros(v.shape[:2] + (1, v.shape[3]), bool)
    np.put_along_axis(keep, idx_v[:, :, None, :].astype(np.int64), True, axis=3)
    v_masked = np.where(keep, v, np.zeros_like(v))
    want = O.decode_attn(q, kp, idx, v_masked, dtype, kt, vt, s_tail)
    got = O.decode_attn_kv(q, kp, idx, vp, idx_v, dtype, kt, vt, s_tail)
    np.testing.assert_allclose(got, want, rtol=1e-13, atol=1e-15)
    if s_tail == 0:
        removed = ~np.broadcast_to(keep[:, :, 0], v.shape[:2] + (v.shape[3],))
        assert np.all(np.repeat(removed, G, axis=1) == (got == 0.0))


def test_decode_kv_identity_index_and_padded_rows():
    """T_v = D with the identity index list is the key-only routine; a padded row
    stride (ld_v > T_v) with junk in the padding changes nothing."""
    q, k, v, kt, vt, idx, idx_v, _ = _decode_case("f64", 2, 3)
    B, N_kv, S, D = v.shape
    kp = np.take_along_axis(k, idx[:, :, None, :].astype(np.int64), axis=3)
    ident = np.broadcast_to(np.arange(D, dtype=np.int16), (B, N_kv, D)).copy()
    a = O.decode_attn_kv(q, kp, idx, v, ident, "f64", kt, vt, 3)
    b = O.decode_attn(q, kp, idx, v, "f64", kt, vt, 3)
    np.testing.assert_allclose(a, b, rtol=1e-14)
    vp = np.take_along_axis(v, idx_v[:, :, None, :].astype(np.int64), axis=3)
    pad = np.concatenate([vp, 1e6 * np.ones(vp.shape[:3] + (5,))], axis=3)
    np.testing.assert_array_equal(O.decode_attn_kv(q, kp, idx, pad, idx_v, "f64", kt, vt, 3),
                                  O.decode_attn_kv(q, kp, idx, vp, idx_v, "f64", kt, vt, 3))
