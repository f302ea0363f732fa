"""Pins for the oracle's descriptor masks (sliding window, prefix, per-batch key lengths).

Nothing here touches the GPU library.  The masked oracle function is fixed against things
other than itself: explicit mask matrices built with numpy's band routines and scipy's
softmax, the already-pinned causal / unmasked oracle, truncated inputs, and closed forms.
"""
import math

import numpy as np
import pytest
import scipy.special

from paper_2410_16663_amd import inputs as I


def bits(x, dtype):
    return I.f32_to_bits(np.asarray(x, dtype=np.float32), dtype)


def rand_qkv(rng, B, H, Nq, Nk, D, dtype, mult=1.0):
    return tuple(bits(rng.standard_normal((B, H, n, D)) * mult, dtype) for n in (Nq, Nk, Nk))


def band_matrix(Nq, Nk, left, right, prefix, klen):
    """Boolean [Nq,Nk] keep-matrix from numpy's triangle routines (no per-element predicate)."""
    off = Nk - Nq
    keep = np.ones((Nq, Nk), dtype=bool)
    if right >= 0:
        keep &= np.tril(np.ones((Nq, Nk), dtype=bool), k=off + right)
    if left >= 0:
        keep &= np.triu(np.ones((Nq, Nk), dtype=bool), k=off - left)
    keep[:, :prefix] = True
    keep[:, klen:] = False
    return keep


def matrix_attention(q, k, v, scale, dtype, keep):
    """keep: [B,Nq,Nk] boolean.  Explicit score matrices, scipy softmax / logsumexp."""
    Q, K, V = (I.bits_to_f64(a, dtype) for a in (q, k, v))
    S = scale * np.einsum("bhid,bhjd->bhij", Q, K)
    S = np.where(keep[:, None], S, -np.inf)
    with np.errstate(invalid="ignore"):
        P = scipy.special.softmax(S, axis=-1)
        lse = scipy.special.logsumexp(S, axis=-1)
    P = np.nan_to_num(P, nan=0.0)
    return np.einsum("bhij,bhjd->bhid", P, V), lse


MASKS = [
    # left, right, prefix, kv_len (None or per-batch list; 2 batch entries)
    (-1, 0, 0, None), (-1, -1, 0, None), (3, 0, 0, None), (0, 0, 0, None), (2, 2, 0, None), (-1, 3, 0, None),
    (5, -1, 0, None), (-1, 0, 4, None), (2, 0, 3, None), (0, 0, 20, None), (-1, -1, 0, [5, 9]), (-1, 0, 0, [0, 7]),
    (3, 1, 2, [6, 1]), (-1, 0, 6, [4, 9]), (100, 100, 0, None),
]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", [(9, 9, 4), (5, 9, 8), (9, 5, 2), (1, 9, 4), (12, 9, 4)])
@pytest.mark.parametrize("mask", MASKS)
def test_matches_explicit_mask_matrices(oracle, mask, shape, dtype):
    left, right, prefix, kv_len = mask
    Nq, Nk, D = shape
    B, H = 2, 2
    if kv_len is not None:
        kv_len = [min(x, Nk) for x in kv_len]
    rng = np.random.default_rng(300 + Nq * 13 + Nk)
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, dtype, 1.5)
    scale = 1.0 / math.sqrt(D)
    keep = np.stack([band_matrix(Nq, Nk, left, right, prefix, Nk if kv_len is None else kv_len[b]) for b in range(B)])
    oref, lref = matrix_attention(q, k, v, scale, dtype, keep)
    o, lse = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
    np.testing.assert_allclose(o, oref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, lref, rtol=1e-12, atol=1e-14)
    # rows without a visible key: zeros and -inf
    empty = ~keep.any(axis=-1)
    assert np.array_equal(np.isneginf(lse), np.broadcast_to(empty[:, None], lse.shape))
    assert (o[np.broadcast_to(empty[:, None], lse.shape)] == 0).all()


@pytest.mark.parametrize("Nq,Nk", [(7, 7), (3, 8), (8, 3)])
def test_descriptor_reduces_to_the_causal_and_unmasked_oracle(oracle, Nq, Nk):
    rng = np.random.default_rng(301)
    q, k, v = rand_qkv(rng, 1, 3, Nq, Nk, 8, I.F16)
    for causal, (left, right) in ((True, (-1, 0)), (False, (-1, -1))):
        o0, l0 = oracle.attention_fwd(q, k, v, 0.3, causal, I.F16)
        o1, l1 = oracle.attention_fwd_masked(q, k, v, 0.3, I.F16, left, right)
        np.testing.assert_allclose(o1, o0, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(l1, l0, rtol=1e-13, atol=1e-15)
    # limits at least as wide as the matrix are no limits
    o2, l2 = oracle.attention_fwd_masked(q, k, v, 0.3, I.F16, Nq + Nk, Nq + Nk)
    np.testing.assert_array_equal(o2, o1)
    np.testing.assert_array_equal(l2, l1)


def test_window_of_one_key_returns_that_value_row(oracle):
    """left = right = 0: row i sees key i + Nk - Nq only -> o = v there exactly, lse = that logit."""
    rng = np.random.default_rng(302)
    Nq, Nk, D = 5, 8, 4
    q, k, v = rand_qkv(rng, 1, 2, Nq, Nk, D, I.BF16)
    o, lse = oracle.attention_fwd_masked(q, k, v, 0.7, I.BF16, 0, 0)
    Q, K, V = (I.bits_to_f64(a, I.BF16) for a in (q, k, v))
    np.testing.assert_array_equal(o, V[:, :, Nk - Nq:])
    np.testing.assert_allclose(lse, 0.7 * np.einsum("bhid,bhid->bhi", Q, K[:, :, Nk - Nq:]), rtol=1e-14)


def test_two_key_window_is_the_logistic_function(oracle):
    """left = 1, right = 0 on a square problem: row i >= 1 mixes v[i-1], v[i] with weight sigmoid(s_i - s_{i-1})."""
    rng = np.random.default_rng(303)
    N, D = 6, 4
    q, k, v = rand_qkv(rng, 1, 1, N, N, D, I.F16)
    o, _ = oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, 1, 0)
    Q, K, V = (I.bits_to_f64(a, I.F16)[0, 0] for a in (q, k, v))
    for i in range(1, N):
        d = 0.5 * (Q[i] @ K[i] - Q[i] @ K[i - 1])
        w = 1.0 / (1.0 + math.exp(-d))
        np.testing.assert_allclose(o[0, 0, i], w * V[i] + (1 - w) * V[i - 1], rtol=1e-13, atol=1e-15)
    np.testing.assert_array_equal(o[0, 0, 0], V[0])


def test_key_lengths_equal_truncated_inputs(oracle):
    """Unmasked with kv_len[b] = L is unmasked attention over the first L keys of that batch entry."""
    rng = np.random.default_rng(304)
    q, k, v = rand_qkv(rng, 3, 2, 4, 10, 8, I.F16)
    lens = [10, 3, 1]
    o, lse = oracle.attention_fwd_masked(q, k, v, 0.4, I.F16, kv_len=lens)
    for b, L in enumerate(lens):
        ob, lb = oracle.attention_fwd(q[b:b + 1], k[b:b + 1, :, :L], v[b:b + 1, :, :L], 0.4, False, I.F16)
        np.testing.assert_allclose(o[b:b + 1], ob, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse[b:b + 1], lb, rtol=1e-13, atol=1e-15)


def test_causal_with_key_length_equals_the_square_causal_problem_on_the_valid_part(oracle):
    """Right-padded batch, Nq = Nk = N, kv_len = L: rows below L are the causal attention of the L x L problem;
    rows from L on see exactly the L valid keys."""
    rng = np.random.default_rng(305)
    N, L, D = 9, 5, 4
    q, k, v = rand_qkv(rng, 1, 2, N, N, D, I.BF16)
    o, lse = oracle.attention_fwd_masked(q, k, v, 0.4, I.BF16, -1, 0, 0, [L])
    o_sq, l_sq = oracle.attention_fwd(q[:, :, :L], k[:, :, :L], v[:, :, :L], 0.4, True, I.BF16)
    np.testing.assert_allclose(o[:, :, :L], o_sq, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse[:, :, :L], l_sq, rtol=1e-13, atol=1e-15)
    o_full, l_full = oracle.attention_fwd(q[:, :, L:], k[:, :, :L], v[:, :, :L], 0.4, False, I.BF16)
    np.testing.assert_allclose(o[:, :, L:], o_full, rtol=1e-13, atol=1e-15)


def test_prefix_rows_attend_the_whole_prefix_and_later_rows_causally(oracle):
    rng = np.random.default_rng(306)
    N, P, D = 10, 4, 4
    q, k, v = rand_qkv(rng, 1, 2, N, N, D, I.F16)
    o, lse = oracle.attention_fwd_masked(q, k, v, 0.6, I.F16, -1, 0, P)
    o_pre, l_pre = oracle.attention_fwd(q[:, :, :P], k[:, :, :P], v[:, :, :P], 0.6, False, I.F16)
    np.testing.assert_allclose(o[:, :, :P], o_pre, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(lse[:, :, :P], l_pre, rtol=1e-13, atol=1e-15)
    o_c, l_c = oracle.attention_fwd(q, k, v, 0.6, True, I.F16)
    np.testing.assert_allclose(o[:, :, P:], o_c[:, :, P:], rtol=1e-13, atol=1e-15)
    # a prefix does not reach past the keys that exist, and a window far from it still sees it
    o2, _ = oracle.attention_fwd_masked(q, k, v, 0.6, I.F16, -1, -1, 3 * N)
    o3, _ = oracle.attention_fwd(q, k, v, 0.6, False, I.F16)
    np.testing.assert_allclose(o2, o3, rtol=1e-13, atol=1e-15)


def test_zero_queries_count_the_visible_keys(oracle):
    """Q = 0: lse = ln(number of visible keys), o = their mean value."""
    rng = np.random.default_rng(307)
    Nq, Nk, D = 7, 12, 4
    _, k, v = rand_qkv(rng, 2, 1, Nq, Nk, D, I.F16)
    q = np.zeros((2, 1, Nq, D), dtype=np.uint16)
    left, right, prefix, lens = 2, 1, 3, [12, 8]
    o, lse = oracle.attention_fwd_masked(q, k, v, 1.0, I.F16, left, right, prefix, lens)
    V = I.bits_to_f64(v, I.F16)
    for b in range(2):
        for i in range(Nq):
            diag = i + Nk - Nq
            js = [j for j in range(lens[b]) if j < prefix or diag - left <= j <= diag + right]
            np.testing.assert_allclose(lse[b, 0, i], math.log(len(js)), rtol=1e-14)
            np.testing.assert_allclose(o[b, 0, i], V[b, 0, js].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_diagonal_at_each_entrys_own_last_key_equals_the_truncated_problem(oracle):
    """diag_from_kv_len: the queries are the last Nq positions of each entry's own kv_len[b] keys, so entry b is
    the same descriptor (without key lengths) applied to that entry's first kv_len[b] keys alone -- the function
    pinned above, on inputs cut by numpy."""
    rng = np.random.default_rng(309)
    q, k, v = rand_qkv(rng, 4, 2, 3, 11, 4, I.BF16)
    lens = [11, 7, 3, 1]
    for left, right, prefix in ((-1, 0, 0), (2, 0, 0), (0, 0, 0), (1, 1, 2), (4, -1, 1), (-1, -1, 0)):
        o, lse = oracle.attention_fwd_masked(q, k, v, 0.6, I.BF16, left, right, prefix, lens, diag_from_kv_len=True)
        for b, L in enumerate(lens):
            ob, lb = oracle.attention_fwd_masked(q[b:b + 1], k[b:b + 1, :, :L], v[b:b + 1, :, :L], 0.6, I.BF16, left,
                                                 right, prefix)
            np.testing.assert_allclose(o[b:b + 1], ob, rtol=1e-13, atol=1e-15)
            np.testing.assert_array_equal(np.isneginf(lse[b:b + 1]), np.isneginf(lb))
            fin = np.isfinite(lb)
            np.testing.assert_allclose(lse[b:b + 1][fin], lb[fin], rtol=1e-13, atol=1e-15)
    # without key lengths the flag changes nothing
    a = oracle.attention_fwd_masked(q, k, v, 0.6, I.BF16, 2, 0, 1)
    c = oracle.attention_fwd_masked(q, k, v, 0.6, I.BF16, 2, 0, 1, diag_from_kv_len=True)
    np.testing.assert_array_equal(a[0], c[0])
    np.testing.assert_array_equal(a[1], c[1])


def test_decoding_step_with_a_window_over_caches_of_different_lengths(oracle):
    """Appendix C's decoding step (one query, the new token) for a batch of caches of different lengths under a
    sliding window of W keys: with Q = 0 the query of entry b weighs the last min(W, L_b) of ITS keys equally --
    lse = ln min(W, L_b), o = their mean -- wherever the cache ends inside the Nk allocated rows.  Without the
    flag the window hangs on key Nk - 1 and misses the short caches altogether."""
    rng = np.random.default_rng(310)
    Nk, D, W = 20, 4, 5
    _, k, v = rand_qkv(rng, 4, 2, 1, Nk, D, I.F16)
    q = np.zeros((4, 2, 1, D), dtype=np.uint16)
    lens = [20, 12, 3, 0]
    o, lse = oracle.attention_fwd_masked(q, k, v, 1.0, I.F16, W - 1, 0, 0, lens, diag_from_kv_len=True)
    V = I.bits_to_f64(v, I.F16)
    for b, L in enumerate(lens):
        n = min(W, L)
        if n == 0:
            assert np.isneginf(lse[b]).all() and (o[b] == 0).all()
            continue
        np.testing.assert_allclose(lse[b, :, 0], math.log(n), rtol=1e-14)
        np.testing.assert_allclose(o[b, :, 0], V[b, :, L - n:L].mean(axis=1), rtol=1e-13, atol=1e-15)
    o2, lse2 = oracle.attention_fwd_masked(q, k, v, 1.0, I.F16, W - 1, 0, 0, lens)
    np.testing.assert_allclose(lse2[0, :, 0], math.log(W), rtol=1e-14)
    assert np.isneginf(lse2[1:]).all()                       # keys 15..19 are padding for the shorter caches


def test_diagonal_flag_against_explicit_matrices(oracle):
    """The same flag against keep-matrices written with numpy's triangle routines, offset L_b - Nq per entry."""
    rng = np.random.default_rng(311)
    B, H, Nq, Nk, D = 3, 2, 4, 9, 4
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, I.F16)
    lens = [9, 6, 2]
    for left, right, prefix in ((1, 0, 0), (-1, 0, 1), (2, 1, 0)):
        keep = np.zeros((B, Nq, Nk), dtype=bool)
        for b, L in enumerate(lens):
            keep[b, :, :L] = band_matrix(Nq, L, left, right, prefix, L)
        o_ref, lse_ref = matrix_attention(q, k, v, 0.5, I.F16, keep)
        o, lse = oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, left, right, prefix, lens, diag_from_kv_len=True)
        np.testing.assert_allclose(o, o_ref, rtol=1e-12, atol=1e-14)
        fin = np.isfinite(lse_ref)
        np.testing.assert_array_equal(np.isneginf(lse), ~fin)
        np.testing.assert_allclose(lse[fin], lse_ref[fin], rtol=1e-12, atol=1e-14)


def test_row_subset_and_bad_arguments(oracle):
    rng = np.random.default_rng(308)
    q, k, v = rand_qkv(rng, 2, 2, 6, 9, 4, I.F16)
    o, lse = oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, 2, 0, 1, [9, 4])
    rows = np.array([0, 7, 23, 12])
    o_s, l_s = oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, 2, 0, 1, [9, 4], rows=rows)
    np.testing.assert_array_equal(o_s, o.reshape(-1, 4)[rows])
    np.testing.assert_array_equal(l_s, lse.reshape(-1)[rows])
    with pytest.raises(RuntimeError):
        oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, kv_len=[10, 1])     # longer than Nk
    with pytest.raises(RuntimeError):
        oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, prefix=-1)
    with pytest.raises(ValueError):
        oracle.attention_fwd_masked(q, k, v, 0.5, I.F16, kv_len=[1, 2, 3])
