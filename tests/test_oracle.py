"""Pins for the CPU oracle: closed forms, invariants, library routines, brute force.

Nothing here touches the GPU library.  Each test fixes one part of the definition in
FastAttention section 5.1 (standard attention), section 4.1 (lower-triangular mask) or
appendix C (decode sees the whole cache) against something other than the oracle itself.
"""
import json
import math
import os

import numpy as np
import pytest
import scipy.special

from paper_2410_16663_amd import inputs as I

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_facts.json")


def bits(x, dtype):
    return I.f32_to_bits(np.asarray(x, dtype=np.float32), dtype)


def rand_qkv(rng, B, H, Nq, Nk, D, dtype, mult=1.0):
    q = bits(rng.standard_normal((B, H, Nq, D)) * mult, dtype)
    k = bits(rng.standard_normal((B, H, Nk, D)) * mult, dtype)
    v = bits(rng.standard_normal((B, H, Nk, D)) * mult, dtype)
    return q, k, v


def numpy_attention(q, k, v, scale, causal, dtype):
    """Independent fp64 reference with explicit score matrices and scipy's softmax/logsumexp."""
    Q, K, V = (I.bits_to_f64(a, dtype) for a in (q, k, v))
    B, H, Nq, D = Q.shape
    Nk = K.shape[2]
    S = scale * np.einsum("bhid,bhjd->bhij", Q, K)
    if causal:
        i = np.arange(Nq)[:, None]
        j = np.arange(Nk)[None, :]
        S = np.where(j <= i + (Nk - Nq), S, -np.inf)
    with np.errstate(invalid="ignore"):
        P = scipy.special.softmax(S, axis=-1)
        lse = scipy.special.logsumexp(S, axis=-1)
    P = np.nan_to_num(P, nan=0.0)
    return np.einsum("bhij,bhjd->bhid", P, V), lse, P


# ---------------------------------------------------------------- format decoding
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_single_key_returns_value_row_for_every_bit_pattern(oracle, dtype):
    """Nk = 1: softmax is 1, so o = v[0] exactly; run over every finite 16-bit pattern."""
    allbits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    ref = I.bits_to_f64(allbits, dtype)
    keep = np.isfinite(ref)
    vb = allbits[keep]
    D = 64
    vb = vb[: (vb.size // D) * D].reshape(1, -1, 1, D)   # heads carry the patterns
    Hh = vb.shape[1]
    q = bits(np.ones((1, Hh, 1, D)), dtype)
    k = bits(np.ones((1, Hh, 1, D)), dtype)
    o, lse = oracle.attention_fwd(q, k, vb, 0.125, False, dtype)
    assert np.array_equal(o, I.bits_to_f64(vb, dtype))
    np.testing.assert_allclose(lse, 0.125 * D, rtol=0, atol=1e-12)


def test_bf16_rounding_of_inputs_is_nearest_even():
    x = np.array([1.0, 1.00390625, 1.01171875, 1.0 + 2**-8 + 2**-20, -3.1415927], dtype=np.float32)
    got = I.bits_to_f64(I.f32_to_bits(x, I.BF16), I.BF16)
    # bf16 spacing near 1 is 2^-7: ties go to even
    assert got[0] == 1.0 and got[1] == 1.0 and got[2] == 1.015625 and got[3] == 1.0078125
    assert abs(got[4] + 3.140625) < 1e-12


# ---------------------------------------------------------------- softmax step
@pytest.mark.parametrize("causal", [False, True])
def test_probabilities_sum_to_one_and_match_scipy(oracle, causal):
    rng = np.random.default_rng(11)
    q, k, v = rand_qkv(rng, 2, 3, 9, 13, 8, I.F16, 2.0)
    _, _, Pref = numpy_attention(q, k, v, 0.3, causal, I.F16)
    for row in range(2 * 3 * 9):
        p = oracle.attention_probs(q, k, 0.3, causal, I.F16, row)
        assert abs(p.sum() - 1.0) < 1e-14
        assert (p >= 0).all()
        np.testing.assert_allclose(p, Pref.reshape(-1, 13)[row], rtol=1e-13, atol=1e-300)


def test_two_keys_is_the_logistic_function(oracle):
    q = bits([[[[1.0, 2.0]]]], I.F16)
    k = bits([[[[0.5, -1.0], [2.0, 0.25]]]], I.F16)
    v = bits([[[[1.0, 0.0], [0.0, 1.0]]]], I.F16)
    scale = 0.7
    s0, s1 = scale * (0.5 - 2.0), scale * (2.0 + 0.5)
    p0 = 1.0 / (1.0 + math.exp(s1 - s0))
    o, lse = oracle.attention_fwd(q, k, v, scale, False, I.F16)
    np.testing.assert_allclose(o[0, 0, 0], [p0, 1.0 - p0], rtol=1e-14)
    assert abs(lse[0, 0, 0] - math.log(math.exp(s0) + math.exp(s1))) < 1e-14


def test_hand_computed_2x2(oracle):
    """Q = K = I, V = [[1,2],[3,4]], scale 1: logits are the identity matrix."""
    eye = bits([[[[1.0, 0.0], [0.0, 1.0]]]], I.F16)
    v = bits([[[[1.0, 2.0], [3.0, 4.0]]]], I.F16)
    e = math.e
    a, b = e / (e + 1.0), 1.0 / (e + 1.0)
    o, lse = oracle.attention_fwd(eye, eye, v, 1.0, False, I.F16)
    np.testing.assert_allclose(o[0, 0], [[a * 1 + b * 3, a * 2 + b * 4], [b * 1 + a * 3, b * 2 + a * 4]], rtol=1e-15)
    np.testing.assert_allclose(lse[0, 0], [math.log(e + 1.0)] * 2, rtol=1e-15)
    o, lse = oracle.attention_fwd(eye, eye, v, 1.0, True, I.F16)
    np.testing.assert_allclose(o[0, 0], [[1.0, 2.0], [b * 1 + a * 3, b * 2 + a * 4]], rtol=1e-15)
    np.testing.assert_allclose(lse[0, 0], [1.0, math.log(e + 1.0)], rtol=1e-15)


# ---------------------------------------------------------------- P.V step
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
def test_constant_v_returns_v(oracle, dtype):
    rng = np.random.default_rng(5)
    q, k, _ = rand_qkv(rng, 1, 2, 17, 23, 16, dtype)
    row = rng.standard_normal(16)
    v = bits(np.broadcast_to(row, (1, 2, 23, 16)), dtype)
    o, _ = oracle.attention_fwd(q, k, v, 0.25, True, dtype)
    expect = I.bits_to_f64(v, dtype)[0, 0, 0]
    np.testing.assert_allclose(o, np.broadcast_to(expect, o.shape), rtol=1e-14)


def test_one_hot_v_column_reads_out_probabilities(oracle):
    rng = np.random.default_rng(6)
    q, k, _ = rand_qkv(rng, 1, 1, 5, 8, 8, I.F16)
    vv = np.zeros((1, 1, 8, 8), dtype=np.float32)
    vv[0, 0, np.arange(8), np.arange(8)] = 1.0          # V = identity: o[i, d] = p[i, d]
    o, _ = oracle.attention_fwd(q, k, bits(vv, I.F16), 0.5, False, I.F16)
    for i in range(5):
        p = oracle.attention_probs(q, k, 0.5, False, I.F16, i)
        np.testing.assert_allclose(o[0, 0, i], p, rtol=1e-15)


# ---------------------------------------------------------------- LSE and mask alignment
@pytest.mark.parametrize("Nq,Nk", [(6, 6), (3, 7), (7, 3), (1, 9)])
@pytest.mark.parametrize("causal", [False, True])
def test_zero_queries_give_log_count_and_mean_of_visible_values(oracle, Nq, Nk, causal):
    rng = np.random.default_rng(7)
    _, k, v = rand_qkv(rng, 1, 2, Nq, Nk, 4, I.F16)
    q = np.zeros((1, 2, Nq, 4), dtype=np.uint16)
    o, lse = oracle.attention_fwd(q, k, v, 0.5, causal, I.F16)
    V = I.bits_to_f64(v, I.F16)
    for i in range(Nq):
        n = min(Nk, max(0, i + Nk - Nq + 1)) if causal else Nk   # bottom-right alignment
        for h in range(2):
            if n == 0:
                assert lse[0, h, i] == -np.inf and (o[0, h, i] == 0).all()
            else:
                assert abs(lse[0, h, i] - math.log(n)) < 1e-14
                np.testing.assert_allclose(o[0, h, i], V[0, h, :n].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_adding_a_vector_to_every_key_shifts_lse_only(oracle):
    rng = np.random.default_rng(8)
    # small integers: k + u stays exactly representable in fp16
    qf = rng.integers(-3, 4, (1, 1, 5, 6)).astype(np.float32)
    kf = rng.integers(-3, 4, (1, 1, 7, 6)).astype(np.float32)
    vf = rng.integers(-3, 4, (1, 1, 7, 6)).astype(np.float32)
    u = rng.integers(-2, 3, 6).astype(np.float32)
    o1, l1 = oracle.attention_fwd(bits(qf, 0), bits(kf, 0), bits(vf, 0), 0.125, False, 0)
    o2, l2 = oracle.attention_fwd(bits(qf, 0), bits(kf + u, 0), bits(vf, 0), 0.125, False, 0)
    np.testing.assert_allclose(o1, o2, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(l2 - l1, 0.125 * (qf[0, 0] @ u)[None, None], rtol=0, atol=1e-13)


def test_causal_row_equals_noncausal_on_its_prefix(oracle):
    rng = np.random.default_rng(9)
    q, k, v = rand_qkv(rng, 1, 2, 12, 12, 8, I.BF16)
    oc, lc = oracle.attention_fwd(q, k, v, 0.35, True, I.BF16)
    for i in range(12):
        on, ln = oracle.attention_fwd(q[:, :, i:i + 1], k[:, :, :i + 1], v[:, :, :i + 1], 0.35, False, I.BF16)
        np.testing.assert_allclose(oc[:, :, i], on[:, :, 0], rtol=1e-14)
        np.testing.assert_allclose(lc[:, :, i], ln[:, :, 0], rtol=1e-14)
    # the first causal row attends to key 0 alone: it IS v[0]
    assert np.array_equal(oc[:, :, 0], I.bits_to_f64(v, I.BF16)[:, :, 0])


def test_decode_query_sees_whole_cache(oracle):
    """Appendix C, decoding: one query against the concatenated cache -- causal == non-causal."""
    rng = np.random.default_rng(10)
    q, k, v = rand_qkv(rng, 2, 2, 1, 33, 8, I.F16)
    a = oracle.attention_fwd(q, k, v, 0.4, True, I.F16)
    b = oracle.attention_fwd(q, k, v, 0.4, False, I.F16)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_noncausal_is_invariant_to_key_value_permutation(oracle):
    rng = np.random.default_rng(12)
    q, k, v = rand_qkv(rng, 1, 1, 4, 10, 8, I.F16)
    perm = rng.permutation(10)
    a = oracle.attention_fwd(q, k, v, 0.3, False, I.F16)
    b = oracle.attention_fwd(q, k[:, :, perm], v[:, :, perm], 0.3, False, I.F16)
    np.testing.assert_allclose(a[0], b[0], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(a[1], b[1], rtol=1e-13)


def test_causal_mask_blocks_match_figure_3(oracle):
    """The set of b x b sub-blocks of the 2M x 2M causal pattern, over all shifts, has the
    size the paper's Figure 3 shows for b = M = 3; the pattern itself is lower triangular."""
    facts = json.load(open(GOLDEN))
    b = facts["fig3_block_size_b"]["value"]
    side = facts["fig3_mmask_side"]["value"]
    q = np.zeros((1, 1, side, 2), dtype=np.uint16)
    k = np.zeros((1, 1, side, 2), dtype=np.uint16)
    mask = np.stack([oracle.attention_probs(q, k, 1.0, True, 0, i) > 0 for i in range(side)])
    assert np.array_equal(mask, np.tril(np.ones((side, side), dtype=bool)))
    blocks = {mask[r:r + b, c:c + b].tobytes() for r in range(side - b + 1) for c in range(side - b + 1)}
    assert len(blocks) == facts["fig3_distinct_bmasks"]["value"]


# ---------------------------------------------------------------- whole thing
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 1, 3, 3, 2), (2, 3, 5, 9, 4), (1, 2, 9, 5, 8), (1, 1, 40, 40, 16)])
def test_matches_explicit_matrix_reference(oracle, dtype, causal, shape):
    B, H, Nq, Nk, D = shape
    rng = np.random.default_rng(100 + Nq + Nk)
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, dtype, 1.5)
    scale = 1.0 / math.sqrt(D)
    o, lse = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    oref, lref, _ = numpy_attention(q, k, v, scale, causal, dtype)
    np.testing.assert_allclose(o, oref, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(lse, lref, rtol=1e-12, atol=1e-14)


def test_asymmetric_operands_catch_a_transposed_product(oracle):
    """Q.K^T contracts over d (not over positions) and P.V contracts over keys."""
    q = bits([[[[1, 0, 0], [0, 2, 0]]]], 0)                       # Nq = 2, D = 3
    k = bits([[[[1, 1, 0], [0, 1, 5], [3, 0, 0], [0, 0, 1]]]], 0)   # Nk = 4
    v = bits([[[[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1]]]], 0)
    S = np.array([[1, 0, 3, 0], [2, 2, 0, 0]], dtype=np.float64)   # by hand
    P = np.exp(S) / np.exp(S).sum(1, keepdims=True)
    V = np.array([[1, 0, 0], [0, 1, 0], [0, 0, 1], [1, 1, 1]], dtype=np.float64)
    o, lse = oracle.attention_fwd(q, k, v, 1.0, False, 0)
    np.testing.assert_allclose(o[0, 0], P @ V, rtol=1e-14)
    np.testing.assert_allclose(lse[0, 0], np.log(np.exp(S).sum(1)), rtol=1e-14)


def test_negative_and_zero_scale(oracle):
    rng = np.random.default_rng(13)
    q, k, v = rand_qkv(rng, 1, 1, 4, 6, 4, I.F16)
    for scale in (-0.5, 0.0):
        o, lse = oracle.attention_fwd(q, k, v, scale, True, I.F16)
        oref, lref, _ = numpy_attention(q, k, v, scale, True, I.F16)
        np.testing.assert_allclose(o, oref, rtol=1e-13, atol=1e-15)
        np.testing.assert_allclose(lse, lref, rtol=1e-13, atol=1e-15)


def test_row_subset_equals_full_run(oracle):
    cfg = I.CONFIGS["C1"]
    q, k, v = I.make_qkv(cfg)
    o, lse = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    rows = I.sample_rows(cfg, per_head=8)
    osub, lsub = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype, rows=rows)
    assert np.array_equal(osub, o.reshape(-1, cfg.D)[rows])
    assert np.array_equal(lsub, lse.reshape(-1)[rows])
    assert 0 in rows and cfg.Nq - 1 in rows


def test_thread_count_does_not_change_results(oracle):
    cfg = I.CONFIGS["C1"]
    q, k, v = I.make_qkv(cfg)
    a = oracle.attention_fwd(q, k, v, cfg.scale, True, cfg.dtype, nthreads=1)
    b = oracle.attention_fwd(q, k, v, cfg.scale, True, cfg.dtype, nthreads=4)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


def test_bad_arguments_are_rejected(oracle):
    q = np.zeros((1, 1, 2, 4), dtype=np.uint16)
    with pytest.raises(RuntimeError):
        oracle.attention_fwd(q, q, q, 1.0, False, 2)
    with pytest.raises(RuntimeError):
        oracle.attention_fwd(q, q, q, 1.0, False, 0, rows=np.array([5]))
    with pytest.raises(TypeError):
        oracle.attention_fwd(q.astype(np.float32), q, q, 1.0, False, 0)
