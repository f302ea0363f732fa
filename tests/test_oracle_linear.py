"""Pins for the oracle's attention + output projection (section 4.2 / appendix C), on the CPU.

The attention part is pinned in test_oracle.py; here the projection and the way the heads are laid side by side
are fixed against closed forms and numpy's matmul on the already-pinned attention output.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import inputs as I


def bits(x, dtype):
    return I.f32_to_bits(np.asarray(x, dtype=np.float32), dtype)


def rand_qkv(rng, B, H, Nq, Nk, D, dtype):
    return tuple(bits(rng.standard_normal((B, H, n, D)), dtype) for n in (Nq, Nk, Nk))


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 1, 3, 3, 2, 4), (2, 3, 5, 9, 4, 7), (1, 2, 9, 5, 8, 3)])
def test_is_the_attention_rows_times_the_matrix(oracle, shape, causal, dtype):
    B, H, Nq, Nk, D, N = shape
    rng = np.random.default_rng(500 + Nq)
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, dtype)
    w = bits(rng.standard_normal((H * D, N)), dtype)
    y = oracle.attention_linear(q, k, v, w, 0.4, causal, dtype)
    o, _ = oracle.attention_fwd(q, k, v, 0.4, causal, dtype)           # [B,H,Nq,D]
    a = o.transpose(0, 2, 1, 3).reshape(B, Nq, H * D)                  # heads side by side
    np.testing.assert_allclose(y, a @ I.bits_to_f64(w, dtype), rtol=1e-12, atol=1e-14)


def test_identity_matrix_returns_the_heads_side_by_side(oracle):
    rng = np.random.default_rng(501)
    B, H, Nq, Nk, D = 2, 3, 4, 6, 2
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, I.F16)
    w = bits(np.eye(H * D), I.F16)
    y = oracle.attention_linear(q, k, v, w, 0.5, True, I.F16)
    o, _ = oracle.attention_fwd(q, k, v, 0.5, True, I.F16)
    for h in range(H):
        np.testing.assert_array_equal(y[:, :, h * D:(h + 1) * D], o[:, h])


def test_one_nonzero_weight_picks_one_head_and_channel(oracle):
    """Catches a transposed matrix or a swapped (head, channel) order."""
    rng = np.random.default_rng(502)
    B, H, Nq, Nk, D, N = 1, 3, 5, 5, 4, 6
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, I.BF16)
    o, _ = oracle.attention_fwd(q, k, v, 0.3, False, I.BF16)
    for (h, d, n, val) in ((0, 1, 5, 2.0), (2, 3, 0, -0.5), (1, 0, 2, 1.0)):
        w = np.zeros((H * D, N), dtype=np.float32)
        w[h * D + d, n] = val
        y = oracle.attention_linear(q, k, v, bits(w, I.BF16), 0.3, False, I.BF16)
        want = np.zeros((B, Nq, N))
        want[:, :, n] = val * o[:, h, :, d]
        np.testing.assert_allclose(y, want, rtol=1e-15, atol=0)


def test_constant_values_give_the_column_sums(oracle):
    """V = 1 everywhere: every attention row is all ones whatever Q and K, so y[t, n] = sum_c w[c, n];
    rows that see no key (causal, Nq > Nk) give zero."""
    rng = np.random.default_rng(503)
    B, H, Nq, Nk, D, N = 1, 2, 6, 4, 4, 5
    q, k, _ = rand_qkv(rng, B, H, Nq, Nk, D, I.F16)
    v = bits(np.ones((B, H, Nk, D)), I.F16)
    wf = rng.standard_normal((H * D, N)).astype(np.float32)
    w = bits(wf, I.F16)
    y = oracle.attention_linear(q, k, v, w, 0.7, True, I.F16)
    colsum = I.bits_to_f64(w, I.F16).sum(axis=0)
    np.testing.assert_array_equal(y[0, :2], np.zeros((2, N)))
    np.testing.assert_allclose(y[0, 2:], np.broadcast_to(colsum, (4, N)), rtol=1e-13)


def test_row_subset_and_bad_arguments(oracle):
    rng = np.random.default_rng(504)
    B, H, Nq, Nk, D, N = 2, 2, 5, 7, 4, 3
    q, k, v = rand_qkv(rng, B, H, Nq, Nk, D, I.F16)
    w = bits(rng.standard_normal((H * D, N)), I.F16)
    y = oracle.attention_linear(q, k, v, w, 0.5, True, I.F16)
    rows = np.array([9, 0, 4])
    np.testing.assert_array_equal(oracle.attention_linear(q, k, v, w, 0.5, True, I.F16, rows=rows), y.reshape(-1, N)[rows])
    with pytest.raises(ValueError):
        oracle.attention_linear(q, k, v, w[:-1], 0.5, True, I.F16)
    with pytest.raises(RuntimeError):
        oracle.attention_linear(q, k, v, w, 0.5, True, I.F16, rows=np.array([B * Nq]))
