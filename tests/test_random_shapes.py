"""GPU parity on seeded random problems: shapes, scales, masks, run counts and block sizes drawn at random
within the documented limits, every entry point against the CPU fp64 oracle element by element.  The
hand-picked cases of the other test files aim at known boundaries (tile edges, diagonals, empty rows); this
file covers the combinations nobody thought of.  Every problem is valid input; the draws are fixed by the seed.

Tolerances as everywhere: O max-abs 1e-2, O mean-abs 1e-3, LSE 1e-3, y as O.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import inputs as I
import options
from gpu_util import (check_against_oracle, run_attn_linear, run_fa_fwd, run_fa_fwd_masked,
                      run_fa_fwd_splitkv)

pytestmark = pytest.mark.gpu

N_CASES = 120


def rand_bits(rng, shape, dtype, mult=1.0):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(mult), dtype)


def draw_problem(rng, max_q=700, max_k=900):
    B = int(rng.integers(1, 4))
    H = int(rng.integers(1, 5))
    # lengths: mostly arbitrary, sometimes exactly on a tile edge or just off it
    def length(hi):
        n = int(rng.integers(1, hi + 1))
        if hi >= 64 and rng.random() < 0.3:
            n = max(1, min(hi, 64 * int(rng.integers(1, hi // 64 + 1)) + int(rng.integers(-1, 2))))
        return n
    Nq, Nk = length(max_q), length(max_k)
    D = int(rng.choice([64, 128]))
    dtype = int(rng.choice([I.F16, I.BF16]))
    scale = float(rng.uniform(0.04, 0.16)) * (1 if rng.random() < 0.9 else -1)
    return B, H, Nq, Nk, D, dtype, scale


@pytest.mark.parametrize("case", range(N_CASES))
def test_fa_fwd_random(oracle, monkeypatch, case):
    rng = np.random.default_rng(7000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_problem(rng)
    causal = bool(rng.integers(0, 2))
    mode = str(rng.choice(["auto", "split", "wide", "fold", "wide64"]))
    if mode != "auto":
        options.set_fwd_mode(mode)
    label = f"fa_fwd case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} scale={scale:.3f} causal={causal} mode={mode}"
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse = run_fa_fwd(q, k, v, scale, causal, dtype)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_CASES))
def test_fa_fwd_splitkv_random(oracle, monkeypatch, case):
    rng = np.random.default_rng(8000 + case)
    few = rng.random() < 0.6
    B, H, Nq, Nk, D, dtype, scale = draw_problem(rng, max_q=4 if few else 600, max_k=3000)
    causal = bool(rng.integers(0, 2))
    nsplit = int(rng.choice([0, 1, 2, 3, 5, 8, 13, 40, 1024]))
    kern = str(rng.choice(["stream", "mfma"]))
    options.set_decode(kern)
    label = (f"splitkv case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} scale={scale:.3f} causal={causal} "
             f"nsplit={nsplit} decode={kern}")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    assert 1 <= plan.nsplit <= (Nk + 63) // 64
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_CASES))
def test_fa_fwd_masked_random(oracle, case):
    rng = np.random.default_rng(9000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_problem(rng)

    def limit():
        r = rng.random()
        return -1 if r < 0.3 else (0 if r < 0.45 else int(rng.integers(1, 400)))
    left, right = limit(), limit()
    prefix = 0 if rng.random() < 0.5 else int(rng.integers(1, Nk + 50))
    kv_len = None if rng.random() < 0.5 else [int(rng.integers(0, Nk + 1)) for _ in range(B)]
    label = (f"masked case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} scale={scale:.3f} "
             f"mask=({left},{right},{prefix},{kv_len}) own_diagonal={int(kv_len is not None and case % 3 == 0)}")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    own = int(kv_len is not None and case % 3 == 0)      # the diagonal at each entry's own last key
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=own)
    o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=own)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_CASES // 2))
def test_fa_attn_linear_random(oracle, monkeypatch, case):
    rng = np.random.default_rng(10000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_problem(rng, max_q=500, max_k=600)
    scale = abs(scale)
    causal = bool(rng.integers(0, 2))
    N = int(rng.choice([256, 512, 768]))
    rpb = int(rng.choice([0, 64, 100, 128, 257]))
    options.set_linear_tile(str(rng.choice(["128", "256"])))
    label = (f"attn_linear case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} N={N} dt={dtype} scale={scale:.3f} "
             f"causal={causal} rows_per_block={rpb}")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    w = rand_bits(rng, (H * D, N), dtype, 1.0 / math.sqrt(H * D))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    y_ref = oracle.attention_linear(q, k, v, w, scale, causal, dtype)
    o, lse, y = run_attn_linear(q, k, v, w, scale, causal, dtype, rows_per_block=rpb)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, label)
    assert np.isfinite(y).all(), label
    err = np.abs(y.astype(np.float64) - y_ref)
    assert err.max() <= 1e-2 and err.mean() <= 1e-3, f"{label}: y max-abs {err.max():.3e} mean-abs {err.mean():.3e}"


# ---- medium problems: several workgroups per head, several rounds of workgroups, long windows; the oracle is
# asked for a seeded sample of rows only (first and last row always included)

N_MEDIUM = 40


def draw_medium(rng):
    B = int(rng.integers(1, 3))
    H = int(rng.integers(1, 9))
    Nq = int(rng.integers(700, 6000))
    Nk = Nq if rng.random() < 0.5 else int(rng.integers(700, 6000))
    D = int(rng.choice([64, 128]))
    dtype = int(rng.choice([I.F16, I.BF16]))
    scale = float(rng.uniform(0.05, 0.12))
    return B, H, Nq, Nk, D, dtype, scale


def sample(rng, B, H, Nq, per_head=24):
    """flat row ids (b*H + h)*Nq + i and the matching (b, h, i) index arrays"""
    ids = []
    for bh in range(B * H):
        rows = np.unique(np.concatenate([rng.integers(0, Nq, size=per_head), [0, Nq - 1]]))
        ids.append(bh * Nq + rows)
    ids = np.concatenate(ids)
    return ids, (ids // Nq) // H, (ids // Nq) % H, ids % Nq


@pytest.mark.parametrize("case", range(N_MEDIUM))
def test_fa_fwd_random_medium(oracle, monkeypatch, case):
    rng = np.random.default_rng(11000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_medium(rng)
    causal = rng.random() < 0.7
    mode = str(rng.choice(["auto", "split", "wide", "fold", "wide64"]))
    if mode != "auto":
        options.set_fwd_mode(mode)
    label = f"fa_fwd medium case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} causal={causal} mode={mode}"
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    ids, b, h, i = sample(rng, B, H, Nq)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype, rows=ids)
    o, lse = run_fa_fwd(q, k, v, scale, causal, dtype)
    check_against_oracle(o[b, h, i], lse[b, h, i], o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_MEDIUM))
def test_fa_fwd_masked_random_medium(oracle, case):
    rng = np.random.default_rng(12000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_medium(rng)

    def limit():
        r = rng.random()
        return -1 if r < 0.25 else (0 if r < 0.4 else int(rng.integers(1, 4500)))
    left, right = limit(), limit()
    prefix = 0 if rng.random() < 0.5 else int(rng.integers(1, 3000))
    kv_len = None if rng.random() < 0.6 else [int(rng.integers(Nk // 2, Nk + 1)) for _ in range(B)]
    label = (f"masked medium case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} "
             f"mask=({left},{right},{prefix},{kv_len})")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    ids, b, h, i = sample(rng, B, H, Nq)
    own = int(kv_len is not None and case % 2 == 0)
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, rows=ids,
                                                 diag_from_kv_len=own)
    o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=own)
    check_against_oracle(o[b, h, i], lse[b, h, i], o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_MEDIUM))
def test_fa_fwd_splitkv_random_medium(oracle, monkeypatch, case):
    rng = np.random.default_rng(13000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_medium(rng)
    Nq = int(rng.choice([1, 1, 2, 7, 64, 300, 1000]))
    Nk = int(rng.integers(3000, 40000))
    causal = bool(rng.integers(0, 2))
    nsplit = int(rng.choice([0, 0, 2, 7, 31, 200]))
    kern = str(rng.choice(["stream", "mfma"]))
    options.set_decode(kern)
    label = (f"splitkv medium case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} causal={causal} "
             f"nsplit={nsplit} decode={kern}")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    ids, b, h, i = sample(rng, B, H, Nq, per_head=min(24, Nq))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype, rows=ids)
    o, lse, _ = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    check_against_oracle(o[b, h, i], lse[b, h, i], o_ref, lse_ref, dtype, label)


@pytest.mark.parametrize("case", range(N_MEDIUM // 2))
def test_fa_attn_linear_random_medium(oracle, monkeypatch, case):
    rng = np.random.default_rng(14000 + case)
    B, H, Nq, Nk, D, dtype, scale = draw_medium(rng)
    Nq = min(Nq, 3000)
    Nk = max(Nk, Nq) if rng.random() < 0.5 else Nq
    causal = bool(rng.integers(0, 2))
    N = int(rng.choice([256, 1024]))
    rpb = int(rng.choice([0, 256, 700, 1024]))
    options.set_linear_tile(str(rng.choice(["128", "256"])))
    label = (f"attn_linear medium case={case} B={B} H={H} Nq={Nq} Nk={Nk} D={D} N={N} dt={dtype} causal={causal} "
             f"rows_per_block={rpb}")
    print("case " + label, flush=True)
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    w = rand_bits(rng, (H * D, N), dtype, 1.0 / math.sqrt(H * D))
    tokens = np.unique(np.concatenate([rng.integers(0, B * Nq, size=40), [0, B * Nq - 1]]))
    y_ref = oracle.attention_linear(q, k, v, w, scale, causal, dtype, rows=tokens)
    o, lse, y = run_attn_linear(q, k, v, w, scale, causal, dtype, rows_per_block=rpb)
    assert np.isfinite(y).all(), label
    err = np.abs(y.reshape(B * Nq, N)[tokens].astype(np.float64) - y_ref)
    assert err.max() <= 1e-2 and err.mean() <= 1e-3, f"{label}: y max-abs {err.max():.3e} mean-abs {err.mean():.3e}"
