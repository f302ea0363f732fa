"""GPU parity of fa_fwd_masked (masks generated per tile from a descriptor: window, prefix, per-batch key
counts) against the CPU fp64 oracle, element by element.

Same tolerances as fa_fwd: O max-abs 1e-2, O mean-abs 1e-3, LSE 1e-3.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import inputs as I
import options
from gpu_util import check_against_oracle, run_fa_decode_masked, run_fa_fwd, run_fa_fwd_masked

pytestmark = pytest.mark.gpu


def rand_bits(rng, shape, dtype, mult=1.0):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(mult), dtype)


# B, H, Nq, Nk, D: one and several workgroups per head, ragged tails, Nq != Nk both ways, decode
SHAPES = [(1, 2, 300, 300, 128), (2, 2, 130, 700, 64), (1, 1, 700, 130, 128), (2, 1, 1, 500, 64), (1, 1, 1000, 1000, 64),
          (2, 1, 520, 777, 128)]
MASKS = [
    # left, right, prefix, kv_len fraction of Nk per batch entry (None: no padding)
    (-1, 0, 0, None), (-1, -1, 0, None), (100, 0, 0, None), (0, 0, 0, None), (63, 0, 0, None), (200, 30, 0, None),
    (-1, 70, 0, None), (40, -1, 0, None), (-1, 0, 130, None), (90, 0, 64, None), (10, 10, 1, None), (0, 0, 500, None),
    (-1, -1, 0, (0.5, 0.9)), (-1, 0, 0, (1.0, 0.3)), (150, 0, 70, (0.8, 0.05)), (-1, 0, 0, (0.0, 1.0)),
]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", MASKS)
@pytest.mark.parametrize("shape", SHAPES)
def test_descriptor_masks_elementwise(oracle, shape, mask, dtype):
    B, H, Nq, Nk, D = shape
    left, right, prefix, frac = mask
    kv_len = None if frac is None else [int(round(f * Nk)) for f in (frac * B)[:B]]
    print(f"case masked shape={shape} mask=({left},{right},{prefix},{kv_len}) dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, mask[:3], dtype)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
    o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} {mask} dt={dtype}")
    empty = np.isneginf(lse_ref)
    assert (I.bits_to_f64(o, dtype)[empty] == 0).all()


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", [(2200, 0, 0), (2048, 300, 0), (2100, 0, 128), (2300, 2300, 0)])
@pytest.mark.parametrize("shape", [(1, 2, 3000, 3000, 128), (1, 1, 2500, 4100, 64)])
def test_long_windows_walked_in_rotated_order(oracle, shape, mask, dtype):
    """Window runs of 32 tiles and more are walked rotated (so that neighbouring query blocks read the same tile
    at the same time): the wrap falls in the middle of a wave's fully visible tiles."""
    B, H, Nq, Nk, D = shape
    left, right, prefix = mask
    print(f"case masked rotated shape={shape} mask={mask} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, mask, dtype)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix)
    o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} {mask} dt={dtype}")


def test_causal_and_unmasked_descriptors_equal_fa_fwd_bit_for_bit(monkeypatch):
    """(-1, 0) and (-1, -1) walk the same tiles with the same arithmetic as fa_fwd's wide mode."""
    print("case masked vs fa_fwd", flush=True)
    options.set_fwd_mode("wide")
    rng = np.random.default_rng(401)
    for dtype, D in ((I.F16, 64), (I.BF16, 128)):
        q, k, v = (rand_bits(rng, (2, 2, n, D), dtype) for n in (600, 900, 900))
        for causal, (left, right) in ((True, (-1, 0)), (False, (-1, -1))):
            o0, l0 = run_fa_fwd(q, k, v, 0.1, causal, dtype)
            o1, l1 = run_fa_fwd_masked(q, k, v, 0.1, dtype, left, right)
            assert np.array_equal(o0, o1) and np.array_equal(l0, l1)


def test_exact_special_cases():
    """left = right = 0: every row is the value row on its diagonal, bit for bit; a key count of one: row = v[0]."""
    print("case masked exact specials", flush=True)
    rng = np.random.default_rng(402)
    for dtype in (I.F16, I.BF16):
        q, k, v = (rand_bits(rng, (1, 2, n, 64), dtype) for n in (200, 330, 330))
        o, lse = run_fa_fwd_masked(q, k, v, 0.125, dtype, 0, 0)
        assert np.array_equal(o, v[:, :, 130:])
        o, lse = run_fa_fwd_masked(q, k, v, 0.125, dtype, -1, -1, 0, [1])
        assert np.array_equal(o, np.broadcast_to(v[:, :, :1], o.shape))


@pytest.mark.parametrize("scale", [-0.12, 0.0, 0.15])
def test_unusual_scales(oracle, scale):
    print(f"case masked scale={scale}", flush=True)
    rng = np.random.default_rng(403)
    q, k, v = (rand_bits(rng, (1, 2, n, 128), I.BF16) for n in (400, 400, 400))
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, I.BF16, 70, 0, 20)
    o, lse = run_fa_fwd_masked(q, k, v, scale, I.BF16, 70, 0, 20)
    check_against_oracle(o, lse, o_ref, lse_ref, I.BF16, f"scale={scale}")


@pytest.mark.parametrize("cfg", [I.SLIDING, I.SLIDING64], ids=["SWA", "SWA64"])
def test_sliding_window_at_full_size_on_sampled_rows(oracle, cfg):
    """The windowed workloads bench.py times (inputs.SLIDING / SLIDING64, same seeded tensors): a stratified sample
    of rows."""
    print("case masked " + cfg.describe(), flush=True)
    q, k, v = I.make_qkv(cfg)
    o, lse = run_fa_fwd_masked(q, k, v, cfg.scale, cfg.dtype, cfg.window - 1, 0)
    rows = I.sample_rows(cfg, per_head=16)
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, cfg.scale, cfg.dtype, cfg.window - 1, 0, rows=rows)
    check_against_oracle(o.reshape(-1, cfg.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, cfg.dtype, cfg.name + " sample",
                         named_config=True)


DECODE_MASKS = [
    # left, right, prefix, per-batch key counts as fractions of Nk (None: no padding)
    (-1, 0, 0, None), (-1, -1, 0, None), (0, 0, 0, None), (99, 0, 0, None), (4000, 0, 0, None), (-1, 0, 0, (1.0, 0.37, 0.0)),
    (500, 0, 0, (0.9, 0.5, 1.0)), (300, 0, 64, None), (300, 0, 1000, None), (10, 0, 5000, None), (0, 0, 1, (0.5, 1.0, 0.001)),
    (2000, 5, 128, (1.0, 0.999, 0.6)),
]


@pytest.mark.parametrize("kernel", ["stream", "mfma"])
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", DECODE_MASKS)
def test_single_query_under_descriptor_masks(oracle, monkeypatch, mask, dtype, kernel):
    """A decoding step (Nq = 1) over caches of different lengths, with a sliding window and / or a prefix that
    stays visible: the streaming kernel walks the prefix and the window as two runs of consecutive keys (one if
    they touch, none if the cache is empty); FA_OPT_DECODE_KERNEL = 1 keeps the tile kernel.  Both against the oracle."""
    options.set_decode(kernel)
    left, right, prefix, frac = mask
    B, H, Nk = 3, 2, 3001
    for D in (64, 128):
        kv_len = None if frac is None else [int(round(f * Nk)) for f in frac]
        print(f"case masked decode D={D} mask=({left},{right},{prefix},{kv_len}) dtype={dtype} kernel={kernel}", flush=True)
        rng = np.random.default_rng(hash((mask[:3], dtype, D)) % (2**32))
        q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (1, Nk, Nk))
        scale = 1.0 / math.sqrt(D)
        o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
        o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
        check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"masked decode D={D} {mask}")


@pytest.mark.parametrize("nsplit", [0, 1, 2, 7, 40])
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", DECODE_MASKS)
def test_decode_masked_in_shares(oracle, mask, dtype, nsplit):
    """fa_decode_masked: the same step with every (batch, head)'s visible keys -- prefix and window laid end to
    end -- cut into nsplit shares and merged.  Entries with few or no keys get shares of few or no keys."""
    left, right, prefix, frac = mask
    B, H, Nk = 3, 2, 3001
    for D in (64, 128):
        kv_len = None if frac is None else [int(round(f * Nk)) for f in frac]
        print(f"case decode masked shares D={D} mask=({left},{right},{prefix},{kv_len}) dtype={dtype} nsplit={nsplit}", flush=True)
        rng = np.random.default_rng(hash((mask[:3], dtype, D, 9)) % (2**32))
        q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (1, Nk, Nk))
        scale = 1.0 / math.sqrt(D)
        o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len)
        o, lse, plan = run_fa_decode_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, nsplit)
        assert plan.nsplit >= 1 and (nsplit == 0 or plan.nsplit == min(nsplit, (Nk + 63) // 64))
        check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"decode masked shares D={D} {mask} nsplit={nsplit}")


OWN_DIAGONAL_MASKS = [
    # left, right, prefix, per-batch key counts as fractions of Nk
    (-1, 0, 0, (1.0, 0.37, 0.0)), (99, 0, 0, (0.9, 0.5, 0.02)), (500, 0, 0, (1.0, 0.1, 0.6)), (0, 0, 0, (0.5, 1.0, 0.001)),
    (300, 0, 64, (0.7, 0.05, 0.3)), (200, 5, 0, (1.0, 0.999, 0.6)),
]


@pytest.mark.parametrize("kernel", ["stream", "mfma"])
@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", OWN_DIAGONAL_MASKS)
def test_decoding_step_with_the_diagonal_at_each_caches_own_last_key(oracle, mask, dtype, kernel):
    """diag_from_kv_len = 1 (include/fa.h): a batch of caches of different lengths in Nk allocated rows, the new
    token's query sitting on the last key of ITS cache, so that a sliding window covers the last W keys of each
    cache (without the flag it hangs on key Nk - 1 and misses the short caches).  Through fa_fwd_masked (both
    kernels) and through fa_decode_masked in shares."""
    options.set_decode(kernel)
    left, right, prefix, frac = mask
    B, H, Nk = 3, 2, 3001
    for D in (64, 128):
        kv_len = [int(round(f * Nk)) for f in frac]
        print(f"case own diagonal decode D={D} mask=({left},{right},{prefix},{kv_len}) dtype={dtype} kernel={kernel}", flush=True)
        rng = np.random.default_rng(hash((mask[:3], dtype, D, 21)) % (2**32))
        q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (1, Nk, Nk))
        scale = 1.0 / math.sqrt(D)
        o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len,
                                                     diag_from_kv_len=True)
        # the case is what it claims to be: short caches are seen (not -inf as they would be without the flag)
        assert np.isfinite(lse_ref[[i for i, n in enumerate(kv_len) if n > 0]]).all()
        o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=1)
        check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"own diagonal decode D={D} {mask}")
        if kernel == "stream":
            for nsplit in (0, 3):
                o, lse, _ = run_fa_decode_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, nsplit, diag_from_kv_len=1)
                check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"own diagonal shares D={D} {mask} nsplit={nsplit}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("mask", [(-1, 0, 0), (100, 0, 0), (63, 0, 40), (300, 20, 0), (-1, -1, 0)])
@pytest.mark.parametrize("shape", [(3, 2, 130, 700, 64), (3, 1, 300, 1000, 128), (3, 1, 520, 777, 128), (3, 2, 300, 300, 64)])
def test_chunk_of_queries_with_the_diagonal_at_each_caches_own_last_key(oracle, shape, mask, dtype):
    """The same flag for Nq > 1 (a chunk of a chunked prefill over caches of different lengths): the Nq queries are
    the last Nq positions of each entry's own keys; an entry with fewer keys than queries leaves its first rows
    without any visible key (o = 0, lse = -inf) unless a prefix covers them."""
    B, H, Nq, Nk, D = shape
    left, right, prefix = mask
    kv_len = [Nk, int(0.55 * Nk), min(Nq // 2, Nk)]
    print(f"case own diagonal chunk shape={shape} mask={mask} kv_len={kv_len} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, mask, dtype, 22)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=True)
    o, lse = run_fa_fwd_masked(q, k, v, scale, dtype, left, right, prefix, kv_len, diag_from_kv_len=1)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"own diagonal chunk {shape} {mask} dt={dtype}")
    empty = np.isneginf(lse_ref)
    assert (I.bits_to_f64(o, dtype)[empty] == 0).all()
