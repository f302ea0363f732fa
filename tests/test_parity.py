"""GPU parity: fa_fwd (through the C ABI) against the CPU fp64 oracle, element by element.

Tolerances (stated by the task for N(0,1) inputs): O max-abs 1e-2, O mean-abs 1e-3, LSE 1e-3.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import binding as fa
import options
from paper_2410_16663_amd import inputs as I
from gpu_util import check_against_oracle, run_fa_fwd

pytestmark = pytest.mark.gpu


def rand_bits(rng, shape, dtype, mult=1.0):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(mult), dtype)


SHAPES = [
    # B, H, Nq, Nk, D      several tiles + ragged tails, Nq != Nk both ways, decode, tiny
    (1, 1, 1, 1, 64), (1, 2, 3, 3, 128), (2, 2, 64, 64, 64), (1, 2, 128, 128, 128),
    (1, 3, 200, 200, 64), (1, 2, 333, 333, 128), (2, 1, 257, 129, 64), (1, 2, 100, 417, 128),
    (1, 2, 1, 300, 128), (3, 1, 7, 1000, 64), (1, 1, 513, 64, 128), (1, 2, 640, 640, 128),
    (1, 1, 31, 65, 64), (1, 1, 129, 63, 128),
]


@pytest.fixture(params=["split", "wide", "fold", "wide64"])
def mode(request, monkeypatch):
    """Force each work decomposition in turn (FA_OPT_FWD_MODE of include/fa.h)."""
    options.set_fwd_mode(request.param)
    return request.param


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", SHAPES)
def test_small_shapes_elementwise(oracle, mode, shape, causal, dtype):
    B, H, Nq, Nk, D = shape
    print(f"case mode={mode} shape={shape} causal={causal} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, causal, dtype)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse = run_fa_fwd(q, k, v, scale, causal, dtype)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} causal={causal} dt={dtype}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", [(1, 2, 2048, 2048, 128), (1, 1, 1500, 1500, 64), (1, 2, 1000, 1300, 128),
                                   (1, 1, 1300, 1000, 128), (2, 1, 1025, 1025, 64), (1, 1, 4096, 4096, 128),
                                   (1, 2, 777, 3000, 64)])
def test_folded_mode_on_longer_causal_shapes(oracle, monkeypatch, shape, dtype):
    """The paired fold has two phases, a mid-kernel change of blocks and a merge: shapes with several workgroups
    per head, ragged ends, more keys than queries (phase A empty for the first workgroups) and fewer (rows
    without keys, expensive blocks that need no second phase)."""
    options.set_fwd_mode("fold")
    B, H, Nq, Nk, D = shape
    print(f"case fold shape={shape} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, dtype, 7)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, True, dtype)
    o, lse = run_fa_fwd(q, k, v, scale, True, dtype)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"fold {shape} dt={dtype}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape", [(1, 2, 2048, 2048, 128), (1, 1, 4096, 4096, 128), (1, 2, 1000, 1300, 128),
                                   (1, 1, 1300, 1000, 128), (2, 1, 1025, 3000, 128), (1, 2, 300, 5000, 128)])
def test_wide64_mode_on_longer_shapes(oracle, shape, causal, dtype):
    """FA_MODE_WIDE64 on walks long enough for its pipelined loop (which takes whole unmasked tiles two at a
    time and leaves the rest to the general loop): several workgroups per head, ragged ends, more keys than
    queries and fewer, waves whose second 32-row block is partly or wholly past the last query."""
    options.set_fwd_mode("wide64")
    B, H, Nq, Nk, D = shape
    print(f"case wide64 shape={shape} causal={causal} dtype={dtype}", flush=True)
    assert fa.fa_fwd_plan(B, H, Nq, Nk, D, int(causal), dtype).mode == fa.FA_MODE_WIDE64
    rng = np.random.default_rng(hash((shape, causal, dtype, 64)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse = run_fa_fwd(q, k, v, scale, causal, dtype)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"wide64 {shape} causal={causal} dt={dtype}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("pattern", ["rising", "late_spike", "staircase"])
def test_wide64_reference_moves_inside_the_pipelined_loop(oracle, pattern, dtype):
    """Row maxima that keep rising over a long walk of unmasked tiles: inside FA_MODE_WIDE64's pipelined loop the
    reference moves through a block out of line that recomputes the unit's logits and rescales accumulators that
    live in the accumulation registers -- here with non-zero accumulators, in both row blocks of a wave, many times."""
    options.set_fwd_mode("wide64")
    print(f"case wide64 moving maximum pattern={pattern} dtype={dtype}", flush=True)
    rng = np.random.default_rng(82)
    D, Nq, Nk = 128, 320, 2048
    qf = rng.standard_normal((1, 2, Nq, D), dtype=np.float32)
    kf = rng.standard_normal((1, 2, Nk, D), dtype=np.float32) * np.float32(0.05)
    vf = rng.standard_normal((1, 2, Nk, D), dtype=np.float32)
    u = qf.mean(axis=2, keepdims=True)
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    qf = qf * np.float32(0.2) + 6.0 * u
    j = np.arange(Nk, dtype=np.float32)
    amp = {"rising": j / 64.0, "late_spike": np.where(j == Nk - 300, 25.0, 0.0),
           "staircase": np.floor(j / 256.0) * 5.0}[pattern].astype(np.float32)
    kf = kf + amp[None, None, :, None] * u
    q, k, v = (I.f32_to_bits(a, dtype) for a in (qf, kf, vf))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, 1.0, False, dtype)
    o, lse = run_fa_fwd(q, k, v, 1.0, False, dtype)
    of = I.bits_to_f64(o, dtype)
    assert np.isfinite(of).all() and np.isfinite(lse).all()
    assert np.abs(of - o_ref).max() <= (1e-2 if dtype == I.F16 else 2e-2)
    assert (np.abs(lse - lse_ref) <= 1e-3 + 1e-6 * np.abs(lse_ref)).all()


@pytest.mark.parametrize("scale", [-0.2, 0.0, 1.0, 1e-3])
def test_unusual_scales(oracle, mode, scale):
    print(f"case mode={mode} scale={scale}", flush=True)
    rng = np.random.default_rng(77)
    q, k, v = (rand_bits(rng, (1, 2, n, 64), I.F16) for n in (150, 210, 210))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, True, I.F16)
    o, lse = run_fa_fwd(q, k, v, scale, True, I.F16)
    check_against_oracle(o, lse, o_ref, lse_ref, I.F16, f"scale={scale}")


def test_rows_without_visible_keys_are_zero_with_minus_inf_lse(oracle, mode):
    print(f"case mode={mode} empty rows", flush=True)
    rng = np.random.default_rng(78)
    q, k, v = (rand_bits(rng, (1, 2, n, 128), I.BF16) for n in (300, 100, 100))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, 0.1, True, I.BF16)
    assert np.isneginf(lse_ref[:, :, :200]).all()
    o, lse = run_fa_fwd(q, k, v, 0.1, True, I.BF16)
    check_against_oracle(o, lse, o_ref, lse_ref, I.BF16, "empty rows")
    assert (I.bits_to_f64(o, I.BF16)[:, :, :200] == 0).all()


def test_exact_special_cases(mode):
    """Properties that hold exactly whatever the summation order."""
    print(f"case mode={mode} exact specials", flush=True)
    rng = np.random.default_rng(79)
    for dtype in (I.F16, I.BF16):
        q, k, v = (rand_bits(rng, (1, 2, n, 64), dtype) for n in (130, 130, 130))
        # causal row 0 sees key 0 only: o = v[0] bit for bit, lse = its logit
        o, lse = run_fa_fwd(q, k, v, 0.125, True, dtype)
        assert np.array_equal(o[:, :, 0], v[:, :, 0])
        # constant V comes back (to within the output rounding of the normalisation)
        vc = np.broadcast_to(v[:, :, :1], v.shape).copy()
        o, _ = run_fa_fwd(q, k, vc, 0.125, False, dtype)
        ref = I.bits_to_f64(vc[:, :, :1], dtype)
        assert np.abs(I.bits_to_f64(o, dtype) - ref).max() <= 2.0 ** -7 * np.abs(ref).max()


def test_large_logits_do_not_overflow(oracle, mode):
    print(f"case mode={mode} large logits", flush=True)
    rng = np.random.default_rng(80)
    q, k, v = (rand_bits(rng, (1, 1, n, 128), I.F16, m) for n, m in ((96, 6.0), (160, 6.0), (160, 1.0)))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, 1.0, False, I.F16)   # logits ~ N(0, 36*sqrt(128))
    o, lse = run_fa_fwd(q, k, v, 1.0, False, I.F16)
    of = I.bits_to_f64(o, I.F16)
    assert np.isfinite(of).all() and np.isfinite(lse).all()
    assert np.abs(of - o_ref).max() <= 1e-2
    assert (np.abs(lse - lse_ref) <= 1e-3 + 2e-7 * np.abs(lse_ref)).all()


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("pattern", ["rising", "falling", "late_spike", "staircase"])
def test_reference_moves_with_the_row_maximum(oracle, mode, pattern, D):
    """Logits whose row maximum keeps moving from tile to tile: the exponent reference has to
    follow it (rescaling what was accumulated) however late and however often it jumps."""
    print(f"case mode={mode} pattern={pattern} D={D}", flush=True)
    rng = np.random.default_rng(81)
    Nq, Nk = 96, 640                                   # ten 64-key tiles
    qf = rng.standard_normal((1, 2, Nq, D), dtype=np.float32)
    kf = rng.standard_normal((1, 2, Nk, D), dtype=np.float32) * np.float32(0.05)
    vf = rng.standard_normal((1, 2, Nk, D), dtype=np.float32)
    # keys get a component along each head's mean query direction, so q.k has a large common part
    u = qf.mean(axis=2, keepdims=True)
    u /= np.linalg.norm(u, axis=-1, keepdims=True)
    qf = qf * np.float32(0.2) + 6.0 * u                 # q.u ~ 6 for every row
    j = np.arange(Nk, dtype=np.float32)
    amp = {"rising": j / 16.0,                          # +4 per tile in q.k/6 ... steadily upward
           "falling": (Nk - j) / 16.0,
           "late_spike": np.where(j == Nk - 3, 30.0, 0.0),
           "staircase": np.floor(j / 64.0) * 6.0}[pattern].astype(np.float32)
    kf = kf + amp[None, None, :, None] * u
    q, k, v = (I.f32_to_bits(a, I.F16) for a in (qf, kf, vf))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, 1.0, False, I.F16)
    o, lse = run_fa_fwd(q, k, v, 1.0, False, I.F16)
    of = I.bits_to_f64(o, I.F16)
    assert np.isfinite(of).all() and np.isfinite(lse).all()
    assert np.abs(of - o_ref).max() <= 1e-2
    # lse values reach the hundreds here: fp32 output and fp32 accumulation of a 128-term dot product
    assert (np.abs(lse - lse_ref) <= 1e-3 + 1e-6 * np.abs(lse_ref)).all()


def test_rerun_is_bitwise_reproducible():
    print("case reproducible", flush=True)
    cfg = I.CONFIGS["C1"]
    q, k, v = I.make_qkv(cfg)
    a = run_fa_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    b = run_fa_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])


@pytest.mark.parametrize("name", ["C1", "C2"])
def test_config_full(oracle, mode, name):
    cfg = I.CONFIGS[name]
    print(f"case mode={mode} {cfg.describe()}", flush=True)
    q, k, v = I.make_qkv(cfg)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    o, lse = run_fa_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    stats = check_against_oracle(o, lse, o_ref, lse_ref, cfg.dtype, name, named_config=True)
    print(name, stats, flush=True)
    assert stats["n_over_1e2"] == 0 and stats["n_allowance"] == 0


@pytest.mark.parametrize("name", ["C4", "C3", "C5"])
def test_config_sampled_rows(oracle, monkeypatch, name):
    """Full-size launch in the mode fa_fwd picks by itself (the one bench.py times); the oracle
    checks a seeded stratified sample of 64 rows per (b,h)."""
    options.set_fwd_mode(None)
    cfg = I.CONFIGS[name]
    print(f"case {cfg.describe()} (sampled rows)", flush=True)
    q, k, v = I.make_qkv(cfg)
    print("  inputs drawn", flush=True)
    rows = I.sample_rows(cfg)
    o, lse = run_fa_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    print("  gpu done", flush=True)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype, rows=rows)
    print("  oracle done", flush=True)
    stats = check_against_oracle(o.reshape(-1, cfg.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, cfg.dtype, name,
                                 named_config=True)
    print(name, stats, flush=True)
    assert stats["n_over_1e2"] == 0 and stats["n_allowance"] == 0
    # cheap whole-tensor properties: everything written and finite
    assert np.isfinite(lse).all()


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("shape", [(1, 1, 1, 128), (2, 3, 77, 64), (3, 5, 1000, 128), (1, 2, 4097, 64), (16, 20, 300, 128)])
def test_single_query_goes_through_the_streaming_kernel(oracle, monkeypatch, shape, dtype):
    """fa_fwd with Nq = 1 (FA_MODE_STREAM): one run per (batch, head) of the streaming kernel, which stores o
    and lse itself.  Causal or not is the same problem (the query sees every key); FA_OPT_DECODE_KERNEL = 1 sends it
    through the tile kernels, whose result differs by the 16-bit rounding of the probabilities at most."""
    B, H, Nk, D = shape
    print(f"case fa_fwd single query shape={shape} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, dtype, 5)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (1, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    assert fa.fa_fwd_plan(B, H, 1, Nk, D, 1, dtype).mode == fa.FA_MODE_STREAM
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, True, dtype)
    o_c, lse_c = run_fa_fwd(q, k, v, scale, True, dtype)
    o_n, lse_n = run_fa_fwd(q, k, v, scale, False, dtype)
    check_against_oracle(o_c, lse_c, o_ref, lse_ref, dtype, f"{shape} stream")
    assert np.array_equal(o_c, o_n) and np.array_equal(lse_c, lse_n)
    options.set_decode("mfma")
    assert fa.fa_fwd_plan(B, H, 1, Nk, D, 1, dtype).mode != fa.FA_MODE_STREAM
    o_t, lse_t = run_fa_fwd(q, k, v, scale, True, dtype)
    check_against_oracle(o_t, lse_t, o_ref, lse_ref, dtype, f"{shape} tile")
    d = np.abs(I.bits_to_f64(o_c, dtype) - I.bits_to_f64(o_t, dtype))
    # lse: the tile kernels' fp16 row sum adds up the probabilities as rounded to fp16 (2^-11 relative per term at worst,
    # far less once a few terms average out); their bf16 row sum is unrounded, like the streaming kernel's
    assert d.max() <= (2e-3 if dtype == I.F16 else 1.6e-2)
    assert np.abs(lse_c - lse_t).max() <= (2.5e-4 if dtype == I.F16 else 1e-5)


def test_tensors_of_more_than_2_to_31_elements(oracle):
    """B = 16, H = 32, N = 32768, D = 128: each tensor holds 2^31 elements (4 GiB), so every offset past the first
    half of the tensors needs more than 32 bits.  The inputs are drawn on the GPU (2^33 bytes of normals would
    take minutes on the host); three heads -- the first, one in the middle, the very last -- are copied back and
    checked against the oracle on sampled rows, the last rows of the last head included."""
    import torch
    B, H, N, D, dtype = 16, 32, 32768, 128, I.BF16
    print(f"case fa_fwd large tensors B={B} H={H} N={N} D={D}", flush=True)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(4242)
    q, k, v = (torch.randn((B, H, N, D), generator=gen, device=dev, dtype=torch.bfloat16) for _ in range(3))
    assert q.numel() == 2**31
    o = torch.full((B, H, N, D), float("nan"), device=dev, dtype=torch.bfloat16)
    lse = torch.full((B, H, N), float("nan"), device=dev, dtype=torch.float32)
    scale = 1.0 / math.sqrt(D)
    fa.fa_fwd(q, k, v, o, lse, B, H, N, N, D, scale, 1, dtype, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    assert not torch.isnan(lse).any().item()
    rng = np.random.default_rng(4243)
    for b, h in ((0, 0), (7, 13), (B - 1, H - 1)):
        bits = [t[b, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16).reshape(1, 1, N, D) for t in (q, k, v)]
        rows = np.unique(np.concatenate([rng.integers(0, N, size=48), [0, 1, N - 2, N - 1]]))
        o_ref, lse_ref = oracle.attention_fwd(bits[0], bits[1], bits[2], scale, True, dtype, rows=rows)
        o_h = o[b, h].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)[rows]
        lse_h = lse[b, h].cpu().numpy()[rows]
        check_against_oracle(o_h, lse_h, o_ref, lse_ref, dtype, f"large tensors head {b},{h}")
