"""GPU parity of fa_fwd_splitkv (few queries against a long K/V, appendix C's decoding shape):
against the CPU fp64 oracle element by element, and against fa_fwd itself.

Same tolerances as fa_fwd: O max-abs 1e-2, O mean-abs 1e-3, LSE 1e-3.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import inputs as I
import options
from gpu_util import check_against_oracle, run_fa_fwd, run_fa_fwd_splitkv

pytestmark = pytest.mark.gpu


def rand_bits(rng, shape, dtype, mult=1.0):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(mult), dtype)


# B, H, Nq, Nk, D
DECODE_SHAPES = [
    (2, 3, 1, 1000, 128), (1, 2, 1, 4097, 64), (1, 4, 1, 20000, 128), (1, 1, 1, 63, 64), (3, 2, 2, 777, 128),
    (1, 1, 1, 1, 128), (2, 2, 1, 5, 64), (1, 3, 1, 257, 128),
]
CHUNK_SHAPES = [
    (1, 2, 37, 1500, 128), (1, 2, 300, 2000, 64), (1, 1, 512, 512, 128), (2, 1, 100, 6000, 64),
]


@pytest.fixture(params=["stream", "mfma"])
def decode_kernel(request, monkeypatch):
    """Both kernels a single-query problem can take: the register-streaming one and (FA_OPT_DECODE_KERNEL = 1 of
    include/fa.h) the tile kernel every other shape runs."""
    options.set_decode(request.param)
    return request.param


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("nsplit", [0, 1, 3, 16, 1024])
@pytest.mark.parametrize("shape", DECODE_SHAPES)
def test_decode_shapes_elementwise(oracle, shape, nsplit, causal, dtype, decode_kernel):
    B, H, Nq, Nk, D = shape
    print(f"case splitkv decode shape={shape} nsplit={nsplit} causal={causal} dtype={dtype} kernel={decode_kernel}", flush=True)
    rng = np.random.default_rng(hash((shape, causal, dtype)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    assert 1 <= plan.nsplit <= (Nk + 63) // 64
    assert plan.streaming == int(Nq == 1 and decode_kernel == "stream")
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} nsplit={nsplit} causal={causal} dt={dtype}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("nsplit", [0, 2, 5, 13])
@pytest.mark.parametrize("shape", CHUNK_SHAPES)
def test_chunked_prefill_shapes_elementwise(oracle, shape, nsplit, causal, dtype):
    """Several query rows (and query blocks) per head; causal runs end on the diagonal at different tiles
    for different waves, and some runs of the early query blocks are empty."""
    B, H, Nq, Nk, D = shape
    print(f"case splitkv chunk shape={shape} nsplit={nsplit} causal={causal} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, causal, dtype, 1)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse, _ = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} nsplit={nsplit} causal={causal} dt={dtype}")


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("shape,nsplit", [((1, 2, 512, 20000, 128), 2), ((1, 2, 512, 20001, 128), 4),
                                          ((1, 1, 700, 13000, 128), 3), ((2, 1, 300, 9000, 128), 2),
                                          ((1, 1, 1100, 12345, 128), 2)])
def test_long_runs_of_several_query_blocks(oracle, shape, nsplit, causal, dtype):
    """Several query blocks per head against runs of 4096 keys and more at D = 128: fa_fwd_splitkv gives those runs
    to the kernel with 64-row waves and the pipelined loop (every other split-KV shape to the tile kernel): runs that
    start and end anywhere in the cache, ragged last tiles, ragged row blocks, runs wholly before or partly above
    the diagonal; and the same call kept on the tile kernel gives the same result to the tolerance."""
    B, H, Nq, Nk, D = shape
    print(f"case splitkv long runs shape={shape} nsplit={nsplit} causal={causal} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, nsplit, causal, dtype, 7)) % (2**32))
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    assert plan.nsplit == nsplit
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"long runs {shape} nsplit={nsplit} causal={causal} dt={dtype}")
    options.set_fwd_mode("wide")          # keeps the tile kernel's split-KV instantiation
    o2, lse2, _ = run_fa_fwd_splitkv(q, k, v, scale, causal, dtype, nsplit)
    check_against_oracle(o2, lse2, o_ref, lse_ref, dtype, f"long runs, tile kernel {shape}")


def test_rows_without_visible_keys(oracle):
    """Causal with Nq > Nk: the first rows see nothing in any run -> o = 0, lse = -inf."""
    print("case splitkv empty rows", flush=True)
    rng = np.random.default_rng(178)
    q, k, v = (rand_bits(rng, (1, 2, n, 128), I.BF16) for n in (300, 200, 200))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, 0.1, True, I.BF16)
    assert np.isneginf(lse_ref[:, :, :100]).all()
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, 0.1, True, I.BF16, 3)
    assert plan.nsplit == 3
    check_against_oracle(o, lse, o_ref, lse_ref, I.BF16, "empty rows")
    assert (I.bits_to_f64(o, I.BF16)[:, :, :100] == 0).all()


@pytest.mark.parametrize("Nq", [1, 5])
@pytest.mark.parametrize("scale", [-0.3, 0.0, 2.0])
def test_unusual_scales_and_large_logits(oracle, scale, Nq):
    """Large logits: the runs end with very different exponent references, which the merge must reconcile
    (Nq = 1: in the streaming kernel, between the lane groups of a workgroup too)."""
    print(f"case splitkv scale={scale} Nq={Nq}", flush=True)
    rng = np.random.default_rng(179)
    q, k, v = (rand_bits(rng, (1, 2, n, 64), I.F16, m) for n, m in ((Nq, 2.0), (3000, 2.0), (3000, 1.0)))
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, True, I.F16)
    o, lse, _ = run_fa_fwd_splitkv(q, k, v, scale, True, I.F16, 9)
    check_against_oracle(o, lse, o_ref, lse_ref, I.F16, f"scale={scale}")


def test_one_dominant_key_in_one_run():
    """A key whose logit towers over the rest: the row is that key's value whichever run holds it (exact:
    every other weight underflows to zero)."""
    print("case splitkv dominant key", flush=True)
    rng = np.random.default_rng(180)
    Nk, D = 5000, 128
    q, k, v = (rand_bits(rng, (1, 1, n, D), I.F16, 0.1) for n in (1, Nk, Nk))
    for pos in (0, 2111, Nk - 1):
        kk = k.copy()
        kk[0, 0, pos] = I.f32_to_bits(I.bits_to_f64(q[0, 0, 0], I.F16).astype(np.float32) * 1000, I.F16)
        o, lse, _ = run_fa_fwd_splitkv(q, kk, v, 1.0, False, I.F16, 11)
        assert np.array_equal(o[0, 0, 0], v[0, 0, pos]), pos


def test_streaming_and_tile_kernels_agree():
    """The two kernels of the single-query case on the same inputs: both within the tolerance of the oracle
    (checked above), and within fp32 rounding of each other apart from the tile kernel's 16-bit probabilities."""
    print("case splitkv streaming vs tile kernel", flush=True)
    import os
    rng = np.random.default_rng(182)
    for dtype, D in ((I.F16, 128), (I.BF16, 64)):
        q, k, v = (rand_bits(rng, (2, 3, n, D), dtype) for n in (1, 9000, 9000))
        res = {}
        for kern in ("stream", "mfma"):
            options.set_decode(kern)
            res[kern] = run_fa_fwd_splitkv(q, k, v, 0.1, True, dtype, 0)
        (o0, lse0, p0), (o1, lse1, p1) = res["stream"], res["mfma"]
        assert p0.streaming == 1 and p1.streaming == 0
        d = np.abs(I.bits_to_f64(o0, dtype) - I.bits_to_f64(o1, dtype))
        assert d.max() <= (1e-3 if dtype == I.F16 else 8e-3)
        # the tile kernels' fp16 row sum adds up the probabilities as rounded to fp16; bf16's and the streaming kernel's do not
        assert np.abs(lse0 - lse1).max() <= (2.5e-4 if dtype == I.F16 else 1e-5)


def test_matches_fa_fwd_and_ignores_workspace_contents(monkeypatch):
    """Same inputs through both entry points: equal up to fp32 rounding order; a larger, NaN-filled
    workspace changes nothing; one run (nsplit = 1) walks the tiles exactly as fa_fwd's wide mode does."""
    print("case splitkv vs fa_fwd", flush=True)
    options.set_fwd_mode("wide")
    rng = np.random.default_rng(181)
    for dtype in (I.F16, I.BF16):
        q, k, v = (rand_bits(rng, (2, 2, n, 128), dtype) for n in (70, 3000, 3000))
        o0, lse0 = run_fa_fwd(q, k, v, 0.09, True, dtype)
        o1, lse1, _ = run_fa_fwd_splitkv(q, k, v, 0.09, True, dtype, 1)
        assert np.array_equal(o0, o1) and np.array_equal(lse0, lse1)
        o2, lse2, _ = run_fa_fwd_splitkv(q, k, v, 0.09, True, dtype, 6)
        o3, lse3, _ = run_fa_fwd_splitkv(q, k, v, 0.09, True, dtype, 6, extra_workspace=4096)
        assert np.array_equal(o2, o3) and np.array_equal(lse2, lse3)
        d = np.abs(I.bits_to_f64(o0, dtype) - I.bits_to_f64(o2, dtype))
        assert d.max() <= (2e-3 if dtype == I.F16 else 1.6e-2)
        assert np.abs(lse0 - lse2).max() <= (2.5e-4 if dtype == I.F16 else 1e-5)


def test_decode_at_cache_size_on_sampled_heads(oracle):
    """The decoding workload bench.py times (inputs.DECODE, same seeded tensors, library-chosen nsplit):
    every head is run, a sample of them is checked."""
    cfg = I.DECODE
    print("case splitkv " + cfg.describe(), flush=True)
    q, k, v = I.make_qkv(cfg)
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, cfg.scale, cfg.causal, cfg.dtype, 0)
    assert plan.nsplit == 4 and plan.grid_x * plan.grid_y == 256
    for b, h in ((0, 0), (1, 17), (1, 31), (0, 8)):
        o_ref, lse_ref = oracle.attention_fwd(q[b:b + 1, h:h + 1], k[b:b + 1, h:h + 1], v[b:b + 1, h:h + 1],
                                              cfg.scale, cfg.causal, cfg.dtype)
        check_against_oracle(o[b:b + 1, h:h + 1], lse[b:b + 1, h:h + 1], o_ref, lse_ref, cfg.dtype, f"DEC head {b},{h}",
                             named_config=True)


def test_chunked_prefill_at_full_size_on_sampled_rows(oracle):
    """The chunked-prefill workload bench.py times (inputs.CHUNKED, same seeded tensors, library-chosen nsplit): 512
    new tokens per head against 32768 keys, bottom-right-aligned causal mask; a stratified sample of rows (16 per head,
    the first and the last row of the chunk among them) is checked."""
    cfg = I.CHUNKED
    print("case splitkv " + cfg.describe(), flush=True)
    q, k, v = I.make_qkv(cfg)
    o, lse, plan = run_fa_fwd_splitkv(q, k, v, cfg.scale, cfg.causal, cfg.dtype, 0)
    assert plan.streaming == 0 and plan.nsplit > 1 and plan.grid_x * plan.grid_y >= 256
    rows = I.sample_rows(cfg, per_head=16, stratum=32)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype, rows=rows)
    stats = check_against_oracle(o.reshape(-1, cfg.D)[rows], lse.reshape(-1)[rows], o_ref, lse_ref, cfg.dtype,
                                 "CHUNK sample", named_config=True)
    print("CHUNK", stats, flush=True)
    assert np.isfinite(lse).all()


@pytest.mark.parametrize("kernel", ["stream", "mfma"])
def test_cache_of_more_than_2_to_31_elements(oracle, monkeypatch, kernel):
    """B = 64, H = 32, Nk = 8192, D = 128: K and V hold 2^31 elements each, so the last heads sit past 32-bit
    offsets.  Inputs drawn on the GPU; the first, a middle and the very last head are checked against the oracle."""
    import torch
    from paper_2410_16663_amd import binding as fa
    options.set_decode(kernel)
    B, H, Nk, D, dtype = 64, 32, 8192, 128, I.F16
    print(f"case splitkv large cache B={B} H={H} Nk={Nk} D={D} kernel={kernel}", flush=True)
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(4343)
    q = torch.randn((B, H, 1, D), generator=gen, device=dev, dtype=torch.float16)
    k, v = (torch.randn((B, H, Nk, D), generator=gen, device=dev, dtype=torch.float16) for _ in range(2))
    assert k.numel() == 2**31
    o = torch.full_like(q, float("nan"))
    lse = torch.full((B, H, 1), float("nan"), device=dev, dtype=torch.float32)
    scale = 1.0 / math.sqrt(D)
    for nsplit in (0, 3):
        plan = fa.fa_fwd_splitkv_plan(B, H, 1, Nk, D, 1, dtype, nsplit)
        ws = torch.empty((plan.workspace_bytes + 3) // 4, device=dev, dtype=torch.float32)
        fa.fa_fwd_splitkv(q, k, v, o, lse, B, H, 1, Nk, D, scale, 1, dtype, nsplit, ws, plan.workspace_bytes,
                          torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        assert not torch.isnan(lse).any().item()
        for b, h in ((0, 0), (31, 17), (B - 1, H - 1)):
            qb, kb, vb = (t[b:b + 1, h:h + 1].contiguous().view(torch.int16).cpu().numpy().view(np.uint16) for t in (q, k, v))
            o_ref, lse_ref = oracle.attention_fwd(qb, kb, vb, scale, True, dtype)
            o_h = o[b:b + 1, h:h + 1].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            check_against_oracle(o_h, lse[b:b + 1, h:h + 1].cpu().numpy(), o_ref, lse_ref, dtype, f"head {b},{h} nsplit={nsplit}")
