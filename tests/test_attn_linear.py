"""GPU parity of fa_attn_linear / fa_attn_linear_block (attention + output projection per block of rows,
section 4.2) against the CPU fp64 oracle.

o and lse: the tolerances of fa_fwd.  y = (heads side by side) x w with w ~ N(0,1)/sqrt(H*D): the error of y is
a sum of H*D errors of o weighted by entries of size 1/sqrt(H*D), i.e. of the size of one error of o: the same
bounds apply, max-abs 1e-2 and mean-abs 1e-3.
"""
import math

import numpy as np
import pytest

from paper_2410_16663_amd import inputs as I
import options
from gpu_util import check_against_oracle, run_attn_linear, run_fa_fwd

pytestmark = pytest.mark.gpu

Y_MAX_ABS = 1e-2
Y_MEAN_ABS = 1e-3


def rand_bits(rng, shape, dtype, mult=1.0):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32) * np.float32(mult), dtype)


def make(rng, B, H, Nq, Nk, D, N, dtype):
    q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
    w = rand_bits(rng, (H * D, N), dtype, 1.0 / math.sqrt(H * D))
    return q, k, v, w


def check_y(y, y_ref, label):
    assert np.isfinite(y).all(), f"{label}: non-finite or unwritten y"
    err = np.abs(y.astype(np.float64) - y_ref)
    assert err.max() <= Y_MAX_ABS, f"{label}: y max-abs {err.max():.3e}"
    assert err.mean() <= Y_MEAN_ABS, f"{label}: y mean-abs {err.mean():.3e}"


@pytest.fixture(params=["128", "256"], autouse=True)
def tile(request, monkeypatch):
    """Force each workgroup tile height of the projection kernel in turn (FA_OPT_LINEAR_TILE of include/fa.h)."""
    options.set_linear_tile(request.param)
    return request.param


# B, H, Nq, Nk, D, N
SHAPES = [(1, 2, 300, 300, 64, 256), (2, 3, 200, 333, 128, 512), (1, 4, 130, 130, 128, 256), (2, 2, 1, 500, 64, 256),
          (1, 1, 257, 129, 128, 768)]


@pytest.mark.parametrize("dtype", [I.F16, I.BF16])
@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("rows_per_block", [0, 128, 100])
@pytest.mark.parametrize("shape", SHAPES)
def test_whole_problem_in_blocks(oracle, shape, rows_per_block, causal, dtype):
    B, H, Nq, Nk, D, N = shape
    print(f"case attn_linear shape={shape} rpb={rows_per_block} causal={causal} dtype={dtype}", flush=True)
    rng = np.random.default_rng(hash((shape, causal, dtype)) % (2**32))
    q, k, v, w = make(rng, B, H, Nq, Nk, D, N, dtype)
    scale = 1.0 / math.sqrt(D)
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, causal, dtype)
    y_ref = oracle.attention_linear(q, k, v, w, scale, causal, dtype)
    o, lse, y = run_attn_linear(q, k, v, w, scale, causal, dtype, rows_per_block=rows_per_block)
    check_against_oracle(o, lse, o_ref, lse_ref, dtype, f"{shape} rpb={rows_per_block}")
    check_y(y, y_ref, f"{shape} rpb={rows_per_block}")


@pytest.mark.parametrize("mode", ["split", "wide", "fold", "wide64"])
def test_blocks_are_independent_and_touch_only_their_rows(oracle, monkeypatch, mode):
    """Arbitrary blocks, out of order, leaving a gap: the gap's rows of o, lse, y stay as they were.  Every
    decomposition of the attention launch is run on a block whose first row is not row 0."""
    options.set_fwd_mode(mode)
    print(f"case attn_linear arbitrary blocks mode={mode}", flush=True)
    rng = np.random.default_rng(601)
    B, H, Nq, Nk, D, N = 2, 2, 1400, 1450, 128, 256
    q, k, v, w = make(rng, B, H, Nq, Nk, D, N, I.F16)
    scale = 0.09
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, scale, True, I.F16)
    y_ref = oracle.attention_linear(q, k, v, w, scale, True, I.F16)
    o, lse, y = run_attn_linear(q, k, v, w, scale, True, I.F16, blocks=[(800, 600), (0, 70), (70, 531)])
    done = np.zeros(Nq, dtype=bool)
    done[0:601] = True
    done[800:1400] = True
    check_against_oracle(o[:, :, done], lse[:, :, done], o_ref[:, :, done], lse_ref[:, :, done], I.F16, "blocks")
    check_y(y[:, done], y_ref[:, done], "blocks")
    assert np.isnan(y[:, ~done]).all() and np.isnan(lse[:, :, ~done]).all() and (o[:, :, ~done] == 0x7E00).all()


def test_tile_order_changes_no_bit(monkeypatch, tile):
    """The order in which the projection's tiles are dealt to the compute units (panels of a few row tiles,
    FA_OPT_LINEAR_PANEL of include/fa.h) decides which workgroup computes a tile, never what it computes: every
    panel height, also ones that do not divide the number of row tiles, gives the same y bit for bit."""
    print(f"case attn_linear tile order tile={tile}", flush=True)
    rng = np.random.default_rng(603)
    B, H, Nq, Nk, D, N = 3, 2, 900, 900, 64, 1024
    q, k, v, w = make(rng, B, H, Nq, Nk, D, N, I.BF16)
    results = []
    for panel in ("1", "3", "4", "7", "1000"):
        options.set_linear_panel(panel)
        o, lse, y = run_attn_linear(q, k, v, w, 0.12, True, I.BF16)
        assert np.isfinite(y).all()
        results.append(y)
    options.set_linear_panel(None)
    o, lse, y = run_attn_linear(q, k, v, w, 0.12, True, I.BF16)
    for r in results:
        assert np.array_equal(r, y)


def test_projections_on_the_second_stream_change_no_bit(tile):
    """fa_attn_linear enqueues the projections on a stream of its own behind events (FA_OPT_LINEAR_OVERLAP of
    include/fa.h): the same kernels on the same data, so o, lse and y are those of the one-stream call bit for
    bit, call after call, and work enqueued on the caller's stream afterwards sees the finished y."""
    import torch
    from paper_2410_16663_amd import binding as fa
    print(f"case attn_linear second stream tile={tile}", flush=True)
    rng = np.random.default_rng(604)
    B, H, Nq, Nk, D, N = 2, 3, 1100, 1100, 128, 512
    q, k, v, w = make(rng, B, H, Nq, Nk, D, N, I.BF16)
    options.set_linear_overlap(False)
    o0, lse0, y0 = run_attn_linear(q, k, v, w, 0.09, True, I.BF16, rows_per_block=256)
    options.set_linear_overlap(None)
    for _ in range(3):
        o1, lse1, y1 = run_attn_linear(q, k, v, w, 0.09, True, I.BF16, rows_per_block=256)
        assert np.array_equal(o0, o1) and np.array_equal(lse0, lse1) and np.array_equal(y0, y1)
    # the caller's stream is ordered after the second stream: a reduction enqueued right after the call, with no
    # synchronisation in between, reads the complete y
    dev = torch.device("cuda:0")
    tq, tk, tv, tw = (torch.from_numpy(a.view(np.int16)).to(dev) for a in (q, k, v, w))
    to = torch.zeros((B, H, Nq, D), dtype=torch.int16, device=dev)
    tl = torch.zeros((B, H, Nq), dtype=torch.float32, device=dev)
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        for _ in range(3):
            ty = torch.full((B, Nq, N), float("nan"), dtype=torch.float32, device=dev)
            fa.fa_attn_linear(tq, tk, tv, tw, to, tl, ty, B, H, Nq, Nk, D, N, 0.09, 1, I.BF16, 256, side.cuda_stream)
            total = ty.double().sum()
            ty.fill_(float("nan"))            # enqueued after the call too: must not overtake its projections
            assert abs(total.item() - y0.astype(np.float64).sum()) < 1e-6 * np.abs(y0).sum()
    side.synchronize()


def test_one_block_gives_fa_fwd_bit_for_bit_and_exact_projections():
    """The whole problem as one block runs the same attention launch as fa_fwd; with w = identity columns the
    projection returns o itself (products with 1 and 0, fp32 sums of one term)."""
    print("case attn_linear exact", flush=True)
    rng = np.random.default_rng(602)
    for dtype, D in ((I.F16, 64), (I.BF16, 128)):
        B, H, Nq, Nk = 1, 256 // D, 333, 333
        q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
        w = I.f32_to_bits(np.eye(H * D, 256, dtype=np.float32), dtype)
        o0, lse0 = run_fa_fwd(q, k, v, 0.11, True, dtype)
        o, lse, y = run_attn_linear(q, k, v, w, 0.11, True, dtype)
        assert np.array_equal(o, o0) and np.array_equal(lse, lse0)
        side_by_side = I.bits_to_f64(o, dtype).transpose(0, 2, 1, 3).reshape(B, Nq, H * D)
        assert np.array_equal(y.astype(np.float64), side_by_side)


def test_llama7b_layer_shape_on_sampled_tokens(oracle):
    """The shape bench.py times: C2's attention (32 heads of 128) and a 4096 x 4096 projection, four blocks."""
    cfg = I.CONFIGS["C2"]
    print("case attn_linear C2 + 4096x4096 projection", flush=True)
    q, k, v = I.make_qkv(cfg)
    w = I.normal_bits((cfg.H * cfg.D, 4096), 2003, cfg.dtype, 1.0 / math.sqrt(cfg.H * cfg.D))
    o, lse, y = run_attn_linear(q, k, v, w, cfg.scale, cfg.causal, cfg.dtype, rows_per_block=1024)
    rows = np.array([0, 1, 127, 128, 255, 256, 300, 511, 512, 1000, 1023, 1024, 1500, 1535, 1536, 2047])   # blocks start at 0, 512, 1536
    y_ref = oracle.attention_linear(q, k, v, w, cfg.scale, cfg.causal, cfg.dtype, rows=rows)
    check_y(y[0, rows], y_ref, "C2 projection sample")
    o_ref, lse_ref = oracle.attention_fwd(q, k, v, cfg.scale, cfg.causal, cfg.dtype)
    check_against_oracle(o, lse, o_ref, lse_ref, cfg.dtype, "C2 in blocks", named_config=True)


def test_blocks_pipeline_with_a_consumer_on_a_second_stream():
    """The use section 4.2 has in mind: after each block an event is recorded, and a second stream (default
    priority) consumes that block's rows of y -- here it copies them, standing in for the exchange between devices
    -- while the first stream goes on with the next block.  The copy must equal the result of running the blocks
    one after another with no second stream, bit for bit."""
    import torch
    from paper_2410_16663_amd import binding as fa
    print("case attn_linear two-stream pipeline", flush=True)
    B, H, Nq, Nk, D, N, dtype = 2, 4, 1100, 1100, 128, 512, I.BF16
    dev = torch.device("cuda:0")
    gen = torch.Generator(device=dev)
    gen.manual_seed(606)
    q, k, v = (torch.randn((B, H, n, D), generator=gen, device=dev, dtype=torch.bfloat16) for n in (Nq, Nk, Nk))
    w = (torch.randn((H * D, N), generator=gen, device=dev, dtype=torch.float32) / math.sqrt(H * D)).to(torch.bfloat16)
    main = torch.cuda.current_stream()
    side = torch.cuda.Stream(device=dev)
    blocks = [(0, 128), (128, 256), (384, 256), (640, 256), (896, 204)]

    def run(two_streams):
        o = torch.zeros_like(q)
        lse = torch.zeros((B, H, Nq), device=dev, dtype=torch.float32)
        y = torch.full((B, Nq, N), float("nan"), device=dev, dtype=torch.float32)
        y_out = torch.full_like(y, float("nan"))
        torch.cuda.synchronize()
        for r, n in blocks:
            fa.fa_attn_linear_block(q, k, v, w, o, lse, y, B, H, Nq, Nk, D, N, 0.09, 1, dtype, r, n, main.cuda_stream)
            if two_streams:
                ev = torch.cuda.Event()
                ev.record(main)
                side.wait_event(ev)
                with torch.cuda.stream(side):
                    y_out[:, r:r + n].copy_(y[:, r:r + n])
            else:
                y_out[:, r:r + n].copy_(y[:, r:r + n])
        if two_streams:
            main.wait_stream(side)
        torch.cuda.synchronize()
        return y_out.cpu().numpy(), y.cpu().numpy()

    serial, y_serial = run(False)
    assert np.isfinite(serial).all() and np.array_equal(serial, y_serial)
    for _ in range(3):
        piped, y_piped = run(True)
        assert np.array_equal(piped, serial) and np.array_equal(y_piped, serial)
