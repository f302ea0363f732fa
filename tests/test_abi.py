"""Host-side checks of the C ABI that need no GPU: the library loads, exports what
include/fa.h declares, and rejects bad arguments before touching the HIP runtime."""
import os
import re

import pytest

from paper_2410_16663_amd import binding as fa
import options

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(fa.LIB_PATH):
        from paper_2410_16663_amd import build
        build.build()
    return fa.load()


def test_library_exports_every_declared_symbol(lib):
    hdr = open(os.path.join(ROOT, "include", "fa.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fa_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(fa.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_version_and_error_strings(lib):
    assert fa.fa_version() >= 100
    seen = set()
    for code in range(0, -12, -1):
        s = fa.fa_strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 12
    assert fa.fa_strerror(-99) == "unknown error code"


GOOD = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=1, H=1, Nq=8, Nk=8, D=64, scale=0.125,
            causal=1, dtype=0)


@pytest.mark.parametrize("change,code", [
    (dict(q=0), fa.FA_ERR_NULL), (dict(k=0), fa.FA_ERR_NULL), (dict(v=0), fa.FA_ERR_NULL),
    (dict(o=0), fa.FA_ERR_NULL), (dict(lse=0), fa.FA_ERR_NULL),
    (dict(B=0), fa.FA_ERR_SHAPE), (dict(H=-1), fa.FA_ERR_SHAPE), (dict(Nq=0), fa.FA_ERR_SHAPE),
    (dict(Nk=0), fa.FA_ERR_SHAPE), (dict(B=70000, H=70000), fa.FA_ERR_SHAPE),
    (dict(Nq=2**31 - 1, Nk=2**31 - 1), fa.FA_ERR_SHAPE), (dict(Nk=2**24, D=128), fa.FA_ERR_SHAPE),
    (dict(D=96), fa.FA_ERR_HEADDIM), (dict(D=0), fa.FA_ERR_HEADDIM), (dict(D=256), fa.FA_ERR_HEADDIM),
    (dict(dtype=2), fa.FA_ERR_DTYPE), (dict(dtype=-1), fa.FA_ERR_DTYPE),
    (dict(scale=float("nan")), fa.FA_ERR_SCALE), (dict(scale=float("inf")), fa.FA_ERR_SCALE),
    (dict(q=0x1008), fa.FA_ERR_ALIGN), (dict(o=0x4004), fa.FA_ERR_ALIGN), (dict(lse=0x5002), fa.FA_ERR_ALIGN),
])
def test_argument_errors_come_back_before_any_launch(lib, change, code):
    args = dict(GOOD)
    args.update(change)
    assert fa.fa_fwd_raw(**args) == code
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd(**args)
    assert e.value.code == code


SPLITKV_GOOD = dict(GOOD, Nq=1, Nk=4096, nsplit=0, workspace=0x6000, workspace_bytes=1 << 30)


@pytest.mark.parametrize("change,code", [
    (dict(q=0), fa.FA_ERR_NULL), (dict(lse=0), fa.FA_ERR_NULL),
    (dict(Nk=0), fa.FA_ERR_SHAPE), (dict(D=96), fa.FA_ERR_HEADDIM), (dict(dtype=3), fa.FA_ERR_DTYPE),
    (dict(scale=float("nan")), fa.FA_ERR_SCALE), (dict(v=0x3004), fa.FA_ERR_ALIGN),
    (dict(workspace=0), fa.FA_ERR_WORKSPACE), (dict(workspace_bytes=16), fa.FA_ERR_WORKSPACE),
    (dict(workspace=0x6008), fa.FA_ERR_ALIGN), (dict(nsplit=1025), fa.FA_ERR_NSPLIT),
])
def test_splitkv_argument_errors_come_back_before_any_launch(lib, change, code):
    args = dict(SPLITKV_GOOD)
    args.update(change)
    assert fa.fa_fwd_splitkv_raw(**args) == code
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_splitkv(**args)
    assert e.value.code == code


@pytest.mark.parametrize("decode_kernel", ["stream", "mfma"])
def test_splitkv_plan(lib, monkeypatch, decode_kernel):
    """Nq = 1 goes to the streaming kernel (one workgroup per (batch, head) and run, no rounding of the grid)
    unless FA_OPT_DECODE_KERNEL = 1 keeps it on the tile kernel; everything else is the tile kernel's either way."""
    options.set_decode(decode_kernel)
    stream = decode_kernel == "stream"
    # given nsplit: kept, clamped to the number of 64-key tiles
    p = fa.fa_fwd_splitkv_plan(2, 4, 1, 64 * 100, 128, 1, 0, 7)
    assert (p.nsplit, p.grid_x, p.grid_y, p.work_items, p.streaming) == (7, 8, 7, 8, int(stream))
    assert p.workspace_bytes == 7 * 2 * 4 * 1 * (128 + 2) * 4
    assert p.combine_grid == 1                                   # 8 rows, 8 rows per block at D = 128
    p = fa.fa_fwd_splitkv_plan(1, 3, 1, 64 * 100, 64, 0, 1, 2)
    assert (p.grid_x, p.grid_y, p.streaming) == ((3, 2, 1) if stream else (8, 2, 0))
    assert fa.fa_fwd_splitkv_plan(1, 1, 1, 130, 64, 0, 0, 50).nsplit == 3
    p = fa.fa_fwd_splitkv_plan(1, 1, 40, 130, 64, 0, 0, 1)
    assert p.combine_grid == 0 and p.streaming == 0                               # one run: nothing to merge
    assert fa.fa_fwd_splitkv_plan(1, 1, 40, 130, 64, 0, 0, 2).combine_grid == 3   # 16 rows per block at D = 64
    # chosen: 256 workgroups, runs of at least four tiles, at least one run
    assert fa.fa_fwd_splitkv_plan(1, 32, 1, 32768, 128, 1, 1).nsplit == 8
    p = fa.fa_fwd_splitkv_plan(8, 32, 1, 32768, 128, 1, 1)
    assert p.nsplit == 1 and p.combine_grid == 0                       # a single run needs no merge
    assert fa.fa_fwd_splitkv_plan(2, 24, 1, 32768, 128, 1, 1).nsplit == 6        # ceil(256 / 48)
    assert fa.fa_fwd_splitkv_plan(1, 8, 1, 2048, 128, 1, 1).nsplit == 8          # 32 tiles / 4
    # D = 64: 512 workgroups of the tile kernel (two fit a compute unit), 256 of the streaming kernel
    assert fa.fa_fwd_splitkv_plan(8, 32, 1, 32768, 64, 1, 1).nsplit == (1 if stream else 2)
    assert fa.fa_fwd_splitkv_plan(8, 32, 2, 32768, 64, 1, 1).nsplit == 2
    assert fa.fa_fwd_splitkv_plan(1, 1, 1, 100, 128, 1, 1).nsplit == 1
    assert fa.fa_fwd_splitkv_plan(64, 32, 300, 4096, 128, 1, 1).nsplit == 1      # enough work items already
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_splitkv_plan(1, 1, 1, 100, 128, 1, 1, 2000)
    assert e.value.code == fa.FA_ERR_NSPLIT
    assert fa.load().fa_fwd_splitkv_plan(1, 1, 8, 8, 64, 0, 0, 0, None) == fa.FA_ERR_NULL


LIN_GOOD = dict(q=0x1000, k=0x2000, v=0x3000, w=0x7000, o=0x4000, lse=0x5000, y=0x8000, B=1, H=2, Nq=300, Nk=300, D=64,
                N=256, scale=0.125, causal=1, dtype=0, row_first=0, row_count=300)


@pytest.mark.parametrize("change,code", [
    (dict(w=0), fa.FA_ERR_NULL), (dict(y=0), fa.FA_ERR_NULL), (dict(o=0), fa.FA_ERR_NULL),
    (dict(N=0), fa.FA_ERR_SHAPE), (dict(N=200), fa.FA_ERR_SHAPE), (dict(N=257), fa.FA_ERR_SHAPE),
    (dict(row_first=-1), fa.FA_ERR_SHAPE), (dict(row_count=0), fa.FA_ERR_SHAPE),
    (dict(row_first=200, row_count=101), fa.FA_ERR_SHAPE), (dict(D=100), fa.FA_ERR_HEADDIM),
    (dict(dtype=2), fa.FA_ERR_DTYPE), (dict(scale=float("nan")), fa.FA_ERR_SCALE),
    (dict(w=0x7008), fa.FA_ERR_ALIGN), (dict(y=0x8002), fa.FA_ERR_ALIGN),
])
def test_attn_linear_argument_errors_come_back_before_any_launch(lib, change, code):
    args = dict(LIN_GOOD)
    args.update(change)
    assert fa.fa_attn_linear_block_raw(**args) == code
    with pytest.raises(fa.FaError) as e:
        fa.fa_attn_linear_block(**args)
    assert e.value.code == code


def test_bench_libraries_export_what_their_header_declares_and_the_product_library_does_not(lib):
    """The measurement aids live in libraries of their own (include/fa_bench.h)."""
    import ctypes
    from paper_2410_16663_amd import bench_binding as fb, build
    build.build_bench(force=False)
    hdr = open(os.path.join(ROOT, "include", "fa_bench.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(fa_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(fb.GPU_EXPORTS) | set(fb.CPU_EXPORTS)
    g, c = fb.load_gpu(), fb.load_cpu()
    assert all(hasattr(g, n) for n in fb.GPU_EXPORTS) and all(hasattr(c, n) for n in fb.CPU_EXPORTS)
    assert not hasattr(lib, "fa_mfma_probe")
    f = ctypes.c_longlong()
    assert g.fa_mfma_probe(0, 0, 10, None, ctypes.byref(f), None) == -1
    assert g.fa_mfma_probe(0, 1, 10, 0x1000, None, None) == -1
    assert g.fa_mfma_probe(2, 0, 10, 0x1000, ctypes.byref(f), None) == -4
    assert g.fa_mfma_probe(0, 0, 0, 0x1000, ctypes.byref(f), None) == -2
    assert g.fa_mfma_probe(0, 2, 10, 0x1000, ctypes.byref(f), None) == -2
    assert g.fa_mfma_probe(0, 1, 10, 0x1002, ctypes.byref(f), None) == -6


def test_options_take_only_their_values_and_return_the_previous_one(lib):
    assert fa.fa_set_option(fa.FA_OPT_FWD_MODE, fa.FA_MODE_WIDE) == fa.FA_AUTO
    assert fa.fa_set_option(fa.FA_OPT_FWD_MODE, fa.FA_MODE_SPLIT) == fa.FA_MODE_WIDE
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 128, 1, 1).mode == fa.FA_MODE_SPLIT
    assert fa.fa_set_option(fa.FA_OPT_FWD_MODE, fa.FA_AUTO) == fa.FA_MODE_SPLIT
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 128, 1, 1).mode == fa.FA_MODE_WIDE64
    L = fa.load()
    for opt, bad in ((fa.FA_OPT_FWD_MODE, 7), (fa.FA_OPT_FWD_MODE, fa.FA_MODE_STREAM), (fa.FA_OPT_DECODE_KERNEL, 2),
                     (fa.FA_OPT_LINEAR_TILE, 64), (fa.FA_OPT_LINEAR_PANEL, 0), (fa.FA_OPT_LINEAR_OVERLAP, 2), (9, 0), (-1, 0)):
        assert L.fa_set_option(opt, bad) == fa.FA_ERR_OPTION
    with pytest.raises(fa.FaError):
        fa.fa_set_option(fa.FA_OPT_LINEAR_TILE, 100)
    for opt in range(5):
        assert L.fa_set_option(opt, fa.FA_AUTO) == fa.FA_AUTO       # the failed calls changed nothing


def test_the_library_reads_no_environment_variable(lib, monkeypatch):
    monkeypatch.setenv("FA_FWD_MODE", "split")
    monkeypatch.setenv("FA_DECODE", "mfma")
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 128, 1, 1).mode == fa.FA_MODE_WIDE64
    assert fa.fa_fwd_plan(2, 4, 1, 6400, 128, 1, 0).mode == fa.FA_MODE_STREAM


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(fa, "_lib", None)
    monkeypatch.setattr(fa, "LIB_PATH", str(tmp_path / "libfa.so"))
    with pytest.raises(FileNotFoundError):
        fa.load()


# ---------------------------------------------------------------- work decomposition (host logic)
def golden():
    import json
    return json.load(open(os.path.join(ROOT, "tests", "golden", "paper_facts.json")))


@pytest.mark.parametrize("mode", ["split", "wide"])
@pytest.mark.parametrize("T", [1, 2, 8, 64, 512])
def test_causal_plan_skips_the_tiles_above_the_diagonal(lib, monkeypatch, mode, T):
    """Square causal problem of T query blocks: block i sees i+1 of the T key blocks, so the
    walked fraction is (T+1)/(2T) -- the paper's "approximately 50%" for long sequences."""
    options.set_fwd_mode(mode)
    bm = 128 if mode == "split" else 256
    N = T * bm
    plan = fa.fa_fwd_plan(2, 3, N, N, 128, 1, 1)
    assert plan.mode == (fa.FA_MODE_SPLIT if mode == "split" else fa.FA_MODE_WIDE)
    assert (plan.block_m, plan.block_n, plan.threads) == (bm, 64, 512)
    assert plan.work_items == 6 * T and plan.grid % 8 == 0 and plan.grid >= plan.work_items
    assert plan.tiles_total == 6 * T * (N // 64)
    assert plan.tiles_visited * 2 * T == plan.tiles_total * (T + 1)
    full = fa.fa_fwd_plan(2, 3, N, N, 128, 0, 1)
    assert full.tiles_visited == full.tiles_total
    if T >= 64:
        fact = golden()["all_zero_blocks_saving"]
        assert abs((1 - plan.tiles_visited / plan.tiles_total) - fact["value"]) <= fact["tolerance"]


def folded_rows(G, g, Nq):
    """Rows of workgroup g of G under the folded assignment: of the head's 8 G blocks of 32 rows, the four
    blocks 4g .. 4g+3 and their mirror images counted from the other end."""
    rows = []
    for j in range(4):
        for blk in (4 * g + j, 8 * G - 1 - 4 * g - j):
            rows.extend(range(blk * 32, min(blk * 32 + 32, Nq)))
    return rows


def test_plan_matches_brute_force_on_ragged_shapes(lib, monkeypatch):
    import itertools
    for mode, bm in (("split", 128), ("wide", 256), ("fold", 256)):
        options.set_fwd_mode(mode)
        for Nq, Nk, causal in itertools.product((1, 100, 257, 640, 2048), (1, 63, 64, 65, 1000, 2048), (0, 1)):
            plan = fa.fa_fwd_plan(1, 1, Nq, Nk, 64, causal, 0)
            G = -(-Nq // bm)
            visited, covered = 0, []
            for g in range(G):
                if mode == "fold" and causal:
                    rows = folded_rows(G, g, Nq)
                else:
                    rows = list(range(g * bm, min(g * bm + bm, Nq)))
                covered.extend(rows)
                tiles = set()
                for i in rows:          # brute force over rows: which 64-key tiles hold a visible key
                    last = min(Nk - 1, i + Nk - Nq) if causal else Nk - 1
                    tiles.update(range(0, last // 64 + 1) if last >= 0 else ())
                visited += (max(tiles) + 1) if tiles else 0
            assert sorted(covered) == list(range(Nq)), (mode, Nq)     # every row is owned exactly once
            assert plan.tiles_visited == visited, (mode, Nq, Nk, causal)


def test_folded_assignment_balances_the_triangle(lib, monkeypatch):
    """Square causal problem: under the folded order every workgroup sees the same number of visible pairs."""
    Nq, G = 2048, 8
    work = [sum(i + 1 for i in folded_rows(G, g, Nq)) for g in range(G)]
    assert max(work) - min(work) <= 32 * 32 * 8          # within one block-diagonal of each other
    plain = [sum(i + 1 for i in range(g * 256, g * 256 + 256)) for g in range(G)]
    assert max(plain) > 10 * min(plain)
    options.set_fwd_mode("fold")
    assert fa.fa_fwd_plan(1, 32, Nq, Nq, 128, 1, 0).mode == fa.FA_MODE_WIDE_FOLD
    assert fa.fa_fwd_plan(1, 32, Nq, Nq, 128, 0, 0).mode == fa.FA_MODE_WIDE     # no triangle to balance


def test_mode_heuristic_and_override(lib, monkeypatch):
    options.set_fwd_mode(None)
    assert fa.fa_fwd_plan(1, 32, 2048, 2048, 128, 1, 0).mode == fa.FA_MODE_WIDE_FOLD  # 256 wide blocks: one per CU
    assert fa.fa_fwd_plan(1, 32, 2048, 2048, 128, 0, 0).mode == fa.FA_MODE_WIDE
    assert fa.fa_fwd_plan(1, 4, 4096, 4096, 128, 1, 0).mode == fa.FA_MODE_SPLIT       # 64 wide blocks: too few
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 128, 1, 1).mode == fa.FA_MODE_WIDE64     # long walks at D = 128
    assert fa.fa_fwd_plan(1, 32, 131072, 131072, 128, 1, 1).mode == fa.FA_MODE_WIDE64
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 64, 1, 1).mode == fa.FA_MODE_WIDE         # D = 64: no such kernel
    assert fa.fa_fwd_plan(16, 32, 2048, 2048, 128, 1, 1).mode == fa.FA_MODE_WIDE       # short walks stay
    assert fa.fa_fwd_plan(8, 32, 4096, 4096, 128, 1, 1).mode == fa.FA_MODE_WIDE        # 2048 keys on average
    assert fa.fa_fwd_plan(4, 32, 4096, 4096, 128, 0, 1).mode == fa.FA_MODE_WIDE64      # not causal: all 4096
    assert fa.fa_fwd_plan(8, 32, 512, 8192, 128, 1, 1).mode == fa.FA_MODE_WIDE64       # a chunk against a long cache
    assert fa.fa_fwd_plan(4, 32, 2048, 2048, 128, 1, 0).mode == fa.FA_MODE_WIDE_FOLD  # four full rounds
    assert fa.fa_fwd_plan(5, 32, 2048, 2048, 128, 1, 0).mode == fa.FA_MODE_WIDE       # more: dynamic dispatch
    assert fa.fa_fwd_plan(1, 40, 2048, 2048, 128, 1, 0).mode == fa.FA_MODE_SPLIT      # 1.25 rounds: fold would idle
    assert fa.fa_fwd_plan(1, 32, 4096, 4096, 128, 1, 0).mode == fa.FA_MODE_WIDE_FOLD
    assert fa.fa_fwd_plan(1, 40, 4096, 4096, 128, 1, 0).mode == fa.FA_MODE_WIDE       # 2.5 rounds: neither
    assert fa.fa_fwd_plan(8, 32, 512, 512, 128, 1, 0).mode == fa.FA_MODE_WIDE         # two blocks per head: nothing to fold
    assert fa.fa_fwd_plan(1, 8, 8192, 8192, 128, 1, 0).mode == fa.FA_MODE_SPLIT
    assert fa.fa_fwd_plan(1, 16, 8192, 8192, 128, 1, 0).mode == fa.FA_MODE_WIDE64
    assert fa.fa_fwd_plan(1, 40, 2048, 2048, 128, 0, 0).mode == fa.FA_MODE_WIDE       # not causal: nothing to even out
    options.set_fwd_mode("wide")
    assert fa.fa_fwd_plan(1, 2, 256, 256, 64, 1, 0).mode == fa.FA_MODE_WIDE
    assert fa.fa_fwd_plan(1, 2, 256, 256, 64, 1, 0).lds_bytes == 4 * 64 * 64 * 2
    options.set_fwd_mode("split")
    assert fa.fa_fwd_plan(8, 32, 8192, 8192, 128, 1, 1).lds_bytes == 2 * 4 * 64 * 128 * 2


def test_no_mask_tensor_is_ever_needed(lib):
    """Section 4.1 quotes 8 GB for a full 64K x 64K mask; the plan's only buffers are the LDS tiles."""
    fact = golden()["full_mask_bytes_at_64k"]
    assert fact["value"] == 65536 * 65536 * 2
    assert fa.fa_fwd_plan(1, 1, 65536, 65536, 128, 1, 0).lds_bytes <= 160 * 1024


def test_plan_rejects_bad_shapes(lib):
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_plan(1, 1, 8, 8, 96, 0, 0)
    assert e.value.code == fa.FA_ERR_HEADDIM
    assert fa.load().fa_fwd_plan(1, 1, 8, 8, 64, 0, 0, None) == fa.FA_ERR_NULL


def test_build_report_shows_register_only_kernels():
    """Every kernel instantiation fits two waves per SIMD (the 64-row kernel, by design, one) and touches no
    scratch memory."""
    from paper_2410_16663_amd import build
    build.build(force=True)
    # attention: 2 dtypes x 2 head dims x (causal x (split, wide, wide + split-KV) + descriptor mask);
    # paired fold: 2 dtypes x 2 head dims; combine: the same; output projection: 2 dtypes x 2 head dims x 2 tile
    # heights; streaming decode: 2 dtypes x 2 head dims x (plain, masked); 64-row waves: 2 dtypes x causal x (plain, split-KV)
    assert len(build.last_report) == 24 + 4 + 4 + 4 + 8 + 8 + 8
    for name, rep in build.last_report.items():
        assert rep["ScratchSize [bytes/lane]"] == 0 and rep["VGPRs Spill"] == 0, name
        assert rep["VGPRs"] + rep.get("AGPRs", 0) <= (512 if "fa_fwd_wide64_kernel" in name else 256), name
        assert rep["LDS Size [bytes/block]"] <= 160 * 1024, name


def test_binding_structures_have_the_headers_sizes_and_offsets(tmp_path):
    """A C program that includes include/fa.h prints sizeof and the offset of the last member of every structure
    the ABI passes; the ctypes mirrors in the binding must agree (a member added on one side only would make the
    library write past the end of the caller's structure)."""
    import ctypes
    import os
    import subprocess
    src = tmp_path / "sizes.c"
    src.write_text(
        '#include <stdio.h>\n#include <stddef.h>\n#include "fa.h"\n'
        'int main(void) {\n'
        '  printf("%zu %zu\\n", sizeof(fa_plan_t), offsetof(fa_plan_t, tiles_total));\n'
        '  printf("%zu %zu\\n", sizeof(fa_splitkv_plan_t), offsetof(fa_splitkv_plan_t, streaming));\n'
        '  printf("%zu %zu\\n", sizeof(fa_mask_t), offsetof(fa_mask_t, kv_len));\n'
        '  return 0;\n}\n')
    exe = tmp_path / "sizes"
    inc = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include")
    subprocess.run(["gcc", "-I", inc, str(src), "-o", str(exe)], check=True)
    lines = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    got = [tuple(int(x) for x in line.split()) for line in lines if line]
    want = [(ctypes.sizeof(fa.FaPlan), fa.FaPlan.tiles_total.offset),
            (ctypes.sizeof(fa.FaSplitKvPlan), fa.FaSplitKvPlan.streaming.offset),
            (ctypes.sizeof(fa.FaMask), fa.FaMask.kv_len.offset)]
    assert got == want
