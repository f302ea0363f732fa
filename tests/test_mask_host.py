"""Host-side checks of the descriptor-mask logic the kernel runs (tile classification and the
workgroup's walk, exposed through the C ABI), by brute force against explicit keep-matrices, and the
argument errors of fa_fwd_masked.  No GPU needed."""
import itertools

import numpy as np
import pytest

from paper_2410_16663_amd import binding as fa

BN = 64


@pytest.fixture(scope="module")
def lib():
    return fa.load()


def keep_matrix(Nq, Nk, left, right, prefix, klen, anchor=0):
    """The predicate of include/fa.h, written out per element (anchor: the diag_from_kv_len member)."""
    i = np.arange(Nq)[:, None]
    j = np.arange(Nk)[None, :]
    diag = i + ((klen if anchor else Nk) - Nq)
    win = np.ones((Nq, Nk), dtype=bool)
    if left >= 0:
        win &= j >= diag - left
    if right >= 0:
        win &= j <= diag + right
    return (j < klen) & ((j < prefix) | win)


DESCRIPTORS = [
    # left, right, prefix
    (-1, 0, 0), (-1, -1, 0), (100, 0, 0), (0, 0, 0), (63, 0, 0), (64, 0, 0), (200, 30, 0), (-1, 70, 0), (40, -1, 0),
    (-1, 0, 130), (90, 0, 64), (10, 10, 1), (0, 0, 500), (-1, 0, 10**6), (2**31 - 1, 2**31 - 1, 0),
]
SHAPES = [(300, 300), (130, 700), (700, 130), (1, 500), (257, 64), (64, 65)]


@pytest.mark.parametrize("anchor", [0, 1])
@pytest.mark.parametrize("Nq,Nk", SHAPES)
@pytest.mark.parametrize("left,right,prefix", DESCRIPTORS)
def test_tile_class_is_never_wrong_and_exact_where_it_must_be(lib, left, right, prefix, Nq, Nk, anchor):
    for klen in sorted({Nk, max(Nk - 37, 0), min(64, Nk), 0}):
        keep = keep_matrix(Nq, Nk, left, right, prefix, klen, anchor)
        for r0 in range(0, Nq, 32):                       # a wave's 32 rows
            r1 = min(r0 + 31, Nq - 1)
            for k0 in range(0, Nk, BN):
                blk = keep[r0:r1 + 1, k0:k0 + BN]
                cls = fa.fa_mask_tile_class(left, right, prefix, klen, Nq, Nk, r0, r1, k0, anchor)
                if cls == fa.FA_TILE_SKIP:
                    assert not blk.any(), (r0, k0, klen)
                elif cls == fa.FA_TILE_FULL:
                    assert blk.all() and blk.shape[1] == BN, (r0, k0, klen)
                else:
                    assert cls == fa.FA_TILE_PARTIAL
                # without a prefix the classification is exact: a mixed tile is the only partial one
                if prefix == 0:
                    want = fa.FA_TILE_SKIP if not blk.any() else (
                        fa.FA_TILE_FULL if blk.all() and blk.shape[1] == BN else fa.FA_TILE_PARTIAL)
                    assert cls == want, (r0, k0, klen, cls, want)


@pytest.mark.parametrize("anchor", [0, 1])
@pytest.mark.parametrize("Nq,Nk", SHAPES)
@pytest.mark.parametrize("left,right,prefix", DESCRIPTORS)
def test_tile_walk_covers_every_visible_tile_once_and_nothing_far_away(lib, left, right, prefix, Nq, Nk, anchor):
    ntiles = (Nk + BN - 1) // BN
    for klen in sorted({Nk, max(Nk - 37, 0), Nk // 2, 0}):
        keep = keep_matrix(Nq, Nk, left, right, prefix, klen, anchor)
        for R0 in range(0, Nq, 256):                      # a workgroup's 256 rows
            R1 = min(R0 + 255, Nq - 1)
            walk = fa.fa_mask_tile_walk(left, right, prefix, klen, Nq, Nk, R0, R1, anchor)
            assert len(set(walk)) == len(walk) and all(0 <= t < ntiles for t in walk)
            assert all(t * BN < klen for t in walk)       # never a tile of pure padding
            needed = {t for t in range(ntiles) if keep[R0:R1 + 1, t * BN:(t + 1) * BN].any()}
            assert needed <= set(walk)
            # the walk is the prefix tiles plus one contiguous run: at most the gap-free hull of what is needed
            if needed and prefix == 0:
                assert set(walk) == set(range(min(needed), max(needed) + 1))
                # ... walked in ascending order from tile 0, or rotated so that position i holds a tile
                # congruent to i modulo the length of the run
                if min(walk) == 0 or len(walk) < 32:
                    assert walk == sorted(walk)
                else:
                    assert all(t % len(walk) == i for i, t in enumerate(walk))


@pytest.mark.parametrize("anchor", [0, 1])
@pytest.mark.parametrize("Nq,Nk", SHAPES + [(1024, 1024), (300, 1100)])
@pytest.mark.parametrize("left,right,prefix", DESCRIPTORS + [(300, 0, 0), (400, 100, 0), (-1, 0, 300), (500, 0, 256)])
def test_interior_run_only_holds_tiles_that_need_no_check(lib, left, right, prefix, Nq, Nk, anchor):
    for klen in sorted({Nk, max(Nk - 37, 0), Nk // 2, 0}):
        for R0 in range(0, Nq, 256):
            R1 = min(R0 + 255, Nq - 1)
            walk = fa.fa_mask_tile_walk(left, right, prefix, klen, Nq, Nk, R0, R1, anchor)
            for r0 in range(R0, R1 + 1, 32):
                r1 = min(r0 + 31, Nq - 1)
                first, count = fa.fa_mask_interior_run(left, right, prefix, klen, Nq, Nk, R0, R1, r0, r1, anchor)
                assert first % 2 == 0 and count % 2 == 0 and first >= 0 and count >= 0
                assert first + count <= max(len(walk) - 1, 0)        # a next position always exists
                cls = [fa.fa_mask_tile_class(left, right, prefix, klen, Nq, Nk, r0, r1, t * BN, anchor) for t in walk]
                for j in range(first, first + count):
                    assert cls[j] == fa.FA_TILE_FULL, (klen, R0, r0, j)
                    assert (walk[j + 1] + 1) * BN <= Nk, (klen, R0, r0, j)   # loaded without a bounds check
                # it is not needlessly short: the longest run of FULL tiles (with a loadable successor) is at most
                # three positions longer (two for evenness at either end, one for the successor)
                ok = [c == fa.FA_TILE_FULL and j + 1 < len(walk) and (walk[j + 1] + 1) * BN <= Nk
                      for j, c in enumerate(cls)]
                best = cur = 0
                for x in ok:
                    cur = cur + 1 if x else 0
                    best = max(best, cur)
                if prefix == 0 or left < 0:      # (a prefix run and a window run that touch are not joined)
                    assert count >= best - 3, (klen, R0, r0, first, count, best)


BIG_SHAPES = [(3000, 3000), (2500, 4100), (4100, 2500)]
BIG_DESCRIPTORS = [(2200, 0, 0), (2048, 300, 0), (2300, 0, 128), (2100, 2100, 0), (2500, 0, 700)]


@pytest.mark.parametrize("Nq,Nk", BIG_SHAPES)
@pytest.mark.parametrize("left,right,prefix", BIG_DESCRIPTORS)
def test_long_windows_are_walked_rotated_and_still_cover_everything(lib, left, right, prefix, Nq, Nk):
    """Window runs of 32 tiles and more: the rotated walk, its classification and its check-free run."""
    for anchor in (0, 1):
        test_tile_walk_covers_every_visible_tile_once_and_nothing_far_away(lib, left, right, prefix, Nq, Nk, anchor)
        test_interior_run_only_holds_tiles_that_need_no_check(lib, left, right, prefix, Nq, Nk, anchor)
    rotated = 0
    for R0 in range(0, Nq, 256):
        R1 = min(R0 + 255, Nq - 1)
        walk = fa.fa_mask_tile_walk(left, right, prefix, Nk, Nq, Nk, R0, R1)
        rotated += walk != sorted(walk)
    if prefix < 512 and Nk >= Nq:                        # (a long prefix or few keys merge the window run into one from tile 0)
        assert rotated > 0                               # the case is exercised at all


def test_causal_walk_matches_the_causal_plan(lib):
    """(-1, 0) walks what fa_fwd's wide mode walks for the same rows."""
    Nq = Nk = 2048
    for R0 in range(0, Nq, 256):
        walk = fa.fa_mask_tile_walk(-1, 0, 0, Nk, Nq, Nk, R0, R0 + 255)
        assert walk == list(range((R0 + 255) // BN + 1))
    total = sum(len(fa.fa_mask_tile_walk(-1, 0, 0, Nk, Nq, Nk, R0, R0 + 255)) for R0 in range(0, Nq, 256))
    import options
    options.set_fwd_mode("wide")
    assert total == fa.fa_fwd_plan(1, 1, Nq, Nk, 128, 1, 0).tiles_visited


def test_sliding_window_walk_is_short(lib):
    """A causal window of W keys: each 256-row workgroup walks about (W + 256) / 64 tiles, whatever N is."""
    N, W = 32768, 4096
    for R0 in (0, 8192, N - 256):
        walk = fa.fa_mask_tile_walk(W - 1, 0, 0, N, N, N, R0, R0 + 255)
        lo, hi = max(0, R0 - (W - 1)) // BN, (R0 + 255) // BN
        assert sorted(walk) == list(range(lo, hi + 1))
    # neighbouring query blocks read their common tiles at the same positions of their walks
    w1 = fa.fa_mask_tile_walk(W - 1, 0, 0, N, N, N, 8192, 8192 + 255)
    w2 = fa.fa_mask_tile_walk(W - 1, 0, 0, N, N, N, 8192 + 256, 8192 + 511)
    assert len(w1) == len(w2) and sum(a == b for a, b in zip(w1, w2)) == len(w1) - 4
    assert len(fa.fa_mask_tile_walk(W - 1, 0, 0, N, N, N, 8192, 8192 + 255)) == (W + 256) // BN


GOOD = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=1, H=1, Nq=8, Nk=8, D=64, scale=0.125,
            left=-1, right=0, prefix=0, kv_len=0, dtype=0)


@pytest.mark.parametrize("change,code", [
    (dict(q=0), fa.FA_ERR_NULL), (dict(lse=0), fa.FA_ERR_NULL), (dict(Nq=0), fa.FA_ERR_SHAPE),
    (dict(D=32), fa.FA_ERR_HEADDIM), (dict(dtype=5), fa.FA_ERR_DTYPE), (dict(scale=float("inf")), fa.FA_ERR_SCALE),
    (dict(prefix=-1), fa.FA_ERR_MASK), (dict(kv_len=0x6002), fa.FA_ERR_ALIGN), (dict(o=0x4008), fa.FA_ERR_ALIGN),
    (dict(Nq=2**30, Nk=64), fa.FA_ERR_SHAPE),
])
def test_masked_argument_errors_come_back_before_any_launch(lib, change, code):
    args = dict(GOOD)
    args.update(change)
    assert fa.fa_fwd_masked_raw(**args) == code
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_masked(**args)
    assert e.value.code == code


DEC_GOOD = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=2, H=4, Nk=6400, D=128, scale=0.1,
                left=-1, right=0, prefix=0, kv_len=0x7000, dtype=1, nsplit=4, workspace=0x8000, workspace_bytes=1 << 30)


@pytest.mark.parametrize("change,code", [
    (dict(k=0), fa.FA_ERR_NULL), (dict(Nk=0), fa.FA_ERR_SHAPE), (dict(D=96), fa.FA_ERR_HEADDIM),
    (dict(dtype=2), fa.FA_ERR_DTYPE), (dict(scale=float("nan")), fa.FA_ERR_SCALE), (dict(prefix=-3), fa.FA_ERR_MASK),
    (dict(kv_len=0x7001), fa.FA_ERR_ALIGN), (dict(nsplit=5000), fa.FA_ERR_NSPLIT),
    (dict(workspace=0), fa.FA_ERR_WORKSPACE), (dict(workspace_bytes=4 * 2 * 4 * 130 * 4 - 1), fa.FA_ERR_WORKSPACE),
    (dict(workspace=0x8004), fa.FA_ERR_ALIGN), (dict(Nk=2**30), fa.FA_ERR_SHAPE),
])
def test_decode_masked_argument_errors_come_back_before_any_launch(lib, change, code):
    args = dict(DEC_GOOD)
    args.update(change)
    assert fa.fa_decode_masked_raw(**args) == code
    with pytest.raises(fa.FaError) as e:
        fa.fa_decode_masked(**args)
    assert e.value.code == code


def test_null_descriptor_and_bad_host_queries(lib):
    L = fa.load()
    assert L.fa_fwd_masked(0x1000, 0x2000, 0x3000, 0x4000, 0x5000, 1, 1, 8, 8, 64, 0.1, None, 0, None) == fa.FA_ERR_NULL
    with pytest.raises(fa.FaError):
        fa.fa_mask_tile_class(-1, 0, 0, 9, 8, 8, 0, 7, 0)        # key count beyond Nk
    with pytest.raises(fa.FaError):
        fa.fa_mask_tile_class(-1, 0, 0, 8, 8, 8, 0, 8, 0)        # row beyond Nq
    with pytest.raises(fa.FaError):
        fa.fa_mask_tile_class(-1, 0, 0, 8, 8, 128, 0, 7, 32)     # not a tile boundary
    with pytest.raises(fa.FaError):
        fa.fa_mask_tile_walk(-1, 0, -2, 8, 8, 8, 0, 7)
    import ctypes
    bad = fa.FaMask(-1, 0, 0, 2, None)                            # the diagonal flag is 0 or 1
    assert fa.load().fa_mask_tile_class(ctypes.byref(bad), 8, 8, 8, 0, 7, 0) == fa.FA_ERR_MASK
    m = fa.FaMask(-1, 0, 0, 0, None)
    tiles, n = (ctypes.c_int * 4)(), ctypes.c_int()
    assert fa.load().fa_mask_tile_walk(ctypes.byref(m), 8, 8, 8, 0, 7, tiles, 4, None) == fa.FA_ERR_NULL
    assert fa.load().fa_mask_tile_walk(ctypes.byref(m), 8, 8, 8, 0, 7, None, 4, ctypes.byref(n)) == fa.FA_ERR_NULL
    assert fa.load().fa_mask_tile_walk(ctypes.byref(m), 8, 8, 8, 0, 7, tiles, -1, ctypes.byref(n)) == fa.FA_ERR_SHAPE
    # a short array gets the first tiles only; the count is the whole walk's
    m2 = fa.FaMask(-1, 0, 0, 0, None)
    assert fa.load().fa_mask_tile_walk(ctypes.byref(m2), 640, 640, 640, 384, 639, tiles, 4, ctypes.byref(n)) == fa.FA_OK
    assert n.value == 10 and list(tiles) == [0, 1, 2, 3]
