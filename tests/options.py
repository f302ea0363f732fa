"""Forcing the library's choices from tests: thin names over fa_set_option of include/fa.h.
tests/conftest.py puts every option back to automatic after each test."""
from paper_2410_16663_amd import binding as fa

_FWD = {"split": fa.FA_MODE_SPLIT, "wide": fa.FA_MODE_WIDE, "fold": fa.FA_MODE_WIDE_FOLD, "wide64": fa.FA_MODE_WIDE64,
        None: fa.FA_AUTO}
_DEC = {"stream": 0, "mfma": 1, None: fa.FA_AUTO}


def set_fwd_mode(name):
    """"split" | "wide" | "fold" | "wide64" | None (automatic)"""
    fa.fa_set_option(fa.FA_OPT_FWD_MODE, _FWD[name])


def set_decode(name):
    """"stream" | "mfma" | None (automatic = streaming)"""
    fa.fa_set_option(fa.FA_OPT_DECODE_KERNEL, _DEC[name])


def set_linear_tile(rows):
    """128 | 256 (int or str) | None"""
    fa.fa_set_option(fa.FA_OPT_LINEAR_TILE, fa.FA_AUTO if rows is None else int(rows))


def set_linear_panel(tiles):
    """>= 1 (int or str) | None"""
    fa.fa_set_option(fa.FA_OPT_LINEAR_PANEL, fa.FA_AUTO if tiles is None else int(tiles))


def set_linear_overlap(on):
    """True / False / None (the library's default: overlapped)"""
    fa.fa_set_option(fa.FA_OPT_LINEAR_OVERLAP, fa.FA_AUTO if on is None else int(bool(on)))


def reset_all():
    for opt in (fa.FA_OPT_FWD_MODE, fa.FA_OPT_DECODE_KERNEL, fa.FA_OPT_LINEAR_TILE, fa.FA_OPT_LINEAR_PANEL,
                fa.FA_OPT_LINEAR_OVERLAP):
        fa.fa_set_option(opt, fa.FA_AUTO)
