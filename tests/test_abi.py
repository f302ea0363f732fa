"""Host-side checks of the C ABI that need no GPU: the library loads, exports what
include/fa.h declares, and rejects bad arguments before touching the HIP runtime."""
import os
import re

import pytest

from paper_2410_16663_amd import binding as fa

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
    for code in range(0, -8, -1):
        s = fa.fa_strerror(code)
        assert s and s != "unknown error code"
        seen.add(s)
    assert len(seen) == 8
    assert fa.fa_strerror(-99) == "unknown error code"


GOOD = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=1, H=1, Nq=8, Nk=8, D=64, scale=0.125,
            causal=1, dtype=0)


@pytest.mark.parametrize("change,code", [
    (dict(q=0), fa.FA_ERR_NULL), (dict(k=0), fa.FA_ERR_NULL), (dict(v=0), fa.FA_ERR_NULL),
    (dict(o=0), fa.FA_ERR_NULL), (dict(lse=0), fa.FA_ERR_NULL),
    (dict(B=0), fa.FA_ERR_SHAPE), (dict(H=-1), fa.FA_ERR_SHAPE), (dict(Nq=0), fa.FA_ERR_SHAPE),
    (dict(Nk=0), fa.FA_ERR_SHAPE), (dict(B=70000, H=70000), fa.FA_ERR_SHAPE),
    (dict(Nq=2**31 - 1, Nk=2**31 - 1), fa.FA_ERR_SHAPE),
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


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    monkeypatch.setattr(fa, "_lib", None)
    monkeypatch.setattr(fa, "LIB_PATH", str(tmp_path / "libfa.so"))
    with pytest.raises(FileNotFoundError):
        fa.load()
