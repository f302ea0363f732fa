"""The host-side C code (the oracle, the host half of the cooperative strategy) under AddressSanitizer and
UndefinedBehaviorSanitizer: a small driver is compiled together with the sources and must exit cleanly.
CPU only; GPU code is not sanitized here."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.parametrize("force_scalar", ["0", "1"])
def test_host_c_code_is_clean_under_asan_and_ubsan(tmp_path, force_scalar):
    exe = str(tmp_path / "driver_host")
    cmd = ["gcc", "-O1", "-g", "-fopenmp", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "tests", "sanitize", "driver_host.c"), os.path.join(ROOT, "oracle", "fa_oracle.c"),
           os.path.join(ROOT, "paper_2410_16663_amd", "csrc", "fa_cpu.c"),
           os.path.join(ROOT, "paper_2410_16663_amd", "csrc", "fa_bench_cpu.c"), "-o", exe, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    env = dict(os.environ)
    # another library may be preloaded ahead of the sanitizer runtime on this machine; leak checking needs ptrace
    env["ASAN_OPTIONS"] = "verify_asan_link_order=0:detect_leaks=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["OMP_NUM_THREADS"] = "4"
    r = subprocess.run([exe, force_scalar], capture_output=True, text=True, env=env, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "clean" in r.stdout


HOST_CALLS = r"""
import ctypes, itertools, sys
lib = ctypes.CDLL(sys.argv[1])
class Plan(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("block_m", ctypes.c_int), ("block_n", ctypes.c_int), ("threads", ctypes.c_int),
                ("grid", ctypes.c_int), ("lds_bytes", ctypes.c_int), ("work_items", ctypes.c_longlong),
                ("tiles_visited", ctypes.c_longlong), ("tiles_total", ctypes.c_longlong)]
class SPlan(ctypes.Structure):
    _fields_ = [("nsplit", ctypes.c_int), ("grid_x", ctypes.c_int), ("grid_y", ctypes.c_int), ("combine_grid", ctypes.c_int),
                ("work_items", ctypes.c_longlong), ("workspace_bytes", ctypes.c_longlong), ("streaming", ctypes.c_int)]
class Mask(ctypes.Structure):
    _fields_ = [("l", ctypes.c_int), ("r", ctypes.c_int), ("p", ctypes.c_int), ("kv", ctypes.c_void_p)]
big = 2**31 - 1
n = 0
for B, H, Nq, Nk, D, causal in itertools.product((1, 7, 70000), (1, 33, 70000), (1, 255, 2048, 2**29, big), (1, 64, 4097, 2**23, big),
                                                 (64, 128, 96), (0, 1)):
    p = Plan(); lib.fa_fwd_plan(B, H, Nq, Nk, D, causal, 0, ctypes.byref(p))
    s = SPlan(); lib.fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, 1, 0, ctypes.byref(s))
    lib.fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, 1, 1024, ctypes.byref(s))
    n += 1
i3 = [ctypes.c_int() for _ in range(4)]
tiles = (ctypes.c_int * 64)()
for l, r, pfx in itertools.product((-1, 0, 63, 5000, big), (-1, 0, 100, big), (0, 1, 700, big)):
    for Nq, Nk in ((1, 1), (300, 300), (130, 70000), (70000, 130), (2**29 - 100, 2**29), (2**30, 64)):
        m = Mask(l, r, pfx, None)
        for klen in (0, Nk // 2, Nk):
            for r0 in (0, max(Nq - 32, 0)):
                r1 = min(r0 + 31, Nq - 1)
                for k0 in (0, (Nk - 1) // 64 * 64):
                    lib.fa_mask_tile_class(ctypes.byref(m), klen, Nq, Nk, r0, r1, k0)
                R1 = min(r0 + 255, Nq - 1)
                lib.fa_mask_tile_walk(ctypes.byref(m), klen, Nq, Nk, r0, R1, tiles, 64, ctypes.byref(i3[2]))
                lib.fa_mask_interior_run(ctypes.byref(m), klen, Nq, Nk, r0, R1, r0, r1, ctypes.byref(i3[0]), ctypes.byref(i3[1]))
                n += 1
# argument errors of the launching entry points (nothing is launched)
vp = ctypes.c_void_p
lib.fa_fwd.argtypes = [vp] * 5 + [ctypes.c_int] * 5 + [ctypes.c_float, ctypes.c_int, ctypes.c_int, vp]
assert lib.fa_fwd(None, 1, 1, 1, 1, 1, 1, 8, 8, 64, 0.1, 1, 0, None) == -1
assert lib.fa_fwd(16, 16, 16, 16, 16, 1, 1, 8, 8, 65, 0.1, 1, 0, None) == -3
print("host calls:", n, "clean")
"""


def test_library_host_logic_is_clean_under_ubsan(tmp_path):
    """The HIP library's host code compiled with -fsanitize=undefined in trap mode (device code untouched): the
    host-only entry points -- plans, mask classification and walks, argument checks -- over extreme sizes."""
    from paper_2410_16663_amd import build
    so = str(tmp_path / "libfa_ubsan.so")
    flags = [f for f in build.HIPCC_FLAGS if not f.startswith("-Rpass")]
    cmd = [os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")] + flags + [
        "-Xarch_host", "-fsanitize=undefined", "-Xarch_host", "-fsanitize-trap=undefined", build.SRC, "-o", so]
    r = subprocess.run(cmd, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr[-2000:]
    import sys
    r = subprocess.run([sys.executable, "-c", HOST_CALLS, so], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "clean" in r.stdout
