"""The library and torch must end up on ONE HIP runtime whichever is loaded first (a PyTorch wheel ships its own
libamdhip64.so; see binding._share_torchs_hip_runtime).  Each order runs in a process of its own."""
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

BODY = r"""
import numpy as np
{first}
{second}
import torch
from paper_2410_16663_amd import binding as fa
runtimes = sorted(set(line.split()[-1] for line in open("/proc/self/maps") if "libamdhip64" in line))
print("hip runtimes mapped:", runtimes, flush=True)
assert len(runtimes) == 1, runtimes
dev = torch.device("cuda:0")
B, H, Nq, Nk, D = 1, 2, 70, 90, 64
q = torch.randn(B, H, Nq, D, device=dev, dtype=torch.float16)
k = torch.randn(B, H, Nk, D, device=dev, dtype=torch.float16)
v = torch.randn(B, H, Nk, D, device=dev, dtype=torch.float16)
o = torch.empty_like(q)
lse = torch.empty(B, H, Nq, device=dev, dtype=torch.float32)
fa.fa_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, 0.125, 0, 0, torch.cuda.current_stream().cuda_stream)
torch.cuda.synchronize()
ref = torch.softmax((q.float() @ k.float().transpose(-1, -2)) * 0.125, dim=-1) @ v.float()
err = (o.float() - ref).abs().max().item()
print("max abs difference to a plain torch attention:", err, flush=True)
assert err < 1e-2
"""

ORDERS = {
    "library first": ("from paper_2410_16663_amd import binding as fa0; fa0.load()", "import torch"),
    "torch first": ("import torch; torch.zeros(1, device='cuda:0')", "from paper_2410_16663_amd import binding as fa0; fa0.load()"),
}


@pytest.mark.parametrize("order", sorted(ORDERS))
def test_library_and_torch_share_one_hip_runtime(order):
    first, second = ORDERS[order]
    print(f"case load order: {order}", flush=True)
    r = subprocess.run([sys.executable, "-c", BODY.format(first=first, second=second)], capture_output=True, text=True,
                       timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
