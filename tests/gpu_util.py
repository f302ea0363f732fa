"""Helpers for the GPU parity tests: device buffers via torch, calls through the C ABI."""
import numpy as np

from paper_2410_16663_amd import binding as fa
from paper_2410_16663_amd import inputs as I

O_MAX_ABS = 1e-2     # tolerance on O, max over elements
O_MEAN_ABS = 1e-3    # tolerance on O, mean over elements
LSE_ABS = 1e-3       # tolerance on log-sum-exp


def run_fa_fwd(q_bits, k_bits, v_bits, scale, causal, dtype, keep_device=False):
    """Copy the uint16 inputs to the GPU, run fa_fwd through the C ABI, return (o_bits, lse) as numpy."""
    import torch
    assert torch.cuda.is_available()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    dev = torch.device("cuda:0")
    tq = torch.from_numpy(q_bits.view(np.int16)).to(dev)
    tk = torch.from_numpy(k_bits.view(np.int16)).to(dev)
    tv = torch.from_numpy(v_bits.view(np.int16)).to(dev)
    # poison the outputs so that anything left unwritten shows up
    to = torch.full((B, H, Nq, D), 0x7E00 if dtype == I.F16 else 0x7FC0, dtype=torch.int16, device=dev)
    tl = torch.full((B, H, Nq), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    fa.fa_fwd(tq, tk, tv, to, tl, B, H, Nq, Nk, D, scale, int(causal), dtype, stream)
    torch.cuda.synchronize()
    if keep_device:
        return (tq, tk, tv, to, tl)
    return to.cpu().numpy().view(np.uint16), tl.cpu().numpy()


def run_fa_fwd_splitkv(q_bits, k_bits, v_bits, scale, causal, dtype, nsplit=0, extra_workspace=0):
    """Same as run_fa_fwd through fa_fwd_splitkv; the workspace is filled with NaN first.

    Returns (o_bits, lse, plan)."""
    import torch
    assert torch.cuda.is_available()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    dev = torch.device("cuda:0")
    tq = torch.from_numpy(q_bits.view(np.int16)).to(dev)
    tk = torch.from_numpy(k_bits.view(np.int16)).to(dev)
    tv = torch.from_numpy(v_bits.view(np.int16)).to(dev)
    to = torch.full((B, H, Nq, D), 0x7E00 if dtype == I.F16 else 0x7FC0, dtype=torch.int16, device=dev)
    tl = torch.full((B, H, Nq), float("nan"), dtype=torch.float32, device=dev)
    plan = fa.fa_fwd_splitkv_plan(B, H, Nq, Nk, D, int(causal), dtype, nsplit)
    nbytes = plan.workspace_bytes + extra_workspace
    ws = torch.full(((nbytes + 3) // 4,), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    fa.fa_fwd_splitkv(tq, tk, tv, to, tl, B, H, Nq, Nk, D, scale, int(causal), dtype, nsplit, ws, nbytes, stream)
    torch.cuda.synchronize()
    return to.cpu().numpy().view(np.uint16), tl.cpu().numpy(), plan


def run_fa_fwd_masked(q_bits, k_bits, v_bits, scale, dtype, left=-1, right=-1, prefix=0, kv_len=None,
                      diag_from_kv_len=0):
    """Same as run_fa_fwd through fa_fwd_masked; kv_len (list of B ints or None) is copied to the GPU."""
    import torch
    assert torch.cuda.is_available()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    dev = torch.device("cuda:0")
    tq = torch.from_numpy(q_bits.view(np.int16)).to(dev)
    tk = torch.from_numpy(k_bits.view(np.int16)).to(dev)
    tv = torch.from_numpy(v_bits.view(np.int16)).to(dev)
    to = torch.full((B, H, Nq, D), 0x7E00 if dtype == I.F16 else 0x7FC0, dtype=torch.int16, device=dev)
    tl = torch.full((B, H, Nq), float("nan"), dtype=torch.float32, device=dev)
    tlen = None if kv_len is None else torch.tensor(list(kv_len), dtype=torch.int32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    fa.fa_fwd_masked(tq, tk, tv, to, tl, B, H, Nq, Nk, D, scale, left, right, prefix, tlen, dtype, stream,
                     diag_from_kv_len)
    torch.cuda.synchronize()
    return to.cpu().numpy().view(np.uint16), tl.cpu().numpy()


def run_fa_decode_masked(q_bits, k_bits, v_bits, scale, dtype, left=-1, right=-1, prefix=0, kv_len=None, nsplit=0,
                         diag_from_kv_len=0):
    """One decoding step through fa_decode_masked (q_bits [B,H,1,D]); the workspace is filled with NaN first.
    Returns (o_bits, lse, plan)."""
    import torch
    assert torch.cuda.is_available()
    B, H, Nq, D = q_bits.shape
    assert Nq == 1
    Nk = k_bits.shape[2]
    dev = torch.device("cuda:0")
    tq = torch.from_numpy(q_bits.view(np.int16)).to(dev)
    tk = torch.from_numpy(k_bits.view(np.int16)).to(dev)
    tv = torch.from_numpy(v_bits.view(np.int16)).to(dev)
    to = torch.full((B, H, 1, D), 0x7E00 if dtype == I.F16 else 0x7FC0, dtype=torch.int16, device=dev)
    tl = torch.full((B, H, 1), float("nan"), dtype=torch.float32, device=dev)
    tlen = None if kv_len is None else torch.tensor(list(kv_len), dtype=torch.int32, device=dev)
    plan = fa.fa_fwd_splitkv_plan(B, H, 1, Nk, D, 0, dtype, nsplit)
    ws = torch.full(((plan.workspace_bytes + 3) // 4 + 4,), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    fa.fa_decode_masked(tq, tk, tv, to, tl, B, H, Nk, D, scale, left, right, prefix, tlen, dtype, nsplit, ws,
                        plan.workspace_bytes, stream, diag_from_kv_len)
    torch.cuda.synchronize()
    return to.cpu().numpy().view(np.uint16), tl.cpu().numpy(), plan


def run_attn_linear(q_bits, k_bits, v_bits, w_bits, scale, causal, dtype, blocks=None, rows_per_block=0):
    """fa_attn_linear (blocks=None) or one fa_attn_linear_block call per (row_first, row_count) in ``blocks``.
    Outputs are poisoned first.  Returns (o_bits, lse, y) as numpy."""
    import torch
    assert torch.cuda.is_available()
    B, H, Nq, D = q_bits.shape
    Nk = k_bits.shape[2]
    N = w_bits.shape[1]
    dev = torch.device("cuda:0")
    tq, tk, tv, tw = (torch.from_numpy(a.view(np.int16)).to(dev) for a in (q_bits, k_bits, v_bits, w_bits))
    to = torch.full((B, H, Nq, D), 0x7E00 if dtype == I.F16 else 0x7FC0, dtype=torch.int16, device=dev)
    tl = torch.full((B, H, Nq), float("nan"), dtype=torch.float32, device=dev)
    ty = torch.full((B, Nq, N), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream().cuda_stream
    if blocks is None:
        fa.fa_attn_linear(tq, tk, tv, tw, to, tl, ty, B, H, Nq, Nk, D, N, scale, int(causal), dtype, rows_per_block,
                          stream)
    else:
        for r0, n in blocks:
            fa.fa_attn_linear_block(tq, tk, tv, tw, to, tl, ty, B, H, Nq, Nk, D, N, scale, int(causal), dtype, r0, n,
                                    stream)
    torch.cuda.synchronize()
    return to.cpu().numpy().view(np.uint16), tl.cpu().numpy(), ty.cpu().numpy()


def bf16_half_ulp(x):
    """Half a unit in the last place of bfloat16 (8 significant bits) at magnitude |x|."""
    ax = np.maximum(np.abs(x), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 8)


# elements that needed the bf16 allowance (see check_against_oracle) since the process started, per label
allowance_used = {}


def check_against_oracle(o_bits, lse, o_ref, lse_ref, dtype, label="", named_config=False):
    """Assert the stated tolerances (O max-abs 1e-2, O mean-abs 1e-3, lse 1e-3). o_bits/o_ref and lse/lse_ref
    have matching shapes.

    One allowance, and only outside the named workloads (``named_config=False``): a bf16 output whose exact
    value is 4 or more in magnitude cannot meet 1e-2 by construction -- half a unit in the last place of bf16 is
    0.0156 there -- so such an element may be off by its half-ulp plus 5e-3.  Everything below 4 in magnitude,
    every fp16 element, and every element of a named workload (``named_config=True``: C1..C5, DEC, SWA, LIN)
    must meet the plain 1e-2.  The number of elements that used the allowance is returned, printed, and kept
    in ``allowance_used``."""
    o = I.bits_to_f64(o_bits, dtype).reshape(o_ref.shape)
    assert np.isfinite(o).all(), f"{label}: non-finite or unwritten output"
    err = np.abs(o - o_ref)
    tol = np.full_like(err, O_MAX_ABS)
    n_allow = 0
    if dtype == I.BF16 and not named_config:
        big = np.abs(o_ref) >= 4.0
        if big.any():
            tol = np.where(big, bf16_half_ulp(o_ref) + 5e-3, tol)
            n_allow = int((big & (err > O_MAX_ABS)).sum())
    worst = np.unravel_index(np.argmax(err - tol), err.shape)
    assert (err <= tol).all(), (f"{label}: O max-abs {err.max():.3e}; {int((err > tol).sum())} element(s) over; worst at "
                                f"{worst}: got {o[worst]!r} want {o_ref[worst]!r} (tol {tol[worst]:.3e})")
    if n_allow:
        allowance_used[label] = allowance_used.get(label, 0) + n_allow
        print(f"{label}: {n_allow} bf16 element(s) of magnitude >= 4 used the half-ulp allowance", flush=True)
    assert err.mean() <= O_MEAN_ABS, f"{label}: O mean-abs {err.mean():.3e}"
    lse = np.asarray(lse, dtype=np.float64).reshape(lse_ref.shape)
    inf = np.isneginf(lse_ref)
    assert np.array_equal(np.isneginf(lse), inf), f"{label}: -inf pattern of lse differs"
    lerr = np.abs(lse[~inf] - lse_ref[~inf])
    assert not np.isnan(lse[~inf]).any(), f"{label}: NaN in lse"
    if lerr.size:
        assert lerr.max() <= LSE_ABS, f"{label}: lse max-abs {lerr.max():.3e}"
    return dict(o_max=float(err.max()), o_mean=float(err.mean()), lse_max=float(lerr.max()) if lerr.size else 0.0,
                n_over_1e2=int((err > O_MAX_ABS).sum()), n_allowance=n_allow)
