"""fa_fwd_splitkv_static, the entry point for callers that cannot allocate: through the C ABI against fa_fwd_splitkv
(same kernels, the library's own array in place of the caller's workspace), on calls in a row that share the array."""
import numpy as np
import pytest

from paper_2410_16663_amd import binding as fa
from paper_2410_16663_amd import inputs as I


def rand_bits(rng, shape, dtype):
    return I.f32_to_bits(rng.standard_normal(shape, dtype=np.float32), dtype)


def test_sizes_beyond_the_limit_are_refused_before_any_gpu_work():
    """nsplit * B * H * Nq * (D + 2) * 4 bytes must fit in 64 MiB; the check is on the host, so fake addresses do."""
    LIMIT = 64 << 20
    args = dict(q=0x1000, k=0x2000, v=0x3000, o=0x4000, lse=0x5000, B=8, H=32, Nq=256, Nk=65536, D=128, scale=0.1,
                causal=1, dtype=1)
    need = fa.fa_fwd_splitkv_plan(8, 32, 256, 65536, 128, 1, 1, 2).workspace_bytes
    assert need == 2 * 8 * 32 * 256 * 130 * 4 and need > LIMIT
    assert fa.fa_fwd_splitkv_static_raw(nsplit=2, **args) == fa.FA_ERR_WORKSPACE
    with pytest.raises(fa.FaError) as e:
        fa.fa_fwd_splitkv_static(nsplit=2, **args)
    assert e.value.code == fa.FA_ERR_WORKSPACE and "64 MiB" in str(e.value)
    # the other argument errors come back as from fa_fwd_splitkv
    assert fa.fa_fwd_splitkv_static_raw(nsplit=2, **dict(args, q=0)) == fa.FA_ERR_NULL
    assert fa.fa_fwd_splitkv_static_raw(nsplit=2, **dict(args, D=96)) == fa.FA_ERR_HEADDIM
    assert fa.fa_fwd_splitkv_static_raw(nsplit=2000, **args) == fa.FA_ERR_NSPLIT
    assert fa.fa_fwd_splitkv_static_raw(nsplit=2, **dict(args, B=1, H=1, Nq=1, scale=float("nan"))) == fa.FA_ERR_SCALE


@pytest.mark.gpu
def test_two_calls_in_a_row_match_the_workspace_entry_point_bit_for_bit(oracle):
    """A decoding step and a chunk of prefill, then a smaller problem of each kind on the array the first call left
    behind: o and lse equal fa_fwd_splitkv's bit for bit (the kernels and the run boundaries are the same), and both
    stay within the stated tolerance of the oracle."""
    import torch
    from gpu_util import check_against_oracle
    dev = torch.device("cuda:0")
    rng = np.random.default_rng(4242)
    stream = torch.cuda.current_stream().cuda_stream
    cases = [  # B, H, Nq, Nk, D, dtype, causal, nsplit -- each followed by a smaller one
        (2, 8, 1, 20000, 128, I.BF16, 1, 0), (1, 3, 1, 777, 128, I.BF16, 1, 5),
        (2, 4, 300, 9000, 128, I.F16, 1, 6), (1, 2, 70, 1500, 64, I.F16, 0, 3),
        (1, 2, 40, 3000, 128, I.BF16, 1, 1),      # a single run: no workspace at all
    ]
    for B, H, Nq, Nk, D, dtype, causal, nsplit in cases:
        print(f"case no-alloc B={B} H={H} Nq={Nq} Nk={Nk} D={D} dt={dtype} causal={causal} nsplit={nsplit}", flush=True)
        q, k, v = (rand_bits(rng, (B, H, n, D), dtype) for n in (Nq, Nk, Nk))
        tq, tk, tv = (torch.from_numpy(a.view(np.int16)).to(dev) for a in (q, k, v))
        poison = 0x7E00 if dtype == I.F16 else 0x7FC0
        outs = []
        for which in ("workspace", "static"):
            to = torch.full((B, H, Nq, D), poison, dtype=torch.int16, device=dev)
            tl = torch.full((B, H, Nq), float("nan"), dtype=torch.float32, device=dev)
            if which == "workspace":
                plan = fa.fa_fwd_splitkv_plan(B, H, Nq, Nk, D, causal, dtype, nsplit)
                ws = torch.full(((plan.workspace_bytes + 3) // 4 + 4,), float("nan"), dtype=torch.float32, device=dev)
                fa.fa_fwd_splitkv(tq, tk, tv, to, tl, B, H, Nq, Nk, D, 0.1, causal, dtype, nsplit, ws,
                                  plan.workspace_bytes, stream)
            else:
                fa.fa_fwd_splitkv_static(tq, tk, tv, to, tl, B, H, Nq, Nk, D, 0.1, causal, dtype, nsplit, stream)
            torch.cuda.synchronize()
            outs.append((to.cpu().numpy().view(np.uint16), tl.cpu().numpy()))
        (o_w, lse_w), (o_s, lse_s) = outs
        assert np.array_equal(o_w, o_s) and np.array_equal(lse_w, lse_s)
        o_ref, lse_ref = oracle.attention_fwd(q, k, v, 0.1, bool(causal), dtype)
        check_against_oracle(o_s, lse_s, o_ref, lse_ref, dtype, f"no-alloc {B, H, Nq, Nk, D}")
