// Measurement aid for the benchmark (include/fa_bench.h): the matrix-only ceiling probe.  Its own small
// library, libfa_bench.so; the attention library neither links nor loads it.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fa.h"
#include "../../include/fa_bench.h"

namespace {

#include "fa_types.inc"
#include "fa_device.inc"
#include "fa_bench_probe_kernel.inc"

}  // namespace

extern "C" int fa_mfma_probe(int dtype, int operands, int iters, float *scratch, long long *flops, void *stream) {
    if (!scratch || !flops) return -1;
    if (dtype != FA_DTYPE_F16 && dtype != FA_DTYPE_BF16) return -4;
    if (operands != 0 && operands != 1) return -2;
    if (iters <= 0 || iters > (1 << 24)) return -2;
    if ((uintptr_t)scratch & 3) return -6;
    const int grid = 256;                                   // one workgroup of 8 waves per compute unit
    hipStream_t st = (hipStream_t)stream;
    switch ((dtype << 1) | operands) {
        case 0: hipLaunchKernelGGL((fa_mfma_probe_kernel<0, false>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        case 1: hipLaunchKernelGGL((fa_mfma_probe_kernel<0, true>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        case 2: hipLaunchKernelGGL((fa_mfma_probe_kernel<1, false>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
        default: hipLaunchKernelGGL((fa_mfma_probe_kernel<1, true>), dim3(grid), dim3(512), 0, st, scratch, iters); break;
    }
    if (hipGetLastError() != hipSuccess) return -7;
    *flops = (long long)grid * 8 * iters * 4 * (2LL * 32 * 32 * 16);
    return 0;
}
