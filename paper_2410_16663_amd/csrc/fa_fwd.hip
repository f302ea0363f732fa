// Exact attention forward for gfx950 (MI355X): kernels and the C ABI of include/fa.h.
//
// Dataflow (FastAttention appendix A, the FlashAttention2 forward): for each block of
// queries, walk the key/value blocks once; per block compute the logits on the matrix
// cores, exponentiate against a running row maximum, multiply by V on the matrix cores,
// and carry the running row maximum / row sum.  Mask handling follows section 4.1:
// blocks that are entirely masked are skipped, blocks that are entirely visible take no
// mask, and only blocks straddling the diagonal (or the ragged end of K) get a
// per-element predicate computed from indices -- no mask tensor exists.
//
// gfx950 mapping (this file's own design):
//  * one wavefront owns 32 query rows; a workgroup is NW wavefronts = 32*NW rows.
//  * logits are produced TRANSPOSED, S^T = K Q^T, with v_mfma_f32_32x32x16: keys on the
//    M side (A operand, read from LDS with ds_read_b128), queries on the N side (B
//    operand, held in registers for the whole kernel).  A lane then owns ONE query
//    column, so row max / row sum are in-lane reductions plus a single cross-half
//    exchange (v_permlane32_swap), and the exponentiated tile is already in the
//    B-operand register layout of the second product O^T = V^T P^T (no shuffle, no LDS
//    round trip -- the MFMA counterpart of the paper's appendix-B layout converter).
//  * V^T fragments come straight out of the row-major V tile with the transposing LDS
//    read ds_read_b64_tr_b16.
//  * K and V tiles (64 keys) are double-buffered in LDS; the next tile's global loads
//    are in flight while the current one is consumed.
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/fa.h"

namespace {

typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

#define LDS_PTR(T, p) ((__attribute__((address_space(3))) T *)(p))

struct FaParams {
    const uint16_t *q, *k, *v;
    uint16_t *o;
    float *lse;
    int H, Nq, Nk;
    int nqt;        // query tiles per (b,h)
    int nwork;      // B*H*nqt
    int per_xcd;    // ceil(nwork / 8)
    float c;        // |scale| * log2(e), or 1 when scale == 0
    float scale_abs;
    int qmode;      // 0: use q as is, 1: negate q (scale < 0), 2: zero q (scale == 0)
};

constexpr int BN = 64;  // keys per tile

template <int DT>
__device__ __forceinline__ f32x16 mfma32(s16x8 a, s16x8 b, f32x16 c) {
    if constexpr (DT == FA_DTYPE_F16)
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
    else
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
}

// two fp32 -> two 16-bit values of the storage type (round to nearest even), packed in 32 bits
template <int DT>
__device__ __forceinline__ s16x2 pack2(float a, float b) {
    f32x2 x = {a, b};
    if constexpr (DT == FA_DTYPE_F16)
        return __builtin_bit_cast(s16x2, __builtin_convertvector(x, f16x2));
    else
        return __builtin_bit_cast(s16x2, __builtin_convertvector(x, bf16x2));
}

// LDS byte offset of 16-byte chunk c of K-tile row r.  The XOR spreads the 16 rows that
// one quarter-wave reads at the same chunk index over all 64 banks.
template <int D>
__device__ __forceinline__ int k_lds_off(int r, int c) {
    if constexpr (D == 128)
        return r * 256 + ((c ^ (r & 15)) << 4);
    else
        return r * 128 + ((c ^ ((r >> 1) & 7)) << 4);
}

// LDS byte offset of byte b (of the row's D*2) of V-tile row r.  The transposing read
// fetches, per half-wave, 4 consecutive rows x 64 bytes: the XOR puts those four 64-byte
// pieces into four different bank groups.
template <int D>
__device__ __forceinline__ int v_lds_off(int r, int b) {
    if constexpr (D == 128)
        return r * 256 + (b ^ ((r & 3) << 6));
    else
        return r * 128 + (b ^ (((r >> 1) & 1) << 6));
}

// v_permlane32_swap exchanges the upper 32 lanes of its first operand with the lower 32
// lanes of its second: fed the same value twice it returns {lo,lo} and {hi,hi}, i.e. every
// lane sees both halves' values of its column.  (The two results are copied to scalars
// before the bit cast: a bit cast applied directly to an element of the returned vector
// reads element 0 whatever the index.)
__device__ __forceinline__ void xhalf_both(float x, float &lo, float &hi) {
    const unsigned a = __builtin_bit_cast(unsigned, x);
    const auto r = __builtin_amdgcn_permlane32_swap(a, a, false, false);
    const unsigned r0 = r[0], r1 = r[1];
    lo = __builtin_bit_cast(float, r0);
    hi = __builtin_bit_cast(float, r1);
}
__device__ __forceinline__ float xhalf_max(float x) {
    float lo, hi;
    xhalf_both(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float xhalf_sum(float x) {
    float lo, hi;
    xhalf_both(x, lo, hi);
    return lo + hi;
}

template <int DT, int D, bool CAUSAL, int NW>
__global__ __launch_bounds__(NW * 64, 2) void fa_fwd_kernel(const FaParams p) {
    constexpr int NT = NW * 64;
    constexpr int BM = NW * 32;
    constexpr int KB = D / 16;   // k-steps of the first product
    constexpr int DB = D / 32;   // 32-row blocks of O^T
    constexpr int ROWB = D * 2;
    constexpr int TILEB = BN * ROWB;
    constexpr int CPR = D / 8;   // 16-byte chunks per row
    constexpr int PER = BN * CPR / NT;
    static_assert(PER >= 1 && BN * CPR % NT == 0, "tile must split evenly over the threads");

    __shared__ __attribute__((aligned(16))) unsigned char smem[4 * TILEB];  // K0 K1 V0 V1

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31;
    const int h = lane >> 5;

    // ---- workgroup -> (b*H+h, query tile).  Workgroup ids are dealt round-robin to the 8
    // XCDs; give each XCD one contiguous run of the head-major work list so that the
    // workgroups sharing an L2 walk the same head's K/V.  Causal: heaviest tile first.
    const int wi = (blockIdx.x & 7) * p.per_xcd + (blockIdx.x >> 3);
    if (wi >= p.nwork) return;
    const int bh = wi / p.nqt;
    const int qt = CAUSAL ? (p.nqt - 1 - wi % p.nqt) : (wi % p.nqt);

    const int Nq = p.Nq, Nk = p.Nk;
    const int off = Nk - Nq;
    const int q_wave = qt * BM + wave * 32;       // first query row of this wave
    const int qrow = q_wave + l32;                // this lane's query row
    const bool wave_has_rows = q_wave < Nq;

    int kmax_wg = Nk - 1, kmax_wave = Nk - 1;     // last key index any row may see
    if (CAUSAL) {
        kmax_wg = min(Nk - 1, min(qt * BM + BM - 1, Nq - 1) + off);
        kmax_wave = min(Nk - 1, min(q_wave + 31, Nq - 1) + off);
    }
    const int nt = kmax_wg >= 0 ? kmax_wg / BN + 1 : 0;

    const size_t kv_head = (size_t)bh * Nk * D;
    const uint16_t *kg = p.k + kv_head;
    const uint16_t *vg = p.v + kv_head;

    // ---- Q fragments (B operand of S^T = K Q^T): lane holds d = 16*kb + 8*h + 0..7 of its row
    s16x8 qf[KB];
    {
        const uint16_t *qp = p.q + ((size_t)bh * Nq + (qrow < Nq ? qrow : 0)) * D + 8 * h;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) {
            s16x8 x = *(const s16x8 *)(qp + kb * 16);
            if (qrow >= Nq || p.qmode == 2) x = (s16x8)(0);
            if (p.qmode == 1) x ^= (s16x8)((short)0x8000);
            qf[kb] = x;
        }
    }

    // ---- staging registers for the next K/V tile
    s16x8 kreg[PER], vreg[PER];
    auto load_tile = [&](int t) {
#pragma unroll
        for (int n = 0; n < PER; ++n) {
            const int id = tid + n * NT;
            const int r = id / CPR, c = id % CPR;
            const int key = t * BN + r;
            if (key < Nk) {
                kreg[n] = *(const s16x8 *)(kg + (size_t)key * D + c * 8);
                vreg[n] = *(const s16x8 *)(vg + (size_t)key * D + c * 8);
            } else {
                kreg[n] = (s16x8)(0);
                vreg[n] = (s16x8)(0);
            }
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int n = 0; n < PER; ++n) {
            const int id = tid + n * NT;
            const int r = id / CPR, c = id % CPR;
            *(s16x8 *)(smem + buf * TILEB + k_lds_off<D>(r, c)) = kreg[n];
            *(s16x8 *)(smem + (2 + buf) * TILEB + v_lds_off<D>(r, c * 16)) = vreg[n];
        }
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db] = (f32x16)(0.f);
    float m_run = -INFINITY;   // running max of the unscaled logits of this lane's query
    float l_run = 0.f;         // this half-wave's share of the running row sum

    if (nt > 0) {
        load_tile(0);
        store_tile(0);
    }
    __syncthreads();

    // per-lane pieces of the LDS read addresses
    const int g2 = (lane >> 4) & 1, li = lane & 15, vi = li >> 2, vc = li & 3;

    for (int t = 0; t < nt; ++t) {
        const int buf = t & 1;
        const bool more = t + 1 < nt;
        if (more) load_tile(t + 1);

        const int k0 = t * BN;
        if (wave_has_rows && k0 <= kmax_wave) {
            const unsigned char *ks = smem + buf * TILEB;
            const unsigned char *vs = smem + (2 + buf) * TILEB;

            // ---- S^T = K Q^T : two 32-key blocks x 32 queries
            f32x16 s[2];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                s[mb] = (f32x16)(0.f);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) {
                    const s16x8 a = *(const s16x8 *)(ks + k_lds_off<D>(mb * 32 + l32, 2 * kb + h));
                    s[mb] = mfma32<DT>(a, qf[kb], s[mb]);
                }
            }

            // ---- mask only when the tile straddles the diagonal or the end of K
            const bool need_mask = (k0 + BN - 1 >= Nk) || (CAUSAL && (k0 + BN - 1 > q_wave + off));
            if (need_mask) {
                int lim = Nk - 1;
                if (CAUSAL) lim = min(lim, qrow + off);
#pragma unroll
                for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int key = k0 + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                        if (key > lim) s[mb][r] = -INFINITY;
                    }
            }

            // ---- online softmax; the lane's 32 logits all belong to one query
            float mx = s[0][0];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[mb][r]);
            mx = xhalf_max(mx);
            const float m_new = fmaxf(m_run, mx);
            const float mc = (m_new == -INFINITY) ? 0.f : m_new * p.c;
            const float alpha = __builtin_amdgcn_exp2f(m_run * p.c - mc);
            m_run = m_new;
            float rs = 0.f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s[mb][r], p.c, -mc));
                    s[mb][r] = e;
                    rs += e;
                }
            l_run = l_run * alpha + rs;
#pragma unroll
            for (int db = 0; db < DB; ++db) oacc[db] *= alpha;

            // ---- P^T fragments: 16-key step j takes logits registers 8*(j%2)..+7 of block j/2,
            // i.e. k-slot (h, v) of step j is key 16*j + 8*(v/4) + 4*h + v%4
            s16x8 pf[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int v2 = 0; v2 < 4; ++v2) {
                    const s16x2 pr = pack2<DT>(s[j >> 1][8 * (j & 1) + 2 * v2], s[j >> 1][8 * (j & 1) + 2 * v2 + 1]);
                    pf[j][2 * v2] = pr[0];
                    pf[j][2 * v2 + 1] = pr[1];
                }
            }

            // ---- O^T += V^T P^T : A operand rows are d, k-slots match the P^T fragments
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const int row = 16 * j + 4 * h + vi;
                    const int bcol = db * 64 + g2 * 32 + vc * 8;
                    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row, bcol)));
                    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row + 8, bcol)));
                    const s16x8 a = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                    oacc[db] = mfma32<DT>(a, pf[j], oacc[db]);
                }
            }
        }

        if (more) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: combine the two half-wave sums, normalise, store
    const float l_tot = xhalf_sum(l_run);
    if (qrow < Nq) {
        const float inv = l_tot > 0.f ? 1.f / l_tot : 0.f;
        uint16_t *op = p.o + ((size_t)bh * Nq + qrow) * D + 4 * h;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                const s16x2 a = pack2<DT>(oacc[db][4 * g] * inv, oacc[db][4 * g + 1] * inv);
                const s16x2 b = pack2<DT>(oacc[db][4 * g + 2] * inv, oacc[db][4 * g + 3] * inv);
                const s16x4 st = {a[0], a[1], b[0], b[1]};
                *(s16x4 *)(op + db * 32 + 8 * g) = st;
            }
        if (h == 0)
            p.lse[(size_t)bh * Nq + qrow] = l_tot > 0.f ? m_run * p.scale_abs + __logf(l_tot) : -INFINITY;
    }
}

template <int DT, int D, bool CAUSAL, int NW>
hipError_t launch(const FaParams &p, int nwork_padded, hipStream_t stream) {
    hipLaunchKernelGGL((fa_fwd_kernel<DT, D, CAUSAL, NW>), dim3(nwork_padded), dim3(NW * 64), 0, stream, p);
    return hipGetLastError();
}

thread_local int g_last_hip_error = 0;

}  // namespace

extern "C" {

int fa_fwd(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nq, int Nk,
           int D, float scale, int causal, int dtype, void *stream) {
    if (!q || !k || !v || !o || !lse) return FA_ERR_NULL;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0) return FA_ERR_SHAPE;
    if (D != 64 && D != 128) return FA_ERR_HEADDIM;
    if (dtype != FA_DTYPE_F16 && dtype != FA_DTYPE_BF16) return FA_ERR_DTYPE;
    if (!isfinite(scale)) return FA_ERR_SCALE;
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15) return FA_ERR_ALIGN;
    if ((uintptr_t)lse & 3) return FA_ERR_ALIGN;

    const int NW = 4;
    const int BM = 32 * NW;
    const long long bh = (long long)B * H;
    const long long nqt = ((long long)Nq + BM - 1) / BM;
    const long long nwork = bh * nqt;
    if (bh > 0x7fffffffLL || nwork > 0x7ffffff0LL) return FA_ERR_SHAPE;
    // Nq + Nk must fit in int arithmetic inside the kernel
    if ((long long)Nq + Nk > 0x7fffff00LL) return FA_ERR_SHAPE;

    FaParams p;
    p.q = (const uint16_t *)q;
    p.k = (const uint16_t *)k;
    p.v = (const uint16_t *)v;
    p.o = (uint16_t *)o;
    p.lse = lse;
    p.H = H;
    p.Nq = Nq;
    p.Nk = Nk;
    p.nqt = (int)nqt;
    p.nwork = (int)nwork;
    p.per_xcd = (int)((nwork + 7) / 8);
    const float LOG2E = 1.4426950408889634f;
    p.qmode = scale > 0.f ? 0 : (scale < 0.f ? 1 : 2);
    p.scale_abs = fabsf(scale);
    p.c = scale == 0.f ? 1.f : fabsf(scale) * LOG2E;
    const int grid = p.per_xcd * 8;
    hipStream_t st = (hipStream_t)stream;

    hipError_t e;
    const int key = (dtype << 2) | ((D == 128) << 1) | (causal ? 1 : 0);
    switch (key) {
        case 0: e = launch<0, 64, false, NW>(p, grid, st); break;
        case 1: e = launch<0, 64, true, NW>(p, grid, st); break;
        case 2: e = launch<0, 128, false, NW>(p, grid, st); break;
        case 3: e = launch<0, 128, true, NW>(p, grid, st); break;
        case 4: e = launch<1, 64, false, NW>(p, grid, st); break;
        case 5: e = launch<1, 64, true, NW>(p, grid, st); break;
        case 6: e = launch<1, 128, false, NW>(p, grid, st); break;
        default: e = launch<1, 128, true, NW>(p, grid, st); break;
    }
    if (e != hipSuccess) {
        g_last_hip_error = (int)e;
        return FA_ERR_LAUNCH;
    }
    return FA_OK;
}

const char *fa_strerror(int code) {
    switch (code) {
        case FA_OK: return "success";
        case FA_ERR_NULL: return "a required pointer is NULL";
        case FA_ERR_SHAPE: return "B, H, Nq, Nk must be positive and the problem must be indexable";
        case FA_ERR_HEADDIM: return "head dimension D must be 64 or 128";
        case FA_ERR_DTYPE: return "dtype must be 0 (fp16) or 1 (bf16)";
        case FA_ERR_SCALE: return "scale must be finite";
        case FA_ERR_ALIGN: return "q, k, v, o must be 16-byte aligned and lse 4-byte aligned";
        case FA_ERR_LAUNCH: return "the HIP runtime rejected the kernel launch";
        default: return "unknown error code";
    }
}

int fa_version(void) { return 100; }

int fa_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
