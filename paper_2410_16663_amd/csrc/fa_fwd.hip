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

// 16 bytes per lane from global memory straight into LDS: lane i's data lands at
// lds_addr + 16*i.  Issued as inline asm so that the compiler does not put a vmcnt(0) wait
// in front of every later LDS read (it cannot tell the buffers apart); the kernel waits
// for vmcnt(0) itself before the barrier that publishes the tile.
__device__ __forceinline__ void dma16_to_lds(const void *gbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase)
                 : "memory", "m0");
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

    // ---- K/V tiles go from global memory straight into LDS (global_load_lds, 16 bytes per
    // lane, no staging registers).  One such instruction fills 1 KiB of LDS contiguously in
    // lane order, so the bank swizzle is applied on the global side: the lane that owns LDS
    // slot (row r, chunk c') fetches the global chunk that the swizzle maps there.
    constexpr int NI = TILEB / 1024 / NW;         // load instructions per wave per tile
    static_assert(TILEB % (1024 * NW) == 0, "tile must split evenly over the waves");
    int k_src[NI], v_src[NI], ld_row[NI];         // per-lane source byte offsets inside a tile row block
#pragma unroll
    for (int n = 0; n < NI; ++n) {
        const int slot = (wave * NI + n) * 1024 + lane * 16;   // LDS byte this lane fills
        const int r = slot / ROWB, cs = (slot % ROWB) >> 4;
        int ck, cv;
        if constexpr (D == 128) {
            ck = cs ^ (r & 15);
            cv = cs ^ ((r & 3) << 2);
        } else {
            ck = cs ^ ((r >> 1) & 7);
            cv = cs ^ (((r >> 1) & 1) << 2);
        }
        ld_row[n] = r;
        k_src[n] = ck * 16;
        v_src[n] = cv * 16;
    }
    const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)LDS_PTR(unsigned char, smem));
    const unsigned char *kgb = (const unsigned char *)kg;
    const unsigned char *vgb = (const unsigned char *)vg;
    auto load_k = [&](int t, int buf) {
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int key = min(t * BN + ld_row[n], Nk - 1);   // rows past the end re-read the last key; they are masked
            dma16_to_lds(kgb, (unsigned)(key * ROWB + k_src[n]), lds_base + buf * TILEB + (wave * NI + n) * 1024);
        }
    };
    auto load_v = [&](int t, int buf) {
#pragma unroll
        for (int n = 0; n < NI; ++n) {
            const int key = min(t * BN + ld_row[n], Nk - 1);
            dma16_to_lds(vgb, (unsigned)(key * ROWB + v_src[n]), lds_base + (2 + buf) * TILEB + (wave * NI + n) * 1024);
        }
    };

    // S^T = K Q^T for one 64-key tile held in K buffer `buf`
    auto qk_tile = [&](int buf, f32x16 (&s)[2]) {
        const unsigned char *ks = smem + buf * TILEB;
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
            s[mb] = (f32x16)(0.f);
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                const s16x8 a = *(const s16x8 *)(ks + k_lds_off<D>(mb * 32 + l32, 2 * kb + h));
                s[mb] = mfma32<DT>(a, qf[kb], s[mb]);
            }
        }
    };

    f32x16 oacc[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) oacc[db] = (f32x16)(0.f);
    // Softmax state, in log2 units (logit * c).  m_ref is the reference actually subtracted
    // before exponentiation; it follows the running maximum lazily (only when the maximum
    // has moved by more than RESCALE_TAU), which keeps exp2 arguments <= RESCALE_TAU and
    // spares the rescale of the accumulator on most tiles.  Any reference gives the same
    // quotient O = acc / l.
    constexpr float RESCALE_TAU = 8.f;
    float m_ref = -1e30f;
    float l_run = 0.f;         // this half-wave's share of the row sum, relative to m_ref

    // per-lane pieces of the LDS read addresses
    const int g2 = (lane >> 4) & 1, li = lane & 15, vi = li >> 2, vc = li & 3;

    // ---- pipeline: K runs one tile ahead of V.  Entering iteration t, tile t's logits are
    // in registers, K(t+1) and V(t) are in LDS.  The iteration issues the loads of K(t+2) and
    // V(t+1), starts the matrix products of tile t+1's logits and, while they run, does the
    // softmax of tile t on the vector unit; then O += V(t)^T P(t)^T.
    f32x16 s_cur[2], s_nxt[2];
    const bool wave_on = wave_has_rows;
    if (nt > 0) {
        load_k(0, 0);
        load_v(0, 0);
        if (nt > 1) load_k(1, 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        if (wave_on && 0 <= kmax_wave) qk_tile(0, s_cur);
    }

    for (int t = 0; t < nt; ++t) {
        const int k0 = t * BN;
        if (t + 2 < nt) load_k(t + 2, t & 1);
        if (t + 1 < nt) load_v(t + 1, (t + 1) & 1);

        const bool act = wave_on && k0 <= kmax_wave;
        const bool act_next = wave_on && (t + 1 < nt) && (k0 + BN <= kmax_wave);
        if (act_next) qk_tile((t + 1) & 1, s_nxt);

        if (act) {
            const unsigned char *vs = smem + (2 + (t & 1)) * TILEB;

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
                        if (key > lim) s_cur[mb][r] = -INFINITY;
                    }
            }

            // ---- online softmax; the lane's 32 logits all belong to one query
            float mx = s_cur[0][0];
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s_cur[mb][r]);
            mx = xhalf_max(mx) * p.c;
            const bool grow = mx > m_ref + RESCALE_TAU;
            if (__builtin_amdgcn_ballot_w64(grow) != 0) {
                const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - mx) : 1.f;
                m_ref = grow ? mx : m_ref;
                l_run *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db) oacc[db] *= alpha;
            }
            float rs = 0.f;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float e = __builtin_amdgcn_exp2f(__builtin_fmaf(s_cur[mb][r], p.c, -m_ref));
                    s_cur[mb][r] = e;
                    rs += e;
                }
            l_run += rs;

            // ---- P^T fragments: 16-key step j takes logits registers 8*(j%2)..+7 of block j/2,
            // i.e. k-slot (h, v) of step j is key 16*j + 8*(v/4) + 4*h + v%4
            s16x8 pf[4];
#pragma unroll
            for (int j = 0; j < 4; ++j) {
#pragma unroll
                for (int v2 = 0; v2 < 4; ++v2) {
                    const s16x2 pr = pack2<DT>(s_cur[j >> 1][8 * (j & 1) + 2 * v2], s_cur[j >> 1][8 * (j & 1) + 2 * v2 + 1]);
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
        s_cur[0] = s_nxt[0];
        s_cur[1] = s_nxt[1];

        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of K(t+2), V(t+1) has landed
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
            p.lse[(size_t)bh * Nq + qrow] = l_tot > 0.f ? (m_ref + __log2f(l_tot)) * 0.6931471805599453f : -INFINITY;
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
