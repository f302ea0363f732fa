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

#include <type_traits>
#include <utility>

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
// lds_addr + IMM + 16*i (the instruction's immediate offset applies to the global address
// and to the LDS address alike).  Issued as inline asm so that the compiler does not put a vmcnt(0) wait
// in front of every later LDS read (it cannot tell the buffers apart); the kernel waits
// for vmcnt(0) itself before the barrier that publishes the tile.
template <int IMM>
__device__ __forceinline__ void dma16_to_lds(const void *gbase, unsigned voff, unsigned lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2 offset:%3"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(gbase), "n"(IMM)
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
    constexpr int RPI = 1024 / ROWB;              // tile rows covered by one load instruction
    // Instruction n of this wave fills LDS bytes [(wave*NI+n)*1024, +1024) of the tile: rows
    // row0 + n*RPI + (lane*16)/ROWB.  The V swizzle does not depend on n; the K swizzle does.
    const int ld_row0 = wave * NI * RPI + (lane * 16) / ROWB;
    const int ld_cs = ((lane * 16) % ROWB) >> 4;
    int k_voff[NI];                               // per-lane byte offset of the K chunk, relative to the tile
    int v_voff;                                   // same for V, relative to row n*RPI of the tile
#pragma unroll
    for (int n = 0; n < NI; ++n) {
        const int r = ld_row0 + n * RPI;
        const int ck = (D == 128) ? (ld_cs ^ (r & 15)) : (ld_cs ^ ((r >> 1) & 7));
        k_voff[n] = ld_row0 * ROWB + ck * 16;
    }
    {
        const int r = ld_row0;   // (r & 3) and ((r >> 1) & 1) are the same for every n: RPI is 4 or 8
        const int cv = (D == 128) ? (ld_cs ^ ((r & 3) << 2)) : (ld_cs ^ (((r >> 1) & 1) << 2));
        v_voff = ld_row0 * ROWB + cv * 16;
    }
    const unsigned lds_base = __builtin_amdgcn_readfirstlane((unsigned)(uintptr_t)LDS_PTR(unsigned char, smem));
    const unsigned char *kgb = (const unsigned char *)kg;
    const unsigned char *vgb = (const unsigned char *)vg;
    // whole tiles take their per-lane offsets as they are (the tile start goes into the scalar
    // base, the row step n*RPI into the instruction's immediate offset); the ragged last tile
    // clamps its rows to the last key -- those rows are masked, they only have to be readable
    auto load_tile = [&](const unsigned char *gb, int t, int lds_off, auto is_k) {
        constexpr bool IS_K = decltype(is_k)::value;
        if (t * BN + BN <= Nk) {
            const unsigned char *tb = gb + (size_t)t * TILEB;
            [&]<int... Ns>(std::integer_sequence<int, Ns...>) {
                (dma16_to_lds<Ns * 1024>(tb, (unsigned)(IS_K ? k_voff[Ns] : v_voff), lds_base + lds_off + wave * NI * 1024), ...);
            }(std::make_integer_sequence<int, NI>{});
        } else {
#pragma unroll
            for (int n = 0; n < NI; ++n) {
                const int key = min(t * BN + ld_row0 + n * RPI, Nk - 1);
                const int src = (IS_K ? k_voff[n] : v_voff) - ld_row0 * ROWB;
                dma16_to_lds<0>(gb, (unsigned)(key * ROWB + src), lds_base + lds_off + (wave * NI + n) * 1024);
            }
        }
    };
    auto load_k = [&](int t, int buf) { load_tile(kgb, t, buf * TILEB, std::true_type{}); };
    auto load_v = [&](int t, int buf) { load_tile(vgb, t, (2 + buf) * TILEB, std::false_type{}); };

    // ---- operand fragments.  K fragment (mb, kb): rows = keys mb*32 + l32, 8 contiguous d.
    auto k_frag = [&](const unsigned char *ks, int mb, int kb) -> s16x8 {
        return *(const s16x8 *)(ks + k_lds_off<D>(mb * 32 + l32, 2 * kb + h));
    };
    // V^T fragment (j, db): rows = d db*32 + l32, k-slot (h, v) = key 16*j + 8*(v/4) + 4*h + v%4,
    // fetched with two transposing reads of 4 keys x 16 d per 16-lane group.
    const int g2 = (lane >> 4) & 1, li = lane & 15, vi = li >> 2, vc = li & 3;
    auto v_frag = [&](const unsigned char *vs, int j, int db) -> s16x8 {
        const int row = 16 * j + 4 * h + vi;
        const int bcol = db * 64 + g2 * 32 + vc * 8;
        const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row, bcol)));
        const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_PTR(s16x4, vs + v_lds_off<D>(row + 8, bcol)));
        return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
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

    // mask + row maximum of 4 logits registers (unit u of 8) of a tile starting at key k0
    auto max_unit = [&](auto mask_c, f32x16 (&s)[2], int u, int k0, int lim, float &mx) {
        constexpr bool MASK = decltype(mask_c)::value;
        const int mb = u >> 2, r0 = (u & 3) * 4;
        if constexpr (MASK) {
#pragma unroll
            for (int r = r0; r < r0 + 4; ++r) {
                const int key = k0 + mb * 32 + 8 * (r >> 2) + 4 * h + (r & 3);
                if (key > lim) s[mb][r] = -INFINITY;
            }
        }
        mx = fmaxf(fmaxf(mx, s[mb][r0]), s[mb][r0 + 1]);
        mx = fmaxf(fmaxf(mx, s[mb][r0 + 2]), s[mb][r0 + 3]);
    };

    auto tile_masked = [&](int t) -> bool {
        const int k0 = t * BN;
        return (k0 + BN - 1 >= Nk) || (CAUSAL && (k0 + BN - 1 > q_wave + off));
    };

    // ---- one tile of the pipeline, for this wave, as an explicit instruction schedule.
    // Entering: tile t's logits are in `sc` and their scaled row maximum in `mx`; K(t+1) and
    // V(t) are in LDS.  The step is a sequence of NM matrix instructions -- first the 2*KB of
    // tile t+1's logits S^T = K Q^T, then the 4*DB of O^T += V(t)^T P(t)^T -- and every matrix
    // instruction carries, in its shadow, a share of the vector work: first the 16 groups of
    // two exponentials of tile t (each yields one packed pair of P), then mask and row maximum
    // of the new logits.  Operand fragments are read from LDS LA instructions ahead.  The
    // scheduling barriers pin this order; registers and wait counts are left to the compiler.
    // The row maximum of the new logits is taken unmasked; a tile that needs the mask applies
    // it, and recomputes its row maximum, in a short pre-pass of its own step (once per wave
    // in a causal run).  The wave's last tile runs the same schedule: its "next logits" are
    // computed from whatever the K buffer holds and never used.
    constexpr int NQK = 2 * KB, NPV = 4 * DB, NM = NQK + NPV;
    constexpr int E_SPAN = NM * 23 / 32;     // the exponentials ride on the first E_SPAN matrix instructions
    constexpr int LA = 2;   // 3 costs a handful of spills at D = 128
    auto tile_step = [&](auto par_c, int t, f32x16 (&sc)[2], f32x16 (&sn)[2], float &mx) {
        constexpr int PAR = decltype(par_c)::value;
        const unsigned char *ksn = smem + (PAR ^ 1) * TILEB;   // K(t+1)
        const unsigned char *vs = smem + (2 + PAR) * TILEB;     // V(t)

        if (tile_masked(t)) {
            int lim = Nk - 1;
            if (CAUSAL) lim = min(lim, qrow + off);
            float mm = -INFINITY;
#pragma unroll
            for (int u = 0; u < 8; ++u) max_unit(std::true_type{}, sc, u, t * BN, lim, mm);
            mx = xhalf_max(mm) * p.c;
        }

        // rare: move the exponent reference up and rescale what has been accumulated
        const bool grow = mx > m_ref + RESCALE_TAU;
        if (__builtin_amdgcn_ballot_w64(grow) != 0) {
            const float alpha = grow ? __builtin_amdgcn_exp2f(m_ref - mx) : 1.f;
            m_ref = grow ? mx : m_ref;
            l_run *= alpha;
#pragma unroll
            for (int db = 0; db < DB; ++db) oacc[db] *= alpha;
        }
        const float nm = -m_ref;
        float rs0 = 0.f, rs1 = 0.f;
        s16x8 pf[4];
        // exponentials of logits registers (j, v2): two elements -> one packed pair of P^T
        auto exp_group = [&](int g) {
            const int j = g >> 2, v2 = g & 3;
            const float e0 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[j >> 1][8 * (j & 1) + 2 * v2], p.c, nm));
            const float e1 = __builtin_amdgcn_exp2f(__builtin_fmaf(sc[j >> 1][8 * (j & 1) + 2 * v2 + 1], p.c, nm));
            rs0 += e0;
            rs1 += e1;
            const s16x2 pr = pack2<DT>(e0, e1);
            pf[j][2 * v2] = pr[0];
            pf[j][2 * v2 + 1] = pr[1];
        };

        {
            float mxn = -INFINITY;
            s16x8 fr[NM];
            auto read_frag = [&](int i) {
                if (i < NQK) fr[i] = k_frag(ksn, i / KB, i % KB);
                else fr[i] = v_frag(vs, (i - NQK) / DB, (i - NQK) % DB);
            };
#pragma unroll
            for (int i = 0; i < LA; ++i) read_frag(i);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                if (i + LA < NM) read_frag(i + LA);
                if (i < NQK) {
                    const int mb = i / KB, kb = i % KB;
                    if (kb == 0) sn[mb] = (f32x16)(0.f);
                    sn[mb] = mfma32<DT>(fr[i], qf[kb], sn[mb]);
                } else {
                    const int j = (i - NQK) / DB, db = (i - NQK) % DB;
                    oacc[db] = mfma32<DT>(fr[i], pf[j], oacc[db]);
                }
#pragma unroll
                for (int g = 0; g < 16; ++g)
                    if (g * E_SPAN / 16 == i) exp_group(g);
#pragma unroll
                for (int u = 0; u < 8; ++u)
                    if (E_SPAN + u * (NM - 1 - E_SPAN) / 8 == i)
                        max_unit(std::false_type{}, sn, u, 0, 0, mxn);
                __builtin_amdgcn_sched_barrier(0);
            }
            mx = xhalf_max(mxn) * p.c;
        }
        l_run += rs0 + rs1;
    };

    // ---- workgroup pipeline: K runs one tile ahead of V.  Iteration t issues the loads of
    // K(t+2) and V(t+1), runs the wave's tile step, then waits for its loads and meets the
    // other waves at the barrier that publishes them.
    const int n_act = (wave_has_rows && kmax_wave >= 0) ? kmax_wave / BN + 1 : 0;   // tiles this wave works on
    f32x16 s_a[2], s_b[2];
    float mx_run = -INFINITY;
    if (nt > 0) {
        load_k(0, 0);
        load_v(0, 0);
        if (nt > 1) load_k(1, 1);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
        __syncthreads();
        if (n_act > 0) {
            // logits and row maximum of tile 0, not overlapped with anything
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) {
                s_a[mb] = (f32x16)(0.f);
#pragma unroll
                for (int kb = 0; kb < KB; ++kb) s_a[mb] = mfma32<DT>(k_frag(smem, mb, kb), qf[kb], s_a[mb]);
            }
            float m0 = -INFINITY;
#pragma unroll
            for (int u = 0; u < 8; ++u) max_unit(std::false_type{}, s_a, u, 0, 0, m0);
            mx_run = xhalf_max(m0) * p.c;
        }
        // tile 0's K buffer is the first one the loop refills: every wave must be done reading it
        __syncthreads();
    }

    using std::integral_constant;
    auto iteration = [&](auto par_c, int t, f32x16 (&sc)[2], f32x16 (&sn)[2]) {
        constexpr int PAR = decltype(par_c)::value;
        if (t + 2 < nt) load_k(t + 2, PAR);
        if (t + 1 < nt) load_v(t + 1, PAR ^ 1);
        if (t < n_act) tile_step(par_c, t, sc, sn, mx_run);
        __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of K(t+2), V(t+1) has landed
        __syncthreads();
    };
    // iterations come in pairs so that the two logits buffers swap roles without copies; an
    // odd tile count is rounded up (the extra iteration has no tile and only meets the barrier)
    for (int t = 0; t < nt; t += 2) {
        iteration(integral_constant<int, 0>{}, t, s_a, s_b);
        iteration(integral_constant<int, 1>{}, t + 1, s_b, s_a);
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
