/*
 * Host-side half of the CPU-GPU cooperative strategy (FastAttention section 4.4, appendix C):
 * the closed-form layer split and the decoding-step attention on the CPU.  C ABI of
 * include/fa_cpu.h.  Built with gcc into libfa_cpu.so; no HIP, no dependence on the GPU library.
 *
 * fa_cpu_decode: the keys of every (batch, head) are cut into runs; OpenMP threads take runs
 * independently, each keeping a running maximum, a running sum and an unnormalised fp32
 * accumulator over blocks of 16 keys (the same online softmax as the GPU kernel's tiles), and a
 * second pass merges the runs of a head.  The inner loops exist twice: AVX-512 (16 fp32 lanes,
 * hardware fp16 conversion, a short polynomial for exp) chosen at run time when the CPU has
 * it, and plain C.
 */
#include <stdatomic.h>
#include <immintrin.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#include "../../include/fa_cpu.h"

#define KEYS_PER_BLOCK 16
#define MAX_D 256

/* ------------------------------------------------------------------ layer split (section 4.4) */

int fa_coop_plan_bytes(double m_gpu, double m_w, double m_mid, double m_vocab, double m_kv, int n, int L,
                       int *l_gpu, int *l_cpu) {
    if (!l_gpu || !l_cpu) return FA_CPU_ERR_NULL;
    if (n <= 0 || L <= 0) return FA_CPU_ERR_SHAPE;
    if (!(m_kv > 0.0) || !(m_gpu >= 0.0) || !(m_w >= 0.0) || !(m_mid >= 0.0) || !(m_vocab >= 0.0)) return FA_CPU_ERR_SHAPE;
    const double room = m_gpu - m_w / n - m_mid - m_vocab;   /* what the KV cache may use on one GPU */
    double layers = floor(room / m_kv);
    if (!(layers > 0.0)) layers = 0.0;                       /* also catches NaN */
    if (layers > L) layers = L;
    *l_gpu = (int)layers;
    *l_cpu = L - *l_gpu;
    return FA_CPU_OK;
}

int fa_coop_plan_fp16(double m_gpu, int n, int L, long long H1, long long H2, long long V, long long B,
                      long long S, long long O, int *l_gpu, int *l_cpu) {
    if (!l_gpu || !l_cpu) return FA_CPU_ERR_NULL;
    if (n <= 0 || L <= 0 || H1 <= 0 || H2 <= 0 || V < 0 || B <= 0 || S <= 0 || O < 0) return FA_CPU_ERR_SHAPE;
    if (!(m_gpu >= 0.0)) return FA_CPU_ERR_SHAPE;
    /* the appendix's last line, numerator and denominator both multiplied by n */
    const double h1 = (double)H1, h2 = (double)H2;
    const double num = n * m_gpu - L * (8.0 * h1 * h1 + 4.0 * h1 * h2) - 6.0 * B * S * h1 - (double)n * V * h1;
    const double den = 4.0 * B * h1 * (double)(S + O);
    double layers = floor(num / den);
    if (!(layers > 0.0)) layers = 0.0;
    if (layers > L) layers = L;
    *l_gpu = (int)layers;
    *l_cpu = L - *l_gpu;
    return FA_CPU_OK;
}

/* ------------------------------------------------------------------ 16-bit formats, scalar */

static float half_bits_to_float(uint16_t h) {
    const uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu, f = h & 0x3ffu, u;
    if (e == 0) {
        if (f == 0) {
            u = sign;
        } else {                                  /* subnormal: renormalise */
            int shift = 0;
            while (!(f & 0x400u)) { f <<= 1; ++shift; }
            u = sign | ((uint32_t)(113 - shift) << 23) | ((f & 0x3ffu) << 13);
        }
    } else if (e == 31) {
        u = sign | 0x7f800000u | (f << 13);
    } else {
        u = sign | ((e + 112) << 23) | (f << 13);
    }
    float x;
    memcpy(&x, &u, 4);
    return x;
}

static float bits_to_float(uint16_t b, int dtype) {
    if (dtype == 0) return half_bits_to_float(b);
    const uint32_t u = (uint32_t)b << 16;
    float x;
    memcpy(&x, &u, 4);
    return x;
}

/* round to nearest even */
static uint16_t float_to_bits(float x, int dtype) {
    uint32_t u;
    memcpy(&u, &x, 4);
    if (dtype == 1) {
        if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x40u);   /* NaN stays NaN */
        return (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
    }
    const uint32_t sign = (u >> 16) & 0x8000u;
    const uint32_t a = u & 0x7fffffffu;
    if (a >= 0x7f800000u) return (uint16_t)(sign | 0x7c00u | (a > 0x7f800000u ? 0x200u : 0));
    if (a >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);                          /* rounds to infinity */
    if (a < 0x33000001u) return (uint16_t)sign;                                       /* below half the smallest subnormal */
    int e = (int)(a >> 23) - 127;
    uint32_t m = (a & 0x7fffffu) | 0x800000u;                                         /* 24-bit significand */
    int shift = e >= -14 ? 13 : 13 + (-14 - e);                                       /* bits to drop */
    uint32_t kept = m >> shift, rem = m & ((1u << shift) - 1), half = 1u << (shift - 1);
    if (rem > half || (rem == half && (kept & 1u))) ++kept;
    if (e >= -14) return (uint16_t)(sign | (uint16_t)((((uint32_t)(e + 15) << 10) + (kept - 0x400u))));
    return (uint16_t)(sign | kept);                                                   /* subnormal (or the smallest normal) */
}

/* ------------------------------------------------------------------ one run of keys, plain C */

static void run_scalar(const float *qf, const uint16_t *k, const uint16_t *v, int n, int D, float scale, int dtype,
                       float *m_out, float *l_out, float *acc) {
    float m = -INFINITY, l = 0.f;
    for (int d = 0; d < D; ++d) acc[d] = 0.f;
    for (int j0 = 0; j0 < n; j0 += KEYS_PER_BLOCK) {
        const int nb = n - j0 < KEYS_PER_BLOCK ? n - j0 : KEYS_PER_BLOCK;
        float s[KEYS_PER_BLOCK];
        float bmax = -INFINITY;
        for (int jj = 0; jj < nb; ++jj) {
            const uint16_t *kr = k + (size_t)(j0 + jj) * D;
            float dot = 0.f;
            for (int d = 0; d < D; ++d) dot += qf[d] * bits_to_float(kr[d], dtype);
            s[jj] = scale * dot;
            if (s[jj] > bmax) bmax = s[jj];
        }
        const float m_new = bmax > m ? bmax : m;
        const float alpha = expf(m - m_new);       /* 0 for the first block */
        l *= alpha;
        for (int d = 0; d < D; ++d) acc[d] *= alpha;
        for (int jj = 0; jj < nb; ++jj) {
            const float p = expf(s[jj] - m_new);
            const uint16_t *vr = v + (size_t)(j0 + jj) * D;
            l += p;
            for (int d = 0; d < D; ++d) acc[d] += p * bits_to_float(vr[d], dtype);
        }
        m = m_new;
    }
    *m_out = m;
    *l_out = l;
}

/* ------------------------------------------------------------------ one run of keys, AVX-512 */

#define AVX512 __attribute__((target("avx512f,avx512bw,avx512dq,avx512vl")))

/* Rows this far ahead are asked for while a row is worked on: K and V are two sequential streams that the
   loop visits in alternating blocks, which the hardware prefetchers alone follow at about two thirds of what
   the cores can draw (a prefetch never faults, so running past the end of a run or of the buffer is harmless). */
#define PREFETCH_KEYS 64

AVX512 static inline __m512 load16_as_float(const uint16_t *p, int dtype) {
    const __m256i h = _mm256_loadu_si256((const __m256i *)p);
    if (dtype == 0) return _mm512_cvtph_ps(h);
    return _mm512_castsi512_ps(_mm512_slli_epi32(_mm512_cvtepu16_epi32(h), 16));
}

/* e^x for x <= 0 (clamped at -87): x = n ln2 + f with n = round(x / ln2), |f| <= 0.347,
   e^f by its Taylor polynomial of degree 6 (error below 1.3e-7 relative), then scaled by 2^n */
AVX512 static inline __m512 exp16(__m512 x) {
    x = _mm512_max_ps(x, _mm512_set1_ps(-87.0f));
    const __m512 n = _mm512_roundscale_ps(_mm512_mul_ps(x, _mm512_set1_ps(1.44269504088896341f)),
                                          _MM_FROUND_TO_NEAREST_INT | _MM_FROUND_NO_EXC);
    __m512 f = _mm512_fnmadd_ps(n, _mm512_set1_ps(0.693145751953125f), x);          /* ln2, high part */
    f = _mm512_fnmadd_ps(n, _mm512_set1_ps(1.42860682030941723212e-6f), f);          /* ln2, low part */
    __m512 p = _mm512_set1_ps(1.0f / 720.0f);
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(1.0f / 120.0f));
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(1.0f / 24.0f));
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(1.0f / 6.0f));
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(0.5f));
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(1.0f));
    p = _mm512_fmadd_ps(p, f, _mm512_set1_ps(1.0f));
    return _mm512_scalef_ps(p, n);
}

AVX512 static void run_avx512(const float *qf, const uint16_t *k, const uint16_t *v, int n, int D, float scale,
                              int dtype, float *m_out, float *l_out, float *acc_out) {
    const int NV = D / 16;                        /* vectors per row, at most 16 */
    __m512 qv[MAX_D / 16], acc[MAX_D / 16];
    for (int c = 0; c < NV; ++c) {
        qv[c] = _mm512_loadu_ps(qf + 16 * c);
        acc[c] = _mm512_setzero_ps();
    }
    float m = -INFINITY, l = 0.f;
    for (int j0 = 0; j0 < n; j0 += KEYS_PER_BLOCK) {
        const int nb = n - j0 < KEYS_PER_BLOCK ? n - j0 : KEYS_PER_BLOCK;
        float s[KEYS_PER_BLOCK] __attribute__((aligned(64)));
        for (int jj = 0; jj < KEYS_PER_BLOCK; ++jj) s[jj] = -INFINITY;    /* absent keys of a ragged block: weight 0 */
        for (int jj = 0; jj < nb; ++jj) {
            const uint16_t *kr = k + (size_t)(j0 + jj) * D;
            for (int b = 0; b < 2 * D; b += 64) _mm_prefetch((const char *)(kr + PREFETCH_KEYS * D) + b, _MM_HINT_T0);
            __m512 d0 = _mm512_setzero_ps(), d1 = _mm512_setzero_ps();
            int c = 0;
            for (; c + 1 < NV; c += 2) {
                d0 = _mm512_fmadd_ps(qv[c], load16_as_float(kr + 16 * c, dtype), d0);
                d1 = _mm512_fmadd_ps(qv[c + 1], load16_as_float(kr + 16 * c + 16, dtype), d1);
            }
            if (c < NV) d0 = _mm512_fmadd_ps(qv[c], load16_as_float(kr + 16 * c, dtype), d0);
            s[jj] = scale * _mm512_reduce_add_ps(_mm512_add_ps(d0, d1));
        }
        const __m512 sv = _mm512_load_ps(s);
        const float bmax = _mm512_reduce_max_ps(sv);
        const float m_new = bmax > m ? bmax : m;
        const float alpha = expf(m - m_new);
        float p[KEYS_PER_BLOCK] __attribute__((aligned(64)));
        const __m512 pv = _mm512_mask_blend_ps(_mm512_cmp_ps_mask(sv, _mm512_set1_ps(-INFINITY), _CMP_EQ_OQ),
                                               exp16(_mm512_sub_ps(sv, _mm512_set1_ps(m_new))), _mm512_setzero_ps());
        _mm512_store_ps(p, pv);
        l = l * alpha + _mm512_reduce_add_ps(pv);
        if (alpha != 1.0f) {
            const __m512 av = _mm512_set1_ps(alpha);
            for (int c = 0; c < NV; ++c) acc[c] = _mm512_mul_ps(acc[c], av);
        }
        for (int jj = 0; jj < nb; ++jj) {
            const uint16_t *vr = v + (size_t)(j0 + jj) * D;
            for (int b = 0; b < 2 * D; b += 64) _mm_prefetch((const char *)(vr + PREFETCH_KEYS * D) + b, _MM_HINT_T0);
            const __m512 pj = _mm512_set1_ps(p[jj]);
            for (int c = 0; c < NV; ++c) acc[c] = _mm512_fmadd_ps(pj, load16_as_float(vr + 16 * c, dtype), acc[c]);
        }
        m = m_new;
    }
    for (int c = 0; c < NV; ++c) _mm512_storeu_ps(acc_out + 16 * c, acc[c]);
    *m_out = m;
    *l_out = l;
}

static atomic_int g_scalar_only;                          /* for tests: run the plain C loops */

int fa_cpu_set_scalar(int on) {
    return atomic_exchange(&g_scalar_only, on != 0);
}

int fa_cpu_has_avx512(void) {
    if (atomic_load(&g_scalar_only)) return 0;
    __builtin_cpu_init();
    return __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
           __builtin_cpu_supports("avx512dq") && __builtin_cpu_supports("avx512vl");
}

/* ------------------------------------------------------------------ decoding-step attention */

int fa_cpu_decode(const void *q, const void *k, const void *v, void *o, float *lse, int B, int H, int Nk, int D,
                  float scale, int dtype, int nthreads) {
    if (!q || !k || !v || !o || !lse) return FA_CPU_ERR_NULL;
    if (B <= 0 || H <= 0 || Nk <= 0) return FA_CPU_ERR_SHAPE;
    if (D <= 0 || D % 16 != 0 || D > MAX_D) return FA_CPU_ERR_HEADDIM;
    if (dtype != 0 && dtype != 1) return FA_CPU_ERR_DTYPE;
    if (!isfinite(scale)) return FA_CPU_ERR_SCALE;
    const uint16_t *qb = (const uint16_t *)q, *kb = (const uint16_t *)k, *vb = (const uint16_t *)v;
    uint16_t *ob = (uint16_t *)o;
#ifdef _OPENMP
    const int threads = nthreads > 0 ? nthreads : omp_get_max_threads();
#else
    const int threads = 1;
    (void)nthreads;
#endif
    /* runs of keys: about eight per thread over the whole problem, 256 .. 8192 keys, whole blocks */
    const long long heads = (long long)B * H;
    long long run = (heads * Nk + 8LL * threads - 1) / (8LL * threads);
    if (run < 256) run = 256;
    if (run > 8192) run = 8192;
    run = (run + KEYS_PER_BLOCK - 1) / KEYS_PER_BLOCK * KEYS_PER_BLOCK;
    const long long nruns = (Nk + run - 1) / run;
    const long long tasks = heads * nruns;
    float *part = (float *)malloc(sizeof(float) * (size_t)tasks * (size_t)(D + 2));
    if (!part) return FA_CPU_ERR_NOMEM;
    const int avx = fa_cpu_has_avx512();

#pragma omp parallel for schedule(dynamic, 1) num_threads(threads)
    for (long long t = 0; t < tasks; ++t) {
        const long long bh = t / nruns, r = t % nruns;
        const long long j0 = r * run;
        const int n = (int)(Nk - j0 < run ? Nk - j0 : run);
        float qf[MAX_D];
        for (int d = 0; d < D; ++d) qf[d] = bits_to_float(qb[bh * D + d], dtype);
        float *pt = part + (size_t)t * (D + 2);
        const uint16_t *kr = kb + ((size_t)bh * Nk + j0) * D, *vr = vb + ((size_t)bh * Nk + j0) * D;
        if (avx) run_avx512(qf, kr, vr, n, D, scale, dtype, pt + D, pt + D + 1, pt);
        else run_scalar(qf, kr, vr, n, D, scale, dtype, pt + D, pt + D + 1, pt);
    }

    /* merge the runs of each head: M = max m_r, L = sum l_r e^(m_r - M), o = sum acc_r e^(m_r - M) / L */
#pragma omp parallel for schedule(static) num_threads(threads)
    for (long long bh = 0; bh < heads; ++bh) {
        const float *p0 = part + (size_t)bh * nruns * (D + 2);
        float M = -INFINITY;
        for (long long r = 0; r < nruns; ++r) {
            const float mr = p0[(size_t)r * (D + 2) + D];
            if (mr > M) M = mr;
        }
        float L = 0.f, acc[MAX_D];
        for (int d = 0; d < D; ++d) acc[d] = 0.f;
        for (long long r = 0; r < nruns; ++r) {
            const float *pr = p0 + (size_t)r * (D + 2);
            const float w = expf(pr[D] - M);
            L += pr[D + 1] * w;
            for (int d = 0; d < D; ++d) acc[d] += pr[d] * w;
        }
        const float inv = 1.0f / L;
        for (int d = 0; d < D; ++d) ob[bh * D + d] = float_to_bits(acc[d] * inv, dtype);
        lse[bh] = M + logf(L);
    }
    free(part);
    return FA_CPU_OK;
}
