/*
 * CPU oracle for exact attention forward -- TEST INFRASTRUCTURE, not a product path.
 *
 * Computes, for every (batch b, head h, query row i), the plain definition of
 * attention that the tiled method must reproduce (FastAttention section 5.1,
 * "standard attention": Softmax(Q K^T / sqrt(d)) V with no fusion and no online
 * softmax; appendix C, prefill equation for X_O; section 4.1: the mask is lower
 * triangular).  Everything is fp64; inputs are fp16/bf16 bit patterns widened
 * exactly.  No blocking, no running maximum, no reordering: one row of logits is
 * materialised, then its maximum, then the weights, then the weighted sum.
 *
 *   J_i   = all keys (non-causal), or { j : j <= i + (Nk - Nq) } (causal,
 *           bottom-right aligned so that a single decode query sees the whole
 *           cache as in appendix C's decoding equations)
 *   s_ij  = scale * sum_d q[i,d] k[j,d]                       j in J_i
 *   m_i   = max_j s_ij ;  w_ij = exp(s_ij - m_i) ;  l_i = sum_j w_ij
 *   o_i   = (sum_j w_ij v_j) / l_i ;  lse_i = m_i + ln(l_i)
 *   rows with empty J_i:  o_i = 0, lse_i = -inf
 *
 * Layout: q [B,H,Nq,D], k,v [B,H,Nk,D], contiguous, D fastest, host pointers,
 * uint16 bit patterns (dtype 0 = IEEE fp16, 1 = bfloat16).
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call this.
 * It shares no code with the GPU library.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double half_to_double(uint16_t h) {
    int sign = (h >> 15) & 1;
    int e = (h >> 10) & 0x1f;
    int f = h & 0x3ff;
    double x;
    if (e == 0) {
        x = ldexp((double)f, -24);             /* zero and subnormals: f * 2^-24 */
    } else if (e == 31) {
        x = f ? NAN : INFINITY;
    } else {
        x = ldexp(1.0 + (double)f / 1024.0, e - 15);
    }
    return sign ? -x : x;
}

static double bf16_to_double(uint16_t h) {
    uint32_t u = (uint32_t)h << 16;            /* bfloat16 is the top half of a binary32 */
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * Decoding is done once per bit pattern: table[dtype][bits] holds the exact value of
 * every 16-bit pattern, filled from the two decoders above on first use.
 */
static double widen_table[2][65536];
static int widen_ready = 0;

static void widen_init(void) {
#pragma omp critical(fa_oracle_widen)
    {
        if (!widen_ready) {
            for (int b = 0; b < 65536; ++b) {
                widen_table[0][b] = half_to_double((uint16_t)b);
                widen_table[1][b] = bf16_to_double((uint16_t)b);
            }
            widen_ready = 1;
        }
    }
}

static double widen(uint16_t bits, int dtype) { return widen_table[dtype][bits]; }

/* number of keys row i may attend to (keys 0 .. count-1) */
static int64_t visible_count(int64_t i, int Nq, int Nk, int causal) {
    if (!causal) return Nk;
    int64_t c = i + ((int64_t)Nk - (int64_t)Nq) + 1;
    if (c < 0) c = 0;
    if (c > Nk) c = Nk;
    return c;
}

/*
 * Steps 1-3 for one row: logits s[0..n), their maximum, the unnormalised
 * weights w[j] = exp(s[j] - m) written over s, and l = sum w.  Returns n.
 */
static int64_t row_weights(const uint16_t *q_row, const uint16_t *k_head, int64_t n, int D,
                           double scale, int dtype, double *s, double *m_out, double *l_out) {
    double m = -INFINITY;
    for (int64_t j = 0; j < n; ++j) {
        const uint16_t *k_row = k_head + j * D;
        double dot = 0.0;
        for (int d = 0; d < D; ++d) dot += widen(q_row[d], dtype) * widen(k_row[d], dtype);
        s[j] = scale * dot;
        if (s[j] > m) m = s[j];
    }
    double l = 0.0;
    for (int64_t j = 0; j < n; ++j) {
        s[j] = exp(s[j] - m);
        l += s[j];
    }
    *m_out = m;
    *l_out = l;
    return n;
}

static int bad_args(const void *q, const void *k, const void *v, int B, int H, int Nq, int Nk, int D,
                    int dtype) {
    if (!q || !k || !v) return -1;
    if (B <= 0 || H <= 0 || Nq <= 0 || Nk <= 0 || D <= 0) return -2;
    if (dtype != 0 && dtype != 1) return -4;
    return 0;
}

/*
 * Full forward.  rows == NULL: every row, o is [B,H,Nq,D], lse is [B,H,Nq].
 * rows != NULL: only the nrows flat row ids (b*H + h)*Nq + i listed; o is
 * [nrows,D], lse is [nrows], in the order listed.
 * nthreads <= 0: OpenMP default.  Returns 0, or <0 on bad arguments.
 */
int fa_oracle_fwd(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *o, double *lse,
                  int B, int H, int Nq, int Nk, int D, double scale, int causal, int dtype,
                  const int64_t *rows, int64_t nrows, int nthreads) {
    int err = bad_args(q, k, v, B, H, Nq, Nk, D, dtype);
    if (err) return err;
    if (!o || !lse) return -1;
    int64_t total = rows ? nrows : (int64_t)B * H * Nq;
    widen_init();
    if (rows) {
        for (int64_t r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= (int64_t)B * H * Nq) return -2;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < total; ++r) {
            if (!s) continue;
            int64_t flat = rows ? rows[r] : r;
            int64_t i = flat % Nq;
            int64_t bh = flat / Nq;
            const uint16_t *q_row = q + flat * D;
            const uint16_t *k_head = k + bh * (int64_t)Nk * D;
            const uint16_t *v_head = v + bh * (int64_t)Nk * D;
            double *o_row = o + r * D;
            int64_t n = visible_count(i, Nq, Nk, causal);
            if (n == 0) {
                for (int d = 0; d < D; ++d) o_row[d] = 0.0;
                lse[r] = -INFINITY;
                continue;
            }
            double m, l;
            row_weights(q_row, k_head, n, D, scale, dtype, s, &m, &l);
            /* o_row[d] = (sum over j, in increasing j, of w_ij v[j,d]) / l_i */
            for (int d = 0; d < D; ++d) o_row[d] = 0.0;
            for (int64_t j = 0; j < n; ++j)
                for (int d = 0; d < D; ++d) o_row[d] += s[j] * widen(v_head[j * D + d], dtype);
            for (int d = 0; d < D; ++d) o_row[d] /= l;
            lse[r] = m + log(l);
        }
        free(s);
    }
    return failed ? -8 : 0;
}

/*
 * Normalised attention probabilities of ONE row (flat id as above):
 * p[j] = w_ij / l_i for j in J_i and 0 for masked keys; p has Nk entries.
 * Exposed so that tests can pin the softmax step on its own.
 */
int fa_oracle_probs(const uint16_t *q, const uint16_t *k, double *p, int B, int H, int Nq, int Nk,
                    int D, double scale, int causal, int dtype, int64_t row) {
    int err = bad_args(q, k, k, B, H, Nq, Nk, D, dtype);
    if (err) return err;
    if (!p) return -1;
    if (row < 0 || row >= (int64_t)B * H * Nq) return -2;
    int64_t i = row % Nq, bh = row / Nq;
    int64_t n = visible_count(i, Nq, Nk, causal);
    for (int64_t j = 0; j < Nk; ++j) p[j] = 0.0;
    if (n == 0) return 0;
    widen_init();
    double m, l;
    row_weights(q + row * D, k + bh * (int64_t)Nk * D, n, D, scale, dtype, p, &m, &l);
    for (int64_t j = 0; j < n; ++j) p[j] /= l;
    return 0;
}

/*
 * Masks generated from a compact descriptor instead of a stored matrix (the idea of section
 * 4.1's mask generator, taken beyond the lower-triangular case): query row i of batch entry b
 * attends to key j exactly when
 *     j < klen_b                              (klen_b = kv_len[b], or Nk if kv_len is NULL:
 *                                              keys at and after klen_b are padding)
 *     and ( j < prefix                        (a prefix every row sees, prefix-LM)
 *           or  diag_i - left <= j <= diag_i + right )   with diag_i = i + (Nk - Nq),
 *                                              a negative left / right meaning "no limit"
 * diag_from_kv_len != 0 puts the diagonal of batch entry b at its own last key instead of the last
 * of the Nk: diag_i = i + (klen_b - Nq), i.e. the Nq queries are the last Nq positions of a sequence
 * of klen_b tokens (appendix C's decoding step, where the new token's query attends its own
 * sequence's cache, for a batch whose caches have different lengths).
 * left < 0, right = 0, prefix = 0, no kv_len is the causal mask; left < 0, right < 0 is no mask.
 * Same plain row-at-a-time evaluation as fa_oracle_fwd, written out on its own: the logits of
 * the visible keys, their maximum, the weights, the weighted sum.
 */
static int key_is_visible(int64_t i, int64_t j, int Nq, int Nk, int64_t left, int64_t right,
                          int64_t prefix, int64_t klen, int diag_from_kv_len) {
    if (j >= klen) return 0;
    if (j < prefix) return 1;
    int64_t diag = i + ((diag_from_kv_len ? klen : (int64_t)Nk) - (int64_t)Nq);
    if (left >= 0 && j < diag - left) return 0;
    if (right >= 0 && j > diag + right) return 0;
    return 1;
}

int fa_oracle_fwd_masked(const uint16_t *q, const uint16_t *k, const uint16_t *v, double *o, double *lse,
                         int B, int H, int Nq, int Nk, int D, double scale, int64_t left, int64_t right,
                         int64_t prefix, const int32_t *kv_len, int diag_from_kv_len, int dtype,
                         const int64_t *rows, int64_t nrows, int nthreads) {
    int err = bad_args(q, k, v, B, H, Nq, Nk, D, dtype);
    if (err) return err;
    if (!o || !lse) return -1;
    if (prefix < 0) return -2;
    int64_t total = rows ? nrows : (int64_t)B * H * Nq;
    widen_init();
    if (rows) {
        for (int64_t r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= (int64_t)B * H * Nq) return -2;
    }
    if (kv_len) {
        for (int b = 0; b < B; ++b)
            if (kv_len[b] < 0 || kv_len[b] > Nk) return -2;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
        if (!s) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 4)
        for (int64_t r = 0; r < total; ++r) {
            if (!s) continue;
            int64_t flat = rows ? rows[r] : r;
            int64_t i = flat % Nq;
            int64_t bh = flat / Nq;
            int64_t klen = kv_len ? kv_len[bh / H] : Nk;
            const uint16_t *q_row = q + flat * D;
            const uint16_t *k_head = k + bh * (int64_t)Nk * D;
            const uint16_t *v_head = v + bh * (int64_t)Nk * D;
            double *o_row = o + r * D;
            /* logits of the visible keys and their maximum */
            double m = -INFINITY;
            int64_t count = 0;
            for (int64_t j = 0; j < Nk; ++j) {
                if (!key_is_visible(i, j, Nq, Nk, left, right, prefix, klen, diag_from_kv_len)) continue;
                double dot = 0.0;
                for (int d = 0; d < D; ++d) dot += widen(q_row[d], dtype) * widen(k_head[j * D + d], dtype);
                s[j] = scale * dot;
                if (s[j] > m) m = s[j];
                ++count;
            }
            for (int d = 0; d < D; ++d) o_row[d] = 0.0;
            if (count == 0) {
                lse[r] = -INFINITY;
                continue;
            }
            /* weights, their sum, the weighted sum of the value rows */
            double l = 0.0;
            for (int64_t j = 0; j < Nk; ++j) {
                if (!key_is_visible(i, j, Nq, Nk, left, right, prefix, klen, diag_from_kv_len)) continue;
                double w = exp(s[j] - m);
                l += w;
                for (int d = 0; d < D; ++d) o_row[d] += w * widen(v_head[j * D + d], dtype);
            }
            for (int d = 0; d < D; ++d) o_row[d] /= l;
            lse[r] = m + log(l);
        }
        free(s);
    }
    return failed ? -8 : 0;
}

/*
 * Attention followed by the output projection (section 4.2: the attention and the Linear that
 * follows it are computed together, block of rows by block of rows; appendix C: X_O contains
 * Softmax(...) X_V W_O).  For token t = (b, i):
 *     a[t, h*D + d] = o[b, h, i, d]            the heads' attention rows side by side
 *     y[t, n]       = sum_c a[t, c] * w[c, n]  c = 0 .. H*D-1,  n = 0 .. N-1
 * with o exactly as fa_oracle_fwd defines it, kept in fp64 (never rounded to 16 bits), and w a
 * [H*D, N] matrix of 16-bit patterns, n fastest.  With the heads of one device this is that
 * device's partial sum of the projection; the sum over devices (the AllReduce) is outside.
 * rows == NULL: every token, y is [B, Nq, N]; else the nrows flat token ids b*Nq + i listed,
 * y is [nrows, N].
 */
int fa_oracle_attn_linear(const uint16_t *q, const uint16_t *k, const uint16_t *v, const uint16_t *w,
                          double *y, int B, int H, int Nq, int Nk, int D, int N, double scale,
                          int causal, int dtype, const int64_t *rows, int64_t nrows, int nthreads) {
    int err = bad_args(q, k, v, B, H, Nq, Nk, D, dtype);
    if (err) return err;
    if (!w || !y) return -1;
    if (N <= 0) return -2;
    int64_t total = rows ? nrows : (int64_t)B * Nq;
    widen_init();
    if (rows) {
        for (int64_t r = 0; r < nrows; ++r)
            if (rows[r] < 0 || rows[r] >= (int64_t)B * Nq) return -2;
    }
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    int failed = 0;
#pragma omp parallel
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)Nk);
        double *a = (double *)malloc(sizeof(double) * (size_t)H * D);
        if (!s || !a) {
#pragma omp atomic write
            failed = 1;
        }
#pragma omp for schedule(dynamic, 1)
        for (int64_t r = 0; r < total; ++r) {
            if (!s || !a) continue;
            int64_t t = rows ? rows[r] : r;
            int64_t b = t / Nq, i = t % Nq;
            int64_t n_vis = visible_count(i, Nq, Nk, causal);
            /* the attention row of every head, side by side */
            for (int h = 0; h < H; ++h) {
                int64_t bh = b * H + h;
                double *a_h = a + (int64_t)h * D;
                for (int d = 0; d < D; ++d) a_h[d] = 0.0;
                if (n_vis == 0) continue;
                const uint16_t *v_head = v + bh * (int64_t)Nk * D;
                double m, l;
                row_weights(q + (bh * Nq + i) * D, k + bh * (int64_t)Nk * D, n_vis, D, scale, dtype, s, &m, &l);
                for (int64_t j = 0; j < n_vis; ++j)
                    for (int d = 0; d < D; ++d) a_h[d] += s[j] * widen(v_head[j * D + d], dtype);
                for (int d = 0; d < D; ++d) a_h[d] /= l;
            }
            /* times the projection matrix */
            double *y_row = y + r * N;
            for (int n = 0; n < N; ++n) y_row[n] = 0.0;
            for (int64_t c = 0; c < (int64_t)H * D; ++c)
                for (int n = 0; n < N; ++n) y_row[n] += a[c] * widen(w[c * N + n], dtype);
        }
        free(s);
        free(a);
    }
    return failed ? -8 : 0;
}

int fa_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
