/*
 * Driver for the sanitizer build of the host-side C code (the oracle, libfa_cpu's and libfa_bench_cpu's sources): runs small
 * cases of every exported function under AddressSanitizer and UndefinedBehaviorSanitizer.  Exit code 0 = clean.
 * Built and run by tests/test_sanitizers.py; not part of any library.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int fa_oracle_fwd(const uint16_t *, const uint16_t *, const uint16_t *, double *, double *, int, int, int, int, int,
                  double, int, int, const int64_t *, int64_t, int);
int fa_oracle_probs(const uint16_t *, const uint16_t *, double *, int, int, int, int, int, double, int, int, int64_t);
int fa_oracle_fwd_masked(const uint16_t *, const uint16_t *, const uint16_t *, double *, double *, int, int, int, int,
                         int, double, int64_t, int64_t, int64_t, const int32_t *, int, int, const int64_t *, int64_t, int);
int fa_oracle_attn_linear(const uint16_t *, const uint16_t *, const uint16_t *, const uint16_t *, double *, int, int,
                          int, int, int, int, double, int, int, const int64_t *, int64_t, int);
int fa_coop_plan_bytes(double, double, double, double, double, int, int, int *, int *);
int fa_coop_plan_fp16(double, int, int, long long, long long, long long, long long, long long, long long, int *, int *);
int fa_cpu_decode(const void *, const void *, const void *, void *, float *, int, int, int, int, float, int, int);
int fa_cpu_stream_read(const void *, long long, int, int, int, double *, unsigned long long *);

static uint32_t rng_state = 12345u;
static uint16_t rand_half(void) {               /* a finite fp16 / bf16 pattern of moderate size */
    rng_state = rng_state * 1664525u + 1013904223u;
    uint16_t mant = (uint16_t)(rng_state >> 20) & 0x3ff;
    uint16_t sign = (uint16_t)((rng_state >> 5) & 1) << 15;
    return (uint16_t)(sign | 0x3800u | mant);   /* fp16: 0.5..1; bf16: tiny but finite */
}
static uint16_t *rand_buf(size_t n) {
    uint16_t *p = (uint16_t *)malloc(n * sizeof(uint16_t));
    for (size_t i = 0; i < n; ++i) p[i] = rand_half();
    return p;
}
#define CHECK(x) do { int rc_ = (x); if (rc_ != 0) { fprintf(stderr, "%s -> %d\n", #x, rc_); return 1; } } while (0)

int main(int argc, char **argv) {
    const int scalar_only = argc > 1 && argv[1][0] == '1';   /* "1": the plain C loops, else what the CPU has */
    fa_cpu_set_scalar(scalar_only);
    for (int dtype = 0; dtype < 2; ++dtype)
        for (int causal = 0; causal < 2; ++causal) {
            const int B = 2, H = 3, Nq = 37, Nk = 53, D = 16, N = 5;
            uint16_t *q = rand_buf((size_t)B * H * Nq * D), *k = rand_buf((size_t)B * H * Nk * D),
                     *v = rand_buf((size_t)B * H * Nk * D), *w = rand_buf((size_t)H * D * N);
            double *o = (double *)malloc(sizeof(double) * B * H * Nq * D), *lse = (double *)malloc(sizeof(double) * B * H * Nq);
            double *p = (double *)malloc(sizeof(double) * Nk), *y = (double *)malloc(sizeof(double) * B * Nq * N);
            CHECK(fa_oracle_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, 0.25, causal, dtype, NULL, 0, 2));
            const int64_t rows[3] = {0, 110, (int64_t)B * H * Nq - 1};
            CHECK(fa_oracle_fwd(q, k, v, o, lse, B, H, Nq, Nk, D, 0.25, causal, dtype, rows, 3, 1));
            CHECK(fa_oracle_probs(q, k, p, B, H, Nq, Nk, D, 0.25, causal, dtype, 17));
            const int32_t lens[2] = {53, 7};
            CHECK(fa_oracle_fwd_masked(q, k, v, o, lse, B, H, Nq, Nk, D, 0.25, 9, causal ? 0 : 4, 3, lens, causal, dtype, NULL, 0, 2));
            CHECK(fa_oracle_fwd_masked(q, k, v, o, lse, B, H, Nq, Nk, D, 0.25, -1, -1, 0, NULL, 0, dtype, rows, 3, 2));
            CHECK(fa_oracle_attn_linear(q, k, v, w, y, B, H, Nq, Nk, D, N, 0.25, causal, dtype, NULL, 0, 2));
            /* Nq > Nk causal: rows without keys */
            CHECK(fa_oracle_fwd(q, k, v, o, lse, B, H, Nq, 20, D, 0.25, 1, dtype, NULL, 0, 2));
            /* host decoding attention: one query per head, several runs of keys, the code path chosen by the first argument */
            uint16_t *q1 = rand_buf((size_t)B * H * 64), *k1 = rand_buf((size_t)B * H * 1000 * 64), *v1 = rand_buf((size_t)B * H * 1000 * 64);
            uint16_t *o1 = (uint16_t *)malloc(sizeof(uint16_t) * B * H * 64);
            float *l1 = (float *)malloc(sizeof(float) * B * H);
            CHECK(fa_cpu_decode(q1, k1, v1, o1, l1, B, H, 1000, 64, 0.125f, dtype, 3));
            CHECK(fa_cpu_decode(q1, k1, v1, o1, l1, B, H, 1, 64, 0.125f, dtype, 1));
            for (int i = 0; i < B * H; ++i)
                if (!isfinite(l1[i])) { fprintf(stderr, "non-finite lse from fa_cpu_decode\n"); return 1; }
            /* the streaming-read yardstick over a buffer that does not end on a 64-byte line */
            double gbs;
            unsigned long long chk;
            CHECK(fa_cpu_stream_read(k1, (long long)sizeof(uint16_t) * B * H * 1000 * 64 - 6, 5, 2, scalar_only, &gbs, &chk));
            free(q); free(k); free(v); free(w); free(o); free(lse); free(p); free(y);
            free(q1); free(k1); free(v1); free(o1); free(l1);
        }
    int a, b;
    CHECK(fa_coop_plan_bytes(100, 80, 10, 5, 7, 4, 12, &a, &b));
    CHECK(fa_coop_plan_fp16(16e9, 8, 40, 5120, 20480, 40000, 1, 262144, 50, &a, &b));
    if (fa_coop_plan_bytes(100, 80, 10, 5, 0, 4, 12, &a, &b) == 0) return 1;   /* must be refused */
    printf("sanitizer driver: clean\n");
    return 0;
}
