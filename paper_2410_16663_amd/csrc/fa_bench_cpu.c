/*
 * Measurement aid for the benchmark (include/fa_bench.h): the streaming-read yardstick for the host-side
 * decoding attention.  Its own small library, libfa_bench_cpu.so (gcc, OpenMP); libfa_cpu.so neither links
 * nor loads it.
 */
#include <immintrin.h>
#include <stdint.h>
#include <string.h>
#include <omp.h>

#include "../../include/fa_bench.h"

#define AVX512 __attribute__((target("avx512f,avx512bw,avx512dq,avx512vl")))

static int has_avx512(void) {
    __builtin_cpu_init();
    return __builtin_cpu_supports("avx512f") && __builtin_cpu_supports("avx512bw") &&
           __builtin_cpu_supports("avx512dq") && __builtin_cpu_supports("avx512vl");
}

/* ------------------------------------------------------------------ streaming-read yardstick */

/* Four lines per step, one from each quarter of the share: a core sustains more bytes per second over several
   concurrent sequential streams than over one (the decoding loop itself reads K and V side by side). */
#define STREAMS 4

AVX512 static uint64_t sum_avx512(const unsigned char *p, size_t n64) {
    const size_t q = n64 / STREAMS;
    __m512i a[STREAMS];
    for (int s = 0; s < STREAMS; ++s) a[s] = _mm512_setzero_si512();
    for (size_t i = 0; i < q; ++i)
        for (int s = 0; s < STREAMS; ++s)
            a[s] = _mm512_add_epi64(a[s], _mm512_loadu_si512((const void *)(p + 64 * (s * q + i))));
    for (size_t i = STREAMS * q; i < n64; ++i) a[0] = _mm512_add_epi64(a[0], _mm512_loadu_si512((const void *)(p + 64 * i)));
    uint64_t lanes[8], t = 0;       /* summed as unsigned words: the wrap-around is meant */
    _mm512_storeu_si512((void *)lanes, _mm512_add_epi64(_mm512_add_epi64(a[0], a[1]), _mm512_add_epi64(a[2], a[3])));
    for (int i = 0; i < 8; ++i) t += lanes[i];
    return t;
}

static uint64_t sum_scalar(const unsigned char *p, size_t n64) {
    const size_t q = n64 / STREAMS;
    uint64_t t[STREAMS] = {0, 0, 0, 0};
    for (size_t i = 0; i < q; ++i)
        for (int s = 0; s < STREAMS; ++s) {
            uint64_t w[8];
            memcpy(w, p + 64 * (s * q + i), 64);
            for (int j = 0; j < 8; ++j) t[s] += w[j];
        }
    for (size_t i = STREAMS * q; i < n64; ++i) {
        uint64_t w[8];
        memcpy(w, p + 64 * i, 64);
        for (int j = 0; j < 8; ++j) t[0] += w[j];
    }
    return t[0] + t[1] + t[2] + t[3];
}

int fa_cpu_stream_read(const void *buf, long long bytes, int nthreads, int reps, int force_scalar, double *gb_per_s,
                       unsigned long long *checksum) {
    if (!buf || !gb_per_s || !checksum) return -1;
    if (bytes < 64 || reps < 1) return -2;
    const int threads = nthreads > 0 ? nthreads : omp_get_max_threads();
    const int avx = !force_scalar && has_avx512();
    const size_t n64 = (size_t)bytes / 64;                 /* whole 64-byte lines */
    uint64_t total = 0;
    const double t0 = omp_get_wtime();
    for (int r = 0; r < reps; ++r) {
#pragma omp parallel for schedule(static) num_threads(threads) reduction(+ : total)
        for (int t = 0; t < threads; ++t) {
            const size_t lo = n64 * (size_t)t / (size_t)threads, hi = n64 * (size_t)(t + 1) / (size_t)threads;
            const unsigned char *p = (const unsigned char *)buf + 64 * lo;
            total += avx ? sum_avx512(p, hi - lo) : sum_scalar(p, hi - lo);
        }
    }
    const double dt = omp_get_wtime() - t0;
    *gb_per_s = (double)n64 * 64.0 * reps / dt / 1e9;
    *checksum = total;
    return 0;
}
