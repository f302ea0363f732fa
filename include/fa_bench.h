/*
 * fa_bench.h -- measurement aids for the benchmark, kept out of the product libraries: a
 * matrix-only kernel that gives the MFMA throughput the chip sustains (the practical ceiling to
 * quote beside the nominal peak of the attention kernels of fa.h), and a streaming-read loop that
 * gives the host-memory ceiling for the CPU-side decoding attention of fa_cpu.h.  Built into
 * libfa_bench.so (HIP) and libfa_bench_cpu.so (plain C); neither is needed, loaded or linked by
 * libfa.so / libfa_cpu.so.
 */
#ifndef FA_BENCH_H
#define FA_BENCH_H

#ifdef __cplusplus
extern "C" {
#endif

/*
 * fa_mfma_probe (libfa_bench.so) -- enqueues a kernel that issues nothing but independent
 * v_mfma_f32_32x32x16 instructions of `dtype` (0 = fp16, 1 = bf16; 256 workgroups of 8 waves,
 * `iters` x 4 instructions per wave) and reports the floating-point operations it performs in
 * *flops (HOST pointer).  Timed by the caller, it gives the matrix throughput the chip sustains
 * under its power limit.  `operands`: 0 = one pair of operands with a few low bits set, the same
 * for every instruction (hardly any switching: the friendliest case for the power limit); 1 = four
 * pairs of pseudo-random operands taken in turn (signs and mantissas toggle from instruction to
 * instruction, as with real data).  `scratch`: DEVICE pointer to one float (never written in
 * practice).  1 <= iters <= 2^24.  `stream`: hipStream_t as void*.
 * Returns 0, or -1 (NULL pointer), -2 (operands / iters out of range), -4 (dtype), -6 (scratch not
 * 4-byte aligned), -7 (the launch failed).
 */
int fa_mfma_probe(int dtype, int operands, int iters, float *scratch, long long *flops, void *stream);

/*
 * fa_cpu_stream_read (libfa_bench_cpu.so) -- `nthreads` threads (<= 0: the OpenMP runtime's
 * default) each add up a contiguous share of the 64-byte lines of `buf` (HOST pointer, `bytes` >=
 * 64, a tail shorter than a line is left out), `reps` times over; *gb_per_s receives the bytes read
 * per second in units of 1e9, *checksum the sum of the 64-bit words modulo 2^64 times `reps` (so
 * that the reads cannot be optimised away, and so that a test can check them).  AVX-512 loads when
 * the CPU has them and force_scalar == 0, plain C otherwise.  Decoding-step attention on the host
 * reads every byte of K and V once and does little else: what this loop reaches over a buffer much
 * larger than the caches is the ceiling for it on the machine at hand.
 * Returns 0, -1 (NULL pointer) or -2 (bytes < 64 or reps < 1).
 */
int fa_cpu_stream_read(const void *buf, long long bytes, int nthreads, int reps, int force_scalar,
                       double *gb_per_s, unsigned long long *checksum);

#ifdef __cplusplus
}
#endif
#endif /* FA_BENCH_H */
