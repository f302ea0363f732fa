/*
 * fa_cpu.h -- C ABI of the host-side half of FastAttention's CPU-GPU cooperative strategy
 * (section 4.4, appendix C): the closed-form split of the transformer layers into those whose
 * KV cache stays in GPU memory and those whose KV cache lives in host memory, and the
 * decoding-step attention that the host computes for the latter, multi-threaded and
 * vectorised, so that only Q, K, V of the new token go down and one output row comes back.
 *
 * Everything here runs on the host CPU (libfa_cpu.so, no HIP); all pointers are HOST pointers.
 */
#ifndef FA_CPU_H
#define FA_CPU_H

#ifdef __cplusplus
extern "C" {
#endif

#define FA_CPU_OK          0
#define FA_CPU_ERR_NULL   -1 /* a required pointer is NULL */
#define FA_CPU_ERR_SHAPE  -2 /* a size is not positive (or negative where zero is allowed) */
#define FA_CPU_ERR_HEADDIM -3 /* D is not a positive multiple of 16, or exceeds 256 */
#define FA_CPU_ERR_DTYPE  -4 /* dtype is not 0 (fp16) or 1 (bf16) */
#define FA_CPU_ERR_SCALE  -5 /* scale is NaN or infinite */
#define FA_CPU_ERR_NOMEM  -8 /* the scratch for the threads' partial results could not be allocated */

/*
 * fa_coop_plan_bytes -- the layer split of section 4.4, general form:
 *     L_GPU = floor( (M_GPU - M_w / n - M_mid - M_vocab) / M_kv ),  clamped to 0 .. L
 *     L_CPU = L - L_GPU
 * The first L_CPU layers keep their KV cache in host memory, the remaining L_GPU layers in GPU
 * memory.  All M_* are bytes on ONE GPU except m_w, the weights of the whole model, which are
 * divided over the n GPUs:
 *   m_gpu   : memory of one GPU;  m_w: all weights;  m_mid: largest intermediate results;
 *   m_vocab : the vocabulary matrix;  m_kv: KV cache of ONE layer on one GPU (> 0)
 * Returns FA_CPU_OK and writes *l_gpu, *l_cpu (host ints), or a negative code.
 */
int fa_coop_plan_bytes(double m_gpu, double m_w, double m_mid, double m_vocab, double m_kv,
                       int n, int L, int *l_gpu, int *l_cpu);

/*
 * fa_coop_plan_fp16 -- the same split with appendix C's FP16 expressions filled in:
 *     M_w     = L (8 H1^2 + 4 H1 H2)        four H1 x H1 and two H1 x H2 matrices per layer, 2 bytes each
 *     M_kv    = 4 B H1 (S + O) / n          K and V, 2 bytes, prompt S plus O generated tokens
 *     M_mid   = 6 B S H1 / n                Q, K, V of the prompt, 2 bytes
 *     M_vocab = V H1                        as the appendix prints it
 *     L_GPU   = (n M_GPU - L (8 H1^2 + 4 H1 H2) - 6 B S H1 - n V H1) / (4 B H1 (S + O)),  floor, clamped
 *   m_gpu : bytes of one GPU;  n: GPUs;  L: layers;  H1: hidden size;  H2: FFN size;
 *   V: vocabulary size;  B: batch;  S: prompt length;  O: tokens to generate
 */
int fa_coop_plan_fp16(double m_gpu, int n, int L, long long H1, long long H2, long long V,
                      long long B, long long S, long long O, int *l_gpu, int *l_cpu);

/*
 * fa_cpu_decode -- attention of one decoding step on the host (section 4.4, step 4; appendix C,
 * decoding equations): for every batch entry b and head h, one query row against the Nk cached
 * keys and values,
 *     o[b,h,:] = softmax_j( scale * q[b,h,:] . k[b,h,j,:] ) v[b,h,j,:],   lse[b,h] = ln sum_j exp(...)
 *   q, o : [B, H, D] 16-bit elements of `dtype` (0 = fp16, 1 = bf16); k, v : [B, H, Nk, D]; lse : [B, H] fp32
 *   D    : a multiple of 16, at most 256
 *   nthreads : OpenMP threads to use; <= 0: the runtime's default
 * Products and sums are fp32; the keys are cut into runs that threads take independently (running
 * maximum and sum per run, as in the tiled GPU kernel) and merged at the end, so the work spreads
 * over the cores even for a single head.  Uses AVX-512 when the CPU has it (checked at run time),
 * plain C otherwise.  The caller owns every buffer; o and lse must not alias the inputs.
 */
int fa_cpu_decode(const void *q, const void *k, const void *v, void *o, float *lse,
                  int B, int H, int Nk, int D, float scale, int dtype, int nthreads);

/* 1 if fa_cpu_decode runs its AVX-512 path on this machine, else 0 */
int fa_cpu_has_avx512(void);

/* Test hook: on != 0 makes fa_cpu_decode run its plain C loops whatever the CPU has, 0 restores the choice at
   run time.  Process-wide, read once per fa_cpu_decode call; returns the previous setting.  The library reads no
   environment variable. */
int fa_cpu_set_scalar(int on);

#ifdef __cplusplus
}
#endif
#endif /* FA_CPU_H */
