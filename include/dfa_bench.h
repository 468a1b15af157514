/*
 * dfa_bench.h - measurement aids of the dilated flash attention library.  They are exported by the
 * same shared library but are no part of the operator's interface (dfa.h): a benchmark harness times
 * launches with them and measures what the matrix cores sustain on their own.
 */
#ifndef DFA_BENCH_H
#define DFA_BENCH_H

#include "dfa.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Times `iters` back-to-back dfa_forward launches with HIP events recorded on `stream`
 * (the stream the kernel runs on) and returns the mean milliseconds per launch in *ms.
 * Arguments as dfa_forward.  Synchronises `stream`.  For benchmarks.
 */
int dfa_forward_timed(const void *q, const void *k, const void *v,
                      dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                      int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                      const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets,
                      void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream,
                      int32_t iters, float *ms);

/*
 * Comparison path of the input-size sweep: dense softmax attention over all N tokens (Eq. 2 with one segment,
 * w = N, r = 1) computed the plain way, with the score matrix held in memory - the "FlashAttention off" side of
 * the paper's ablation (section 4.3, Fig. 4).  Four launches on `stream`: S = Q K^T (batched matrix-core
 * product), row softmax in place, a transpose of V, O = P V.
 *   q, k, v, strides, B, H, N, D, scale   as in dfa_forward, bf16 only; N % 256 == 0 and N <= 4096
 *   out         device bf16 [B, N, H, D];  lse device fp32 [B, H, N] or NULL
 *   workspace   device, 16-byte aligned, dfa_dense_unfused_workspace_bytes() = room for the bf16 scores
 *               [B, H, N, N] and V^T [B, H, D, N]; DFA_ERR_WORKSPACE when smaller
 * Scores and probabilities are rounded to bf16 on their way through memory.
 */
size_t dfa_dense_unfused_workspace_bytes(int32_t B, int32_t H, int32_t N, int32_t D);
int dfa_dense_unfused(const void *q, const void *k, const void *v,
                      dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                      int32_t B, int32_t H, int32_t N, int32_t D, float scale,
                      void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Measurement aid (no part of the operator): what the matrix cores sustain on their own, the
 * ceiling that the kernels' MFMA rooflines are also quoted against.  Runs a loop of
 * independent v_mfma_f32_32x32x16_bf16 on the whole chip (two waves per SIMD, no memory
 * traffic) on the default stream and synchronises.
 *   random_operands  0: small constant operands; 1: pseudo-random bf16 operands (more bits
 *                    toggle, the sustained clock is lower)
 *   tflops           out, host: achieved TFLOP/s
 *   shader_mhz       out, host: shader clock during the loop (cycle counter / 100 MHz wall counter)
 * Allocates and frees a few bytes of device memory.
 */
int dfa_mfma_peak(int32_t random_operands, float *tflops, float *shader_mhz);

#ifdef __cplusplus
}
#endif
#endif /* DFA_BENCH_H */
