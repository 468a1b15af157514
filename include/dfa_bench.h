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
