// Dense attention the plain way, with the score matrix materialised in memory: the "FlashAttention off" side of
// the paper's ablation over input sizes (section 4.3, Fig. 4), built from this library's own pieces so that the
// size sweep can put it beside the fused kernel on the same chip:
//   1. S = Q K^T per (b, h)                batched matrix-core product, S bf16 [B, H, N, N]
//   2. P = softmax(scale * S) row by row   in place (fp32 arithmetic, P rounded to bf16), lse written
//   3. V^T per (b, h)                      small transpose, so that both operands of step 4 have the contraction
//                                          index contiguous
//   4. O = P V                             batched matrix-core product, written at [B, N, H, D]
// Scores and probabilities pass through memory as bf16, as a framework's unfused attention in bf16 would hold
// them: a scaled score of magnitude below 8 is off by at most 2^-6 after its rounding, which bounds the error
// of lse (measured some 1e-3) and sits well inside the bars of the outputs.
#include "dfa_device.h"
#include "dfa_mfma.h"

namespace dfa {

namespace {

// One wave per row of S (N <= 4096: at most 8 chunks of 8 scores per lane, held in registers).
__global__ __launch_bounds__(256) void softmax_rows_kernel(uint16_t* __restrict__ s, float* __restrict__ lse, int64_t rows,
                                                           int32_t N, float scale_log2e) {
    const int lane = threadIdx.x & 63;
    const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    uint16_t* rp = s + row * N;
    const int chunks = N / 8;                  // 16-byte chunks of the row
    u32x4 raw[8];
    float x[8][8];
    float mx = -INFINITY;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int ch = lane + 64 * c;
        if (ch < chunks) {
            raw[c] = *reinterpret_cast<const u32x4*>(rp + 8 * ch);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                x[c][2 * e] = __builtin_bit_cast(float, raw[c][e] << 16);
                x[c][2 * e + 1] = __builtin_bit_cast(float, raw[c][e] & 0xffff0000u);
                mx = fmaxf(mx, fmaxf(x[c][2 * e], x[c][2 * e + 1]));
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) mx = fmaxf(mx, __shfl_xor(mx, off));
    const float m2 = mx * scale_log2e;         // scale > 0: the largest scaled score
    float sum = 0.f;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int ch = lane + 64 * c;
        if (ch < chunks) {
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                x[c][e] = __builtin_amdgcn_exp2f(fmaf(x[c][e], scale_log2e, -m2));
                sum += x[c][e];
            }
        }
    }
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) sum += __shfl_xor(sum, off);
    const float inv = 1.0f / sum;
#pragma unroll
    for (int c = 0; c < 8; ++c) {
        const int ch = lane + 64 * c;
        if (ch < chunks) {
            u32x4 o;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const bf16x2 pr = {(__bf16)(x[c][2 * e] * inv), (__bf16)(x[c][2 * e + 1] * inv)};
                o[e] = __builtin_bit_cast(uint32_t, pr);
            }
            *reinterpret_cast<u32x4*>(rp + 8 * ch) = o;
        }
    }
    if (lane == 0 && lse) lse[row] = (m2 + __builtin_amdgcn_logf(sum)) * kLn2;
}

// V [B, N, H, D] (strided) -> V^T [B, H, D, N]: a workgroup transposes 64 tokens x 64 features of one (b, h)
// through LDS; reads and writes are 128-byte rows.
__global__ __launch_bounds__(256) void transpose_v_kernel(const uint16_t* __restrict__ v, int64_t svb, int64_t svn, int64_t svh,
                                                          int32_t H, int32_t N, uint16_t* __restrict__ vt) {
    __shared__ uint16_t tile[64][kD + 2];
    const int bh = blockIdx.y, b = bh / H, h = bh % H, n0 = blockIdx.x * 64;
    const uint16_t* src = v + (int64_t)b * svb + (int64_t)h * svh;
    for (int i = threadIdx.x; i < 64 * kD; i += 256) {
        const int n = i / kD, d = i % kD;
        tile[n][d] = src[(int64_t)(n0 + n) * svn + d];
    }
    __syncthreads();
    uint16_t* dst = vt + (int64_t)bh * kD * N;
    for (int i = threadIdx.x; i < 64 * kD; i += 256) {
        const int d = i / 64, n = i % 64;
        dst[(int64_t)d * N + n0 + n] = tile[n][d];
    }
}

}  // namespace

hipError_t launch_dense_unfused(const void* q, const void* k, const void* v, int64_t sqb, int64_t sqn, int64_t sqh,
                                int64_t skb, int64_t skn, int64_t skh, int64_t svb, int64_t svn, int64_t svh,
                                int32_t B, int32_t H, int32_t N, float scale, void* out, float* lse,
                                void* scores, void* vt, hipStream_t st) {
    const int64_t NN = (int64_t)N * N;
    // 1. S = Q K^T: rows of Q against rows of K, contraction over the D features
    hipError_t e = launch_linear_bf16_batched(q, k, scores, N, N, kD, sqn, skn, N, B, H, sqb, sqh, skb, skh, H * NN, NN, st);
    if (e != hipSuccess) return e;
    // 2. row softmax in place
    const int64_t rows = (int64_t)B * H * N;
    hipLaunchKernelGGL(softmax_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, st,
                       static_cast<uint16_t*>(scores), lse, rows, N, scale * kLog2e);
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // 3. V^T
    hipLaunchKernelGGL(transpose_v_kernel, dim3(N / 64, B * H), dim3(256), 0, st, static_cast<const uint16_t*>(v),
                       svb, svn, svh, H, N, static_cast<uint16_t*>(vt));
    if ((e = hipGetLastError()) != hipSuccess) return e;
    // 4. O = P V: rows of P against rows of V^T, contraction over the N keys; row n of (b, h) lands at out[b, n, h, :]
    return launch_linear_bf16_batched(scores, vt, out, N, kD, N, N, N, (int64_t)H * kD, B, H, H * NN, NN,
                                      (int64_t)H * kD * N, (int64_t)kD * N, (int64_t)N * H * kD, kD, st);
}

}  // namespace dfa
