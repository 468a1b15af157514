// Fused dilated flash attention forward in fp32 (plain vector FMAs, no matrix cores).
//
// Same tiling and the same single online-softmax state per query row across all member
// branches as the bf16 kernel; here one lane owns one query row (its q row and its output
// accumulator live in registers) and the 64-key K/V tiles are staged in LDS, where every
// lane reads the same address (a broadcast).  The exponent is taken on (s - m) so that its
// rounding error scales with the distance from the row maximum, not with the logit.
#include "dfa_device.h"

namespace dfa {

namespace {

constexpr int kSub = 16;   // keys per online-softmax step

__global__ __launch_bounds__(256)
void dfa_fwd_f32_kernel(const FwdParams p) {
    __shared__ __attribute__((aligned(16))) float k_lds[kKeyTile * kD];
    __shared__ __attribute__((aligned(16))) float v_lds[kKeyTile * kD];

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = item.t;
    const int tid = threadIdx.x;
    const int h = tile.h, b = item.b;
    const bool live = tid < tile.nrows;
    const int64_t n = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];

    float* const out = static_cast<float*>(p.out) + (((int64_t)b * p.N + n) * p.H + h) * kD;
    float* const lse = p.lse ? p.lse + ((int64_t)b * p.H + h) * p.N + n : nullptr;

    if (tile.nseg == 0) {
        if (live) {
#pragma unroll
            for (int d = 0; d < kD; d += 4) *reinterpret_cast<float4*>(out + d) = make_float4(0.f, 0.f, 0.f, 0.f);
            if (lse) *lse = -INFINITY;
        }
        return;
    }

    float qv[kD], acc[kD];
    {
        const float* qp = static_cast<const float*>(p.q) + (int64_t)b * p.sqb + n * p.sqn + (int64_t)h * p.sqh;
#pragma unroll
        for (int d = 0; d < kD; d += 4) {
            const float4 x = *reinterpret_cast<const float4*>(qp + d);
            qv[d] = x.x; qv[d + 1] = x.y; qv[d + 2] = x.z; qv[d + 3] = x.w;
        }
#pragma unroll
        for (int d = 0; d < kD; ++d) acc[d] = 0.f;
    }
    float m_run = -INFINITY, l_run = 0.f;

    const float* kp = static_cast<const float*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const float* vp = static_cast<const float*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;

    for (int s = 0; s < tile.nseg; ++s) {
        const KeySeg seg = p.segs[tile.seg_begin + s];
        const float ln_mult = seg.log2_mult * kLn2;   // a key that counts m times: weight m exp(s) = exp(s + ln m)
        for (int t = 0; t * kKeyTile < seg.count; ++t) {
            __syncthreads();               // previous tile fully consumed
            // thread -> (key tid/16 + 16u, 16-byte chunk tid%16)
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int kr = (tid >> 4) + 16 * u;
                const int j = min(t * kKeyTile + kr, seg.count - 1);
                const int64_t row = kept_row(seg.key0, seg.stride, j);
                const int cch = (tid & 15) * 4;
                *reinterpret_cast<float4*>(k_lds + kr * kD + cch) =
                    *reinterpret_cast<const float4*>(kp + row * p.skn + cch);
                *reinterpret_cast<float4*>(v_lds + kr * kD + cch) =
                    *reinterpret_cast<const float4*>(vp + row * p.svn + cch);
            }
            __syncthreads();
            const int nvalid = min(kKeyTile, seg.count - t * kKeyTile);
            for (int c0 = 0; c0 < nvalid; c0 += kSub) {
                float sc[kSub];
                float mx = -INFINITY;
#pragma unroll
                for (int jj = 0; jj < kSub; ++jj) {
                    const float* kr = k_lds + (c0 + jj) * kD;
                    // four interleaved partial sums: shorter rounding chains, more ILP
                    float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;
#pragma unroll
                    for (int d = 0; d < kD; d += 4) {
                        const float4 x = *reinterpret_cast<const float4*>(kr + d);
                        d0 = fmaf(qv[d], x.x, d0);
                        d1 = fmaf(qv[d + 1], x.y, d1);
                        d2 = fmaf(qv[d + 2], x.z, d2);
                        d3 = fmaf(qv[d + 3], x.w, d3);
                    }
                    const float dot = (d0 + d1) + (d2 + d3);
                    sc[jj] = (c0 + jj < nvalid) ? dot * p.scale + ln_mult : -INFINITY;
                    mx = fmaxf(mx, sc[jj]);
                }
                const float m_new = fmaxf(m_run, mx);
                const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * kLog2e);
                m_run = m_new;
                l_run *= alpha;
#pragma unroll
                for (int d = 0; d < kD; ++d) acc[d] *= alpha;
#pragma unroll
                for (int jj = 0; jj < kSub; ++jj) {
                    const float pj = __builtin_amdgcn_exp2f((sc[jj] - m_new) * kLog2e);
                    l_run += pj;
                    const float* vr = v_lds + (c0 + jj) * kD;
#pragma unroll
                    for (int d = 0; d < kD; d += 4) {
                        const float4 x = *reinterpret_cast<const float4*>(vr + d);
                        acc[d] = fmaf(pj, x.x, acc[d]);
                        acc[d + 1] = fmaf(pj, x.y, acc[d + 1]);
                        acc[d + 2] = fmaf(pj, x.z, acc[d + 2]);
                        acc[d + 3] = fmaf(pj, x.w, acc[d + 3]);
                    }
                }
            }
        }
    }

    if (live) {
        const float inv = 1.0f / l_run;
#pragma unroll
        for (int d = 0; d < kD; d += 4)
            *reinterpret_cast<float4*>(out + d) =
                make_float4(acc[d] * inv, acc[d + 1] * inv, acc[d + 2] * inv, acc[d + 3] * inv);
        if (lse) *lse = m_run + __builtin_amdgcn_logf(l_run) * kLn2;
    }
}

}  // namespace

hipError_t launch_fwd_f32(const FwdParams& p, int n_items, hipStream_t st) {
    hipLaunchKernelGGL(dfa_fwd_f32_kernel, dim3(n_items), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace dfa
