// Stand-alone stages of dilated attention: device indexer, gather (Eq. 1), placement
// (the MAP of Eq. 3) and the log-sum-exp branch merge.  All are memory-bound streaming
// kernels: 16-byte accesses, consecutive lanes on consecutive bytes of a row.
#include "dfa_device.h"

namespace dfa {

namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x4v __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int32_t offset_of(const HeadOffsets& offs, int32_t h, int32_t r) {
    return offs.explicit_table ? offs.o[h] : h % r;
}

// idx[h][slot], slot = i * (w/r) + j  ->  token i*w + o_h + j*r
__global__ __launch_bounds__(256)
void index_map_kernel(int32_t N, int32_t H, int32_t w, int32_t r, const HeadOffsets offs, int32_t* idx) {
    const int32_t per_head = N / r, per_seg = w / r;
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (x >= (int64_t)H * per_head) return;
    const int32_t h = (int32_t)(x / per_head), slot = (int32_t)(x % per_head);
    const int32_t i = slot / per_seg, j = slot % per_seg;
    idx[x] = kept_row(segment_first(i, w, offset_of(offs, h, r)), r, j);
}

// The three streaming kernels below index with 32-bit arithmetic inside one image (grid.y or
// grid.z carries b and h), so a thread spends a handful of integer instructions per 16 bytes.

// xg[b][h][slot][:] = x[b][token(slot)][h][:]; one 16-byte chunk per thread.
// grid = (chunks of one (b, h) / 256, H, B)
__global__ __launch_bounds__(256)
void gather_kernel(const char* x, int64_t sb, int64_t sn, int64_t sh, int32_t N, int esize, int chunk_shift,
                   int32_t w, int32_t r, const HeadOffsets offs, char* xg) {
    const int32_t per_head = N / r, per_seg = w / r;
    const uint32_t c = blockIdx.x * 256u + threadIdx.x;        // chunk within this (b, h)
    const uint32_t slot = c >> chunk_shift;
    if (slot >= (uint32_t)per_head) return;
    const uint32_t ch = c & ((1u << chunk_shift) - 1u);
    const int32_t h = blockIdx.y, H = gridDim.y;
    const int64_t b = blockIdx.z;
    const uint32_t seg = slot / (uint32_t)per_seg;
    const int32_t n = kept_row(segment_first((int32_t)seg, w, offset_of(offs, h, r)), r, (int32_t)(slot - seg * per_seg));
    const char* src = x + (b * sb + (int64_t)n * sn + (int64_t)h * sh) * esize + 16 * ch;
    char* dst = xg + ((b * H + h) * per_head + slot) * (int64_t)(kD * esize) + 16 * ch;
    *reinterpret_cast<u32x4*>(dst) = *reinterpret_cast<const u32x4*>(src);
}

// out[b][n][h][:] = og[b][h][slot(n)][:] if the branch keeps token n, else 0.
// grid = (chunks of one image / 256, B)
__global__ __launch_bounds__(256)
void scatter_kernel(const char* og, int32_t H, int32_t N, int esize, int chunk_shift, int32_t w, int32_t r,
                    const HeadOffsets offs, char* out) {
    const uint32_t c = blockIdx.x * 256u + threadIdx.x;        // chunk within this image
    const uint32_t t = c >> chunk_shift;                       // n * H + h
    if (t >= (uint32_t)N * (uint32_t)H) return;
    const uint32_t ch = c & ((1u << chunk_shift) - 1u);
    const uint32_t n = t / (uint32_t)H, h = t - n * (uint32_t)H;
    const int64_t b = blockIdx.y;
    const int32_t i = (int32_t)n / w;
    const int32_t pos = (int32_t)n - segment_first(i, w, offset_of(offs, (int32_t)h, r));
    const int32_t q = pos / r;
    u32x4 val = {0u, 0u, 0u, 0u};
    if (pos >= 0 && q * r == pos) {
        const int64_t slot = (int64_t)i * (w / r) + q;
        val = *reinterpret_cast<const u32x4*>(og + ((b * H + h) * (N / r) + slot) * (kD * esize) + 16 * ch);
    }
    *reinterpret_cast<u32x4*>(out + (b * N * H + t) * (int64_t)(kD * esize) + 16 * ch) = val;
}

// L = log sum_b exp(lse_b); out = sum_b exp(lse_b - L) out_b.  16 lanes per row, 4 d each.
// grid = (16 * rows of one image / 256, B)
template <bool kOutBf16>
__global__ __launch_bounds__(256)
void merge_kernel(const float* out_b, const float* lse_b, int32_t nb, int32_t H, int32_t N,
                  int64_t rows, void* out, float* lse) {
    const uint32_t x = blockIdx.x * 256u + threadIdx.x;
    const uint32_t t = x >> 4;                                 // n * H + h
    if (t >= (uint32_t)N * (uint32_t)H) return;
    const int part = (int)(x & 15u);
    const uint32_t n = t / (uint32_t)H, h = t - n * (uint32_t)H;
    const int64_t b = blockIdx.y;
    const int64_t rowid = b * N * H + t;                       // (b, n, h) flattened
    const int64_t lidx = (b * H + h) * N + n;
    float lb[DFA_MAX_BRANCHES];
    float m = -INFINITY;
#pragma unroll
    for (int s = 0; s < DFA_MAX_BRANCHES; ++s) {
        lb[s] = s < nb ? lse_b[(int64_t)s * rows + lidx] : -INFINITY;
        m = fmaxf(m, lb[s]);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = -INFINITY;
    if (m > -INFINITY) {
        float z = 0.f;
        float wgt[DFA_MAX_BRANCHES];
#pragma unroll
        for (int s = 0; s < DFA_MAX_BRANCHES; ++s) {
            wgt[s] = __builtin_amdgcn_exp2f((lb[s] - m) * kLog2e);   // 0 for branches that do not keep the row
            z += wgt[s];
        }
        const float inv = 1.0f / z;
        L = m + __builtin_amdgcn_logf(z) * kLn2;
#pragma unroll
        for (int s = 0; s < DFA_MAX_BRANCHES; ++s) {
            if (s >= nb || lb[s] == -INFINITY) continue;
            const float4 o = *reinterpret_cast<const float4*>(out_b + ((int64_t)s * rows + rowid) * kD + 4 * part);
            const float ws = wgt[s] * inv;
            acc.x = fmaf(ws, o.x, acc.x);
            acc.y = fmaf(ws, o.y, acc.y);
            acc.z = fmaf(ws, o.z, acc.z);
            acc.w = fmaf(ws, o.w, acc.w);
        }
    }
    if (kOutBf16) {
        bf16x4v o = {(__bf16)acc.x, (__bf16)acc.y, (__bf16)acc.z, (__bf16)acc.w};
        *reinterpret_cast<bf16x4v*>(static_cast<__bf16*>(out) + rowid * kD + 4 * part) = o;
    } else {
        *reinterpret_cast<float4*>(static_cast<float*>(out) + rowid * kD + 4 * part) = acc;
    }
    if (lse && part == 0) lse[lidx] = L;
}

inline unsigned blocks_for(int64_t threads) { return (unsigned)((threads + 255) / 256); }

}  // namespace

hipError_t launch_index_map(int32_t N, int32_t H, int32_t w, int32_t r, const HeadOffsets& offs,
                            int32_t* d_idx, hipStream_t st) {
    const int64_t total = (int64_t)H * (N / r);
    hipLaunchKernelGGL(index_map_kernel, dim3(blocks_for(total)), dim3(256), 0, st, N, H, w, r, offs, d_idx);
    return hipGetLastError();
}

hipError_t launch_gather(const void* x, int64_t sb, int64_t sn, int64_t sh, int32_t B, int32_t H,
                         int32_t N, int esize, int32_t w, int32_t r, const HeadOffsets& offs,
                         void* xg, hipStream_t st) {
    const int chunk_shift = esize == 2 ? 3 : 4;               // 16-byte chunks per row: 8 (bf16) or 16 (fp32)
    const int64_t per_bh = (int64_t)(N / r) << chunk_shift;
    hipLaunchKernelGGL(gather_kernel, dim3(blocks_for(per_bh), H, B), dim3(256), 0, st,
                       static_cast<const char*>(x), sb, sn, sh, N, esize, chunk_shift, w, r, offs,
                       static_cast<char*>(xg));
    return hipGetLastError();
}

hipError_t launch_scatter(const void* og, int32_t B, int32_t H, int32_t N, int esize, int32_t w,
                          int32_t r, const HeadOffsets& offs, void* out, hipStream_t st) {
    const int chunk_shift = esize == 2 ? 3 : 4;
    const int64_t per_image = ((int64_t)N * H) << chunk_shift;
    hipLaunchKernelGGL(scatter_kernel, dim3(blocks_for(per_image), B), dim3(256), 0, st,
                       static_cast<const char*>(og), H, N, esize, chunk_shift, w, r, offs, static_cast<char*>(out));
    return hipGetLastError();
}

hipError_t launch_merge(const float* out_b, const float* lse_b, int32_t nb, int32_t B, int32_t H,
                        int32_t N, bool out_bf16, void* out, float* lse, hipStream_t st) {
    const int64_t rows = (int64_t)B * N * H;
    const dim3 grid(blocks_for((int64_t)N * H * 16), B);
    if (out_bf16)
        hipLaunchKernelGGL(merge_kernel<true>, grid, dim3(256), 0, st, out_b, lse_b, nb, H, N, rows, out, lse);
    else
        hipLaunchKernelGGL(merge_kernel<false>, grid, dim3(256), 0, st, out_b, lse_b, nb, H, N, rows, out, lse);
    return hipGetLastError();
}

}  // namespace dfa
