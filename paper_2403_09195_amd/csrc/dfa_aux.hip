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

// xg[b][h][slot][:] = x[b][token(slot)][h][:]; one 16-byte chunk per thread
__global__ __launch_bounds__(256)
void gather_kernel(const char* x, int64_t sb, int64_t sn, int64_t sh, int32_t H, int32_t N, int esize,
                   int32_t w, int32_t r, const HeadOffsets offs, char* xg, int64_t total_chunks) {
    const int chunks = kD * esize / 16;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= total_chunks) return;
    const int32_t per_head = N / r, per_seg = w / r;
    const int64_t rowid = c / chunks;                 // (b, h, slot) flattened
    const int ch = (int)(c % chunks);
    const int32_t slot = (int32_t)(rowid % per_head);
    const int64_t bh = rowid / per_head;
    const int32_t h = (int32_t)(bh % H);
    const int64_t b = bh / H;
    const int64_t n = kept_row(segment_first(slot / per_seg, w, offset_of(offs, h, r)), r, slot % per_seg);
    const char* src = x + (b * sb + n * sn + h * sh) * esize + 16 * ch;
    *reinterpret_cast<u32x4*>(xg + rowid * (kD * esize) + 16 * ch) = *reinterpret_cast<const u32x4*>(src);
}

// out[b][n][h][:] = og[b][h][slot(n)][:] if the branch keeps token n, else 0
__global__ __launch_bounds__(256)
void scatter_kernel(const char* og, int32_t H, int32_t N, int esize, int32_t w, int32_t r,
                    const HeadOffsets offs, char* out, int64_t total_chunks) {
    const int chunks = kD * esize / 16;
    const int64_t c = (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (c >= total_chunks) return;
    const int64_t rowid = c / chunks;                 // (b, n, h) flattened
    const int ch = (int)(c % chunks);
    const int32_t h = (int32_t)(rowid % H);
    const int64_t bn = rowid / H;
    const int32_t n = (int32_t)(bn % N);
    const int64_t b = bn / N;
    const int32_t i = n / w;
    const int32_t pos = n - segment_first(i, w, offset_of(offs, h, r));
    u32x4 val = {0u, 0u, 0u, 0u};
    if (pos >= 0 && pos % r == 0) {
        const int64_t slot = (int64_t)i * (w / r) + pos / r;
        val = *reinterpret_cast<const u32x4*>(og + ((b * H + h) * (N / r) + slot) * (kD * esize) + 16 * ch);
    }
    *reinterpret_cast<u32x4*>(out + rowid * (kD * esize) + 16 * ch) = val;
}

// L = log sum_b exp(lse_b); out = sum_b exp(lse_b - L) out_b.  16 lanes per row, 4 d each.
template <bool kOutBf16>
__global__ __launch_bounds__(256)
void merge_kernel(const float* out_b, const float* lse_b, int32_t nb, int32_t H, int32_t N,
                  int64_t rows, void* out, float* lse) {
    const int64_t x = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t rowid = x >> 4;                     // (b, n, h) flattened
    if (rowid >= rows) return;
    const int part = (int)(x & 15);
    const int32_t h = (int32_t)(rowid % H);
    const int64_t bn = rowid / H;
    const int32_t n = (int32_t)(bn % N);
    const int64_t b = bn / N;
    const int64_t lidx = (b * H + h) * N + n;
    float lb[DFA_MAX_BRANCHES];
    float m = -INFINITY;
    for (int s = 0; s < nb; ++s) {
        lb[s] = lse_b[(int64_t)s * rows + lidx];
        m = fmaxf(m, lb[s]);
    }
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    float L = -INFINITY;
    if (m > -INFINITY) {
        float z = 0.f;
        for (int s = 0; s < nb; ++s) z += __builtin_amdgcn_exp2f((lb[s] - m) * kLog2e);
        const float inv = 1.0f / z;
        L = m + __builtin_amdgcn_logf(z) * kLn2;
        for (int s = 0; s < nb; ++s) {
            if (lb[s] == -INFINITY) continue;
            const float wgt = __builtin_amdgcn_exp2f((lb[s] - m) * kLog2e) * inv;
            const float4 o = *reinterpret_cast<const float4*>(out_b + ((int64_t)s * rows + rowid) * kD + 4 * part);
            acc.x = fmaf(wgt, o.x, acc.x);
            acc.y = fmaf(wgt, o.y, acc.y);
            acc.z = fmaf(wgt, o.z, acc.z);
            acc.w = fmaf(wgt, o.w, acc.w);
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
    const int64_t total = (int64_t)B * H * (N / r) * (kD * esize / 16);
    hipLaunchKernelGGL(gather_kernel, dim3(blocks_for(total)), dim3(256), 0, st,
                       static_cast<const char*>(x), sb, sn, sh, H, N, esize, w, r, offs,
                       static_cast<char*>(xg), total);
    return hipGetLastError();
}

hipError_t launch_scatter(const void* og, int32_t B, int32_t H, int32_t N, int esize, int32_t w,
                          int32_t r, const HeadOffsets& offs, void* out, hipStream_t st) {
    const int64_t total = (int64_t)B * N * H * (kD * esize / 16);
    hipLaunchKernelGGL(scatter_kernel, dim3(blocks_for(total)), dim3(256), 0, st,
                       static_cast<const char*>(og), H, N, esize, w, r, offs, static_cast<char*>(out), total);
    return hipGetLastError();
}

hipError_t launch_merge(const float* out_b, const float* lse_b, int32_t nb, int32_t B, int32_t H,
                        int32_t N, bool out_bf16, void* out, float* lse, hipStream_t st) {
    const int64_t rows = (int64_t)B * N * H;
    if (out_bf16)
        hipLaunchKernelGGL(merge_kernel<true>, dim3(blocks_for(rows * 16)), dim3(256), 0, st,
                           out_b, lse_b, nb, H, N, rows, out, lse);
    else
        hipLaunchKernelGGL(merge_kernel<false>, dim3(blocks_for(rows * 16)), dim3(256), 0, st,
                           out_b, lse_b, nb, H, N, rows, out, lse);
    return hipGetLastError();
}

}  // namespace dfa
