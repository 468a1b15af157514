// Backward of the fused dilated attention: dq, dk, dv for a gradient dout of the merged output.
//
// The paper states no backward pass; this is the chain rule on Eq. 2 and the branch merge.  The
// merged operator is a softmax over the multiset union of a row's key lists, so with the merged
// lse of the forward pass, P(n, j) = exp(scale q_n.k_j - lse_n) per (branch, n, j) pair and
// delta_n = dout_n . out_n:
//   dv_j += P dout_n,   ds = P (dout_n . v_j - delta_n),   dq_n += scale ds k_j,   dk_j += scale ds q_n.
// P is recomputed from lse, nothing of the forward pass is stored besides out and lse.  Where the
// plan visits a pair once for the m branches that hold it, P carries the factor m (every formula
// above is linear in P).
//
// This file: the per-row preparation of the fp32 path (delta, and lse in base-2 units; the bf16 path does it in
// its dq kernel) and
// the fp32 path, correctness-first kernels in fp32 vector arithmetic on the same launch plan as
// the forward pass, one lane per row of a tile.  bf16 operands go to the matrix-core kernels.  In a
// segment the kept rows are queries and keys alike, so a tile's key lists are also the lists of
// queries that see its rows as keys: the dq kernel walks them as keys, the dk and dv kernels walk
// them as queries, and no gradient needs an atomic or a second pass over partial sums.
#include "dfa_device.h"

namespace dfa {

namespace {

template <typename T>
__device__ __forceinline__ float4 load4(const T* p);
template <>
__device__ __forceinline__ float4 load4<float>(const float* p) { return *reinterpret_cast<const float4*>(p); }
template <typename T>
__device__ __forceinline__ void store4v(T* p, float a, float b, float c, float d);
template <>
__device__ __forceinline__ void store4v<float>(float* p, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(p) = make_float4(a, b, c, d);
}

template <typename T>
__device__ __forceinline__ void load_row(const T* p, float (&x)[kD]) {
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
        const float4 t = load4<T>(p + d);
        x[d] = t.x; x[d + 1] = t.y; x[d + 2] = t.z; x[d + 3] = t.w;
    }
}
template <typename T>
__device__ __forceinline__ void store_row(T* p, const float (&x)[kD]) {
#pragma unroll
    for (int d = 0; d < kD; d += 4) store4v<T>(p + d, x[d], x[d + 1], x[d + 2], x[d + 3]);
}

__device__ __forceinline__ float dot_row(const float (&a)[kD], const float* b) {
    float d0 = 0.f, d1 = 0.f, d2 = 0.f, d3 = 0.f;               // four interleaved partial sums
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
        const float4 x = *reinterpret_cast<const float4*>(b + d);
        d0 = fmaf(a[d], x.x, d0);
        d1 = fmaf(a[d + 1], x.y, d1);
        d2 = fmaf(a[d + 2], x.z, d2);
        d3 = fmaf(a[d + 3], x.w, d3);
    }
    return (d0 + d1) + (d2 + d3);
}
__device__ __forceinline__ void axpy_row(float s, const float* b, float (&acc)[kD]) {
#pragma unroll
    for (int d = 0; d < kD; d += 4) {
        const float4 x = *reinterpret_cast<const float4*>(b + d);
        acc[d] = fmaf(s, x.x, acc[d]);
        acc[d + 1] = fmaf(s, x.y, acc[d + 1]);
        acc[d + 2] = fmaf(s, x.z, acc[d + 2]);
        acc[d + 3] = fmaf(s, x.w, acc[d + 3]);
    }
}

// ndelta[b][h][n] = -(dout[b][n][h][:] . out[b][n][h][:]) and lse2 = lse * log2(e); 16 lanes per row, 4 d each.
// grid = (16 * rows of one image / 256, B): one image is indexed with 32-bit arithmetic.
template <typename T>
__global__ __launch_bounds__(256)
void bwd_delta_kernel(const T* out, const T* dout, const float* lse, float* ndelta, float* lse2, int32_t H, int32_t N) {
    const uint32_t x = blockIdx.x * 256u + threadIdx.x;
    const uint32_t t = x >> 4;                                       // n * H + h
    const int part = (int)(x & 15u);
    const bool in = t < (uint32_t)N * (uint32_t)H;
    const int64_t b = blockIdx.y;
    const int64_t rowid = b * N * H + t;                             // (b, n, h) flattened
    float s = 0.f;
    if (in) {
        const float4 a = load4<T>(out + rowid * kD + 4 * part), g = load4<T>(dout + rowid * kD + 4 * part);
        s = (a.x * g.x + a.y * g.y) + (a.z * g.z + a.w * g.w);
    }
#pragma unroll
    for (int m = 8; m >= 1; m >>= 1) s += __shfl_xor(s, m, 16);
    if (in && part == 0) {
        const uint32_t n = t / (uint32_t)H, h = t - n * (uint32_t)H;
        const int64_t at = (b * H + h) * N + n;
        ndelta[at] = -s;
        lse2[at] = lse[at] * kLog2e;
    }
}

// Stages 64 rows of a strided tensor (rows key0 + stride * j of image b, head h) into LDS as fp32;
// positions past the end of the list re-read its last row.
template <typename T>
__device__ __forceinline__ void stage_rows(const T* base, int64_t sn, const KeySeg& seg, int t, float* lds, int tid) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int kr = (tid >> 4) + 16 * u;
        const int j = min(t * kKeyTile + kr, seg.count - 1);
        const int64_t row = kept_row(seg.key0, seg.stride, j);
        const int cch = (tid & 15) * 4;
        *reinterpret_cast<float4*>(lds + kr * kD + cch) = load4<T>(base + row * sn + cch);
    }
}

// kMode 0: dq of the tile's rows (they are queries; the lists are walked as keys)
// kMode 1: dv of the tile's rows (they are keys; the lists are walked as queries)
// kMode 2: dk of the tile's rows (likewise)
template <typename T, int kMode>
__global__ __launch_bounds__(256)
void bwd_kernel(const BwdParams p) {
    __shared__ __attribute__((aligned(16))) float a_lds[kKeyTile * kD];   // k rows (mode 0) or q rows (modes 1, 2)
    __shared__ __attribute__((aligned(16))) float b_lds[kKeyTile * kD];   // v rows (mode 0) or dout rows
    __shared__ float l_lds[kKeyTile], d_lds[kKeyTile];                     // lse and -delta of the staged queries

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = item.t;
    const int tid = threadIdx.x;
    const int h = tile.h, b = item.b;
    const bool live = tid < tile.nrows;
    const int64_t n = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    const int64_t row_c = (((int64_t)b * p.N + n) * p.H + h) * kD;         // this row in a contiguous [B,N,H,D] tensor
    T* const grad = static_cast<T*>(kMode == 0 ? p.dq : kMode == 1 ? p.dv : p.dk) + row_c;

    float acc[kD];
#pragma unroll
    for (int d = 0; d < kD; ++d) acc[d] = 0.f;
    if (tile.nseg == 0) {                    // rows that no branch keeps take and give no gradient
        if (live) store_row<T>(grad, acc);
        return;
    }

    const T* const qb = static_cast<const T*>(p.q) + (int64_t)b * p.sqb + (int64_t)h * p.sqh;
    const T* const kb = static_cast<const T*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const T* const vb = static_cast<const T*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;
    const T* const gb = static_cast<const T*>(p.dout) + ((int64_t)b * p.N * p.H + h) * kD;   // row n at n * H * D
    const float* const lse_bh = p.lse + ((int64_t)b * p.H + h) * p.N;
    const float* const ndelta_bh = p.ndelta + ((int64_t)b * p.H + h) * p.N;

    float x0[kD], x1[kD];                    // mode 0: q, dout of this row; mode 1: k; mode 2: k, v
    float my_l = 0.f, my_d = 0.f;
    if (kMode == 0) {
        load_row<T>(qb + n * p.sqn, x0);
        load_row<T>(gb + n * p.H * kD, x1);
        my_l = lse_bh[n] * kLog2e;
        my_d = ndelta_bh[n];
    } else {
        load_row<T>(kb + n * p.skn, x0);
        if (kMode == 2) load_row<T>(vb + n * p.svn, x1);
    }

    for (int s = 0; s < tile.nseg; ++s) {
        const KeySeg seg = p.segs[tile.seg_begin + s];
        for (int t = 0; t * kKeyTile < seg.count; ++t) {
            __syncthreads();                 // previous tile fully consumed
            if (kMode == 0) {
                stage_rows<T>(kb, p.skn, seg, t, a_lds, tid);
                stage_rows<T>(vb, p.svn, seg, t, b_lds, tid);
            } else {
                stage_rows<T>(qb, p.sqn, seg, t, a_lds, tid);
                stage_rows<T>(gb, (int64_t)p.H * kD, seg, t, b_lds, tid);
                if (tid < kKeyTile) {
                    const int64_t row = kept_row(seg.key0, seg.stride, min(t * kKeyTile + tid, seg.count - 1));
                    l_lds[tid] = lse_bh[row] * kLog2e;
                    d_lds[tid] = ndelta_bh[row];
                }
            }
            __syncthreads();
            const int nvalid = min(kKeyTile, seg.count - t * kKeyTile);
            for (int c = 0; c < nvalid; ++c) {
                const float* ar = a_lds + c * kD;
                const float* br = b_lds + c * kD;
                const float sc = dot_row(x0, ar) * p.scale;                       // scale q.k
                if (kMode == 0) {
                    const float pr = __builtin_amdgcn_exp2f(sc * kLog2e + seg.log2_mult - my_l);
                    const float ds = pr * (dot_row(x1, br) + my_d) * p.scale;
                    axpy_row(ds, ar, acc);                                        // dq += scale ds k
                } else {
                    const float pr = __builtin_amdgcn_exp2f(sc * kLog2e + seg.log2_mult - l_lds[c]);
                    if (kMode == 1) {
                        axpy_row(pr, br, acc);                                    // dv += P dout
                    } else {
                        const float ds = pr * (dot_row(x1, br) + d_lds[c]) * p.scale;
                        axpy_row(ds, ar, acc);                                    // dk += scale ds q
                    }
                }
            }
        }
    }
    if (live) store_row<T>(grad, acc);
}

}  // namespace

// fp32 operands: the per-row preparation, then one vector kernel per gradient.  bf16 operands go to the
// matrix-core kernels, whose dq kernel prepares the per-row values itself.
hipError_t launch_bwd(const BwdParams& p, int n_items, int32_t B, bool bf16, hipStream_t st) {
    if (bf16) return launch_bwd_bf16(p, n_items, st);
    hipLaunchKernelGGL((bwd_delta_kernel<float>), dim3((unsigned)(((int64_t)p.N * p.H * 16 + 255) / 256), B), dim3(256), 0, st,
                       static_cast<const float*>(p.out), static_cast<const float*>(p.dout), p.lse, p.ndelta, p.lse2, p.H, p.N);
    hipLaunchKernelGGL((bwd_kernel<float, 0>), dim3(n_items), dim3(256), 0, st, p);
    hipLaunchKernelGGL((bwd_kernel<float, 1>), dim3(n_items), dim3(256), 0, st, p);
    hipLaunchKernelGGL((bwd_kernel<float, 2>), dim3(n_items), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace dfa
