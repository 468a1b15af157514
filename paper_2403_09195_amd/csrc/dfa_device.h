// Shared device-side declarations of the dilated-attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <cstdint>
#include "dfa_plan.h"

namespace dfa {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kD = DFA_HEAD_DIM;        // head dimension
constexpr int kKeyTile = 64;            // keys staged in LDS per step
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// Arguments of the fused forward kernels.  Strides are in elements.
struct FwdParams {
    const void* q;
    const void* k;
    const void* v;
    int64_t sqb, sqn, sqh;
    int64_t skb, skn, skh;
    int64_t svb, svn, svh;
    void* out;          // [B, N, H, D] contiguous
    float* lse;         // [B, H, N] or nullptr
    const int32_t* rows;
    const KeySeg* segs;
    const Item* items;
    // bf16 kernel only: log2 of the multiplicity of each progression's keys for the rows of each of the tile's eight
    // 32-row blocks, [segs][8]; -inf = the block's rows do not attend to these keys (tiles that pack several row groups)
    const float* block_mult;
    int32_t H, N;
    float scale;        // multiplies q.k
    // Split launches only (few workgroups, see launch_fwd_bf16_split): workgroup g walks the share of a tile's
    // 64-key steps that split_wgs[g] names and leaves its partial result in block g of split_ws;
    // launch_merge_split then writes out and lse.
    const SplitWg* split_wgs;
    const ItemParts* item_parts;
    float* split_ws;
};

// Arguments of the backward kernels.  out, dout, dq, dk, dv are contiguous [B, N, H, D].
struct BwdParams {
    const void* q;
    const void* k;
    const void* v;
    const void* out;
    const void* dout;
    int64_t sqb, sqn, sqh;
    int64_t skb, skn, skh;
    int64_t svb, svn, svh;
    const float* lse;   // [B, H, N], merged, from the forward pass
    float* ndelta;      // [B, H, N] workspace: -(dout . out) per row (negated: it is added to dP, in the dk/dv kernel as
                        // the start value of the dP accumulators)
    float* lse2;        // [B, H, N] workspace: lse * log2(e) per row
    void* dq;
    void* dk;
    void* dv;
    const int32_t* rows;
    const KeySeg* segs;
    const Item* items;
    int32_t H, N;
    float scale;
};

// Per-head start offsets of the stand-alone indexer / gather / scatter kernels, passed by
// value: explicit tables are limited to kMaxExplicitHeads heads, h mod r has no limit.
constexpr int kMaxExplicitHeads = 128;
struct HeadOffsets {
    int32_t explicit_table;             // 0: o = h mod r
    int32_t o[kMaxExplicitHeads];
};

// Kept-row indexer of Eq. 1: row j of the segment whose first kept row is `first`.
__device__ __forceinline__ int32_t kept_row(int32_t first, int32_t stride, int32_t j) {
    return first + stride * j;
}
// First kept row of segment i for start offset o.
__device__ __forceinline__ int32_t segment_first(int32_t i, int32_t w, int32_t o) {
    return i * w + o;
}

// Launchers (defined in the .hip files); every one returns the hipError_t of the launch.
hipError_t launch_fwd_bf16(const FwdParams& p, int n_items, bool out_f32, bool packed, hipStream_t st);
hipError_t launch_fwd_bf16_split(const FwdParams& p, int n_split_wgs, bool packed, hipStream_t st);
hipError_t launch_merge_split(const FwdParams& p, int n_items, hipStream_t st);
hipError_t launch_fwd_f32(const FwdParams& p, int n_items, hipStream_t st);
hipError_t launch_bwd(const BwdParams& p, int n_items, int32_t B, bool bf16, hipStream_t st);
hipError_t launch_bwd_bf16(const BwdParams& p, int n_items, hipStream_t st);
hipError_t launch_linear_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                              int64_t ldx, int64_t ldw, int64_t ldy, const ChipShape& chip, hipStream_t st);
// batch of products of one shape: matrix (z0, z1) starts at x + z0 * xs0 + z1 * xs1 etc.; M % 256 == 0, N % 64 == 0, K % 64 == 0
hipError_t launch_linear_bf16_batched(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                                      int64_t ldx, int64_t ldw, int64_t ldy, int32_t batch_outer, int32_t batch_inner,
                                      int64_t xs0, int64_t xs1, int64_t ws0, int64_t ws1, int64_t ys0, int64_t ys1,
                                      hipStream_t st);
// dense attention with the scores materialised in memory (comparison path of the size sweep)
hipError_t launch_dense_unfused(const void* q, const void* k, const void* v, int64_t sqb, int64_t sqn, int64_t sqh,
                                int64_t skb, int64_t skn, int64_t skh, int64_t svb, int64_t svn, int64_t svh,
                                int32_t B, int32_t H, int32_t N, float scale, void* out, float* lse,
                                void* scores, void* vt, hipStream_t st);
hipError_t launch_index_map(int32_t N, int32_t H, int32_t w, int32_t r, const HeadOffsets& offs,
                            int32_t* d_idx, hipStream_t st);
hipError_t launch_gather(const void* x, int64_t sb, int64_t sn, int64_t sh, int32_t B, int32_t H,
                         int32_t N, int esize, int32_t w, int32_t r, const HeadOffsets& offs,
                         void* xg, hipStream_t st);
hipError_t launch_scatter(const void* og, int32_t B, int32_t H, int32_t N, int esize, int32_t w,
                          int32_t r, const HeadOffsets& offs, void* out, hipStream_t st);
hipError_t launch_merge(const float* out_b, const float* lse_b, int32_t nb, int32_t B, int32_t H,
                        int32_t N, bool out_bf16, void* out, float* lse, hipStream_t st);

}  // namespace dfa
