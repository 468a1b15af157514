// Device-side building blocks shared by the matrix-core kernels of the attention path (gfx950):
// direct global->LDS copies with hand-placed waits, the LDS swizzle, the walk over a tile's key
// lists, transposed fragment reads and the lane ^ 32 exchange.
#pragma once
#include "dfa_device.h"

namespace dfa {

constexpr int kRowElems = kD;              // LDS rows are the 128-byte rows of memory, unpadded
constexpr int kStageElems = kKeyTile * kRowElems;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

#define DFA_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define DFA_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

// The two lanes that share a query (lane and lane ^ 32, each with 16 of a block's 32 keys)
// combine their values.  v_permlane32_swap exchanges the upper half of its first operand with
// the lower half of its second; fed x twice it leaves x of the lower half in both halves of
// the first and x of the upper half in both halves of the second.  Written as inline assembly
// (with the idle states a vector write before it and a vector read after it need): the
// compiler's builtin hands back the first result for both.
__device__ __forceinline__ void wave_half_pair(float x, float& lo, float& hi) {
    lo = x;
    hi = x;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(lo), "+v"(hi));
}
__device__ __forceinline__ float wave_half_max(float x) {
    float lo, hi;
    wave_half_pair(x, lo, hi);
    return fmaxf(lo, hi);
}
__device__ __forceinline__ float wave_half_sum(float x) {
    float lo, hi;
    wave_half_pair(x, lo, hi);
    return lo + hi;
}

// 16-byte chunk swizzle of the K stage: chunk c of LDS row rho sits at chunk c ^ k_swizzle(rho).
// Sixteen consecutive rows then spread one chunk column over all 64 banks.
__device__ __forceinline__ int k_swizzle(int rho) { return (rho >> 1) & 7; }

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// Walks the 64-key steps of a tile's key list, progression after progression.
// All fields are wave-uniform and kept in scalar registers.
struct KeyCursor {
    int s, t;                  // progression index within the tile, 64-key step within the progression
    int key0, stride, count;   // the progression: keys key0 + stride * j, j < count
    float bias;                // log2 of the multiplicity of its keys, added to the base-2 scaled score
};

__device__ __forceinline__ void cursor_load(KeyCursor& c, const KeySeg* seg_lds) {
    c.key0 = __builtin_amdgcn_readfirstlane(seg_lds[c.s].key0);
    c.stride = __builtin_amdgcn_readfirstlane(seg_lds[c.s].stride);
    c.count = __builtin_amdgcn_readfirstlane(seg_lds[c.s].count);
    c.bias = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, seg_lds[c.s].log2_mult)));
}

__device__ __forceinline__ void cursor_next(KeyCursor& c, const KeySeg* seg_lds, int nseg) {
    if ((c.t + 1) * kKeyTile < c.count) {
        ++c.t;
    } else {
        c.t = 0;
        ++c.s;
        if (c.s < nseg) cursor_load(c, seg_lds);
    }
}

// 16 bytes per lane from global memory straight into LDS.  gbase and lds_addr are
// wave-uniform; lane L's bytes land at lds_addr + 16*L.  Issued as inline assembly so that the
// compiler's wait-count insertion does not see it: it would otherwise drain the vector-memory
// counter before every LDS read and serialise the copy pipeline.  The waits are placed by
// hand (wait_vmcnt) in the main loop.
__device__ __forceinline__ void copy16_to_lds(const void* gbase, uint32_t lane_byte_offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_byte_offset), "s"(gbase)
                 : "memory", "m0");
}

__device__ __forceinline__ const void* uniform_ptr(const void* p) {
    const uint64_t x = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}

// Transposed 8-element fragment out of a row-major, unswizzled 16-bit tile: within a 16-lane group
// lane i supplies the address of T[R + i/4][C + 4*(i%4) ..] and receives T[R .. R+3][C + i]; the
// second read continues four rows further down.
__device__ __forceinline__ bf16x8 read_v_frag(const uint16_t* vp) {
    const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DFA_LDS_PTR(short4v, vp));
    const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DFA_LDS_PTR(short4v, vp + 4 * kRowElems));
    const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, both);
}

}  // namespace dfa
