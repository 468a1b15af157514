// Projections either side of the attention operator inside an encoder layer (the ViT
// self-attention block of section 3.1: a fused QKV projection before the operator, an output
// projection after it): y = x . w^T, bf16 operands on the gfx950 matrix cores, fp32
// accumulation, result rounded to bf16 (nearest even).
//
// One workgroup of 4 waves owns a BM x BN tile of y (256 x 128, or 128 x 128 when that fills
// the chip more evenly) and walks K in steps of 32.  Both operand tiles have their K elements
// contiguous in memory (x rows and w rows), so both go global -> LDS as 64-byte rows
// (global_load_lds, 16 bytes per lane, no staging registers) into a ring of three stages, two
// in flight while the third is consumed, with the 16-byte chunks of a row XOR-swizzled so that
// the fragment reads are free of bank conflicts, and both are read back as 16-byte MFMA
// fragments.  Two workgroups share a CU (72 KB of LDS each), so that one's epilogue (the
// stores of its tile, a quarter of the launch if nothing overlaps them) runs under the other's
// matrix work.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16): A operand = 32 weight rows (output
// features) x 16 k, B operand = 16 k x 32 x-rows.  The result then has one x-row (one row of
// y) per lane and 4 consecutive output features in 4 consecutive registers, which the
// epilogue stores as 8-byte pieces.  A wave computes BM/2 rows x BN/2 features.
#include "dfa_device.h"

namespace dfa {

namespace {

constexpr int kLinBK = 32;                 // k elements per stage: one 64-byte LDS row
constexpr int kLinStages = 3;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

#define DFA_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))

// 16-byte chunk swizzle: chunk c (0..3) of LDS row rho sits at chunk c ^ swizzle(rho).  Sixteen
// consecutive rows then spread one chunk column over all 64 banks.
__device__ __forceinline__ int lin_swizzle(int rho) { return (rho >> 2) & 3; }

template <int N>
__device__ __forceinline__ void lin_wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// 16 bytes per lane from global memory straight into LDS: lane L's bytes land at lds_addr +
// 16*L.  gbase and lds_addr are wave-uniform.  Inline assembly, so that the compiler's
// wait-count insertion does not see the copy and drain it before every LDS read; the waits are
// placed by hand.
__device__ __forceinline__ void lin_copy16(const void* gbase, uint32_t lane_byte_offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_byte_offset), "s"(gbase)
                 : "memory", "m0");
}

__device__ __forceinline__ const void* lin_uniform_ptr(const void* p) {
    const uint64_t x = reinterpret_cast<uint64_t>(p);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)x);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(x >> 32));
    return reinterpret_cast<const void*>(((uint64_t)hi << 32) | lo);
}

// y[m][n] = sum_k x[m][k] * w[n][k].  Requires M % BM == 0, N % BN == 0, K % 32 == 0, every
// row of x, w and y starting on a 16-byte boundary.  grid = (M/BM) * (N/BN) workgroups,
// workgroup i on die i % 8; tiles are dealt so that one die walks all feature tiles of a row
// band before moving on (the x band is then read from memory once per die, w stays in its L2).
template <int BM, int BN>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void linear_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, uint16_t* __restrict__ y,
                        int K, int64_t ldx, int64_t ldw, int64_t ldy, int tiles_m, int tiles_n) {
    constexpr int MB = BM / 64, NB = BN / 64;          // 32-row / 32-feature blocks per wave
    __shared__ __attribute__((aligned(1024))) uint16_t x_lds[kLinStages][BM * kLinBK];
    __shared__ __attribute__((aligned(1024))) uint16_t w_lds[kLinStages][BN * kLinBK];

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, j = lane & 31, g = lane >> 5;

    // tile of this workgroup
    const int die = blockIdx.x % kNumXcd, local = blockIdx.x / kNumXcd;
    const int per_die = (tiles_m * tiles_n + kNumXcd - 1) / kNumXcd;   // tiles are numbered band by band
    const int t = die * per_die + local;
    if (t >= tiles_m * tiles_n) return;
    const int tm = t / tiles_n, tn = t % tiles_n;
    const int64_t m0 = (int64_t)tm * BM, n0 = (int64_t)tn * BN;

    // ---- copies: a copy fills 16 rows of 64 bytes; lane L lands at row L/4, chunk L%4 and fetches
    // the source chunk that the swizzle puts there (the swizzle only sees L/4: copies start on
    // multiples of 16 rows).  Wave `wave` fills x rows (BM/4)*wave .. and w rows (BN/4)*wave .. .
    constexpr int kXCopies = BM / 64, kWCopies = BN / 64, kCopies = kXCopies + kWCopies;   // per wave per stage
    const int r16 = lane >> 2;
    const int src_chunk = (lane & 3) ^ lin_swizzle(r16);
    const uint32_t x_off = (uint32_t)(r16 * ldx * 2 + 16 * src_chunk);
    const uint32_t w_off = (uint32_t)(r16 * ldw * 2 + 16 * src_chunk);
    const uint32_t x_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &x_lds[0][0]);
    const uint32_t w_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &w_lds[0][0]);
    constexpr uint32_t kXStageBytes = BM * kLinBK * 2, kWStageBytes = BN * kLinBK * 2;

    auto issue = [&](int ks, int stage) {
#pragma unroll
        for (int u = 0; u < kXCopies; ++u) {
            const int row = (BM / 4) * wave + 16 * u;
            lin_copy16(lin_uniform_ptr(x + (m0 + row) * ldx + (int64_t)ks * kLinBK), x_off,
                       x_lds_addr + stage * kXStageBytes + row * 64);
        }
#pragma unroll
        for (int u = 0; u < kWCopies; ++u) {
            const int row = (BN / 4) * wave + 16 * u;
            lin_copy16(lin_uniform_ptr(w + (n0 + row) * ldw + (int64_t)ks * kLinBK), w_off,
                       w_lds_addr + stage * kWStageBytes + row * 64);
        }
    };

    // ---- fragments: lane (j, g) reads row j of a 32-row block, chunk (2*kk + g) ^ swizzle(j)
    const int wm = wave >> 1, wn = wave & 1;
    const int frag = j * kLinBK + 8 * (g ^ lin_swizzle(j));            // element offset for kk = 0; kk = 1 xors 16 in
    const int x_rows = (BM / 2) * wm, w_rows = (BN / 2) * wn;          // first row of this wave in the two tiles

    floatx16 acc[NB][MB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[nb][mb][v] = 0.f;

    const int n_k = K / kLinBK;
#pragma unroll
    for (int ks = 0; ks < kLinStages - 1; ++ks)
        if (ks < n_k) issue(ks, ks);
    int stage = 0;
    for (int ks = 0; ks < n_k; ++ks) {
        // this wave's share of stage ks has landed once only the copies of the next stage are outstanding
        if (ks + 1 < n_k) lin_wait_vmcnt<kCopies>(); else lin_wait_vmcnt<0>();
        __syncthreads();           // everyone's has, and everyone is done reading the stage consumed last
        if (ks + kLinStages - 1 < n_k) issue(ks + kLinStages - 1, stage == 0 ? kLinStages - 1 : stage - 1);
        const uint16_t* xs = x_lds[stage] + x_rows * kLinBK;
        const uint16_t* ws = w_lds[stage] + w_rows * kLinBK;
#pragma unroll
        for (int kk = 0; kk < 2; ++kk) {
            bf16x8 xf[MB], wf[NB];
#pragma unroll
            for (int mb = 0; mb < MB; ++mb)
                xf[mb] = *reinterpret_cast<const bf16x8*>(xs + 32 * mb * kLinBK + (frag ^ (16 * kk)));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
                wf[nb] = *reinterpret_cast<const bf16x8*>(ws + 32 * nb * kLinBK + (frag ^ (16 * kk)));
#pragma unroll
            for (int nb = 0; nb < NB; ++nb)
#pragma unroll
                for (int mb = 0; mb < MB; ++mb)
                    acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(wf[nb], xf[mb], acc[nb][mb], 0, 0, 0);
        }
        stage = stage == kLinStages - 1 ? 0 : stage + 1;
    }

    // ---- epilogue: lane (j, g) holds row m0 + x_rows + 32*mb + j; registers 4*vq .. 4*vq+3 are
    // features n0 + w_rows + 32*nb + 8*vq + 4*g .. +3
#pragma unroll
    for (int mb = 0; mb < MB; ++mb) {
        uint16_t* yrow = y + (m0 + x_rows + 32 * mb + j) * ldy + n0 + w_rows + 4 * g;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
                const bf16x4 o = {(__bf16)acc[nb][mb][4 * vq], (__bf16)acc[nb][mb][4 * vq + 1],
                                  (__bf16)acc[nb][mb][4 * vq + 2], (__bf16)acc[nb][mb][4 * vq + 3]};
                *reinterpret_cast<bf16x4*>(yrow + 32 * nb + 8 * vq) = o;
            }
    }
}

template <int BM, int BN>
hipError_t launch_tiles(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                        int64_t ldx, int64_t ldw, int64_t ldy, hipStream_t st) {
    const int tiles_m = (int)(M / BM), tiles_n = N / BN;
    const int per_die = (tiles_m * tiles_n + kNumXcd - 1) / kNumXcd;
    hipLaunchKernelGGL((linear_bf16_kernel<BM, BN>), dim3(per_die * kNumXcd), dim3(256), 0, st,
                       static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w), static_cast<uint16_t*>(y),
                       K, ldx, ldw, ldy, tiles_m, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                              int64_t ldx, int64_t ldw, int64_t ldy, hipStream_t st) {
    // 512 workgroups run at a time (2 per CU).  The 256-row tile moves fewer bytes per flop; the
    // 128-row tile is taken when the last round of 256-row tiles would leave too much of the chip idle.
    const int64_t big = (M / 256) * (N / 128);
    const int64_t rounds = (big + 511) / 512;
    const bool small_tiles = M % 256 != 0 || big * 10 < rounds * 512 * 8;
    return small_tiles ? launch_tiles<128, 128>(x, w, y, M, N, K, ldx, ldw, ldy, st)
                       : launch_tiles<256, 128>(x, w, y, M, N, K, ldx, ldw, ldy, st);
}

}  // namespace dfa
