// Projections either side of the attention operator inside an encoder layer (the ViT
// self-attention block of section 3.1: a fused QKV projection before the operator, an output
// projection after it): y = x . w^T, bf16 operands on the gfx950 matrix cores, fp32
// accumulation, result rounded to bf16 (nearest even).
//
// One workgroup of 8 waves owns a 256 x BN tile of y (BN = 256 or 128) and walks K in steps
// of 64.  Both operand tiles have their K elements contiguous in memory (x rows and w rows),
// so both go global -> LDS as 128-byte rows (global_load_lds, 16 bytes per lane, no staging
// registers) into two alternating stages, with the 16-byte chunks of a row XOR-swizzled so
// that the fragment reads are free of bank conflicts, and both are read back as 16-byte MFMA
// fragments.  What limits the kernel is the byte rate of the CU's vector memory path (copies in,
// results out), so the tile is as large as LDS allows and the results leave as whole 128-byte
// lines.
//
// Matrix-core mapping (v_mfma_f32_16x16x32_bf16; lane = 16*g4 + r16): A operand = 16 weight rows (output
// features) x 32 k, B operand = 32 k x 16 x-rows, each lane supplying 8 consecutive k of row r16.  The result
// then has one x-row (one row of y) per lane and 4 consecutive output features in its 4 registers.  A wave
// computes 128 rows x BN/4 features: per 32 k it reads 8 + BN/64 fragments and issues 8 * BN/64 MFMAs.  (The
// 32x32x16 instruction does the same work in half as many issues but with twice the accumulator traffic
// per FLOP; under this part's power limit the 16x16x32 form is the faster one: 115 us against 123 us on the
// QKV projection of the stack workload.)
// Epilogue: each wave rounds its results to bf16, lays them out row-major in its own piece of
// LDS (the stages are free by then) and stores them 16 bytes per lane, eight lanes to a row.
#include "dfa_device.h"
#include "dfa_mfma.h"

namespace dfa {

namespace {

constexpr int kLinBM = 256;                // rows of y per workgroup
constexpr int kLinBK = 64;                 // k elements per stage: one 128-byte LDS row
constexpr int kLinStages = 2;

typedef float floatx4 __attribute__((ext_vector_type(4)));

// 16-byte chunk swizzle: chunk c of LDS row rho sits at chunk c ^ swizzle(rho).  Eight consecutive
// rows then spread one chunk column over all 64 banks (a fragment read takes row r16 of a 16-row block).
__device__ __forceinline__ int lin_swizzle(int rho) { return rho & 7; }

// The 256 x BN tile of y at (m0, n0): y[m][n] = sum_k x[m][k] * w[n][k].  lds: the workgroup's LDS (two stages
// of a 256-row x tile and a BN-row w tile).
template <int BN>
__device__ __forceinline__ void linear_tile(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                            uint16_t* __restrict__ y, int K, int64_t ldx, int64_t ldw, int64_t ldy,
                                            int64_t m0, int64_t n0, char* lds) {
    constexpr int NT = BN / 64;            // 16-feature blocks per wave
    constexpr uint32_t kXStageBytes = kLinBM * kLinBK * 2, kWStageBytes = BN * kLinBK * 2;
    constexpr uint32_t kXBytes = kLinStages * kXStageBytes;

    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;

    // ---- copies: a copy fills 8 rows of 128 bytes; lane L lands at row L/8, chunk L%8 and fetches
    // the source chunk that the swizzle puts there.  Wave `wave` fills x rows 32*wave .. +31
    // (4 copies) and w rows (BN/8)*wave .. (BN/64 copies: 4 + BN/64 per wave and stage); both starts are multiples of 8, so
    // the swizzle of row 8u + L/8 of a wave's share is L/8.
    const int r8 = lane >> 3;
    const int chunk = (lane & 7) ^ lin_swizzle(r8);
    const uint32_t x_off = (uint32_t)(r8 * ldx * 2 + 16 * chunk);      // byte offset of this lane inside an 8-row group
    const uint32_t w_off = (uint32_t)(r8 * ldw * 2 + 16 * chunk);
    const uint32_t lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &lds[0]);

    auto issue = [&](int ks, int stage) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int row = 32 * wave + 8 * u;
            copy16_to_lds(uniform_ptr(x + (m0 + row) * ldx + (int64_t)ks * kLinBK), x_off,
                       lds_addr + stage * kXStageBytes + row * 128);
        }
#pragma unroll
        for (int u = 0; u < BN / 64; ++u) {
            const int row = (BN / 8) * wave + 8 * u;
            copy16_to_lds(uniform_ptr(w + (n0 + row) * ldw + (int64_t)ks * kLinBK), w_off,
                       lds_addr + kXBytes + stage * kWStageBytes + row * 128);
        }
    };

    // ---- fragments: lane (j, g) reads row j of a 32-row block, chunk (2*kk + g) ^ swizzle(j)
    const int wm = wave >> 2, wn = wave & 3;
    const int frag = r16 * kLinBK + 8 * (g4 ^ lin_swizzle(r16));       // element offset for k half 0; half 1 xors 32 in
    const int x_rows = 128 * wm, w_rows = (BN / 4) * wn;               // first row of this wave in the two tiles

    floatx4 acc[NT][8];                    // [16-feature block][16-row block]: lane (g4, r16), register i = y[row r16][feature 4*g4 + i]
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_k = K / kLinBK;
    issue(0, 0);
    for (int ks = 0; ks < n_k; ++ks) {
        const int stage = ks & 1;
        wait_vmcnt<0>();       // this wave's share of stage ks has landed
        __syncthreads();           // everyone's has, and everyone is done reading the other stage
        if (ks + 1 < n_k) issue(ks + 1, stage ^ 1);
        const uint16_t* xs = reinterpret_cast<const uint16_t*>(lds + stage * kXStageBytes) + x_rows * kLinBK;
        const uint16_t* ws = reinterpret_cast<const uint16_t*>(lds + kXBytes + stage * kWStageBytes) + w_rows * kLinBK;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            bf16x8 wf[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                wf[nt] = *reinterpret_cast<const bf16x8*>(ws + 16 * nt * kLinBK + (frag ^ (32 * kh)));
#pragma unroll
            for (int mh = 0; mh < 2; ++mh) {
                bf16x8 xf[4];
#pragma unroll
                for (int m4 = 0; m4 < 4; ++m4)
                    xf[m4] = *reinterpret_cast<const bf16x8*>(xs + 16 * (4 * mh + m4) * kLinBK + (frag ^ (32 * kh)));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int m4 = 0; m4 < 4; ++m4)
                        acc[nt][4 * mh + m4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt], xf[m4], acc[nt][4 * mh + m4], 0, 0, 0);
            }
        }
    }

    // ---- epilogue.  Lane (g4, r16) holds row x_rows + 16*mt + r16 of the tile; its registers 0..3 of
    // block nt are features w_rows + 16*nt + 4*g4 .. +3.  Each wave transposes 64 rows at a time through
    // its own piece of LDS: rows of BN/4 features (64 or 128 bytes) at a pitch of 16 bytes more, written 8
    // bytes per lane, read back 16 bytes per lane with consecutive lanes along a row, and stored as whole
    // rows of the wave's tile.
    __syncthreads();               // every wave is done with the stages
    constexpr int kRowBytes = (BN / 4) * 2, kPitch = kRowBytes + 16, kLanesPerRow = kRowBytes / 16;
    constexpr int kRowsPerStore = 64 / kLanesPerRow;
    char* mine = lds + wave * (64 * kPitch);
    const int srow = lane / kLanesPerRow, schunk = lane % kLanesPerRow;
#pragma unroll
    for (int half = 0; half < 2; ++half) {
#pragma unroll
        for (int m4 = 0; m4 < 4; ++m4)
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const floatx4& a = acc[nt][4 * half + m4];
                const bf16x4 o = {(__bf16)a[0], (__bf16)a[1], (__bf16)a[2], (__bf16)a[3]};
                *reinterpret_cast<bf16x4*>(mine + (16 * m4 + r16) * kPitch + (16 * nt + 4 * g4) * 2) = o;
            }
        // the wave reads only what it wrote itself: LDS operations of a wave complete in order
#pragma unroll
        for (int s = 0; s < 64 / kRowsPerStore; ++s) {
            const int row = s * kRowsPerStore + srow;                      // row within this half
            const u32x4 v = *reinterpret_cast<const u32x4*>(mine + row * kPitch + 16 * schunk);
            uint16_t* dst = y + (m0 + x_rows + 64 * half + row) * ldy + n0 + w_rows + 8 * schunk;
            *reinterpret_cast<u32x4*>(dst) = v;
        }
    }
}

// ---- the resident form used by the projections -------------------------------------------------------------
// One workgroup per CU stays for the whole launch and works through its CU's tiles one after the other.  The
// tiles of a launch all cost the same, so the fixed round-robin deal below is also the balanced one, and a
// resident workgroup can do what a fresh one cannot: fetch the first k-step of its next tile while the last
// k-step of the current one is computed, so that neither the first trip to memory of a tile nor the write-out of
// the one before it leaves the CU's matrix cores idle.
// LDS: two stages of a 256-row x tile and a (up to) 256-row w tile, at fixed places whatever the width of the
// tile in hand, and a piece per wave for the write-out (16 rows at a time), apart from the stages because the
// next tile's first stage is already arriving while the results leave.
constexpr uint32_t kResXStage = kLinBM * kLinBK * 2;                 // 32 KB
constexpr uint32_t kResWStage = 256 * kLinBK * 2;                    // 32 KB (a 128-feature tile uses half)
constexpr uint32_t kResWBase = kLinStages * kResXStage;
constexpr uint32_t kResOutBase = kResWBase + kLinStages * kResWStage;
constexpr int kResOutPitch = 64 * 2 + 16;                            // a wave's 64 features of one row, padded
constexpr uint32_t kResLdsBytes = kResOutBase + 8 * 16 * kResOutPitch;

// One work item of a die's list: local index j < wide: the 256-feature tile j; beyond, the halves of the tiles
// after them (see launch_tiles).  Returns false past the end of the die's list.
struct ResItem {
    int64_t m0, n0;
    bool wide;
};
__device__ __forceinline__ bool res_item(int die, int j, int per_die, int wide_per_die, int tiles_m, int tiles_n, int bn,
                                         ResItem* it) {
    const bool whole = bn == 128 || j < wide_per_die;
    const int in_die = whole ? j : wide_per_die + (j - wide_per_die) / 2;
    const int t = die * per_die + in_die;
    if (in_die >= per_die || t >= tiles_m * tiles_n) return false;
    it->m0 = (int64_t)(t / tiles_n) * kLinBM;
    it->n0 = (int64_t)(t % tiles_n) * bn + (whole ? 0 : 128 * ((j - wide_per_die) & 1));
    it->wide = whole && bn == 256;
    return true;
}

// The copies of k-step ks of the tile at (m0, n0), `bn` features wide, into stage `stage`.
template <int BN>
__device__ __forceinline__ void res_issue(const uint16_t* x, const uint16_t* w, int64_t ldx, int64_t ldw, int64_t m0,
                                          int64_t n0, int ks, int stage, int wave, uint32_t x_off, uint32_t w_off,
                                          uint32_t lds_addr) {
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int row = 32 * wave + 8 * u;
        copy16_to_lds(uniform_ptr(x + (m0 + row) * ldx + (int64_t)ks * kLinBK), x_off, lds_addr + stage * kResXStage + row * 128);
    }
#pragma unroll
    for (int u = 0; u < BN / 64; ++u) {
        const int row = (BN / 8) * wave + 8 * u;
        copy16_to_lds(uniform_ptr(w + (n0 + row) * ldw + (int64_t)ks * kLinBK), w_off, lds_addr + kResWBase + stage * kResWStage + row * 128);
    }
}

// All k-steps and the write-out of one tile whose first k-step is already on its way into stage `stage`
// (updated to the stage the next tile starts in).  `next`: the tile to prefetch during the last k-step, if any.
template <int BN>
__device__ __forceinline__ void res_tile(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w,
                                         uint16_t* __restrict__ y, int K, int64_t ldx, int64_t ldw, int64_t ldy,
                                         const ResItem& cur, bool have_next, const ResItem& next, int& stage, char* lds) {
    constexpr int NT = BN / 64;            // 16-feature blocks per wave
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, r16 = lane & 15, g4 = lane >> 4;
    const int r8 = lane >> 3;
    const int chunk = (lane & 7) ^ lin_swizzle(r8);
    const uint32_t x_off = (uint32_t)(r8 * ldx * 2 + 16 * chunk);
    const uint32_t w_off = (uint32_t)(r8 * ldw * 2 + 16 * chunk);
    const uint32_t lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &lds[0]);
    const int wm = wave >> 2, wn = wave & 3;
    const int frag = r16 * kLinBK + 8 * (g4 ^ lin_swizzle(r16));
    const int x_rows = 128 * wm, w_rows = (BN / 4) * wn;

    floatx4 acc[NT][8];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt)
#pragma unroll
        for (int mt = 0; mt < 8; ++mt) acc[nt][mt] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int n_k = K / kLinBK;
    for (int ks = 0; ks < n_k; ++ks) {
        wait_vmcnt<0>();           // this wave's share of stage ks has landed (and the stores of the tile before have left)
        __syncthreads();           // everyone's has, and everyone is done reading the other stage
        if (ks + 1 < n_k) {
            res_issue<BN>(x, w, ldx, ldw, cur.m0, cur.n0, ks + 1, stage ^ 1, wave, x_off, w_off, lds_addr);
        } else if (have_next) {    // the next tile's first k-step, under this tile's last one and its write-out
            if (next.wide) res_issue<256>(x, w, ldx, ldw, next.m0, next.n0, 0, stage ^ 1, wave, x_off, w_off, lds_addr);
            else res_issue<128>(x, w, ldx, ldw, next.m0, next.n0, 0, stage ^ 1, wave, x_off, w_off, lds_addr);
        }
        const uint16_t* xs = reinterpret_cast<const uint16_t*>(lds + stage * kResXStage) + x_rows * kLinBK;
        const uint16_t* ws = reinterpret_cast<const uint16_t*>(lds + kResWBase + stage * kResWStage) + w_rows * kLinBK;
#pragma unroll
        for (int kh = 0; kh < 2; ++kh) {
            bf16x8 wf[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
                wf[nt] = *reinterpret_cast<const bf16x8*>(ws + 16 * nt * kLinBK + (frag ^ (32 * kh)));
#pragma unroll
            for (int mh = 0; mh < 2; ++mh) {
                bf16x8 xf[4];
#pragma unroll
                for (int m4 = 0; m4 < 4; ++m4)
                    xf[m4] = *reinterpret_cast<const bf16x8*>(xs + 16 * (4 * mh + m4) * kLinBK + (frag ^ (32 * kh)));
#pragma unroll
                for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                    for (int m4 = 0; m4 < 4; ++m4)
                        acc[nt][4 * mh + m4] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(wf[nt], xf[m4], acc[nt][4 * mh + m4], 0, 0, 0);
            }
        }
        stage ^= 1;
    }

    // ---- write-out, 16 rows of the wave's tile at a time through the wave's own piece of LDS: lane (g4, r16) holds
    // row 16*mt + r16, features 16*nt + 4*g4 .. +3; written 8 bytes per lane, read back 16 bytes per lane with
    // consecutive lanes along a row, stored as whole rows of the wave's tile.  No barrier: the piece belongs to
    // this wave alone, and LDS operations of a wave complete in order.
    constexpr int kRowBytes = (BN / 4) * 2, kLanesPerRow = kRowBytes / 16, kRowsPerStore = 64 / kLanesPerRow;
    char* mine = lds + kResOutBase + wave * (16 * kResOutPitch);
    const int srow = lane / kLanesPerRow, schunk = lane % kLanesPerRow;
#pragma unroll
    for (int mt = 0; mt < 8; ++mt) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) {
            const floatx4& a = acc[nt][mt];
            const bf16x4 o = {(__bf16)a[0], (__bf16)a[1], (__bf16)a[2], (__bf16)a[3]};
            *reinterpret_cast<bf16x4*>(mine + r16 * kResOutPitch + (16 * nt + 4 * g4) * 2) = o;
        }
#pragma unroll
        for (int s = 0; s < (16 + kRowsPerStore - 1) / kRowsPerStore; ++s) {
            const int row = s * kRowsPerStore + srow;                      // row within these 16
            if (kRowsPerStore <= 16 || row < 16) {
                const u32x4 v = *reinterpret_cast<const u32x4*>(mine + row * kResOutPitch + 16 * schunk);
                uint16_t* dst = y + (cur.m0 + x_rows + 16 * mt + row) * ldy + cur.n0 + w_rows + 8 * schunk;
                *reinterpret_cast<u32x4*>(dst) = v;
            }
        }
    }
}

// Requires M % 256 == 0, N % BN == 0, K % 64 == 0, every row of x, w and y starting on a 16-byte boundary.
// Workgroup i stays on CU (i / dies) of die i % dies; tiles (256 x BN) are numbered band by band and dealt so that one
// die walks all feature tiles of a row band before moving on (the x band is then read from memory once per die, w stays
// in its L2), the CUs of a die taking them round-robin.  When the last round of a die would be at most half full
// (wide tiles only), its tiles are cut into two 128-feature halves, which fill the die for a round half as long: the
// first `wide_per_die` items of a die are whole tiles, the others halves.
template <int BN>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void linear_bf16_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, uint16_t* __restrict__ y,
                        int K, int64_t ldx, int64_t ldw, int64_t ldy, int tiles_m, int tiles_n, int wide_per_die, int dies,
                        int cus_per_die) {
    __shared__ __attribute__((aligned(1024))) char lds[kResLdsBytes];
    const int die = blockIdx.x % dies, cu = blockIdx.x / dies;
    const int per_die = (tiles_m * tiles_n + dies - 1) / dies;
    ResItem cur, next;
    int j = cu;
    if (!res_item(die, j, per_die, wide_per_die, tiles_m, tiles_n, BN, &cur)) return;
    // the first tile's first k-step
    {
        const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6), lane = threadIdx.x & 63, r8 = lane >> 3;
        const int chunk = (lane & 7) ^ lin_swizzle(r8);
        const uint32_t x_off = (uint32_t)(r8 * ldx * 2 + 16 * chunk), w_off = (uint32_t)(r8 * ldw * 2 + 16 * chunk);
        const uint32_t lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &lds[0]);
        if (cur.wide) res_issue<256>(x, w, ldx, ldw, cur.m0, cur.n0, 0, 0, wave, x_off, w_off, lds_addr);
        else res_issue<128>(x, w, ldx, ldw, cur.m0, cur.n0, 0, 0, wave, x_off, w_off, lds_addr);
    }
    int stage = 0;
    for (;;) {                     // ends: j grows by cus_per_die >= 1 every trip, res_item fails past the die's list
        j += cus_per_die;
        const bool have_next = res_item(die, j, per_die, wide_per_die, tiles_m, tiles_n, BN, &next);
        if (cur.wide) res_tile<256>(x, w, y, K, ldx, ldw, ldy, cur, have_next, next, stage, lds);
        else res_tile<128>(x, w, y, K, ldx, ldw, ldy, cur, have_next, next, stage, lds);
        if (!have_next) break;
        cur = next;
    }
}

// A batch of independent products of one shape: workgroup (t, z) computes tile t of matrix z = z0 * batch_inner + z1,
// whose operands start at x + z0 * xs0 + z1 * xs1 (elements), and likewise for w and y.  Plain tile order.
template <int BN>
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void linear_bf16_batched_kernel(const uint16_t* __restrict__ x, const uint16_t* __restrict__ w, uint16_t* __restrict__ y,
                                int K, int64_t ldx, int64_t ldw, int64_t ldy, int tiles_n, int batch_inner,
                                int64_t xs0, int64_t xs1, int64_t ws0, int64_t ws1, int64_t ys0, int64_t ys1) {
    __shared__ __attribute__((aligned(1024))) char lds[kLinStages * (kLinBM + BN) * kLinBK * 2];
    const int z0 = blockIdx.y / batch_inner, z1 = blockIdx.y % batch_inner;
    const int64_t m0 = (int64_t)(blockIdx.x / tiles_n) * kLinBM, n0 = (int64_t)(blockIdx.x % tiles_n) * BN;
    linear_tile<BN>(x + z0 * xs0 + z1 * xs1, w + z0 * ws0 + z1 * ws1, y + z0 * ys0 + z1 * ys1, K, ldx, ldw, ldy, m0, n0, lds);
}

template <int BN>
hipError_t launch_tiles(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                        int64_t ldx, int64_t ldw, int64_t ldy, const ChipShape& chip, hipStream_t st) {
    const int dies = chip.dies > 0 ? chip.dies : 1, cus_per_die = chip.cus / dies > 0 ? chip.cus / dies : 1;
    const int tiles_m = (int)(M / kLinBM), tiles_n = N / BN;
    const int per_die = (tiles_m * tiles_n + dies - 1) / dies;
    // wide tiles: whole rounds of a die's CUs as they are, a last round that is at most half full in halves
    const int rem = per_die % cus_per_die;
    const int wide_per_die = (BN == 256 && rem > 0 && 2 * rem <= cus_per_die) ? per_die - rem : per_die;
    const int items_per_die = wide_per_die + 2 * (per_die - wide_per_die);
    const int wg_per_die = items_per_die < cus_per_die ? items_per_die : cus_per_die;      // one resident workgroup per CU
    hipLaunchKernelGGL((linear_bf16_kernel<BN>), dim3(wg_per_die * dies), dim3(512), 0, st,
                       static_cast<const uint16_t*>(x), static_cast<const uint16_t*>(w), static_cast<uint16_t*>(y),
                       K, ldx, ldw, ldy, tiles_m, tiles_n, wide_per_die, dies, cus_per_die);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_linear_bf16(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                              int64_t ldx, int64_t ldw, int64_t ldy, const ChipShape& chip, hipStream_t st) {
    // One workgroup per CU at a time.  The 256-feature tile moves fewer bytes per flop; the 128-feature
    // tile is taken when the last round of wide tiles would leave too much of the chip idle.
    bool wide = N % 256 == 0;
    if (wide) {
        const int64_t cus = chip.cus > 0 ? chip.cus : 1;
        const int64_t tiles = (M / kLinBM) * (N / 256), rounds = (tiles + cus - 1) / cus;
        wide = tiles * 10 >= rounds * cus * 8;
    }
    return wide ? launch_tiles<256>(x, w, y, M, N, K, ldx, ldw, ldy, chip, st)
                : launch_tiles<128>(x, w, y, M, N, K, ldx, ldw, ldy, chip, st);
}

hipError_t launch_linear_bf16_batched(const void* x, const void* w, void* y, int64_t M, int32_t N, int32_t K,
                                      int64_t ldx, int64_t ldw, int64_t ldy, int32_t batch_outer, int32_t batch_inner,
                                      int64_t xs0, int64_t xs1, int64_t ws0, int64_t ws1, int64_t ys0, int64_t ys1,
                                      hipStream_t st) {
    const uint16_t* xp = static_cast<const uint16_t*>(x);
    const uint16_t* wp = static_cast<const uint16_t*>(w);
    uint16_t* yp = static_cast<uint16_t*>(y);
    const dim3 block(512);
    if (N % 256 == 0) {
        const dim3 grid((unsigned)((M / kLinBM) * (N / 256)), (unsigned)(batch_outer * batch_inner));
        hipLaunchKernelGGL((linear_bf16_batched_kernel<256>), grid, block, 0, st, xp, wp, yp, K, ldx, ldw, ldy, N / 256,
                           batch_inner, xs0, xs1, ws0, ws1, ys0, ys1);
    } else if (N % 128 == 0) {
        const dim3 grid((unsigned)((M / kLinBM) * (N / 128)), (unsigned)(batch_outer * batch_inner));
        hipLaunchKernelGGL((linear_bf16_batched_kernel<128>), grid, block, 0, st, xp, wp, yp, K, ldx, ldw, ldy, N / 128,
                           batch_inner, xs0, xs1, ws0, ws1, ys0, ys1);
    } else {
        const dim3 grid((unsigned)((M / kLinBM) * (N / 64)), (unsigned)(batch_outer * batch_inner));
        hipLaunchKernelGGL((linear_bf16_batched_kernel<64>), grid, block, 0, st, xp, wp, yp, K, ldx, ldw, ldy, N / 64,
                           batch_inner, xs0, xs1, ws0, ws1, ys0, ys1);
    }
    return hipGetLastError();
}

}  // namespace dfa
