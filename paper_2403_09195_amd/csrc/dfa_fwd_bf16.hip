// Fused dilated flash attention forward, bf16 on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns a tile of up to 256 query rows that share the same key lists
// (section 3.1: all of them are kept by the same branches and fall into the same segment of
// each).  It walks the key lists of its member branches one after the other, 64 keys at a
// time, carrying ONE online-softmax state (reference exponent, running sum, accumulator) per
// query row across all of them: continuing the softmax over the next branch's keys is the
// log-sum-exp merge of the branches, so no partial result ever leaves the registers.
//
// Gather (Eq. 1) happens in the global->LDS copies (key j of a segment is row first + r*j),
// placement (Eq. 3) in the final store (each query row is written back at its own token).
//
// Data movement: K and V rows go from global memory straight into LDS (global_load_lds, 16
// bytes per lane, no staging registers), three 64-key stages deep, so a copy has two full
// compute steps to land.  Each wave-level copy fills 1 KB = 8 rows of 128 bytes; which
// global row and 16-byte chunk a lane fetches is free, which is how the row permutation and
// the bank swizzle below are applied.
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, wave64; lane = 32*g + j):
//   S^T = K~ Q~^T : A = K rows (32 keys x 16 d), B = Q^T (16 d x 32 queries).  The result puts
//                   query j in lane j: register v of lane (j, g) is key row 8*(v/4)+4*g+v%4,
//                   so row statistics are 16 in-lane values plus one exchange with lane^32.
//   O^T += V~^T P^T: A = V^T (32 d x 16 keys), B = P^T (16 keys x 32 queries).  B wants 8
//                   consecutive contraction slots per lane; the S^T registers 8*st .. 8*st+7
//                   of a lane serve directly, which fixes which key sits in which slot: MFMA row
//                   i of the first product is contraction slot sigma(i) of the second (sigma swaps
//                   bits 2 and 3).  K is therefore kept in LDS with the key of tile position p in
//                   row sigma(p); V stays in position order, row-major as in memory, and its
//                   transposed operand is fetched with ds_read_b64_tr_b16 (4 keys x 16 d per
//                   16-lane group, delivered key-contiguous per lane).
// Each wave handles 64 query rows (two 32-row blocks), so every K / V^T fragment read from
// LDS feeds two MFMAs.
#include "dfa_device.h"

namespace dfa {

namespace {

constexpr int kStages = 3;                 // 64-key K/V stages in flight
constexpr int kRowElems = kD;              // LDS rows are the 128-byte rows of memory, unpadded
constexpr int kStageElems = kKeyTile * kRowElems;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef short short8v __attribute__((ext_vector_type(8)));

#define DFA_LDS_PTR(T, p) ((__attribute__((address_space(3))) T*)(p))
#define DFA_GLOBAL_PTR(p) ((const __attribute__((address_space(1))) void*)(p))

__device__ __forceinline__ float wave_half_xchg(float x) {
    // value held by the lane that owns the other 16 keys of the same query (lane ^ 32)
    return __shfl_xor(x, 32, 64);
}

// 16-byte chunk swizzle of the K stage: chunk c of LDS row rho sits at chunk c ^ k_swizzle(rho).
// Sixteen consecutive rows then spread one chunk column over all 64 banks.
__device__ __forceinline__ int k_swizzle(int rho) { return (rho >> 1) & 7; }

// s_waitcnt on the vector-memory counter only (gfx9 encoding: vmcnt in bits 3:0 and 15:14).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

// Walks the 64-key steps of a tile's key lists: segment after segment (one per member branch).
// All fields are wave-uniform and kept in scalar registers.
struct KeyCursor {
    int s, t;                  // segment index within the tile, 64-key step within the segment
    int key0, stride, count;   // the segment: kept keys are key0 + stride * j, j < count
};

__device__ __forceinline__ void cursor_load(KeyCursor& c, const KeySeg* seg_lds) {
    c.key0 = __builtin_amdgcn_readfirstlane(seg_lds[c.s].key0);
    c.stride = __builtin_amdgcn_readfirstlane(seg_lds[c.s].stride);
    c.count = __builtin_amdgcn_readfirstlane(seg_lds[c.s].count);
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

// Per-lane constants of the global->LDS copies.  A wave issues 2 K copies and 2 V copies per
// step; copy u of wave w fills LDS rows 8*(2w+u) .. +7, lane L lands at row L/8, chunk L%8.
struct CopyLane {
    int kpos[2];       // tile position of the key whose row this lane fetches (K copies)
    int kchunk[2];     // byte offset of the 16-byte chunk of that row
    int vpos[2];       // same for V (position order, chunks in place)
    int vchunk;
};

__device__ __forceinline__ void issue_stage(const FwdParams& p, const uint16_t* kp, const uint16_t* vp,
                                            const KeyCursor& c, const CopyLane& cl, int wave,
                                            uint32_t k_stage, uint32_t v_stage) {
    const int j0 = c.t * kKeyTile;
    const int room = c.count - 1 - j0;       // keys past the end of the list re-read the last one
    // uniform base: first key of this step; per-lane offsets stay below 64 * stride * row pitch
    const int64_t first = kept_row(c.key0, c.stride, j0);
    const void* kb = uniform_ptr(kp + first * p.skn);
    const void* vb = uniform_ptr(vp + first * p.svn);
    const uint32_t kpitch = (uint32_t)(c.stride * p.skn * 2);
    const uint32_t vpitch = (uint32_t)(c.stride * p.svn * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const uint32_t blk = (uint32_t)(2 * wave + u) * 1024u;
        copy16_to_lds(kb, (uint32_t)min(cl.kpos[u], room) * kpitch + cl.kchunk[u], k_stage + blk);
        copy16_to_lds(vb, (uint32_t)min(cl.vpos[u], room) * vpitch + cl.vchunk, v_stage + blk);
    }
}

// If a lane's partial row sum of one 32-key block exceeds this, some exponent may have left
// the comfortable range and the reference exponent is moved up (see rebase_block).
constexpr float kRebaseThreshold = 256.0f;

// Softmax numerators of one 32-key block against the current reference exponents m_ref (no
// row maximum is taken here): p = exp2(c*s - m_ref), rounded to bf16 (nearest even) and packed
// straight into the B operands of the second product.  psum = this lane's share of the row
// sums, taken over the rounded values with a packed dot product.
__device__ __forceinline__ void exp_block(const floatx16 (&s)[2], float c, const float (&m_ref)[2],
                                          u32x4 (&pb)[2][2], float (&psum)[2]) {
    const bf16x2 ones = {(__bf16)1.0f, (__bf16)1.0f};
    // Written stage by stage (all exponents, then all exponentials, then all conversions) and
    // with four independent partial sums: a vector instruction that needs the result of the one
    // just before it stalls the wave, so dependent instructions are kept far apart.
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float t[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) t[v] = fmaf(s[qb][v], c, -m_ref[qb]);
#pragma unroll
        for (int v = 0; v < 16; ++v) t[v] = __builtin_amdgcn_exp2f(t[v]);
        bf16x2 pr[8];
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            pr[v] = bf16x2{(__bf16)t[2 * v], (__bf16)t[2 * v + 1]};
            pb[qb][v >> 2][v & 3] = __builtin_bit_cast(uint32_t, pr[v]);   // slots 2v%8, 2v%8+1 of step v/4
        }
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        a0 = __builtin_amdgcn_fdot2_f32_bf16(pr[0], ones, a0, false);
        a1 = __builtin_amdgcn_fdot2_f32_bf16(pr[1], ones, a1, false);
        a2 = __builtin_amdgcn_fdot2_f32_bf16(pr[2], ones, a2, false);
        a3 = __builtin_amdgcn_fdot2_f32_bf16(pr[3], ones, a3, false);
        a0 = __builtin_amdgcn_fdot2_f32_bf16(pr[4], ones, a0, false);
        a1 = __builtin_amdgcn_fdot2_f32_bf16(pr[5], ones, a1, false);
        a2 = __builtin_amdgcn_fdot2_f32_bf16(pr[6], ones, a2, false);
        a3 = __builtin_amdgcn_fdot2_f32_bf16(pr[7], ones, a3, false);
        psum[qb] = (a0 + a1) + (a2 + a3);
    }
}

// Rare path of the online softmax: take the exact row maximum of this block, move the
// reference exponent up to it, rescale the running sum and the accumulator.
__device__ __forceinline__ void rebase_block(const floatx16 (&s)[2], float c, float (&m_ref)[2],
                                             float (&l_run)[2], floatx16 (&oacc)[2][2]) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float mx = s[qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[qb][v]);
        mx = fmaxf(mx, wave_half_xchg(mx));
        const float m_new = fmaxf(m_ref[qb], mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m_ref[qb] - m_new);   // exp2(-inf) = 0 at the start
        m_ref[qb] = m_new;
        l_run[qb] *= alpha;
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= alpha;
    }
}

// One 64-key step: S^T, softmax numerators, O^T accumulation, in two 32-key blocks.  The
// scheduling fences keep the phases apart so that at most two score blocks, two packed
// probability blocks and one set of LDS fragments are alive at a time (256 registers per lane
// are all there is at two waves per SIMD); inside a phase the matrix cores work on one block
// while the vector ALU exponentiates the other.
__device__ __forceinline__ void tile_step(const uint16_t* kl, const uint16_t* vl, const bf16x8 (&qf)[2][4],
                                          int lane, int nvalid, float c, float (&m_ref)[2],
                                          float (&l_run)[2], floatx16 (&oacc)[2][2]) {
    const int j = lane & 31, g = lane >> 5;
    floatx16 sacc[2][2];                   // [key block][query block]
    u32x4 pb[2][2][2];                     // [key block][query block][16-key step], bf16 pairs

    auto scores = [&](int ks) {
        const int rho = 32 * ks + j;
        const uint16_t* krow = kl + rho * kRowElems;
        const int swz = k_swizzle(rho);
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(krow + 8 * ((2 * kk + g) ^ swz));
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                if (kk == 0) {
                    floatx16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.f;
                    sacc[ks][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][kk], z, 0, 0, 0);
                } else {
                    sacc[ks][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][kk], sacc[ks][qb], 0, 0, 0);
                }
            }
        }
    };
    auto mask_tail = [&](int ks) {
        // end of a key list: register v of lane (j, g) is tile position 32*ks + 16*(v/8) + 8*g + v%8
        asm volatile("" ::: "memory");     // keeps this a branch: full steps must not pay for the selects
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int pos = 32 * ks + 16 * (v >> 3) + 8 * g + (v & 7);
            if (pos >= nvalid) {
                sacc[ks][0][v] = -INFINITY;
                sacc[ks][1][v] = -INFINITY;
            }
        }
    };
    auto numerators = [&](int ks) {
        float psum[2];
        for (int attempt = 0;; ++attempt) {
            exp_block(sacc[ks], c, m_ref, pb[ks], psum);
            // wave-uniform test; written so that NaN (-inf - -inf before the first rebase) trips it
            const bool calm = psum[0] <= kRebaseThreshold && psum[1] <= kRebaseThreshold;
            // one rebase always suffices for finite inputs (every p of the block is <= 1 after it);
            // the bound keeps the loop finite when the inputs hold NaN or infinities
            if (__builtin_expect(__ballot(!calm) == 0ull, 1) || attempt == 1) break;
            rebase_block(sacc[ks], c, m_ref, l_run, oacc);
        }
        l_run[0] += psum[0];
        l_run[1] += psum[1];
    };
    // transposed V fragments: within a 16-lane group lane i supplies the address of
    // V[R + i/4][C + 4*(i%4) ..] and receives V[R .. R+3][C + i]
    const int i16 = lane & 15;
    const uint16_t* vbase = vl + ((i16 >> 2) + 8 * g) * kRowElems + 16 * ((lane >> 4) & 1) + 4 * (i16 & 3);
    auto accumulate = [&](int ks) {
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int st = 0; st < 2; ++st) {
                const uint16_t* vp = vbase + (32 * ks + 16 * st) * kRowElems + 32 * db;
                const short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DFA_LDS_PTR(short4v, vp));
                const short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(DFA_LDS_PTR(short4v, vp + 4 * kRowElems));
                const short8v both = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, both);
#pragma unroll
                for (int qb = 0; qb < 2; ++qb)
                    oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pb[ks][qb][st]), oacc[db][qb], 0, 0, 0);
            }
    };

    scores(0);
    if (nvalid < kKeyTile) mask_tail(0);
    __builtin_amdgcn_sched_barrier(0);
    scores(1);                             // matrix cores: block 1 scores | vector ALU: block 0 exponentials
    if (nvalid < kKeyTile) mask_tail(1);
    numerators(0);
    __builtin_amdgcn_sched_barrier(0);
    accumulate(0);                         // matrix cores: block 0 second product | vector ALU: block 1 exponentials
    numerators(1);
    __builtin_amdgcn_sched_barrier(0);
    accumulate(1);
}

template <typename OutT>
__device__ __forceinline__ void store4(OutT* dst, float a, float b, float c, float d);

template <>
__device__ __forceinline__ void store4<float>(float* dst, float a, float b, float c, float d) {
    *reinterpret_cast<float4*>(dst) = make_float4(a, b, c, d);
}
template <>
__device__ __forceinline__ void store4<__bf16>(__bf16* dst, float a, float b, float c, float d) {
    bf16x4 o = {(__bf16)a, (__bf16)b, (__bf16)c, (__bf16)d};   // round to nearest even
    *reinterpret_cast<bf16x4*>(dst) = o;
}

template <typename OutT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void dfa_fwd_bf16_kernel(const FwdParams p) {
    __shared__ __attribute__((aligned(1024))) uint16_t k_lds[kStages][kStageElems];
    __shared__ __attribute__((aligned(1024))) uint16_t v_lds[kStages][kStageElems];
    __shared__ int32_t row_idx[kTileRows];
    __shared__ KeySeg seg_lds[DFA_MAX_BRANCHES];

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = p.tiles[item.tile];
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int h = tile.h, b = item.b;

    row_idx[tid] = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    if (tid < tile.nseg) seg_lds[tid] = p.segs[tile.seg_begin + tid];
    __syncthreads();

    OutT* const out = static_cast<OutT*>(p.out);
    const int64_t out_bh = (int64_t)b * p.N * p.H + h;   // in rows; row n adds n * H

    if (tile.nseg == 0) {
        // rows that no branch keeps: the zero matrix of Eq. 3 shows through, lse = -inf
        constexpr int kChunks = kD * sizeof(OutT) / 16;
        for (int x = tid; x < tile.nrows * kChunks; x += 256) {
            const int rr = x / kChunks, ch = x % kChunks;
            char* dst = reinterpret_cast<char*>(out + (out_bh + (int64_t)row_idx[rr] * p.H) * kD) + 16 * ch;
            *reinterpret_cast<u32x4*>(dst) = u32x4{0u, 0u, 0u, 0u};
        }
        if (p.lse && tid < tile.nrows)
            p.lse[((int64_t)b * p.H + h) * p.N + row_idx[tid]] = -INFINITY;
        return;
    }

    const uint16_t* const kp = static_cast<const uint16_t*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const uint16_t* const vp = static_cast<const uint16_t*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;

    // what this lane fetches in each copy (see CopyLane)
    CopyLane cl;
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int rho = 8 * (2 * wave + u) + (lane >> 3);                       // LDS row
        cl.kpos[u] = (rho & 0x33) | ((rho & 4) << 1) | ((rho & 8) >> 1);        // sigma(rho)
        cl.kchunk[u] = 16 * ((lane & 7) ^ k_swizzle(rho));
        cl.vpos[u] = rho;
    }
    cl.vchunk = 16 * (lane & 7);

    int n_steps = 0;
    for (int s = 0; s < tile.nseg; ++s)
        n_steps += (__builtin_amdgcn_readfirstlane(seg_lds[s].count) + kKeyTile - 1) / kKeyTile;

    const uint32_t k_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &k_lds[0][0]);
    const uint32_t v_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &v_lds[0][0]);
    constexpr uint32_t kStageBytes = kStageElems * 2;

    // first two stages on their way before anything else
    KeyCursor pf;
    pf.s = 0;
    pf.t = 0;
    cursor_load(pf, seg_lds);
    KeyCursor cur = pf;
    issue_stage(p, kp, vp, pf, cl, wave, k_lds_addr, v_lds_addr);
    cursor_next(pf, seg_lds, tile.nseg);
    if (n_steps > 1) {
        issue_stage(p, kp, vp, pf, cl, wave, k_lds_addr + kStageBytes, v_lds_addr + kStageBytes);
        cursor_next(pf, seg_lds, tile.nseg);
    }

    // Q fragments: B operand of S^T, lane (j, g) holds Q[row j][16*kk + 8*g .. +7]
    bf16x8 qf[2][4];
    {
        const uint16_t* qp = static_cast<const uint16_t*>(p.q) + (int64_t)b * p.sqb + (int64_t)h * p.sqh;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int64_t row = row_idx[wave * 64 + qb * 32 + j];
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + row * p.sqn + 16 * kk + 8 * g);
        }
        // pin the fragments here: the compiler then waits for these loads before the main loop
        // and places no vector-memory wait of its own inside it (it cannot see the copies above,
        // and a wait sized for these eight loads would drain the copy pipeline every step)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[qb][kk]));
    }

    const float c = p.scale * kLog2e;          // exponent scale: exp(s*x) = exp2(c*x)

    floatx16 oacc[2][2];                       // [d block][query block], O^T layout
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][qb][v] = 0.f;
    // Online softmax state per query block.  m_ref is a reference exponent, not the running
    // maximum: it is only moved (to the exact maximum seen so far) when a block's sums show
    // that exponents got large, so that the common case needs no row maximum at all.  Between
    // moves every p stays below kRebaseThreshold, which fp32 and bf16 carry without loss.
    float m_ref[2] = {-INFINITY, -INFINITY};
    float l_run[2] = {0.f, 0.f};               // this lane's share of the running sum

    const bool wave_live = wave * 64 < tile.nrows;   // waves past the end of a short tile only help copying

    int stage = 0;
    for (int i = 0; i < n_steps; ++i) {
        // stage i has landed once at most the 4 copies of stage i+1 are still outstanding
        // (the Q loads were issued after the first two stages, so the first wait covers them)
        if (i == 0 || i + 1 >= n_steps) wait_vmcnt<0>(); else wait_vmcnt<4>();
        __syncthreads();       // every wave's share is in LDS, and everyone is done with stage i-1
        if (i + 2 < n_steps) {
            const int st2 = stage == 0 ? 2 : stage - 1;        // (stage + 2) % 3
            issue_stage(p, kp, vp, pf, cl, wave, k_lds_addr + st2 * kStageBytes, v_lds_addr + st2 * kStageBytes);
            cursor_next(pf, seg_lds, tile.nseg);
        }
        const int nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
        if (wave_live) tile_step(k_lds[stage], v_lds[stage], qf, lane, nvalid, c, m_ref, l_run, oacc);
        cursor_next(cur, seg_lds, tile.nseg);
        stage = stage == 2 ? 0 : stage + 1;
    }

    // ---- epilogue: normalise, log-sum-exp, place each row at its own token (Eq. 3)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int slot = wave * 64 + qb * 32 + j;
        const float l_tot = l_run[qb] + wave_half_xchg(l_run[qb]);
        const float inv = 1.0f / l_tot;
        if (slot < tile.nrows) {
            const int64_t n = row_idx[slot];
            OutT* op = out + (out_bh + n * p.H) * kD;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq)
                    store4<OutT>(op + 32 * db + 8 * vq + 4 * g,
                                 oacc[db][qb][4 * vq] * inv, oacc[db][qb][4 * vq + 1] * inv,
                                 oacc[db][qb][4 * vq + 2] * inv, oacc[db][qb][4 * vq + 3] * inv);
            if (p.lse && g == 0)
                p.lse[((int64_t)b * p.H + h) * p.N + n] = (m_ref[qb] + __builtin_amdgcn_logf(l_tot)) * kLn2;
        }
    }
}

}  // namespace

hipError_t launch_fwd_bf16(const FwdParams& p, int n_items, bool out_f32, hipStream_t st) {
    if (out_f32)
        hipLaunchKernelGGL(dfa_fwd_bf16_kernel<float>, dim3(n_items), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL(dfa_fwd_bf16_kernel<__bf16>, dim3(n_items), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace dfa
