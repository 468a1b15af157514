// Backward of the fused dilated attention for bf16 operands, on the gfx950 matrix cores.
//
// The paper states no backward pass; this is the chain rule on Eq. 2 and the branch merge.  With
// the merged lse of the forward pass, P(n, j) = exp(scale q_n.k_j - lse_n) per (branch, n, j)
// pair of the definition and delta_n = dout_n . out_n:
//   dv_j += P dout_n,   ds = P (dout_n . v_j - delta_n),   dq_n += scale ds k_j,   dk_j += scale ds q_n.
//
// Two launches on the forward's plan, one for dq (which also leaves -delta and lse in base-2 units of every
// row in the workspace) and then one for dk and dv together; a workgroup owns
// a tile of up to 256 rows and walks the tile's lists 64 rows at a time.  In a segment the kept
// rows are queries and keys alike, so the lists are the tile's keys when its rows act as
// queries (dq) and the queries that see its rows when they act as keys (dk, dv): no gradient
// needs an atomic.  The rows of the tile stay in registers as B operands; the walked rows go
// global -> LDS (global_load_lds) three stages deep, each tensor in the layout its use needs:
//   "A" layout: rows permuted by sigma and 16-byte chunks swizzled, read back as 32 rows x 16 d
//               A operands of the first products (S^T and dP^T, walked row = MFMA row),
//   "T" layout: rows in list order, unswizzled, read back transposed (ds_read_b64_tr_b16) as
//               32 d x 16 rows A operands of the second product, whose B operand is the packed
//               bf16 result of the first products straight from registers (the register order
//               of the first product's result is the contraction order sigma fixes).
// Per 32 walked rows:
//   dq:  S^T = K~ Q^T, dP^T = V~ dO^T, dS^T = P (dP - delta), dQ^T += K~^T dS^T   (times scale at the end)
//   dk, dv:  S = Q~ K^T, dP - delta = dO~ V^T started from -delta, P = exp2(..), dS = P (dP - delta),
//            dV^T += dO~^T P,  dK^T += Q~^T dS   (times scale at the end)
// (~ marks the walked rows).  lse and delta of the walked queries travel with the rows as 4-byte
// copies.  P is recomputed from lse; there is no online softmax and no rescaling here.
#include "dfa_device.h"
#include "dfa_mfma.h"

namespace dfa {

namespace {

constexpr int kBwdStages = 3;

// 4 bytes per lane from global memory straight into LDS: lane L's word lands at lds_addr + 4*L.
__device__ __forceinline__ void copy4_to_lds(const void* gbase, uint32_t lane_byte_offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_byte_offset), "s"(gbase)
                 : "memory", "m0");
}

// What a lane fetches in the two 1 KB copies a wave contributes to one 8 KB tensor stage: copy u
// of wave w fills LDS rows rho = 8*(2w+u) .. +7, lane L lands at row L/8, chunk L%8.
struct BwdCopyLane {
    int a_pos, a_chunk;    // "A" layout: list position sigma(rho) and byte offset of the swizzled chunk (copy 0;
                           // copy 1: position + 4, chunk ^ 64)
    int t_pos, t_chunk;    // "T" layout: position rho, chunk in place (copy 1: position + 8)
};

template <bool kLayoutA>
__device__ __forceinline__ void issue_tensor(const uint16_t* base, int64_t row_pitch, const KeyCursor& c,
                                             const BwdCopyLane& cl, int wave, uint32_t lds_stage) {
    const int j0 = c.t * kKeyTile;
    const int room = c.count - 1 - j0;       // positions past the end of the list re-read its last row
    const int64_t first = kept_row(c.key0, c.stride, j0);
    const void* gb = uniform_ptr(base + first * row_pitch);
    const uint32_t pitch = (uint32_t)(c.stride * row_pitch * 2);
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const uint32_t blk = (uint32_t)(2 * wave + u) * 1024u;
        if (kLayoutA)
            copy16_to_lds(gb, (uint32_t)min(cl.a_pos + 4 * u, room) * pitch + (cl.a_chunk ^ (64 * u)), lds_stage + blk);
        else
            copy16_to_lds(gb, (uint32_t)min(cl.t_pos + 8 * u, room) * pitch + cl.t_chunk, lds_stage + blk);
    }
}

// one fp32 per walked row (position order): lane L fetches the value of list position L
__device__ __forceinline__ void issue_scalars(const float* per_row, const KeyCursor& c, int lane, uint32_t lds_addr) {
    const int j0 = c.t * kKeyTile;
    const int room = c.count - 1 - j0;
    const int64_t first = kept_row(c.key0, c.stride, j0);
    copy4_to_lds(uniform_ptr(per_row + first), (uint32_t)(min(lane, room) * c.stride * 4), lds_addr);
}

// Every value of a 32-row block at or past list position nvalid becomes -inf (its P is then 0).
// Register v of lane (j, g) is block position 16*(v/8) + 8*g + v%8.
__device__ __forceinline__ void mask_rows(floatx16& s, int g, int nvalid) {
#pragma unroll
    for (int v = 0; v < 16; ++v)
        if (16 * (v >> 3) + 8 * g + (v & 7) >= nvalid) s[v] = -INFINITY;
}

__device__ __forceinline__ floatx16 zero16() {
    floatx16 z;
#pragma unroll
    for (int v = 0; v < 16; ++v) z[v] = 0.f;
    return z;
}

// packs 16 fp32 values into the two B operands (16-row steps) of the second product
__device__ __forceinline__ void pack_block(const float (&x)[16], u32x4 (&pb)[2]) {
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const bf16x2 pr = {(__bf16)x[2 * v], (__bf16)x[2 * v + 1]};
        pb[v >> 2][v & 3] = __builtin_bit_cast(uint32_t, pr);
    }
}

// P and dS of one 32 x 32 block of the dk/dv kernel.  lp: lse (base-2 units) of the walked queries in LDS;
// register v of a lane is block position 16*(v/8) + 8*g + v%8, lp points at position 8*g.  dpd holds
// dP - delta already (the accumulators of dP start from -delta).  kBias: the pairs of this step count m
// times, log2 m = bias (see KeySeg).  The factor scale of dS goes onto the dk accumulator at the end.
template <bool kBias>
__device__ __forceinline__ void probs_block(const floatx16& s, const floatx16& dpd, const float* lp,
                                            float c, float bias, float (&pr)[16], float (&ds)[16]) {
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            const float4 l2 = *reinterpret_cast<const float4*>(lp + 16 * hf + e);
            const float l2a[4] = {l2.x, l2.y, l2.z, l2.w};
#pragma unroll
            for (int x = 0; x < 4; ++x) {
                const int v = 8 * hf + e + x;
                pr[v] = __builtin_amdgcn_exp2f(fmaf(s[v], c, kBias ? bias - l2a[x] : -l2a[x]));
                ds[v] = pr[v] * dpd[v];
            }
        }
}

// -delta of the 32 walked queries of a block as the start value of the dP accumulators: register v of a
// lane is block position 16*(v/8) + 8*g + v%8, dl points at position 8*g.
__device__ __forceinline__ floatx16 load_ndelta(const float* dl) {
    floatx16 r;
#pragma unroll
    for (int hf = 0; hf < 2; ++hf)
#pragma unroll
        for (int e = 0; e < 8; e += 4) {
            const float4 d = *reinterpret_cast<const float4*>(dl + 16 * hf + e);
            r[8 * hf + e] = d.x; r[8 * hf + e + 1] = d.y; r[8 * hf + e + 2] = d.z; r[8 * hf + e + 3] = d.w;
        }
    return r;
}

// dq of a tile: its rows are queries, the lists are walked as keys (K in "A" and "T" layout, V in "A"
// layout).  Four waves of 64 rows each.
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void bwd_dq_bf16_kernel(const BwdParams p) {
    constexpr int kTensors = 3;
    constexpr int kCopies = 2 * kTensors;                            // per wave per stage
    __shared__ __attribute__((aligned(1024))) uint16_t t_lds[kTensors][kBwdStages][kStageElems];
    __shared__ int32_t row_idx[kTileRows];
    __shared__ KeySeg seg_lds[kMaxTileSegs];

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = item.t;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int h = tile.h, b = item.b;

    row_idx[tid] = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    if (tid < tile.nseg) seg_lds[tid] = p.segs[tile.seg_begin + tid];
    __syncthreads();

    uint16_t* const grad = static_cast<uint16_t*>(p.dq);
    const int64_t out_bh = (int64_t)b * p.N * p.H + h;   // in rows of a contiguous [B,N,H,D] tensor; row n adds n * H

    if (tile.nseg == 0) {
        // rows that no branch keeps take and give no gradient
        constexpr int kChunks = kD * 2 / 16;
        for (int x = tid; x < tile.nrows * kChunks; x += 256) {
            const int rr = x / kChunks, ch = x % kChunks;
            char* dst = reinterpret_cast<char*>(grad + (out_bh + (int64_t)row_idx[rr] * p.H) * kD) + 16 * ch;
            *reinterpret_cast<u32x4*>(dst) = u32x4{0u, 0u, 0u, 0u};
        }
        return;
    }

    const uint16_t* const qp = static_cast<const uint16_t*>(p.q) + (int64_t)b * p.sqb + (int64_t)h * p.sqh;
    const uint16_t* const kp = static_cast<const uint16_t*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const uint16_t* const vp = static_cast<const uint16_t*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;
    const uint16_t* const gp = static_cast<const uint16_t*>(p.dout) + out_bh * kD;          // row n at n * H * D
    const int64_t g_pitch = (int64_t)p.H * kD;
    const uint16_t* const op = static_cast<const uint16_t*>(p.out) + out_bh * kD;           // row n at n * H * D
    const float* const lse_bh = p.lse + ((int64_t)b * p.H + h) * p.N;
    float* const ndelta_bh = p.ndelta + ((int64_t)b * p.H + h) * p.N;
    float* const lse2_bh = p.lse2 + ((int64_t)b * p.H + h) * p.N;

    // The lane constants of the copies are worked out afresh at every issue, from a copy of the lane number
    // the compiler cannot see through: kept across the main loop they are spilled to scratch memory, and the
    // reloads (vector memory operations the compiler waits for) would drain the copy pipeline every step.
    auto copy_lane = [&]() {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        BwdCopyLane cl;
        const int rho = 16 * wave + (ln >> 3);                                  // LDS row of copy 0 (bit 3 clear)
        cl.a_pos = (rho & 0x33) | ((rho & 4) << 1);                             // sigma(rho)
        cl.a_chunk = 16 * ((ln & 7) ^ k_swizzle(rho));
        cl.t_pos = rho;
        cl.t_chunk = 16 * (ln & 7);
        return cl;
    };
    // fragment reads: "A" layout row j of a 32-row block, chunk (2*kk + g) ^ swizzle(j); "T" layout as
    // read_v_frag describes
    const int frag_a = j * kRowElems + 8 * (g ^ k_swizzle(j));
    const int frag_t = (((lane & 15) >> 2) + 8 * g) * kRowElems + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    int n_steps = tile.n_steps;

    const uint32_t t_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &t_lds[0][0][0]);
    constexpr uint32_t kStageBytes = kStageElems * 2, kTensorBytes = kBwdStages * kStageBytes;

    auto issue = [&](const KeyCursor& c, int slot) {
        const uint32_t st = t_addr + slot * kStageBytes;
        const BwdCopyLane cl = copy_lane();
        issue_tensor<true>(kp, p.skn, c, cl, wave, st);
        issue_tensor<true>(vp, p.svn, c, cl, wave, st + kTensorBytes);
        issue_tensor<false>(kp, p.skn, c, cl, wave, st + 2 * kTensorBytes);
    };

    // first two stages on their way before anything else
    KeyCursor pf;
    pf.s = 0;
    pf.t = 0;
    cursor_load(pf, seg_lds);
    KeyCursor cur = pf;
    issue(pf, 0);
    cursor_next(pf, seg_lds, tile.nseg);
    if (n_steps > 1) {
        issue(pf, 1);
        cursor_next(pf, seg_lds, tile.nseg);
    }

    // ---- lse in base-2 units and -delta = -(dout . out) of the wave's rows: worked out here (a lane and its
    // partner lane ^ 32 hold the two halves of a row) and left in the workspace for the dk/dv kernel, which
    // reads them for the rows it walks.  Done before the B operands are loaded so that the two do not
    // need registers at the same time.
    float my_l2[2], my_nd[2];
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        const int64_t row = row_idx[wave * 64 + blk * 32 + j];
        my_l2[blk] = lse_bh[row] * kLog2e;
        float part = 0.f;
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            const bf16x8 gv = *reinterpret_cast<const bf16x8*>(gp + row * g_pitch + 16 * kk + 8 * g);
            const bf16x8 ov = *reinterpret_cast<const bf16x8*>(op + row * g_pitch + 16 * kk + 8 * g);
#pragma unroll
            for (int t = 0; t < 8; ++t) part = fmaf((float)gv[t], (float)ov[t], part);
        }
        my_nd[blk] = -wave_half_sum(part);
        if (g == 0 && wave * 64 + blk * 32 + j < tile.nrows) {
            ndelta_bh[row] = my_nd[blk];
            lse2_bh[row] = my_l2[blk];
        }
    }
    __builtin_amdgcn_sched_barrier(0);

    // ---- the tile's own rows as B operands (16 d x 32 rows): lane (j, g) holds row j, d 16*kk + 8*g .. +7
    bf16x8 qf[2][4], gf[2][4];           // q and dout of the wave's two 32-row blocks
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
        const int64_t row = row_idx[wave * 64 + blk * 32 + j];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            qf[blk][kk] = *reinterpret_cast<const bf16x8*>(qp + row * p.sqn + 16 * kk + 8 * g);
            gf[blk][kk] = *reinterpret_cast<const bf16x8*>(gp + row * g_pitch + 16 * kk + 8 * g);
        }
    }
    // pin them: the compiler then waits for these loads here and places no vector-memory wait of
    // its own inside the main loop (it cannot see the copies, and its wait would drain them)
#pragma unroll
    for (int blk = 0; blk < 2; ++blk) {
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            asm volatile("" : "+v"(qf[blk][kk]));
            asm volatile("" : "+v"(gf[blk][kk]));
        }
        asm volatile("" : "+v"(my_l2[blk]));
        asm volatile("" : "+v"(my_nd[blk]));
    }

    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale * kLog2e)));
    const float scale = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale)));

    floatx16 acc[2][2];                    // [d block][own 32-row block], transposed like the forward's accumulator
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int blk = 0; blk < 2; ++blk) acc[db][blk] = zero16();

    const bool wave_live = wave * 64 < tile.nrows;   // waves past the end of a short tile only help copying

    // pairs that count m times (see KeySeg): P carries the factor m, i.e. log2 m is taken off the row's
    // lse while the walk is inside such a progression
    float bias_cur = 0.f;
    int slot = 0;
    for (int i = 0; i < n_steps; ++i) {
        if (cur.bias != bias_cur) {
            my_l2[0] -= cur.bias - bias_cur;
            my_l2[1] -= cur.bias - bias_cur;
            bias_cur = cur.bias;
        }
        // stage i has landed once at most the copies of stage i+1 are still outstanding (the loads of
        // the own rows were issued after the first two stages, so the first wait covers them)
        if (i == 0 || i + 1 >= n_steps) wait_vmcnt<0>(); else wait_vmcnt<kCopies>();
        __syncthreads();       // every wave's share is in LDS, and everyone is done with stage i-1
        if (i + 2 < n_steps) {
            issue(pf, slot == 0 ? 2 : slot - 1);               // (slot + 2) % 3
            cursor_next(pf, seg_lds, tile.nseg);
        }
        const int nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
        if (wave_live) {
#pragma unroll
            for (int ws = 0; ws < 2; ++ws) {                   // 32 walked keys at a time
                const int nv = nvalid - 32 * ws;
                const uint16_t* const ka = t_lds[0][slot] + 32 * ws * kRowElems;
                const uint16_t* const va = t_lds[1][slot] + 32 * ws * kRowElems;
                u32x4 pb[2][2];                                // [own block][16-key step], packed bf16 pairs
                floatx16 s[2], dp[2];
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8 kfr = *reinterpret_cast<const bf16x8*>(ka + (frag_a ^ (16 * kk)));
                    const bf16x8 vfr = *reinterpret_cast<const bf16x8*>(va + (frag_a ^ (16 * kk)));
#pragma unroll
                    for (int blk = 0; blk < 2; ++blk) {
                        s[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kfr, qf[blk][kk], kk == 0 ? zero16() : s[blk], 0, 0, 0);
                        dp[blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vfr, gf[blk][kk], kk == 0 ? zero16() : dp[blk], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int blk = 0; blk < 2; ++blk) {
                    if (nv < 32) mask_rows(s[blk], g, nv);
                    float ds[16];
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const float pr = __builtin_amdgcn_exp2f(fmaf(s[blk][v], c, -my_l2[blk]));
                        ds[v] = pr * (dp[blk][v] + my_nd[blk]);    // the factor scale goes onto the accumulator at the end
                    }
                    pack_block(ds, pb[blk]);
                }
                // dQ^T[d][query] += K~^T[d][key] . dS^T[key][query]
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int st = 0; st < 2; ++st) {
                        const bf16x8 kt = read_v_frag(t_lds[2][slot] + (32 * ws + 16 * st) * kRowElems + frag_t + 32 * db);
#pragma unroll
                        for (int blk = 0; blk < 2; ++blk)
                            acc[db][blk] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kt, __builtin_bit_cast(bf16x8, pb[blk][st]), acc[db][blk], 0, 0, 0);
                    }
            }
        }
        cursor_next(cur, seg_lds, tile.nseg);
        slot = slot == kBwdStages - 1 ? 0 : slot + 1;
    }

    // ---- epilogue: each wave lays its 64 rows out row-major in a piece of the (now idle) stages, at a
    // pitch of 144 bytes, and stores them 16 bytes per lane, eight lanes to a row, at the rows' tokens
    __syncthreads();           // every wave is done with the stages
    constexpr int kPitch = kD * 2 + 16;
    char* mine = reinterpret_cast<char*>(&t_lds[wave >> 1][0][0]) + (wave & 1) * (64 * kPitch);
    if (wave_live) {
#pragma unroll
        for (int blk = 0; blk < 2; ++blk)
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const bf16x4 o = {(__bf16)(acc[db][blk][4 * vq] * scale), (__bf16)(acc[db][blk][4 * vq + 1] * scale),
                                      (__bf16)(acc[db][blk][4 * vq + 2] * scale), (__bf16)(acc[db][blk][4 * vq + 3] * scale)};
                    *reinterpret_cast<bf16x4*>(mine + (32 * blk + j) * kPitch + (32 * db + 8 * vq + 4 * g) * 2) = o;
                }
        // the wave reads back only what it wrote itself; LDS operations of a wave complete in order
        const int srow = lane >> 3, schunk = lane & 7;
#pragma unroll
        for (int s = 0; s < 8; ++s) {
            const int row = 8 * s + srow, slot_r = wave * 64 + row;
            const u32x4 val = *reinterpret_cast<const u32x4*>(mine + row * kPitch + 16 * schunk);
            if (slot_r < tile.nrows) {
                const int64_t n = row_idx[slot_r];
                *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(grad + (out_bh + n * p.H) * kD) + 16 * schunk) = val;
            }
        }
    }
}

// dk and dv of a tile in one walk over its query lists.  Eight waves of 32 rows each (both
// gradients of 64 rows would not fit a wave's registers): the scores are computed once for both,
// and the walked Q and dO rows are copied once, each in both layouts.
__global__ __launch_bounds__(512) __attribute__((amdgpu_waves_per_eu(2, 2)))
void bwd_dkdv_bf16_kernel(const BwdParams p) {
    constexpr int kTensors = 4;                                      // Q "A", dO "A", Q "T", dO "T"
    constexpr int kCopies = kTensors + 2;                            // per wave per stage, with lse and delta
    __shared__ __attribute__((aligned(1024))) uint16_t t_lds[kTensors][kBwdStages][kStageElems];
    __shared__ __attribute__((aligned(256))) float sc_lds[2][kBwdStages][kKeyTile];
    __shared__ int32_t row_idx[kTileRows];
    __shared__ KeySeg seg_lds[kMaxTileSegs];

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = item.t;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int h = tile.h, b = item.b;

    if (tid < kTileRows) row_idx[tid] = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    if (tid < tile.nseg) seg_lds[tid] = p.segs[tile.seg_begin + tid];
    __syncthreads();

    uint16_t* const grad_k = static_cast<uint16_t*>(p.dk);
    uint16_t* const grad_v = static_cast<uint16_t*>(p.dv);
    const int64_t out_bh = (int64_t)b * p.N * p.H + h;   // in rows of a contiguous [B,N,H,D] tensor; row n adds n * H

    if (tile.nseg == 0) {
        // rows that no branch keeps take and give no gradient
        constexpr int kChunks = kD * 2 / 16;
        for (int x = tid; x < tile.nrows * kChunks; x += 512) {
            const int rr = x / kChunks, ch = x % kChunks;
            const int64_t at = (out_bh + (int64_t)row_idx[rr] * p.H) * kD;
            *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(grad_k + at) + 16 * ch) = u32x4{0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(grad_v + at) + 16 * ch) = u32x4{0u, 0u, 0u, 0u};
        }
        return;
    }

    const uint16_t* const qp = static_cast<const uint16_t*>(p.q) + (int64_t)b * p.sqb + (int64_t)h * p.sqh;
    const uint16_t* const kp = static_cast<const uint16_t*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const uint16_t* const vp = static_cast<const uint16_t*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;
    const uint16_t* const gp = static_cast<const uint16_t*>(p.dout) + out_bh * kD;          // row n at n * H * D
    const int64_t g_pitch = (int64_t)p.H * kD;
    const float* const ndelta_bh = p.ndelta + ((int64_t)b * p.H + h) * p.N;
    const float* const lse2_bh = p.lse2 + ((int64_t)b * p.H + h) * p.N;

    // one 1 KB copy per wave and tensor: wave w fills LDS rows rho = 8w .. 8w+7, lane L lands at row L/8, chunk L%8
    const int rho = 8 * wave + (lane >> 3);
    const int a_pos = (rho & 0x33) | ((rho & 4) << 1) | ((rho & 8) >> 1);      // sigma(rho)
    const int a_chunk = 16 * ((lane & 7) ^ k_swizzle(rho));
    const int t_chunk = 16 * (lane & 7);
    const int frag_a = j * kRowElems + 8 * (g ^ k_swizzle(j));
    const int frag_t = (((lane & 15) >> 2) + 8 * g) * kRowElems + 16 * ((lane >> 4) & 1) + 4 * (lane & 3);

    int n_steps = tile.n_steps;

    const uint32_t t_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &t_lds[0][0][0]);
    const uint32_t sc_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &sc_lds[0][0][0]);
    constexpr uint32_t kStageBytes = kStageElems * 2, kTensorBytes = kBwdStages * kStageBytes;

    auto issue = [&](const KeyCursor& c, int slot) {
        const int j0 = c.t * kKeyTile;
        const int room = c.count - 1 - j0;   // positions past the end of the list re-read its last row
        const int64_t first = kept_row(c.key0, c.stride, j0);
        const uint32_t qpitch = (uint32_t)(c.stride * p.sqn * 2), gpitch = (uint32_t)(c.stride * g_pitch * 2);
        const void* qb = uniform_ptr(qp + first * p.sqn);
        const void* gb = uniform_ptr(gp + first * g_pitch);
        const uint32_t st = t_addr + slot * kStageBytes + wave * 1024u;
        const uint32_t pa = (uint32_t)min(a_pos, room), pt = (uint32_t)min(rho, room);
        copy16_to_lds(qb, pa * qpitch + a_chunk, st);
        copy16_to_lds(gb, pa * gpitch + a_chunk, st + kTensorBytes);
        copy16_to_lds(qb, pt * qpitch + t_chunk, st + 2 * kTensorBytes);
        copy16_to_lds(gb, pt * gpitch + t_chunk, st + 3 * kTensorBytes);
        issue_scalars(lse2_bh, c, lane, sc_addr + slot * (kKeyTile * 4));
        issue_scalars(ndelta_bh, c, lane, sc_addr + (kBwdStages + slot) * (kKeyTile * 4));
    };

    KeyCursor pf;
    pf.s = 0;
    pf.t = 0;
    cursor_load(pf, seg_lds);
    KeyCursor cur = pf;
    issue(pf, 0);
    cursor_next(pf, seg_lds, tile.nseg);
    if (n_steps > 1) {
        issue(pf, 1);
        cursor_next(pf, seg_lds, tile.nseg);
    }

    // the wave's own 32 rows as B operands (16 d x 32 rows): lane (j, g) holds row j, d 16*kk + 8*g .. +7
    bf16x8 kf[4], vf[4];
    {
        const int64_t row = row_idx[wave * 32 + j];
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            kf[kk] = *reinterpret_cast<const bf16x8*>(kp + row * p.skn + 16 * kk + 8 * g);
            vf[kk] = *reinterpret_cast<const bf16x8*>(vp + row * p.svn + 16 * kk + 8 * g);
        }
        // pinned: the compiler waits for these loads here and places no vector-memory wait of its own in the loop
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) {
            asm volatile("" : "+v"(kf[kk]));
            asm volatile("" : "+v"(vf[kk]));
        }
    }

    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale * kLog2e)));
    const float scale = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale)));

    floatx16 dk_acc[2], dv_acc[2];         // [d block], transposed: lane = own row
#pragma unroll
    for (int db = 0; db < 2; ++db) {
        dk_acc[db] = zero16();
        dv_acc[db] = zero16();
    }
    const bool wave_live = wave * 32 < tile.nrows;

    int slot = 0;
    for (int i = 0; i < n_steps; ++i) {
        if (i == 0 || i + 1 >= n_steps) wait_vmcnt<0>(); else wait_vmcnt<kCopies>();
        __syncthreads();       // every wave's share is in LDS, and everyone is done with stage i-1
        if (i + 2 < n_steps) {
            issue(pf, slot == 0 ? 2 : slot - 1);               // (slot + 2) % 3
            cursor_next(pf, seg_lds, tile.nseg);
        }
        const int nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
        if (wave_live) {
#pragma unroll
            for (int ws = 0; ws < 2; ++ws) {                   // 32 walked queries at a time
                const int nv = nvalid - 32 * ws;
                const uint16_t* const qa = t_lds[0][slot] + 32 * ws * kRowElems;
                const uint16_t* const ga = t_lds[1][slot] + 32 * ws * kRowElems;
                floatx16 s, dp = load_ndelta(&sc_lds[1][slot][32 * ws + 8 * g]);   // dp ends up as dP - delta
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) {
                    const bf16x8 qf = *reinterpret_cast<const bf16x8*>(qa + (frag_a ^ (16 * kk)));
                    const bf16x8 gf = *reinterpret_cast<const bf16x8*>(ga + (frag_a ^ (16 * kk)));
                    s = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf, kf[kk], kk == 0 ? zero16() : s, 0, 0, 0);
                    dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gf, vf[kk], dp, 0, 0, 0);
                }
                if (nv < 32) mask_rows(s, g, nv);
                // lse and delta of the walked queries: register v is block position 16*(v/8) + 8*g + v%8
                float pr[16], ds[16];
                {
                    const float* lp = &sc_lds[0][slot][32 * ws + 8 * g];
                    if (cur.bias == 0.f) probs_block<false>(s, dp, lp, c, 0.f, pr, ds);
                    else probs_block<true>(s, dp, lp, c, cur.bias, pr, ds);
                }
                u32x4 pp[2], ps[2];
                pack_block(pr, pp);
                pack_block(ds, ps);
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int st = 0; st < 2; ++st) {
                        const int off = (32 * ws + 16 * st) * kRowElems + frag_t + 32 * db;
                        const bf16x8 qt = read_v_frag(t_lds[2][slot] + off);
                        const bf16x8 gt = read_v_frag(t_lds[3][slot] + off);
                        dv_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(gt, __builtin_bit_cast(bf16x8, pp[st]), dv_acc[db], 0, 0, 0);
                        dk_acc[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qt, __builtin_bit_cast(bf16x8, ps[st]), dk_acc[db], 0, 0, 0);
                    }
            }
        }
        cursor_next(cur, seg_lds, tile.nseg);
        slot = slot == kBwdStages - 1 ? 0 : slot + 1;
    }

    // ---- epilogue: each wave lays its 32 rows of both gradients out row-major in a piece of the idle
    // stages (pitch 144 bytes) and stores them 16 bytes per lane, eight lanes to a row
    __syncthreads();           // every wave is done with the stages
    constexpr int kPitch = kD * 2 + 16;
    char* mine = reinterpret_cast<char*>(&t_lds[wave >> 1][0][0]) + (wave & 1) * (64 * kPitch);   // 2 x 32 rows
    if (wave_live) {
#pragma unroll
        for (int which = 0; which < 2; ++which)
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int vq = 0; vq < 4; ++vq) {
                    const floatx16& a = which == 0 ? dk_acc[db] : dv_acc[db];
                    const float f = which == 0 ? scale : 1.0f;     // dk = scale dS^T q
                    const bf16x4 o = {(__bf16)(a[4 * vq] * f), (__bf16)(a[4 * vq + 1] * f), (__bf16)(a[4 * vq + 2] * f), (__bf16)(a[4 * vq + 3] * f)};
                    *reinterpret_cast<bf16x4*>(mine + (32 * which + j) * kPitch + (32 * db + 8 * vq + 4 * g) * 2) = o;
                }
        // the wave reads back only what it wrote itself; LDS operations of a wave complete in order
        const int srow = lane >> 3, schunk = lane & 7;
#pragma unroll
        for (int which = 0; which < 2; ++which)
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const int row = 8 * s + srow, slot_r = wave * 32 + row;
                const u32x4 val = *reinterpret_cast<const u32x4*>(mine + (32 * which + row) * kPitch + 16 * schunk);
                if (slot_r < tile.nrows) {
                    const int64_t n = row_idx[slot_r];
                    uint16_t* dst = (which == 0 ? grad_k : grad_v) + (out_bh + n * p.H) * kD;
                    *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(dst) + 16 * schunk) = val;
                }
            }
    }
}

}  // namespace

hipError_t launch_bwd_bf16(const BwdParams& p, int n_items, hipStream_t st) {
    hipLaunchKernelGGL(bwd_dq_bf16_kernel, dim3(n_items), dim3(256), 0, st, p);
    hipLaunchKernelGGL(bwd_dkdv_bf16_kernel, dim3(n_items), dim3(512), 0, st, p);
    return hipGetLastError();
}

}  // namespace dfa
