// Fused dilated flash attention forward, bf16 on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns a tile of up to 256 query rows that share the same key lists
// (section 3.1: all of them are kept by the same branches and fall into the same segment of
// each).  It walks the key lists of its member branches one after the other (keys that several of
// them keep are visited once and weighted by their multiplicity, see KeySeg), carrying ONE
// online-softmax state (reference exponent, running sum, accumulator) per query row across all
// of them: continuing the softmax over the next branch's keys is the log-sum-exp merge of the
// branches, so no partial result ever leaves the registers.
//
// Gather (Eq. 1) happens in the global->LDS copies (key j of a segment is row first + r*j),
// placement (Eq. 3) in the final store (each query row is written back at its own token).
//
// Data movement: K and V rows go from global memory straight into LDS (global_load_lds, 16
// bytes per lane, no staging registers) in stages of 64 keys, four stages in LDS, two of them
// in flight while a third is being consumed.  Each wave-level copy fills 1 KB = 8 rows of 128
// bytes; which global row and 16-byte chunk a lane fetches is free, which is how the row
// permutation and the bank swizzle below are applied.
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
//
// Schedule: the key walk is software-pipelined in beats of 32 keys.  In one beat a wave issues
// the MFMAs of the NEXT block's scores and of the PREVIOUS block's accumulation while its
// vector ALU turns the CURRENT block's scores into probabilities, all in one hand-ordered
// instruction stream (see beat()), so matrix cores and vector ALU overlap inside each wave
// and not only between the two waves that share a SIMD.  The first beat of a walk (nothing to
// accumulate yet) and the last (nothing left to score) stand outside the loop in trimmed form.
//
// Row sums: the vector ALU's issue slots are what a beat runs out of first (an exponent, an exponential
// and half a rounding per score already fill the time of the MFMAs beside them), so the softmax
// denominators are not added up there.  The rounded probabilities sit in registers as B operands of the
// second product; one more small MFMA per 16-key group (v_mfma_f32_16x16x32_bf16 against a constant 0/1
// selector, see `sel` in the kernel) sums them per query on the matrix cores, which have time to spare.
// The denominator is therefore the sum of the bf16-rounded numerators, the same values the accumulator
// is built from: out is their exact weighted mean, and lse carries their rounding (each numerator is off
// by at most 2^-9 relative on average and 2^-8 at worst, so |error of lse| <= 2^-8 when one key dominates
// and far less when many keys share the weight).
#include "dfa_device.h"
#include "dfa_mfma.h"

namespace dfa {

namespace {

typedef float floatx4 __attribute__((ext_vector_type(4)));
constexpr int kStages = 4;                 // 64-key K/V stages in LDS

// Per-lane constants of the global->LDS copies.  A wave issues 2 K copies and 2 V copies per
// step; copy u of wave w fills LDS rows rho = 8*(2w+u) .. +7, lane L lands at row L/8, chunk
// L%8.  Stored for u = 0; for u = 1 (rho + 8) the key position sigma(rho) grows by 4, the
// swizzled chunk flips its top bit and the V position grows by 8.
struct CopyLane {
    int kpos;          // tile position of the key whose row this lane fetches (K copy 0)
    int kchunk;        // byte offset of the 16-byte chunk of that row
    int vpos;          // same for V (position order, chunks in place)
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
        copy16_to_lds(kb, (uint32_t)min(cl.kpos + 4 * u, room) * kpitch + (cl.kchunk ^ (64 * u)), k_stage + blk);
        copy16_to_lds(vb, (uint32_t)min(cl.vpos + 8 * u, room) * vpitch + cl.vchunk, v_stage + blk);
    }
}

// If a lane's partial row sum of one 32-key block exceeds this, some exponent may have left
// the comfortable range and the reference exponent is moved up (see rebase_block).
constexpr float kRebaseThreshold = 256.0f;
// Reference exponent before the first score of a row (kernel variant for packed tiles): below any scaled score
// that fp32 holds with room to spare, and finite.
constexpr float kRefStart = -3.0e38f;

// Softmax numerators of one 32-key block against the current reference exponents m_ref (no
// row maximum is taken here): p = exp2(c*s - m_ref), rounded to bf16 (nearest even) and packed
// straight into the B operands of the second product; psum = the row sums of the block (whole rows:
// both lanes that share a query hold the same value), in fp32 over the unrounded values.  Plain form,
// used after a rebase; beat() takes the numerators the same way in its hand-ordered stream and has
// the matrix cores add them up.
__device__ __forceinline__ void exp_block(const floatx16 (&s)[2], float c, const float (&m_ref)[2],
                                          u32x4 (&pb)[2][2], float (&psum)[2]) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        float a0 = 0.f, a1 = 0.f;
#pragma unroll
        for (int v = 0; v < 8; ++v) {
            const float e0 = __builtin_amdgcn_exp2f(fmaf(s[qb][2 * v], c, -m_ref[qb]));
            const float e1 = __builtin_amdgcn_exp2f(fmaf(s[qb][2 * v + 1], c, -m_ref[qb]));
            const bf16x2 pr = {(__bf16)e0, (__bf16)e1};
            pb[qb][v >> 2][v & 3] = __builtin_bit_cast(uint32_t, pr);   // slots 2v%8, 2v%8+1 of step v/4
            a0 += e0;
            a1 += e1;
        }
        psum[qb] = wave_half_sum(a0 + a1);
    }
}

// Rare path of the online softmax: take the exact row maximum of this block, move the
// reference exponent up to it, rescale the running sum and the accumulator.
// kSkips: a query block may be skipping the progression in hand (m_ref = +inf, see the kernel): it stays as it is.
template <bool kSkips>
__device__ __forceinline__ void rebase_block(const floatx16 (&s)[2], float c, float (&m_ref)[2],
                                             float (&l_run)[2], floatx16 (&oacc)[2][2]) {
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        if (kSkips && m_ref[qb] == INFINITY) continue;      // wave-uniform: a block skips as a whole
        float mx = s[qb][0];
#pragma unroll
        for (int v = 1; v < 16; ++v) mx = fmaxf(mx, s[qb][v]);
        mx = wave_half_max(mx);
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

// Lane constants of the LDS fragment reads.
struct FragLane {
    int k;        // element offset inside a 32-key K block of the 16-byte chunk for d-step 0; the chunk
                  // of d-step kk is (2*kk + g) ^ swizzle, i.e. this offset with 16*kk xor-ed in
    int v;        // element offset inside a 32-key V block of this lane's transposed-read address
};

// End of a key list: every score of a 32-key block at or past position nvalid becomes -inf.
// Register v of lane (j, g) is block position 16*(v/8) + 8*g + v%8.
__device__ __forceinline__ void mask_block(floatx16 (&s)[2], int g, int nvalid) {
#pragma unroll
    for (int v = 0; v < 16; ++v) {
        const int pos = 16 * (v >> 3) + 8 * g + (v & 7);
        if (pos >= nvalid) {
            s[0][v] = -INFINITY;
            s[1][v] = -INFINITY;
        }
    }
}

// Scores of one 32-key block, S^T = K~ Q~^T, on their own (pipeline prologue).
__device__ __forceinline__ void scores_block(const uint16_t* kblk, const FragLane& fl, const bf16x8 (&qf)[2][4],
                                             floatx16 (&s)[2]) {
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
        const bf16x8 kf = *reinterpret_cast<const bf16x8*>(kblk + (fl.k ^ (16 * kk)));
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            floatx16 z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.f;
            s[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][kk], kk == 0 ? z : s[qb], 0, 0, 0);
        }
    }
}


// Second product of one 32-key block on its own (pipeline epilogue).
__device__ __forceinline__ void accumulate_block(const uint16_t* vblk, const FragLane& fl, const u32x4 (&pb)[2][2],
                                                 floatx16 (&oacc)[2][2]) {
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int st = 0; st < 2; ++st) {
            const bf16x8 vf = read_v_frag(vblk + fl.v + 16 * st * kRowElems + 32 * db);
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
                oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, __builtin_bit_cast(bf16x8, pb[qb][st]), oacc[db][qb], 0, 0, 0);
        }
}

// One pipeline beat (32 keys).  Three independent pieces of work are woven into one
// instruction stream, so that the matrix cores and the vector ALU of the SIMD are busy at the
// same time from within a single wave:
//   matrix cores : S^T of the NEXT block (K at k_next -> s_next), and O^T += V~^T P^T of the
//                  PREVIOUS block (V at v_prev, probabilities p_prev);
//   vector ALU   : softmax numerators of the CURRENT block (s_cur -> p_cur).
// The stream is laid out slot by slot: one MFMA, then the exponent, exponential and rounding
// instructions of three different score pairs (a vector instruction that needs the
// result of the one just before it stalls the wave, so each pair moves one stage per slot).
// Whenever a 16-key group of p_cur is complete, one row-sum MFMA (selector `sel` times that group)
// adds it to psum: register 0 of its result is the sum over the group's 16 keys of the lane's query.
// Scheduling fences keep the compiler from regrouping the slots.
// kScores / kAccumulate: the beat has a next block to score / a previous block to accumulate (the first
// beat of a walk has no previous block, the last one no next block; their MFMAs and fragment reads are
// left out).
template <bool kScores, bool kAccumulate>
__device__ __forceinline__ void beat(const uint16_t* k_next, const uint16_t* v_prev, const FragLane& fl,
                                     const bf16x8 (&qf)[2][4], const floatx16 (&s_cur)[2], floatx16 (&s_next)[2],
                                     const u32x4 (&p_prev)[2][2], u32x4 (&p_cur)[2][2], floatx16 (&oacc)[2][2],
                                     float c, const float (&m_ref)[2], float (&psum)[2], const bf16x8& sel) {
    bf16x8 kf[2], vf[2];           // fragments of MFMA group r live in slot r & 1
    float t[16][2];                // exponents, then exponentials, of score pair q
    floatx4 rs[2];                 // row sums of the rounded numerators, from the matrix cores (register 0)

    auto load_group = [&](int r) {     // group r: d-step r of the scores, (d block r/2, 16-key step r%2) of the accumulation
        if (kScores) kf[r & 1] = *reinterpret_cast<const bf16x8*>(k_next + (fl.k ^ (16 * r)));
        if (kAccumulate) vf[r & 1] = read_v_frag(v_prev + fl.v + 16 * (r & 1) * kRowElems + 32 * (r >> 1));
    };
    auto mfma = [&](int k) {           // MFMA k of the beat: group r = k/4; scores for query block 0, 1, then accumulation for 0, 1
        const int r = k >> 2, qb = k & 1;
        if ((k & 2) == 0) {
            if (!kScores) return;
            floatx16 z;
#pragma unroll
            for (int v = 0; v < 16; ++v) z[v] = 0.f;
            s_next[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf[r & 1], qf[qb][r], r == 0 ? z : s_next[qb], 0, 0, 0);
        } else {
            if (!kAccumulate) return;
            const int db = r >> 1, st = r & 1;
            oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf[r & 1], __builtin_bit_cast(bf16x8, p_prev[qb][st]), oacc[db][qb], 0, 0, 0);
        }
    };

    load_group(0);
#pragma unroll
    for (int m = 0; m < 18; ++m) {
        // fragment reads run four slots ahead of their first MFMA
        if (m >= 2 && m < 14 && ((m - 2) & 3) == 0) load_group(((m - 2) >> 2) + 1);
        if (m >= 2 && m < 18) mfma(m - 2);
        if (m < 16) {                                   // exponents of pair m
            const int qb = m >> 3, v = 2 * (m & 7);
            t[m][0] = fmaf(s_cur[qb][v], c, -m_ref[qb]);
            t[m][1] = fmaf(s_cur[qb][v + 1], c, -m_ref[qb]);
        }
        if (m >= 1 && m < 17) {                         // exponentials of pair m - 1
            t[m - 1][0] = __builtin_amdgcn_exp2f(t[m - 1][0]);
            t[m - 1][1] = __builtin_amdgcn_exp2f(t[m - 1][1]);
        }
        if (m >= 2 && m < 18) {                         // pair m - 2: round into its B-operand slot, add to the row sums
            const int q = m - 2, qb = q >> 3, pr = q & 7;
            const bf16x2 w = {(__bf16)t[q][0], (__bf16)t[q][1]};
            p_cur[qb][pr >> 2][pr & 3] = __builtin_bit_cast(uint32_t, w);
        }
        if (m == 7 || m == 11 || m == 15) {             // row sums of the 16-key group finished two slots ago
            const int grp = (m - 7) >> 2, qb = grp >> 1, st = grp & 1;
            rs[qb] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, __builtin_bit_cast(bf16x8, p_cur[qb][st]),
                                                             st == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : rs[qb], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    rs[1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(sel, __builtin_bit_cast(bf16x8, p_cur[1][1]), rs[1], 0, 0, 0);
    psum[0] = rs[0][0];
    psum[1] = rs[1][0];
}

// The wave-uniform end of a beat: accept the numerators, or (rarely) move the reference
// exponent and redo them.  oacc already holds every earlier block under the old reference.
template <bool kSkips>
__device__ __forceinline__ void settle(const floatx16 (&s_cur)[2], u32x4 (&p_cur)[2][2], float c, float (&m_ref)[2],
                                       float (&l_run)[2], floatx16 (&oacc)[2][2], float (&psum)[2]) {
    // written so that NaN (-inf - -inf before the first rebase) trips the test
    const bool calm = psum[0] <= kRebaseThreshold && psum[1] <= kRebaseThreshold;
    if (__builtin_expect(__ballot(!calm) != 0ull, 0)) {
        // one rebase always suffices for finite inputs (every p of the block is <= 1 after it)
        rebase_block<kSkips>(s_cur, c, m_ref, l_run, oacc);
        exp_block(s_cur, c, m_ref, p_cur, psum);
    }
    l_run[0] += psum[0];
    l_run[1] += psum[1];
}

// kSplit: the workgroup walks only its share of the tile's steps (see FwdParams::split_wgs) and leaves a partial
// result (rows in tile order: out normalised, divided by the row's largest magnitude and rounded to fp16; lse and
// those row scales in fp32) in its own block of the workspace; a tile that the launch leaves whole (one part) is
// written out as in any other launch.  OutT is bf16 then.
// kPacked: the plan has tiles that pack several row groups (multiplicities per 32-row block, filler slots); plans
// without such tiles run the variant that has none of that in its way.
template <typename OutT, bool kSplit, bool kPacked>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2, 2)))
void dfa_fwd_bf16_kernel(const FwdParams p) {
    __shared__ __attribute__((aligned(1024))) uint16_t k_lds[kStages][kStageElems];
    __shared__ __attribute__((aligned(1024))) uint16_t v_lds[kStages][kStageElems];
    __shared__ int32_t row_idx[kTileRows];      // token of each slot; < 0: a filler slot, nothing to store
    // the tile's key progressions, one copy per wave: log2_mult of wave w's copy is the figure for w's rows
    // (-inf: they do not attend to the progression's keys)
    __shared__ KeySeg seg_all[kPacked ? 4 : 1][kMaxTileSegs];
    __shared__ float bias1_all[kPacked ? 4 : 1][kMaxTileSegs];   // kPacked: log2 m of the wave's second 32-row block

    int part = 0, nparts = 1, item_index = blockIdx.x;
    if (kSplit) {
        const SplitWg sw = p.split_wgs[blockIdx.x];
        item_index = sw.item;
        part = sw.part_nparts & 0xffff;
        nparts = sw.part_nparts >> 16;
    }
    const Item item = p.items[item_index];
    if (item.tile < 0) return;
    const Tile tile = item.t;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int h = tile.h, b = item.b;

    // What the tile's start waits for, in as few round trips as the data allows: the row numbers (this
    // thread's entry of the tile's list and the two rows whose Q fragments this lane holds) and the key
    // progressions in one go, then the Q fragments, which go out before anything else: theirs is the
    // longest wait, and the set-up of the K/V stages below runs under it.  (The plan's progression
    // array ends with one spare entry, so a tile without progressions still reads inside it.)
    const int32_t my_row = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    int32_t q_row[2] = {p.rows[tile.row_begin + min(wave * 64 + j, tile.nrows - 1)],
                        p.rows[tile.row_begin + min(wave * 64 + 32 + j, tile.nrows - 1)]};
    // a filler slot of a packed tile holds ~n of a row n of its group: loaded like any row, never stored
    if (kPacked) {
        q_row[0] ^= q_row[0] >> 31;
        q_row[1] ^= q_row[1] >> 31;
    }
    KeySeg my_seg = p.segs[tile.seg_begin + min(tid, max(tile.nseg, 1) - 1)];
    float4 my_wmult = make_float4(0.f, 0.f, 0.f, 0.f), my_wmult2 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (kPacked) {
        const float4* bm = reinterpret_cast<const float4*>(p.block_mult + 8 * (int64_t)(tile.seg_begin + min(tid, max(tile.nseg, 1) - 1)));
        my_wmult = bm[0];
        my_wmult2 = bm[1];
    }
    // held here so that the compiler does not move these loads behind the Q loads (whose wait would then
    // sit in front of the barrier)
    asm volatile("" : "+v"(my_seg.key0), "+v"(my_seg.stride), "+v"(my_seg.count), "+v"(my_seg.log2_mult));
    if (kPacked) {
        asm volatile("" : "+v"(my_wmult.x), "+v"(my_wmult.y), "+v"(my_wmult.z), "+v"(my_wmult.w));
        asm volatile("" : "+v"(my_wmult2.x), "+v"(my_wmult2.y), "+v"(my_wmult2.z), "+v"(my_wmult2.w));
    }
    // Q fragments: B operand of S^T, lane (j, g) holds Q[row j][16*kk + 8*g .. +7]
    bf16x8 qf[2][4];
    {
        const uint16_t* qp = static_cast<const uint16_t*>(p.q) + (int64_t)item.b * p.sqb + (int64_t)tile.h * p.sqh;
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                qf[qb][kk] = *reinterpret_cast<const bf16x8*>(qp + (int64_t)q_row[qb] * p.sqn + 16 * kk + 8 * g);
    }
    row_idx[tid] = my_row;
    if (tid < tile.nseg) {
        if constexpr (kPacked) {
            // wave w holds blocks 2w and 2w + 1 of the tile
            my_seg.log2_mult = my_wmult.x; seg_all[0][tid] = my_seg; bias1_all[0][tid] = my_wmult.y;
            my_seg.log2_mult = my_wmult.z; seg_all[1][tid] = my_seg; bias1_all[1][tid] = my_wmult.w;
            my_seg.log2_mult = my_wmult2.x; seg_all[2][tid] = my_seg; bias1_all[2][tid] = my_wmult2.y;
            my_seg.log2_mult = my_wmult2.z; seg_all[3][tid] = my_seg; bias1_all[3][tid] = my_wmult2.w;
        } else {
            seg_all[0][tid] = my_seg;
        }
    }
    const KeySeg* const seg_lds = seg_all[kPacked ? wave : 0];
    __syncthreads();

    OutT* const out = static_cast<OutT*>(p.out);
    float* const lse_out = p.lse;
    const int64_t out_bh = (int64_t)b * p.N * p.H + h;   // in rows; row n adds n * H
    // split launches: this workgroup's block of partial results, out [256][64] then lse [256], rows in tile order
    char* const blk = kSplit ? reinterpret_cast<char*>(p.split_ws) + (int64_t)blockIdx.x * kSplitBlockBytes : nullptr;
    float* const blk_lse = reinterpret_cast<float*>(blk + kTileRows * kD * 2);
    float* const blk_scale = blk_lse + kTileRows;
    // a tile that the split launch walks whole (one part) is finished here like in any other launch
    const bool partial = kSplit && nparts > 1;

    if (partial && tile.nseg == 0) {
        blk_lse[tid] = -INFINITY;     // the merge writes the zero rows
        return;
    }
    if (tile.nseg == 0) {
        // rows that no branch keeps: the zero matrix of Eq. 3 shows through, lse = -inf
        constexpr int kChunks = kD * sizeof(OutT) / 16;
        for (int x = tid; x < tile.nrows * kChunks; x += 256) {
            const int rr = x / kChunks, ch = x % kChunks;
            char* dst = reinterpret_cast<char*>(out + (out_bh + (int64_t)row_idx[rr] * p.H) * kD) + 16 * ch;
            *reinterpret_cast<u32x4*>(dst) = u32x4{0u, 0u, 0u, 0u};
        }
        if (lse_out && tid < tile.nrows)
            lse_out[((int64_t)b * p.H + h) * p.N + row_idx[tid]] = -INFINITY;
        return;
    }

    const uint16_t* const kp = static_cast<const uint16_t*>(p.k) + (int64_t)b * p.skb + (int64_t)h * p.skh;
    const uint16_t* const vp = static_cast<const uint16_t*>(p.v) + (int64_t)b * p.svb + (int64_t)h * p.svh;

    // What this lane fetches in each copy (see CopyLane): worked out afresh at every issue, from a copy of the
    // lane number the compiler cannot see through.  Kept across the main loop these four values are spilled
    // to scratch memory, and their reloads (vector memory operations the compiler waits for) would drain
    // the copy pipeline every step.
    auto copy_lane = [&]() {
        int ln = lane;
        asm volatile("" : "+v"(ln));
        CopyLane cl;
        const int rho = 16 * wave + (ln >> 3);                                  // LDS row of copy 0 (bit 3 clear)
        cl.kpos = (rho & 0x33) | ((rho & 4) << 1);                              // sigma(rho)
        cl.kchunk = 16 * ((ln & 7) ^ k_swizzle(rho));
        cl.vpos = rho;
        cl.vchunk = 16 * (ln & 7);
        return cl;
    };

    // what this lane reads back as MFMA fragments
    auto frag_lane = [](int ln) {
        FragLane f;
        const int jj = ln & 31, gg = ln >> 5, i16 = ln & 15;
        f.k = jj * kRowElems + 8 * (gg ^ k_swizzle(jj));
        // transposed V fragments: within a 16-lane group lane i supplies the address of
        // V[R + i/4][C + 4*(i%4) ..] and receives V[R .. R+3][C + i]
        f.v = ((i16 >> 2) + 8 * gg) * kRowElems + 16 * ((ln >> 4) & 1) + 4 * (i16 & 3);
        return f;
    };
    const FragLane fl = frag_lane(lane);

    int n_steps = tile.n_steps;

    const uint32_t k_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &k_lds[0][0]);
    const uint32_t v_lds_addr = (uint32_t)(uintptr_t)DFA_LDS_PTR(void, &v_lds[0][0]);
    constexpr uint32_t kStageBytes = kStageElems * 2;

    KeyCursor pf;
    pf.s = 0;
    pf.t = 0;
    if (kSplit) {
        // this workgroup's share of the steps: [first, last) of the tile's n_steps
        const int first = part * n_steps / nparts, last = (part + 1) * n_steps / nparts;
        n_steps = last - first;
        if (n_steps == 0) {        // a tile with fewer steps than parts: this part has no keys
            blk_lse[tid] = -INFINITY;
            return;
        }
        int skip = first;
        for (;;) {                 // ends: first < the tile's step count
            const int in_seg = (__builtin_amdgcn_readfirstlane(seg_lds[pf.s].count) + kKeyTile - 1) / kKeyTile;
            if (skip < in_seg) break;
            skip -= in_seg;
            ++pf.s;
        }
        pf.t = skip;
    }
    // the first three stages on their way before anything else
    cursor_load(pf, seg_lds);
    KeyCursor cur = pf;
#pragma unroll
    for (int s = 0; s <= 2; ++s)
        if (s < n_steps) {
            issue_stage(p, kp, vp, pf, copy_lane(), wave, k_lds_addr + s * kStageBytes, v_lds_addr + s * kStageBytes);
            cursor_next(pf, seg_lds, tile.nseg);
        }

    // pin the Q fragments here: the compiler then waits for their loads (and, as the counter is
    // shared and loads complete in order, for the stages issued after them) before the main loop and
    // places no vector-memory wait of its own inside it (it cannot see the copies, and a wait sized
    // for these eight loads would drain the copy pipeline every step)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(qf[qb][kk]));
    wait_vmcnt<0>();           // all three stages
    __syncthreads();           // stages 0 to 2 complete in LDS; from the first refill on, two stages are in flight at every wait

    // exponent scale, exp(s*x) = exp2(c*x); wave-uniform, so it is kept in a scalar register
    const float c = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, p.scale * kLog2e)));

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
    // A progression whose keys count m times adds log2(m) to its scaled scores.  That is done by holding
    // m_ref as (reference exponent - log2 m of the progression being walked) and moving it when the
    // walk enters a progression of another multiplicity; sums and accumulator stay on the true reference.
    // The start value is finite (any score moves the reference up to itself at once, the factor exp2(start - new)
    // being an exact 0): a wave whose rows skip the first progressions of a packed tile sees only masked scores
    // there, and -inf - start is a clean -inf where -inf - -inf would not be.
    float m_ref[2] = {kPacked ? kRefStart : -INFINITY, kPacked ? kRefStart : -INFINITY};
    float l_run[2] = {0.f, 0.f};               // running sum of the row (the two lanes of a query hold the same value)
    float bias_cur = 0.f;                      // log2 m held in m_ref (wave-uniform)
    // kPacked: the same per 32-row block of the wave, -inf while the block skips the progression in hand: m_ref is
    // then +inf (every exponent -inf, every numerator an exact 0, no instruction spent on it) and the block's
    // reference exponent waits in m_kept
    float bias_q[2] = {0.f, 0.f};
    float m_kept[2] = {kRefStart, kRefStart};
    float bias1 = 0.f;                         // kPacked: log2 m of the progression in hand for the second block

    const bool wave_live = wave * 64 < tile.nrows;   // waves past the end of a short tile only help copying

    // Software pipeline over 32-key blocks (two per stage).  Block 2s of step s is turned into probabilities in
    // beat A(s), block 2s+1 in beat B(s); A(s) also scores block 2s+1 and accumulates block 2s-1, B(s) scores
    // block 2s+2 and accumulates block 2s.  The first A has nothing to accumulate and the last B nothing to
    // score, so both stand outside the loop, whose trip s runs B(s) and A(s+1).
    // A operand of the row-sum products (v_mfma_f32_16x16x32_bf16 on a B operand of the second product, lane =
    // 16*g4 + n): that instruction reads lane (n, g4) as contraction slots 8*g4 .. +7 of column n, so column n
    // gathers the 8 keys each of lanes n, 16+n, 32+n, 48+n, which are query n of the block (slots 0-7 and
    // 16-23) and query 16+n (slots 8-15 and 24-31).  Result row 4*g4 goes to register 0 of lane group g4:
    // rows 0 and 8 select the slots of query n, rows 4 and 12 those of query 16+n, all other rows are zero,
    // so register 0 of every lane receives the sum over all 16 keys of its own query.  (An infinite
    // numerator of one query turns its neighbour's sum into NaN through a zero of the selector; either
    // fails the test in settle(), which then redoes the block without the matrix cores.)
    bf16x8 sel;
    {
        const int mrow = lane & 15, g4 = lane >> 4;
        const bool on = (mrow & 3) == 0 && ((mrow >> 2) & 1) == (g4 & 1);
        const uint32_t w = on ? 0x3f803f80u : 0u;
        sel = __builtin_bit_cast(bf16x8, u32x4{w, w, w, w});
    }
    floatx16 s_a[2], s_b[2];
    u32x4 p_a[2][2], p_b[2][2];
    float psum[2];
    int stage = 0;
    int nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
    // a progression whose keys count m times for this wave's rows: log2 m comes off the reference exponents held
    // in m_ref; m = 0 (log2 m = -inf): the rows do not attend to these keys, every score of the step is masked
    auto enter_step = [&]() {
        nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
        if (cur.bias != bias_cur) {            // both blocks of this step still hold raw scores
            m_ref[0] -= cur.bias - bias_cur;
            m_ref[1] -= cur.bias - bias_cur;
            bias_cur = cur.bias;
        }
    };
    auto enter_step_packed = [&](bool first) {
        nvalid = min(kKeyTile, cur.count - cur.t * kKeyTile);
        // cur.bias (from the wave's copy of the list) is the first block's figure; the second block's is read when
        // the walk enters a progression
        if (first || cur.t == 0)
            bias1 = __builtin_bit_cast(float, __builtin_amdgcn_readfirstlane(__builtin_bit_cast(int, bias1_all[wave][cur.s])));
        const float now[2] = {cur.bias, bias1};
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
            if (now[qb] != bias_q[qb]) {       // wave-uniform; both key blocks of this step still hold raw scores
                const float ref = bias_q[qb] > -INFINITY ? m_ref[qb] + bias_q[qb] : m_kept[qb];
                if (now[qb] > -INFINITY) {
                    m_ref[qb] = ref - now[qb];
                } else {
                    m_kept[qb] = ref;
                    m_ref[qb] = INFINITY;
                }
                bias_q[qb] = now[qb];
            }
    };
    if constexpr (kPacked) enter_step_packed(true); else enter_step();
    if (wave_live) {
        scores_block(k_lds[0], fl, qf, s_a);
        if (nvalid < 32) mask_block(s_a, g, nvalid);
        beat<true, false>(k_lds[0] + 32 * kRowElems, v_lds[0], fl, qf, s_a, s_b, p_b, p_a, oacc, c, m_ref, psum, sel);
        settle<kPacked>(s_a, p_a, c, m_ref, l_run, oacc, psum);
    }
    for (int s = 0; s + 1 < n_steps; ++s) {
        const int stage_prev = stage == 0 ? kStages - 1 : stage - 1;
        const int stage_next = stage == kStages - 1 ? 0 : stage + 1;
        // stage s+1 has landed once at most the 4 copies of stage s+2 are still outstanding
        if (s + 2 < n_steps) wait_vmcnt<4>(); else wait_vmcnt<0>();
        __syncthreads();       // every wave's share of stage s+1 is in LDS, and everyone is done with stage s-1
        if (s + 3 < n_steps) {
            issue_stage(p, kp, vp, pf, copy_lane(), wave, k_lds_addr + stage_prev * kStageBytes, v_lds_addr + stage_prev * kStageBytes);
            cursor_next(pf, seg_lds, tile.nseg);
        }
        if (wave_live) {
            // B(s): scores of block 2s+2, accumulation of block 2s, numerators of block 2s+1
            if (nvalid < 64) mask_block(s_b, g, nvalid - 32);
            beat<true, true>(k_lds[stage_next], v_lds[stage], fl, qf, s_b, s_a, p_a, p_b, oacc, c, m_ref, psum, sel);
            settle<kPacked>(s_b, p_b, c, m_ref, l_run, oacc, psum);
        }
        cursor_next(cur, seg_lds, tile.nseg);
        if constexpr (kPacked) enter_step_packed(false); else enter_step();
        if (wave_live) {
            // A(s+1): scores of block 2s+3, accumulation of block 2s+1, numerators of block 2s+2
            if (nvalid < 32) mask_block(s_a, g, nvalid);
            beat<true, true>(k_lds[stage_next] + 32 * kRowElems, v_lds[stage] + 32 * kRowElems, fl, qf, s_a, s_b, p_b, p_a, oacc, c, m_ref, psum, sel);
            settle<kPacked>(s_a, p_a, c, m_ref, l_run, oacc, psum);
        }
        stage = stage_next;
    }
    if (wave_live) {
        // B of the last step: accumulation of its first block, numerators of its second
        if (nvalid < 64) mask_block(s_b, g, nvalid - 32);
        beat<false, true>(k_lds[stage], v_lds[stage], fl, qf, s_b, s_a, p_a, p_b, oacc, c, m_ref, psum, sel);
        settle<kPacked>(s_b, p_b, c, m_ref, l_run, oacc, psum);
    }
    // From here on the lane constants are worked out afresh, from a copy of the lane number the
    // compiler cannot see through: carried across the loop they would cost it registers that
    // the loop needs, and spills to scratch memory.
    int lane_e = lane;
    asm volatile("" : "+v"(lane_e));
    // accumulation of the last block
    if (wave_live) {
        accumulate_block(v_lds[stage] + 32 * kRowElems, frag_lane(lane_e), p_b, oacc);
    }

    // ---- epilogue: normalise, log-sum-exp, place each row at its own token (Eq. 3)
    const int j_e = lane_e & 31, g_e = lane_e >> 5;
    float inv[2];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
        const int slot = wave * 64 + qb * 32 + j_e;
        const float l_tot = l_run[qb];
        inv[qb] = 1.0f / l_tot;
        const float ref = !kPacked ? m_ref[qb] + bias_cur : bias_q[qb] > -INFINITY ? m_ref[qb] + bias_q[qb] : m_kept[qb];
        const float lse_row = (ref + __builtin_amdgcn_logf(l_tot)) * kLn2;
        if (partial) {
            if (g_e == 0) blk_lse[slot] = slot < tile.nrows ? lse_row : -INFINITY;
        } else if (lse_out && g_e == 0 && slot < tile.nrows && (!kPacked || row_idx[slot] >= 0)) {
            lse_out[((int64_t)b * p.H + h) * p.N + row_idx[slot]] = lse_row;
        }
    }
    if (partial) {
        // Partial rows leave as fp16, each divided by its largest magnitude (kept in fp32 beside the row's lse): half
        // the bytes of fp32 rows, which is what a split launch is short of, at an error of 2^-12 of the row's largest
        // value per element.  Same detour through LDS as for bf16 rows below: whole 128-byte lines.
        typedef _Float16 halfx4 __attribute__((ext_vector_type(4)));
        float factor[2];
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = 0.f;
#pragma unroll
            for (int db = 0; db < 2; ++db)
#pragma unroll
                for (int v = 0; v < 16; ++v) mx = fmaxf(mx, fabsf(oacc[db][qb][v]));
            mx = wave_half_max(mx) * inv[qb];            // the two lanes of a query hold the halves of its row
            const float scale_row = mx > 0.f ? mx : 1.f;
            factor[qb] = inv[qb] / scale_row;
            const int slot = wave * 64 + qb * 32 + j_e;
            if (g_e == 0) blk_scale[slot] = scale_row;
        }
        __syncthreads();           // every wave is done with the stages
        constexpr int kPitch = kD * 2 + 16;
        char* mine = reinterpret_cast<char*>(wave < 2 ? &k_lds[0][0] : &v_lds[0][0]) + (wave & 1) * (64 * kPitch);
        if (wave_live) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const halfx4 o = {(_Float16)(oacc[db][qb][4 * vq] * factor[qb]), (_Float16)(oacc[db][qb][4 * vq + 1] * factor[qb]),
                                          (_Float16)(oacc[db][qb][4 * vq + 2] * factor[qb]), (_Float16)(oacc[db][qb][4 * vq + 3] * factor[qb])};
                        *reinterpret_cast<halfx4*>(mine + (32 * qb + j_e) * kPitch + (32 * db + 8 * vq + 4 * g_e) * 2) = o;
                    }
            // the wave reads back only what it wrote itself; LDS operations of a wave complete in order
            const int srow = lane_e >> 3, schunk = lane_e & 7;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int row = 8 * s + srow, slot = wave * 64 + row;
                const u32x4 val = *reinterpret_cast<const u32x4*>(mine + row * kPitch + 16 * schunk);
                if (slot < tile.nrows) *reinterpret_cast<u32x4*>(blk + slot * (kD * 2) + 16 * schunk) = val;
            }
        }
    } else if constexpr (sizeof(OutT) == 2) {
        // bf16 rows are 128 bytes.  A lane holds 4 consecutive d of one row per register quad; written
        // out directly that would be 8-byte pieces of 32 different lines per store.  Each wave
        // instead lays its 64 rows out row-major in a piece of the (now idle) K / V stages, at a
        // pitch of 144 bytes, and stores them 16 bytes per lane, eight lanes to a row: whole lines.
        __syncthreads();           // every wave is done with the stages
        constexpr int kPitch = kD * 2 + 16;
        char* mine = reinterpret_cast<char*>(wave < 2 ? &k_lds[0][0] : &v_lds[0][0]) + (wave & 1) * (64 * kPitch);
        if (wave_live) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb)
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq) {
                        const bf16x4 o = {(__bf16)(oacc[db][qb][4 * vq] * inv[qb]), (__bf16)(oacc[db][qb][4 * vq + 1] * inv[qb]),
                                          (__bf16)(oacc[db][qb][4 * vq + 2] * inv[qb]), (__bf16)(oacc[db][qb][4 * vq + 3] * inv[qb])};
                        *reinterpret_cast<bf16x4*>(mine + (32 * qb + j_e) * kPitch + (32 * db + 8 * vq + 4 * g_e) * 2) = o;
                    }
            // the wave reads back only what it wrote itself; LDS operations of a wave complete in order
            const int srow = lane_e >> 3, schunk = lane_e & 7;
#pragma unroll
            for (int s = 0; s < 8; ++s) {
                const int row = 8 * s + srow, slot = wave * 64 + row;
                const u32x4 val = *reinterpret_cast<const u32x4*>(mine + row * kPitch + 16 * schunk);
                if (slot < tile.nrows && (!kPacked || row_idx[slot] >= 0)) {
                    const int64_t n = row_idx[slot];
                    *reinterpret_cast<u32x4*>(reinterpret_cast<char*>(out + (out_bh + n * p.H) * kD) + 16 * schunk) = val;
                }
            }
        }
    } else {
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            const int slot = wave * 64 + qb * 32 + j_e;
            if (slot < tile.nrows && (!kPacked || row_idx[slot] >= 0)) {
                const int64_t n = row_idx[slot];
                OutT* op = out + (out_bh + n * p.H) * kD;
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int vq = 0; vq < 4; ++vq)
                        *reinterpret_cast<float4*>(op + 32 * db + 8 * vq + 4 * g_e) =
                            make_float4(oacc[db][qb][4 * vq] * inv[qb], oacc[db][qb][4 * vq + 1] * inv[qb],
                                        oacc[db][qb][4 * vq + 2] * inv[qb], oacc[db][qb][4 * vq + 3] * inv[qb]);
            }
        }
    }
}

// Merge of a split launch: combines the partial results of a launch item's shares by their log-sum-exp weights (the
// same formula as the stand-alone branch merge: a share is attention over a part of the row's keys) and writes the
// rows at their tokens.  Grid (items, 8): a workgroup takes 32 rows of the tile, eight lanes to a row with eight
// features each.  The shares' blocks are addressed from the item's entry of item_parts alone, so their loads go out
// together with that of the row's token (every block has all 256 rows, whatever the tile's count).
__global__ __launch_bounds__(256) void merge_split_kernel(const FwdParams p) {
    const ItemParts ip = p.item_parts[blockIdx.x];
    const Item item = p.items[blockIdx.x];
    if (ip.nparts <= 1) return;         // padding item, or a tile walked whole (its workgroup wrote the rows itself)
    const int r = blockIdx.y * 32 + (threadIdx.x >> 3), sub = threadIdx.x & 7;
    const char* blk0 = reinterpret_cast<const char*>(p.split_ws) + (int64_t)ip.first_wg * kSplitBlockBytes;
    float lb[kMaxSplit];
    typedef _Float16 halfx8 __attribute__((ext_vector_type(8)));
    float sc[kMaxSplit];
    halfx8 o[kMaxSplit];
#pragma unroll
    for (int x = 0; x < kMaxSplit; ++x) {
        lb[x] = -INFINITY;
        sc[x] = 0.f;
        o[x] = halfx8{};
        if (x < ip.nparts) {
            const char* b = blk0 + (int64_t)x * kSplitBlockBytes;
            lb[x] = reinterpret_cast<const float*>(b + kTileRows * kD * 2)[r];
            sc[x] = reinterpret_cast<const float*>(b + kTileRows * kD * 2)[kTileRows + r];
            o[x] = *reinterpret_cast<const halfx8*>(b + (r * kD + 8 * sub) * 2);
        }
    }
    const Tile tile = item.t;
    if (r >= tile.nrows) return;
    const int32_t n = p.rows[tile.row_begin + r];
    if (n < 0) return;                  // filler slot of a packed tile
    float m = -INFINITY;
#pragma unroll
    for (int x = 0; x < kMaxSplit; ++x) m = fmaxf(m, lb[x]);
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    float L = -INFINITY;
    if (m > -INFINITY) {
        float w[kMaxSplit], z = 0.f;
#pragma unroll
        for (int x = 0; x < kMaxSplit; ++x) {
            w[x] = __builtin_amdgcn_exp2f((lb[x] - m) * kLog2e);      // 0 for shares without keys
            z += w[x];
        }
        const float inv = 1.0f / z;
        L = m + __builtin_amdgcn_logf(z) * kLn2;
#pragma unroll
        for (int x = 0; x < kMaxSplit; ++x) {
            if (lb[x] == -INFINITY) continue;      // such a share has written no rows: its block holds anything
            const float ws = w[x] * inv * sc[x];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(ws, (float)o[x][e], acc[e]);
        }
    }
    bf16x8 ob;
#pragma unroll
    for (int e = 0; e < 8; ++e) ob[e] = (__bf16)acc[e];
    *reinterpret_cast<bf16x8*>(static_cast<__bf16*>(p.out) + (((int64_t)item.b * p.N + n) * p.H + tile.h) * kD + 8 * sub) = ob;
    if (p.lse && sub == 0) p.lse[((int64_t)item.b * p.H + tile.h) * p.N + n] = L;
}

}  // namespace

hipError_t launch_fwd_bf16(const FwdParams& p, int n_items, bool out_f32, bool packed, hipStream_t st) {
    if (out_f32 && packed) return hipErrorInvalidValue;      // fp32 output is launched on plain plans only
    if (out_f32)
        hipLaunchKernelGGL((dfa_fwd_bf16_kernel<float, false, false>), dim3(n_items), dim3(256), 0, st, p);
    else if (packed)
        hipLaunchKernelGGL((dfa_fwd_bf16_kernel<__bf16, false, true>), dim3(n_items), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((dfa_fwd_bf16_kernel<__bf16, false, false>), dim3(n_items), dim3(256), 0, st, p);
    return hipGetLastError();
}

// Launches with few workgroups are bound by the longest tile's walk, not by throughput: there the tiles are walked by
// several workgroups each (p.split_wgs), every one over a share of the steps, into partial results (p.split_ws)
// that launch_merge_split combines.
hipError_t launch_fwd_bf16_split(const FwdParams& p, int n_split_wgs, bool packed, hipStream_t st) {
    if (packed)
        hipLaunchKernelGGL((dfa_fwd_bf16_kernel<__bf16, true, true>), dim3(n_split_wgs), dim3(256), 0, st, p);
    else
        hipLaunchKernelGGL((dfa_fwd_bf16_kernel<__bf16, true, false>), dim3(n_split_wgs), dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t launch_merge_split(const FwdParams& p, int n_items, hipStream_t st) {
    hipLaunchKernelGGL(merge_split_kernel, dim3(n_items, kTileRows / 32), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace dfa
