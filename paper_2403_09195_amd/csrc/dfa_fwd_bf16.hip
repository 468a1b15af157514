// Fused dilated flash attention forward, bf16 on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns a tile of up to 256 query rows that share the same key lists
// (section 3.1: all of them are kept by the same branches and fall into the same segment of
// each).  It walks the key lists of its member branches one after the other, 64 keys at a
// time, carrying ONE online-softmax state (running max m, running sum l, accumulator) per
// query row across all of them: continuing the softmax over the next branch's keys is the
// log-sum-exp merge of the branches, so no partial result ever leaves the registers.
//
// Gather (Eq. 1) happens in the global->LDS loads (key j of a segment is row first + r*j),
// placement (Eq. 3) in the final store (each query row is written back at its own token).
//
// Matrix-core mapping (v_mfma_f32_32x32x16_bf16, wave64; lane = 32*g + j):
//   S^T = K~ Q~^T : A = K rows (32 keys x 16 d), B = Q^T (16 d x 32 queries).  The result puts
//                   query j in lane j: register v of lane (j, g) is key row 8*(v/4)+4*g+v%4,
//                   so a row max / row sum is 16 in-lane values plus one exchange with lane^32.
//   O^T += V~^T P^T: A = V^T (32 d x 16 keys), B = P^T (16 keys x 32 queries).  B wants 8
//                   consecutive contraction slots per lane; the S^T registers 8*st .. 8*st+7
//                   of a lane serve directly, which fixes which key sits in which slot.  V^T is
//                   stored in LDS with the keys of a 32-key block permuted (bits 2 and 3 of the
//                   position swapped relative to the MFMA row) so that a lane's 8 slots are 16
//                   contiguous bytes, and K rows are read through the same permutation.
// Each wave handles 64 query rows (two 32-row blocks), so every K / V^T fragment read from
// LDS feeds two MFMAs.
#include "dfa_device.h"

namespace dfa {

namespace {

constexpr int kLdsStride = kD + 8;   // bf16 elements per LDS row: 144 bytes, keeps 16-byte
                                     // alignment and spreads consecutive rows over the banks

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

__device__ __forceinline__ float wave_half_xchg(float x) {
    // value held by the lane that owns the other 16 keys of the same query (lane ^ 32)
    return __shfl_xor(x, 32, 64);
}

struct TileRegs {   // one 64-key K/V tile in flight between global memory and LDS
    u32x4 k[2];
    u32x2 v[4];
};

__device__ __forceinline__ void load_tile(const FwdParams& p, int64_t kbase, int64_t vbase,
                                          const KeySeg& seg, int t, int tid, TileRegs& r) {
    const uint16_t* kp = static_cast<const uint16_t*>(p.k) + kbase;
    const uint16_t* vp = static_cast<const uint16_t*>(p.v) + vbase;
    const int last = seg.count - 1;
    // K: thread -> (row tid/8 + 32u, 16-byte chunk tid%8)
#pragma unroll
    for (int u = 0; u < 2; ++u) {
        const int j = min(t * kKeyTile + (tid >> 3) + 32 * u, last);
        const int64_t row = kept_row(seg.key0, seg.stride, j);
        r.k[u] = *reinterpret_cast<const u32x4*>(kp + row * p.skn + (tid & 7) * 8);
    }
    // V: thread -> (keys 4*(tid/16) .. +3, d 4*(tid%16) .. +3)
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int j = min(t * kKeyTile + 4 * (tid >> 4) + u, last);
        const int64_t row = kept_row(seg.key0, seg.stride, j);
        r.v[u] = *reinterpret_cast<const u32x2*>(vp + row * p.svn + (tid & 15) * 4);
    }
}

__device__ __forceinline__ void store_tile(uint16_t* k_lds, uint16_t* vt_lds, int tid, const TileRegs& r) {
#pragma unroll
    for (int u = 0; u < 2; ++u)
        *reinterpret_cast<u32x4*>(k_lds + ((tid >> 3) + 32 * u) * kLdsStride + (tid & 7) * 8) = r.k[u];
    // 4x4 transpose of bf16 in registers: r.v[u] = V[key 4kq+u][d 4dq .. 4dq+3]
    const int kq = tid >> 4, dq = tid & 15;
    const uint32_t a0 = r.v[0].x, a1 = r.v[1].x, a2 = r.v[2].x, a3 = r.v[3].x;
    const uint32_t b0 = r.v[0].y, b1 = r.v[1].y, b2 = r.v[2].y, b3 = r.v[3].y;
    u32x2 o0, o1, o2, o3;
    o0.x = (a0 & 0xffffu) | (a1 << 16);          o0.y = (a2 & 0xffffu) | (a3 << 16);          // d + 0
    o1.x = (a0 >> 16) | (a1 & 0xffff0000u);      o1.y = (a2 >> 16) | (a3 & 0xffff0000u);      // d + 1
    o2.x = (b0 & 0xffffu) | (b1 << 16);          o2.y = (b2 & 0xffffu) | (b3 << 16);          // d + 2
    o3.x = (b0 >> 16) | (b1 & 0xffff0000u);      o3.y = (b2 >> 16) | (b3 & 0xffff0000u);      // d + 3
    uint16_t* base = vt_lds + (4 * dq) * kLdsStride + 4 * kq;
    *reinterpret_cast<u32x2*>(base) = o0;
    *reinterpret_cast<u32x2*>(base + kLdsStride) = o1;
    *reinterpret_cast<u32x2*>(base + 2 * kLdsStride) = o2;
    *reinterpret_cast<u32x2*>(base + 3 * kLdsStride) = o3;
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
    __shared__ __attribute__((aligned(16))) uint16_t k_lds[2][kKeyTile * kLdsStride];
    __shared__ __attribute__((aligned(16))) uint16_t vt_lds[2][kD * kLdsStride];
    __shared__ int32_t row_idx[kTileRows];

    const Item item = p.items[blockIdx.x];
    if (item.tile < 0) return;
    const Tile tile = p.tiles[item.tile];
    const int tid = threadIdx.x;
    const int wave = tid >> 6, lane = tid & 63, j = lane & 31, g = lane >> 5;
    const int h = tile.h, b = item.b;

    row_idx[tid] = p.rows[tile.row_begin + min(tid, tile.nrows - 1)];
    __syncthreads();

    OutT* const out = static_cast<OutT*>(p.out);
    const int64_t out_bh = (int64_t)b * p.N * p.H + h;   // in rows; row n adds n * H

    if (tile.nseg == 0) {
        // rows that no branch keeps: the zero matrix of Eq. 3 shows through, lse = -inf
        constexpr int kChunks = kD * sizeof(OutT) / 16;
        for (int x = tid; x < tile.nrows * kChunks; x += 256) {
            const int rr = x / kChunks, c = x % kChunks;
            char* dst = reinterpret_cast<char*>(out + (out_bh + (int64_t)row_idx[rr] * p.H) * kD) + 16 * c;
            *reinterpret_cast<u32x4*>(dst) = u32x4{0u, 0u, 0u, 0u};
        }
        if (p.lse && tid < tile.nrows)
            p.lse[((int64_t)b * p.H + h) * p.N + row_idx[tid]] = -INFINITY;
        return;
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
    }

    const int64_t kbase = (int64_t)b * p.skb + (int64_t)h * p.skh;
    const int64_t vbase = (int64_t)b * p.svb + (int64_t)h * p.svh;
    const float c = p.scale * kLog2e;          // exponent scale: exp(s*x) = exp2(c*x)

    floatx16 oacc[2][2];                       // [d block][query block], O^T layout
#pragma unroll
    for (int db = 0; db < 2; ++db)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
            for (int v = 0; v < 16; ++v) oacc[db][qb][v] = 0.f;
    float m_run[2] = {-INFINITY, -INFINITY};   // running max of c * s, per query block
    float l_run[2] = {0.f, 0.f};               // this lane's share of the running sum

    // LDS row of the key that MFMA row j reads: bits 2 and 3 swapped
    const int jperm = (j & 0x13) | ((j & 4) << 1) | ((j & 8) >> 1);

    int s = 0, t = 0, buf = 0;
    KeySeg seg = p.segs[tile.seg_begin];
    {
        TileRegs r;
        load_tile(p, kbase, vbase, seg, 0, tid, r);
        store_tile(k_lds[0], vt_lds[0], tid, r);
    }
    __syncthreads();

    while (true) {
        // next tile: same segment, or first tile of the next member branch
        int ns = s, nt = t + 1;
        bool has_next = true;
        if (nt * kKeyTile >= seg.count) {
            ns = s + 1;
            nt = 0;
            has_next = ns < tile.nseg;
        }
        KeySeg nseg = seg;
        TileRegs r;
        if (has_next) {
            if (ns != s) nseg = p.segs[tile.seg_begin + ns];
            load_tile(p, kbase, vbase, nseg, nt, tid, r);
        }

        const int nvalid = min(kKeyTile, seg.count - t * kKeyTile);
        const uint16_t* kl = k_lds[buf];
        const uint16_t* vl = vt_lds[buf];

        // ---- S^T = K~ Q~^T for 64 keys x 64 queries
        floatx16 sacc[2][2];                   // [key block][query block]
#pragma unroll
        for (int ks = 0; ks < 2; ++ks) {
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) {
                const bf16x8 kf = *reinterpret_cast<const bf16x8*>(
                    kl + (32 * ks + jperm) * kLdsStride + 16 * kk + 8 * g);
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
        }
        if (nvalid < kKeyTile) {
            // ragged end of a key list: register v of lane (j, g) is tile position
            // 32*ks + 16*(v/8) + 8*g + v%8
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int pos = 32 * ks + 16 * (v >> 3) + 8 * g + (v & 7);
                    if (pos >= nvalid) {
                        sacc[ks][0][v] = -INFINITY;
                        sacc[ks][1][v] = -INFINITY;
                    }
                }
        }

        // ---- online softmax, per query block; P^T is packed straight into B operands
        bf16x8 pb[2][2][2];                    // [key block][query block][16-key step]
#pragma unroll
        for (int qb = 0; qb < 2; ++qb) {
            float mx = sacc[0][qb][0];
#pragma unroll
            for (int v = 1; v < 16; ++v) mx = fmaxf(mx, sacc[0][qb][v]);
#pragma unroll
            for (int v = 0; v < 16; ++v) mx = fmaxf(mx, sacc[1][qb][v]);
            mx = fmaxf(mx, wave_half_xchg(mx));
            const float m_new = fmaxf(m_run[qb], mx * c);
            const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
            m_run[qb] = m_new;
            float psum = 0.f;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(sacc[ks][qb][v], c, -m_new));
                    psum += pv;
                    pb[ks][qb][v >> 3][v & 7] = (__bf16)pv;   // round to nearest even
                }
            l_run[qb] = l_run[qb] * alpha + psum;
            if (__ballot(alpha != 1.0f) != 0ull) {   // wave-uniform: skip when no max moved
#pragma unroll
                for (int db = 0; db < 2; ++db)
#pragma unroll
                    for (int v = 0; v < 16; ++v) oacc[db][qb][v] *= alpha;
            }
        }

        // ---- O^T += V~^T P^T
#pragma unroll
        for (int db = 0; db < 2; ++db)
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int st = 0; st < 2; ++st) {
                    const bf16x8 vf = *reinterpret_cast<const bf16x8*>(
                        vl + (32 * db + j) * kLdsStride + 32 * ks + 16 * st + 8 * g);
#pragma unroll
                    for (int qb = 0; qb < 2; ++qb)
                        oacc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pb[ks][qb][st], oacc[db][qb], 0, 0, 0);
                }

        if (has_next) store_tile(k_lds[buf ^ 1], vt_lds[buf ^ 1], tid, r);
        __syncthreads();
        if (!has_next) break;
        s = ns;
        t = nt;
        seg = nseg;
        buf ^= 1;
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
                p.lse[((int64_t)b * p.H + h) * p.N + n] = (m_run[qb] + __builtin_amdgcn_logf(l_tot)) * kLn2;
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
