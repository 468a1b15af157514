/*
 * dfa.h - C ABI of the MI355X (gfx950) Dilated Flash Attention forward library.
 *
 * The operation is the attention operator of SAM-Lightening, section 3.1:
 *   - Segmentation + sparsification (Eq. 1): the N tokens of one image are cut into N/w
 *     segments of length w; inside segment i the rows i*w + o + j*r (j = 0 .. w/r-1) of
 *     Q, K and V are kept.  The paper writes o = 0; here o depends on the head
 *     (o = h mod r by default, or an explicit per-head table).
 *   - Per-segment attention (Eq. 2): softmax(scale * Q~_i K~_i^T) V~_i over the kept rows.
 *     Eq. 2 prints no scale factor: pass scale = 1.0f for the literal equation,
 *     1/sqrt(D) for the usual flash-attention convention.
 *   - Recomposition (Eq. 3): results are placed at the token positions they were taken
 *     from in a zero matrix of the input's shape; rows that nothing keeps are 0.
 *   - The paper cuts the sequence into equal-length parts.  The attention entry points also
 *     take other shapes: token n lies in part floor(n / w) and is kept iff
 *     n - floor(n / w) * w - o is a non-negative multiple of r, so the last part is shorter
 *     when w does not divide N (the same as padding the sequence and giving padded keys no
 *     weight), w > N gives a single part, and r need not divide w.  The index map, gather and
 *     placement entry points keep the regular case (w <= N, N % w == 0, w % r == 0).
 *   - Several (w, r) branches are merged with their log-sum-exp weights:
 *     L = log sum_b exp(lse_b), out = sum_b exp(lse_b - L) * out_b over the branches that
 *     keep the row (the paper treats a single branch; nb = 1 reproduces it).
 *
 * Conventions shared by all entry points
 *   - Pointers marked "device" are device memory of the current HIP device, "host" are
 *     ordinary host memory read before the call returns.  The caller owns every buffer.
 *   - Work is enqueued on `stream` (a hipStream_t passed as void*; NULL = default stream)
 *     and the call returns without synchronising, unless stated otherwise.
 *   - Tensors q, k, v are addressed as base + b*stride.b + n*stride.n + h*stride.h + d
 *     (strides in elements, the D elements of one row contiguous).  Every row must start
 *     on a 16-byte boundary.  Outputs are contiguous: out [B, N, H, D], lse [B, H, N].
 *   - D must be 64.  Non-causal, no mask, no bias.
 *   - Return value: DFA_OK (0) or a negative dfa_status_t.  Argument errors are found on
 *     the host before anything is enqueued.  No C++ exception crosses this boundary.
 *   - The attention entry points keep a per-process cache of launch plans (tile lists in
 *     device memory, read-only once built, a few hundred KB each), keyed by device and
 *     problem shape.  The first call with a new shape allocates and uploads its plan
 *     (synchronously); later calls with that shape allocate nothing and only enqueue
 *     kernels, so they can be recorded into a HIP graph (call once before capturing).  The
 *     cache holds the 64 most recently used plans (at most 256 MiB); a plan that falls out is
 *     freed (which synchronises its device) once no call is using it.  dfa_release_plans()
 *     empties the cache.  Calls may come from several threads and on several streams at once:
 *     a plan is shared and never written after its upload.
 *   - Workspace.  A bf16 dfa_forward with fewer workgroups than the chip has room for (a single
 *     image, say) is faster when the long key walks are shared out over several workgroups
 *     whose partial results (out in fp16 with a scale per row, lse in fp32) are merged afterwards.  Those partial results live in a workspace that the caller
 *     owns: dfa_workspace_bytes() says how much the shape needs (0 = none), and each call that
 *     may overlap another one needs a workspace of its own.  With workspace == NULL the call
 *     runs unsplit: same results to within rounding, slower for such shapes.
 */
#ifndef DFA_H
#define DFA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DFA_MAX_BRANCHES 8
#define DFA_HEAD_DIM 64

typedef enum {
    DFA_OK = 0,
    DFA_ERR_NULL = -1,      /* a required pointer is NULL                                    */
    DFA_ERR_SHAPE = -2,     /* B, H, N <= 0; D != 64; w < 1; r < 1; head offset outside      */
                            /* [0, r); scale not finite or <= 0; for the index map, gather   */
                            /* and placement also w > N, N % w != 0, w % r != 0; for the     */
                            /* projections sizes that the tiles do not divide                */
    DFA_ERR_BRANCHES = -3,  /* nb < 1 or nb > DFA_MAX_BRANCHES                               */
    DFA_ERR_DTYPE = -4,     /* unknown dfa_dtype_t                                           */
    DFA_ERR_ALIGN = -5,     /* a base pointer or stride breaks the 16-byte row alignment     */
    DFA_ERR_LAUNCH = -6,    /* the HIP runtime refused an allocation, copy or launch         */
    DFA_ERR_TOO_LARGE = -7, /* index arithmetic would overflow the kernel's 32-bit counters  */
    DFA_ERR_WORKSPACE = -8  /* a workspace was passed that is smaller than dfa_workspace_bytes() */
} dfa_status_t;

typedef enum { DFA_BF16 = 0, DFA_F32 = 1 } dfa_dtype_t;

/* One (segment length, sparsification interval) pair of section 3.1. */
typedef struct { int32_t w; int32_t r; } dfa_branch_t;

/* Element strides of a [B, N, H, D]-addressed tensor; D is contiguous. */
typedef struct { int64_t b; int64_t n; int64_t h; } dfa_strides_t;

int dfa_version(void);
const char *dfa_error_string(int code);

/*
 * Kept-row indexer, host (Eq. 1 with the per-head start).
 * out_idx (host, int32 [H][N/r]): out_idx[h][i*(w/r) + j] = i*w + o_h + j*r.
 * head_offsets (host, int32 [H]) or NULL for o_h = h mod r.  Uses no GPU.
 */
int dfa_index_map(int32_t N, int32_t H, dfa_branch_t br, const int32_t *head_offsets,
                  int32_t *out_idx);

/*
 * The same map computed by the device indexer (the routine the gather, scatter and
 * attention kernels address kept rows with), written to d_out_idx (device, int32
 * [H][N/r]).  head_offsets is host memory or NULL.  Asynchronous on `stream`.
 */
int dfa_index_map_device(int32_t N, int32_t H, dfa_branch_t br, const int32_t *head_offsets,
                         int32_t *d_out_idx, void *stream);

/*
 * Bytes of device workspace that dfa_forward / dfa_encoder_stack use for this shape on the current
 * device (section 3.1's operator has no such notion: this is the room for the partial results
 * of a launch whose tiles are each walked by several workgroups, see "Workspace" above).  0 when the
 * shape needs none, for dt = DFA_F32, and for arguments dfa_forward would reject.  Host only: builds
 * the launch plan on the host, allocates nothing on the device; asks the current device for its
 * compute-unit count (the MI355X's when there is no device).
 */
size_t dfa_workspace_bytes(int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                           const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets);

/*
 * Main entry: gather (Eq. 1) + per-segment attention (Eq. 2) + placement (Eq. 3) +
 * log-sum-exp merge of the nb branches, in one fused kernel.
 *   q, k, v       device, dtype dt, strided as described above
 *   branches      host, nb entries; head_offsets host int32 [nb][H] or NULL (o = h mod r)
 *   out           device, dtype dt, contiguous [B, N, H, D]; rows kept by no branch get 0
 *   lse           device, fp32 contiguous [B, H, N], natural log of the sum of
 *                 exp(scale * q.k) over the row's keys (each key counted once per branch
 *                 that pairs it with the row); -inf for rows kept by no branch.  May be NULL.
 *   workspace     device, 16-byte aligned, at least dfa_workspace_bytes() of this shape, written and
 *                 read by this call only (contents need not be kept between calls); or NULL.  Too
 *                 small a non-NULL workspace is DFA_ERR_WORKSPACE.
 * dt = DFA_BF16: bf16 operands on the matrix cores, fp32 accumulation and softmax
 * statistics, probabilities rounded to bf16 before the product with V, result rounded to
 * bf16.  The softmax denominator is the fp32 sum of those rounded probabilities, so out is
 * their exact weighted mean of V rows, and lse is within 2^-8 (3.9e-3) of the exact value
 * in the worst case (one key carrying the row), a few 1e-4 when many keys share the
 * weight.  dt = DFA_F32: fp32 throughout.
 */
int dfa_forward(const void *q, const void *k, const void *v,
                dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets,
                void *out, float *lse, void *workspace, size_t workspace_bytes, void *stream);

/*
 * dfa_forward for callers that cannot allocate device memory (code under HIP graph capture set-up rules,
 * tight serving loops, harnesses that forbid hipMalloc): same arguments without the workspace, same kernels
 * and same results as dfa_forward with a workspace, but it never calls hipMalloc / hipFree or anything else
 * that allocates device memory.  The launch plan and the partial results of a split launch live in a static
 * device array of DFA_STATIC_SCRATCH_BYTES (40 MiB) that each GPU the entry point runs on holds until the
 * process ends; a shape whose plan and partial results do not fit returns DFA_ERR_WORKSPACE before anything
 * is enqueued (every shape that is split fits; the limit is met by plans of some 700 000 workgroups).
 * The first call with a shape other than the previous call's on that GPU synchronises the device and copies
 * the new plan in (not capturable; call once before capturing); calls that repeat the shape only enqueue.
 * All calls on one GPU share the array: calls that overlap on one GPU (two streams, two threads) race on it
 * and must be serialised by the caller.
 */
#define DFA_STATIC_SCRATCH_BYTES ((size_t)40 << 20)
int dfa_forward_static(const void *q, const void *k, const void *v,
                       dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                       int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                       const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets,
                       void *out, float *lse, void *stream);

/*
 * Backward of dfa_forward: gradients with respect to q, k, v for a gradient dout of the merged
 * output (lse takes no gradient).  The paper gives no backward pass; this is the chain rule on
 * Eq. 2 and the branch merge: with P = exp(scale q_n.k_j - lse_n) per (branch, n, j) pair of
 * the definition and delta_n = dout_n . out_n,  dv_j += P dout_n,  ds = P (dout_n . v_j - delta_n),
 * dq_n += scale ds k_j,  dk_j += scale ds q_n.
 *   q, k, v, strides, shapes, dt, scale, branches, head_offsets   exactly as passed to dfa_forward
 *   out, lse       device, what dfa_forward returned (out dtype dt [B, N, H, D], lse fp32 [B, H, N])
 *   dout           device, dtype dt, contiguous [B, N, H, D]
 *   delta_ws       device, fp32 [2][B, H, N] workspace (receives -(dout . out) and lse * log2(e) per row)
 *   dq, dk, dv     device, dtype dt, contiguous [B, N, H, D]; rows kept by no branch get 0
 * dt = DFA_BF16: bf16 operands on the matrix cores, fp32 accumulation, P and dS rounded to bf16
 * before their second products, gradients rounded to bf16.  dt = DFA_F32: fp32 vector arithmetic
 * (correctness path).  Two (bf16) or four (fp32) launches on `stream`; uses the plan cache of dfa_forward.
 */
int dfa_backward(const void *q, const void *k, const void *v, const void *out, const float *lse,
                 const void *dout, dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                 int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                 const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets,
                 float *delta_ws, void *dq, void *dk, void *dv, void *stream);

/*
 * One branch, unmerged (Eq. 1-3 for a single (w, r)): out_b device fp32 [B, N, H, D]
 * (0 on rows the branch does not keep), lse_b device fp32 [B, H, N] (-inf there).
 * head_offsets host int32 [H] or NULL.  Inputs of dtype dt as in dfa_forward.
 */
int dfa_forward_branch(const void *q, const void *k, const void *v,
                       dfa_strides_t sq, dfa_strides_t sk, dfa_strides_t sv,
                       int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt, float scale,
                       dfa_branch_t br, const int32_t *head_offsets,
                       float *out_b, float *lse_b, void *stream);

/*
 * Stand-alone log-sum-exp merge of nb unmerged branch results.
 *   out_b device fp32 [nb][B, N, H, D], lse_b device fp32 [nb][B, H, N]
 *   out   device dtype dt [B, N, H, D], lse device fp32 [B, H, N] (may be NULL)
 */
int dfa_merge(const float *out_b, const float *lse_b, int32_t nb,
              int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
              void *out, float *lse, void *stream);

/*
 * Stand-alone gather (Eq. 1): kept rows of one strided tensor x into a dense
 * xg (device, dtype dt, contiguous [B, H, N/r, D]), rows in index-map order.
 */
int dfa_gather(const void *x, dfa_strides_t sx, int32_t B, int32_t H, int32_t N, int32_t D,
               dfa_dtype_t dt, dfa_branch_t br, const int32_t *head_offsets,
               void *xg, void *stream);

/*
 * Stand-alone placement (the MAP of Eq. 3): dense og (device, dtype dt, [B, H, N/r, D])
 * back to token positions in out (device, dtype dt, contiguous [B, N, H, D]); rows the
 * branch does not keep are written as 0, so out needs no initialisation.
 */
int dfa_scatter(const void *og, int32_t B, int32_t H, int32_t N, int32_t D, dfa_dtype_t dt,
                dfa_branch_t br, const int32_t *head_offsets, void *out, void *stream);

/*
 * Host-side view of the launch plan of the fp32 forward kernel and of dfa_backward (no GPU needed;
 * the bf16 dfa_forward refines it, see dfa_plan_describe_forward): the query
 * rows of each head are grouped by the set of (branch, segment) pairs that keep them and
 * cut into tiles; every tile carries its keys as arithmetic progressions: one per member
 * branch, or, where the member branches keep some keys more than once, the multiset union of
 * those cut into progressions of one multiplicity each (a key kept by m branches is visited
 * once and its softmax weight multiplied by m: the same sum as m visits, section 3.1's merge
 * being a softmax over the multiset union of the branches' keys).
 * Pass NULL arrays to query the sizes only.
 *   n_tiles, n_rows, n_segs, n_items   out, host: entry counts
 *   tiles  host int32 [n_tiles][6] = (h, row_begin, nrows, seg_begin, nseg, 64-key steps of the list)
 *   rows   host int32 [n_rows]     token positions, tile after tile
 *   segs   host int32 [n_segs][4]  = (first key, key stride, key count, multiplicity)
 *   items  host int32 [n_items][2] = (tile or -1 for padding, b) in launch order
 */
int dfa_plan_describe(int32_t B, int32_t H, int32_t N, const dfa_branch_t *branches, int32_t nb,
                      const int32_t *head_offsets, int32_t *n_tiles, int32_t *n_rows,
                      int32_t *n_segs, int32_t *n_items, int32_t *tiles, int32_t *rows,
                      int32_t *segs, int32_t *items);

/*
 * The same view of the plan the bf16 dfa_forward launches.  It differs where row groups fill only part of a
 * 256-row tile (small images: the rows of one window of the narrowest branch fall into several groups by which
 * dilated branches also keep them): groups that share most of their keys are packed into one tile, each group
 * on 32-row blocks of its own (half a wave: the unit with its own softmax state), and the tile walks the union of
 * their key lists once.  A progression then has a multiplicity per block, 0 where that block's rows do not attend
 * to its keys (their scores are masked).
 * Arguments as dfa_plan_describe, with
 *   rows       an entry < 0 is a filler slot between two groups of a packed tile (it holds ~n of a row n of the
 *              group before it; nothing is stored for it)
 *   segs       [n_segs][4] = (first key, key stride, key count, largest multiplicity over the blocks)
 *   block_mult host int32 [n_segs][8]: multiplicity of the progression's keys for the rows of block 0..7
 *              (slots 32k .. 32k+31 of the tile); NULL to skip
 */
int dfa_plan_describe_forward(int32_t B, int32_t H, int32_t N, const dfa_branch_t *branches, int32_t nb,
                              const int32_t *head_offsets, int32_t *n_tiles, int32_t *n_rows,
                              int32_t *n_segs, int32_t *n_items, int32_t *tiles, int32_t *rows,
                              int32_t *segs, int32_t *block_mult, int32_t *items);

/*
 * Projection either side of the operator inside an encoder layer (the ViT self-attention
 * block the paper's encoder is built from, section 3.1): y = x . w^T, one weight ROW per
 * output feature, no bias.  bf16 operands on the matrix cores, fp32 accumulation, y rounded
 * to bf16.
 *   x device bf16 [M][K] with row pitch ldx, w device bf16 [N][K] with row pitch ldw,
 *   y device bf16 [M][N] with row pitch ldy (pitches in elements, each a multiple of 8;
 *   base pointers 16-byte aligned).  M % 256 == 0, N % 128 == 0, K % 64 == 0, else
 *   DFA_ERR_SHAPE.  y must not overlap x or w.  Asynchronous on `stream`.
 */
int dfa_linear(const void *x, const void *w, void *y, int64_t M, int32_t N, int32_t K,
               int64_t ldx, int64_t ldw, int64_t ldy, void *stream);

/*
 * `layers` encoder attention layers back to back (the "encoder attention stack" workload):
 * per layer  qkv = x_l . w_qkv[l]^T  (features ordered [3][H][D]: q heads, k heads, v heads),
 * attn = dfa_forward(q, k, v read in place from qkv through strides),  x_{l+1} = attn . w_o[l]^T.
 * No bias, residual or normalisation.  E = H * D.
 *   x        device bf16 [B][N][E], read only
 *   w_qkv    device bf16 [layers][3E][E];  w_o  device bf16 [layers][E][E]
 *   qkv_ws   device bf16 [B][N][3][H][D]   workspace, holds the last layer's qkv on return
 *   attn_ws  device bf16 [B][N][H][D]      workspace, holds the last layer's attention output
 *   y        device bf16 [B][N][E]         x_layers; also used for every intermediate x_l
 *                                          (y may be the same buffer as x: x is then overwritten)
 *   branches, head_offsets, scale, workspace, workspace_bytes    as in dfa_forward (one workspace
 *                                          serves every layer)
 * (B * N) % 256 == 0 and E % 128 == 0 are required (DFA_ERR_SHAPE otherwise); D must be 64.
 * Every argument is checked before the first launch.  Three launches per layer on `stream` (four
 * where the attention launch is split); allocates only what the plan cache allocates on first use.
 */
int dfa_encoder_stack(const void *x, const void *w_qkv, const void *w_o, int32_t layers,
                      int32_t B, int32_t H, int32_t N, int32_t D, float scale,
                      const dfa_branch_t *branches, int32_t nb, const int32_t *head_offsets,
                      void *qkv_ws, void *attn_ws, void *y, void *workspace, size_t workspace_bytes,
                      void *stream);

/* Empties the plan cache of every device; a plan is freed (its device synchronised) as soon as no
 * call is using it any more. */
int dfa_release_plans(void);

#ifdef __cplusplus
}
#endif
#endif /* DFA_H */
