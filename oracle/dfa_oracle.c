/*
 * fp64 CPU oracle for Dilated Flash Attention (SAM-Lightening, section 3.1).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  It shares no code with the GPU path and is
 * called only from tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * What it computes, for every batch b and head h independently:
 *   1. Segmentation + sparsification (section 3.1, Eq. 1): the N tokens are cut
 *      into N/w segments of length w; inside segment i the rows
 *      i*w + o + j*r, j = 0 .. w/r-1, are kept.  The paper writes the case
 *      o = 0; the per-head start o = h mod r (or an explicit table) is the
 *      workload definition's extension.  The same rows are taken from Q, K, V.
 *   2. Per-segment attention (Eq. 2): softmax(scale * Q~ K~^T) V~ over the kept
 *      rows of one segment.  Eq. 2 prints no scale; `scale` is an argument
 *      (1.0 reproduces Eq. 2 literally, 1/sqrt(D) is the usual convention).
 *   3. Recomposition (Eq. 3 and its steps (1)-(3)): a zero matrix of the input's
 *      shape receives every segment's rows at the token positions they were
 *      taken from; rows that no segment keeps stay zero (their lse is -inf).
 *      The paper cuts the sequence into "equal-length parts"; where w does not
 *      divide N the attention functions take the last part shorter (the same as
 *      padding the sequence to a multiple of w and giving padded keys weight
 *      zero), w > N gives one part, and where r does not divide w a part keeps
 *      its rows o, o + r, o + 2r, ... below its end.  Token n is in part
 *      floor(n / w) and is kept iff n - floor(n / w) * w - o is a non-negative
 *      multiple of r.  The index map keeps the regular case only (w | N, r | w).
 *   4. Branch merge (workload definition; the paper treats one (w, r) only):
 *      L = log sum_b exp(lse_b), out = sum_b exp(lse_b - L) * out_b over the
 *      branches that keep the row.
 *
 * All arithmetic is fp64; nothing is tiled, fused or reordered beyond the
 * loops above.  Layouts: q, k, v, out are [B, N, H, D] contiguous; lse is
 * [B, H, N].  Every function returns 0 on success, -1 on bad arguments.
 *
 * Parity pins (tests marked "not gpu"): dense-softmax closed form for w = N,
 * r = 1; brute-force multiplicity-weighted softmax on tiny inputs; softmax
 * rows summing to one; merge of disjoint branches = attention over the union;
 * zero-query closed form; locality and key-shift invariants.  No function
 * here is unpinned.
 */
#include <math.h>
#include <stdlib.h>
#include <string.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static int branch_ok(int N, int w, int r) {
    return N > 0 && w > 0 && r > 0 && w <= N && (N % w) == 0 && (w % r) == 0;
}

/* The attention functions also take ragged partitions (see the header). */
static int branch_general_ok(int N, int w, int r) {
    return N > 0 && w > 0 && r > 0;
}

/* Kept rows of part i of a branch, ascending, into rows[]; returns how many. */
static int kept_rows_of_part(int N, int w, int r, int o, int i, int *rows) {
    const long long first = (long long)i * w + o;
    long long end = (long long)(i + 1) * w;
    if (end > N) end = N;
    int n_keep = 0;
    for (long long n = first; n < end; n += r) rows[n_keep++] = (int)n;
    return n_keep;
}

static int head_offset(const int *head_offsets, int h, int r) {
    return head_offsets ? head_offsets[h] : (h % r);
}

int dfa_oracle_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Eq. 1 with the per-head start: idx[h][i*(w/r) + j] = i*w + o_h + j*r. */
int dfa_oracle_index_map(int N, int H, int w, int r, const int *head_offsets, int *idx) {
    if (!branch_ok(N, w, r) || H <= 0 || !idx) return -1;
    const int per_seg = w / r;
    for (int h = 0; h < H; ++h) {
        const int o = head_offset(head_offsets, h, r);
        if (o < 0 || o >= r) return -1;
        for (int i = 0; i < N / w; ++i)
            for (int j = 0; j < per_seg; ++j)
                idx[(size_t)h * (N / r) + (size_t)i * per_seg + j] = i * w + o + j * r;
    }
    return 0;
}

/*
 * Eq. 2 for one sparsified segment: `rows` lists the n_keep kept token
 * positions; attention of each kept query over all kept keys.  Writes the
 * result rows and their log-sum-exp straight to the token positions they came
 * from (the MAP of Eq. 3).  If probs != NULL it receives the n_keep x n_keep
 * softmax matrix (debug aid for the rows-sum-to-one pin).
 */
static void segment_attention(const double *q, const double *k, const double *v,
                              size_t tok_stride, int D, double scale,
                              const int *rows, int n_keep,
                              double *out, double *lse, double *t, double *probs) {
    for (int a = 0; a < n_keep; ++a) {
        const double *qa = q + (size_t)rows[a] * tok_stride;
        double m = -INFINITY;
        for (int c = 0; c < n_keep; ++c) {
            const double *kc = k + (size_t)rows[c] * tok_stride;
            double s = 0.0;
            for (int d = 0; d < D; ++d) s += qa[d] * kc[d];
            s *= scale;
            t[c] = s;
            if (s > m) m = s;
        }
        double l = 0.0;
        for (int c = 0; c < n_keep; ++c) {
            t[c] = exp(t[c] - m);
            l += t[c];
        }
        double *oa = out + (size_t)rows[a] * tok_stride;
        for (int d = 0; d < D; ++d) oa[d] = 0.0;
        for (int c = 0; c < n_keep; ++c) {
            const double p = t[c] / l;
            const double *vc = v + (size_t)rows[c] * tok_stride;
            for (int d = 0; d < D; ++d) oa[d] += p * vc[d];
            if (probs) probs[(size_t)a * n_keep + c] = p;
        }
        lse[rows[a]] = m + log(l);
    }
}

/*
 * One (w, r) branch, unmerged: out_b [B,N,H,D] (zero where no segment keeps the
 * row), lse_b [B,H,N] (-inf there).
 */
int dfa_oracle_branch(const double *q, const double *k, const double *v,
                      int B, int H, int N, int D, double scale,
                      int w, int r, const int *head_offsets,
                      double *out_b, double *lse_b) {
    if (!q || !k || !v || !out_b || !lse_b || B <= 0 || H <= 0 || D <= 0 || !branch_general_ok(N, w, r)) return -1;
    for (int h = 0; h < H; ++h) {
        const int o = head_offset(head_offsets, h, r);
        if (o < 0 || o >= r) return -1;
    }
    const size_t tok = (size_t)H * D;
    const int per_seg = (w < N ? w : N) / r + 1;                   /* room for the kept rows of one part */
    const int n_parts = (N + w - 1) / w;
    memset(out_b, 0, sizeof(double) * (size_t)B * N * H * D);      /* O_init = 0 */
    for (size_t x = 0; x < (size_t)B * H * N; ++x) lse_b[x] = -INFINITY;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int *rows = (int *)malloc(sizeof(int) * per_seg);
            double *t = (double *)malloc(sizeof(double) * per_seg);
            if (!rows || !t) {
                failed = 1;
            } else {
                const int o = head_offset(head_offsets, h, r);
                const size_t base = (size_t)b * N * tok + (size_t)h * D;
                for (int i = 0; i < n_parts; ++i) {
                    const int n_keep = kept_rows_of_part(N, w, r, o, i, rows);
                    segment_attention(q + base, k + base, v + base, tok, D, scale, rows, n_keep,
                                      out_b + base, lse_b + ((size_t)b * H + h) * N, t, NULL);
                }
            }
            free(rows);
            free(t);
        }
    }
    return failed ? -1 : 0;
}

/* Softmax matrix of one segment of one (b, h): probs [w/r, w/r]. Debug aid. */
int dfa_oracle_segment_probs(const double *q, const double *k, const double *v,
                             int B, int H, int N, int D, double scale,
                             int w, int r, int offset, int b, int h, int seg, double *probs) {
    if (!q || !k || !v || !probs || !branch_ok(N, w, r) || offset < 0 || offset >= r) return -1;
    if (b < 0 || b >= B || h < 0 || h >= H || seg < 0 || seg >= N / w) return -1;
    const size_t tok = (size_t)H * D;
    const int per_seg = w / r;
    int *rows = (int *)malloc(sizeof(int) * per_seg);
    double *t = (double *)malloc(sizeof(double) * per_seg);
    double *o_tmp = (double *)calloc((size_t)N * tok, sizeof(double));
    double *l_tmp = (double *)malloc(sizeof(double) * N);
    if (!rows || !t || !o_tmp || !l_tmp) { free(rows); free(t); free(o_tmp); free(l_tmp); return -1; }
    for (int j = 0; j < per_seg; ++j) rows[j] = seg * w + offset + j * r;
    const size_t base = (size_t)b * N * tok + (size_t)h * D;
    segment_attention(q + base, k + base, v + base, tok, D, scale, rows, per_seg,
                      o_tmp + (size_t)h * D, l_tmp, t, probs);
    free(rows); free(t); free(o_tmp); free(l_tmp);
    return 0;
}

/*
 * Log-sum-exp merge of nb branch results.  out_b is [nb][rows][D], lse_b is
 * [nb][rows] (rows = any flattening shared by both), out [rows][D], lse [rows].
 * A branch with lse = -inf does not take part; a row no branch keeps gives
 * out = 0, lse = -inf.
 */
int dfa_oracle_merge(int nb, size_t rows, int D, const double *out_b, const double *lse_b,
                     double *out, double *lse) {
    if (nb <= 0 || D <= 0 || !out_b || !lse_b || !out || !lse) return -1;
    for (size_t x = 0; x < rows; ++x) {
        double m = -INFINITY;
        for (int b = 0; b < nb; ++b) {
            const double l = lse_b[(size_t)b * rows + x];
            if (l > m) m = l;
        }
        double *o = out + x * D;
        for (int d = 0; d < D; ++d) o[d] = 0.0;
        if (m == -INFINITY) { lse[x] = -INFINITY; continue; }
        double z = 0.0;
        for (int b = 0; b < nb; ++b) z += exp(lse_b[(size_t)b * rows + x] - m);
        const double L = m + log(z);
        for (int b = 0; b < nb; ++b) {
            const double l = lse_b[(size_t)b * rows + x];
            if (l == -INFINITY) continue;
            const double wgt = exp(l - L);
            const double *ob = out_b + ((size_t)b * rows + x) * D;
            for (int d = 0; d < D; ++d) o[d] += wgt * ob[d];
        }
        lse[x] = L;
    }
    return 0;
}

/*
 * Whole operator: every branch, then the merge.  head_offsets is NULL
 * (o = h mod r) or [nb][H].  branch_out / branch_lse may be NULL, else they
 * receive the per-branch results ([nb][B,N,H,D] and [nb][B,H,N]).
 * The merge works on rows flattened as (b, n, h) for out and (b, h, n) for lse,
 * so the branch lse planes are transposed to (b, n, h) order first.
 */
int dfa_oracle_forward(const double *q, const double *k, const double *v,
                       int B, int H, int N, int D, double scale,
                       int nb, const int *w, const int *r, const int *head_offsets,
                       double *out, double *lse, double *branch_out, double *branch_lse) {
    if (nb <= 0 || !w || !r || !out || !lse) return -1;
    const size_t rows = (size_t)B * N * H;
    double *ob = branch_out ? branch_out : (double *)malloc(sizeof(double) * rows * D * nb);
    double *lb = branch_lse ? branch_lse : (double *)malloc(sizeof(double) * rows * nb);
    double *lt = (double *)malloc(sizeof(double) * rows * nb);   /* lse in (b,n,h) order */
    double *lm = (double *)malloc(sizeof(double) * rows);
    int rc = (ob && lb && lt && lm) ? 0 : -1;
    for (int x = 0; rc == 0 && x < nb; ++x)
        rc = dfa_oracle_branch(q, k, v, B, H, N, D, scale, w[x], r[x],
                               head_offsets ? head_offsets + (size_t)x * H : NULL,
                               ob + (size_t)x * rows * D, lb + (size_t)x * rows);
    if (rc == 0) {
        for (int x = 0; x < nb; ++x)
            for (int b = 0; b < B; ++b)
                for (int h = 0; h < H; ++h)
                    for (int n = 0; n < N; ++n)
                        lt[(size_t)x * rows + ((size_t)b * N + n) * H + h] =
                            lb[(size_t)x * rows + ((size_t)b * H + h) * N + n];
        rc = dfa_oracle_merge(nb, rows, D, ob, lt, out, lm);
        if (rc == 0)
            for (int b = 0; b < B; ++b)
                for (int h = 0; h < H; ++h)
                    for (int n = 0; n < N; ++n)
                        lse[((size_t)b * H + h) * N + n] = lm[((size_t)b * N + n) * H + h];
    }
    if (!branch_out) free(ob);
    if (!branch_lse) free(lb);
    free(lt);
    free(lm);
    return rc;
}

/*
 * The same operator for a list of sampled output rows only (full-size parity
 * checks): bhn is [n_rows][3] = (b, h, n); out_rows [n_rows][D]; lse_rows
 * [n_rows].  Per row: for every branch that keeps token n, attention of q_n
 * over the kept keys of n's segment (Eq. 1-2), then the merge.
 */
int dfa_oracle_forward_rows(const double *q, const double *k, const double *v,
                            int B, int H, int N, int D, double scale,
                            int nb, const int *w, const int *r, const int *head_offsets,
                            int n_rows, const int *bhn, double *out_rows, double *lse_rows) {
    if (!q || !k || !v || nb <= 0 || !w || !r || !bhn || !out_rows || !lse_rows || D <= 0) return -1;
    for (int x = 0; x < nb; ++x) if (!branch_general_ok(N, w[x], r[x])) return -1;
    const size_t tok = (size_t)H * D;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int a = 0; a < n_rows; ++a) {
        const int b = bhn[3 * a], h = bhn[3 * a + 1], n = bhn[3 * a + 2];
        double *ob = (double *)malloc(sizeof(double) * nb * D);
        double *lb = (double *)malloc(sizeof(double) * nb);
        double *t = (double *)malloc(sizeof(double) * N);
        if (!ob || !lb || !t || b < 0 || b >= B || h < 0 || h >= H || n < 0 || n >= N) {
            failed = 1;
        } else {
            const size_t base = (size_t)b * N * tok + (size_t)h * D;
            const double *qn = q + base + (size_t)n * tok;
            for (int x = 0; x < nb; ++x) {
                const int o = head_offset(head_offsets ? head_offsets + (size_t)x * H : NULL, h, r[x]);
                const int seg = n / w[x];
                const int pos = n - seg * w[x] - o;
                lb[x] = -INFINITY;
                for (int d = 0; d < D; ++d) ob[x * D + d] = 0.0;
                if (pos < 0 || pos % r[x] != 0) continue;           /* row not kept by this branch */
                long long part_end = (long long)(seg + 1) * w[x];
                if (part_end > N) part_end = N;
                const int per_seg = (int)((part_end - 1 - ((long long)seg * w[x] + o)) / r[x]) + 1;
                double m = -INFINITY;
                for (int j = 0; j < per_seg; ++j) {
                    const double *kc = k + base + (size_t)(seg * w[x] + o + j * r[x]) * tok;
                    double s = 0.0;
                    for (int d = 0; d < D; ++d) s += qn[d] * kc[d];
                    t[j] = s * scale;
                    if (t[j] > m) m = t[j];
                }
                double l = 0.0;
                for (int j = 0; j < per_seg; ++j) { t[j] = exp(t[j] - m); l += t[j]; }
                for (int j = 0; j < per_seg; ++j) {
                    const double *vc = v + base + (size_t)(seg * w[x] + o + j * r[x]) * tok;
                    const double p = t[j] / l;
                    for (int d = 0; d < D; ++d) ob[x * D + d] += p * vc[d];
                }
                lb[x] = m + log(l);
            }
            dfa_oracle_merge(nb, 1, D, ob, lb, out_rows + (size_t)a * D, lse_rows + a);
        }
        free(ob); free(lb); free(t);
    }
    return failed ? -1 : 0;
}


/*
 * Gradients of the operator with respect to q, k and v for a given gradient dout of its
 * output (lse takes no gradient).  The paper states no backward pass (it distils through
 * the FlashAttention library, section 4.3); this is the chain rule applied to Eq. 2 and the
 * branch merge.  The merged operator is a softmax over the multiset union of a row's key
 * sets:  out_n = sum over branches x and keys j of part_x(n) of P_x(n,j) v_j  with
 * P_x(n,j) = exp(scale q_n.k_j - lse_n), lse_n the merged log-sum-exp.  With
 * delta_n = dout_n . out_n:
 *   dv_j += P dout_n
 *   ds    = P (dout_n . v_j - delta_n)
 *   dq_n += scale ds k_j,   dk_j += scale ds q_n
 * summed over every (branch, n, j) pair of the definition.  Plain loops, fp64; one (b, h) per
 * thread.  dq, dk, dv are [B,N,H,D] like q.
 */
int dfa_oracle_backward(const double *q, const double *k, const double *v, const double *dout,
                        int B, int H, int N, int D, double scale,
                        int nb, const int *w, const int *r, const int *head_offsets,
                        double *dq, double *dk, double *dv) {
    if (!q || !k || !v || !dout || !dq || !dk || !dv || nb <= 0 || !w || !r || B <= 0 || H <= 0 || D <= 0) return -1;
    for (int x = 0; x < nb; ++x) if (!branch_general_ok(N, w[x], r[x])) return -1;
    const size_t total = (size_t)B * N * H * D, rows_total = (size_t)B * N * H;
    double *out = (double *)malloc(sizeof(double) * total);
    double *lse = (double *)malloc(sizeof(double) * rows_total);
    if (!out || !lse) { free(out); free(lse); return -1; }
    int rc = dfa_oracle_forward(q, k, v, B, H, N, D, scale, nb, w, r, head_offsets, out, lse, NULL, NULL);
    if (rc != 0) { free(out); free(lse); return rc; }
    memset(dq, 0, sizeof(double) * total);
    memset(dk, 0, sizeof(double) * total);
    memset(dv, 0, sizeof(double) * total);
    const size_t tok = (size_t)H * D;
    int failed = 0;
#pragma omp parallel for collapse(2) schedule(dynamic, 1)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int *rows = (int *)malloc(sizeof(int) * (N + 1));
            if (!rows) { failed = 1; continue; }
            const size_t base = (size_t)b * N * tok + (size_t)h * D;
            const double *L = lse + ((size_t)b * H + h) * N;
            for (int x = 0; x < nb; ++x) {
                const int o = head_offset(head_offsets ? head_offsets + (size_t)x * H : NULL, h, r[x]);
                const int n_parts = (N + w[x] - 1) / w[x];
                for (int i = 0; i < n_parts; ++i) {
                    const int n_keep = kept_rows_of_part(N, w[x], r[x], o, i, rows);
                    for (int a = 0; a < n_keep; ++a) {
                        const size_t rn = base + (size_t)rows[a] * tok;
                        double delta = 0.0;
                        for (int d = 0; d < D; ++d) delta += dout[rn + d] * out[rn + d];
                        for (int c = 0; c < n_keep; ++c) {
                            const size_t rj = base + (size_t)rows[c] * tok;
                            double t = 0.0, dp = 0.0;
                            for (int d = 0; d < D; ++d) { t += q[rn + d] * k[rj + d]; dp += dout[rn + d] * v[rj + d]; }
                            const double P = exp(scale * t - L[rows[a]]);
                            const double ds = P * (dp - delta);
                            for (int d = 0; d < D; ++d) {
                                dv[rj + d] += P * dout[rn + d];
                                dq[rn + d] += scale * ds * k[rj + d];
                                dk[rj + d] += scale * ds * q[rn + d];
                            }
                        }
                    }
                }
            }
            free(rows);
        }
    }
    free(out);
    free(lse);
    return failed ? -1 : 0;
}
