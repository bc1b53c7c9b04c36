/*
 * fp64 CPU oracle for the partial self-attention of one sequence segment
 * (LSS Transformer, Section 3 "Principle 3", Eq. 2; the full-sequence case
 * s0 = 0, l_s = l_x is Eq. 1 of Section 2.2).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the checker for the HIP library, not a
 * fallback for it: only tests, the smoke entry and the benchmark's
 * cpu_baseline leg may call it.  It shares no code with the HIP path.
 *
 * The method is exact (Section 3, Principle 3: concatenating per-segment
 * outputs equals the sequential result), so the oracle is the definition
 * written out: plain loops, two-pass softmax (max, then sum), nothing tiled,
 * nothing fused, nothing online.  Everything is double precision.
 *
 * Layout of every activation: [B, L, H, d] contiguous, d fastest (token-major
 * rows of E_m = H*d columns, the paper's l x E_m matrices; one head is a
 * column slice of width d = E_m / H).  lse is [B, H, l_s].
 *
 * Readings of points the paper leaves open:
 *   - d_k of Eq. 1 is the per-head width d; scores are divided by sqrt(d).
 *   - "decoder-only (GPT)" (Section 5.1) means a causal mask: the query at
 *     global position g = s0 + r sees keys j <= g.  Masked pairs have weight
 *     exactly 0 (they are simply left out of the sums).
 *   - no dropout on the attention weights in the functions of the headline
 *     path; the *_dropout functions at the end of this file add it.
 *   - the backward pass is the textbook gradient of Eq. 2; a segment's
 *     dK/dV "partial" is the contribution of its own query rows only, and the
 *     sum over segments (the arithmetic of the reduce-scatter in Fig. 2(v))
 *     is the full-sequence gradient.
 *
 * Threads: OpenMP over query rows, and over key rows for dK/dV.  Every sum
 * is taken by one thread in increasing index order, so results do not depend
 * on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define IDX4(b, l, h, c, L, H, d) ((((int64_t)(b) * (L) + (l)) * (H) + (h)) * (d) + (c))

int lss_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* number of keys visible to local row r of segment (s0, .): Eq. 2 with the
 * causal reading above; all l_x keys when not causal. */
static int64_t visible(int64_t s0, int64_t r, int64_t l_x, int causal)
{
    if (!causal) return l_x;
    int64_t n = s0 + r + 1;
    return n < l_x ? n : l_x;
}

/* One row of Eq. 2: scores S[j], their softmax P[j] and lse.  P must hold nj. */
static double row_softmax(const double *q_row, const double *k, int64_t b, int64_t h,
                          int64_t l_x, int64_t H, int64_t d, int64_t nj, double *P)
{
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    double m = -INFINITY;
    for (int64_t j = 0; j < nj; ++j) {
        const double *k_row = k + IDX4(b, j, h, 0, l_x, H, d);
        double s = 0.0;
        for (int64_t c = 0; c < d; ++c) s += q_row[c] * k_row[c];
        s *= inv_sqrt_d;
        P[j] = s;
        if (s > m) m = s;
    }
    double ell = 0.0;
    for (int64_t j = 0; j < nj; ++j) ell += exp(P[j] - m);
    const double lse = m + log(ell);
    for (int64_t j = 0; j < nj; ++j) P[j] = exp(P[j] - lse);
    return lse;
}

/*
 * Forward of Eq. 2 for one segment.
 *   q_seg [B, l_s, H, d], k, v [B, l_x, H, d]  ->  out [B, l_s, H, d], lse [B, H, l_s]
 * returns 0, or -1 on a bad shape.
 */
int lss_oracle_segment_fwd(const double *q_seg, const double *k, const double *v,
                           int64_t s0, int64_t l_s, int64_t l_x, int64_t B, int64_t H,
                           int64_t d, int causal, double *out, double *lse)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || d < 1) return -1;
    const int64_t rows = B * H * l_s;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)l_x);
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < rows; ++t) {
            const int64_t r = t % l_s, h = (t / l_s) % H, b = t / (l_s * H);
            const int64_t nj = visible(s0, r, l_x, causal);
            const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
            lse[(b * H + h) * l_s + r] = row_softmax(q_row, k, b, h, l_x, H, d, nj, P);
            double *o_row = out + IDX4(b, r, h, 0, l_s, H, d);
            for (int64_t c = 0; c < d; ++c) o_row[c] = 0.0;
            for (int64_t j = 0; j < nj; ++j) {
                const double *v_row = v + IDX4(b, j, h, 0, l_x, H, d);
                for (int64_t c = 0; c < d; ++c) o_row[c] += P[j] * v_row[c];
            }
        }
        free(P);
    }
    return 0;
}

/*
 * Backward of Eq. 2 for one segment, given dO = d(loss)/d(out).
 *   -> dq [B, l_s, H, d]; dk_part, dv_part [B, l_x, H, d] (all l_x rows
 *      written; rows no query of this segment sees are 0).
 * With P the softmax row and dP[j] = dO[r].v[j]:
 *   D = sum_j P[j] dP[j];  dS[j] = P[j] (dP[j] - D);
 *   dq[r] = sum_j dS[j] k[j] / sqrt(d);
 *   dk_part[j] = sum_r dS[r][j] q[r] / sqrt(d);  dv_part[j] = sum_r P[r][j] dO[r].
 * Like the paper's own implementation (Section 2.2) the l_s x l_x weight
 * matrix of one head is materialised: first all rows (P, dS, dq), then all
 * key columns (dk_part, dv_part), each sum taken in increasing index order.
 */
int lss_oracle_segment_bwd(const double *q_seg, const double *k, const double *v,
                           int64_t s0, int64_t l_s, int64_t l_x, int64_t B, int64_t H,
                           int64_t d, int causal, const double *dO,
                           double *dq, double *dk_part, double *dv_part)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || d < 1) return -1;
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const size_t w_elems = (size_t)(l_s > 0 ? l_s : 1) * (size_t)l_x;
    double *Pm = (double *)malloc(sizeof(double) * w_elems);
    double *dSm = (double *)malloc(sizeof(double) * w_elems);
    if (!Pm || !dSm) { free(Pm); free(dSm); return -2; }
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
#pragma omp parallel for schedule(dynamic, 4)
            for (int64_t r = 0; r < l_s; ++r) {
                const int64_t nj = visible(s0, r, l_x, causal);
                double *P = Pm + r * l_x, *dS = dSm + r * l_x;
                const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
                const double *do_row = dO + IDX4(b, r, h, 0, l_s, H, d);
                row_softmax(q_row, k, b, h, l_x, H, d, nj, P);
                double D = 0.0;
                for (int64_t j = 0; j < nj; ++j) {
                    const double *v_row = v + IDX4(b, j, h, 0, l_x, H, d);
                    double dp = 0.0;
                    for (int64_t c = 0; c < d; ++c) dp += do_row[c] * v_row[c];
                    dS[j] = dp;
                    D += P[j] * dp;
                }
                for (int64_t j = 0; j < nj; ++j) dS[j] = P[j] * (dS[j] - D);
                for (int64_t j = nj; j < l_x; ++j) { P[j] = 0.0; dS[j] = 0.0; }
                double *dq_row = dq + IDX4(b, r, h, 0, l_s, H, d);
                for (int64_t c = 0; c < d; ++c) dq_row[c] = 0.0;
                for (int64_t j = 0; j < nj; ++j) {
                    const double *k_row = k + IDX4(b, j, h, 0, l_x, H, d);
                    for (int64_t c = 0; c < d; ++c) dq_row[c] += dS[j] * k_row[c];
                }
                for (int64_t c = 0; c < d; ++c) dq_row[c] *= inv_sqrt_d;
            }
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < l_x; ++j) {
                double *dk_row = dk_part + IDX4(b, j, h, 0, l_x, H, d);
                double *dv_row = dv_part + IDX4(b, j, h, 0, l_x, H, d);
                for (int64_t c = 0; c < d; ++c) { dk_row[c] = 0.0; dv_row[c] = 0.0; }
                for (int64_t r = 0; r < l_s; ++r) {
                    const double ds = dSm[r * l_x + j], p = Pm[r * l_x + j];
                    if (ds == 0.0 && p == 0.0) continue; /* masked pair */
                    const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
                    const double *do_row = dO + IDX4(b, r, h, 0, l_s, H, d);
                    for (int64_t c = 0; c < d; ++c) {
                        dk_row[c] += ds * q_row[c];
                        dv_row[c] += p * do_row[c];
                    }
                }
                for (int64_t c = 0; c < d; ++c) dk_row[c] *= inv_sqrt_d;
            }
        }
    free(Pm);
    free(dSm);
    return 0;
}

/*
 * Softmax rows themselves (the partial score matrix A_w of Section 2.2 for one
 * segment), for tests that look at the weights: P [B, H, l_s, l_x], masked
 * entries 0.
 */
int lss_oracle_segment_weights(const double *q_seg, const double *k, int64_t s0, int64_t l_s,
                               int64_t l_x, int64_t B, int64_t H, int64_t d, int causal, double *P)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || d < 1) return -1;
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h)
            for (int64_t r = 0; r < l_s; ++r) {
                const int64_t nj = visible(s0, r, l_x, causal);
                double *row = P + ((b * H + h) * l_s + r) * l_x;
                for (int64_t j = 0; j < l_x; ++j) row[j] = 0.0;
                row_softmax(q_seg + IDX4(b, r, h, 0, l_s, H, d), k, b, h, l_x, H, d, nj, row);
            }
    return 0;
}

/*
 * Segment sum (the arithmetic of the reduce-scatter of Fig. 2(v)):
 * out = parts[0] + parts[1] + ... in that order, elementwise, n_elems each.
 */
int lss_oracle_reduce_partials(const double *const *parts, int n, int64_t n_elems, double *out)
{
    if (n < 0 || n_elems < 0) return -1;
    for (int64_t e = 0; e < n_elems; ++e) {
        double s = 0.0;
        for (int i = 0; i < n; ++i) s += parts[i][e];
        out[e] = s;
    }
    return 0;
}

/* ------------------------------------------------------------------------
 * Dropout on the attention weights.  Section 2.2 names a dropout next to
 * the softmax in the normalisation of the scores; the reading taken here is
 * the usual one of the framework the paper was written in: the softmax row
 * A_w is computed first, then each weight is kept with probability 1 - p and
 * the kept ones are divided by 1 - p, and E = dropout(A_w) V.  lse stays the
 * logsumexp of the scores.
 *
 * The keep decision of a weight is a function of (seed, b*H + h, GLOBAL query
 * position, key position) alone, so that a segment drops exactly what the
 * sequential computation would drop at those positions and the segments'
 * outputs still concatenate to the full-sequence result (Section 3,
 * Principle 3).  The paper does not say how the random numbers are drawn.
 * DEFINITION used here: a counter-based generator, not a stream (nothing
 * depends on the order of evaluation), built from a published 32-bit integer
 * mixing function mix32 (two multiply-xorshift rounds):
 *     row_key(seed, bh, row) = mix32(mix32(lo32(seed) + 0x9e3779b9 (bh + 1)) ^ row)
 *     col_key(seed, col)     = mix32(mix32(hi32(seed) + 0x85ebca6b) ^ col)
 *     u(seed, bh, row, col)  = mix32(row_key + col_key)            (mod 2^32)
 *     keep                   = u >= round(p 2^32)
 * The argument of the last mix is a sum of a row term and a column term; the
 * pins check that the mix removes that structure (the parity of the keep bits
 * at the four corners of any rectangle of rows and columns behaves like that
 * of four independent coin flips).
 * ------------------------------------------------------------------------ */
static uint32_t mix32(uint32_t x)
{
    x ^= x >> 16; x *= 0x7feb352dU;
    x ^= x >> 15; x *= 0x846ca68bU;
    x ^= x >> 16;
    return x;
}
static uint32_t row_key(uint64_t seed, uint32_t bh, uint32_t row)
{
    return mix32(mix32((uint32_t)seed + 0x9e3779b9U * (bh + 1U)) ^ row);
}
static uint32_t col_key(uint64_t seed, uint32_t col)
{
    return mix32(mix32((uint32_t)(seed >> 32) + 0x85ebca6bU) ^ col);
}
static uint32_t drop_threshold(double p)
{
    const double t = floor(p * 4294967296.0 + 0.5);
    return t >= 4294967295.0 ? 4294967295U : (t <= 0.0 ? 0U : (uint32_t)t);
}
/* 1 if the weight of (row key rk, key position col) is kept */
static int keep(uint32_t rk, uint64_t seed, uint32_t col, uint32_t thr)
{
    return mix32(rk + col_key(seed, col)) >= thr;
}

/* keep mask of one segment: mask [B, H, l_s, l_x] bytes (1 = kept), all key positions */
int lss_oracle_dropout_mask(double p, uint64_t seed, int64_t s0, int64_t l_s, int64_t l_x, int64_t B,
                            int64_t H, unsigned char *mask)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || !(p >= 0.0 && p < 1.0)) return -1;
    const uint32_t thr = drop_threshold(p);
    for (int64_t bh = 0; bh < B * H; ++bh)
        for (int64_t r = 0; r < l_s; ++r) {
            const uint32_t rk = row_key(seed, (uint32_t)bh, (uint32_t)(s0 + r));
            for (int64_t j = 0; j < l_x; ++j) mask[(bh * l_s + r) * l_x + j] = (unsigned char)keep(rk, seed, (uint32_t)j, thr);
        }
    return 0;
}

/* keep mask for dropout on a segment's activations [B, l_s, E] (the residual branches of a layer):
 * element (b, r, c) is decided as the weight of (batch*head b, global row s0 + r, key c) would be */
int lss_oracle_activation_keep(double p, uint64_t seed, int64_t s0, int64_t l_s, int64_t E, int64_t B,
                               unsigned char *mask)
{
    if (l_s < 0 || E < 1 || s0 < 0 || B < 0 || !(p >= 0.0 && p < 1.0)) return -1;
    const uint32_t thr = drop_threshold(p);
    for (int64_t b = 0; b < B; ++b)
        for (int64_t r = 0; r < l_s; ++r) {
            const uint32_t rk = row_key(seed, (uint32_t)b, (uint32_t)(s0 + r));
            for (int64_t c = 0; c < E; ++c) mask[(b * l_s + r) * E + c] = (unsigned char)keep(rk, seed, (uint32_t)c, thr);
        }
    return 0;
}

/* Forward with dropout: as lss_oracle_segment_fwd, with out = sum_j keep_j P[j] / (1 - p) v[j]. */
int lss_oracle_segment_fwd_dropout(const double *q_seg, const double *k, const double *v,
                                   int64_t s0, int64_t l_s, int64_t l_x, int64_t B, int64_t H,
                                   int64_t d, int causal, double p, uint64_t seed, double *out, double *lse)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || d < 1 || !(p >= 0.0 && p < 1.0)) return -1;
    const uint32_t thr = drop_threshold(p);
    const double inv_keep = 1.0 / (1.0 - p);
    const int64_t rows = B * H * l_s;
#pragma omp parallel
    {
        double *P = (double *)malloc(sizeof(double) * (size_t)l_x);
#pragma omp for schedule(dynamic, 4)
        for (int64_t t = 0; t < rows; ++t) {
            const int64_t r = t % l_s, h = (t / l_s) % H, b = t / (l_s * H);
            const int64_t nj = visible(s0, r, l_x, causal);
            const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
            lse[(b * H + h) * l_s + r] = row_softmax(q_row, k, b, h, l_x, H, d, nj, P);
            const uint32_t rk = row_key(seed, (uint32_t)(b * H + h), (uint32_t)(s0 + r));
            double *o_row = out + IDX4(b, r, h, 0, l_s, H, d);
            for (int64_t c = 0; c < d; ++c) o_row[c] = 0.0;
            for (int64_t j = 0; j < nj; ++j) {
                if (!keep(rk, seed, (uint32_t)j, thr)) continue;
                const double w = P[j] * inv_keep;
                const double *v_row = v + IDX4(b, j, h, 0, l_x, H, d);
                for (int64_t c = 0; c < d; ++c) o_row[c] += w * v_row[c];
            }
        }
        free(P);
    }
    return 0;
}

/*
 * Backward with dropout.  With A = softmax row, M_j = keep_j / (1 - p), out = sum_j A_j M_j v_j:
 *   dA[j] = M_j (dO[r].v[j]);  D = sum_j A[j] dA[j];  dS[j] = A[j] (dA[j] - D);
 *   dq[r] = sum_j dS[j] k[j] / sqrt(d);
 *   dk_part[j] = sum_r dS[r][j] q[r] / sqrt(d);  dv_part[j] = sum_r A[r][j] M[r][j] dO[r].
 */
int lss_oracle_segment_bwd_dropout(const double *q_seg, const double *k, const double *v,
                                   int64_t s0, int64_t l_s, int64_t l_x, int64_t B, int64_t H,
                                   int64_t d, int causal, double p, uint64_t seed, const double *dO,
                                   double *dq, double *dk_part, double *dv_part)
{
    if (l_s < 0 || l_x < 1 || s0 < 0 || s0 + l_s > l_x || B < 0 || H < 1 || d < 1 || !(p >= 0.0 && p < 1.0)) return -1;
    const uint32_t thr = drop_threshold(p);
    const double inv_keep = 1.0 / (1.0 - p);
    const double inv_sqrt_d = 1.0 / sqrt((double)d);
    const size_t w_elems = (size_t)(l_s > 0 ? l_s : 1) * (size_t)l_x;
    double *AMm = (double *)malloc(sizeof(double) * w_elems);   /* A_j M_j */
    double *dSm = (double *)malloc(sizeof(double) * w_elems);
    if (!AMm || !dSm) { free(AMm); free(dSm); return -2; }
    for (int64_t b = 0; b < B; ++b)
        for (int64_t h = 0; h < H; ++h) {
#pragma omp parallel for schedule(dynamic, 4)
            for (int64_t r = 0; r < l_s; ++r) {
                const int64_t nj = visible(s0, r, l_x, causal);
                double *AM = AMm + r * l_x, *dS = dSm + r * l_x;
                const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
                const double *do_row = dO + IDX4(b, r, h, 0, l_s, H, d);
                row_softmax(q_row, k, b, h, l_x, H, d, nj, AM);     /* AM holds A for now */
                const uint32_t rk = row_key(seed, (uint32_t)(b * H + h), (uint32_t)(s0 + r));
                double D = 0.0;
                for (int64_t j = 0; j < nj; ++j) {
                    const double *v_row = v + IDX4(b, j, h, 0, l_x, H, d);
                    double dp = 0.0;
                    for (int64_t c = 0; c < d; ++c) dp += do_row[c] * v_row[c];
                    const double mj = keep(rk, seed, (uint32_t)j, thr) ? inv_keep : 0.0;
                    dS[j] = mj * dp;                                 /* dA[j] */
                    D += AM[j] * dS[j];
                }
                for (int64_t j = 0; j < nj; ++j) {
                    const double a = AM[j];
                    dS[j] = a * (dS[j] - D);
                    AM[j] = keep(rk, seed, (uint32_t)j, thr) ? a * inv_keep : 0.0;
                }
                for (int64_t j = nj; j < l_x; ++j) { AM[j] = 0.0; dS[j] = 0.0; }
                double *dq_row = dq + IDX4(b, r, h, 0, l_s, H, d);
                for (int64_t c = 0; c < d; ++c) dq_row[c] = 0.0;
                for (int64_t j = 0; j < nj; ++j) {
                    const double *k_row = k + IDX4(b, j, h, 0, l_x, H, d);
                    for (int64_t c = 0; c < d; ++c) dq_row[c] += dS[j] * k_row[c];
                }
                for (int64_t c = 0; c < d; ++c) dq_row[c] *= inv_sqrt_d;
            }
#pragma omp parallel for schedule(static)
            for (int64_t j = 0; j < l_x; ++j) {
                double *dk_row = dk_part + IDX4(b, j, h, 0, l_x, H, d);
                double *dv_row = dv_part + IDX4(b, j, h, 0, l_x, H, d);
                for (int64_t c = 0; c < d; ++c) { dk_row[c] = 0.0; dv_row[c] = 0.0; }
                for (int64_t r = 0; r < l_s; ++r) {
                    const double ds = dSm[r * l_x + j], am = AMm[r * l_x + j];
                    if (ds == 0.0 && am == 0.0) continue;
                    const double *q_row = q_seg + IDX4(b, r, h, 0, l_s, H, d);
                    const double *do_row = dO + IDX4(b, r, h, 0, l_s, H, d);
                    for (int64_t c = 0; c < d; ++c) {
                        dk_row[c] += ds * q_row[c];
                        dv_row[c] += am * do_row[c];
                    }
                }
                for (int64_t c = 0; c < d; ++c) dk_row[c] *= inv_sqrt_d;
            }
        }
    free(AMm);
    free(dSm);
    return 0;
}
