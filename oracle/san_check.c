/*
 * Memory- and undefined-behaviour check of the fp64 oracle (test infrastructure, like the oracle itself).
 *
 * Built together with lss_oracle.c under -fsanitize=address,undefined (oracle.build_sanitized()) into a
 * stand-alone program: it calls every exported function of the oracle on small seeded inputs with tight
 * heap buffers -- ragged segments, a single row, l_s = 0, causal and not, dropout -- so that an
 * out-of-bounds index, a misused buffer or an overflowing shift in the oracle aborts the run, and checks
 * on the way a few relations the mathematics fixes (softmax rows sum to 1, the first causal row returns
 * v_0, partials add up to the full-sequence gradient, p = 0 is the plain call).  Exit status 0 = clean.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int lss_oracle_threads(void);
int lss_oracle_segment_fwd(const double *, const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                           int64_t, int, double *, double *);
int lss_oracle_segment_bwd(const double *, const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t,
                           int64_t, int, const double *, double *, double *, double *);
int lss_oracle_segment_weights(const double *, const double *, int64_t, int64_t, int64_t, int64_t, int64_t, int64_t, int,
                               double *);
int lss_oracle_reduce_partials(const double *const *, int, int64_t, double *);
int lss_oracle_dropout_mask(double, uint64_t, int64_t, int64_t, int64_t, int64_t, int64_t, unsigned char *);
int lss_oracle_activation_keep(double, uint64_t, int64_t, int64_t, int64_t, int64_t, unsigned char *);
int lss_oracle_segment_fwd_dropout(const double *, const double *, const double *, int64_t, int64_t, int64_t, int64_t,
                                   int64_t, int64_t, int, double, uint64_t, double *, double *);
int lss_oracle_segment_bwd_dropout(const double *, const double *, const double *, int64_t, int64_t, int64_t, int64_t,
                                   int64_t, int64_t, int, double, uint64_t, const double *, double *, double *, double *);

static uint64_t g_state = 0x1234567ULL;
static double rnd(void)     /* a small linear congruential generator: uniform in [-1, 1) */
{
    g_state = g_state * 6364136223846793005ULL + 1442695040888963407ULL;
    return (double)(int64_t)(g_state >> 11) / 4503599627370496.0 - 1.0;
}
static double *fresh(int64_t n, int random)
{
    double *p = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
    if (!p) exit(3);
    for (int64_t i = 0; i < n; ++i) p[i] = random ? rnd() : NAN;   /* outputs start as NaN: unwritten entries show */
    return p;
}
static int g_fail = 0;
static void expect(int ok, const char *what, int line)
{
    if (!ok) { fprintf(stderr, "san_check: line %d: %s\n", line, what); g_fail = 1; }
}
#define EXPECT(c) expect((c), #c, __LINE__)
static double maxdiff(const double *a, const double *b, int64_t n)
{
    double m = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        const double e = fabs(a[i] - b[i]);
        if (!(e <= m)) m = e;      /* NaN propagates */
    }
    return m;
}

/* one sequence split into the given segments: forward and backward per segment against the unsegmented call */
static void run_case(int64_t B, int64_t l_x, int64_t H, int64_t d, int causal, const int64_t *cuts, int n_seg, double p,
                     uint64_t seed)
{
    const int64_t nkv = B * l_x * H * d;
    double *q = fresh(nkv, 1), *k = fresh(nkv, 1), *v = fresh(nkv, 1), *g = fresh(nkv, 1);
    double *fo = fresh(nkv, 0), *fl = fresh(B * H * l_x, 0), *fdq = fresh(nkv, 0), *fdk = fresh(nkv, 0), *fdv = fresh(nkv, 0);
    if (p > 0.0) {
        EXPECT(lss_oracle_segment_fwd_dropout(q, k, v, 0, l_x, l_x, B, H, d, causal, p, seed, fo, fl) == 0);
        EXPECT(lss_oracle_segment_bwd_dropout(q, k, v, 0, l_x, l_x, B, H, d, causal, p, seed, g, fdq, fdk, fdv) == 0);
    } else {
        EXPECT(lss_oracle_segment_fwd(q, k, v, 0, l_x, l_x, B, H, d, causal, fo, fl) == 0);
        EXPECT(lss_oracle_segment_bwd(q, k, v, 0, l_x, l_x, B, H, d, causal, g, fdq, fdk, fdv) == 0);
    }
    double **pk = (double **)malloc(sizeof(double *) * (size_t)n_seg), **pv = (double **)malloc(sizeof(double *) * (size_t)n_seg);
    for (int i = 0; i < n_seg; ++i) {
        const int64_t s0 = cuts[i], l_s = cuts[i + 1] - cuts[i], nq = B * l_s * H * d;
        /* the segment's rows of q and dO as tensors of their own ([B, l_s, H, d]) */
        double *qs = fresh(nq, 0), *gs = fresh(nq, 0), *o = fresh(nq, 0), *l = fresh(B * H * l_s, 0), *dq = fresh(nq, 0);
        for (int64_t b = 0; b < B; ++b)
            for (int64_t r = 0; r < l_s; ++r) {
                memcpy(qs + (b * l_s + r) * H * d, q + (b * l_x + s0 + r) * H * d, sizeof(double) * (size_t)(H * d));
                memcpy(gs + (b * l_s + r) * H * d, g + (b * l_x + s0 + r) * H * d, sizeof(double) * (size_t)(H * d));
            }
        pk[i] = fresh(nkv, 0);
        pv[i] = fresh(nkv, 0);
        if (p > 0.0) {
            EXPECT(lss_oracle_segment_fwd_dropout(qs, k, v, s0, l_s, l_x, B, H, d, causal, p, seed, o, l) == 0);
            EXPECT(lss_oracle_segment_bwd_dropout(qs, k, v, s0, l_s, l_x, B, H, d, causal, p, seed, gs, dq, pk[i], pv[i]) == 0);
        } else {
            EXPECT(lss_oracle_segment_fwd(qs, k, v, s0, l_s, l_x, B, H, d, causal, o, l) == 0);
            EXPECT(lss_oracle_segment_bwd(qs, k, v, s0, l_s, l_x, B, H, d, causal, gs, dq, pk[i], pv[i]) == 0);
            /* the weights of every row sum to 1 */
            double *w = fresh(B * H * l_s * l_x, 0);
            EXPECT(lss_oracle_segment_weights(qs, k, s0, l_s, l_x, B, H, d, causal, w) == 0);
            for (int64_t t = 0; t < B * H * l_s; ++t) {
                double sum = 0.0;
                for (int64_t j = 0; j < l_x; ++j) sum += w[t * l_x + j];
                EXPECT(fabs(sum - 1.0) < 1e-12);
            }
            free(w);
        }
        /* segment rows equal the unsegmented result's rows (Section 3, Principle 3) */
        for (int64_t b = 0; b < B; ++b)
            for (int64_t r = 0; r < l_s; ++r) {
                EXPECT(maxdiff(o + (b * l_s + r) * H * d, fo + (b * l_x + s0 + r) * H * d, H * d) < 1e-12);
                EXPECT(maxdiff(dq + (b * l_s + r) * H * d, fdq + (b * l_x + s0 + r) * H * d, H * d) < 1e-11);
                for (int64_t h = 0; h < H; ++h)
                    EXPECT(fabs(l[(b * H + h) * l_s + r] - fl[(b * H + h) * l_x + s0 + r]) < 1e-12);
            }
        if (causal && p == 0.0 && s0 == 0 && l_s > 0)       /* the first causal row sees key 0 only */
            EXPECT(maxdiff(o, v, d) < 1e-15);
        free(qs); free(gs); free(o); free(l); free(dq);
    }
    /* the partials add up to the gradient of the unsegmented call (Principle 4, Fig. 2(v)) */
    double *sk = fresh(nkv, 0), *sv = fresh(nkv, 0);
    EXPECT(lss_oracle_reduce_partials((const double *const *)pk, n_seg, nkv, sk) == 0);
    EXPECT(lss_oracle_reduce_partials((const double *const *)pv, n_seg, nkv, sv) == 0);
    EXPECT(maxdiff(sk, fdk, nkv) < 1e-11);
    EXPECT(maxdiff(sv, fdv, nkv) < 1e-11);
    for (int i = 0; i < n_seg; ++i) { free(pk[i]); free(pv[i]); }
    free(pk); free(pv); free(sk); free(sv);
    free(q); free(k); free(v); free(g); free(fo); free(fl); free(fdq); free(fdk); free(fdv);
}

int main(void)
{
    EXPECT(lss_oracle_threads() >= 1);
    const int64_t even[] = {0, 4, 8, 12, 16}, ragged[] = {0, 1, 1, 7, 19, 23}, one[] = {0, 5};
    run_case(1, 16, 2, 4, 1, even, 4, 0.0, 0);
    run_case(2, 23, 3, 5, 1, ragged, 5, 0.0, 0);        /* a single-row and an empty segment, odd head width */
    run_case(2, 23, 1, 8, 0, ragged, 5, 0.0, 0);
    run_case(1, 5, 1, 1, 1, one, 1, 0.0, 0);
    run_case(2, 23, 2, 4, 1, ragged, 5, 0.3, 0xfedcba9876543210ULL);
    run_case(1, 16, 2, 4, 0, even, 4, 0.9, 7);

    /* dropout masks: p = 0 keeps everything; the forward with p = 0 is the plain forward; positions beyond 2^31 */
    {
        unsigned char *m = (unsigned char *)malloc(2 * 3 * 7 * 11);
        EXPECT(lss_oracle_dropout_mask(0.0, 99, 2, 7, 11, 2, 3, m) == 0);
        for (int i = 0; i < 2 * 3 * 7 * 11; ++i) EXPECT(m[i] == 1);
        EXPECT(lss_oracle_dropout_mask(0.5, ~0ULL, 4, 7, 11, 2, 3, m) == 0);
        EXPECT(lss_oracle_dropout_mask(1.0, 1, 0, 7, 11, 2, 3, m) == -1);
        EXPECT(lss_oracle_dropout_mask(0.5, 1, 5, 7, 11, 2, 3, m) == -1);      /* 5 + 7 > 11 */
        free(m);
        unsigned char *a = (unsigned char *)malloc(2 * 3 * 13);
        EXPECT(lss_oracle_activation_keep(0.25, 0x8000000080000000ULL, 4000000000LL, 3, 13, 2, a) == 0);
        EXPECT(lss_oracle_activation_keep(0.25, 1, -1, 3, 13, 2, a) == -1);
        free(a);
    }
    /* bad shapes are refused before anything is touched */
    EXPECT(lss_oracle_segment_fwd(NULL, NULL, NULL, 3, 4, 6, 1, 1, 4, 1, NULL, NULL) == -1);
    EXPECT(lss_oracle_segment_bwd(NULL, NULL, NULL, 0, 4, 0, 1, 1, 4, 1, NULL, NULL, NULL, NULL) == -1);
    EXPECT(lss_oracle_reduce_partials(NULL, -1, 4, NULL) == -1);
    if (g_fail) return 1;
    puts("san_check: clean");
    return 0;
}
