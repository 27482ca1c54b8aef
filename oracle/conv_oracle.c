/*
 * CPU oracle for direct 2-D convolution, the three training passes.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path (the HIP library or
 * its Python binding) may include, link or call this file; it shares no code,
 * header, table or helper with the GPU kernels.  It exists so that the GPU
 * results can be compared against the plain definition.
 *
 * Every function is one of the paper's naive seven-loop nests written out:
 *   forward          -- Algorithm 1 (Section II-A)
 *   backward by data -- Algorithm 6 (Section II-I)
 *   weight update    -- Algorithm 8 (Section II-J)
 * over the logical tensors of Section II: I[N][C][H][W], W[K][C][R][S],
 * O[N][K][P][Q] (row-major, last index fastest), in fp64 throughout.
 *
 * Readings where the paper is silent (all three are the usual conventions):
 *   - zero padding, symmetric on each axis (one value per axis, so that the
 *     1xS and Rx1 filters of Inception-style layers can pad along their long
 *     side only): the input position touched by output (oj,oi) and tap (r,s) is
 *         ij = stride*oj - pad_h + r ,  ii = stride*oi - pad_w + s ,
 *     and a term whose (ij,ii) falls outside [0,H)x[0,W) is skipped.  The
 *     printed loops are the pad = 0 case.
 *   - P = floor((H + 2 pad_h - R)/stride) + 1, Q = floor((W + 2 pad_w - S)/stride) + 1.
 *   - the "+=" targets start from zero: outputs are overwritten.
 *
 * No blocking, no reordering, no vectorisation tricks: loop order is the
 * paper's (n,k,c,oj,oi,r,s).  OpenMP splits only the outermost loop whose
 * iterations write disjoint outputs (n for forward/backward, k for update),
 * so the summation order of every output element is independent of the
 * number of threads.
 *
 * Parity pins (see tests/test_oracle_*.py): brute-force gather evaluator on
 * tiny shapes, 1x1 == GEMM, delta-filter shifts, adjoint identities, the
 * paper's two duality statements, all-ones closed forms, N-additivity,
 * separable closed forms against scipy's correlate2d, torch's fp64 conv2d and
 * its autograd gradients.
 */
#include <stddef.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int N, C, K, H, W, R, S, stride, pad_h, pad_w;
} oracle_shape_t;

static int out_extent(int in, int pad, int filt, int stride)
{
    int span = in + 2 * pad - filt;
    if (span < 0) return 0;
    return span / stride + 1;
}

int oracle_out_h(const oracle_shape_t *g) { return out_extent(g->H, g->pad_h, g->R, g->stride); }
int oracle_out_w(const oracle_shape_t *g) { return out_extent(g->W, g->pad_w, g->S, g->stride); }

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Algorithm 1: O[n][k][oj][oi] += I[n][c][ij+r][ii+s] * W[k][c][r][s]. */
void oracle_conv_fwd(const oracle_shape_t *g, const double *I, const double *Wt, double *O)
{
    const int N = g->N, C = g->C, K = g->K, H = g->H, W = g->W, R = g->R, S = g->S;
    const int stride = g->stride, pad_h = g->pad_h, pad_w = g->pad_w;
    const int P = oracle_out_h(g), Q = oracle_out_w(g);
    memset(O, 0, sizeof(double) * (size_t)N * K * P * Q);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < C; ++c)
                for (int oj = 0; oj < P; ++oj)
                    for (int oi = 0; oi < Q; ++oi) {
                        const int ij = stride * oj - pad_h;
                        const int ii = stride * oi - pad_w;
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                if (ij + r < 0 || ij + r >= H) continue;
                                if (ii + s < 0 || ii + s >= W) continue;
                                O[(((size_t)n * K + k) * P + oj) * Q + oi] +=
                                    I[(((size_t)n * C + c) * H + (ij + r)) * W + (ii + s)] *
                                    Wt[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    }
}

/* Algorithm 6: dI[n][c][ij+r][ii+s] += dO[n][k][oj][oi] * W[k][c][r][s]. */
void oracle_conv_bwd_data(const oracle_shape_t *g, const double *dO, const double *Wt, double *dI)
{
    const int N = g->N, C = g->C, K = g->K, H = g->H, W = g->W, R = g->R, S = g->S;
    const int stride = g->stride, pad_h = g->pad_h, pad_w = g->pad_w;
    const int P = oracle_out_h(g), Q = oracle_out_w(g);
    memset(dI, 0, sizeof(double) * (size_t)N * C * H * W);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int k = 0; k < K; ++k)
            for (int c = 0; c < C; ++c)
                for (int oj = 0; oj < P; ++oj)
                    for (int oi = 0; oi < Q; ++oi) {
                        const int ij = stride * oj - pad_h;
                        const int ii = stride * oi - pad_w;
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                if (ij + r < 0 || ij + r >= H) continue;
                                if (ii + s < 0 || ii + s >= W) continue;
                                dI[(((size_t)n * C + c) * H + (ij + r)) * W + (ii + s)] +=
                                    dO[(((size_t)n * K + k) * P + oj) * Q + oi] *
                                    Wt[(((size_t)k * C + c) * R + r) * S + s];
                            }
                    }
}

/* Algorithm 8: dW[k][c][r][s] += I[n][c][ij+r][ii+s] * dO[n][k][oj][oi].
 * The printed loop order has n outermost; every dW element is written by all
 * n, so threads split k (the outermost loop with disjoint outputs) and each
 * thread runs the remaining loops in the printed order. */
void oracle_conv_upd(const oracle_shape_t *g, const double *I, const double *dO, double *dW)
{
    const int N = g->N, C = g->C, K = g->K, H = g->H, W = g->W, R = g->R, S = g->S;
    const int stride = g->stride, pad_h = g->pad_h, pad_w = g->pad_w;
    const int P = oracle_out_h(g), Q = oracle_out_w(g);
    memset(dW, 0, sizeof(double) * (size_t)K * C * R * S);
#pragma omp parallel for schedule(static)
    for (int k = 0; k < K; ++k)
        for (int n = 0; n < N; ++n)
            for (int c = 0; c < C; ++c)
                for (int oj = 0; oj < P; ++oj)
                    for (int oi = 0; oi < Q; ++oi) {
                        const int ij = stride * oj - pad_h;
                        const int ii = stride * oi - pad_w;
                        for (int r = 0; r < R; ++r)
                            for (int s = 0; s < S; ++s) {
                                if (ij + r < 0 || ij + r >= H) continue;
                                if (ii + s < 0 || ii + s >= W) continue;
                                dW[(((size_t)k * C + c) * R + r) * S + s] +=
                                    I[(((size_t)n * C + c) * H + (ij + r)) * W + (ii + s)] *
                                    dO[(((size_t)n * K + k) * P + oj) * Q + oi];
                            }
                    }
}

/* Algorithm 8 restricted to a list of dW entries: entry e is
 * (k,c,r,s) = idx[4e..4e+3]; out[e] is that element of the full result.
 * Used when the full tensor at minibatch 256 is too slow to evaluate. */
void oracle_conv_upd_entries(const oracle_shape_t *g, const double *I, const double *dO,
                             int n_entries, const int *idx, double *out)
{
    const int N = g->N, C = g->C, K = g->K, H = g->H, W = g->W;
    const int stride = g->stride, pad_h = g->pad_h, pad_w = g->pad_w;
    const int P = oracle_out_h(g), Q = oracle_out_w(g);
#pragma omp parallel for schedule(dynamic, 8)
    for (int e = 0; e < n_entries; ++e) {
        const int k = idx[4 * e + 0], c = idx[4 * e + 1], r = idx[4 * e + 2], s = idx[4 * e + 3];
        double acc = 0.0;
        for (int n = 0; n < N; ++n)
            for (int oj = 0; oj < P; ++oj)
                for (int oi = 0; oi < Q; ++oi) {
                    const int ij = stride * oj - pad_h;
                    const int ii = stride * oi - pad_w;
                    if (ij + r < 0 || ij + r >= H) continue;
                    if (ii + s < 0 || ii + s >= W) continue;
                    acc += I[(((size_t)n * C + c) * H + (ij + r)) * W + (ii + s)] *
                           dO[(((size_t)n * K + k) * P + oj) * Q + oi];
                }
        out[e] = acc;
    }
}
