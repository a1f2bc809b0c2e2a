/*
 * CPU oracle for the GNN aggregation / combination hot path.  TEST INFRASTRUCTURE ONLY:
 * it is called by the tests, by the smoke check and by the benchmark's CPU-baseline leg, never
 * by the product library, and it shares no code with the GPU kernels.
 *
 * Everything here is the plain definition, written as slow per-destination loops with fp64
 * accumulation:
 *   - aggregation f(h(X)) over an in-edge CSR (pointer array indexed by destination, vertex
 *     array of sources; paper, Preliminaries "Data representation" and "Algorithm model"),
 *   - its derivative, an aggregation whose outputs live on the source vertices (paper,
 *     "Training for GNNs"), done here by scattering so it needs no transposed structure,
 *   - the transposed structure (CSC) itself, as a stable counting sort,
 *   - the combination (MLP: linear transform, bias, non-linearity; paper "Algorithm model"
 *     and the GNN Kernel Orchestrator section's sigma(W f(h(X)) + b)).
 *
 * Readings the paper leaves open:
 *   mean divides by the number of in-edges of the row (empty row -> 0); the symmetric
 *   normalisation uses 1/sqrt(d(u) d(v)) with d = in-degree taken from the given CSR for both
 *   ends (square graphs only); a per-edge scalar weight multiplies each term in every mode.
 *
 * OpenMP `parallel for` over independent outputs only (destinations, or feature columns for
 * the scatter); each output's sum is accumulated sequentially in edge order.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { GTO_SUM = 0, GTO_MEAN = 1, GTO_SYMNORM = 2 };

static inline double get(const void *p, int is_f32, size_t i) {
    return is_f32 ? (double)((const float *)p)[i] : ((const double *)p)[i];
}

/* in-degree of every destination, out-degree of every source */
void gto_degrees(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx,
                 int32_t *deg_in, int32_t *deg_out) {
    for (int64_t u = 0; u < n_src; ++u) deg_out[u] = 0;
    for (int64_t v = 0; v < n_dst; ++v) {
        deg_in[v] = rowptr[v + 1] - rowptr[v];
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) deg_out[colidx[e]] += 1;
    }
}

/* Transposed structure: row u lists the destinations of u's out-edges, ordered by the edge's
 * position e in the given CSR (stable); perm[k] is that position. */
void gto_transpose(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx,
                   int32_t *rowptr_t, int32_t *colidx_t, int32_t *perm) {
    int32_t *next = (int32_t *)calloc((size_t)n_src + 1, sizeof(int32_t));
    for (int64_t u = 0; u <= n_src; ++u) rowptr_t[u] = 0;
    for (int64_t v = 0; v < n_dst; ++v)
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) rowptr_t[colidx[e] + 1] += 1;
    for (int64_t u = 0; u < n_src; ++u) rowptr_t[u + 1] += rowptr_t[u];
    for (int64_t u = 0; u < n_src; ++u) next[u] = rowptr_t[u];
    for (int64_t v = 0; v < n_dst; ++v)
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int32_t k = next[colidx[e]]++;
            colidx_t[k] = (int32_t)v;
            perm[k] = e;
        }
    free(next);
}

static double dinv_of(const int32_t *rowptr, int64_t i) {
    int32_t d = rowptr[i + 1] - rowptr[i];
    return d > 0 ? 1.0 / sqrt((double)d) : 0.0;
}

/* Y[i,:] = aggregation of destination v = rows ? rows[i] : i, for i < n_rows.
 * Returns 0, or -1 for an unsupported request (symmetric norm on a non-square graph). */
int gto_aggregate_fwd(int64_t n_dst, int64_t n_src, const int32_t *rowptr,
                      const int32_t *colidx, const float *ew, int reduce, int64_t F,
                      const void *X, int x_is_f32, int64_t ldx, double *Y, int64_t ldy,
                      const int64_t *rows, int64_t n_rows) {
    if (reduce == GTO_SYMNORM && n_dst != n_src) return -1;
    if (!rows) n_rows = n_dst;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_rows; ++i) {
        int64_t v = rows ? rows[i] : i;
        int32_t deg = rowptr[v + 1] - rowptr[v];
        for (int64_t f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int64_t u = colidx[e];
                double term = get(X, x_is_f32, (size_t)u * ldx + f);
                if (ew) term *= (double)ew[e];
                if (reduce == GTO_SYMNORM) term *= dinv_of(rowptr, u);
                acc += term;
            }
            if (reduce == GTO_MEAN) acc = deg > 0 ? acc / (double)deg : 0.0;
            if (reduce == GTO_SYMNORM) acc *= dinv_of(rowptr, v);
            Y[(size_t)i * ldy + f] = acc;
        }
    }
    return 0;
}

/* dX[u,:] = sum over edges e = (u -> v) of c_e * dY[v,:], c_e the forward coefficient of e.
 * Loops over destination rows and scatters.  If src_rows is given only those source rows are
 * produced: dX[i,:] is the gradient of source src_rows[i]. */
int gto_aggregate_bwd(int64_t n_dst, int64_t n_src, const int32_t *rowptr,
                      const int32_t *colidx, const float *ew, int reduce, int64_t F,
                      const void *dY, int dy_is_f32, int64_t lddy, double *dX, int64_t lddx,
                      const int64_t *src_rows, int64_t n_src_rows) {
    if (reduce == GTO_SYMNORM && n_dst != n_src) return -1;
    int64_t *slot = NULL;
    int64_t n_out = n_src;
    if (src_rows) {
        slot = (int64_t *)malloc((size_t)n_src * sizeof(int64_t));
        for (int64_t u = 0; u < n_src; ++u) slot[u] = -1;
        for (int64_t i = 0; i < n_src_rows; ++i) slot[src_rows[i]] = i;
        n_out = n_src_rows;
    }
    for (int64_t i = 0; i < n_out; ++i)
        for (int64_t f = 0; f < F; ++f) dX[(size_t)i * lddx + f] = 0.0;
    const int64_t FB = 16; /* column block per thread: disjoint outputs, no races */
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t f0 = 0; f0 < F; f0 += FB) {
        int64_t f1 = f0 + FB < F ? f0 + FB : F;
        for (int64_t v = 0; v < n_dst; ++v) {
            int32_t deg = rowptr[v + 1] - rowptr[v];
            for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
                int64_t u = colidx[e];
                int64_t o = slot ? slot[u] : u;
                if (o < 0) continue;
                double c = ew ? (double)ew[e] : 1.0;
                if (reduce == GTO_MEAN) c = c / (double)deg;
                if (reduce == GTO_SYMNORM) c *= dinv_of(rowptr, u) * dinv_of(rowptr, v);
                for (int64_t f = f0; f < f1; ++f)
                    dX[(size_t)o * lddx + f] += c * get(dY, dy_is_f32, (size_t)v * lddy + f);
            }
        }
    }
    free(slot);
    return 0;
}

/* C[M,N] = op(A) op(B) (+ bias[N]) (then max(.,0) if relu); op(A) is M x K, op(B) is K x N.
 * transA: A is stored K x M (lda >= M); transB: B is stored N x K (ldb >= K). */
void gto_combine(int64_t M, int64_t N, int64_t K, const double *A, int64_t lda, int transA,
                 const double *B, int64_t ldb, int transB, const double *bias, int relu,
                 double *C, int64_t ldc) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        double *c = C + (size_t)i * ldc;
        if (!transB) {
            /* k outside j so the row of B is walked contiguously; every C[i,j] still sums its
             * K products in increasing k */
            for (int64_t j = 0; j < N; ++j) c[j] = 0.0;
            for (int64_t k = 0; k < K; ++k) {
                double a = transA ? A[(size_t)k * lda + i] : A[(size_t)i * lda + k];
                const double *b = B + (size_t)k * ldb;
                for (int64_t j = 0; j < N; ++j) c[j] += a * b[j];
            }
        } else {
            for (int64_t j = 0; j < N; ++j) {
                double acc = 0.0;
                for (int64_t k = 0; k < K; ++k) {
                    double a = transA ? A[(size_t)k * lda + i] : A[(size_t)i * lda + k];
                    acc += a * B[(size_t)j * ldb + k];
                }
                c[j] = acc;
            }
        }
        for (int64_t j = 0; j < N; ++j) {
            double z = c[j];
            if (bias) z += bias[j];
            if (relu && !(z > 0.0)) z = 0.0;
            c[j] = z;
        }
    }
}

/* ---------------------------------------------------------------------------------------------
 * Edge weighting (paper: Preliminaries, "edge weighting": a function g of the source and
 * destination embeddings per edge, and a function h that transforms the source embedding with
 * g's output before the aggregation f; Frontend section: NeighborApply computes g, Pull applies
 * h and f).  Edge e = (u -> v) is position e of the given CSR.
 *   g:  GTO_G_DOT  w_e    = sum_f Xs[u,f] * Xd[v,f]      (scalar; the SDDMM (D D^T) o S of the paper)
 *       GTO_G_MUL  w_e[f] = Xs[u,f] * Xd[v,f]            (vector; NGCF's element-wise product)
 *   h:  GTO_H_SCALE  w_e * Xs[u]   (scalar weight),  GTO_H_ADD  Xs[u] + w_e,  GTO_H_MUL  Xs[u] (.) w_e
 *   f:  sum or mean over the in-edges of v (mean divides by the in-degree; empty row -> 0).
 * ------------------------------------------------------------------------------------------- */
enum { GTO_G_DOT = 0, GTO_G_MUL = 1 };
enum { GTO_H_SCALE = 0, GTO_H_ADD = 1, GTO_H_MUL = 2 };

/* W: [E] for DOT, [E, F] (row stride F) for MUL */
void gto_neighbor_apply(int64_t n_dst, const int32_t *rowptr, const int32_t *colidx, int g, int64_t F,
                        const double *Xs, const double *Xd, double *W) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_dst; ++v)
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int64_t u = colidx[e];
            if (g == GTO_G_DOT) {
                double acc = 0.0;
                for (int64_t f = 0; f < F; ++f) acc += Xs[(size_t)u * F + f] * Xd[(size_t)v * F + f];
                W[e] = acc;
            } else {
                for (int64_t f = 0; f < F; ++f) W[(size_t)e * F + f] = Xs[(size_t)u * F + f] * Xd[(size_t)v * F + f];
            }
        }
}

/* Derivative of g for upstream dW (same shape as W): edge by edge, applied to both ends
 * (paper, "Training for GNNs": g' is applied for both dst and src nodes).
 * dXs[n_src, F], dXd[n_dst, F] are overwritten. */
void gto_neighbor_apply_bwd(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx, int g,
                            int64_t F, const double *dW, const double *Xs, const double *Xd, double *dXs,
                            double *dXd) {
    for (size_t i = 0; i < (size_t)n_src * F; ++i) dXs[i] = 0.0;
    for (size_t i = 0; i < (size_t)n_dst * F; ++i) dXd[i] = 0.0;
    for (int64_t v = 0; v < n_dst; ++v)
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int64_t u = colidx[e];
            for (int64_t f = 0; f < F; ++f) {
                double d = (g == GTO_G_DOT) ? dW[e] : dW[(size_t)e * F + f];
                dXs[(size_t)u * F + f] += d * Xd[(size_t)v * F + f];
                dXd[(size_t)v * F + f] += d * Xs[(size_t)u * F + f];
            }
        }
}

static double h_apply(int h, double x, const double *W, int64_t e, int64_t F, int64_t f) {
    if (h == GTO_H_SCALE) return W[e] * x;
    if (h == GTO_H_ADD) return x + W[(size_t)e * F + f];
    return x * W[(size_t)e * F + f];
}

/* Y[v,:] = f_{e in in(v)} h(Xs[u,:], W_e);  mean != 0 divides by the in-degree */
void gto_pull(int64_t n_dst, const int32_t *rowptr, const int32_t *colidx, int mean, int h, int64_t F,
              const double *Xs, const double *W, double *Y) {
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t v = 0; v < n_dst; ++v) {
        int32_t deg = rowptr[v + 1] - rowptr[v];
        for (int64_t f = 0; f < F; ++f) {
            double acc = 0.0;
            for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e)
                acc += h_apply(h, Xs[(size_t)colidx[e] * F + f], W, e, F, f);
            if (mean) acc = deg > 0 ? acc / (double)deg : 0.0;
            Y[(size_t)v * F + f] = acc;
        }
    }
}

/* Derivative of Pull for upstream dY: dXs[n_src,F] (scatter over the edges) and dW (shape of W). */
void gto_pull_bwd(int64_t n_dst, int64_t n_src, const int32_t *rowptr, const int32_t *colidx, int mean, int h,
                  int64_t F, const double *dY, const double *Xs, const double *W, double *dXs, double *dW) {
    for (size_t i = 0; i < (size_t)n_src * F; ++i) dXs[i] = 0.0;
    for (int64_t v = 0; v < n_dst; ++v) {
        int32_t deg = rowptr[v + 1] - rowptr[v];
        double c = mean ? 1.0 / (double)deg : 1.0;
        for (int32_t e = rowptr[v]; e < rowptr[v + 1]; ++e) {
            int64_t u = colidx[e];
            if (h == GTO_H_SCALE) dW[e] = 0.0;
            for (int64_t f = 0; f < F; ++f) {
                double up = c * dY[(size_t)v * F + f];          /* d loss / d h(...)[f] */
                double x = Xs[(size_t)u * F + f];
                if (h == GTO_H_SCALE) {
                    dXs[(size_t)u * F + f] += up * W[e];
                    dW[e] += up * x;
                } else if (h == GTO_H_ADD) {
                    dXs[(size_t)u * F + f] += up;
                    dW[(size_t)e * F + f] = up;
                } else {
                    dXs[(size_t)u * F + f] += up * W[(size_t)e * F + f];
                    dW[(size_t)e * F + f] = up * x;
                }
            }
        }
    }
}

/* fp64 -> nearest bf16 value (ties to even), returned as fp64.  bf16 has 8 significant bits
 * and the fp32 exponent range; values below the smallest normal round on the subnormal grid. */
void gto_round_bf16(int64_t n, const double *x, double *y) {
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        if (v == 0.0 || isnan(v) || isinf(v)) { y[i] = v; continue; }
        int e;
        (void)frexp(v, &e);          /* |v| = m * 2^e, m in [0.5, 1)  ->  exponent e-1 */
        int ex = e - 1;
        if (ex < -126) ex = -126;
        double q = ldexp(1.0, ex - 7); /* spacing of bf16 numbers in this binade */
        double r = nearbyint(v / q) * q; /* default rounding mode: ties to even */
        if (fabs(r) > 3.3895313892515355e38) r = v > 0 ? INFINITY : -INFINITY;
        y[i] = r;
    }
}

int gto_num_threads(void) {
    int n = 1;
#ifdef _OPENMP
#pragma omp parallel
    {
#pragma omp single
        n = omp_get_num_threads();
    }
#endif
    return n;
}
