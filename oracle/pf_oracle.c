/*
 * pf_oracle.c -- TEST INFRASTRUCTURE, not the product.
 *
 * Plain, slow, double-precision CPU statement of what Pufferfish's
 * pre-factorized low-rank layers compute (forward and backward), written
 * out from the paper's layer definitions as nested loops.  It exists so the
 * GPU library can be checked against something that can be read by eye; it
 * shares no code with that library and only tests, the smoke check and the
 * benchmark's CPU-baseline leg may call it.
 *
 * Conventions (every array dense row-major, last index fastest, all double):
 *   linear / LSTM : X[M x in], V[in x r] (input-side factor),
 *                   U[out x r] (output-side factor), W = U V^T (out x in),
 *                   T = X V  (M x r),  Y = T U^T + b  (M x out).
 *   conv          : X[N,C,H,W], Uk[r,C,k,k] (thin k x k filters, the paper's
 *                   conv_u), Vp[Cout,r] (1x1 filters, the paper's conv_v),
 *                   T[N,r,Ho,Wo], Y[N,Cout,Ho,Wo]; cross-correlation, zero
 *                   padding, stride on the k x k stage only.
 *
 * Every function names the passage of the paper it restates.  Parity pins
 * for each function live in tests/test_oracle_*.py (library routines, closed
 * forms, finite differences, hand-worked fixtures); no function here is
 * "parity unpinned".
 *
 * The "omp parallel for" pragmas split an outer loop whose iterations write
 * disjoint outputs; they change neither the arithmetic nor its order within
 * one output element.
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

typedef int64_t i64;

int pfo_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void pfo_set_num_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* ------------------------------------------------------------------ */
/* Fully connected layer (Section 2.1; Appendix B "FC layer")          */
/* ------------------------------------------------------------------ */

/* Dense layer  Y = X W^T + b  with W[out x in]: the layer before
 * factorization (Section 2.1, h = sigma(W x) without the activation). */
void pfo_dense_linear_fwd(i64 M, i64 in, i64 out, const double *X,
                          const double *W, const double *bias, double *Y)
{
#pragma omp parallel for schedule(static)
    for (i64 m = 0; m < M; ++m)
        for (i64 o = 0; o < out; ++o) {
            double acc = 0.0;
            for (i64 i = 0; i < in; ++i) acc += X[m * in + i] * W[o * in + i];
            Y[m * out + o] = acc + (bias ? bias[o] : 0.0);
        }
}

/* Factorized layer, W replaced by U V^T (Section 2.1): first the rank-r
 * projection T = X V, then Y = T U^T + b.  T is returned because the
 * backward pass consumes it. */
void pfo_lowrank_linear_fwd(i64 M, i64 in, i64 out, i64 r, const double *X,
                            const double *V, const double *U,
                            const double *bias, double *Y, double *T)
{
#pragma omp parallel for schedule(static)
    for (i64 m = 0; m < M; ++m) {
        for (i64 p = 0; p < r; ++p) {
            double acc = 0.0;
            for (i64 i = 0; i < in; ++i) acc += X[m * in + i] * V[i * r + p];
            T[m * r + p] = acc;
        }
        for (i64 o = 0; o < out; ++o) {
            double acc = 0.0;
            for (i64 p = 0; p < r; ++p) acc += T[m * r + p] * U[o * r + p];
            Y[m * out + o] = acc + (bias ? bias[o] : 0.0);
        }
    }
}

/* Gradients of L through Y = (X V) U^T + b given dY = dL/dY (the chain rule
 * through the two products of Section 2.1; the paper trains U and V, so all
 * of dX, dU, dV, db are needed).  Any output pointer may be NULL. */
void pfo_lowrank_linear_bwd(i64 M, i64 in, i64 out, i64 r, const double *X,
                            const double *V, const double *U, const double *dY,
                            double *dX, double *dU, double *dV, double *db)
{
    double *T = (double *)malloc(sizeof(double) * (size_t)(M * r + 1));
    double *dT = (double *)malloc(sizeof(double) * (size_t)(M * r + 1));
#pragma omp parallel for schedule(static)
    for (i64 m = 0; m < M; ++m)
        for (i64 p = 0; p < r; ++p) {
            double t = 0.0, g = 0.0;
            for (i64 i = 0; i < in; ++i) t += X[m * in + i] * V[i * r + p];
            for (i64 o = 0; o < out; ++o) g += dY[m * out + o] * U[o * r + p];
            T[m * r + p] = t;   /* T  = X V      */
            dT[m * r + p] = g;  /* dT = dY U     */
        }
    if (dX) {
#pragma omp parallel for schedule(static)
        for (i64 m = 0; m < M; ++m)
            for (i64 i = 0; i < in; ++i) {
                double acc = 0.0; /* dX = dT V^T */
                for (i64 p = 0; p < r; ++p) acc += dT[m * r + p] * V[i * r + p];
                dX[m * in + i] = acc;
            }
    }
    if (dU) {
#pragma omp parallel for schedule(static)
        for (i64 o = 0; o < out; ++o)
            for (i64 p = 0; p < r; ++p) {
                double acc = 0.0; /* dU = dY^T T */
                for (i64 m = 0; m < M; ++m) acc += dY[m * out + o] * T[m * r + p];
                dU[o * r + p] = acc;
            }
    }
    if (dV) {
#pragma omp parallel for schedule(static)
        for (i64 i = 0; i < in; ++i)
            for (i64 p = 0; p < r; ++p) {
                double acc = 0.0; /* dV = X^T dT */
                for (i64 m = 0; m < M; ++m) acc += X[m * in + i] * dT[m * r + p];
                dV[i * r + p] = acc;
            }
    }
    if (db) {
        for (i64 o = 0; o < out; ++o) {
            double acc = 0.0;
            for (i64 m = 0; m < M; ++m) acc += dY[m * out + o];
            db[o] = acc;
        }
    }
    free(T);
    free(dT);
}

/* ------------------------------------------------------------------ */
/* Convolution layer (Section 2.2; Appendix B "Convolution layer")     */
/* ------------------------------------------------------------------ */

static i64 conv_out_dim(i64 H, int k, int s, int p)
{
    return (H + 2 * (i64)p - k) / s + 1;
}

i64 pfo_conv_out_dim(i64 H, int k, int s, int p) { return conv_out_dim(H, k, s, p); }

/* Dense k x k convolution with Wd[Cout,C,k,k]: the layer before
 * factorization (Section 2.2 "Basics on convolution layers"). */
void pfo_dense_conv_fwd(i64 N, i64 C, i64 H, i64 W, i64 Cout, int k, int s,
                        int p, const double *X, const double *Wd, double *Y)
{
    const i64 Ho = conv_out_dim(H, k, s, p), Wo = conv_out_dim(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 o = 0; o < Cout; ++o)
            for (i64 y = 0; y < Ho; ++y)
                for (i64 x = 0; x < Wo; ++x) {
                    double acc = 0.0;
                    for (i64 c = 0; c < C; ++c)
                        for (int i = 0; i < k; ++i)
                            for (int j = 0; j < k; ++j) {
                                i64 yy = y * s + i - p, xx = x * s + j - p;
                                if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                acc += Wd[((o * C + c) * k + i) * k + j] *
                                       X[((n * C + c) * H + yy) * W + xx];
                            }
                    Y[((n * Cout + o) * Ho + y) * Wo + x] = acc;
                }
}

/* Factorized convolution (Section 2.2 "Factorizing a convolution layer"):
 * a thin k x k convolution with r filters (stride s, zero padding p)
 * followed by a 1x1 convolution r -> Cout (stride 1, no padding), nothing
 * in between. */
void pfo_lowrank_conv_fwd(i64 N, i64 C, i64 H, i64 W, i64 Cout, i64 r, int k,
                          int s, int p, const double *X, const double *Uk,
                          const double *Vp, double *Y, double *T)
{
    const i64 Ho = conv_out_dim(H, k, s, p), Wo = conv_out_dim(W, k, s, p);
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 q = 0; q < r; ++q)
            for (i64 y = 0; y < Ho; ++y)
                for (i64 x = 0; x < Wo; ++x) {
                    double acc = 0.0;
                    for (i64 c = 0; c < C; ++c)
                        for (int i = 0; i < k; ++i)
                            for (int j = 0; j < k; ++j) {
                                i64 yy = y * s + i - p, xx = x * s + j - p;
                                if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                acc += Uk[((q * C + c) * k + i) * k + j] *
                                       X[((n * C + c) * H + yy) * W + xx];
                            }
                    T[((n * r + q) * Ho + y) * Wo + x] = acc;
                }
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 o = 0; o < Cout; ++o)
            for (i64 y = 0; y < Ho; ++y)
                for (i64 x = 0; x < Wo; ++x) {
                    double acc = 0.0;
                    for (i64 q = 0; q < r; ++q)
                        acc += Vp[o * r + q] * T[((n * r + q) * Ho + y) * Wo + x];
                    Y[((n * Cout + o) * Ho + y) * Wo + x] = acc;
                }
}

/* Gradients through the two stages of the factorized convolution, given
 * dY = dL/dY.  dT is the gradient at the rank-r feature map. */
void pfo_lowrank_conv_bwd(i64 N, i64 C, i64 H, i64 W, i64 Cout, i64 r, int k,
                          int s, int p, const double *X, const double *Uk,
                          const double *Vp, const double *dY, double *dX,
                          double *dUk, double *dVp)
{
    const i64 Ho = conv_out_dim(H, k, s, p), Wo = conv_out_dim(W, k, s, p);
    const size_t nT = (size_t)(N * r * Ho * Wo + 1);
    double *T = (double *)malloc(sizeof(double) * nT);
    double *dT = (double *)malloc(sizeof(double) * nT);
    double *Ytmp = (double *)malloc(sizeof(double) * (size_t)(N * Cout * Ho * Wo + 1));
    pfo_lowrank_conv_fwd(N, C, H, W, Cout, r, k, s, p, X, Uk, Vp, Ytmp, T);
    free(Ytmp);
    /* dT[n,q,y,x] = sum_o Vp[o,q] dY[n,o,y,x] */
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 n = 0; n < N; ++n)
        for (i64 q = 0; q < r; ++q)
            for (i64 y = 0; y < Ho; ++y)
                for (i64 x = 0; x < Wo; ++x) {
                    double acc = 0.0;
                    for (i64 o = 0; o < Cout; ++o)
                        acc += Vp[o * r + q] * dY[((n * Cout + o) * Ho + y) * Wo + x];
                    dT[((n * r + q) * Ho + y) * Wo + x] = acc;
                }
    if (dVp) {
        /* dVp[o,q] = sum_{n,y,x} dY[n,o,y,x] T[n,q,y,x] */
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 o = 0; o < Cout; ++o)
            for (i64 q = 0; q < r; ++q) {
                double acc = 0.0;
                for (i64 n = 0; n < N; ++n)
                    for (i64 y = 0; y < Ho; ++y)
                        for (i64 x = 0; x < Wo; ++x)
                            acc += dY[((n * Cout + o) * Ho + y) * Wo + x] *
                                   T[((n * r + q) * Ho + y) * Wo + x];
                dVp[o * r + q] = acc;
            }
    }
    if (dUk) {
        /* dUk[q,c,i,j] = sum_{n,y,x} dT[n,q,y,x] Xpad[n,c,y s+i-p,x s+j-p] */
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 q = 0; q < r; ++q)
            for (i64 c = 0; c < C; ++c)
                for (int i = 0; i < k; ++i)
                    for (int j = 0; j < k; ++j) {
                        double acc = 0.0;
                        for (i64 n = 0; n < N; ++n)
                            for (i64 y = 0; y < Ho; ++y)
                                for (i64 x = 0; x < Wo; ++x) {
                                    i64 yy = y * s + i - p, xx = x * s + j - p;
                                    if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                    acc += dT[((n * r + q) * Ho + y) * Wo + x] *
                                           X[((n * C + c) * H + yy) * W + xx];
                                }
                        dUk[((q * C + c) * k + i) * k + j] = acc;
                    }
    }
    if (dX) {
        /* dX[n,c,yy,xx] = sum over every (q,y,x,i,j) whose window touches
         * (yy,xx): scatter form of the definition, one image/channel plane
         * per iteration so planes never overlap between threads. */
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 n = 0; n < N; ++n)
            for (i64 c = 0; c < C; ++c) {
                double *plane = dX + (n * C + c) * H * W;
                for (i64 e = 0; e < H * W; ++e) plane[e] = 0.0;
                for (i64 q = 0; q < r; ++q)
                    for (i64 y = 0; y < Ho; ++y)
                        for (i64 x = 0; x < Wo; ++x) {
                            double g = dT[((n * r + q) * Ho + y) * Wo + x];
                            for (int i = 0; i < k; ++i)
                                for (int j = 0; j < k; ++j) {
                                    i64 yy = y * s + i - p, xx = x * s + j - p;
                                    if (yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                                    plane[yy * W + xx] +=
                                        g * Uk[((q * C + c) * k + i) * k + j];
                                }
                        }
            }
    }
    free(T);
    free(dT);
}

/* ------------------------------------------------------------------ */
/* LSTM cell (Section 2.3, eq. (1) dense and eq. (2) factorized)       */
/* ------------------------------------------------------------------ */

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* One step of the textbook LSTM, eq. (1).  Wx[4h x d], Wh[4h x h], gate
 * blocks stacked in the order i, f, g, o; one bias vector b[4h] standing
 * for the sum of the equation's two. */
void pfo_dense_lstm_cell_fwd(i64 B, i64 d, i64 h, const double *x,
                             const double *hprev, const double *cprev,
                             const double *Wx, const double *Wh,
                             const double *bias, double *h_out, double *c_out)
{
#pragma omp parallel for schedule(static)
    for (i64 b = 0; b < B; ++b)
        for (i64 j = 0; j < h; ++j) {
            double z[4];
            for (int g = 0; g < 4; ++g) {
                i64 row = g * h + j;
                double acc = bias ? bias[row] : 0.0;
                for (i64 i = 0; i < d; ++i) acc += Wx[row * d + i] * x[b * d + i];
                for (i64 i = 0; i < h; ++i) acc += Wh[row * h + i] * hprev[b * h + i];
                z[g] = acc;
            }
            double ig = sigmoid(z[0]), fg = sigmoid(z[1]), gg = tanh(z[2]),
                   og = sigmoid(z[3]);
            double c = fg * cprev[b * h + j] + ig * gg;
            c_out[b * h + j] = c;
            h_out[b * h + j] = og * tanh(c);
        }
}

/* One step of the factorized LSTM, eq. (2).
 *   groups == 4: every gate has its own factor pair, as eq. (2) and the
 *     paper's LSTM architecture table have it: Vx[d x 4r], gate g uses
 *     columns g r .. (g+1) r - 1; Ux[4h x r], rows g h .. (g+1) h - 1.
 *   groups == 1: the stacked 4h x d matrix is factorized as one rank-r
 *     product: Vx[d x r] shared by the four gates, Ux[4h x r].
 * Tx[B x groups r] = x Vx, Th[B x groups r] = hprev Vh.
 * gates[B x 4h] holds the activated i, f, g, o. */
void pfo_lowrank_lstm_cell_fwd(i64 B, i64 d, i64 h, i64 r, int groups,
                               const double *x, const double *hprev,
                               const double *cprev, const double *Vx,
                               const double *Ux, const double *Vh,
                               const double *Uh, const double *bias,
                               double *h_out, double *c_out, double *gates,
                               double *Tx, double *Th)
{
    const i64 gr = (i64)groups * r;
#pragma omp parallel for schedule(static)
    for (i64 b = 0; b < B; ++b) {
        for (i64 q = 0; q < gr; ++q) {
            double ax = 0.0, ah = 0.0;
            for (i64 i = 0; i < d; ++i) ax += x[b * d + i] * Vx[i * gr + q];
            for (i64 i = 0; i < h; ++i) ah += hprev[b * h + i] * Vh[i * gr + q];
            Tx[b * gr + q] = ax;
            Th[b * gr + q] = ah;
        }
        for (i64 j = 0; j < h; ++j) {
            double z[4];
            for (int g = 0; g < 4; ++g) {
                i64 row = g * h + j;
                i64 off = (groups == 4) ? g * r : 0;
                double acc = bias ? bias[row] : 0.0;
                for (i64 q = 0; q < r; ++q) acc += Ux[row * r + q] * Tx[b * gr + off + q];
                for (i64 q = 0; q < r; ++q) acc += Uh[row * r + q] * Th[b * gr + off + q];
                z[g] = acc;
            }
            double ig = sigmoid(z[0]), fg = sigmoid(z[1]), gg = tanh(z[2]),
                   og = sigmoid(z[3]);
            double c = fg * cprev[b * h + j] + ig * gg;
            gates[b * 4 * h + 0 * h + j] = ig;
            gates[b * 4 * h + 1 * h + j] = fg;
            gates[b * 4 * h + 2 * h + j] = gg;
            gates[b * 4 * h + 3 * h + j] = og;
            c_out[b * h + j] = c;
            h_out[b * h + j] = og * tanh(c);
        }
    }
}

/* Backward of one factorized LSTM step (derivative of eq. (2)).
 * Inputs dh = dL/dh_t (sum of the gradient from the layer above and from
 * step t+1), dc_next = dL/dc_t arriving from step t+1 (NULL = 0).
 * Outputs: dx, dh_prev, dc_prev, and the parameter gradients, which are
 * written (accumulate == 0) or added to (accumulate != 0), since the same
 * factors serve every time step. */
void pfo_lowrank_lstm_cell_bwd(i64 B, i64 d, i64 h, i64 r, int groups,
                               const double *x, const double *hprev,
                               const double *cprev, const double *c_out,
                               const double *gates, const double *Tx,
                               const double *Th, const double *Vx,
                               const double *Ux, const double *Vh,
                               const double *Uh, const double *dh,
                               const double *dc_next, double *dx,
                               double *dh_prev, double *dc_prev, double *dVx,
                               double *dUx, double *dVh, double *dUh,
                               double *dbias, int accumulate)
{
    const i64 gr = (i64)groups * r;
    double *dz = (double *)malloc(sizeof(double) * (size_t)(B * 4 * h + 1));
    double *dTx = (double *)malloc(sizeof(double) * (size_t)(B * gr + 1));
    double *dTh = (double *)malloc(sizeof(double) * (size_t)(B * gr + 1));
    /* gate derivatives */
#pragma omp parallel for schedule(static)
    for (i64 b = 0; b < B; ++b)
        for (i64 j = 0; j < h; ++j) {
            double ig = gates[b * 4 * h + 0 * h + j], fg = gates[b * 4 * h + 1 * h + j];
            double gg = gates[b * 4 * h + 2 * h + j], og = gates[b * 4 * h + 3 * h + j];
            double tc = tanh(c_out[b * h + j]);
            double dhv = dh[b * h + j];
            double dc = (dc_next ? dc_next[b * h + j] : 0.0) + dhv * og * (1.0 - tc * tc);
            double d_o = dhv * tc, d_i = dc * gg, d_f = dc * cprev[b * h + j], d_g = dc * ig;
            if (dc_prev) dc_prev[b * h + j] = dc * fg;
            dz[b * 4 * h + 0 * h + j] = d_i * ig * (1.0 - ig);
            dz[b * 4 * h + 1 * h + j] = d_f * fg * (1.0 - fg);
            dz[b * 4 * h + 2 * h + j] = d_g * (1.0 - gg * gg);
            dz[b * 4 * h + 3 * h + j] = d_o * og * (1.0 - og);
        }
    /* dTx = dz Ux, dTh = dz Uh (per gate group when groups == 4) */
#pragma omp parallel for collapse(2) schedule(static)
    for (i64 b = 0; b < B; ++b)
        for (i64 q = 0; q < gr; ++q) {
            double ax = 0.0, ah = 0.0;
            int g0 = (groups == 4) ? (int)(q / r) : 0;
            int g1 = (groups == 4) ? g0 + 1 : 4;
            i64 qq = (groups == 4) ? q % r : q;
            for (int g = g0; g < g1; ++g)
                for (i64 j = 0; j < h; ++j) {
                    double v = dz[b * 4 * h + g * h + j];
                    ax += v * Ux[(g * h + j) * r + qq];
                    ah += v * Uh[(g * h + j) * r + qq];
                }
            dTx[b * gr + q] = ax;
            dTh[b * gr + q] = ah;
        }
    if (dx)
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 b = 0; b < B; ++b)
            for (i64 i = 0; i < d; ++i) {
                double acc = 0.0;
                for (i64 q = 0; q < gr; ++q) acc += dTx[b * gr + q] * Vx[i * gr + q];
                dx[b * d + i] = acc;
            }
    if (dh_prev)
#pragma omp parallel for collapse(2) schedule(static)
        for (i64 b = 0; b < B; ++b)
            for (i64 i = 0; i < h; ++i) {
                double acc = 0.0;
                for (i64 q = 0; q < gr; ++q) acc += dTh[b * gr + q] * Vh[i * gr + q];
                dh_prev[b * h + i] = acc;
            }
    /* parameter gradients */
#pragma omp parallel for schedule(static)
    for (i64 row = 0; row < 4 * h; ++row) {
        i64 off = (groups == 4) ? (row / h) * r : 0;
        for (i64 q = 0; q < r; ++q) {
            double ax = 0.0, ah = 0.0;
            for (i64 b = 0; b < B; ++b) {
                ax += dz[b * 4 * h + row] * Tx[b * gr + off + q];
                ah += dz[b * 4 * h + row] * Th[b * gr + off + q];
            }
            if (dUx) dUx[row * r + q] = (accumulate ? dUx[row * r + q] : 0.0) + ax;
            if (dUh) dUh[row * r + q] = (accumulate ? dUh[row * r + q] : 0.0) + ah;
        }
        if (dbias) {
            double acc = 0.0;
            for (i64 b = 0; b < B; ++b) acc += dz[b * 4 * h + row];
            dbias[row] = (accumulate ? dbias[row] : 0.0) + acc;
        }
    }
    if (dVx)
#pragma omp parallel for schedule(static)
        for (i64 i = 0; i < d; ++i)
            for (i64 q = 0; q < gr; ++q) {
                double acc = 0.0;
                for (i64 b = 0; b < B; ++b) acc += x[b * d + i] * dTx[b * gr + q];
                dVx[i * gr + q] = (accumulate ? dVx[i * gr + q] : 0.0) + acc;
            }
    if (dVh)
#pragma omp parallel for schedule(static)
        for (i64 i = 0; i < h; ++i)
            for (i64 q = 0; q < gr; ++q) {
                double acc = 0.0;
                for (i64 b = 0; b < B; ++b) acc += hprev[b * h + i] * dTh[b * gr + q];
                dVh[i * gr + q] = (accumulate ? dVh[i * gr + q] : 0.0) + acc;
            }
    free(dz);
    free(dTx);
    free(dTh);
}

/* ------------------------------------------------------------------ */
/* Factor initialisation (Algorithm 1, the SVD step; Section 3          */
/* "Vanilla warm-up training")                                         */
/* ------------------------------------------------------------------ */

/* Truncated SVD of W[m x n] (W = Ut S Vt^T) by one-sided Jacobi rotations
 * on the columns, then the balanced split of Algorithm 1:
 *   U = Ut_r S_r^(1/2)  (m x r),   V = Vt_r S_r^(1/2)  (n x r),
 * so that U V^T is the best rank-r approximation of W.  sigma receives all
 * min(m,n) singular values in descending order.  Returns the sweep count,
 * or -1 if it did not converge. */
int pfo_svd_split(i64 m, i64 n, i64 r, const double *W, double *U, double *V,
                  double *sigma)
{
    /* Work on A = W (m x n) if m >= n, else on W^T, so rows >= cols. */
    const int transposed = m < n;
    const i64 rows = transposed ? n : m, cols = transposed ? m : n;
    double *A = (double *)malloc(sizeof(double) * (size_t)(rows * cols + 1));
    double *Q = (double *)calloc((size_t)(cols * cols + 1), sizeof(double));
    for (i64 i = 0; i < rows; ++i)
        for (i64 j = 0; j < cols; ++j)
            A[i * cols + j] = transposed ? W[j * n + i] : W[i * n + j];
    for (i64 j = 0; j < cols; ++j) Q[j * cols + j] = 1.0;

    int sweep, converged = 0;
    for (sweep = 0; sweep < 60 && !converged; ++sweep) {
        converged = 1;
        for (i64 a = 0; a < cols - 1; ++a)
            for (i64 b = a + 1; b < cols; ++b) {
                double alpha = 0.0, beta = 0.0, gamma = 0.0;
                for (i64 i = 0; i < rows; ++i) {
                    double va = A[i * cols + a], vb = A[i * cols + b];
                    alpha += va * va;
                    beta += vb * vb;
                    gamma += va * vb;
                }
                if (fabs(gamma) <= 1e-15 * sqrt(alpha * beta) || gamma == 0.0) continue;
                converged = 0;
                double zeta = (beta - alpha) / (2.0 * gamma);
                double t = (zeta >= 0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                double c = 1.0 / sqrt(1.0 + t * t), s = c * t;
                for (i64 i = 0; i < rows; ++i) {
                    double va = A[i * cols + a], vb = A[i * cols + b];
                    A[i * cols + a] = c * va - s * vb;
                    A[i * cols + b] = s * va + c * vb;
                }
                for (i64 i = 0; i < cols; ++i) {
                    double va = Q[i * cols + a], vb = Q[i * cols + b];
                    Q[i * cols + a] = c * va - s * vb;
                    Q[i * cols + b] = s * va + c * vb;
                }
            }
    }
    /* column norms = singular values; order them descending */
    double *sv = (double *)malloc(sizeof(double) * (size_t)(cols + 1));
    i64 *order = (i64 *)malloc(sizeof(i64) * (size_t)(cols + 1));
    for (i64 j = 0; j < cols; ++j) {
        double acc = 0.0;
        for (i64 i = 0; i < rows; ++i) acc += A[i * cols + j] * A[i * cols + j];
        sv[j] = sqrt(acc);
        order[j] = j;
    }
    for (i64 a = 0; a < cols; ++a)
        for (i64 b = a + 1; b < cols; ++b)
            if (sv[order[b]] > sv[order[a]]) {
                i64 t = order[a];
                order[a] = order[b];
                order[b] = t;
            }
    for (i64 j = 0; j < cols; ++j) sigma[j] = sv[order[j]];
    /* A[:,j] = sigma_j * left vector, Q[:,j] = right vector (of A).
     * For the transposed case left/right swap roles for W. */
    for (i64 q = 0; q < r; ++q) {
        i64 j = order[q];
        double s = sv[j], rs = sqrt(s);
        for (i64 i = 0; i < rows; ++i) {
            double left = (s > 0.0) ? A[i * cols + j] / s : 0.0;
            if (transposed) V[i * r + q] = left * rs; else U[i * r + q] = left * rs;
        }
        for (i64 i = 0; i < cols; ++i) {
            double right = Q[i * cols + j];
            if (transposed) U[i * r + q] = right * rs; else V[i * r + q] = right * rs;
        }
    }
    free(A);
    free(Q);
    free(sv);
    free(order);
    return converged ? sweep : -1;
}
