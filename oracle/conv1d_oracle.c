/*
 * FP64 direct-summation oracle for the 1D dilated convolution layer.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call this file;
 * it exists so that tests, the smoke check and the benchmark's CPU-baseline
 * leg have an independent, slow, obviously-correct answer.  It shares no
 * code, header, table or helper with the HIP kernels.
 *
 * What it computes (paper Section 2, Eq. 2, read as the cross-correlation
 * that Algorithm 1 / Algorithm 2 actually index: input column q + s*d feeds
 * output column q through tap s; zero padding at the edges, Section 2 last
 * paragraph):
 *
 *   fwd        Y [n,k,q] = sum_c sum_s X[n,c,q + s*d - P] * Wt[k,c,s]      X = 0 outside [0,W)
 *   bwd_data   dX[n,c,i] = sum_k sum_s Wt[k,c,s] * dY[n,k,i + P - s*d]     dY = 0 outside [0,Q)
 *              (Section 3.2: the adjoint of fwd in X)
 *   bwd_weight dW[k,c,s] = sum_n sum_q X[n,c,q + s*d - P] * dY[n,k,q]
 *              (Section 3.3, Algorithm 4: the adjoint of fwd in Wt)
 *
 * with Q = W + 2P - (S-1)*d.  Every function optionally fills a companion
 * array with the same sum taken over |product|; that is the denominator of
 * the parity metric  |gpu - oracle| / sum|products|.
 *
 * Layouts (row-major, contiguous):  X[N][C][W], Wt[K][C][S], Y/dY[N][K][Q],
 * dX[N][C][W], dW[K][C][S].  Plain nested loops, no blocking, no GEMM call.
 * OpenMP splits independent output elements across threads and never splits
 * a reduction, so results do not depend on the thread count.
 *
 * Epilogue (conv1d_oracle_epilogue): what a framework does to the layer's
 * output next.  Section 3 leaves the bias to the framework: z = y + bias[k].
 * Section 4.4 follows the layer with a ReLU that stays in BF16: a = max(z, 0),
 * stored as bfloat16 (nearest value, ties to the even significand).  Each of
 * the three steps is optional.  The magnitude companion gains |bias[k]|.
 *
 * The *_at variants evaluate the same definitions at a caller-given list of
 * output coordinates (for full-size workloads where the whole output would
 * take minutes).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int conv1d_oracle_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Q from Section 2 / Fig. 1: stride 1, P zeros on each side. */
long conv1d_oracle_out_width(long W, long S, long d, long P)
{
    return W + 2 * P - (S - 1) * d;
}

/* ---- forward: Eq. 2 with Algorithm 1's indexing ------------------------- */
void conv1d_oracle_fwd(const double *x, const double *wt, double *y, double *yabs,
                       long N, long C, long K, long W, long S, long d, long P)
{
    const long Q = conv1d_oracle_out_width(W, S, d, P);
    if (Q <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (long n = 0; n < N; ++n)
        for (long k = 0; k < K; ++k) {
            double *yr = y + (n * K + k) * Q;
            double *ar = yabs ? yabs + (n * K + k) * Q : NULL;
            for (long q = 0; q < Q; ++q) {
                double acc = 0.0, aacc = 0.0;
                for (long c = 0; c < C; ++c) {
                    const double *xr = x + (n * C + c) * W;
                    const double *wr = wt + (k * C + c) * S;
                    for (long s = 0; s < S; ++s) {
                        const long i = q + s * d - P;
                        if (i >= 0 && i < W) {
                            const double p = xr[i] * wr[s];
                            acc += p;
                            aacc += fabs(p);
                        }
                    }
                }
                yr[q] = acc;
                if (ar) ar[q] = aacc;
            }
        }
}

/* ---- backward data: adjoint of fwd with respect to X (Section 3.2) ------ */
void conv1d_oracle_bwd_data(const double *dy, const double *wt, double *dx, double *dxabs,
                            long N, long C, long K, long W, long S, long d, long P)
{
    const long Q = conv1d_oracle_out_width(W, S, d, P);
    if (Q <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (long n = 0; n < N; ++n)
        for (long c = 0; c < C; ++c) {
            double *dr = dx + (n * C + c) * W;
            double *ar = dxabs ? dxabs + (n * C + c) * W : NULL;
            for (long i = 0; i < W; ++i) {
                double acc = 0.0, aacc = 0.0;
                for (long k = 0; k < K; ++k) {
                    const double *gr = dy + (n * K + k) * Q;
                    const double *wr = wt + (k * C + c) * S;
                    for (long s = 0; s < S; ++s) {
                        const long q = i + P - s * d;
                        if (q >= 0 && q < Q) {
                            const double p = wr[s] * gr[q];
                            acc += p;
                            aacc += fabs(p);
                        }
                    }
                }
                dr[i] = acc;
                if (ar) ar[i] = aacc;
            }
        }
}

/* ---- backward weight: adjoint of fwd with respect to Wt (Section 3.3) --- */
void conv1d_oracle_bwd_weight(const double *x, const double *dy, double *dw, double *dwabs,
                              long N, long C, long K, long W, long S, long d, long P)
{
    const long Q = conv1d_oracle_out_width(W, S, d, P);
    if (Q <= 0) return;
#pragma omp parallel for collapse(3) schedule(static)
    for (long k = 0; k < K; ++k)
        for (long c = 0; c < C; ++c)
            for (long s = 0; s < S; ++s) {
                double acc = 0.0, aacc = 0.0;
                for (long n = 0; n < N; ++n) {
                    const double *xr = x + (n * C + c) * W;
                    const double *gr = dy + (n * K + k) * Q;
                    for (long q = 0; q < Q; ++q) {
                        const long i = q + s * d - P;
                        if (i >= 0 && i < W) {
                            const double p = xr[i] * gr[q];
                            acc += p;
                            aacc += fabs(p);
                        }
                    }
                }
                dw[(k * C + c) * S + s] = acc;
                if (dwabs) dwabs[(k * C + c) * S + s] = aacc;
            }
}

/* ---- the same three definitions at sampled output coordinates ----------- */
/* idx holds `count` triples: (n,k,q) for fwd, (n,c,i) for bwd_data,
 * (k,c,s) for bwd_weight.  out/outabs receive one value per triple. */
void conv1d_oracle_fwd_at(const double *x, const double *wt, const int64_t *idx, long count,
                          double *out, double *outabs,
                          long N, long C, long K, long W, long S, long d, long P)
{
    (void)N;
    (void)K;
#pragma omp parallel for schedule(static)
    for (long t = 0; t < count; ++t) {
        const long n = idx[3 * t], k = idx[3 * t + 1], q = idx[3 * t + 2];
        double acc = 0.0, aacc = 0.0;
        for (long c = 0; c < C; ++c)
            for (long s = 0; s < S; ++s) {
                const long i = q + s * d - P;
                if (i >= 0 && i < W) {
                    const double p = x[(n * C + c) * W + i] * wt[(k * C + c) * S + s];
                    acc += p;
                    aacc += fabs(p);
                }
            }
        out[t] = acc;
        if (outabs) outabs[t] = aacc;
    }
}

void conv1d_oracle_bwd_data_at(const double *dy, const double *wt, const int64_t *idx, long count,
                               double *out, double *outabs,
                               long N, long C, long K, long W, long S, long d, long P)
{
    (void)N;
    (void)W;
    const long Q = conv1d_oracle_out_width(W, S, d, P);
#pragma omp parallel for schedule(static)
    for (long t = 0; t < count; ++t) {
        const long n = idx[3 * t], c = idx[3 * t + 1], i = idx[3 * t + 2];
        double acc = 0.0, aacc = 0.0;
        for (long k = 0; k < K; ++k)
            for (long s = 0; s < S; ++s) {
                const long q = i + P - s * d;
                if (q >= 0 && q < Q) {
                    const double p = wt[(k * C + c) * S + s] * dy[(n * K + k) * Q + q];
                    acc += p;
                    aacc += fabs(p);
                }
            }
        out[t] = acc;
        if (outabs) outabs[t] = aacc;
    }
}

void conv1d_oracle_bwd_weight_at(const double *x, const double *dy, const int64_t *idx, long count,
                                 double *out, double *outabs,
                                 long N, long C, long K, long W, long S, long d, long P)
{
    (void)S;
    const long Q = conv1d_oracle_out_width(W, S, d, P);
#pragma omp parallel for schedule(dynamic, 1)
    for (long t = 0; t < count; ++t) {
        const long k = idx[3 * t], c = idx[3 * t + 1], s = idx[3 * t + 2];
        double acc = 0.0, aacc = 0.0;
        for (long n = 0; n < N; ++n)
            for (long q = 0; q < Q; ++q) {
                const long i = q + s * d - P;
                if (i >= 0 && i < W) {
                    const double p = x[(n * C + c) * W + i] * dy[(n * K + k) * Q + q];
                    acc += p;
                    aacc += fabs(p);
                }
            }
        out[t] = acc;
        if (outabs) outabs[t] = aacc;
    }
}

/* ---- epilogue: bias (Section 3), ReLU and BF16 storage (Section 4.4) ----- */
/* Nearest bfloat16 (8 significant bits, exponent range of binary32), ties to
 * even, written from the definition: scale the significand to 8 bits, round
 * to the nearest integer in the default (ties-to-even) mode, scale back.
 * Below 2^-126 the spacing stays 2^-133 (subnormals); beyond the largest
 * finite bfloat16 the result is +-infinity. */
double conv1d_oracle_round_bf16(double v)
{
    if (v == 0.0 || isnan(v) || isinf(v)) return v;
    int e;
    (void)frexp(v, &e);               /* |v| = m * 2^e, m in [0.5, 1) */
    int lsb = e - 8;                  /* exponent of the last kept bit */
    if (lsb < -133) lsb = -133;
    const double r = ldexp(nearbyint(ldexp(v, -lsb)), lsb);
    const double max_bf16 = ldexp(255.0, 120);   /* (2 - 2^-7) * 2^127 */
    if (fabs(r) > max_bf16) return v > 0 ? INFINITY : -INFINITY;
    return r;
}

/* y[n][k][q] (rows = N*K, each of `width` columns) is updated in place:
 * + bias[row % K] if bias != NULL, then max(.,0) if relu, then rounded to
 * bfloat16 if round_bf16.  yabs (may be NULL) gains |bias|. */
void conv1d_oracle_epilogue(double *y, double *yabs, const double *bias, long N, long K, long width,
                            int relu, int round_bf16)
{
#pragma omp parallel for schedule(static)
    for (long r = 0; r < N * K; ++r) {
        const double b = bias ? bias[r % K] : 0.0;
        for (long q = 0; q < width; ++q) {
            double z = y[r * width + q] + b;
            if (relu && z < 0.0) z = 0.0;
            if (round_bf16) z = conv1d_oracle_round_bf16(z);
            y[r * width + q] = z;
            if (yabs) yabs[r * width + q] += fabs(b);
        }
    }
}
