/*
 * TEST INFRASTRUCTURE ONLY -- the slow CPU oracle's convolution primitives.
 *
 * Direct-loop 2-D cross-correlation and its two adjoints, in fp64, NCHW.
 * Nothing here is blocked, fused or reordered: every function is the plain
 * definition of a convolutional layer (the "standard 3-convolutional-layer
 * network" of the paper's appendix "Atari Frame Processing") written as nested
 * loops, so that it can be checked against the definition by eye.
 *
 * Only tests, the smoke check and the CPU-baseline leg of the benchmark may
 * link this file.  The GPU library shares no code with it.
 *
 * Definition (no kernel flip, zero padding `pad` on every side, stride `s`):
 *
 *   OH = floor((H + 2 pad - k) / s) + 1,  OW likewise
 *   pre[n,co,oy,ox] = b[co] + sum_{ci,ky,kx} W[co,ci,ky,kx] *
 *                     x[n,ci, oy*s + ky - pad, ox*s + kx - pad]
 *
 * with x taken as zero outside [0,H) x [0,Wd).
 *
 * Parallelism: OpenMP over samples only (each sample is independent in the
 * forward and input-gradient passes; the weight gradient is accumulated per
 * fixed group of samples and the groups are summed in order afterwards, so the
 * result does not depend on the thread count).
 */
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int orc_out_size(int H, int k, int s, int pad) {
    int span = H + 2 * pad - k;
    if (span < 0) return 0;
    return span / s + 1;
}

/* pre = b + W (*) x          x:[N,Cin,H,Wd]  W:[Cout,Cin,k,k]  pre:[N,Cout,OH,OW] */
void orc_conv2d_forward(const double *x, const double *W, const double *b, double *pre,
                        int N, int Cin, int H, int Wd, int Cout, int k, int s, int pad) {
    const int OH = orc_out_size(H, k, s, pad), OW = orc_out_size(Wd, k, s, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Cout; ++co)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    double acc = b ? b[co] : 0.0;
                    for (int ci = 0; ci < Cin; ++ci)
                        for (int ky = 0; ky < k; ++ky) {
                            const int y = oy * s + ky - pad;
                            if (y < 0 || y >= H) continue;
                            for (int kx = 0; kx < k; ++kx) {
                                const int xx = ox * s + kx - pad;
                                if (xx < 0 || xx >= Wd) continue;
                                acc += W[(((size_t)co * Cin + ci) * k + ky) * k + kx] *
                                       x[(((size_t)n * Cin + ci) * H + y) * Wd + xx];
                            }
                        }
                    pre[(((size_t)n * Cout + co) * OH + oy) * OW + ox] = acc;
                }
}

/* dx[n,ci,y,xx] = sum over every (co,oy,ox,ky,kx) whose window touches (y,xx) of
 *                 W[co,ci,ky,kx] * dpre[n,co,oy,ox]
 * written as a scatter that walks the forward loop nest.                         */
void orc_conv2d_input_grad(const double *W, const double *dpre, double *dx,
                           int N, int Cin, int H, int Wd, int Cout, int k, int s, int pad) {
    const int OH = orc_out_size(H, k, s, pad), OW = orc_out_size(Wd, k, s, pad);
#pragma omp parallel for schedule(static)
    for (int n = 0; n < N; ++n) {
        double *dxn = dx + (size_t)n * Cin * H * Wd;
        memset(dxn, 0, sizeof(double) * (size_t)Cin * H * Wd);
        for (int co = 0; co < Cout; ++co)
            for (int oy = 0; oy < OH; ++oy)
                for (int ox = 0; ox < OW; ++ox) {
                    const double g = dpre[(((size_t)n * Cout + co) * OH + oy) * OW + ox];
                    if (g == 0.0) continue;
                    for (int ci = 0; ci < Cin; ++ci)
                        for (int ky = 0; ky < k; ++ky) {
                            const int y = oy * s + ky - pad;
                            if (y < 0 || y >= H) continue;
                            for (int kx = 0; kx < k; ++kx) {
                                const int xx = ox * s + kx - pad;
                                if (xx < 0 || xx >= Wd) continue;
                                dxn[((size_t)ci * H + y) * Wd + xx] +=
                                    W[(((size_t)co * Cin + ci) * k + ky) * k + kx] * g;
                            }
                        }
                }
    }
}

/* dW[co,ci,ky,kx] = sum_{n,oy,ox} dpre[n,co,oy,ox] * x[n,ci,oy*s+ky-pad,ox*s+kx-pad]
 * db[co]          = sum_{n,oy,ox} dpre[n,co,oy,ox]
 * Samples are taken in fixed groups of ORC_GROUP; each group's contribution is
 * accumulated on its own (in sample order) and the groups are then added in
 * group order, so the sum order is fixed whatever the thread count.              */
#define ORC_GROUP 32
void orc_conv2d_weight_grad(const double *x, const double *dpre, double *dW, double *db,
                            int N, int Cin, int H, int Wd, int Cout, int k, int s, int pad) {
    const int OH = orc_out_size(H, k, s, pad), OW = orc_out_size(Wd, k, s, pad);
    const size_t wsz = (size_t)Cout * Cin * k * k;
    const int G = (N + ORC_GROUP - 1) / ORC_GROUP;
    double *per = (double *)calloc((size_t)(G > 0 ? G : 1) * (wsz + Cout), sizeof(double));
#pragma omp parallel for schedule(static)
    for (int g_ = 0; g_ < G; ++g_) {
        double *w = per + (size_t)g_ * (wsz + Cout);
        double *bb = w + wsz;
        const int n_end = (g_ + 1) * ORC_GROUP < N ? (g_ + 1) * ORC_GROUP : N;
        for (int n = g_ * ORC_GROUP; n < n_end; ++n)
            for (int co = 0; co < Cout; ++co)
                for (int oy = 0; oy < OH; ++oy)
                    for (int ox = 0; ox < OW; ++ox) {
                        const double g = dpre[(((size_t)n * Cout + co) * OH + oy) * OW + ox];
                        bb[co] += g;
                        if (g == 0.0) continue;
                        for (int ci = 0; ci < Cin; ++ci)
                            for (int ky = 0; ky < k; ++ky) {
                                const int y = oy * s + ky - pad;
                                if (y < 0 || y >= H) continue;
                                for (int kx = 0; kx < k; ++kx) {
                                    const int xx = ox * s + kx - pad;
                                    if (xx < 0 || xx >= Wd) continue;
                                    w[(((size_t)co * Cin + ci) * k + ky) * k + kx] +=
                                        g * x[(((size_t)n * Cin + ci) * H + y) * Wd + xx];
                                }
                            }
                    }
    }
    memset(dW, 0, sizeof(double) * wsz);
    memset(db, 0, sizeof(double) * Cout);
    for (int g_ = 0; g_ < G; ++g_) {
        const double *w = per + (size_t)g_ * (wsz + Cout);
        for (size_t i = 0; i < wsz; ++i) dW[i] += w[i];
        for (int co = 0; co < Cout; ++co) db[co] += w[wsz + co];
    }
    free(per);
}
