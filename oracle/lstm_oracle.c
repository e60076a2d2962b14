/*
 * CPU oracle for the stacked LSTM forward pass.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision loops that follow the cell equations of the paper
 * (Section 4, the equation block defining f_t, i_t, o_t, g_t, c_t, h_t) with zero
 * hidden layers inside each gate (the "*" of H* taken as zero, i.e. the conventional
 * LSTM cell the paper uses as its baseline, Section 5):
 *
 *     a_q  = b_q + W_q . [x_t , h_{t-1}]          q in {f, i, o, g}
 *     f,i,o = sigmoid(a_f), sigmoid(a_i), sigmoid(a_o) ;  g = tanh(a_g)
 *     c_t  = f * c_{t-1} + i * g
 *     h_t  = o * tanh(c_t)
 *
 * The weight of each gate acts on the concatenation [x_t, h_{t-1}]; it is passed here
 * as its two column blocks Wx (acting on x_t) and Wh (acting on h_{t-1}).  The four
 * gates are stacked along the rows in the paper's order f, i, o, g.
 *
 * Masks (Section 4, "mask-based approach": every weight matrix has a binary mask of the
 * same size, and the effective weight is W (x) Msk): an entry whose mask byte is 0 is
 * skipped, so whatever value is stored under it never enters the sum.  A NULL mask
 * means every entry is kept.
 *
 * Stacking (Section 5.1: stacked LSTM layers; Section 5.2: bidirectional recurrent
 * layers): layer l+1 reads the hidden-state sequence of layer l.  With two directions,
 * direction 1 walks t = T-1 .. 0, its state is stored at the input position it was
 * computed for, and the two directions are concatenated on the feature axis
 * (forward first) to form the next layer's input.
 *
 * Nothing here is blocked, fused or reordered: one dot product per gate row, summed in
 * index order (bias, then the x terms k = 0.., then the h terms k = 0..).  OpenMP only
 * distributes independent (batch, hidden-unit) outputs of one timestep over threads, so
 * the result does not depend on the thread count.
 *
 * This file shares no code, header or table with the GPU library and must never be
 * linked into or called from it.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static double sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/* b + sum_k Wx[k]*xv[k] (kept entries only) + sum_k Wh[k]*hv[k] (kept entries only) */
static double gate_preact(double bias,
                          const float *wx, const unsigned char *mx, const double *xv, int D,
                          const float *wh, const unsigned char *mh, const double *hv, int H)
{
    double a = bias;
    for (int k = 0; k < D; ++k) {
        if (mx == NULL || mx[k]) a += (double)wx[k] * xv[k];
    }
    for (int k = 0; k < H; ++k) {
        if (mh == NULL || mh[k]) a += (double)wh[k] * hv[k];
    }
    return a;
}

/*
 * L layers, ndir in {1,2} directions, D0 = width of x, H = hidden width.
 * Per (layer l, direction d), index n = l*ndir + d:
 *   Wx[n] float [4H, D_l] row-major (D_0 = D0, D_l = ndir*H for l > 0), Mx[n] bytes or NULL
 *   Wh[n] float [4H, H],  Mh[n] bytes or NULL,  bias[n] float [4H]
 * x float [T,B,D0];  h0,c0 float [L*ndir,B,H] or NULL (zeros)
 * y double [T,B,ndir*H];  hT,cT double [L*ndir,B,H] or NULL
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int lstm_oracle_forward(int L, int ndir, int D0, int H, int T, int B,
                        const float *const *Wx, const unsigned char *const *Mx,
                        const float *const *Wh, const unsigned char *const *Mh,
                        const float *const *bias,
                        const float *x, const float *h0, const float *c0,
                        double *y, double *hT, double *cT, int nthreads)
{
    if (L < 1 || (ndir != 1 && ndir != 2) || D0 < 1 || H < 1 || T < 0 || B < 0) return -1;
    if (!Wx || !Wh || !bias || !y || (!x && T * B > 0)) return -1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    const size_t Dmax = (size_t)(D0 > ndir * H ? D0 : ndir * H);
    const size_t seq = (size_t)T * B;
    double *X = (double *)malloc((seq * Dmax + 1) * sizeof(double));        /* input of the current layer */
    double *Y = (double *)malloc((seq * ndir * H + 1) * sizeof(double));    /* output of the current layer */
    double *h = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *c = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *hn = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *cn = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    if (!X || !Y || !h || !c || !hn || !cn) { free(X); free(Y); free(h); free(c); free(hn); free(cn); return -1; }

    int D = D0;
    for (size_t i = 0; i < seq * D0; ++i) X[i] = (double)x[i];

    for (int l = 0; l < L; ++l) {
        for (int d = 0; d < ndir; ++d) {
            const int n = l * ndir + d;
            const float *wx = Wx[n], *wh = Wh[n], *bb = bias[n];
            const unsigned char *mx = Mx ? Mx[n] : NULL, *mh = Mh ? Mh[n] : NULL;
            for (size_t i = 0; i < (size_t)B * H; ++i) {
                h[i] = h0 ? (double)h0[(size_t)n * B * H + i] : 0.0;
                c[i] = c0 ? (double)c0[(size_t)n * B * H + i] : 0.0;
            }
            for (int s = 0; s < T; ++s) {
                const int t = (d == 0) ? s : T - 1 - s;
#pragma omp parallel for collapse(2) schedule(static)
                for (int b = 0; b < B; ++b) {
                    for (int j = 0; j < H; ++j) {
                        const double *xv = X + ((size_t)t * B + b) * D;
                        const double *hv = h + (size_t)b * H;
                        double a[4];
                        for (int q = 0; q < 4; ++q) {
                            const size_t r = (size_t)q * H + j;
                            a[q] = gate_preact((double)bb[r],
                                               wx + r * D, mx ? mx + r * D : NULL, xv, D,
                                               wh + r * H, mh ? mh + r * H : NULL, hv, H);
                        }
                        const double f = sigmoid(a[0]), i = sigmoid(a[1]), o = sigmoid(a[2]), g = tanh(a[3]);
                        const double cnew = f * c[(size_t)b * H + j] + i * g;
                        const double hnew = o * tanh(cnew);
                        cn[(size_t)b * H + j] = cnew;
                        hn[(size_t)b * H + j] = hnew;
                        Y[((size_t)t * B + b) * (ndir * H) + (size_t)d * H + j] = hnew;
                    }
                }
                double *tmp = h; h = hn; hn = tmp;
                tmp = c; c = cn; cn = tmp;
            }
            if (hT) memcpy(hT + (size_t)n * B * H, h, (size_t)B * H * sizeof(double));
            if (cT) memcpy(cT + (size_t)n * B * H, c, (size_t)B * H * sizeof(double));
        }
        /* the concatenated directions become the next layer's input */
        D = ndir * H;
        memcpy(X, Y, seq * D * sizeof(double));
    }
    memcpy(y, Y, seq * ndir * H * sizeof(double));
    free(X); free(Y); free(h); free(c); free(hn); free(cn);
    return 0;
}

int lstm_oracle_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
