/*
 * CPU oracle for the stacked H-LSTM forward pass.  TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, double-precision loops that follow the cell equations of the paper
 * (Section 4, the equation block defining f_t, i_t, o_t, g_t, c_t, h_t) with ONE hidden
 * layer H inside each gate (the "*" of H* taken as one; the paper's experiments use one
 * hidden layer per control gate whose width equals the hidden-state width, Sections 5.1
 * and 5.2) and ReLU as the hidden layer's activation (Section 4 names the ReLU as the
 * choice that brings zero outputs):
 *
 *     u_q  = relu( b1_q + W1_q . [x_t , h_{t-1}] )        hidden layer of gate q, width G
 *     a_q  = b2_q + W2_q . u_q                             q in {f, i, o, g}
 *     f,i,o = sigmoid(a_f), sigmoid(a_i), sigmoid(a_o) ;  g = tanh(a_g)
 *     c_t  = f * c_{t-1} + i * g
 *     h_t  = o * tanh(c_t)
 *
 * Every gate has its own hidden layer: u_q feeds gate q only.  W1_q acts on the
 * concatenation [x_t, h_{t-1}] and is passed as its two column blocks W1x and W1h.  The
 * four gates are stacked along the rows in the paper's order f, i, o, g: row q*G + g of
 * W1x / W1h / b1 is hidden unit g of gate q, row q*H + j of W2 / b2 is output j of gate q.
 *
 * Masks (Section 4, "mask-based approach"): an entry whose mask byte is 0 is skipped, so
 * whatever value is stored under it never enters a sum.  A NULL mask keeps every entry.
 *
 * Stacking and directions as in the LSTM oracle (Sections 5.1, 5.2): layer l+1 reads the
 * hidden-state sequence of layer l; direction 1 walks t = T-1 .. 0, its state is stored at
 * the input position it was computed for; directions are concatenated forward first.
 *
 * Nothing is blocked, fused or reordered: per (timestep, sequence) the 4G hidden-layer
 * values are computed one dot product each (bias, then x terms k = 0.., then h terms
 * k = 0..), then one dot product per gate output row (bias, then g = 0..).  OpenMP only
 * distributes independent rows over threads; the result does not depend on the thread count.
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

static double hl_sigmoid(double z) { return 1.0 / (1.0 + exp(-z)); }

/*
 * L layers, ndir in {1,2} directions, D0 = width of x, H = hidden-state width, G = width of
 * each gate's hidden layer.  Per (layer l, direction d), index n = l*ndir + d:
 *   W1x[n] float [4G, D_l] row-major (D_0 = D0, D_l = ndir*H for l > 0), M1x[n] bytes or NULL
 *   W1h[n] float [4G, H],  M1h[n] bytes or NULL,  b1[n] float [4G]
 *   W2[n]  float [4H, G],  M2[n]  bytes or NULL,  b2[n] float [4H]
 * x float [T,B,D0];  h0,c0 float [L*ndir,B,H] or NULL (zeros)
 * y double [T,B,ndir*H];  hT,cT double [L*ndir,B,H] or NULL
 * Returns 0, or -1 on bad arguments / allocation failure.
 */
int hlstm_oracle_forward(int L, int ndir, int D0, int H, int G, int T, int B,
                         const float *const *W1x, const unsigned char *const *M1x,
                         const float *const *W1h, const unsigned char *const *M1h,
                         const float *const *b1,
                         const float *const *W2, const unsigned char *const *M2,
                         const float *const *b2,
                         const float *x, const float *h0, const float *c0,
                         double *y, double *hT, double *cT, int nthreads)
{
    if (L < 1 || (ndir != 1 && ndir != 2) || D0 < 1 || H < 1 || G < 1 || T < 0 || B < 0) return -1;
    if (!W1x || !W1h || !b1 || !W2 || !b2 || !y || (!x && T * B > 0)) return -1;
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#else
    (void)nthreads;
#endif
    const size_t Dmax = (size_t)(D0 > ndir * H ? D0 : ndir * H);
    const size_t seq = (size_t)T * B;
    double *X = (double *)malloc((seq * Dmax + 1) * sizeof(double));
    double *Y = (double *)malloc((seq * ndir * H + 1) * sizeof(double));
    double *h = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *c = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *hn = (double *)malloc(((size_t)B * H + 1) * sizeof(double));
    double *u = (double *)malloc(((size_t)B * 4 * G + 1) * sizeof(double));
    if (!X || !Y || !h || !c || !hn || !u) { free(X); free(Y); free(h); free(c); free(hn); free(u); return -1; }

    int D = D0;
    for (size_t i = 0; i < seq * D0; ++i) X[i] = (double)x[i];

    for (int l = 0; l < L; ++l) {
        for (int d = 0; d < ndir; ++d) {
            const int n = l * ndir + d;
            const float *w1x = W1x[n], *w1h = W1h[n], *bb1 = b1[n], *w2 = W2[n], *bb2 = b2[n];
            const unsigned char *m1x = M1x ? M1x[n] : NULL, *m1h = M1h ? M1h[n] : NULL, *m2 = M2 ? M2[n] : NULL;
            for (size_t i = 0; i < (size_t)B * H; ++i) {
                h[i] = h0 ? (double)h0[(size_t)n * B * H + i] : 0.0;
                c[i] = c0 ? (double)c0[(size_t)n * B * H + i] : 0.0;
            }
            for (int s = 0; s < T; ++s) {
                const int t = (d == 0) ? s : T - 1 - s;
                /* hidden layers of the four gates */
#pragma omp parallel for collapse(2) schedule(static)
                for (int b = 0; b < B; ++b) {
                    for (int r = 0; r < 4 * G; ++r) {
                        const double *xv = X + ((size_t)t * B + b) * D;
                        const double *hv = h + (size_t)b * H;
                        double a = (double)bb1[r];
                        for (int k = 0; k < D; ++k)
                            if (m1x == NULL || m1x[(size_t)r * D + k]) a += (double)w1x[(size_t)r * D + k] * xv[k];
                        for (int k = 0; k < H; ++k)
                            if (m1h == NULL || m1h[(size_t)r * H + k]) a += (double)w1h[(size_t)r * H + k] * hv[k];
                        u[(size_t)b * 4 * G + r] = a > 0.0 ? a : 0.0;
                    }
                }
                /* gate outputs, cell and hidden state */
#pragma omp parallel for collapse(2) schedule(static)
                for (int b = 0; b < B; ++b) {
                    for (int j = 0; j < H; ++j) {
                        double a[4];
                        for (int q = 0; q < 4; ++q) {
                            const size_t r = (size_t)q * H + j;
                            const double *uq = u + (size_t)b * 4 * G + (size_t)q * G;
                            double acc = (double)bb2[r];
                            for (int g = 0; g < G; ++g)
                                if (m2 == NULL || m2[r * G + g]) acc += (double)w2[r * G + g] * uq[g];
                            a[q] = acc;
                        }
                        const double f = hl_sigmoid(a[0]), i = hl_sigmoid(a[1]), o = hl_sigmoid(a[2]), g = tanh(a[3]);
                        const double cnew = f * c[(size_t)b * H + j] + i * g;
                        const double hnew = o * tanh(cnew);
                        c[(size_t)b * H + j] = cnew;      /* c_{t-1}[b][j] is read by this (b, j) only */
                        hn[(size_t)b * H + j] = hnew;     /* h_{t-1} was consumed by the hidden layers above */
                        Y[((size_t)t * B + b) * (ndir * H) + (size_t)d * H + j] = hnew;
                    }
                }
                double *tmp = h; h = hn; hn = tmp;
            }
            if (hT) memcpy(hT + (size_t)n * B * H, h, (size_t)B * H * sizeof(double));
            if (cT) memcpy(cT + (size_t)n * B * H, c, (size_t)B * H * sizeof(double));
        }
        D = ndir * H;
        memcpy(X, Y, seq * D * sizeof(double));
    }
    memcpy(y, Y, seq * ndir * H * sizeof(double));
    free(X); free(Y); free(h); free(c); free(hn); free(u);
    return 0;
}
