/*
 * fp64 CPU oracle for the pre-scan step of the LBMamba block: depthwise
 * convolution along the sequence followed by SiLU (paper = arXiv 2506.15976,
 * Algorithm 1, the line that forms x' from x before B, C and Delta are projected).
 *
 * TEST INFRASTRUCTURE ONLY, like lbscan_oracle.c: it shares nothing with the
 * HIP path and only the tests load it.
 *
 * The paper names the operation (Conv1d, then SiLU) and nothing else.  Readings:
 *   - the convolution is depthwise (one filter per channel; x and x' have the
 *     same shape (B, L, E) in Algorithm 1) with a bias per channel;
 *   - it is causal, as in the Mamba block that Algorithm 1 extends: output t
 *     sees inputs t-K+1 .. t, inputs before the start count as zero;
 *         pre[b,d,t] = bias[d] + sum_{k=0}^{K-1} w[d,k] x[b,d,t-(K-1)+k]
 *         y = pre * sigmoid(pre)      (or y = pre when the activation is off)
 *   - K is a free argument (Mamba's default is 4);
 *   - reverse = 1 is the same operator on the time-reversed sequence (output t
 *     sees inputs t .. t+K-1), for blocks that scan right to left.
 *
 * Layout: x, y, dy, dx (batch, dim, seqlen); w, dw (dim, width); bias, dbias (dim);
 * all host fp64, dense, last index contiguous.
 *
 * Parity status: pinned by tests/test_oracle_conv_pins.py (library FIR filter,
 * hand-written sums, flip identity, finite differences).
 */
#include <math.h>
#include <string.h>

static double sigmoid64(double v) { return 1.0 / (1.0 + exp(-v)); }

/* input index that tap k of output t reads; may fall outside [0, L) */
static long tap_index(long t, int k, int K, int reverse)
{
    return reverse ? t + (K - 1) - k : t - (K - 1) + k;
}

int lbconv_ref_fwd(int batch, int dim, int seqlen, int width, int activation, int reverse,
                   const double *x, const double *w, const double *bias, double *y)
{
    if (batch < 0 || dim < 0 || seqlen < 0 || width < 1) return -1;
    if ((long)batch * dim * seqlen == 0) return 0;
    if (!x || !w || !y) return -1;
    for (long row = 0; row < (long)batch * dim; ++row) {
        const int d = (int)(row % dim);
        const double *xr = x + row * seqlen;
        double *yr = y + row * seqlen;
        for (long t = 0; t < seqlen; ++t) {
            double pre = bias ? bias[d] : 0.0;
            for (int k = 0; k < width; ++k) {
                const long s = tap_index(t, k, width, reverse);
                if (s >= 0 && s < seqlen) pre += w[(long)d * width + k] * xr[s];
            }
            yr[t] = activation ? pre * sigmoid64(pre) : pre;
        }
    }
    return 0;
}

/*
 * Gradient of lbconv_ref_fwd.  With dpre_t = dy_t * d(act)/d(pre_t), where
 * d SiLU(p)/dp = sigma(p) (1 + p (1 - sigma(p))):
 *   dx_s    = sum over the outputs t whose tap k reads s of w[k] dpre_t
 *   dw[d,k] = sum_{b,t} dpre_t x[tap(t,k)]       dbias[d] = sum_{b,t} dpre_t
 * Every output is overwritten; dbias may be NULL iff bias is.
 */
int lbconv_ref_bwd(int batch, int dim, int seqlen, int width, int activation, int reverse,
                   const double *x, const double *w, const double *bias, const double *dy,
                   double *dx, double *dw, double *dbias)
{
    if (batch < 0 || dim < 0 || seqlen < 0 || width < 1) return -1;
    if (!dw || (bias && !dbias)) return -1;
    memset(dw, 0, sizeof(double) * (size_t)dim * width);
    if (dbias) memset(dbias, 0, sizeof(double) * (size_t)dim);
    if ((long)batch * dim * seqlen == 0) return 0;
    if (!x || !w || !dy || !dx) return -1;
    memset(dx, 0, sizeof(double) * (size_t)batch * dim * seqlen);
    for (long row = 0; row < (long)batch * dim; ++row) {
        const int d = (int)(row % dim);
        const double *xr = x + row * seqlen, *gr = dy + row * seqlen;
        double *dxr = dx + row * seqlen;
        for (long t = 0; t < seqlen; ++t) {
            double pre = bias ? bias[d] : 0.0;
            for (int k = 0; k < width; ++k) {
                const long s = tap_index(t, k, width, reverse);
                if (s >= 0 && s < seqlen) pre += w[(long)d * width + k] * xr[s];
            }
            double dpre = gr[t];
            if (activation) {
                const double sg = sigmoid64(pre);
                dpre *= sg * (1.0 + pre * (1.0 - sg));
            }
            for (int k = 0; k < width; ++k) {
                const long s = tap_index(t, k, width, reverse);
                if (s >= 0 && s < seqlen) {
                    dxr[s] += w[(long)d * width + k] * dpre;
                    dw[(long)d * width + k] += dpre * xr[s];
                }
            }
            if (dbias) dbias[d] += dpre;
        }
    }
    return 0;
}
