/*
 * CPU oracle for 2-D convolution forward.  TEST INFRASTRUCTURE ONLY: it is called by the tests,
 * the smoke check and the bench's cpu_baseline leg, never by the product path, and it shares no
 * code with the HIP kernels.
 *
 * What it computes is the plain definition of the layer in the paper's section 2.1 (C_I input
 * maps of H_I x W_I, a sliding H_F x W_F kernel, C_O output maps, batch N), which the implicit
 * channel-first method reproduces exactly up to summation order (section 3.1, "General
 * Principle": permuting the lowered matrix's columns together with the filter rows leaves the
 * GEMM result unchanged; section 3.2: the taps may be accumulated in any order):
 *
 *   y[n,p,q,k] = sum_{r<R} sum_{s<S} sum_{c<C}
 *                  x[n, p*stride + r*dil - pad, q*stride + s*dil - pad, c] * w[k,r,s,c]
 *
 * with x read as zero outside 0<=h<H, 0<=w<W, no filter flip (the worked 5x5 example of
 * section 3.1 reads the first window as 1A..3C with tap <1,1> on 1A), symmetric zero padding,
 * and P = floor((H + 2*pad - dil*(R-1) - 1)/stride) + 1 (Q alike).  The paper itself states
 * neither padding nor dilation formulas; these are the usual DNN conventions.
 *
 * Layouts are dense NHWC / KRSC / NPQK.  Inputs arrive as fp32 values that the caller has
 * already rounded to the layer's input type; they are promoted to fp64, multiplied and
 * accumulated in fp64 in the loop order n,p,q,k,r,s,c.  No blocking, no lowering, no GEMM.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int conv_ref_out_dim(int in, int filt, int stride, int pad, int dil)
{
    int span = in + 2 * pad - dil * (filt - 1) - 1;
    if (span < 0) return 0;
    return span / stride + 1;
}

int conv_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* returns 0 on success, -1 on a bad argument */
int conv_ref_f64(const float *x, const float *w, double *y,
                 int N, int H, int W, int C, int K, int R, int S,
                 int stride, int pad, int dil)
{
    if (!x || !w || !y) return -1;
    if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1) return -1;
    if (stride < 1 || dil < 1 || pad < 0) return -1;
    const int P = conv_ref_out_dim(H, R, stride, pad, dil);
    const int Q = conv_ref_out_dim(W, S, stride, pad, dil);
    if (P < 1 || Q < 1) return -1;

#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int p = 0; p < P; ++p) {
            for (int q = 0; q < Q; ++q) {
                for (int k = 0; k < K; ++k) {
                    double acc = 0.0;
                    for (int r = 0; r < R; ++r) {
                        const int h = p * stride + r * dil - pad;
                        if (h < 0 || h >= H) continue;
                        for (int s = 0; s < S; ++s) {
                            const int ww = q * stride + s * dil - pad;
                            if (ww < 0 || ww >= W) continue;
                            const float *xp = x + (((size_t)n * H + h) * W + ww) * C;
                            const float *wp = w + (((size_t)k * R + r) * S + s) * C;
                            for (int c = 0; c < C; ++c)
                                acc += (double)xp[c] * (double)wp[c];
                        }
                    }
                    y[(((size_t)n * P + p) * Q + q) * K + k] = acc;
                }
            }
        }
    }
    return 0;
}
