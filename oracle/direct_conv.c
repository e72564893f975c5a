/* CPU oracle, C form: float64 direct convolution (zero-padded
 * cross-correlation), the same definition as oracle/direct.py, written as
 * plain loops so it can be timed on the host cores next to the GPU run.
 * TEST INFRASTRUCTURE ONLY: used by the tests (cross-checked against the
 * numpy oracle) and by the benchmark's CPU-baseline leg.
 *
 *   y[n,k,p,q] = b[k] + sum_{c,r,s} x[n, g*Cg + c, p*stride-pad+r, q*stride-pad+s] * w[k,c,r,s]
 *
 * Inputs are float32 (as stored in a model file), widened to double on use;
 * the accumulator and the output are double.  Threads split the (n,k) planes.
 */
#include <stddef.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_conv2d_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_conv2d_f64(const float *x, const float *w, const double *bias, double *y,
                       int N, int C, int H, int W, int K, int R, int S,
                       int stride, int pad, int groups) {
    const int Cg = C / groups, Kg = K / groups;
    const int P = (H + 2 * pad - R) / stride + 1;
    const int Q = (W + 2 * pad - S) / stride + 1;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n) {
        for (int k = 0; k < K; ++k) {
            const int g = k / Kg;
            double *yp = y + ((size_t)n * K + k) * P * Q;
            for (int i = 0; i < P * Q; ++i) yp[i] = bias ? bias[k] : 0.0;
            for (int c = 0; c < Cg; ++c) {
                const float *xp = x + ((size_t)n * C + (size_t)g * Cg + c) * H * W;
                const float *wp = w + ((size_t)k * Cg + c) * R * S;
                for (int r = 0; r < R; ++r) {
                    for (int s = 0; s < S; ++s) {
                        const double wv = (double)wp[r * S + s];
                        for (int p = 0; p < P; ++p) {
                            const int ih = p * stride - pad + r;
                            if (ih < 0 || ih >= H) continue;
                            for (int q = 0; q < Q; ++q) {
                                const int iw = q * stride - pad + s;
                                if (iw < 0 || iw >= W) continue;
                                yp[p * Q + q] += (double)xp[(size_t)ih * W + iw] * wv;
                            }
                        }
                    }
                }
            }
        }
    }
}
