/*
 * CPU oracle for the Jasper-style 1D time-convolution sub-block.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It exists so that the GPU
 * kernels can be checked against a plain, slow, obviously correct evaluation
 * of the same mathematics.  It shares no code with the GPU path and must only
 * be called from tests, the smoke check and the benchmark's CPU-baseline leg.
 *
 * What it computes.  The paper (Section 3, "Neural Module"; Section 3.3, mixed
 * precision; Section 4.1.1, the Jasper encoder) delegates the forward and the
 * two gradient passes of its convolutional encoder to the deep-learning
 * backend and prints no formula for them, so the oracle is the textbook
 * definition of the operation written out as loops in double precision:
 *
 *   T_out        = floor((T + 2*pad - dilation*(K-1) - 1)/stride) + 1
 *   tau(t,k)     = t*stride - pad + k*dilation          (cross-correlation)
 *   z[b,co,t]    = sum_ci sum_k w[co,ci,k] * x[b,ci,tau(t,k)],  x == 0 outside [0,T)
 *   u            = scale[co]*z + shift[co]               (folded BatchNorm affine)
 *   v            = u + residual[b,co,t]                  (optional)
 *   y            = max(v,0)                              (optional ReLU)
 *   m            = [y > 0]  (1 when no ReLU);  dres = dy*m;  dz = dy*m*scale[co]
 *   dx[b,ci,tau] = sum over (co,t,k) with tau(t,k)==tau of w[co,ci,k]*dz[b,co,t]
 *   dw[co,ci,k]  = sum_b sum_t dz[b,co,t] * x[b,ci,tau(t,k)]
 *
 * Layouts: activations [B][C][T] (T innermost), weights [Cout][Cin][K],
 * all dense, all `double`.  Nothing is rounded anywhere.
 *
 * Parity pins (tests/test_oracle_pins.py): K=1 against a library matmul, impulse
 * input recovering every weight, all-ones closed-form edge counts, brute-force
 * padded/dilated index enumeration, stride = subsampling, dilation = zero-stuffed
 * kernel, shift equivariance, adjoint identities, central finite differences of
 * the whole block, epilogue closed forms, and torch's CPU float64 conv1d with
 * autograd as a library special case.  The sampled (`*_at`) evaluators are pinned
 * to the full-tensor ones.
 */
#include <stddef.h>
#include <stdint.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the parallel loops below will use (reported next to CPU timings). */
int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

int oracle_conv1d_out_len(int T, int K, int stride, int dilation, int pad)
{
    if (T <= 0 || K <= 0 || stride <= 0 || dilation <= 0 || pad < 0) return -1;
    long span = (long)T + 2L * pad - (long)dilation * (K - 1) - 1;
    if (span < 0) return -1;
    return (int)(span / stride) + 1;
}

/* One pre-activation value z[b,co,t] straight from the definition. */
static double conv_at(int Cin, int T, int K, int stride, int dilation, int pad,
                      const double *xb /* [Cin][T] of batch item b */,
                      const double *wco /* [Cin][K] of output channel co */, int t)
{
    double z = 0.0;
    for (int ci = 0; ci < Cin; ++ci) {
        for (int k = 0; k < K; ++k) {
            long tau = (long)t * stride - pad + (long)k * dilation;
            if (tau >= 0 && tau < T) z += wco[(size_t)ci * K + k] * xb[(size_t)ci * T + tau];
        }
    }
    return z;
}

static double epilogue(double z, const double *scale, const double *shift,
                       const double *residual, int relu, int co, size_t out_index)
{
    double u = (scale ? scale[co] * z : z) + (shift ? shift[co] : 0.0);
    double v = residual ? u + residual[out_index] : u;
    if (relu) return v > 0.0 ? v : 0.0;
    return v;
}

/* Block forward.  y (and, if non-NULL, the pre-affine z) are [B][Cout][T_out]. */
void oracle_conv1d_block_fwd(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                             int pad, const double *x, const double *w, const double *scale,
                             const double *shift, const double *residual, int relu, double *y,
                             double *z_out)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int co = 0; co < Cout; ++co) {
            const double *xb = x + (size_t)b * Cin * T;
            const double *wco = w + (size_t)co * Cin * K;
            for (int t = 0; t < To; ++t) {
                size_t o = ((size_t)b * Cout + co) * To + t;
                double z = conv_at(Cin, T, K, stride, dilation, pad, xb, wco, t);
                if (z_out) z_out[o] = z;
                y[o] = epilogue(z, scale, shift, residual, relu, co, o);
            }
        }
    }
}

/* Block forward at n chosen flat output indices (into [B][Cout][T_out]). */
void oracle_conv1d_block_fwd_at(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                                int pad, const double *x, const double *w, const double *scale,
                                const double *shift, const double *residual, int relu, long n,
                                const int64_t *index, double *y)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
    (void)B;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        size_t o = (size_t)index[i];
        int t = (int)(o % To);
        int co = (int)((o / To) % Cout);
        int b = (int)(o / ((size_t)To * Cout));
        double z = conv_at(Cin, T, K, stride, dilation, pad, x + (size_t)b * Cin * T,
                           w + (size_t)co * Cin * K, t);
        y[i] = epilogue(z, scale, shift, residual, relu, co, o);
    }
}

/* Backward of the epilogue: upstream gradient of y -> gradient of z and of the residual. */
void oracle_conv1d_epilogue_bwd(int B, int Cout, int To, const double *dy, const double *y_saved,
                                const double *scale, int relu, double *dz, double *dres)
{
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int co = 0; co < Cout; ++co) {
            for (int t = 0; t < To; ++t) {
                size_t o = ((size_t)b * Cout + co) * To + t;
                double m = 1.0;
                if (relu) m = (y_saved[o] > 0.0) ? 1.0 : 0.0;
                double g = dy[o] * m;
                if (dres) dres[o] = g;
                if (dz) dz[o] = scale ? g * scale[co] : g;
            }
        }
    }
}

/* Input gradient, scatter form: every (co,t,k) term is pushed to the sample it read. */
void oracle_conv1d_bwd_data(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                            int pad, const double *dz, const double *w, double *dx)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b) {
        for (int ci = 0; ci < Cin; ++ci) {
            double *dxr = dx + ((size_t)b * Cin + ci) * T;
            for (int tau = 0; tau < T; ++tau) dxr[tau] = 0.0;
            for (int co = 0; co < Cout; ++co) {
                const double *dzr = dz + ((size_t)b * Cout + co) * To;
                const double *wr = w + ((size_t)co * Cin + ci) * K;
                for (int t = 0; t < To; ++t) {
                    for (int k = 0; k < K; ++k) {
                        long tau = (long)t * stride - pad + (long)k * dilation;
                        if (tau >= 0 && tau < T) dxr[tau] += wr[k] * dzr[t];
                    }
                }
            }
        }
    }
}

/* Input gradient at n chosen flat indices of [B][Cin][T], gather form:
 * the taps that reach sample tau are those with (tau + pad - k*dilation) divisible by
 * the stride and the quotient a valid output position. */
void oracle_conv1d_bwd_data_at(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                               int pad, const double *dz, const double *w, long n,
                               const int64_t *index, double *dx)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
    (void)B;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        size_t o = (size_t)index[i];
        int tau = (int)(o % T);
        int ci = (int)((o / T) % Cin);
        int b = (int)(o / ((size_t)T * Cin));
        double s = 0.0;
        for (int co = 0; co < Cout; ++co) {
            const double *dzr = dz + ((size_t)b * Cout + co) * To;
            const double *wr = w + ((size_t)co * Cin + ci) * K;
            for (int k = 0; k < K; ++k) {
                long num = (long)tau + pad - (long)k * dilation;
                if (num < 0 || num % stride != 0) continue;
                long t = num / stride;
                if (t < To) s += wr[k] * dzr[t];
            }
        }
        dx[i] = s;
    }
}

/* Weight gradient: dw[co][ci][k], summed over batch and time. */
void oracle_conv1d_bwd_weight(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                              int pad, const double *x, const double *dz, double *dw)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
#pragma omp parallel for collapse(2) schedule(static)
    for (int co = 0; co < Cout; ++co) {
        for (int ci = 0; ci < Cin; ++ci) {
            for (int k = 0; k < K; ++k) {
                double s = 0.0;
                for (int b = 0; b < B; ++b) {
                    const double *dzr = dz + ((size_t)b * Cout + co) * To;
                    const double *xr = x + ((size_t)b * Cin + ci) * T;
                    for (int t = 0; t < To; ++t) {
                        long tau = (long)t * stride - pad + (long)k * dilation;
                        if (tau >= 0 && tau < T) s += dzr[t] * xr[tau];
                    }
                }
                dw[((size_t)co * Cin + ci) * K + k] = s;
            }
        }
    }
}

/* Weight gradient at n chosen flat indices of [Cout][Cin][K]. */
void oracle_conv1d_bwd_weight_at(int B, int Cin, int Cout, int T, int K, int stride, int dilation,
                                 int pad, const double *x, const double *dz, long n,
                                 const int64_t *index, double *dw)
{
    const int To = oracle_conv1d_out_len(T, K, stride, dilation, pad);
    if (To <= 0) return;
#pragma omp parallel for schedule(static)
    for (long i = 0; i < n; ++i) {
        size_t o = (size_t)index[i];
        int k = (int)(o % K);
        int ci = (int)((o / K) % Cin);
        int co = (int)(o / ((size_t)K * Cin));
        double s = 0.0;
        for (int b = 0; b < B; ++b) {
            const double *dzr = dz + ((size_t)b * Cout + co) * To;
            const double *xr = x + ((size_t)b * Cin + ci) * T;
            for (int t = 0; t < To; ++t) {
                long tau = (long)t * stride - pad + (long)k * dilation;
                if (tau >= 0 && tau < T) s += dzr[t] * xr[tau];
            }
        }
        dw[i] = s;
    }
}
