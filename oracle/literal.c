/*
 * Loop-by-loop statement of the DoRA module in double precision.
 *
 * TEST INFRASTRUCTURE ONLY: built with gcc by oracle/build.py and called from
 * the CPU tests to cross-check the numpy oracle on small shapes (every sum is
 * an explicit loop over explicit indices, so a transposed operand or a wrong
 * axis in either version shows up as a disagreement).  Nothing in the product
 * path links or loads this file.
 *
 * Layout everywhere: row-major, W[d_out][d_in], A[r][d_in], B[d_out][r],
 * m[d_out], x[T][d_in], y/dy[T][d_out].
 *
 * Definitions followed: Eq. (1) (adapted weight, row norm over d_in), Eq. (6)
 * (g = m / max(norm, eps)), App. A item 1 (compose equation), Sec. 3.2 and
 * App. C item 2 (compose gradients), norm treated as a constant (App. A item 2).
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>

/* c[j] = || W[j,:] + s * sum_l B[j,l] A[l,:] ||_2 */
void lit_row_norm(const double* W, const double* A, const double* B, double s,
                  long d_out, long d_in, long r, double* c)
{
    for (long j = 0; j < d_out; ++j) {
        double acc = 0.0;
        for (long k = 0; k < d_in; ++k) {
            double ba = 0.0;
            for (long l = 0; l < r; ++l) ba += B[j * r + l] * A[l * d_in + k];
            double d = W[j * d_in + k] + s * ba;
            acc += d * d;
        }
        c[j] = sqrt(acc);
    }
}

/* y[t,j] = sum_k x[t,k] * W'[j,k], with W' = g[j] * (W + sBA)[j,k]  (Eq. 1 applied as a linear layer) */
void lit_forward_via_adapted_weight(const double* x, const double* W, const double* A, const double* B,
                                    const double* m, double s, double eps,
                                    long T, long d_out, long d_in, long r, double* y)
{
    double* c = (double*)malloc(sizeof(double) * (size_t)d_out);
    lit_row_norm(W, A, B, s, d_out, d_in, r, c);
    for (long t = 0; t < T; ++t) {
        for (long j = 0; j < d_out; ++j) {
            double cc = c[j] > eps ? c[j] : eps;
            double g = m[j] / cc;
            double acc = 0.0;
            for (long k = 0; k < d_in; ++k) {
                double ba = 0.0;
                for (long l = 0; l < r; ++l) ba += B[j * r + l] * A[l * d_in + k];
                acc += x[t * d_in + k] * (g * (W[j * d_in + k] + s * ba));
            }
            y[t * d_out + j] = acc;
        }
    }
    free(c);
}

/* delta[t,j] = (g-1)*base + g*s*lora with base = x W^T, lora = (x A^T) B^T; also inner = s*lora + base */
void lit_forward_compose(const double* x, const double* W, const double* A, const double* B,
                         const double* m, double s, double eps,
                         long T, long d_out, long d_in, long r,
                         double* delta, double* inner)
{
    double* c = (double*)malloc(sizeof(double) * (size_t)d_out);
    double* h = (double*)malloc(sizeof(double) * (size_t)r);
    lit_row_norm(W, A, B, s, d_out, d_in, r, c);
    for (long t = 0; t < T; ++t) {
        for (long l = 0; l < r; ++l) {
            double acc = 0.0;
            for (long k = 0; k < d_in; ++k) acc += x[t * d_in + k] * A[l * d_in + k];
            h[l] = acc;
        }
        for (long j = 0; j < d_out; ++j) {
            double base = 0.0, lora = 0.0;
            for (long k = 0; k < d_in; ++k) base += x[t * d_in + k] * W[j * d_in + k];
            for (long l = 0; l < r; ++l) lora += h[l] * B[j * r + l];
            double cc = c[j] > eps ? c[j] : eps;
            double g = m[j] / cc;
            delta[t * d_out + j] = (g - 1.0) * base + g * (s * lora);
            inner[t * d_out + j] = s * lora + base;
        }
    }
    free(h);
    free(c);
}

/*
 * Gradients of L = sum_{t,j} dy[t,j] * y[t,j], y = base + delta, norm c held constant.
 *   y[t,j] = g[j] * ( sum_k x[t,k] W[j,k] + s * sum_l (sum_k x[t,k] A[l,k]) B[j,l] )
 * so, index by index,
 *   dx[t,k] = sum_j dy[t,j] g[j] ( W[j,k] + s sum_l B[j,l] A[l,k] )
 *   dA[l,k] = sum_t sum_j dy[t,j] g[j] s B[j,l] x[t,k]
 *   dB[j,l] = sum_t dy[t,j] g[j] s h[t,l]
 *   dm[j]   = sum_t dy[t,j] inner[t,j] / max(c[j], eps)
 */
void lit_backward(const double* dy, const double* x, const double* W, const double* A, const double* B,
                  const double* m, double s, double eps,
                  long T, long d_out, long d_in, long r,
                  double* dx, double* dA, double* dB, double* dm)
{
    double* c = (double*)malloc(sizeof(double) * (size_t)d_out);
    double* g = (double*)malloc(sizeof(double) * (size_t)d_out);
    double* h = (double*)malloc(sizeof(double) * (size_t)(T * r));
    lit_row_norm(W, A, B, s, d_out, d_in, r, c);
    for (long j = 0; j < d_out; ++j) g[j] = m[j] / (c[j] > eps ? c[j] : eps);
    for (long t = 0; t < T; ++t)
        for (long l = 0; l < r; ++l) {
            double acc = 0.0;
            for (long k = 0; k < d_in; ++k) acc += x[t * d_in + k] * A[l * d_in + k];
            h[t * r + l] = acc;
        }
    for (long t = 0; t < T; ++t)
        for (long k = 0; k < d_in; ++k) {
            double acc = 0.0;
            for (long j = 0; j < d_out; ++j) {
                double ba = 0.0;
                for (long l = 0; l < r; ++l) ba += B[j * r + l] * A[l * d_in + k];
                acc += dy[t * d_out + j] * g[j] * (W[j * d_in + k] + s * ba);
            }
            dx[t * d_in + k] = acc;
        }
    for (long l = 0; l < r; ++l)
        for (long k = 0; k < d_in; ++k) {
            double acc = 0.0;
            for (long t = 0; t < T; ++t)
                for (long j = 0; j < d_out; ++j)
                    acc += dy[t * d_out + j] * g[j] * s * B[j * r + l] * x[t * d_in + k];
            dA[l * d_in + k] = acc;
        }
    for (long j = 0; j < d_out; ++j)
        for (long l = 0; l < r; ++l) {
            double acc = 0.0;
            for (long t = 0; t < T; ++t) acc += dy[t * d_out + j] * g[j] * s * h[t * r + l];
            dB[j * r + l] = acc;
        }
    for (long j = 0; j < d_out; ++j) {
        double acc = 0.0;
        for (long t = 0; t < T; ++t) {
            double base = 0.0, lora = 0.0;
            for (long k = 0; k < d_in; ++k) base += x[t * d_in + k] * W[j * d_in + k];
            for (long l = 0; l < r; ++l) lora += h[t * r + l] * B[j * r + l];
            acc += dy[t * d_out + j] * (s * lora + base);
        }
        dm[j] = acc / (c[j] > eps ? c[j] : eps);
    }
    free(h);
    free(g);
    free(c);
}
