/*
 * TEST INFRASTRUCTURE ONLY.  Plain fp64 CPU definitions of the three tensor
 * operators the tuner evaluates.  Nothing in the product library links,
 * includes or calls this file; only tests, the smoke check and the
 * cpu_baseline leg of the benchmark do.
 *
 * Every function is the operator's definition written out as nested loops with
 * one scalar fp64 accumulator per output element, reduction index innermost and
 * ascending.  No blocking, no vectorisation tricks, no loop interchange.  An
 * OpenMP "parallel for" over the outermost output index only spreads whole
 * output elements over cores; it changes no sum.
 *
 *   MatMul       Z[n,m]   = sum_k X[n,k] Y[k,m]                (App. B.1)
 *   BatchMatMul  Z[b,n,m] = sum_k X[b,n,k] Y[b,k,m]            (App. B.2)
 *   Conv2d       Z[i,j,k,l] = sum_p sum_m sum_n I[i,p,k*S+m-P,l*S+n-P] K[j,p,m,n]
 *                with taps that fall outside the image contributing zero, and
 *                H_out = floor((H_in + 2P - H_k)/S) + 1, same for W (App. B.3, Eq. 5;
 *                the printed equation omits S and P although the text defines
 *                them; this is the reading with both put back, no kernel flip).
 *
 * All tensors are dense, contiguous, row-major (NCHW image, OIHW kernel).
 * In this file the matrix product is written C[M,N] = A[M,K] B[K,N].
 */
#include <stddef.h>
#include <stdint.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

void oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/* C[i,j] = sum_k A[i,k] * B[k,j]   (App. B.1) */
void oracle_matmul(const double *A, const double *B, double *C,
                   int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < M; ++i) {
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += A[i * K + k] * B[k * N + j];
            C[i * N + j] = s;
        }
    }
}

/* The same definition for a chosen list of full rows of C:
 * out[r, j] = sum_k A[rows[r], k] * B[k, j].  Used where the full product is
 * too large for the host; every value is still computed by the plain sum. */
void oracle_matmul_rows(const double *A, const double *B, double *out,
                        const int64_t *rows, int64_t n_rows,
                        int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < n_rows; ++r) {
        const int64_t i = rows[r];
        for (int64_t j = 0; j < N; ++j) {
            double s = 0.0;
            for (int64_t k = 0; k < K; ++k)
                s += A[i * K + k] * B[k * N + j];
            out[r * N + j] = s;
        }
    }
}

/* The same definition for a chosen list of single entries (is[e], js[e]). */
void oracle_matmul_entries(const double *A, const double *B, double *out,
                           const int64_t *is, const int64_t *js, int64_t n_entries,
                           int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n_entries; ++e) {
        double s = 0.0;
        for (int64_t k = 0; k < K; ++k)
            s += A[is[e] * K + k] * B[k * N + js[e]];
        out[e] = s;
    }
}

/* C[b,i,j] = sum_k A[b,i,k] * B[b,k,j]; no term crosses batches (App. B.2) */
void oracle_bmm(const double *A, const double *B, double *C,
                int64_t batch, int64_t M, int64_t N, int64_t K)
{
#pragma omp parallel for schedule(static)
    for (int64_t b = 0; b < batch; ++b) {
        const double *Ab = A + b * M * K;
        const double *Bb = B + b * K * N;
        double *Cb = C + b * M * N;
        for (int64_t i = 0; i < M; ++i) {
            for (int64_t j = 0; j < N; ++j) {
                double s = 0.0;
                for (int64_t k = 0; k < K; ++k)
                    s += Ab[i * K + k] * Bb[k * N + j];
                Cb[i * N + j] = s;
            }
        }
    }
}

/* Output extent along one spatial axis (App. B.3, the two floor formulas). */
int64_t oracle_conv_out_extent(int64_t in, int64_t k, int64_t stride, int64_t pad)
{
    const int64_t span = in + 2 * pad - k;
    if (span < 0 || stride <= 0) return 0;
    return span / stride + 1;
}

/* Direct convolution (App. B.3, Eq. 5 with stride and padding restored).
 * img [B, Cin, H, W], ker [Cout, Cin, Hk, Wk], out [B, Cout, Hout, Wout]. */
void oracle_conv2d(const double *img, const double *ker, double *out,
                   int64_t B, int64_t Cin, int64_t H, int64_t W,
                   int64_t Cout, int64_t Hk, int64_t Wk,
                   int64_t stride, int64_t pad)
{
    const int64_t Hout = oracle_conv_out_extent(H, Hk, stride, pad);
    const int64_t Wout = oracle_conv_out_extent(W, Wk, stride, pad);
#pragma omp parallel for collapse(2) schedule(static)
    for (int64_t i = 0; i < B; ++i) {
        for (int64_t j = 0; j < Cout; ++j) {
            for (int64_t k = 0; k < Hout; ++k) {
                for (int64_t l = 0; l < Wout; ++l) {
                    double s = 0.0;
                    for (int64_t p = 0; p < Cin; ++p) {
                        for (int64_t m = 0; m < Hk; ++m) {
                            const int64_t y = k * stride + m - pad;
                            if (y < 0 || y >= H) continue;
                            for (int64_t n = 0; n < Wk; ++n) {
                                const int64_t x = l * stride + n - pad;
                                if (x < 0 || x >= W) continue;
                                s += img[((i * Cin + p) * H + y) * W + x] *
                                     ker[((j * Cin + p) * Hk + m) * Wk + n];
                            }
                        }
                    }
                    out[((i * Cout + j) * Hout + k) * Wout + l] = s;
                }
            }
        }
    }
}
