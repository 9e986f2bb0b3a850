/*
 * oracle_tensor.h -- entry points of the fp64 CPU oracle (oracle/liboracle_tensor.so).
 *
 * TEST INFRASTRUCTURE.  The oracle is a library of its own, built from oracle/tensor_oracle.c with gcc; the product
 * library (opevo.h) neither includes this header nor links that library.  Only the tests, the smoke check and the
 * cpu_baseline / reference leg of the benchmark call it.
 *
 * Every function is the operator's definition written as nested loops with one fp64 accumulator per output element,
 * reduction index innermost and ascending; OpenMP spreads whole output elements over cores and changes no sum.
 * All pointers are HOST pointers to dense, contiguous, row-major fp64 arrays owned by the caller; inputs are read
 * only, outputs are written completely; nothing is allocated or retained.  Sizes are element counts per axis and
 * must be >= 0 (a zero extent writes nothing).  The functions have no error path: shapes are the caller's contract.
 */
#ifndef ORACLE_TENSOR_H
#define ORACLE_TENSOR_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Threads the OpenMP loops will use / set that number (n <= 0 is ignored). */
int oracle_num_threads(void);
void oracle_set_threads(int n);

/* MatMul (App. B.1): C[i,j] = sum_k A[i,k] * B[k,j];  A [M,K], B [K,N], C [M,N]. */
void oracle_matmul(const double *A, const double *B, double *C, int64_t M, int64_t N, int64_t K);

/* The same sums for chosen full rows, out[r,j] = C[rows[r], j] (out [n_rows, N]), and for chosen single entries,
 * out[e] = C[is[e], js[e]]: for products too large to form on the host.  Indices must lie inside C. */
void oracle_matmul_rows(const double *A, const double *B, double *out, const int64_t *rows, int64_t n_rows,
                        int64_t N, int64_t K);
void oracle_matmul_entries(const double *A, const double *B, double *out, const int64_t *is, const int64_t *js,
                           int64_t n_entries, int64_t N, int64_t K);

/* BatchMatMul (App. B.2): C[b,i,j] = sum_k A[b,i,k] * B[b,k,j];  A [batch,M,K], B [batch,K,N], C [batch,M,N]. */
void oracle_bmm(const double *A, const double *B, double *C, int64_t batch, int64_t M, int64_t N, int64_t K);

/* Output extent of a convolution along one spatial axis (App. B.3): floor((in + 2 pad - k) / stride) + 1, 0 if the
 * kernel does not fit. */
int64_t oracle_conv_out_extent(int64_t in, int64_t k, int64_t stride, int64_t pad);

/* Conv2d (App. B.3, Eq. 5 with stride and padding put back, cross-correlation, taps outside the image contribute 0):
 * out[i,j,k,l] = sum_p sum_m sum_n img[i,p,k*stride+m-pad,l*stride+n-pad] * ker[j,p,m,n];
 * img [B,Cin,H,W], ker [Cout,Cin,Hk,Wk], out [B,Cout,Hout,Wout] with the extents of oracle_conv_out_extent. */
void oracle_conv2d(const double *img, const double *ker, double *out, int64_t B, int64_t Cin, int64_t H, int64_t W,
                   int64_t Cout, int64_t Hk, int64_t Wk, int64_t stride, int64_t pad);

#ifdef __cplusplus
}
#endif
#endif
