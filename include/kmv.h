/*
 * kmv — dense matrix-vector products for AMD Instinct MI355X (gfx950).
 *
 * C ABI of the library.  Every product is the BLAS level-2 operation of the
 * paper's Section 5.2 ("Routines and APIs"):
 *
 *        y  <-  alpha * op(A) * x  +  beta * y
 *
 * with A general (GEMV; the non-transposed and transposed kernels of
 * Section 6.1) or symmetric / Hermitian with ONE stored triangle (SYMV for
 * s,d and HEMV for c,z; Sections 6.1, 6.5 and 7: only the upper or only the
 * lower triangle is read).  The argument lists are the standard column-major
 * BLAS ones, which the paper's routines follow (Section 5.2), followed by a
 * caller-owned workspace and a stream (the paper's "_async" variants,
 * Section 5.2, take the stream as an extra last argument as well).
 *
 * Memory and ownership
 *   A, x, y, workspace : DEVICE pointers, owned by the caller, valid until
 *                        the work enqueued on `stream` has completed.
 *   alpha, beta        : HOST pointers, read before the call returns.
 *   stream             : a hipStream_t passed as void* (NULL = null stream).
 *   Calls only enqueue kernels: no allocation, no memset, no host
 *   synchronisation, no hidden global state, so a sequence of calls can be
 *   recorded into a HIP graph and replayed.  A and x must not overlap y or
 *   the workspace.
 *   Concurrent calls must use distinct workspaces.
 *
 * Layout (Section 5.3, single-GPU routines)
 *   A is column major: element (i,j) is A[i + j*lda], lda >= max(1, rows).
 *   A may point anywhere inside a larger matrix (a sub-block at arbitrary
 *   row / column offsets, Section 6.6): the kernels derive the 128-byte
 *   alignment of the columns from the pointer value and lda, start their
 *   row tiles on the aligned boundary and mask the leading rows, so the
 *   "_offset" entry points further down are a convenience, not a faster
 *   path.  No byte outside the m x n
 *   block (GEMV) or outside the stored triangle (SYMV/HEMV) is ever read.
 *   Complex numbers are interleaved (re, im) pairs.
 *   Vectors: element k of a length-len vector with increment inc is
 *   v[k*inc] for inc > 0 and v[(k-(len-1))*inc] for inc < 0 (reference BLAS).
 *
 * Semantics of special values (reference-BLAS conventions)
 *   m == 0 or n == 0, or (alpha == 0 and beta == 1): nothing is enqueued.
 *   alpha == 0 : A and x are not read,  y <- beta*y.
 *   beta  == 0 : y is not read (NaN / Inf in y do not propagate).
 *   HEMV ignores the imaginary part of the diagonal of A.
 *
 * Return value
 *   0                    success (work enqueued)
 *   -k                   the k-th BLAS argument is illegal, numbered as the
 *                        reference BLAS numbers them
 *                          GEMV     : trans 1, m 2, n 3, lda 6, incx 8, incy 11
 *                          SYMV/HEMV: uplo 1, n 2, lda 5, incx 7, incy 10
 *   KMV_ERR_WORKSPACE    the call needs its workspace and it is NULL, not
 *                        256-byte aligned or smaller than the size the
 *                        matching *_workspace_bytes call reports.  A call
 *                        needs it when x is strided (incx != 1) or when its
 *                        kernels exchange partial sums: GEMV with split
 *                        columns or rows, SYMV/HEMV beyond the size of the
 *                        one-launch kernel (kmv_symv_kernel_variant == 2);
 *                        otherwise workspace may be NULL
 *   KMV_ERR_NULL         A, x, y, alpha or beta is NULL
 *   KMV_ERR_HIP + e      the HIP runtime reported error e at launch
 *   On any error nothing is enqueued and y is untouched.
 *
 * Families declared below, in this order: GEMV; SYMV / HEMV; complex
 * symmetric SYMV; the "_offset" forms that name the parent matrix; the
 * "_devscalars" forms (alpha, beta in device memory) - both also for the
 * complex symmetric product (kmv_csymv_*, kmv_zsymv_*); panel steps of the
 * tridiagonal and the bidiagonal reduction built on these calls; strided
 * batches; pointer-array batches; workspace sizes; the work partition; the bandwidth probe; tuning.
 *
 * Determinism: for fixed arguments (including the alignment of A modulo 128
 * bytes) and fixed tuning values the result is bitwise reproducible; partial
 * sums of different workgroups meet in a workspace and are added in a fixed
 * order (no floating-point atomics).
 */
#ifndef KMV_H
#define KMV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct { float re, im; } kmv_complex64;
typedef struct { double re, im; } kmv_complex128;

#define KMV_OK 0
#define KMV_ERR_WORKSPACE 1001
#define KMV_ERR_NULL 1002
#define KMV_ERR_HIP 2000

/* ---- GEMV: y <- alpha*op(A)*x + beta*y,  A is m x n (Section 6.1, kernels 1
 * and 2; Algorithms "Non-transposed GEMV" and "Transposed GEMV").
 * trans: 'N' op(A)=A (x has n, y has m elements); 'T' op(A)=A^T; 'C'
 * op(A)=A^H (x has m, y has n elements); lower case accepted; for the real
 * precisions 'C' is the same as 'T'. */
int kmv_sgemv(char trans, int64_t m, int64_t n, const float* alpha, const float* A, int64_t lda,
              const float* x, int64_t incx, const float* beta, float* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_dgemv(char trans, int64_t m, int64_t n, const double* alpha, const double* A, int64_t lda,
              const double* x, int64_t incx, const double* beta, double* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_cgemv(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_zgemv(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);

/* ---- SYMV (real symmetric) and HEMV (complex Hermitian): A is n x n and only
 * its `uplo` triangle ('L' or 'U', lower case accepted) is read (Section 6.1
 * kernel 3, Section 6.5 for the diagonal blocks, Algorithm "Upper/Lower
 * SYMV/HEMV").  Each stored off-diagonal element is read once and used for
 * both a_ij*x_j and op(a_ij)*x_i (matrices of at most about 2000 rows go to a
 * one-launch kernel that reads the cache-resident triangle twice instead).
 * n beyond what the kernels' tables index (about 139000 rows of 16-byte
 * elements, more for the others: more than fits the device) is refused with
 * KMV_ERR_HIP + hipErrorInvalidValue. */
int kmv_ssymv(char uplo, int64_t n, const float* alpha, const float* A, int64_t lda,
              const float* x, int64_t incx, const float* beta, float* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_dsymv(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda,
              const double* x, int64_t incx, const double* beta, double* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_chemv(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_zhemv(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);

/* ---- SYMV for complex symmetric matrices (A = A^T, no conjugation, the
 * diagonal taken as stored).  The routine table of Section 5.2 lists SYMV for
 * s,d and HEMV for c,z only; these two complete the set of the standard BLAS
 * extension and run the HEMV kernels with the conjugation switched off.
 * Arguments, workspace (kmv_symv_workspace_bytes with prec 'c' / 'z') and
 * errors as for kmv_chemv / kmv_zhemv. */
int kmv_csymv(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);
int kmv_zsymv(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* workspace, size_t workspace_bytes, void* stream);

/* ---- Sub-block calls that name the parent matrix (Section 6.6, "Multiplication
 * by a Submatrix"; the GEMV-OFFSET / SYMV-OFFSET / HEMV-OFFSET rows
 * of the routine table in Section 5.2).  A, m, n (and x, y) describe the
 * PARENT; the product is taken with the block of its rows offset_r..m-1 and
 * columns offset_c..n-1 (SYMV/HEMV: the trailing diagonal block from `offset`
 * on).  x and y are the parent's vectors: of a vector with increment inc the
 * logical elements from the offset on take part, the others are neither read
 * nor written ('N': x from offset_c, y from offset_r; 'T','C': x from
 * offset_r, y from offset_c).  The paper does not print the argument list;
 * this one is the standard list followed by the offsets.
 * The call equals the standard call on the pointer A + offset_r + offset_c*lda
 * with the reduced sizes: the standard calls here already derive the tile grid
 * from the pointer's misalignment, and, unlike the paper's kernels, neither
 * form loads parent elements outside the block.  Workspace: the size for the
 * block's dimensions (m - offset_r, n - offset_c; n - offset).  Errors as for
 * the standard calls; an offset below 0 or beyond the dimension returns the
 * negated number of that argument (-12 / -13 for GEMV, -11 for SYMV/HEMV). */
int kmv_sgemv_offset(char trans, int64_t m, int64_t n, const float* alpha, const float* A, int64_t lda,
                     const float* x, int64_t incx, const float* beta, float* y, int64_t incy,
                     int64_t offset_r, int64_t offset_c, void* workspace, size_t workspace_bytes, void* stream);
int kmv_dgemv_offset(char trans, int64_t m, int64_t n, const double* alpha, const double* A, int64_t lda,
                     const double* x, int64_t incx, const double* beta, double* y, int64_t incy,
                     int64_t offset_r, int64_t offset_c, void* workspace, size_t workspace_bytes, void* stream);
int kmv_cgemv_offset(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A,
                     int64_t lda, const kmv_complex64* x, int64_t incx, const kmv_complex64* beta,
                     kmv_complex64* y, int64_t incy, int64_t offset_r, int64_t offset_c, void* workspace,
                     size_t workspace_bytes, void* stream);
int kmv_zgemv_offset(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A,
                     int64_t lda, const kmv_complex128* x, int64_t incx, const kmv_complex128* beta,
                     kmv_complex128* y, int64_t incy, int64_t offset_r, int64_t offset_c, void* workspace,
                     size_t workspace_bytes, void* stream);
int kmv_ssymv_offset(char uplo, int64_t n, const float* alpha, const float* A, int64_t lda, const float* x,
                     int64_t incx, const float* beta, float* y, int64_t incy, int64_t offset, void* workspace,
                     size_t workspace_bytes, void* stream);
int kmv_dsymv_offset(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x,
                     int64_t incx, const double* beta, double* y, int64_t incy, int64_t offset, void* workspace,
                     size_t workspace_bytes, void* stream);
int kmv_chemv_offset(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
                     const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y,
                     int64_t incy, int64_t offset, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zhemv_offset(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
                     const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y,
                     int64_t incy, int64_t offset, void* workspace, size_t workspace_bytes, void* stream);
int kmv_csymv_offset(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
                     const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y,
                     int64_t incy, int64_t offset, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zsymv_offset(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
                     const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y,
                     int64_t incy, int64_t offset, void* workspace, size_t workspace_bytes, void* stream);

/* ---- The same products with alpha and beta in DEVICE memory (one element
 * each, read by the kernels when they run, so a scalar that an earlier kernel
 * on the stream computes needs no host synchronisation; the paper's routines
 * take host scalars only, Section 5.2).  Everything else as for the standard
 * calls, except that nothing can depend on the scalars' values at enqueue
 * time: alpha == 0 still yields beta*y exactly (A and x are read, their
 * values - NaN, Inf - do not enter), beta == 0 still means y is not read,
 * alpha == 0 with beta == 1 rewrites y with its own values.  The scalars must
 * not be written while the call is in flight. */
int kmv_sgemv_devscalars(char trans, int64_t m, int64_t n, const float* alpha, const float* A, int64_t lda,
                         const float* x, int64_t incx, const float* beta, float* y, int64_t incy,
                         void* workspace, size_t workspace_bytes, void* stream);
int kmv_dgemv_devscalars(char trans, int64_t m, int64_t n, const double* alpha, const double* A, int64_t lda,
                         const double* x, int64_t incx, const double* beta, double* y, int64_t incy,
                         void* workspace, size_t workspace_bytes, void* stream);
int kmv_cgemv_devscalars(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A,
                         int64_t lda, const kmv_complex64* x, int64_t incx, const kmv_complex64* beta,
                         kmv_complex64* y, int64_t incy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zgemv_devscalars(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A,
                         int64_t lda, const kmv_complex128* x, int64_t incx, const kmv_complex128* beta,
                         kmv_complex128* y, int64_t incy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_ssymv_devscalars(char uplo, int64_t n, const float* alpha, const float* A, int64_t lda, const float* x,
                         int64_t incx, const float* beta, float* y, int64_t incy, void* workspace,
                         size_t workspace_bytes, void* stream);
int kmv_dsymv_devscalars(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x,
                         int64_t incx, const double* beta, double* y, int64_t incy, void* workspace,
                         size_t workspace_bytes, void* stream);
int kmv_chemv_devscalars(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
                         const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y,
                         int64_t incy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zhemv_devscalars(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
                         const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y,
                         int64_t incy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_csymv_devscalars(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
                         const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y,
                         int64_t incy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zsymv_devscalars(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
                         const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y,
                         int64_t incy, void* workspace, size_t workspace_bytes, void* stream);

/* ---- Panel step of the symmetric tridiagonal reduction (Section 10: the
 * two-sided reductions are where these products are spent; SYMV on the
 * trailing block and GEMV on the reflector panels, all on sub-blocks at
 * arbitrary offsets, Section 6.6).  A second workload built on the entry
 * points above, for s and d (and c, z: see the Hermitian form below).  The
 * description is for lower storage (uplo 'L'); 'U' follows it.
 * For the first nb columns of the symmetric n x n matrix A (device, lower
 * triangle referenced, never the strict upper one): column i is brought up to
 * date with the reflectors before it, a Householder reflector H_i = I - tau_i
 * v_i v_i^T annihilates its entries below the subdiagonal, and w_i is formed so
 * that A - V W^T - W V^T on the trailing block is the transformed block.
 * On exit (all device memory): A[i][i] = d_i; A[i+1][i] = 1 and A[i+2..][i] =
 * the rest of v_i; e[i] the subdiagonal entry, tau[i]; W (n x nb, leading
 * dimension ldw >= n) holds w_i in W[i+1..n-1][i] (rows 0..i of column i are
 * scratch).  Columns nb..n-1 of A are not modified.  A column without entries
 * below the subdiagonal gets tau = 0 (e = the subdiagonal entry as it stands;
 * both 0 for the last column of the matrix).  Norms are formed without
 * rescaling against underflow or overflow.
 * uplo 'U' (upper triangle referenced, never the strict lower one) is the
 * mirror image: the LAST nb columns are reduced, from column n-1 down to n-nb;
 * column i = n-nb+k uses slot k of e, tau and W; its reflector annihilates
 * A[0..i-2][i], so on exit A[i][i] = d_i, A[i-1][i] = 1, A[0..i-2][i] = the
 * rest of v_i, e[k] the superdiagonal entry, W[0..i-1][k] = w_i (rows i.. of
 * that column are scratch); columns 0..n-nb-1 of A are not modified and
 * A - V W^T - W V^T on the LEADING (n-nb) x (n-nb) block is the transformed
 * block; column 0 of the matrix has no reflector (e = tau = 0).
 * Only enqueues kernels on `stream` (five per column: the symmetric product's
 * two and three of the panel's own; tau, the norms and the inner products stay
 * on the device), so a panel can be captured in a graph.
 * Workspace: kmv_sytrd_panel_workspace_bytes(prec, n, nb), 256-byte aligned.
 * Errors: negated argument number (uplo 1, n 2, nb 3 (0 <= nb <= min(n, 1024)), lda 5,
 * ldw 9), KMV_ERR_NULL, KMV_ERR_WORKSPACE, or the code of a failing launch,
 * in which case the columns before it are done and A is left in between. */
int kmv_ssytrd_panel(char uplo, int64_t n, int64_t nb, float* A, int64_t lda, float* e, float* tau, float* W,
                     int64_t ldw, void* workspace, size_t workspace_bytes, void* stream);
int kmv_dsytrd_panel(char uplo, int64_t n, int64_t nb, double* A, int64_t lda, double* e, double* tau, double* W,
                     int64_t ldw, void* workspace, size_t workspace_bytes, void* stream);
/* The same step for a complex Hermitian matrix (HETRD): H_i = I - tau_i v_i v_i^H with a real e_i and a
 * complex tau_i, A - V W^H - W V^H on the trailing block; the diagonal entries d_i come out real (their
 * imaginary parts, never used, are set to zero for the panel's columns).  e is a REAL array. */
int kmv_chetrd_panel(char uplo, int64_t n, int64_t nb, kmv_complex64* A, int64_t lda, float* e, kmv_complex64* tau,
                     kmv_complex64* W, int64_t ldw, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zhetrd_panel(char uplo, int64_t n, int64_t nb, kmv_complex128* A, int64_t lda, double* e,
                     kmv_complex128* tau, kmv_complex128* W, int64_t ldw, void* workspace, size_t workspace_bytes,
                     void* stream);
size_t kmv_sytrd_panel_workspace_bytes(char prec, int64_t n, int64_t nb);

/* ---- Panel step of the bidiagonal reduction (Section 10: GEMV on the trailing
 * block and on the accumulated panels, on sub-blocks at arbitrary row and
 * column offsets, with strided vectors).  The description is for m >= n
 * (upper bidiagonal) in s and d; m < n and the complex forms follow it.  For the first nb columns and rows of the m x n matrix A
 * (device): column i is brought up to date, a reflector H_i = I - tauq_i v_i
 * v_i^T annihilates it below the diagonal, y_i is formed from the trailing
 * block (transposed product); row i is brought up to date, a reflector G_i =
 * I - taup_i u_i u_i^T annihilates it right of the superdiagonal, x_i is
 * formed from the trailing block; so that A - V Y^T - X U^T on the trailing
 * block is Q^T A P there.
 * On exit (all device memory): A[i..m-1][i] = v_i with A[i][i] = 1, A[i][i+1..
 * n-1] = u_i with A[i][i+1] = 1; d[i] the diagonal and e[i] the superdiagonal
 * entry of the bidiagonal form, tauq[i], taup[i]; X (m x nb, ldx >= m) holds
 * x_i in X[i+1..m-1][i], Y (n x nb, ldy >= n) holds y_i in Y[i+1..n-1][i]
 * (rows 0..i of column i of X and Y are scratch).  Rows and columns nb.. of A
 * beyond the panel are not modified.  The last column of the matrix has no
 * row reflector (e = taup = 0).  Norms are formed without rescaling.
 * Only enqueues kernels on `stream` (eight per column for nb <= 256: the two
 * products with the trailing block, their second stages and four launches of
 * the panel's own kernels, which do not write the scratch rows of X and Y;
 * about twenty GEMV-sized launches per column beyond), capturable.
 * m < n reduces to LOWER bidiagonal form with the roles of rows and columns
 * exchanged: row i is brought up to date and reflected first (G_i annihilates
 * A[i][i+1..n-1]; A[i][i..n-1] = u_i with A[i][i] = 1, d[i] the diagonal
 * entry), x_i follows, then column i below the diagonal (H_i annihilates
 * A[i+2..m-1][i]; A[i+1..m-1][i] = v_i with A[i+1][i] = 1, e[i] the
 * subdiagonal entry) and y_i; X[i+1..m-1][i] = x_i, Y[i+1..n-1][i] = y_i; the
 * last row of the matrix has no column reflector (e = tauq = 0).
 * Workspace: kmv_gebrd_panel_workspace_bytes(prec, m, n, nb), 256-byte
 * aligned.  Errors: negated argument number (m 1, n 2, nb 3
 * (0 <= nb <= min(m, n)), lda 5, ldx 11, ldy 13), KMV_ERR_NULL, KMV_ERR_WORKSPACE, or
 * the code of a failing launch (the columns before it are done). */
int kmv_sgebrd_panel(int64_t m, int64_t n, int64_t nb, float* A, int64_t lda, float* d, float* e, float* tauq,
                     float* taup, float* X, int64_t ldx, float* Y, int64_t ldy, void* workspace,
                     size_t workspace_bytes, void* stream);
int kmv_dgebrd_panel(int64_t m, int64_t n, int64_t nb, double* A, int64_t lda, double* d, double* e, double* tauq,
                     double* taup, double* X, int64_t ldx, double* Y, int64_t ldy, void* workspace,
                     size_t workspace_bytes, void* stream);
/* Complex matrices: H_i = I - tauq_i v_i v_i^H is applied as H_i^H from the
 * left and G_i = I - taup_i u_i u_i^H from the right, A - V Y^H - X U^H on
 * the trailing block is Q^H A P there.  A reflector for the vector (alpha, x)
 * has the real beta = -sign(Re alpha) * ||(alpha, x)||, so d and e are REAL
 * arrays; tauq and taup are complex; row i of A right of the diagonal holds
 * u_i^H (the conjugated vector, A[i][i+1] = 1).  Everything else as above. */
int kmv_cgebrd_panel(int64_t m, int64_t n, int64_t nb, kmv_complex64* A, int64_t lda, float* d, float* e,
                     kmv_complex64* tauq, kmv_complex64* taup, kmv_complex64* X, int64_t ldx, kmv_complex64* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);
int kmv_zgebrd_panel(int64_t m, int64_t n, int64_t nb, kmv_complex128* A, int64_t lda, double* d, double* e,
                     kmv_complex128* tauq, kmv_complex128* taup, kmv_complex128* X, int64_t ldx, kmv_complex128* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream);
size_t kmv_gebrd_panel_workspace_bytes(char prec, int64_t m, int64_t n, int64_t nb);

/* ---- Strided batches: `batch` products of one shape in one call; member b
 * uses A + b*strideA, x + b*stridex, y + b*stridey (strides in elements, >= 0;
 * 0 shares an input among the members; the outputs of two members must not
 * overlap: stridey >= 1 + (len(y)-1)*|incy| when batch > 1).  alpha and beta
 * (host) are common to all members.  The paper has no batched routines; these
 * serve the many-small-matrices case, where a launch per product would cost
 * more than the product: one launch covers the whole batch (65535 members per
 * launch, more are split), each member runs a single-launch form of the
 * kernels (GEMV without column or row splits; SYMV/HEMV with one workgroup
 * per member up to n = 1024, 512 for z, and the small-matrix kernel beyond),
 * so no workspace is needed and member results do not depend on the batch
 * size.  kmv_csymv_ / kmv_zsymv_strided_batched are the complex symmetric
 * products.  Restriction: incx must be 1.  Errors: negated argument number
 * (GEMV: trans 1, m 2, n 3, lda 6, strideA 7, incx 9, stridex 10, incy 13,
 * stridey 14, batch 15; SYMV/HEMV: uplo 1, n 2, lda 5, strideA 6, incx 8,
 * stridex 9, incy 12, stridey 13, batch 14), KMV_ERR_NULL, KMV_ERR_HIP + code. */
int kmv_sgemv_strided_batched(char trans, int64_t m, int64_t n, const float* alpha, const float* A, int64_t lda,
                              int64_t strideA, const float* x, int64_t incx, int64_t stridex, const float* beta,
                              float* y, int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_dgemv_strided_batched(char trans, int64_t m, int64_t n, const double* alpha, const double* A, int64_t lda,
                              int64_t strideA, const double* x, int64_t incx, int64_t stridex, const double* beta,
                              double* y, int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_cgemv_strided_batched(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
                              int64_t strideA, const kmv_complex64* x, int64_t incx, int64_t stridex, const kmv_complex64* beta,
                              kmv_complex64* y, int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_zgemv_strided_batched(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
                              int64_t strideA, const kmv_complex128* x, int64_t incx, int64_t stridex, const kmv_complex128* beta,
                              kmv_complex128* y, int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_ssymv_strided_batched(char uplo, int64_t n, const float* alpha, const float* A, int64_t lda, int64_t strideA,
                              const float* x, int64_t incx, int64_t stridex, const float* beta, float* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_dsymv_strided_batched(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, int64_t strideA,
                              const double* x, int64_t incx, int64_t stridex, const double* beta, double* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_chemv_strided_batched(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda, int64_t strideA,
                              const kmv_complex64* x, int64_t incx, int64_t stridex, const kmv_complex64* beta, kmv_complex64* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_zhemv_strided_batched(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda, int64_t strideA,
                              const kmv_complex128* x, int64_t incx, int64_t stridex, const kmv_complex128* beta, kmv_complex128* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_csymv_strided_batched(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda, int64_t strideA,
                              const kmv_complex64* x, int64_t incx, int64_t stridex, const kmv_complex64* beta, kmv_complex64* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);
int kmv_zsymv_strided_batched(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda, int64_t strideA,
                              const kmv_complex128* x, int64_t incx, int64_t stridex, const kmv_complex128* beta, kmv_complex128* y,
                              int64_t incy, int64_t stridey, int64_t batch, void* stream);

/* ---- Pointer-array batches: `batch` products of one shape; member b uses the
 * matrix A[b], the vectors x[b] and y[b].  A, x and y are arrays of `batch`
 * DEVICE pointers that themselves live in DEVICE memory (the kernels read
 * them; the host never does, so the arrays may be filled by an earlier kernel
 * on the stream).  For callers whose members do not lie at a constant stride;
 * everything else as for the strided batches above: one launch per 65535
 * members, single-launch kernels (in instances of their own that fetch the
 * operand pointers from the arrays), no workspace, alpha and beta on the host,
 * incx = 1, the outputs of two members must not overlap.  The members'
 * alignment is not known at enqueue time: the tile grids start at row 0 and
 * columns that are not 16-byte aligned are read with unaligned 16-byte loads.
 * Errors: negated argument number (GEMV: trans 1, m 2, n 3, lda 6, incx 8,
 * incy 11, batch 12; SYMV/HEMV: uplo 1, n 2, lda 5, incx 7, incy 10, batch
 * 11), KMV_ERR_NULL (also for a NULL array; the pointers inside the arrays
 * are not looked at), KMV_ERR_HIP + code. */
int kmv_sgemv_batched(char trans, int64_t m, int64_t n, const float* alpha, const float* const* A, int64_t lda,
                      const float* const* x, int64_t incx, const float* beta, float* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_dgemv_batched(char trans, int64_t m, int64_t n, const double* alpha, const double* const* A, int64_t lda,
                      const double* const* x, int64_t incx, const double* beta, double* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_cgemv_batched(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* const* A, int64_t lda,
                      const kmv_complex64* const* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_zgemv_batched(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* const* A, int64_t lda,
                      const kmv_complex128* const* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_ssymv_batched(char uplo, int64_t n, const float* alpha, const float* const* A, int64_t lda,
                      const float* const* x, int64_t incx, const float* beta, float* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_dsymv_batched(char uplo, int64_t n, const double* alpha, const double* const* A, int64_t lda,
                      const double* const* x, int64_t incx, const double* beta, double* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_chemv_batched(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* const* A, int64_t lda,
                      const kmv_complex64* const* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_zhemv_batched(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* const* A, int64_t lda,
                      const kmv_complex128* const* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_csymv_batched(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* const* A, int64_t lda,
                      const kmv_complex64* const* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* const* y, int64_t incy,
                      int64_t batch, void* stream);
int kmv_zsymv_batched(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* const* A, int64_t lda,
                      const kmv_complex128* const* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* const* y, int64_t incy,
                      int64_t batch, void* stream);

/* ---- Workspace sizes (bytes; an upper bound valid for every pointer
 * alignment, every increment and every tuning value).  prec is 's','d','c'
 * or 'z'.  The workspace holds the packed copy of a strided x and the
 * per-workgroup partial sums that the final pass adds in a fixed order (the
 * deterministic replacement of the atomic accumulation of Section 6.2).
 * The pointer passed as workspace must be 256-byte aligned.  Returns 0 for
 * an unknown prec, a negative dimension or an empty product. */
size_t kmv_gemv_workspace_bytes(char prec, char trans, int64_t m, int64_t n);
size_t kmv_symv_workspace_bytes(char prec, char uplo, int64_t n);

/* ---- Work partition of Section 6.2 (Eqs. local_workload and starting_point,
 * read with W in place of the misprinted d): share `w` and first item `s` of
 * worker `y` when `W` items are split over `Y` workers in contiguous,
 * balanced pieces.  Host-only helper, exported so that its invariants
 * (shares sum to W, pieces are contiguous, sizes differ by at most one) can
 * be tested; the kernels use the same formula for their row / column /
 * tile splits. */
void kmv_partition(int64_t W, int64_t Y, int64_t y, int64_t* w, int64_t* s);

/* ---- Bandwidth probe (the STREAM measurement of Section 7 that defines the
 * sustained bandwidth of the roofline): enqueues one pass of
 *   kind 0 "read"  : sum-reduce a[0..n)   (reads  n*8 bytes)
 *   kind 1 "copy"  : b[i] = a[i]          (moves 2*n*8 bytes)
 *   kind 2 "triad" : c[i] = a[i] + s*b[i] (moves 3*n*8 bytes)
 *   kind 3 "read, few workgroups": kind 0 in the launch shape of the fastest
 *                    matrix kernel - 192 workgroups (or the tuning value
 *                    wg_target), 16 vector loads in flight per lane
 * over n doubles.  a, b, c: device pointers to n doubles each (b, c may be
 * NULL for kinds 0 and 3; c for kind 1); `sink` a device pointer to at least
 * 8192 doubles (kinds 0 and 3 write per-workgroup sums there).  Returns 0 or
 * an error code as above. */
int kmv_stream_probe(int kind, int64_t n, const double* a, double* b, double* c, double* sink, void* stream);

/* ---- Tuning values for sweeps (Section 9: the tuning parameters are kept
 * apart from the kernel templates).  Keys are listed by kmv_tuning_keys()
 * as a comma separated string; kmv_set_tuning returns 0, or -1 for an
 * unknown key or a value outside the compiled set; value 0 = choose
 * automatically.  Process-wide; not thread safe against concurrent calls.
 *   gemv_n_splits, gemv_t_splits  column / row splits of the GEMV kernels
 *   gemv_n_row_tiles              row tiles per wave of GEMV-N (1, 2, 4)
 *   gemv_t_wgs                    workgroups of the transposed kernel (each
 *                                 takes every gemv_t_wgs-th group of columns;
 *                                 0 or more than there are groups: one each)
 *   gemv_short                    kernels for matrices of a few row tiles:
 *                                 1 = never, 2 = whenever they apply
 *   gemv_align_classes            GEMV with a leading dimension that is no
 *                                 multiple of 128 bytes: columns grouped by
 *                                 their alignment (1 = never, 2 = always)
 *   symv_variant                  SYMV/HEMV main kernel, see below (2, 3)
 *   symv_tiles_per_wave           row-chunk height, in units of 4 row tiles (1 .. 4;
 *                                 3 and 4 with one-tile units only)
 *   symv_unit_tiles               variant 2: row tiles per prefetch unit (1, 2)
 *   symv_piece_fixed              variant 2: fixed part of a piece's weight on
 *                                 the work line, plus one (1..17)
 *   symv_edge_weight              variant 2: extra weight per edge tile of a
 *                                 piece, plus one (1..17)
 *   wg_target                     workgroups the split heuristics aim for; for
 *                                 SYMV variant 2 the number of workgroups
 *   symv_member_rows              strided batches: largest n that gets one
 *                                 workgroup per member (up to 1024; 512 for z)
 *   symv_member_waves             waves of that workgroup (4, 8; a value
 *                                 also keeps the smallest members away from
 *                                 the one-wave-per-member kernel)
 *   symv_small_waves              variant 3: waves per workgroup (4, 8, 16)
 *   gemv_tiny_rows                strided batches: members with fewer rows
 *                                 than this get one wave each (1 = never)
 *   tuned_table                   1 = ignore the compiled-in table of measured
 *                                 per-size settings (see kmv_tuned_settings) */
int kmv_set_tuning(const char* key, int64_t value);
int64_t kmv_get_tuning(const char* key);
const char* kmv_tuning_keys(void);

/* The table of measured per-size settings (Section 9: the best tuning
 * parameters of every routine, precision and size found by a coarse and a
 * fine sweep, kept apart from the kernels).  The tuning tool writes its rows
 * (python -m paper_1410_1726_amd.tune table --save), the build compiles them
 * in, and the planners of the single-product entry points consult them for
 * square products (m == n) whose leading dimension is a whole number of
 * 128-byte lines: a row fills the tuning keys that the caller left at 0, for
 * that one call.  This query returns 1 and the row's values if a row applies
 * to routine op ('N'; 'T' for both transposed forms; 'L' or 'U' for
 * SYMV/HEMV) in precision prec at size n under the current tuning values, 0
 * if none does (the planner's rules decide), -1 for an unknown op or prec, a
 * negative n or a null pointer.  values (host, 7 entries, written only when
 * 1 is returned) = gemv_n_splits, gemv_n_row_tiles, gemv_t_splits,
 * symv_variant, symv_tiles_per_wave, symv_unit_tiles, wg_target; 0 = left to
 * the planner.  Host only: nothing is read from the device or launched. */
int kmv_tuned_settings(char prec, char op, int64_t n, int64_t* values);

/* Which main kernel a kmv_<prec>symv / hemv call with these arguments would
 * launch under the current tuning values: 2 = balanced shares of (row chunk,
 * panel) pieces (the balanced partition of Section 6.2 applied to the stored
 * triangle), 3 = the single-launch kernel for small matrices (no workspace
 * traffic; every stored element is read twice, which only pays while the
 * triangle stays in cache, hence its size limit of about 2000 rows).  Only the address
 * of A is used (its alignment decides), nothing is read or launched.  Returns
 * 0 for an unknown prec or uplo, n < 0 or lda < max(1, n).  For benchmarks
 * and profiles that have to name the kernel they time. */
int kmv_symv_kernel_variant(char prec, char uplo, int64_t n, const void* A, int64_t lda);

/* The balanced SYMV/HEMV kernel deals the pieces (row chunk x panel of 16
 * columns) of the stored triangle to its workgroups in contiguous shares of a
 * work line (Section 6.2, Eqs. local_workload / starting_point), on which a
 * piece weighs the row tiles it really holds (`unit_tiles` at a time) plus
 * `fixed`, plus `edge` for every edge tile among them (a tile with rows
 * before row 0, when shift > 0, or beyond row n - 1).  This call returns the table the planner computes for such a call:
 * start[y] = (chunk << 20) | piece inside the chunk for y = 0 .. workers (the
 * last entry is (number of chunks, 0)); first[k] / last[k] = the workers that
 * hold the first and the last piece of chunk k (arrays of 272 entries); *work
 * = length of the line.  Host arrays owned by the caller, any of them may be
 * NULL.  shift = leading masked slots of row tile 0 (0 .. rows per tile - 1),
 * chunk_tiles 4 or 8, unit_tiles 1 or 2, slots = workgroups wanted (at most
 * 800 are used).  Returns the number of workers, -1 for arguments out of
 * range.  Nothing is launched; exported for the tests of the host logic. */
int kmv_symv_shares(char prec, char uplo, int64_t n, int shift, int chunk_tiles, int unit_tiles, int64_t slots,
                    int fixed, int edge, uint32_t* start, uint16_t* first, uint16_t* last, int64_t* work);

/* kmv_dsymv for callers that cannot allocate or pass a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, results and errors as kmv_dsymv without the workspace pair:
 * the partial sums (and the packed copy of a strided x) go to a device array
 * of KMV_STATIC_SCRATCH_BYTES that is part of the library's code object (each
 * device the library runs on holds its copy until the process ends).  The
 * call allocates nothing and frees nothing.  A product whose plan needs more
 * than the array holds is refused with KMV_ERR_WORKSPACE before anything is
 * enqueued: with the default tuning DSYMV fits up to about n = 54000
 * (kmv_symv_workspace_bytes('d', uplo, n) is an upper bound of the need).
 * The first call on a device looks up the array's address (make it outside a
 * graph capture).  All calls on a device share the one array: two calls whose
 * kernels may overlap in time (different streams, or graph branches) race
 * and give wrong results; calls on one stream are safe.  Nothing in the array
 * has to be cleared between calls: every slot is written before it is read. */
#define KMV_STATIC_SCRATCH_BYTES (16u << 20)
int kmv_dsymv_static(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x,
                     int64_t incx, const double* beta, double* y, int64_t incy, void* stream);

const char* kmv_version(void);

#ifdef __cplusplus
}
#endif
#endif /* KMV_H */
