// CPU oracle for the dense matrix-vector products  y = alpha*op(A)*x + beta*y.
//
// TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
// GPU library is checked against.  It shares no code with the GPU library and
// must never be called from the product path.
//
// What it computes (paper, Section 5.2 "KBLAS routines", the operation
// y = alpha*A*x + beta*y for a general or Hermitian/symmetric A, and
// Section 7, which states that a symmetric/Hermitian product reads only the
// upper or only the lower triangle):
//
//   GEMV  N :  y_i = alpha * sum_j a_ij     * x_j + beta*y_i     i < m
//   GEMV  T :  y_j = alpha * sum_i a_ij     * x_i + beta*y_j     j < n
//   GEMV  C :  y_j = alpha * sum_i conj(a_ij)*x_i + beta*y_j     j < n
//   SYMV    :  y_i = alpha * sum_j s_ij * x_j + beta*y_i,  s_ij = a_ij when
//              (i,j) lies in the stored triangle, a_ji otherwise
//   HEMV    :  same with s_ij = conj(a_ji) outside the stored triangle and
//              s_ii = Re(a_ii)
//   The paper's routine table lists SYMV for s,d and HEMV for c,z; the
//   complex *symmetric* product (no conjugation anywhere, the diagonal taken
//   as stored) is the same definition with the s,d rule applied to c,z and is
//   offered through mvo_symv_complex_symmetric.
//
// A is column major with leading dimension lda (Section 5.3, single-GPU
// layout): a_ij = A[i + j*lda].  Vectors follow the reference-BLAS increment
// rule: element k of a length-len vector with increment inc lives at
// v[k*inc] when inc > 0 and at v[(k-(len-1))*inc] when inc < 0.
//
// Each output element is one plain left-to-right sum.  There is no blocking,
// no reordering and no vectorisation by hand.  OpenMP only distributes
// *different output elements* over threads.
//
// Readings of points the paper leaves open (standard BLAS conventions):
//   * beta == 0  : y is not read (NaN/Inf in y do not propagate).
//   * alpha == 0 : A and x are not read.
//   * HEMV ignores the imaginary part of the diagonal.
//   * only the stored triangle of a symmetric/Hermitian matrix is indexed.
//
// Accumulation modes:
//   MODE_W (0)  accumulate and return in the working precision (this is the
//               mode that is timed as the CPU baseline);
//   MODE_X (1)  accumulate in extended precision (double for s/c, long
//               double for d/z) and return double / complex double, so the
//               oracle's own rounding does not consume the parity tolerance;
//   MODE_ABS(2) the same loops on absolute values, returning in double
//               |alpha| * sum |a||x| + |beta||y| : the denominator of the
//               componentwise error bound.
//
// Pins (tests/test_oracle_*.py): exact rational brute force on tiny integer
// inputs, numpy products on the explicitly completed matrix, closed forms for
// A = I and A = ones, alpha = 0, beta = 0, transpose identities, NaN poison
// in the unreferenced triangle.

#include <complex>
#include <cstdint>
#include <cstddef>
#include <cmath>

namespace {

enum { MODE_W = 0, MODE_X = 1, MODE_ABS = 2 };

template <class T> struct is_cplx { static const bool value = false; };
template <class R> struct is_cplx<std::complex<R> > { static const bool value = true; };

template <class T> inline T conj_of(const T& v) { return v; }
template <class R> inline std::complex<R> conj_of(const std::complex<R>& v) { return std::conj(v); }

template <class T> inline T real_only(const T& v) { return v; }
template <class R> inline std::complex<R> real_only(const std::complex<R>& v) { return std::complex<R>(v.real(), R(0)); }

template <class T> inline bool is_zero(const T& v) { return v == T(0); }

// position of logical element k in a strided vector (reference-BLAS rule)
inline int64_t vpos(int64_t k, int64_t len, int64_t inc) {
    return inc > 0 ? k * inc : (k - (len - 1)) * inc;
}

// convert a stored value to the accumulation type (plain widening)
template <class ACC, class T> struct widen {
    static ACC get(const T& v) { return ACC(v); }
};
template <class RA, class R> struct widen<std::complex<RA>, std::complex<R> > {
    static std::complex<RA> get(const std::complex<R>& v) { return std::complex<RA>(RA(v.real()), RA(v.imag())); }
};
// absolute-value mode: everything becomes a non-negative double
template <class T> inline double absval(const T& v) { return std::fabs(double(v)); }
template <class R> inline double absval(const std::complex<R>& v) { return std::hypot(double(v.real()), double(v.imag())); }

// ---------------------------------------------------------------------------
// GEMV.  OUT is the output element type, ACC the accumulation type.
// ---------------------------------------------------------------------------
template <class T, class ACC, class OUT>
void gemv_loops(char trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda,
                const T* x, int64_t incx, T beta, const T* yin, int64_t incy,
                OUT* yout, const int64_t* sample, int64_t nsample) {
    const bool notrans = (trans == 'N' || trans == 'n');
    const bool conjt = (trans == 'C' || trans == 'c');
    const int64_t leny = notrans ? m : n;
    const int64_t lenx = notrans ? n : m;
    const int64_t nout = sample ? nsample : leny;
    const ACC al = widen<ACC, T>::get(alpha);
    const ACC be = widen<ACC, T>::get(beta);
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nout; ++t) {
        const int64_t k = sample ? sample[t] : t;   // output index
        ACC sum = ACC(0);
        if (!is_zero(alpha)) {
            if (notrans) {
                for (int64_t j = 0; j < lenx; ++j)
                    sum += widen<ACC, T>::get(A[k + j * lda]) * widen<ACC, T>::get(x[vpos(j, lenx, incx)]);
            } else {
                for (int64_t i = 0; i < lenx; ++i) {
                    T a = A[i + k * lda];
                    if (conjt) a = conj_of(a);
                    sum += widen<ACC, T>::get(a) * widen<ACC, T>::get(x[vpos(i, lenx, incx)]);
                }
            }
        }
        ACC r = is_zero(alpha) ? ACC(0) : al * sum;
        if (!is_zero(beta)) r += be * widen<ACC, T>::get(yin[vpos(k, leny, incy)]);
        yout[vpos(k, leny, incy)] = OUT(r);
    }
}

template <class T>
void gemv_abs(char trans, int64_t m, int64_t n, T alpha, const T* A, int64_t lda,
              const T* x, int64_t incx, T beta, const T* yin, int64_t incy,
              double* yout, const int64_t* sample, int64_t nsample) {
    const bool notrans = (trans == 'N' || trans == 'n');
    const int64_t leny = notrans ? m : n;
    const int64_t lenx = notrans ? n : m;
    const int64_t nout = sample ? nsample : leny;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < nout; ++t) {
        const int64_t k = sample ? sample[t] : t;
        double sum = 0.0;
        if (!is_zero(alpha)) {
            for (int64_t l = 0; l < lenx; ++l) {
                const T a = notrans ? A[k + l * lda] : A[l + k * lda];
                sum += absval(a) * absval(x[vpos(l, lenx, incx)]);
            }
        }
        double r = absval(alpha) * sum;
        if (!is_zero(beta)) r += absval(beta) * absval(yin[vpos(k, leny, incy)]);
        yout[vpos(k, leny, incy)] = r;
    }
}

// ---------------------------------------------------------------------------
// SYMV / HEMV.  Only A[i + j*lda] with (i,j) inside the uplo triangle is read.
// ---------------------------------------------------------------------------
template <class T, class ACC, class OUT>
void symv_loops(bool herm, char uplo, int64_t n, T alpha, const T* A, int64_t lda,
                const T* x, int64_t incx, T beta, const T* yin, int64_t incy,
                OUT* yout, const int64_t* sample, int64_t nsample) {
    const bool lower = (uplo == 'L' || uplo == 'l');
    const int64_t nout = sample ? nsample : n;
    const ACC al = widen<ACC, T>::get(alpha);
    const ACC be = widen<ACC, T>::get(beta);
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < nout; ++t) {
        const int64_t i = sample ? sample[t] : t;
        ACC sum = ACC(0);
        if (!is_zero(alpha)) {
            for (int64_t j = 0; j < n; ++j) {
                T s;
                if (j == i) {
                    s = A[i + i * lda];
                    if (herm) s = real_only(s);
                } else {
                    // (i,j) is in the lower triangle when i > j
                    const bool stored = lower ? (i > j) : (i < j);
                    if (stored) {
                        s = A[i + j * lda];
                    } else {
                        s = A[j + i * lda];
                        if (herm) s = conj_of(s);
                    }
                }
                sum += widen<ACC, T>::get(s) * widen<ACC, T>::get(x[vpos(j, n, incx)]);
            }
        }
        ACC r = is_zero(alpha) ? ACC(0) : al * sum;
        if (!is_zero(beta)) r += be * widen<ACC, T>::get(yin[vpos(i, n, incy)]);
        yout[vpos(i, n, incy)] = OUT(r);
    }
}

template <class T>
void symv_abs(bool herm, char uplo, int64_t n, T alpha, const T* A, int64_t lda,
              const T* x, int64_t incx, T beta, const T* yin, int64_t incy,
              double* yout, const int64_t* sample, int64_t nsample) {
    const bool lower = (uplo == 'L' || uplo == 'l');
    const int64_t nout = sample ? nsample : n;
#pragma omp parallel for schedule(dynamic, 16)
    for (int64_t t = 0; t < nout; ++t) {
        const int64_t i = sample ? sample[t] : t;
        double sum = 0.0;
        if (!is_zero(alpha)) {
            for (int64_t j = 0; j < n; ++j) {
                const bool stored = (j == i) || (lower ? (i > j) : (i < j));
                const T s = stored ? A[i + j * lda] : A[j + i * lda];
                // HEMV uses only the real part of the diagonal
                const double as = (j == i && herm) ? absval(real_only(s)) : absval(s);
                sum += as * absval(x[vpos(j, n, incx)]);
            }
        }
        double r = absval(alpha) * sum;
        if (!is_zero(beta)) r += absval(beta) * absval(yin[vpos(i, n, incy)]);
        yout[vpos(i, n, incy)] = r;
    }
}

// --- per-precision dispatch -------------------------------------------------
// XT = extended accumulation type, XO = type returned in MODE_X.
template <class T, class XT, class XO>
int gemv_any(int mode, char trans, int64_t m, int64_t n, const void* alpha, const void* A, int64_t lda,
             const void* x, int64_t incx, const void* beta, const void* yin, int64_t incy, void* yout,
             const int64_t* sample, int64_t nsample) {
    const T al = *static_cast<const T*>(alpha), be = *static_cast<const T*>(beta);
    const T *a = static_cast<const T*>(A), *xv = static_cast<const T*>(x), *yi = static_cast<const T*>(yin);
    if (mode == MODE_W) gemv_loops<T, T, T>(trans, m, n, al, a, lda, xv, incx, be, yi, incy, static_cast<T*>(yout), sample, nsample);
    else if (mode == MODE_X) gemv_loops<T, XT, XO>(trans, m, n, al, a, lda, xv, incx, be, yi, incy, static_cast<XO*>(yout), sample, nsample);
    else if (mode == MODE_ABS) gemv_abs<T>(trans, m, n, al, a, lda, xv, incx, be, yi, incy, static_cast<double*>(yout), sample, nsample);
    else return -100;
    return 0;
}

template <class T, class XT, class XO>
int symv_any(int mode, bool herm, char uplo, int64_t n, const void* alpha, const void* A, int64_t lda,
             const void* x, int64_t incx, const void* beta, const void* yin, int64_t incy, void* yout,
             const int64_t* sample, int64_t nsample) {
    const T al = *static_cast<const T*>(alpha), be = *static_cast<const T*>(beta);
    const T *a = static_cast<const T*>(A), *xv = static_cast<const T*>(x), *yi = static_cast<const T*>(yin);
    if (mode == MODE_W) symv_loops<T, T, T>(herm, uplo, n, al, a, lda, xv, incx, be, yi, incy, static_cast<T*>(yout), sample, nsample);
    else if (mode == MODE_X) symv_loops<T, XT, XO>(herm, uplo, n, al, a, lda, xv, incx, be, yi, incy, static_cast<XO*>(yout), sample, nsample);
    else if (mode == MODE_ABS) symv_abs<T>(herm, uplo, n, al, a, lda, xv, incx, be, yi, incy, static_cast<double*>(yout), sample, nsample);
    else return -100;
    return 0;
}

typedef std::complex<float> cf;
typedef std::complex<double> cd;
typedef std::complex<long double> cl;

}  // namespace

// ---------------------------------------------------------------------------
// C entry points (all pointers are HOST pointers).
//   prec : 's','d','c','z'
//   yin  : y on entry (working precision, never written)
//   yout : result; element type depends on mode (see top of file); laid out
//          with the same increment incy as y.  Elements that are not computed
//          (when `sample` selects a subset of output indices) are untouched.
//   sample/nsample : optional list of output indices to compute; NULL = all.
// Returns 0, or a negative number for an unknown prec/mode.
// ---------------------------------------------------------------------------
extern "C" int mvo_gemv(char prec, int mode, char trans, int64_t m, int64_t n, const void* alpha,
                        const void* A, int64_t lda, const void* x, int64_t incx, const void* beta,
                        const void* yin, int64_t incy, void* yout, const int64_t* sample, int64_t nsample) {
    switch (prec) {
        case 's': return gemv_any<float, double, double>(mode, trans, m, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'd': return gemv_any<double, long double, double>(mode, trans, m, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'c': return gemv_any<cf, cd, cd>(mode, trans, m, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'z': return gemv_any<cd, cl, cd>(mode, trans, m, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
    }
    return -101;
}

// SYMV for prec 's','d'; HEMV for prec 'c','z'.
extern "C" int mvo_symv(char prec, int mode, char uplo, int64_t n, const void* alpha,
                        const void* A, int64_t lda, const void* x, int64_t incx, const void* beta,
                        const void* yin, int64_t incy, void* yout, const int64_t* sample, int64_t nsample) {
    switch (prec) {
        case 's': return symv_any<float, double, double>(mode, false, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'd': return symv_any<double, long double, double>(mode, false, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'c': return symv_any<cf, cd, cd>(mode, true, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'z': return symv_any<cd, cl, cd>(mode, true, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
    }
    return -101;
}

// Complex symmetric SYMV (prec 'c','z'): the SYMV rule without any conjugation.
extern "C" int mvo_symv_complex_symmetric(char prec, int mode, char uplo, int64_t n, const void* alpha,
                                          const void* A, int64_t lda, const void* x, int64_t incx, const void* beta,
                                          const void* yin, int64_t incy, void* yout, const int64_t* sample,
                                          int64_t nsample) {
    switch (prec) {
        case 'c': return symv_any<cf, cd, cd>(mode, false, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
        case 'z': return symv_any<cd, cl, cd>(mode, false, uplo, n, alpha, A, lda, x, incx, beta, yin, incy, yout, sample, nsample);
    }
    return -101;
}

#ifdef _OPENMP
#include <omp.h>
extern "C" int mvo_num_threads(void) { return omp_get_max_threads(); }
extern "C" void mvo_set_num_threads(int t) { omp_set_num_threads(t); }
#else
extern "C" int mvo_num_threads(void) { return 1; }
extern "C" void mvo_set_num_threads(int) {}
#endif
