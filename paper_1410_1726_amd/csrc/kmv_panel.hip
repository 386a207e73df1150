// Panel steps of the two-sided reductions - symmetric tridiagonal (below) and
// bidiagonal (further down) - built on the library's own
// SYMV and GEMV calls (paper, Section 10: the two-sided reductions spend their
// memory-bound time in exactly these products - SYMV on the trailing block once
// per column, GEMV on the tall panels of accumulated reflectors - and always on
// sub-blocks that start at arbitrary offsets inside the matrix, Section 6.6).
//
// The step is the published "latrd" panel of the blocked Householder
// tridiagonalisation, lower storage, written from its definition:
//   column i:  a  = A[i:,i] - V[i:,:i] W[i,:i]^T - W[i:,:i] V[i,:i]^T        (2 GEMV-N, strided x)
//              reflector (beta, tau, v) that annihilates a[2:]                (one small kernel)
//              w  = A[i+1:,i+1:] v                                            (SYMV, trailing block)
//              w -= V[i+1:,:i] (W[i+1:,:i]^T v) + W[i+1:,:i] (V[i+1:,:i]^T v) (2 GEMV-T, 2 GEMV-N)
//              w  = tau w;  w -= (tau/2)(w.v) v                               (one small kernel)
// Upper storage runs the mirror image (last nb columns, from the right), complex types the Hermitian form
// (conjugated transposes, real e); the bidiagonal step further down exists for all four precisions as well.
// Everything stays on the device and on the caller's stream: tau and the dot
// product never visit the host, so a whole panel is one uninterrupted sequence of
// launches (and can be captured in a graph).  The matrix-vector products go
// through the public entry points, i.e. through the same argument checks,
// planners and kernels as any other caller's.
#include "../../include/kmv.h"
#include "kmv_common.hpp"

namespace kmv {
namespace {

constexpr int PT = 1024;   // threads of the two single-workgroup vector kernels

// Sum over the workgroup in a fixed order: lanes by DPP, then the waves' sums in wave order.
template <class T> __device__ __forceinline__ T block_sum(T v, T* red) {
    const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
    const T s = wave_sum(v);
    __syncthreads();             // red may still be read from an earlier call
    if (lane == 0) red[w] = s;
    __syncthreads();
    T tot = red[0];
#pragma unroll
    for (int k = 1; k < PT / WAVE; ++k) tot += red[k];
    return tot;
}

// The two vector kernels run in one workgroup (their sums need no second launch then); each thread
// keeps PU independent loads in flight per pass, which is what their time depends on.
constexpr int PU = 8;

// Householder reflector for the vector (alpha, x): alpha at *head, the m-1 elements of x at tail[k*inc].
// On exit *head = 1, x <- x / (alpha - beta), *e = beta = -sign(alpha) * ||(alpha, x)||,
// *tau = (beta - alpha) / beta; a zero x gives tau = 0, beta = alpha.
template <class T>
__global__ __launch_bounds__(PT) void reflector_kernel(int64_t m, T* head, T* tail, int64_t inc, T* e, T* tau) {
    __shared__ T red[PT / WAVE];
    const T alpha = *head;
    T ss = 0;
    for (int64_t base = threadIdx.x; base < m - 1; base += (int64_t)PU * PT) {
        T x[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            x[u] = k < m - 1 ? tail[k * inc] : T(0);
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) ss += x[u] * x[u];
    }
    const T xnorm = sqrt(block_sum(ss, red));    // every thread has read *head once this returns
    T beta = alpha, t = 0;
    if (xnorm != 0) {
        beta = -copysign(sqrt(alpha * alpha + xnorm * xnorm), alpha);
        t = (beta - alpha) / beta;
        const T scale = T(1) / (alpha - beta);
        for (int64_t base = threadIdx.x; base < m - 1; base += (int64_t)PU * PT) {
            T x[PU];
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int64_t k = base + (int64_t)u * PT;
                x[u] = k < m - 1 ? tail[k * inc] : T(0);
            }
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int64_t k = base + (int64_t)u * PT;
                if (k < m - 1) tail[k * inc] = x[u] * scale;
            }
        }
    }
    if (threadIdx.x == 0) {
        *head = 1;
        *e = beta;
        *tau = t;
    }
}

// dst[k*dinc] = src[k*sinc] (conjugated with CONJ): a row of a column-major matrix to a contiguous vector and back
template <class T, bool CONJ = false>
__global__ void strided_copy_kernel(int64_t len, const T* src, int64_t sinc, T* dst, int64_t dinc) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) {
        T v = src[k * sinc];
        if constexpr (CONJ && Traits<T>::cplx) v.im = -v.im;
        dst[k * dinc] = v;
    }
}

// v <- (*s) v, the scalar in device memory
template <class T> __global__ void scale_kernel(int64_t len, const T* s, T* v) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) v[k] = mul_of(*s, v[k]);
}

// w <- tau w - (tau/2) ((tau w).v) v.  Then, for the next column's update, the first `cnt` entries of the
// next row of W and of V (element j at wnext[j*ldw], vnext[j*ldv]; the last one of W is w[0], just written)
// are copied to the contiguous wrow / vrow, which spares that column two launches for packing strided rows.
template <class T>
__global__ __launch_bounds__(PT) void finish_w_kernel(int64_t m, const T* tau, const T* v, T* w, const T* wnext,
                                                      int64_t ldw, const T* vnext, int64_t ldv, int cnt, T* wrow,
                                                      T* vrow) {
    __shared__ T red[PT / WAVE];
    const T t = *tau;
    T part = 0;
    for (int64_t base = threadIdx.x; base < m; base += (int64_t)PU * PT) {
        T wv[PU], vv[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            wv[u] = k < m ? w[k] : T(0);
            vv[u] = k < m ? v[k] : T(0);
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) part += (t * wv[u]) * vv[u];
    }
    const T c = T(-0.5) * t * block_sum(part, red);
    for (int64_t base = threadIdx.x; base < m; base += (int64_t)PU * PT) {
        T wv[PU], vv[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            wv[u] = k < m ? w[k] : T(0);
            vv[u] = k < m ? v[k] : T(0);
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            if (k < m) w[k] = t * wv[u] + c * vv[u];
        }
    }
    __syncthreads();     // w[0] is in place for every thread of the workgroup
    if ((int)threadIdx.x < cnt) {
        wrow[threadIdx.x] = wnext[threadIdx.x * ldw];
        vrow[threadIdx.x] = vnext[threadIdx.x * ldv];
    }
}

// ---- the same two kernels for complex vectors (C = cf32 / cf64, R its real type) ----
// Reflector for (alpha, x), alpha at *head, x at tail[0..m-2]: beta = -sign(Re alpha) ||(alpha, x)|| is real,
// tau = (beta - alpha) / beta, x <- x / (alpha - beta), *head = 1; x = 0 with a real alpha gives tau = 0,
// beta = alpha.  The diagonal element above the head (*diag, the d_i of this column; may be null) loses its
// imaginary part here: it is real for a Hermitian matrix and was only carried along by the column update.
template <class C, class R>
__global__ __launch_bounds__(PT) void reflector_kernel_c(int64_t m, C* diag, C* head, C* tail, R* e, C* tau) {
    __shared__ R red[PT / WAVE];
    const C alpha = *head;
    R ss = 0;
    for (int64_t base = threadIdx.x; base < m - 1; base += (int64_t)PU * PT) {
        C x[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            x[u] = k < m - 1 ? tail[k] : C{0, 0};
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) ss += x[u].re * x[u].re + x[u].im * x[u].im;
    }
    const R xnorm = sqrt(block_sum(ss, red));
    R beta = alpha.re;
    C t{0, 0};
    if (xnorm != 0 || alpha.im != 0) {
        beta = -copysign(sqrt(alpha.re * alpha.re + alpha.im * alpha.im + xnorm * xnorm), alpha.re);
        t = C{(beta - alpha.re) / beta, -alpha.im / beta};
        // 1 / (alpha - beta)
        const R dr = alpha.re - beta, di = alpha.im, den = dr * dr + di * di;
        const C scale{dr / den, -di / den};
        for (int64_t base = threadIdx.x; base < m - 1; base += (int64_t)PU * PT) {
            C x[PU];
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int64_t k = base + (int64_t)u * PT;
                x[u] = k < m - 1 ? tail[k] : C{0, 0};
            }
#pragma unroll
            for (int u = 0; u < PU; ++u) {
                const int64_t k = base + (int64_t)u * PT;
                if (k < m - 1) tail[k] = C{x[u].re * scale.re - x[u].im * scale.im, x[u].re * scale.im + x[u].im * scale.re};
            }
        }
    }
    if (threadIdx.x == 0) {
        *head = C{1, 0};
        if (diag) diag->im = 0;
        *e = beta;
        *tau = t;
    }
}

// w <- tau w - (tau/2) ((tau w)^H v) v, then the conjugated next rows of W and V packed for the next column.
// The next diagonal element (*diag_next) loses its imaginary part before that column's update reads it: the
// caller need not have set it, and a product with it would carry whatever it holds into the real part
// (null for the last column of the panel: the element after it is not the panel's).
template <class C, class R>
__global__ __launch_bounds__(PT) void finish_w_kernel_c(int64_t m, const C* tau, const C* v, C* w, const C* wnext,
                                                        int64_t ldw, const C* vnext, int64_t ldv, int cnt, C* wrow,
                                                        C* vrow, C* diag_next) {
    __shared__ R red[PT / WAVE];
    const C t = *tau;
    R pr = 0, pi = 0;       // sum of conj(t w_k) v_k
    for (int64_t base = threadIdx.x; base < m; base += (int64_t)PU * PT) {
        C wv[PU], vv[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            wv[u] = k < m ? w[k] : C{0, 0};
            vv[u] = k < m ? v[k] : C{0, 0};
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const R sr = t.re * wv[u].re - t.im * wv[u].im, si = t.re * wv[u].im + t.im * wv[u].re;   // t w
            pr += sr * vv[u].re + si * vv[u].im;
            pi += sr * vv[u].im - si * vv[u].re;
        }
    }
    const R dr = block_sum(pr, red), di = block_sum(pi, red);
    // c = -(t/2) * dot
    const C c{R(-0.5) * (t.re * dr - t.im * di), R(-0.5) * (t.re * di + t.im * dr)};
    for (int64_t base = threadIdx.x; base < m; base += (int64_t)PU * PT) {
        C wv[PU], vv[PU];
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            wv[u] = k < m ? w[k] : C{0, 0};
            vv[u] = k < m ? v[k] : C{0, 0};
        }
#pragma unroll
        for (int u = 0; u < PU; ++u) {
            const int64_t k = base + (int64_t)u * PT;
            if (k < m)
                w[k] = C{t.re * wv[u].re - t.im * wv[u].im + c.re * vv[u].re - c.im * vv[u].im,
                         t.re * wv[u].im + t.im * wv[u].re + c.re * vv[u].im + c.im * vv[u].re};
        }
    }
    __syncthreads();
    if ((int)threadIdx.x < cnt) {
        const C a = wnext[threadIdx.x * ldw], b = vnext[threadIdx.x * ldv];
        wrow[threadIdx.x] = C{a.re, -a.im};
        vrow[threadIdx.x] = C{b.re, -b.im};
    }
    if (threadIdx.x == 0 && diag_next) diag_next->im = 0;
}

// a column without a reflector: e = tau = 0, the diagonal element real
template <class C, class R> __global__ void no_reflector_kernel_c(C* diag, R* e, C* tau) {
    diag->im = 0;
    *e = 0;
    *tau = C{0, 0};
}

// e and tau of a column that has no reflector (a fill kernel rather than a memset node, so that a
// captured panel holds kernels only)
template <class R, class T> __global__ void no_reflector_kernel(R* e, T* tau) {
    *e = 0;
    *tau = zero_of<T>();
}

template <class T> inline T from_real(double v) {
    if constexpr (Traits<T>::cplx) return T{(typename Traits<T>::real)v, 0};
    else return (T)v;
}

template <class T> struct Calls;
template <> struct Calls<float> {
    static constexpr char prec = 's';
    static constexpr auto gemv = kmv_sgemv;
    static constexpr auto symv = kmv_ssymv;
};
template <> struct Calls<double> {
    static constexpr char prec = 'd';
    static constexpr auto gemv = kmv_dgemv;
    static constexpr auto symv = kmv_dsymv;
};

template <> struct Calls<cf32> {
    static constexpr char prec = 'c';
    static int gemv(char trans, int64_t m, int64_t n, const cf32* alpha, const cf32* A, int64_t lda, const cf32* x,
                    int64_t incx, const cf32* beta, cf32* y, int64_t incy, void* ws, size_t wsb, void* stream) {
        return kmv_cgemv(trans, m, n, (const kmv_complex64*)alpha, (const kmv_complex64*)A, lda, (const kmv_complex64*)x, incx,
                         (const kmv_complex64*)beta, (kmv_complex64*)y, incy, ws, wsb, stream);
    }
    static int symv(char uplo, int64_t n, const cf32* alpha, const cf32* A, int64_t lda, const cf32* x, int64_t incx,
                    const cf32* beta, cf32* y, int64_t incy, void* ws, size_t wsb, void* stream) {
        return kmv_chemv(uplo, n, (const kmv_complex64*)alpha, (const kmv_complex64*)A, lda, (const kmv_complex64*)x, incx,
                         (const kmv_complex64*)beta, (kmv_complex64*)y, incy, ws, wsb, stream);
    }
};
template <> struct Calls<cf64> {
    static constexpr char prec = 'z';
    static int gemv(char trans, int64_t m, int64_t n, const cf64* alpha, const cf64* A, int64_t lda, const cf64* x,
                    int64_t incx, const cf64* beta, cf64* y, int64_t incy, void* ws, size_t wsb, void* stream) {
        return kmv_zgemv(trans, m, n, (const kmv_complex128*)alpha, (const kmv_complex128*)A, lda, (const kmv_complex128*)x,
                         incx, (const kmv_complex128*)beta, (kmv_complex128*)y, incy, ws, wsb, stream);
    }
    static int symv(char uplo, int64_t n, const cf64* alpha, const cf64* A, int64_t lda, const cf64* x, int64_t incx,
                    const cf64* beta, cf64* y, int64_t incy, void* ws, size_t wsb, void* stream) {
        return kmv_zhemv(uplo, n, (const kmv_complex128*)alpha, (const kmv_complex128*)A, lda, (const kmv_complex128*)x, incx,
                         (const kmv_complex128*)beta, (kmv_complex128*)y, incy, ws, wsb, stream);
    }
};

inline size_t max_of(size_t a, size_t b) { return a > b ? a : b; }

// bytes at the front of the workspace for the two packed rows (nb elements each)
template <class T> size_t rows_bytes(int64_t nb) {
    return (size_t)((2 * nb * sizeof(T) + 255) / 256) * 256;
}

// the packed rows plus the largest workspace any product of the panel asks for
template <class T> size_t panel_workspace(int64_t n, int64_t nb) {
    if (n <= 0 || nb <= 0) return 0;
    if (nb > n) nb = n;
    size_t need = 0;
    for (int64_t i = 0; i < nb; ++i) {
        need = max_of(need, kmv_gemv_workspace_bytes(Calls<T>::prec, 'N', n - i, i));
        if (i < n - 1) {
            need = max_of(need, kmv_symv_workspace_bytes(Calls<T>::prec, 'L', n - i - 1));
            need = max_of(need, kmv_gemv_workspace_bytes(Calls<T>::prec, 'T', n - i - 1, i));
            need = max_of(need, kmv_gemv_workspace_bytes(Calls<T>::prec, 'N', n - i - 1, i));
        }
    }
    return rows_bytes<T>(nb) + need;
}

// T real: SYTRD panel; T complex (cf32 / cf64): HETRD panel, e real, transposes conjugated
template <class T>
int sytrd_panel(char uplo, int64_t n, int64_t nb, T* A, int64_t lda, typename Traits<T>::real* e, T* tau, T* W,
                int64_t ldw, void* ws, size_t wsb, void* stream) {
    using R = typename Traits<T>::real;
    constexpr bool CPLX = Traits<T>::cplx;
    constexpr char TC = CPLX ? 'C' : 'T';
    const bool lower = (uplo == 'L' || uplo == 'l');
    if (!lower && uplo != 'U' && uplo != 'u') return -1;
    if (n < 0) return -2;
    if (nb < 0 || nb > n) return -3;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (ldw < (n > 1 ? n : 1)) return -9;
    if (n == 0 || nb == 0) return KMV_OK;
    if (!A || !e || !tau || !W) return KMV_ERR_NULL;
    if (!ws || wsb < panel_workspace<T>(n, nb) || ((uintptr_t)ws % 256) != 0) return KMV_ERR_WORKSPACE;
    static_assert(PT >= 1024, "the row copy at the end of finish_w_kernel uses one thread per column of the panel");
    if (nb > PT) return -3;
    T* wrow = static_cast<T*>(ws);           // row i of W and of V, packed by the column before
    T* vrow = wrow + nb;
    ws = static_cast<char*>(ws) + rows_bytes<T>(nb);
    wsb -= rows_bytes<T>(nb);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const T one = from_real<T>(1), zero = from_real<T>(0), minus = from_real<T>(-1);
    const auto gemv = Calls<T>::gemv;
    const auto symv = Calls<T>::symv;
    int rc = KMV_OK;
    if (!lower) {
        // Upper storage: the mirror image.  The LAST nb columns are reduced, from column n-1 down to n-nb; column
        // i has slot iw = i - (n - nb) in e, tau and W; its reflector annihilates A[0:i-1, i], v = A[0:i, i] with
        // the one at row i-1; the k = n-1-i columns to its right are the reflectors and W columns done before.
        const int64_t first = n - nb;
        for (int64_t i = n - 1; i >= first; --i) {
            const int64_t iw = i - first, k = n - 1 - i;
            T* col = A + i * lda;                    // A[0:i+1, i]
            if (k > 0) {
                rc = gemv('N', i + 1, k, &minus, A + (i + 1) * lda, lda, wrow, 1, &one, col, 1, ws, wsb, stream);
                if (rc) return rc;
                rc = gemv('N', i + 1, k, &minus, W + (iw + 1) * ldw, ldw, vrow, 1, &one, col, 1, ws, wsb, stream);
                if (rc) return rc;
            }
            if (i == 0) {   // first column of the matrix: no reflector
                if constexpr (CPLX) hipLaunchKernelGGL((no_reflector_kernel_c<T, R>), dim3(1), dim3(1), 0, s, col, e + iw, tau + iw);
                else hipLaunchKernelGGL((no_reflector_kernel<T, T>), dim3(1), dim3(1), 0, s, e + iw, tau + iw);
                const hipError_t he = hipGetLastError();
                if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
                continue;
            }
            const int64_t m = i;                     // length of v
            T* head = col + (i - 1);                 // A[i-1, i]
            T* w = W + iw * ldw;                     // W[0:i, iw]
            T* small = W + (i + 1) + iw * ldw;       // W[i+1:, iw]: the k-vector of the corrections
            if constexpr (CPLX) hipLaunchKernelGGL((reflector_kernel_c<T, R>), dim3(1), dim3(PT), 0, s, m, col + i, head, col, e + iw, tau + iw);
            else hipLaunchKernelGGL((reflector_kernel<T>), dim3(1), dim3(PT), 0, s, m, head, col, (int64_t)1, e + iw, tau + iw);
            hipError_t he = hipGetLastError();
            if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
            rc = symv('U', m, &one, A, lda, col, 1, &zero, w, 1, ws, wsb, stream);
            if (rc) return rc;
            if (k > 0) {
                rc = gemv(TC, m, k, &one, W + (iw + 1) * ldw, ldw, col, 1, &zero, small, 1, ws, wsb, stream);
                if (rc) return rc;
                rc = gemv('N', m, k, &minus, A + (i + 1) * lda, lda, small, 1, &one, w, 1, ws, wsb, stream);
                if (rc) return rc;
                rc = gemv(TC, m, k, &one, A + (i + 1) * lda, lda, col, 1, &zero, small, 1, ws, wsb, stream);
                if (rc) return rc;
                rc = gemv('N', m, k, &minus, W + (iw + 1) * ldw, ldw, small, 1, &one, w, 1, ws, wsb, stream);
                if (rc) return rc;
            }
            // w finished; row i-1 of W (slots iw..) and of V (columns i..) packed for column i-1
            if constexpr (CPLX)
                hipLaunchKernelGGL((finish_w_kernel_c<T, R>), dim3(1), dim3(PT), 0, s, m, tau + iw, col, w, W + (i - 1) + iw * ldw,
                                   ldw, A + (i - 1) + i * lda, lda, (int)(k + 1), wrow, vrow,
                                   i - 1 >= first ? A + (i - 1) + (i - 1) * lda : (T*)nullptr);
            else
                hipLaunchKernelGGL((finish_w_kernel<T>), dim3(1), dim3(PT), 0, s, m, tau + iw, col, w, W + (i - 1) + iw * ldw, ldw,
                                   A + (i - 1) + i * lda, lda, (int)(k + 1), wrow, vrow);
            he = hipGetLastError();
            if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
        }
        return KMV_OK;
    }
    for (int64_t i = 0; i < nb; ++i) {
        T* col = A + i + i * lda;               // A[i:, i]
        if (i > 0) {
            // column i catches up with the reflectors before it; x is row i of W, then row i of V (= of A),
            // both packed (and conjugated in the complex case) by the last kernel of column i-1
            rc = gemv('N', n - i, i, &minus, A + i, lda, wrow, 1, &one, col, 1, ws, wsb, stream);
            if (rc) return rc;
            rc = gemv('N', n - i, i, &minus, W + i, ldw, vrow, 1, &one, col, 1, ws, wsb, stream);
            if (rc) return rc;
        }
        if (i >= n - 1) {   // last column of the matrix: no reflector; its slots are defined all the same
            if constexpr (CPLX) hipLaunchKernelGGL((no_reflector_kernel_c<T, R>), dim3(1), dim3(1), 0, s, col, e + i, tau + i);
            else hipLaunchKernelGGL((no_reflector_kernel<T, T>), dim3(1), dim3(1), 0, s, e + i, tau + i);
            const hipError_t he = hipGetLastError();
            if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
            continue;
        }
        const int64_t m = n - i - 1;
        T* v = col + 1;                         // A[i+1:, i]
        T* w = W + (i + 1) + i * ldw;           // W[i+1:, i]
        T* small = W + i * ldw;                 // W[:i, i]: the i-vector of the corrections
        if constexpr (CPLX) hipLaunchKernelGGL((reflector_kernel_c<T, R>), dim3(1), dim3(PT), 0, s, m, col, v, v + 1, e + i, tau + i);
        else hipLaunchKernelGGL((reflector_kernel<T>), dim3(1), dim3(PT), 0, s, m, v, v + 1, (int64_t)1, e + i, tau + i);
        hipError_t he = hipGetLastError();
        if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
        rc = symv('L', m, &one, A + (i + 1) + (i + 1) * lda, lda, v, 1, &zero, w, 1, ws, wsb, stream);
        if (rc) return rc;
        if (i > 0) {
            rc = gemv(TC, m, i, &one, W + i + 1, ldw, v, 1, &zero, small, 1, ws, wsb, stream);
            if (rc) return rc;
            rc = gemv('N', m, i, &minus, A + i + 1, lda, small, 1, &one, w, 1, ws, wsb, stream);
            if (rc) return rc;
            rc = gemv(TC, m, i, &one, A + i + 1, lda, v, 1, &zero, small, 1, ws, wsb, stream);
            if (rc) return rc;
            rc = gemv('N', m, i, &minus, W + i + 1, ldw, small, 1, &one, w, 1, ws, wsb, stream);
            if (rc) return rc;
        }
        if constexpr (CPLX)
            hipLaunchKernelGGL((finish_w_kernel_c<T, R>), dim3(1), dim3(PT), 0, s, m, tau + i, v, w, W + (i + 1), ldw,
                               A + (i + 1), lda, (int)(i + 1), wrow, vrow,
                               i + 1 < nb ? A + (i + 1) + (i + 1) * lda : (T*)nullptr);
        else
            hipLaunchKernelGGL((finish_w_kernel<T>), dim3(1), dim3(PT), 0, s, m, tau + i, v, w, W + (i + 1), ldw,
                               A + (i + 1), lda, (int)(i + 1), wrow, vrow);
        he = hipGetLastError();
        if (he != hipSuccess) return KMV_ERR_HIP + (int)he;
    }
    return KMV_OK;
}

// bytes at the front of the workspace for the contiguous copy of the current row
template <class T> size_t row_bytes(int64_t n) { return (size_t)((n * sizeof(T) + 255) / 256) * 256; }

// complex panels: three conjugated copies of short strided rows (at most nb elements each)
template <class T> size_t short_rows_bytes(int64_t nb) {
    return Traits<T>::cplx ? (size_t)((3 * nb * sizeof(T) + 255) / 256) * 256 : 0;
}

// the row copy plus the largest workspace any product of the bidiagonal panel asks for
template <class T> size_t gebrd_workspace(int64_t m, int64_t n, int64_t nb) {
    if (m <= 0 || n <= 0 || nb <= 0) return 0;
    const int64_t mn = m < n ? m : n;
    if (nb > mn) nb = mn;
    const char p = Calls<T>::prec;
    size_t need = 0;
    if (m < n) {     // lower bidiagonal: rows first
        for (int64_t i = 0; i < nb; ++i) {
            const int64_t mi = m - i - 1, ni = n - i;
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', ni, i));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', i, ni));
            if (mi <= 0) continue;
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi, ni));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', ni, i));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi, i + 1));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', i, ni));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, ni - 1));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, i + 1));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', ni - 1, i));
            need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', i + 1, ni - 1));
        }
        return row_bytes<T>(n) + short_rows_bytes<T>(nb) + need;
    }
    for (int64_t i = 0; i < nb; ++i) {
        const int64_t mi = m - i, ni = n - i - 1;
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi, i));
        if (ni <= 0) continue;
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, ni));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, i));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', ni, i + 1));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', i, ni));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi - 1, ni));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', ni, i + 1));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi - 1, i + 1));
        need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', i, ni));
    }
    return row_bytes<T>(n) + short_rows_bytes<T>(nb) + need;
}

// Panel step of the bidiagonal reduction (m >= n: upper bidiagonal; m < n: lower bidiagonal, see the branch
// below): the published "labrd" step written
// from its definition on top of the GEMV entry points.  Per column two products with the whole trailing
// block (transposed from the left, plain from the right, the latter with a strided x: a row of A) and
// eleven with the tall or wide panels of vectors accumulated so far, two reflectors and two scalings by
// tau; everything on the device and on the caller's stream.  The row that becomes u_i is worked on in a
// contiguous copy (one strided gather before, one scatter after): a reflector along a row of stride lda took
// 36 us on average at n = 16384, and the three products that take u_i as x need no packing this way.
// Complex T: H_i = I - tauq v v^H is applied as H_i^H, G_i = I - taup u u^H from the right, the update is
// A - V Y^H - X U^H, so every transposed product is a conjugate-transposed one.  Row i of A stores u_i^H;
// the row is updated and reflected as its conjugate (the contiguous copy holds conj(row), then u_i), and
// the three short strided rows that enter products conjugated (row i of Y, of V and of X) are copied
// conjugated into the workspace first; d and e are real.
template <class T>
int gebrd_panel(int64_t m, int64_t n, int64_t nb, T* A, int64_t lda, typename Traits<T>::real* d,
                typename Traits<T>::real* e, T* tauq, T* taup, T* X, int64_t ldx, T* Y, int64_t ldy, void* ws,
                size_t wsb, void* stream) {
    using R = typename Traits<T>::real;
    constexpr bool CPLX = Traits<T>::cplx;
    if (m < 0) return -1;
    if (n < 0) return -2;
    if (nb < 0 || nb > (m < n ? m : n)) return -3;
    if (lda < (m > 1 ? m : 1)) return -5;
    if (ldx < (m > 1 ? m : 1)) return -11;
    if (ldy < (n > 1 ? n : 1)) return -13;
    if (m == 0 || n == 0 || nb == 0) return KMV_OK;
    if (!A || !d || !e || !tauq || !taup || !X || !Y) return KMV_ERR_NULL;
    if (!ws || wsb < gebrd_workspace<T>(m, n, nb) || ((uintptr_t)ws % 256) != 0) return KMV_ERR_WORKSPACE;
    T* urow = static_cast<T*>(ws);            // row i right of the diagonal, contiguous
    ws = static_cast<char*>(ws) + row_bytes<T>(n);
    wsb -= row_bytes<T>(n);
    T* yrow = static_cast<T*>(ws);            // complex only: conj of row i of Y, of V (= A), of X
    T* vrow = yrow + nb;
    T* xrow = vrow + nb;
    ws = static_cast<char*>(ws) + short_rows_bytes<T>(nb);
    wsb -= short_rows_bytes<T>(nb);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const T one = from_real<T>(1), zero = from_real<T>(0), minus = from_real<T>(-1);
    const char TR = CPLX ? 'C' : 'T';
    auto a_ = [&](int64_t i, int64_t j) { return A + i + j * lda; };
    auto x_ = [&](int64_t i, int64_t j) { return X + i + j * ldx; };
    auto y_ = [&](int64_t i, int64_t j) { return Y + i + j * ldy; };
    int rc = KMV_OK;
    hipError_t he = hipSuccess;
#define KMV_GEMV(...)                                          \
    do {                                                       \
        rc = Calls<T>::gemv(__VA_ARGS__, ws, wsb, stream);     \
        if (rc) return rc;                                     \
    } while (0)
#define KMV_LAUNCHED()                                         \
    do {                                                       \
        he = hipGetLastError();                                \
        if (he != hipSuccess) return KMV_ERR_HIP + (int)he;    \
    } while (0)
    // conjugated copy of `len` elements with stride `inc` (complex panels only)
    auto conj_row = [&](int64_t len, const T* src, int64_t inc, T* dst) {
        hipLaunchKernelGGL((strided_copy_kernel<T, true>), dim3((unsigned)ceil_div(len, (int64_t)256)), dim3(256), 0, s,
                           len, src, inc, dst, (int64_t)1);
    };
    auto reflector = [&](int64_t len, T* head, R* beta, T* tau) {
        if constexpr (CPLX)
            hipLaunchKernelGGL((reflector_kernel_c<T, R>), dim3(1), dim3(PT), 0, s, len, (T*)nullptr, head, head + 1, beta, tau);
        else
            hipLaunchKernelGGL((reflector_kernel<T>), dim3(1), dim3(PT), 0, s, len, head, head + 1, (int64_t)1, beta, tau);
    };
    if (m < n) {
        // More columns than rows: lower bidiagonal form, the roles of rows and columns exchanged.  Row i is
        // brought up to date and reflected first (in its contiguous, conjugated copy), x_i follows from the
        // trailing block; then column i below the diagonal, its reflector (the one at row i+1) and y_i.
        for (int64_t i = 0; i < nb; ++i) {
            const int64_t mi = m - i - 1, ni = n - i;       // rows below row i, columns from column i on
            const dim3 cgrid((unsigned)ceil_div(ni, (int64_t)256));
            hipLaunchKernelGGL((strided_copy_kernel<T, CPLX>), cgrid, dim3(256), 0, s, ni, a_(i, i), lda, urow, (int64_t)1);
            KMV_LAUNCHED();
            if (i > 0) {
                if constexpr (CPLX) {
                    conj_row(i, a_(i, 0), lda, vrow);
                    KMV_LAUNCHED();
                    conj_row(i, x_(i, 0), ldx, xrow);
                    KMV_LAUNCHED();
                    KMV_GEMV('N', ni, i, &minus, y_(i, 0), ldy, vrow, (int64_t)1, &one, urow, (int64_t)1);
                    KMV_GEMV('C', i, ni, &minus, a_(0, i), lda, xrow, (int64_t)1, &one, urow, (int64_t)1);
                } else {
                    KMV_GEMV('N', ni, i, &minus, y_(i, 0), ldy, a_(i, 0), lda, &one, urow, (int64_t)1);
                    KMV_GEMV('T', i, ni, &minus, a_(0, i), lda, x_(i, 0), ldx, &one, urow, (int64_t)1);
                }
            }
            reflector(ni, urow, d + i, taup + i);
            KMV_LAUNCHED();
            hipLaunchKernelGGL((strided_copy_kernel<T, CPLX>), cgrid, dim3(256), 0, s, ni, urow, (int64_t)1, a_(i, i), lda);
            KMV_LAUNCHED();
            if (mi <= 0) {     // last row of the matrix: no column reflector
                hipLaunchKernelGGL((no_reflector_kernel<R, T>), dim3(1), dim3(1), 0, s, e + i, tauq + i);
                KMV_LAUNCHED();
                continue;
            }
            // x = taup * (trailing block u - corrections)
            KMV_GEMV('N', mi, ni, &one, a_(i + 1, i), lda, urow, (int64_t)1, &zero, x_(i + 1, i), (int64_t)1);
            if (i > 0) {
                KMV_GEMV(TR, ni, i, &one, y_(i, 0), ldy, urow, (int64_t)1, &zero, x_(0, i), (int64_t)1);
                KMV_GEMV('N', mi, i, &minus, a_(i + 1, 0), lda, x_(0, i), (int64_t)1, &one, x_(i + 1, i), (int64_t)1);
                KMV_GEMV('N', i, ni, &one, a_(0, i), lda, urow, (int64_t)1, &zero, x_(0, i), (int64_t)1);
                KMV_GEMV('N', mi, i, &minus, x_(i + 1, 0), ldx, x_(0, i), (int64_t)1, &one, x_(i + 1, i), (int64_t)1);
            }
            hipLaunchKernelGGL((scale_kernel<T>), dim3((unsigned)ceil_div(mi, (int64_t)256)), dim3(256), 0, s, mi, taup + i,
                               x_(i + 1, i));
            KMV_LAUNCHED();
            // column i below the diagonal catches up (x_i just computed takes part) and gets its reflector
            if (i > 0) {
                if constexpr (CPLX) {
                    conj_row(i, y_(i, 0), ldy, yrow);
                    KMV_LAUNCHED();
                    KMV_GEMV('N', mi, i, &minus, a_(i + 1, 0), lda, yrow, (int64_t)1, &one, a_(i + 1, i), (int64_t)1);
                } else {
                    KMV_GEMV('N', mi, i, &minus, a_(i + 1, 0), lda, y_(i, 0), ldy, &one, a_(i + 1, i), (int64_t)1);
                }
            }
            KMV_GEMV('N', mi, i + 1, &minus, x_(i + 1, 0), ldx, a_(0, i), (int64_t)1, &one, a_(i + 1, i), (int64_t)1);
            reflector(mi, a_(i + 1, i), e + i, tauq + i);
            KMV_LAUNCHED();
            // y = tauq * (trailing block^H v - corrections)
            KMV_GEMV(TR, mi, ni - 1, &one, a_(i + 1, i + 1), lda, a_(i + 1, i), (int64_t)1, &zero, y_(i + 1, i), (int64_t)1);
            if (i > 0) {
                KMV_GEMV(TR, mi, i, &one, a_(i + 1, 0), lda, a_(i + 1, i), (int64_t)1, &zero, y_(0, i), (int64_t)1);
                KMV_GEMV('N', ni - 1, i, &minus, y_(i + 1, 0), ldy, y_(0, i), (int64_t)1, &one, y_(i + 1, i), (int64_t)1);
            }
            KMV_GEMV(TR, mi, i + 1, &one, x_(i + 1, 0), ldx, a_(i + 1, i), (int64_t)1, &zero, y_(0, i), (int64_t)1);
            KMV_GEMV(TR, i + 1, ni - 1, &minus, a_(0, i + 1), lda, y_(0, i), (int64_t)1, &one, y_(i + 1, i), (int64_t)1);
            hipLaunchKernelGGL((scale_kernel<T>), dim3((unsigned)ceil_div(ni - 1, (int64_t)256)), dim3(256), 0, s, ni - 1,
                               tauq + i, y_(i + 1, i));
            KMV_LAUNCHED();
        }
        return KMV_OK;
    }
    for (int64_t i = 0; i < nb; ++i) {
        const int64_t mi = m - i, ni = n - i - 1;
        if (i > 0) {   // column i catches up with the panels
            if constexpr (CPLX) {
                conj_row(i, y_(i, 0), ldy, yrow);
                KMV_LAUNCHED();
                KMV_GEMV('N', mi, i, &minus, a_(i, 0), lda, yrow, (int64_t)1, &one, a_(i, i), (int64_t)1);
            } else {
                KMV_GEMV('N', mi, i, &minus, a_(i, 0), lda, y_(i, 0), ldy, &one, a_(i, i), (int64_t)1);
            }
            KMV_GEMV('N', mi, i, &minus, x_(i, 0), ldx, a_(0, i), (int64_t)1, &one, a_(i, i), (int64_t)1);
        }
        reflector(mi, a_(i, i), d + i, tauq + i);
        KMV_LAUNCHED();
        if (ni <= 0) {     // last column of the matrix: no row reflector
            hipLaunchKernelGGL((no_reflector_kernel<R, T>), dim3(1), dim3(1), 0, s, e + i, taup + i);
            KMV_LAUNCHED();
            continue;
        }
        // y = tauq * (trailing block^H v - corrections)
        KMV_GEMV(TR, mi, ni, &one, a_(i, i + 1), lda, a_(i, i), (int64_t)1, &zero, y_(i + 1, i), (int64_t)1);
        if (i > 0) {
            KMV_GEMV(TR, mi, i, &one, a_(i, 0), lda, a_(i, i), (int64_t)1, &zero, y_(0, i), (int64_t)1);
            KMV_GEMV('N', ni, i, &minus, y_(i + 1, 0), ldy, y_(0, i), (int64_t)1, &one, y_(i + 1, i), (int64_t)1);
            KMV_GEMV(TR, mi, i, &one, x_(i, 0), ldx, a_(i, i), (int64_t)1, &zero, y_(0, i), (int64_t)1);
            KMV_GEMV(TR, i, ni, &minus, a_(0, i + 1), lda, y_(0, i), (int64_t)1, &one, y_(i + 1, i), (int64_t)1);
        }
        hipLaunchKernelGGL((scale_kernel<T>), dim3((unsigned)ceil_div(ni, (int64_t)256)), dim3(256), 0, s, ni, tauq + i,
                           y_(i + 1, i));
        KMV_LAUNCHED();
        // row i catches up and gets its reflector, in a contiguous copy that then goes back into the row
        const dim3 cgrid((unsigned)ceil_div(ni, (int64_t)256));
        hipLaunchKernelGGL((strided_copy_kernel<T, CPLX>), cgrid, dim3(256), 0, s, ni, a_(i, i + 1), lda, urow, (int64_t)1);
        KMV_LAUNCHED();
        if constexpr (CPLX) {
            conj_row(i + 1, a_(i, 0), lda, vrow);
            KMV_LAUNCHED();
            KMV_GEMV('N', ni, i + 1, &minus, y_(i + 1, 0), ldy, vrow, (int64_t)1, &one, urow, (int64_t)1);
            if (i > 0) {
                conj_row(i, x_(i, 0), ldx, xrow);
                KMV_LAUNCHED();
                KMV_GEMV('C', i, ni, &minus, a_(0, i + 1), lda, xrow, (int64_t)1, &one, urow, (int64_t)1);
            }
        } else {
            KMV_GEMV('N', ni, i + 1, &minus, y_(i + 1, 0), ldy, a_(i, 0), lda, &one, urow, (int64_t)1);
            if (i > 0) KMV_GEMV('T', i, ni, &minus, a_(0, i + 1), lda, x_(i, 0), ldx, &one, urow, (int64_t)1);
        }
        reflector(ni, urow, e + i, taup + i);
        KMV_LAUNCHED();
        hipLaunchKernelGGL((strided_copy_kernel<T, CPLX>), cgrid, dim3(256), 0, s, ni, urow, (int64_t)1, a_(i, i + 1), lda);
        KMV_LAUNCHED();
        // x = taup * (trailing block u - corrections)
        KMV_GEMV('N', mi - 1, ni, &one, a_(i + 1, i + 1), lda, urow, (int64_t)1, &zero, x_(i + 1, i), (int64_t)1);
        KMV_GEMV(TR, ni, i + 1, &one, y_(i + 1, 0), ldy, urow, (int64_t)1, &zero, x_(0, i), (int64_t)1);
        KMV_GEMV('N', mi - 1, i + 1, &minus, a_(i + 1, 0), lda, x_(0, i), (int64_t)1, &one, x_(i + 1, i), (int64_t)1);
        if (i > 0) {
            KMV_GEMV('N', i, ni, &one, a_(0, i + 1), lda, urow, (int64_t)1, &zero, x_(0, i), (int64_t)1);
            KMV_GEMV('N', mi - 1, i, &minus, x_(i + 1, 0), ldx, x_(0, i), (int64_t)1, &one, x_(i + 1, i), (int64_t)1);
        }
        hipLaunchKernelGGL((scale_kernel<T>), dim3((unsigned)ceil_div(mi - 1, (int64_t)256)), dim3(256), 0, s, mi - 1,
                           taup + i, x_(i + 1, i));
        KMV_LAUNCHED();
    }
#undef KMV_GEMV
#undef KMV_LAUNCHED
    return KMV_OK;
}

}  // namespace
}  // namespace kmv

extern "C" {

int kmv_ssytrd_panel(char uplo, int64_t n, int64_t nb, float* A, int64_t lda, float* e, float* tau, float* W,
                     int64_t ldw, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::sytrd_panel<float>(uplo, n, nb, A, lda, e, tau, W, ldw, workspace, workspace_bytes, stream);
}
int kmv_dsytrd_panel(char uplo, int64_t n, int64_t nb, double* A, int64_t lda, double* e, double* tau, double* W,
                     int64_t ldw, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::sytrd_panel<double>(uplo, n, nb, A, lda, e, tau, W, ldw, workspace, workspace_bytes, stream);
}
int kmv_sgebrd_panel(int64_t m, int64_t n, int64_t nb, float* A, int64_t lda, float* d, float* e, float* tauq, float* taup,
                     float* X, int64_t ldx, float* Y, int64_t ldy, void* workspace, size_t workspace_bytes,
                     void* stream) {
    return kmv::gebrd_panel<float>(m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy, workspace, workspace_bytes, stream);
}
int kmv_dgebrd_panel(int64_t m, int64_t n, int64_t nb, double* A, int64_t lda, double* d, double* e, double* tauq,
                     double* taup, double* X, int64_t ldx, double* Y, int64_t ldy, void* workspace,
                     size_t workspace_bytes, void* stream) {
    return kmv::gebrd_panel<double>(m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy, workspace, workspace_bytes, stream);
}
int kmv_cgebrd_panel(int64_t m, int64_t n, int64_t nb, kmv_complex64* A, int64_t lda, float* d, float* e,
                     kmv_complex64* tauq, kmv_complex64* taup, kmv_complex64* X, int64_t ldx, kmv_complex64* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::gebrd_panel<kmv::cf32>(m, n, nb, (kmv::cf32*)A, lda, d, e, (kmv::cf32*)tauq, (kmv::cf32*)taup, (kmv::cf32*)X,
                                       ldx, (kmv::cf32*)Y, ldy, workspace, workspace_bytes, stream);
}
int kmv_zgebrd_panel(int64_t m, int64_t n, int64_t nb, kmv_complex128* A, int64_t lda, double* d, double* e,
                     kmv_complex128* tauq, kmv_complex128* taup, kmv_complex128* X, int64_t ldx, kmv_complex128* Y,
                     int64_t ldy, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::gebrd_panel<kmv::cf64>(m, n, nb, (kmv::cf64*)A, lda, d, e, (kmv::cf64*)tauq, (kmv::cf64*)taup, (kmv::cf64*)X,
                                       ldx, (kmv::cf64*)Y, ldy, workspace, workspace_bytes, stream);
}
size_t kmv_gebrd_panel_workspace_bytes(char prec, int64_t m, int64_t n, int64_t nb) {
    if (prec == 's') return kmv::gebrd_workspace<float>(m, n, nb);
    if (prec == 'd') return kmv::gebrd_workspace<double>(m, n, nb);
    if (prec == 'c') return kmv::gebrd_workspace<kmv::cf32>(m, n, nb);
    if (prec == 'z') return kmv::gebrd_workspace<kmv::cf64>(m, n, nb);
    return 0;
}
int kmv_chetrd_panel(char uplo, int64_t n, int64_t nb, kmv_complex64* A, int64_t lda, float* e, kmv_complex64* tau,
                     kmv_complex64* W, int64_t ldw, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::sytrd_panel<kmv::cf32>(uplo, n, nb, (kmv::cf32*)A, lda, e, (kmv::cf32*)tau, (kmv::cf32*)W, ldw, workspace,
                                       workspace_bytes, stream);
}
int kmv_zhetrd_panel(char uplo, int64_t n, int64_t nb, kmv_complex128* A, int64_t lda, double* e, kmv_complex128* tau,
                     kmv_complex128* W, int64_t ldw, void* workspace, size_t workspace_bytes, void* stream) {
    return kmv::sytrd_panel<kmv::cf64>(uplo, n, nb, (kmv::cf64*)A, lda, e, (kmv::cf64*)tau, (kmv::cf64*)W, ldw, workspace,
                                       workspace_bytes, stream);
}
size_t kmv_sytrd_panel_workspace_bytes(char prec, int64_t n, int64_t nb) {
    if (prec == 's') return kmv::panel_workspace<float>(n, nb);
    if (prec == 'd') return kmv::panel_workspace<double>(n, nb);
    if (prec == 'c') return kmv::panel_workspace<kmv::cf32>(n, nb);
    if (prec == 'z') return kmv::panel_workspace<kmv::cf64>(n, nb);
    return 0;
}

}  // extern "C"
