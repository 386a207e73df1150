// Panel steps of the two-sided reductions - symmetric tridiagonal (below) and
// bidiagonal (further down) (paper, Section 10: the two-sided reductions spend their
// memory-bound time in exactly these products - SYMV on the trailing block once
// per column, GEMV on the tall panels of accumulated reflectors - and always on
// sub-blocks that start at arbitrary offsets inside the matrix, Section 6.6).
//
// The tridiagonal step is the published "latrd" panel of the blocked Householder
// tridiagonalisation, lower storage, written from its definition:
//   column i:  a  = A[i:,i] - V[i:,:i] W[i,:i]^T - W[i:,:i] V[i,:i]^T
//              reflector (beta, tau, v) that annihilates a[2:]
//              w  = A[i+1:,i+1:] v                                            (SYMV, trailing block)
//              w -= V[i+1:,:i] (W[i+1:,:i]^T v) + W[i+1:,:i] (V[i+1:,:i]^T v)
//              w  = tau w;  w -= (tau/2)(w.v) v
// The symmetric product, which holds 97% of the bytes, goes through the public entry point (the same
// argument checks, planner and kernels as any other caller's).  The products with the two tall panels
// (at most nb columns wide) and the vector steps between them are three kernels of this file per column:
// as six GEMV launches, their second-stage sums and two vector kernels they were eleven launches of 4-11 us
// each, a quarter of the panel's time for 3% of its bytes.
// Upper storage runs the mirror image (last nb columns, from the right), complex types the Hermitian form
// (conjugated transposes, real e).  The bidiagonal step further down follows the same plan in all four
// precisions: the two products with the trailing block per column go through the public GEMV entry points,
// everything else of a column is four launches of two kernels of this file (a panel wider than 256 columns
// runs the step built from GEMV calls alone, about twenty launches per column).
// Everything stays on the device and on the caller's stream: tau, the norms and the inner
// products never visit the host, so a whole panel is one uninterrupted sequence of
// launches (and can be captured in a graph).
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

// ---- the reflector kernel for complex vectors (C = cf32 / cf64, R its real type) ----
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

// ---- The tridiagonal panel's own kernels ------------------------------------------------------------------
// Everything of a column except the symmetric product runs in three launches over row chunks, each launch
// ending where the next step needs a sum over all rows; the sums travel as one partial per workgroup and are
// added up in workgroup order by every consumer, so the result does not depend on scheduling:
//   panel_reflector_kernel  norm of the column from the partials -> beta, tau; scales the reflector's tail;
//                           partial products  W^H v, V^H v  of its chunk with the panels of earlier columns
//   (SYMV / HEMV            w = A22 v, the public entry point)
//   panel_correct_kernel    W^H v, V^H v from the partials;  w <- tau (w - V (W^H v) - W (V^H v)),  partial w^H v
//   panel_column_kernel     w <- w - (tau/2)(w^H v) v;  the next column catches up with all reflectors so far,
//                           a <- a - V conj(W[d,:]) - W conj(V[d,:])  (d = its diagonal row), its diagonal
//                           entry made real, partial sums of squares of its entries beyond the subdiagonal
// The two tall panels V (in A) and W are read three times per column instead of being the operands of six
// matrix-vector launches with two vector kernels in between.  All three are bound by the latency of the panel
// loads, so their shapes aim at many loads in flight: the correct and column kernels run one workgroup per 64
// rows (up to FG_MAX workgroups), its four waves taking every fourth column of the panels and adding their
// parts through LDS; the reflector kernel, whose output is 2k sums PER WORKGROUP that every workgroup of the
// next launch has to add up, runs at most DG_MAX workgroups of 16 waves over 256 rows, the waves again
// splitting the columns.
// Row space: the kernels of one column see the rows of its reflector vector v (m rows) and everything that is
// row-aligned with it; the next column `a` has the same rows, its diagonal entry in row d = 0 (lower storage,
// HEAD_FIRST) or d = m-1 (upper), its subdiagonal entry next to it.
constexpr int FT = 256;        // correct / column kernels: threads,
constexpr int FR = WAVE;       //   rows per pass (one per lane),
constexpr int FG_MAX = 256;    //   most workgroups
constexpr int DT = 1024;       // reflector kernel: threads,
constexpr int DR = 256;        //   rows per pass,
constexpr int DG_MAX = 64;     //   most workgroups
constexpr int NB_MAX = 1024;
// reflector kernels: panel columns a wave works on at a time (16 waves per workgroup leave 128 registers per lane: two
// columns for 16-byte elements, four otherwise),
template <class T> constexpr int rc_of() { return sizeof(T) == 16 ? 2 : 4; }
constexpr int RQ = DR / WAVE; //   rows per lane in the first DR rows of a chunk (what is fetched ahead)
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
inline int64_t thin_rows(int64_t m) { return FR * ceil_div(m > 0 ? m : 1, (int64_t)FR * FG_MAX); }
inline unsigned thin_chunks(int64_t m) { return (unsigned)ceil_div(m > 0 ? m : 1, thin_rows(m)); }
inline int64_t fat_rows(int64_t m) { return DR * ceil_div(m > 0 ? m : 1, (int64_t)DR * DG_MAX); }
inline unsigned fat_chunks(int64_t m) { return (unsigned)ceil_div(m > 0 ? m : 1, fat_rows(m)); }

template <class T> __device__ __forceinline__ T conj_of(T a) {
    if constexpr (Traits<T>::cplx) return T{a.re, -a.im};
    else return a;
}
template <class T> __device__ __forceinline__ T from_one() {
    if constexpr (Traits<T>::cplx) return T{1, 0};
    else return T(1);
}
template <class T> __device__ __forceinline__ T neg_of(T a) {
    if constexpr (Traits<T>::cplx) return T{-a.re, -a.im};
    else return -a;
}
template <class T> __device__ __forceinline__ typename Traits<T>::real abs2_of(T a) {
    if constexpr (Traits<T>::cplx) return a.re * a.re + a.im * a.im;
    else return a * a;
}
template <class T> __device__ __forceinline__ T half_neg_of(T a) {      // -a/2
    if constexpr (Traits<T>::cplx) return T{(typename Traits<T>::real)(-0.5) * a.re, (typename Traits<T>::real)(-0.5) * a.im};
    else return T(-0.5) * a;
}
// sum over the NT threads of the workgroup in a fixed order (lanes by DPP, then the waves in wave order);
// red holds one slot per wave
template <int NT, class T> __device__ __forceinline__ T group_sum(T v, T* red) {
    const int lane = threadIdx.x % WAVE, w = threadIdx.x / WAVE;
    const T s = wave_sum(v);
    __syncthreads();
    if (lane == 0) red[w] = s;
    __syncthreads();
    T tot = red[0];
#pragma unroll
    for (int q = 1; q < NT / WAVE; ++q) tot = add_of(tot, red[q]);
    return tot;
}

// s1[0 .. kp), s2[0 .. kk - kp) <- the column sums of the gd partial rows of `dots` (kk entries each), for a workgroup
// of FT threads: wave w adds the rows g = w, w + 4, ... of 64 columns at a time (all its loads in flight at once), the
// four waves' sums are added in wave order through tmp - a fixed order, whatever the scheduling.
template <class T>
__device__ __forceinline__ void sum_partial_rows(const T* __restrict__ dots, int gd, int kk, int kp, T* s1, T* s2, T (*tmp)[FR]) {
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    for (int jb = 0; jb < kk; jb += WAVE) {
        const int j = jb + lane;
        T s = zero_of<T>();
        if (j < kk) {
#pragma unroll 16
            for (int g = wv; g < gd; g += FT / WAVE) s = add_of(s, dots[(int64_t)g * kk + j]);
        }
        tmp[wv][lane] = s;
        __syncthreads();
        if (wv == 0 && j < kk) {
            T tot = tmp[0][lane];
#pragma unroll
            for (int q = 1; q < FT / WAVE; ++q) tot = add_of(tot, tmp[q][lane]);
            if (j < kp) s1[j] = tot;
            else s2[j - kp] = tot;
        }
        __syncthreads();
    }
}

// The update kernel of the bidiagonal panel starts with a prologue (sums of partials, coefficients, barriers) that
// the panel entries themselves do not depend on, and a barrier keeps the compiler from moving loads across it: so the
// first PF columns a wave takes of each panel are fetched by hand before the prologue, for the lane's row of the
// workgroup's first pass (its only one up to 16384 rows), and used in the same order as the loop would have used
// them (10.8 -> 8.9 us per launch at 16384 rows, nb = 64).  The same in the correct and column kernels of the
// tridiagonal panel, which follow the symmetric product's final pass, measured slower (6.1 -> 10.2 us) and is not done.
constexpr int PF = 16;
template <class T>
__device__ __forceinline__ void fetch_ahead(T (&pre)[PF], const T* __restrict__ P, int64_t ld, int k, int64_t r, bool in) {
    const int wv = threadIdx.x / WAVE;
#pragma unroll
    for (int u = 0; u < PF; ++u) {
        const int j = wv + u * (FT / WAVE);
        pre[u] = in && j < k ? P[r + j * ld] : zero_of<T>();
    }
}

template <class T, bool HEAD_FIRST>
__global__ __launch_bounds__(FT) void panel_column_kernel(int64_t m, int64_t rpw, int k, const T* __restrict__ Vp, int64_t ldv,
                                                          const T* __restrict__ Wp, int64_t ldw, const T* __restrict__ v, T* w,
                                                          const T* tau, const T* wdot, int gw, const T* whead, T* a,
                                                          typename Traits<T>::real* normpart, T* alpha_out, int finalize,
                                                          int has_next) {
    using R = typename Traits<T>::real;
    __shared__ T wr[NB_MAX + 1], vr[NB_MAX + 1];
    __shared__ T part[FT / WAVE][FR];
    __shared__ T red[FT / WAVE];
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    const int64_t rd = HEAD_FIRST ? 0 : m - 1, ra = HEAD_FIRST ? 1 : m - 2;
    const bool update = finalize && has_next;
    const int64_t r0 = (int64_t)blockIdx.x * rpw;
    const int64_t r1 = r0 + rpw < m ? r0 + rpw : m;
    T c = zero_of<T>();
    if (finalize) {
        T d = zero_of<T>();
        for (int g = threadIdx.x; g < gw; g += FT) d = add_of(d, wdot[g]);
        c = mul_of(half_neg_of(*tau), group_sum<FT>(d, red));
        if (has_next) {
            for (int j = threadIdx.x; j < k; j += FT) {
                wr[j] = conj_of(Wp[rd + j * ldw]);
                vr[j] = conj_of(Vp[rd + j * ldv]);
            }
            if (threadIdx.x == 0) {
                T wf = *whead;
                fma_acc(wf, c, v[rd]);
                wr[k] = conj_of(wf);
                vr[k] = conj_of(v[rd]);
            }
            __syncthreads();
        }
    }
    R nrm = 0;
    for (int64_t rb = r0; rb < r1; rb += FR) {
        const int64_t r = rb + lane;
        const bool in = r < r1;
        if (update) {
            T sub = zero_of<T>();
            if (in) {
#pragma unroll 8
                for (int j = wv; j < k; j += FT / WAVE) {
                    fma_acc(sub, Vp[r + j * ldv], wr[j]);
                    fma_acc(sub, Wp[r + j * ldw], vr[j]);
                }
            }
            part[wv][lane] = sub;
            __syncthreads();
        }
        if (wv == 0 && in) {
            T vv = zero_of<T>(), wf = zero_of<T>();
            if (finalize) {
                vv = v[r];
                wf = w[r];
                fma_acc(wf, c, vv);
                w[r] = wf;
            }
            if (has_next) {
                T acc = a[r];
                if (finalize) {
                    T sub = part[0][lane];
#pragma unroll
                    for (int q = 1; q < FT / WAVE; ++q) sub = add_of(sub, part[q][lane]);
                    fma_acc(sub, vv, wr[k]);
                    fma_acc(sub, wf, vr[k]);
                    acc = add_of(acc, neg_of(sub));
                }
                if (r == rd) acc = real_part_only(acc);
                a[r] = acc;
                if (r == ra) *alpha_out = acc;
                if (r != rd && r != ra) nrm += abs2_of(acc);
            }
        }
        if (update) __syncthreads();     // part is written again in the next pass
    }
    if (has_next && wv == 0) {
        nrm = wave_sum(nrm);
        if (lane == 0) normpart[blockIdx.x] = nrm;
    }
}

// Reflector of the column `a` (m rows, diagonal entry in row rd, alpha next to it, x the rest): beta = -sign(Re alpha)
// ||(alpha, x)||, tau = (beta - alpha) / beta, x <- x / (alpha - beta), a[ra] = 1; x = 0 (and a real alpha) gives
// tau = 0, beta = alpha.  alpha and ||x||^2 come from the launch before (every workgroup overwrites its part of
// the column, so none may read another's).  Then the chunk's share of  W^H v  and  V^H v  for the kp columns of
// the panels: dots[g][j] and dots[g][kp + j].
template <class T, bool HEAD_FIRST>
__global__ __launch_bounds__(DT) void panel_reflector_kernel(int64_t m, int64_t rpw, int kp, const T* __restrict__ Vp, int64_t ldv,
                                                             const T* __restrict__ Wp, int64_t ldw, T* a,
                                                             const typename Traits<T>::real* normpart, int gn, const T* alpha_in,
                                                             typename Traits<T>::real* e, T* tau, T* dots) {
    using R = typename Traits<T>::real;
    constexpr int RC = rc_of<T>();
    __shared__ R red[DT / WAVE];
    __shared__ T xs[DT];       // the finished vector, first DT rows of the chunk (all of it up to 65536 rows)
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    const int64_t rd = HEAD_FIRST ? 0 : m - 1, ra = HEAD_FIRST ? 1 : m - 2;
    const int64_t r0 = (int64_t)blockIdx.x * rpw;
    const int64_t r1 = r0 + rpw < m ? r0 + rpw : m;
    // the panel entries of the wave's first group of columns do not depend on the norm: fetched ahead of it
    T pw[RC / 2][RQ], pv[RC / 2][RQ];
#pragma unroll
    for (int c = 0; c < RC / 2; ++c) {
        const int j = wv + c * (DT / WAVE);
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            const int64_t r = r0 + lane + q * WAVE;
            const bool in = j < kp && r < r1;
            pw[c][q] = in ? Wp[r + j * ldw] : zero_of<T>();
            pv[c][q] = in ? Vp[r + j * ldv] : zero_of<T>();
        }
    }
    R x2 = 0;
    for (int g = threadIdx.x; g < gn; g += DT) x2 += normpart[g];
    const R xn2 = group_sum<DT>(x2, red);
    const T alpha = *alpha_in;
    R beta, are, aim = 0;
    if constexpr (Traits<T>::cplx) { are = alpha.re; aim = alpha.im; }
    else are = alpha;
    beta = are;
    T t = zero_of<T>(), scale = zero_of<T>();
    const bool have = xn2 != 0 || aim != 0;
    if (have) {
        beta = -copysign(sqrt(are * are + aim * aim + xn2), are);
        const R dr = are - beta, den = dr * dr + aim * aim;      // 1 / (alpha - beta)
        if constexpr (Traits<T>::cplx) {
            t = T{(beta - are) / beta, -aim / beta};
            scale = T{dr / den, -aim / den};
        } else {
            t = (beta - are) / beta;
            scale = R(1) / dr;
        }
    }
    for (int64_t r = r0 + threadIdx.x; r < r1; r += DT) {
        T x = zero_of<T>();          // the diagonal row is not part of v
        if (r == ra) {
            x = from_one<T>();
            a[r] = x;
        } else if (r != rd) {
            x = a[r];
            if (have) {
                x = mul_of(x, scale);
                a[r] = x;
            }
        }
        if (r - r0 < DT) xs[r - r0] = x;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *e = beta;
        *tau = t;
    }
    if (kp == 0) return;
    __syncthreads();     // the chunk of v is in place for all waves of the workgroup
    // a wave takes RC / 2 columns of each panel at a time, so that their loads are in flight together (a column past
    // the end repeats the wave's first one and is not stored)
    for (int jb = wv; jb < kp; jb += (RC / 2) * (DT / WAVE)) {
        const T *cw[RC / 2], *cv[RC / 2];
        T aw[RC / 2], av[RC / 2];
#pragma unroll
        for (int c = 0; c < RC / 2; ++c) {
            const int j = jb + c * (DT / WAVE) < kp ? jb + c * (DT / WAVE) : jb;
            cw[c] = Wp + j * ldw;
            cv[c] = Vp + j * ldv;
            aw[c] = av[c] = zero_of<T>();
        }
        int64_t r = r0 + lane;
        if (jb == wv) {      // the group fetched ahead
#pragma unroll
            for (int q = 0; q < RQ; ++q, r += WAVE) {
                if (r < r1) {
                    const T x = xs[r - r0];
#pragma unroll
                    for (int c = 0; c < RC / 2; ++c) {
                        fma_acc_conj(aw[c], pw[c][q], x);
                        fma_acc_conj(av[c], pv[c][q], x);
                    }
                }
            }
        }
#pragma unroll 4
        for (; r < r1; r += WAVE) {
            const T x = r - r0 < DT ? xs[r - r0] : (r == rd ? zero_of<T>() : a[r]);
#pragma unroll
            for (int c = 0; c < RC / 2; ++c) {
                fma_acc_conj(aw[c], cw[c][r], x);
                fma_acc_conj(av[c], cv[c][r], x);
            }
        }
#pragma unroll
        for (int c = 0; c < RC / 2; ++c) {
            const T sw = wave_sum(aw[c]), sv = wave_sum(av[c]);
            const int j = jb + c * (DT / WAVE);
            if (lane == 0 && j < kp) {
                dots[(int64_t)blockIdx.x * 2 * kp + j] = sw;
                dots[(int64_t)blockIdx.x * 2 * kp + kp + j] = sv;
            }
        }
    }
}

// w <- tau (w - V s1 - W s2) with s1 = W^H v, s2 = V^H v summed from the gd partial rows of `dots`; the chunk's
// share of w^H v goes to wdot[g], the entry of w in row rd (the next column's diagonal row) to *whead as well:
// the next launch rewrites w, and all its workgroups need that one entry as it is now.
template <class T>
__global__ __launch_bounds__(FT) void panel_correct_kernel(int64_t m, int64_t rpw, int k, const T* __restrict__ Vp, int64_t ldv,
                                                           const T* __restrict__ Wp, int64_t ldw, const T* __restrict__ v, T* w,
                                                           const T* tau, const T* __restrict__ dots, int gd, int64_t rd, T* wdot,
                                                           T* whead) {
    __shared__ T s1[NB_MAX], s2[NB_MAX];
    __shared__ T part[FT / WAVE][FR];
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    const int64_t r0 = (int64_t)blockIdx.x * rpw;
    const int64_t r1 = r0 + rpw < m ? r0 + rpw : m;
    sum_partial_rows(dots, gd, 2 * k, k, s1, s2, part);
    const T t = *tau;
    T dot = zero_of<T>();
    for (int64_t rb = r0; rb < r1; rb += FR) {
        const int64_t r = rb + lane;
        const bool in = r < r1;
        T sub = zero_of<T>();
        if (in) {
#pragma unroll 8
            for (int j = wv; j < k; j += FT / WAVE) {
                fma_acc(sub, Vp[r + j * ldv], s1[j]);
                fma_acc(sub, Wp[r + j * ldw], s2[j]);
            }
        }
        part[wv][lane] = sub;
        __syncthreads();
        if (wv == 0 && in) {
            T tot = part[0][lane];
#pragma unroll
            for (int q = 1; q < FT / WAVE; ++q) tot = add_of(tot, part[q][lane]);
            const T wn = mul_of(t, add_of(w[r], neg_of(tot)));
            w[r] = wn;
            if (r == rd) *whead = wn;
            fma_acc_conj(dot, wn, v[r]);
        }
        __syncthreads();     // part is written again in the next pass
    }
    if (wv == 0) {
        dot = wave_sum(dot);
        if (lane == 0) wdot[blockIdx.x] = dot;
    }
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

// ---- The bidiagonal panel's own kernels -------------------------------------------------------------------
// A column of the bidiagonal step has two halves of the same shape, one along the rows of the matrix (the
// column reflector v_i, then x_i) and one along its columns (the row reflector u_i, then y_i).  Each half is a
// long vector index r and two tall panels that are contiguous in r:
//     along the rows:     V = A[:, :i] (the column reflectors) and X
//     along the columns:  Y and U, where U[j][k] = u_k[j] is a contiguous copy of the row reflectors kept in the
//                         workspace (row k of A holds u_k^H with stride lda, which no wave can read coalesced)
// and runs as  update -> reflector -> product with the trailing block (the public GEMV entry point) -> the
// other half's update, ...: two launches of this file per half, four per column, where the step built from
// GEMV calls took about twenty.
//   bd_update_kernel      finishes the vector z the product before it left behind,
//                             z <- tau (z - P s1 - Q s2),   s1 = P^H w, s2 = Q^H w summed from the partials of the
//                             reflector kernel before (w = the reflector the product was formed with),
//                         and brings the next vector to reflect up to date with all reflectors so far,
//                             t <- t - P c1 - Q c2 - z cz   (c1, c2, cz: the entries of the other half's panels
//                             in the row or column of t, conjugated as the update A - V Y^H - X U^H asks),
//                         reading both panels once for the two sums; t is taken from a strided, conjugated
//                         row of A (GATHER) or updated in place; its first entry goes to *alpha_out, the
//                         partial sums of squares of the others to normpart (one per workgroup)
//   bd_reflector_kernel   beta, tau and the scaling from alpha and the partial norms; scales the vector in
//                         place (first entry = 1), optionally scatters its conjugate into the row of A, and
//                         leaves the partial products P^H w, Q^H w of its row chunk in `dots`
// Partial sums are added in workgroup order by every consumer, so results do not depend on scheduling.
constexpr int BD_NB = 256;     // widest panel the two kernels hold coefficients for; wider panels take the GEMV-built step

template <class T, bool GATHER>
__global__ __launch_bounds__(FT) void bd_update_kernel(int64_t len, int64_t rpw, int kp, const T* __restrict__ P, int64_t ldp, int kq,
                                                       const T* __restrict__ Q, int64_t ldq, T* z, const T* tau,
                                                       const T* __restrict__ dots, int gd, const T* c1src, int64_t c1inc,
                                                       const T* c2src, int64_t c2inc, int conj2, const T* czsrc, const T* src,
                                                       int64_t sinc, T* dst, typename Traits<T>::real* normpart, T* alpha_out,
                                                       int fin, int has_next) {
    using R = typename Traits<T>::real;
    __shared__ T s1[BD_NB], s2[BD_NB], c1[BD_NB], c2[BD_NB];
    __shared__ T partf[FT / WAVE][FR], partu[FT / WAVE][FR];
    __shared__ T czs;
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    const bool update = fin && has_next;
    const int64_t r0 = (int64_t)blockIdx.x * rpw;
    const int64_t r1 = r0 + rpw < len ? r0 + rpw : len;
    T pp[PF], pq[PF];
    fetch_ahead(pp, P, ldp, kp, r0 + lane, fin && r0 + lane < r1);
    fetch_ahead(pq, Q, ldq, kq, r0 + lane, fin && r0 + lane < r1);
    if (fin) {
        sum_partial_rows(dots, gd, kp + kq, kp, s1, s2, partf);
        if (has_next) {
            for (int j = threadIdx.x; j < kp; j += FT) c1[j] = conj_of(c1src[j * c1inc]);
            for (int j = threadIdx.x; j < kq; j += FT) c2[j] = conj2 ? conj_of(c2src[j * c2inc]) : c2src[j * c2inc];
            if (threadIdx.x == 0) czs = conj2 ? conj_of(*czsrc) : *czsrc;
        }
        __syncthreads();
    }
    const T t = fin ? *tau : zero_of<T>();
    const T cz = update ? czs : zero_of<T>();
    R nrm = 0;
    for (int64_t rb = r0; rb < r1; rb += FR) {
        const int64_t r = rb + lane;
        const bool in = r < r1;
        if (fin) {
            T sf = zero_of<T>(), su = zero_of<T>();
            if (in) {
                int j0 = wv;
                if (rb == r0) {
#pragma unroll
                    for (int u = 0; u < PF; ++u) {
                        const int j = wv + u * (FT / WAVE);
                        if (j < kp) {
                            fma_acc(sf, pp[u], s1[j]);
                            if (update) fma_acc(su, pp[u], c1[j]);
                        }
                    }
#pragma unroll
                    for (int u = 0; u < PF; ++u) {
                        const int j = wv + u * (FT / WAVE);
                        if (j < kq) {
                            fma_acc(sf, pq[u], s2[j]);
                            if (update) fma_acc(su, pq[u], c2[j]);
                        }
                    }
                    j0 = wv + PF * (FT / WAVE);
                }
#pragma unroll 16
                for (int j = j0; j < kp; j += FT / WAVE) {
                    const T p = P[r + j * ldp];
                    fma_acc(sf, p, s1[j]);
                    if (update) fma_acc(su, p, c1[j]);
                }
#pragma unroll 16
                for (int j = j0; j < kq; j += FT / WAVE) {
                    const T q = Q[r + j * ldq];
                    fma_acc(sf, q, s2[j]);
                    if (update) fma_acc(su, q, c2[j]);
                }
            }
            partf[wv][lane] = sf;
            partu[wv][lane] = su;
            __syncthreads();
        }
        if (wv == 0 && in) {
            T zf = zero_of<T>();
            if (fin) {
                T tot = partf[0][lane];
#pragma unroll
                for (int q = 1; q < FT / WAVE; ++q) tot = add_of(tot, partf[q][lane]);
                zf = mul_of(t, add_of(z[r], neg_of(tot)));
                z[r] = zf;
            }
            if (has_next) {
                T acc = src[r * sinc];
                if constexpr (GATHER) acc = conj_of(acc);
                if (fin) {
                    T sub = partu[0][lane];
#pragma unroll
                    for (int q = 1; q < FT / WAVE; ++q) sub = add_of(sub, partu[q][lane]);
                    fma_acc(sub, zf, cz);
                    acc = add_of(acc, neg_of(sub));
                }
                dst[r] = acc;
                if (r == 0) *alpha_out = acc;
                else nrm += abs2_of(acc);
            }
        }
        if (fin) __syncthreads();     // the part arrays are written again in the next pass
    }
    if (has_next && wv == 0) {
        nrm = wave_sum(nrm);
        if (lane == 0) normpart[blockIdx.x] = nrm;
    }
}

// Reflector of the vector a (len entries, alpha = a[0], x the rest), alpha and ||x||^2 from the update kernel
// before: beta = -sign(Re alpha) ||(alpha, x)||, tau = (beta - alpha) / beta, x <- x / (alpha - beta), a[0] = 1;
// x = 0 (and a real alpha) gives tau = 0, beta = alpha.  With `scat` the conjugate of the finished vector goes to
// scat[r * scinc] as well (the row of A).  Then the chunk's share of P^H a (kp sums) and Q^H a (kq sums):
// dots[g][0 .. kp) and dots[g][kp .. kp + kq).
template <class T>
__global__ __launch_bounds__(DT) void bd_reflector_kernel(int64_t len, int64_t rpw, int kp, const T* __restrict__ P, int64_t ldp, int kq,
                                                          const T* __restrict__ Q, int64_t ldq, T* a,
                                                          const typename Traits<T>::real* normpart, int gn, const T* alpha_in,
                                                          typename Traits<T>::real* e, T* tau, T* scat, int64_t scinc, T* dots) {
    using R = typename Traits<T>::real;
    constexpr int RC = rc_of<T>();
    __shared__ R red[DT / WAVE];
    __shared__ T xs[DT];       // the finished vector, first DT rows of the chunk (all of it up to 65536 rows)
    const int lane = threadIdx.x % WAVE, wv = threadIdx.x / WAVE;
    const int kk = kp + kq;
    const int64_t r0 = (int64_t)blockIdx.x * rpw;
    const int64_t r1 = r0 + rpw < len ? r0 + rpw : len;
    // the panel entries of the wave's first group of columns do not depend on the norm: fetched ahead of it
    T pc[RC][RQ];
#pragma unroll
    for (int c = 0; c < RC; ++c) {
        const int j = wv + c * (DT / WAVE), jc = j < kk ? j : 0;
        const T* col = jc < kp ? P + jc * ldp : Q + (jc - kp) * ldq;
#pragma unroll
        for (int q = 0; q < RQ; ++q) {
            const int64_t r = r0 + lane + q * WAVE;
            pc[c][q] = j < kk && r < r1 ? col[r] : zero_of<T>();
        }
    }
    R x2 = 0;
    for (int g = threadIdx.x; g < gn; g += DT) x2 += normpart[g];
    const R xn2 = group_sum<DT>(x2, red);
    const T alpha = *alpha_in;
    R beta, are, aim = 0;
    if constexpr (Traits<T>::cplx) { are = alpha.re; aim = alpha.im; }
    else are = alpha;
    beta = are;
    T t = zero_of<T>(), scale = zero_of<T>();
    const bool have = xn2 != 0 || aim != 0;
    if (have) {
        beta = -copysign(sqrt(are * are + aim * aim + xn2), are);
        const R dr = are - beta, den = dr * dr + aim * aim;      // 1 / (alpha - beta)
        if constexpr (Traits<T>::cplx) {
            t = T{(beta - are) / beta, -aim / beta};
            scale = T{dr / den, -aim / den};
        } else {
            t = (beta - are) / beta;
            scale = R(1) / dr;
        }
    }
    for (int64_t r = r0 + threadIdx.x; r < r1; r += DT) {
        T x = from_one<T>();
        if (r != 0) {
            x = a[r];
            if (have) x = mul_of(x, scale);
        }
        a[r] = x;
        if (scat) scat[r * scinc] = conj_of(x);
        if (r - r0 < DT) xs[r - r0] = x;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) {
        *e = beta;
        *tau = t;
    }
    if (kk == 0) return;
    __syncthreads();     // the chunk of the vector is in place for all waves of the workgroup
    // a wave takes RC columns at a time, so that their loads are in flight together (a column past the end repeats
    // the wave's first one and is not stored)
    for (int jb = wv; jb < kk; jb += RC * (DT / WAVE)) {
        const T* col[RC];
        T acc[RC];
#pragma unroll
        for (int c = 0; c < RC; ++c) {
            const int j = jb + c * (DT / WAVE) < kk ? jb + c * (DT / WAVE) : jb;
            col[c] = j < kp ? P + j * ldp : Q + (j - kp) * ldq;
            acc[c] = zero_of<T>();
        }
        int64_t r = r0 + lane;
        if (jb == wv) {      // the group fetched ahead
#pragma unroll
            for (int q = 0; q < RQ; ++q, r += WAVE) {
                if (r < r1) {
                    const T x = xs[r - r0];
#pragma unroll
                    for (int c = 0; c < RC; ++c) fma_acc_conj(acc[c], pc[c][q], x);
                }
            }
        }
#pragma unroll 4
        for (; r < r1; r += WAVE) {
            const T x = r - r0 < DT ? xs[r - r0] : a[r];
#pragma unroll
            for (int c = 0; c < RC; ++c) fma_acc_conj(acc[c], col[c][r], x);
        }
#pragma unroll
        for (int c = 0; c < RC; ++c) {
            const T sum = wave_sum(acc[c]);
            const int j = jb + c * (DT / WAVE);
            if (lane == 0 && j < kk) dots[(int64_t)blockIdx.x * kk + j] = sum;
        }
    }
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

// Front of the workspace: what the panel's own kernels hand to each other.  alpha and the entry of w in the
// next diagonal row (256 bytes), then one partial per workgroup of the norms and of w^H v, then the partial
// products with the panels (2 nb per workgroup of the reflector kernel).
template <class T> struct PanelScratch {
    using R = typename Traits<T>::real;
    T* alpha;
    T* whead;
    R* normpart;
    T* wdot;
    T* dots;
    static size_t bytes(int64_t nb) {
        return 256 + round_up(FG_MAX * sizeof(R), 256) + round_up(FG_MAX * sizeof(T), 256) +
               round_up((size_t)DG_MAX * 2 * (size_t)nb * sizeof(T), 256);
    }
    explicit PanelScratch(void* base) {
        char* p = static_cast<char*>(base);
        alpha = reinterpret_cast<T*>(p);
        whead = alpha + 1;
        normpart = reinterpret_cast<R*>(p + 256);
        wdot = reinterpret_cast<T*>(p + 256 + round_up(FG_MAX * sizeof(R), 256));
        dots = reinterpret_cast<T*>(p + 256 + round_up(FG_MAX * sizeof(R), 256) + round_up(FG_MAX * sizeof(T), 256));
    }
};

// the panel's own scratch plus the largest workspace a symmetric product of the panel asks for
template <class T> size_t panel_workspace(int64_t n, int64_t nb) {
    if (n <= 0 || nb <= 0) return 0;
    if (nb > n) nb = n;
    size_t need = 0;
    for (int64_t i = 0; i < nb && i < n - 1; ++i)
        need = max_of(need, kmv_symv_workspace_bytes(Calls<T>::prec, 'L', n - i - 1));
    return PanelScratch<T>::bytes(nb) + need;
}

// T real: SYTRD panel; T complex (cf32 / cf64): HETRD panel, e real, transposes conjugated
template <class T>
int sytrd_panel(char uplo, int64_t n, int64_t nb, T* A, int64_t lda, typename Traits<T>::real* e, T* tau, T* W,
                int64_t ldw, void* ws, size_t wsb, void* stream) {
    using R = typename Traits<T>::real;
    constexpr bool CPLX = Traits<T>::cplx;
    const bool lower = (uplo == 'L' || uplo == 'l');
    if (!lower && uplo != 'U' && uplo != 'u') return -1;
    if (n < 0) return -2;
    if (nb < 0 || nb > n) return -3;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (ldw < (n > 1 ? n : 1)) return -9;
    if (n == 0 || nb == 0) return KMV_OK;
    if (!A || !e || !tau || !W) return KMV_ERR_NULL;
    if (!ws || wsb < panel_workspace<T>(n, nb) || ((uintptr_t)ws % 256) != 0) return KMV_ERR_WORKSPACE;
    if (nb > NB_MAX) return -3;
    const PanelScratch<T> sc(ws);
    ws = static_cast<char*>(ws) + PanelScratch<T>::bytes(nb);
    wsb -= PanelScratch<T>::bytes(nb);
    hipStream_t s = static_cast<hipStream_t>(stream);
    const T one = from_real<T>(1), zero = from_real<T>(0);
    const auto symv = Calls<T>::symv;
    const T* nullc = nullptr;
    T* nullm = nullptr;
#define KMV_PANEL_CHECK()                                        \
    do {                                                         \
        const hipError_t he_ = hipGetLastError();                \
        if (he_ != hipSuccess) return KMV_ERR_HIP + (int)he_;    \
    } while (0)
    if (!lower) {
        // Upper storage: the mirror image.  The LAST nb columns are reduced, from column n-1 down to n-nb; column
        // i has slot iw = i - (n - nb) in e, tau and W; its reflector annihilates A[0:i-1, i], v = A[0:i, i] with
        // the one at row i-1; the k = n-1-i columns to its right are the reflectors and W columns done before.
        const int64_t first = n - nb;
        // norm and alpha of the first column to go (it has nothing to catch up with)
        hipLaunchKernelGGL((panel_column_kernel<T, false>), dim3(thin_chunks(n)), dim3(FT), 0, s, n, thin_rows(n), 0, nullc,
                           (int64_t)0, nullc, (int64_t)0, nullc, nullm, nullc, nullc, 0, nullc, A + (n - 1) * lda, sc.normpart,
                           sc.alpha, 0, 1);
        KMV_PANEL_CHECK();
        for (int64_t i = n - 1; i >= first; --i) {
            const int64_t iw = i - first, k = n - 1 - i, mp = i + 1;
            T* col = A + i * lda;                    // A[0:i+1, i], the diagonal entry last
            if (i == 0) {   // first column of the matrix: no reflector
                if constexpr (CPLX) hipLaunchKernelGGL((no_reflector_kernel_c<T, R>), dim3(1), dim3(1), 0, s, col, e + iw, tau + iw);
                else hipLaunchKernelGGL((no_reflector_kernel<T, T>), dim3(1), dim3(1), 0, s, e + iw, tau + iw);
                KMV_PANEL_CHECK();
                continue;
            }
            const T* Vp = A + (i + 1) * lda;         // the k columns to the right: reflectors ...
            const T* Wp = W + (iw + 1) * ldw;        // ... and their companions
            hipLaunchKernelGGL((panel_reflector_kernel<T, false>), dim3(fat_chunks(mp)), dim3(DT), 0, s, mp, fat_rows(mp), (int)k,
                               Vp, lda, Wp, ldw, col, sc.normpart, (int)thin_chunks(mp), sc.alpha, e + iw, tau + iw, sc.dots);
            KMV_PANEL_CHECK();
            const int64_t m = i;                     // length of v = A[0:i, i]
            T* w = W + iw * ldw;                     // W[0:i, iw]
            const int rc = symv('U', m, &one, A, lda, col, 1, &zero, w, 1, ws, wsb, stream);
            if (rc) return rc;
            hipLaunchKernelGGL((panel_correct_kernel<T>), dim3(thin_chunks(m)), dim3(FT), 0, s, m, thin_rows(m), (int)k, Vp, lda, Wp,
                               ldw, col, w, tau + iw, sc.dots, (int)fat_chunks(mp), m - 1, sc.wdot, sc.whead);
            KMV_PANEL_CHECK();
            hipLaunchKernelGGL((panel_column_kernel<T, false>), dim3(thin_chunks(m)), dim3(FT), 0, s, m, thin_rows(m), (int)k, Vp, lda,
                               Wp, ldw, col, w, tau + iw, sc.wdot, (int)thin_chunks(m), sc.whead, A + (i - 1) * lda, sc.normpart,
                               sc.alpha, 1, i - 1 >= first ? 1 : 0);
            KMV_PANEL_CHECK();
        }
        return KMV_OK;
    }
    hipLaunchKernelGGL((panel_column_kernel<T, true>), dim3(thin_chunks(n)), dim3(FT), 0, s, n, thin_rows(n), 0, nullc, (int64_t)0,
                       nullc, (int64_t)0, nullc, nullm, nullc, nullc, 0, nullc, A, sc.normpart, sc.alpha, 0, 1);
    KMV_PANEL_CHECK();
    for (int64_t i = 0; i < nb; ++i) {
        T* col = A + i + i * lda;               // A[i:, i], up to date: the diagonal entry first
        const int64_t mp = n - i;
        if (i >= n - 1) {   // last column of the matrix: no reflector; its slots are defined all the same
            if constexpr (CPLX) hipLaunchKernelGGL((no_reflector_kernel_c<T, R>), dim3(1), dim3(1), 0, s, col, e + i, tau + i);
            else hipLaunchKernelGGL((no_reflector_kernel<T, T>), dim3(1), dim3(1), 0, s, e + i, tau + i);
            KMV_PANEL_CHECK();
            continue;
        }
        hipLaunchKernelGGL((panel_reflector_kernel<T, true>), dim3(fat_chunks(mp)), dim3(DT), 0, s, mp, fat_rows(mp), (int)i, A + i,
                           lda, W + i, ldw, col, sc.normpart, (int)thin_chunks(mp), sc.alpha, e + i, tau + i, sc.dots);
        KMV_PANEL_CHECK();
        const int64_t m = n - i - 1;
        T* v = col + 1;                         // A[i+1:, i]
        T* w = W + (i + 1) + i * ldw;           // W[i+1:, i]
        const int rc = symv('L', m, &one, A + (i + 1) + (i + 1) * lda, lda, v, 1, &zero, w, 1, ws, wsb, stream);
        if (rc) return rc;
        const T* Vp = A + i + 1;                // rows i+1.. of the i reflectors before ...
        const T* Wp = W + i + 1;                // ... and of their companions
        hipLaunchKernelGGL((panel_correct_kernel<T>), dim3(thin_chunks(m)), dim3(FT), 0, s, m, thin_rows(m), (int)i, Vp, lda, Wp, ldw,
                           v, w, tau + i, sc.dots, (int)fat_chunks(mp), (int64_t)0, sc.wdot, sc.whead);
        KMV_PANEL_CHECK();
        hipLaunchKernelGGL((panel_column_kernel<T, true>), dim3(thin_chunks(m)), dim3(FT), 0, s, m, thin_rows(m), (int)i, Vp, lda, Wp,
                           ldw, v, w, tau + i, sc.wdot, (int)thin_chunks(m), sc.whead, A + (i + 1) + (i + 1) * lda, sc.normpart,
                           sc.alpha, 1, i + 1 < nb ? 1 : 0);
        KMV_PANEL_CHECK();
    }
    return KMV_OK;
#undef KMV_PANEL_CHECK
}

// bytes at the front of the workspace for the contiguous copy of the current row
template <class T> size_t row_bytes(int64_t n) { return (size_t)((n * sizeof(T) + 255) / 256) * 256; }

// complex panels: three conjugated copies of short strided rows (at most nb elements each)
template <class T> size_t short_rows_bytes(int64_t nb) {
    return Traits<T>::cplx ? (size_t)((3 * nb * sizeof(T) + 255) / 256) * 256 : 0;
}

// the contiguous copy U of the row reflectors (n x nb, U[j][k] = u_k[j]) that the fused step keeps
inline int64_t bd_ldu(int64_t n) { return (n + 31) / 32 * 32; }
template <class T> size_t bd_u_bytes(int64_t n, int64_t nb) { return round_up((size_t)bd_ldu(n) * (size_t)nb * sizeof(T), 256); }

// Workspace of the bidiagonal panel.  Panels of at most BD_NB columns run the fused step: the hand-over scratch
// of its kernels, U, and the largest workspace of the two products with the trailing block; wider panels the
// step built from GEMV calls: the row copy plus the largest workspace any of its products asks for.
template <class T> size_t gebrd_workspace(int64_t m, int64_t n, int64_t nb) {
    if (m <= 0 || n <= 0 || nb <= 0) return 0;
    const int64_t mn = m < n ? m : n;
    if (nb > mn) nb = mn;
    const char p = Calls<T>::prec;
    size_t need = 0;
    if (nb <= BD_NB) {
        for (int64_t i = 0; i < nb; ++i) {
            const int64_t mi = m < n ? m - i - 1 : m - i, ni = m < n ? n - i : n - i - 1;
            if (mi <= 0 || ni <= 0) continue;
            if (m < n) {
                need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi, ni));
                need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, ni - 1));
            } else {
                need = max_of(need, kmv_gemv_workspace_bytes(p, 'T', mi, ni));
                need = max_of(need, kmv_gemv_workspace_bytes(p, 'N', mi - 1, ni));
            }
        }
        return PanelScratch<T>::bytes(nb) + bd_u_bytes<T>(n, nb) + need;
    }
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

// The bidiagonal panel step with the kernels above (panels of at most BD_NB columns): per column
//   m >= n:  reflector of column i (d, tauq; partial V^H v, X^H v) - y_i = A22^H v (GEMV) - update along the columns
//            (y_i finished; row i gathered, conjugated, brought up to date into U[:, i]) - reflector of the row (e,
//            taup; scattered back into A; partial Y^H u, U^H u) - x_i = A22 u (GEMV) - update along the rows (x_i
//            finished; column i+1 brought up to date)
//   m <  n:  the same with rows and columns exchanged, the row first.
// Arguments are checked by the caller.
template <class T>
int gebrd_panel_fused(int64_t m, int64_t n, int64_t nb, T* A, int64_t lda, typename Traits<T>::real* d,
                      typename Traits<T>::real* e, T* tauq, T* taup, T* X, int64_t ldx, T* Y, int64_t ldy, void* ws, size_t wsb,
                      void* stream) {
    using R = typename Traits<T>::real;
    constexpr bool CPLX = Traits<T>::cplx;
    const PanelScratch<T> sc(ws);
    T* U = reinterpret_cast<T*>(static_cast<char*>(ws) + PanelScratch<T>::bytes(nb));
    const int64_t ldu = bd_ldu(n);
    const size_t front = PanelScratch<T>::bytes(nb) + bd_u_bytes<T>(n, nb);
    ws = static_cast<char*>(ws) + front;
    wsb -= front;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const T one = from_real<T>(1), zero = from_real<T>(0);
    const char TR = CPLX ? 'C' : 'T';
    auto a_ = [&](int64_t i, int64_t j) { return A + i + j * lda; };
    auto x_ = [&](int64_t i, int64_t j) { return X + i + j * ldx; };
    auto y_ = [&](int64_t i, int64_t j) { return Y + i + j * ldy; };
    auto u_ = [&](int64_t j, int64_t k) { return U + j + k * ldu; };
    const T* nullc = nullptr;
    T* nullm = nullptr;
    int rc = KMV_OK;
#define KMV_BD_CHECK()                                           \
    do {                                                         \
        const hipError_t he_ = hipGetLastError();                \
        if (he_ != hipSuccess) return KMV_ERR_HIP + (int)he_;    \
    } while (0)
    // update along the rows of A: finishes x (column kq of X, `fin`) and brings column c of A up to date (`next`),
    // both from row r0 on; kp = columns of V, kq = columns of X in the sums
    auto rows_update = [&](int64_t r0, int64_t c, int kp, int kq, const T* tau, int gd, int fin, int next) {
        const int64_t len = m - r0;
        hipLaunchKernelGGL((bd_update_kernel<T, false>), dim3(thin_chunks(len)), dim3(FT), 0, s, len, thin_rows(len), kp, a_(r0, 0), lda,
                           kq, x_(r0, 0), ldx, fin ? x_(r0, kq) : nullm, tau, sc.dots, gd, next && fin ? y_(c, 0) : nullc, ldy,
                           next && fin ? a_(0, c) : nullc, (int64_t)1, 0, next && fin ? a_(kq, c) : nullc,
                           next ? a_(r0, c) : nullc, (int64_t)1, next ? a_(r0, c) : nullm, sc.normpart, sc.alpha, fin, next);
    };
    // update along the columns of A: finishes y (column yc of Y, `fin`) and gathers row r of A from column j0 on,
    // conjugated and brought up to date, into U[j0:, r] (`next`); P and Q are (Y, U) or (U, Y), see the callers
    auto cols_update = [&](int64_t j0, int64_t r, int kp, const T* P, int64_t ldp, int kq, const T* Q, int64_t ldq, T* z,
                           const T* tau, int gd, const T* c1src, int64_t c1inc, const T* c2src, int64_t c2inc, const T* czsrc, int fin,
                           int next) {
        const int64_t len = n - j0;
        hipLaunchKernelGGL((bd_update_kernel<T, true>), dim3(thin_chunks(len)), dim3(FT), 0, s, len, thin_rows(len), kp, P, ldp, kq, Q,
                           ldq, z, tau, sc.dots, gd, c1src, c1inc, c2src, c2inc, 1, czsrc, next ? a_(r, j0) : nullc, lda,
                           next ? u_(j0, r) : nullm, sc.normpart, sc.alpha, fin, next);
    };
    auto reflect = [&](int64_t len, int kp, const T* P, int64_t ldp, int kq, const T* Q, int64_t ldq, T* a, R* beta, T* tau, T* scat) {
        hipLaunchKernelGGL((bd_reflector_kernel<T>), dim3(fat_chunks(len)), dim3(DT), 0, s, len, fat_rows(len), kp, P, ldp, kq, Q, ldq, a,
                           sc.normpart, (int)thin_chunks(len), sc.alpha, beta, tau, scat, lda, sc.dots);
    };
    if (m < n) {
        // lower bidiagonal: the row first
        cols_update(0, 0, 0, nullc, 0, 0, nullc, 0, nullm, nullc, 0, nullc, 0, nullc, 0, nullc, 0, 1);
        KMV_BD_CHECK();
        for (int64_t i = 0; i < nb; ++i) {
            const int64_t mi = m - i - 1, ni = n - i;       // rows below row i, columns from column i on
            const int k = (int)i;
            reflect(ni, k, y_(i, 0), ldy, k, u_(i, 0), ldu, u_(i, i), d + i, taup + i, a_(i, i));
            KMV_BD_CHECK();
            if (mi <= 0) {     // last row of the matrix: no column reflector
                hipLaunchKernelGGL((no_reflector_kernel<R, T>), dim3(1), dim3(1), 0, s, e + i, tauq + i);
                KMV_BD_CHECK();
                continue;
            }
            rc = Calls<T>::gemv('N', mi, ni, &one, a_(i + 1, i), lda, u_(i, i), (int64_t)1, &zero, x_(i + 1, i), (int64_t)1, ws, wsb,
                                stream);
            if (rc) return rc;
            // x_i = taup (x - V (Y^H u) - X (U^H u)); column i below the diagonal catches up, x_i taking part
            rows_update(i + 1, i, k, k, taup + i, (int)fat_chunks(ni), 1, 1);
            KMV_BD_CHECK();
            reflect(mi, k + 1, x_(i + 1, 0), ldx, k, a_(i + 1, 0), lda, a_(i + 1, i), e + i, tauq + i, nullm);
            KMV_BD_CHECK();
            rc = Calls<T>::gemv(TR, mi, ni - 1, &one, a_(i + 1, i + 1), lda, a_(i + 1, i), (int64_t)1, &zero, y_(i + 1, i), (int64_t)1,
                                ws, wsb, stream);
            if (rc) return rc;
            // y_i = tauq (y - U (X^H v) - Y (V^H v)); row i+1 catches up, y_i taking part
            cols_update(i + 1, i + 1, k + 1, u_(i + 1, 0), ldu, k, y_(i + 1, 0), ldy, y_(i + 1, i), tauq + i, (int)fat_chunks(mi),
                        x_(i + 1, 0), ldx, a_(i + 1, 0), lda, a_(i + 1, i), 1, i + 1 < nb ? 1 : 0);
            KMV_BD_CHECK();
        }
        return KMV_OK;
    }
    rows_update(0, 0, 0, 0, nullc, 0, 0, 1);
    KMV_BD_CHECK();
    for (int64_t i = 0; i < nb; ++i) {
        const int64_t mi = m - i, ni = n - i - 1;
        const int k = (int)i;
        reflect(mi, k, a_(i, 0), lda, k, x_(i, 0), ldx, a_(i, i), d + i, tauq + i, nullm);
        KMV_BD_CHECK();
        if (ni <= 0) {     // last column of the matrix: no row reflector
            hipLaunchKernelGGL((no_reflector_kernel<R, T>), dim3(1), dim3(1), 0, s, e + i, taup + i);
            KMV_BD_CHECK();
            continue;
        }
        rc = Calls<T>::gemv(TR, mi, ni, &one, a_(i, i + 1), lda, a_(i, i), (int64_t)1, &zero, y_(i + 1, i), (int64_t)1, ws, wsb, stream);
        if (rc) return rc;
        // y_i = tauq (y - Y (V^H v) - U (X^H v)); row i right of the diagonal catches up, y_i taking part
        cols_update(i + 1, i, k, y_(i + 1, 0), ldy, k, u_(i + 1, 0), ldu, y_(i + 1, i), tauq + i, (int)fat_chunks(mi), a_(i, 0), lda,
                    x_(i, 0), ldx, a_(i, i), 1, 1);
        KMV_BD_CHECK();
        reflect(ni, k + 1, y_(i + 1, 0), ldy, k, u_(i + 1, 0), ldu, u_(i + 1, i), e + i, taup + i, a_(i, i + 1));
        KMV_BD_CHECK();
        rc = Calls<T>::gemv('N', mi - 1, ni, &one, a_(i + 1, i + 1), lda, u_(i + 1, i), (int64_t)1, &zero, x_(i + 1, i), (int64_t)1, ws,
                            wsb, stream);
        if (rc) return rc;
        // x_i = taup (x - V (Y^H u) - X (U^H u)); column i+1 catches up, x_i taking part
        rows_update(i + 1, i + 1, k + 1, k, taup + i, (int)fat_chunks(ni), 1, i + 1 < nb ? 1 : 0);
        KMV_BD_CHECK();
    }
#undef KMV_BD_CHECK
    return KMV_OK;
}

// Panel step of the bidiagonal reduction (m >= n: upper bidiagonal; m < n: lower bidiagonal, see the branch
// below): the published "labrd" step written from its definition.  Argument checks, then the fused step above
// for panels of at most BD_NB columns; beyond that the step on top of the GEMV entry points that follows,
// which is also the plain statement of what the fused kernels compute.  Per column two products with the whole trailing
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
    if (nb <= BD_NB) return gebrd_panel_fused<T>(m, n, nb, A, lda, d, e, tauq, taup, X, ldx, Y, ldy, ws, wsb, stream);
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
