// SYMV / HEMV kernels for gfx950: y <- alpha*A*x + beta*y with A symmetric
// (real) or Hermitian (complex) and only one triangle stored.
//
// The paper (Section 6.1 kernel 3, Section 6.2 Eq. total_workload_symv,
// Section 6.3 and Algorithm "Upper/Lower SYMV/HEMV") walks the off-diagonal
// blocks of a block column vertically, uses every loaded element twice (the
// "non-transposed" product a_ij*x_j for y_i and the "transposed" product
// op(a_ij)*x_i for y_j), keeps the transposed partial sums in registers over
// the whole walk, but has to reduce and write the non-transposed ones after
// every block because they belong to different pieces of y; diagonal blocks go
// to a separate kernel that mirrors them in shared memory (Section 6.5).
//
// Kept: the vertical walk of a column panel, the dual use of each element, the
// register accumulators for the transposed part, the register double buffer.
// Different: lanes map to 16-byte row vectors (wave64 streams 1 KiB of a
// column per instruction); the waves of a workgroup share the rows and split
// the panel's columns, their non-transposed row sums meet in LDS and are
// flushed every KT row tiles to a workspace indexed [panel][row] (one barrier
// per KT tiles instead of two per block, and no atomics); the diagonal tiles
// are handled in the same kernel by predicated element loads that never touch
// the other triangle, so the mirrored copy of Section 6.5 is never built; the
// triangle is cut into (panel, chunk of row tiles) workgroups of bounded size
// instead of a fixed (X, Y) grid, which balances the triangular workload.
// A second kernel adds, in a fixed order, all row sums and column sums that
// belong to y_i and applies alpha and beta.
#include "kmv_launch.hpp"

namespace kmv {

namespace {
constexpr int SY_NW = 4;    // waves per workgroup
constexpr int SY_CW = 16;   // columns per wave  -> panel of 64 columns
constexpr int SY_KT = 4;    // row tiles between two flushes of the row sums
constexpr int64_t DEFAULT_CHUNK_TILES = 8;
constexpr int64_t MAX_CHUNK_TILES = 64;
constexpr int RED_ROWS = 64, RED_PARTS = 4;
}  // namespace

template <class T> int panel_cols() { return SY_NW * SY_CW; }

// first / one-past-last row tile that a panel's stored part touches
template <bool LOWER>
__host__ __device__ __forceinline__ void panel_tiles(int64_t J0, int64_t C, int64_t n, int shift, int64_t TR,
                                                     int64_t ntiles, int64_t& tlo, int64_t& thi) {
    if (LOWER) {
        tlo = (J0 + shift) / TR;
        thi = ntiles;
    } else {
        const int64_t jend = (J0 + C < n) ? (J0 + C) : n;
        tlo = 0;
        thi = (jend - 1 + shift) / TR + 1;
    }
}

template <class T, bool HERM, bool LOWER, int CW, int NW, int KT>
__global__ __launch_bounds__(NW * WAVE) void symv_kernel(SymvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    constexpr int C = CW * NW;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int64_t n = a.n, lda = a.lda;
    const int shift = a.plan.shift;
    const T* __restrict__ x = a.x;

    // long panels first: panel 0 is the longest for 'L', the last one for 'U'
    const int64_t p = LOWER ? (int64_t)blockIdx.y : (a.plan.npanels - 1 - (int64_t)blockIdx.y);
    const int64_t J0 = p * C;
    int64_t tlo, thi;
    panel_tiles<LOWER>(J0, C, n, shift, TR, a.plan.ntiles, tlo, thi);
    const int64_t tbeg = tlo + (int64_t)blockIdx.x * a.plan.chunk_tiles;
    int64_t tend = tbeg + a.plan.chunk_tiles;
    if (tend > thi) tend = thi;
    if (tbeg >= tend) return;   // whole workgroup leaves together, before any barrier

    const int64_t jw = J0 + (int64_t)w * CW;   // first column of this wave
    const bool ragged_panel = (J0 + C > n);
    T xj[CW];
    const T* __restrict__ col[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const bool ok = jw + c < n;
        xj[c] = ok ? x[jw + c] : zero_of<T>();
        col[c] = a.A + (ok ? (jw + c) : (n - 1)) * lda;
    }
    T accT[CW];
#pragma unroll
    for (int c = 0; c < CW; ++c) accT[c] = zero_of<T>();

    __shared__ Vec<T> nbuf[2][NW][KT][WAVE];
    int q = 0, buf = 0;
    int64_t gstart = tbeg;
    T* __restrict__ wsn = a.wsn + p * a.plan.rows_padded;

    // hand the row sums of tile t to LDS; every KT tiles (and after the last
    // tile) add the NW waves' contributions in wave order and store them.
    auto emit = [&](const T(&accN)[VEC], int64_t t) {
        Vec<T> o;
#pragma unroll
        for (int v = 0; v < VEC; ++v) o.e[v] = accN[v];
        nbuf[buf][w][q][lane] = o;
        ++q;
        if (q == KT || t == tend - 1) {
            __syncthreads();
            for (int e = threadIdx.x; e < q * WAVE; e += NW * WAVE) {
                const int qt = e / WAVE, ln = e % WAVE;
                Vec<T> s = nbuf[buf][0][qt][ln];
#pragma unroll
                for (int ww = 1; ww < NW; ++ww) {
                    const Vec<T> o2 = nbuf[buf][ww][qt][ln];
#pragma unroll
                    for (int v = 0; v < VEC; ++v) s.e[v] = add_of(s.e[v], o2.e[v]);
                }
                store_vec(wsn + (gstart + qt) * TR + (int64_t)ln * VEC, s);
            }
            buf ^= 1;
            gstart += q;
            q = 0;
        }
    };

    // a tile is interior when all its rows exist, the panel is full width and
    // every (row, column) pair lies strictly inside the stored triangle
    auto is_interior = [&](int64_t t) {
        const int64_t r0 = t * TR - shift;
        if (ragged_panel || r0 < 0 || r0 + TR > n) return false;
        return LOWER ? (r0 > J0 + C - 1) : (r0 + TR - 1 < J0);
    };
    auto masked_tile = [&](int64_t t) {
        const int64_t r = t * TR - shift + (int64_t)lane * VEC;
        T accN[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            accN[v] = zero_of<T>();
            const int64_t row = r + v;
            const bool rowok = row >= 0 && row < n;
            const T xi = rowok ? x[row] : zero_of<T>();
#pragma unroll
            for (int c = 0; c < CW; ++c) {
                const int64_t j = jw + c;
                const bool inside = rowok && j < n && (LOWER ? row >= j : row <= j);
                if (inside) {
                    T av = load_elem_stream(col[c] + row);
                    if (row == j) {
                        if (HERM) av = real_part_only(av);
                        fma_acc(accN[v], av, xj[c]);
                    } else {
                        fma_acc(accN[v], av, xj[c]);
                        fma_op<HERM>(accT[c], av, xi);
                    }
                }
            }
        }
        emit(accN, t);
    };

    Vec<T> xi0, xi1, b0[CW], b1[CW];
    auto load_tile = [&](Vec<T>& xi, Vec<T>(&bb)[CW], int64_t t) {
        const int64_t r = t * TR - shift + (int64_t)lane * VEC;
        xi = load_cached(x + r);
#pragma unroll
        for (int c = 0; c < CW; ++c) bb[c] = load_stream(col[c] + r);
    };
    auto compute_tile = [&](const Vec<T>& xi, const Vec<T>(&bb)[CW], int64_t t) {
        T accN[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) accN[v] = zero_of<T>();
#pragma unroll
        for (int c = 0; c < CW; ++c)
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                fma_acc(accN[v], bb[c].e[v], xj[c]);
                fma_op<HERM>(accT[c], bb[c].e[v], xi.e[v]);
            }
        emit(accN, t);
    };

    // masked prefix, interior run (register double buffer), masked suffix
    int64_t t = tbeg;
    while (t < tend && !is_interior(t)) { masked_tile(t); ++t; }
    int64_t tin_end = t;
    while (tin_end < tend && is_interior(tin_end)) ++tin_end;
    if (t < tin_end) load_tile(xi0, b0, t);
    for (; t < tin_end; t += 2) {
        if (t + 1 < tin_end) load_tile(xi1, b1, t + 1);
        compute_tile(xi0, b0, t);
        if (t + 1 < tin_end) {
            if (t + 2 < tin_end) load_tile(xi0, b0, t + 2);
            compute_tile(xi1, b1, t + 1);
        }
    }
    for (t = tin_end; t < tend; ++t) masked_tile(t);

    // transposed part: one wave reduction per column, this wave owns its columns
    T* __restrict__ wst = a.wst + (p * a.plan.max_chunks + (int64_t)blockIdx.x) * C + (int64_t)w * CW;
#pragma unroll
    for (int c = 0; c < CW; ++c) {
        const T s = wave_sum(accT[c]);
        if (lane == 0) wst[c] = s;
    }
}

// y_i = alpha * ( sum over panels of wsn[panel][i] + sum over chunks of
// wst[panel(i)][chunk][i] ) + beta*y_i, every sum in ascending index order.
// blockDim = (RED_ROWS, RED_PARTS): the panel range of a row is cut into
// RED_PARTS interleaved parts that meet in LDS in part order.
template <class T, bool LOWER>
__global__ __launch_bounds__(RED_ROWS * RED_PARTS) void symv_reduce_kernel(SymvArgs<T> a, int C) {
    constexpr int TR = tile_rows<T>();
    const int lx = threadIdx.x, g = threadIdx.y;
    const int64_t i = (int64_t)blockIdx.x * RED_ROWS + lx;
    const int shift = a.plan.shift;
    __shared__ T part[RED_PARTS][RED_ROWS];
    T s = zero_of<T>();
    if (i < a.n) {
        const int64_t slot = i + shift;
        const int64_t ti = slot / TR;
        int64_t pbeg, pend;   // panels whose tile range contains tile ti
        if (LOWER) {
            pbeg = 0;
            pend = ((ti + 1) * TR - shift - 1) / C + 1;
            if (pend > a.plan.npanels) pend = a.plan.npanels;
        } else {
            const int64_t need = ti * TR - shift + 1;   // panels with (p+1)*C >= need
            pbeg = need > 0 ? (need + C - 1) / C - 1 : 0;
            pend = a.plan.npanels;
        }
        const T* __restrict__ wsn = a.wsn + slot;
        for (int64_t p = pbeg + g; p < pend; p += RED_PARTS) s = add_of(s, wsn[p * a.plan.rows_padded]);
    }
    part[g][lx] = s;
    __syncthreads();
    if (g == 0 && i < a.n) {
        T tot = part[0][lx];
#pragma unroll
        for (int gg = 1; gg < RED_PARTS; ++gg) tot = add_of(tot, part[gg][lx]);
        const int64_t pi = i / C;
        int64_t tlo, thi;
        panel_tiles<LOWER>(pi * C, C, a.n, shift, TR, a.plan.ntiles, tlo, thi);
        const int64_t nch = ceil_div(thi - tlo, a.plan.chunk_tiles);
        const T* __restrict__ wst = a.wst + pi * a.plan.max_chunks * C + (i - pi * C);
        for (int64_t k = 0; k < nch; ++k) tot = add_of(tot, wst[k * C]);
        T* yp = a.y + i * a.incy;
        *yp = epilogue(a.alpha, tot, a.beta, yp);
    }
}

// ------------------------------------------------------------- host side ----
template <class T> SymvPlan<T> plan_symv(bool lower, int64_t n, const void* A, int64_t lda) {
    (void)lower;
    constexpr int TR = tile_rows<T>();
    const int64_t C = panel_cols<T>();
    SymvPlan<T> p;
    const bool sizing = (A == nullptr);
    p.shift = sizing ? max_row_shift<T>() : row_shift<T>(A, lda);
    p.ntiles = ceil_div(n + p.shift, TR);
    p.npanels = ceil_div(n, C);
    int64_t ct = tuning().symv_chunk_tiles > 0 ? tuning().symv_chunk_tiles : DEFAULT_CHUNK_TILES;
    if (ct > MAX_CHUNK_TILES) ct = MAX_CHUNK_TILES;
    p.chunk_tiles = ct;
    p.max_chunks = ceil_div(p.ntiles, ct);
    p.rows_padded = p.ntiles * TR;
    p.xpack_off = 0;
    p.wsn_off = round_up((size_t)n * sizeof(T), WS_ALIGN);
    p.wst_off = p.wsn_off + round_up((size_t)p.npanels * p.rows_padded * sizeof(T), WS_ALIGN);
    // sizing: one chunk per tile is the largest column-sum area any tuning needs
    const int64_t size_chunks = sizing ? p.ntiles : p.max_chunks;
    p.total_bytes = p.wst_off + round_up((size_t)p.npanels * size_chunks * C * sizeof(T), WS_ALIGN);
    return p;
}

template <class T, bool HERM> static hipError_t launch_symv_impl(const SymvArgs<T>& a, bool lower, hipStream_t s) {
    const dim3 grid((unsigned)a.plan.max_chunks, (unsigned)a.plan.npanels);
    if (lower)
        hipLaunchKernelGGL((symv_kernel<T, HERM, true, SY_CW, SY_NW, SY_KT>), grid, dim3(SY_NW * WAVE), 0, s, a);
    else
        hipLaunchKernelGGL((symv_kernel<T, HERM, false, SY_CW, SY_NW, SY_KT>), grid, dim3(SY_NW * WAVE), 0, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 rgrid((unsigned)ceil_div(a.n, RED_ROWS));
    const dim3 rblock(RED_ROWS, RED_PARTS);
    if (lower)
        hipLaunchKernelGGL((symv_reduce_kernel<T, true>), rgrid, rblock, 0, s, a, (int)panel_cols<T>());
    else
        hipLaunchKernelGGL((symv_reduce_kernel<T, false>), rgrid, rblock, 0, s, a, (int)panel_cols<T>());
    return hipGetLastError();
}

template <class T> hipError_t launch_symv(const SymvArgs<T>& a, bool lower, hipStream_t s) {
    return launch_symv_impl<T, Traits<T>::cplx>(a, lower, s);
}

#define KMV_INSTANTIATE_SYMV(T)                                                       \
    template int panel_cols<T>();                                                     \
    template SymvPlan<T> plan_symv<T>(bool, int64_t, const void*, int64_t);           \
    template hipError_t launch_symv<T>(const SymvArgs<T>&, bool, hipStream_t);
KMV_INSTANTIATE_SYMV(float)
KMV_INSTANTIATE_SYMV(double)
KMV_INSTANTIATE_SYMV(cf32)
KMV_INSTANTIATE_SYMV(cf64)

}  // namespace kmv
