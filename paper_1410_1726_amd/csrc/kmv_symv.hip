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
// register double buffer.  Different, to fit wave64 and the HBM behaviour of
// the MI355X (a workgroup that touches many columns at the same row offset
// loses bandwidth, a workgroup that reads a few columns over several KiB of
// consecutive rows does not):
//  * lanes map to 16-byte row vectors, a wave streams 1 KiB of a column per
//    instruction;
//  * a workgroup owns (panel of C columns) x (chunk of NW*KTW row tiles); each
//    wave owns KTW of those row tiles for the whole task and sweeps the panel
//    in groups of NC columns, so at any moment the workgroup reads NC columns
//    over NW consecutive KiB;
//  * the non-transposed row sums of a wave's tiles therefore stay in registers
//    for the whole panel width and are stored once per task into a workspace
//    indexed [panel][row] - no shared memory, no barrier and no atomics in the
//    loop (the paper needs a sync-and-reduce per block);
//  * the transposed column sums are reduced across the wave once per column
//    group (DPP), meet the other waves' in LDS and go to a second workspace
//    indexed [panel][chunk][column];
//  * diagonal tiles are handled in the same kernel by predicated element loads
//    that never touch the other triangle, so the mirrored copy of Section 6.5
//    is never built;
//  * the triangle is cut into bounded (panel, chunk) tasks instead of a fixed
//    (X, Y) grid, which balances the triangular workload.
// A second kernel adds, in a fixed order, all row sums and column sums that
// belong to y_i and applies alpha and beta.
#include "kmv_launch.hpp"

namespace kmv {

namespace {
constexpr int SY_NW = 4;    // waves per workgroup
constexpr int SY_NC = 8;    // columns per column group
constexpr int DEFAULT_PANEL_COLS = 64;
constexpr int DEFAULT_TILES_PER_WAVE = 2;
constexpr int RED_ROWS = 32, RED_PARTS = 8;
}  // namespace

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

template <class T, bool HERM, bool LOWER, int NC, int CGS, int KTW, int NW>
__global__ __launch_bounds__(NW * WAVE) void symv_kernel(SymvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    constexpr int C = NC * CGS;
    constexpr int CT = NW * KTW;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int64_t n = a.n, lda = a.lda;
    const int shift = a.plan.shift;
    const T* __restrict__ x = a.x;

    // Workgroup ids are dealt round robin to the 8 XCDs, each with its own L2.
    // All chunks of a panel go to one XCD (panel index = XCD modulo 8), so every
    // L2 sees the whole range of row offsets: with a power-of-two leading
    // dimension the lines of one row range in all columns share few L2 sets.
    // Long panels first: panel 0 is the longest for 'L', the last one for 'U'.
    const int64_t lin = blockIdx.x;
    const int64_t slot = lin / XCDS, xcd = lin % XCDS;
    const int64_t pord = (slot / a.plan.max_chunks) * XCDS + xcd;
    const int64_t chunk = slot % a.plan.max_chunks;
    if (pord >= a.plan.npanels) return;
    const int64_t p = LOWER ? pord : (a.plan.npanels - 1 - pord);
    const int64_t J0 = p * C;
    int64_t tlo, thi;
    panel_tiles<LOWER>(J0, C, n, shift, TR, a.plan.ntiles, tlo, thi);
    const int64_t tbeg = tlo + chunk * CT;
    int64_t tend = tbeg + CT;
    if (tend > thi) tend = thi;
    if (tbeg >= tend) return;   // whole workgroup leaves together, before any barrier

    const bool ragged_panel = (J0 + C > n);
    // a tile is "fast" when all its rows exist, the panel is full width and every
    // (row, column) pair of the panel lies strictly inside the stored triangle
    auto is_interior = [&](int64_t t) {
        const int64_t r0 = t * TR - shift;
        if (ragged_panel || r0 < 0 || r0 + TR > n) return false;
        return LOWER ? (r0 > J0 + C - 1) : (r0 + TR - 1 < J0);
    };

    // this wave's row tiles, their x segment and their row-sum accumulators
    int64_t rq[KTW];
    bool valid[KTW], fast[KTW];
    Vec<T> xi[KTW];
    T accN[KTW][VEC];
#pragma unroll
    for (int q = 0; q < KTW; ++q) {
        const int64_t t = tbeg + w + (int64_t)NW * q;
        valid[q] = t < tend;
        fast[q] = valid[q] && is_interior(t);
        rq[q] = t * TR - shift + (int64_t)lane * VEC;
        if (fast[q]) {
            xi[q] = load_cached(x + rq[q]);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const int64_t row = rq[q] + v;
                const int64_t rc = row < 0 ? 0 : (row >= n ? n - 1 : row);
                xi[q].e[v] = select_of(valid[q] && row >= 0 && row < n, x[rc], zero_of<T>());
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) accN[q][v] = zero_of<T>();
    }

    __shared__ T tpart[NW][C];
    const T* __restrict__ colbase = a.A + J0 * lda;

    // one unit of work = one column group (NC columns) over all KTW tiles of the
    // wave; the next unit's matrix vectors and x_j scalars are in flight while
    // the current one is being used
    Vec<T> b0[KTW][NC], b1[KTW][NC];
    T xj0[NC], xj1[NC];
    auto load_cg = [&](Vec<T>(&buf)[KTW][NC], T(&xjb)[NC], int cg) {
        const int64_t jg = J0 + (int64_t)cg * NC;
#pragma unroll
        for (int q = 0; q < KTW; ++q) {
            if (fast[q]) {
                const T* src = colbase + (int64_t)cg * NC * lda + rq[q];
#pragma unroll
                for (int c = 0; c < NC; ++c) buf[q][c] = load_stream(src + (int64_t)c * lda);
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) xjb[c] = select_of(jg + c < n, x[jg + c < n ? jg + c : n - 1], zero_of<T>());
    };
    auto compute_cg = [&](const Vec<T>(&buf)[KTW][NC], const T(&xjb)[NC], int cg) {
        const int64_t jg = J0 + (int64_t)cg * NC;
        T accT[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) accT[c] = zero_of<T>();
#pragma unroll
        for (int q = 0; q < KTW; ++q) {
            if (fast[q]) {
#pragma unroll
                for (int c = 0; c < NC; ++c)
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        fma_acc(accN[q][v], buf[q][c].e[v], xjb[c]);
                        fma_op<HERM>(accT[c], buf[q][c].e[v], xi[q].e[v]);
                    }
            } else if (valid[q]) {
                // edge / diagonal tile: element loads, all issued before the first
                // use; a pair outside the stored triangle loads the (always
                // stored) diagonal element of its column instead and is skipped
                T av[VEC][NC];
                bool ins[VEC][NC], dia[VEC][NC];
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const int64_t row = rq[q] + v;
                    const bool rowok = row >= 0 && row < n;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int64_t j = jg + c;
                        const int64_t jc = j < n ? j : n - 1;
                        ins[v][c] = rowok && j < n && (LOWER ? row >= j : row <= j);
                        dia[v][c] = (row == j);
                        av[v][c] = load_elem_stream(a.A + (ins[v][c] ? row : jc) + jc * lda);
                    }
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v)
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const T an = select_of(HERM && dia[v][c], real_part_only(av[v][c]), av[v][c]);
                        T nn = accN[q][v], nt = accT[c];
                        fma_acc(nn, an, xjb[c]);
                        fma_op<HERM>(nt, av[v][c], xi[q].e[v]);
                        accN[q][v] = select_of(ins[v][c], nn, accN[q][v]);
                        accT[c] = select_of(ins[v][c] && !dia[v][c], nt, accT[c]);
                    }
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const T s = wave_sum(accT[c]);
            if (lane == 0) tpart[w][cg * NC + c] = s;
        }
    };

    load_cg(b0, xj0, 0);
    for (int cg = 0; cg < CGS; cg += 2) {
        if (cg + 1 < CGS) load_cg(b1, xj1, cg + 1);
        compute_cg(b0, xj0, cg);
        if (cg + 1 < CGS) {
            if (cg + 2 < CGS) load_cg(b0, xj0, cg + 2);
            compute_cg(b1, xj1, cg + 1);
        }
    }

    // row sums: one 16-byte store per lane and tile into wsn[panel][row slot]
    T* __restrict__ wsn = a.wsn + p * a.plan.rows_padded + a.plan.shift;
#pragma unroll
    for (int q = 0; q < KTW; ++q) {
        if (valid[q]) {
            Vec<T> o;
#pragma unroll
            for (int v = 0; v < VEC; ++v) o.e[v] = accN[q][v];
            store_vec(wsn + rq[q], o);
        }
    }
    // column sums of the NW waves meet in LDS and are added in wave order
    __syncthreads();
    if (threadIdx.x < C) {
        const int c = threadIdx.x;
        T s = tpart[0][c];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) s = add_of(s, tpart[ww][c]);
        a.wst[(p * a.plan.max_chunks + chunk) * C + c] = s;
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
#pragma unroll 4
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
    SymvPlan<T> p;
    const bool sizing = (A == nullptr);
    p.shift = sizing ? max_row_shift<T>() : row_shift<T>(A, lda);
    p.ntiles = ceil_div(n + p.shift, TR);
    // sizing takes the settings that need the most room: narrow panels, one tile per wave
    int64_t C = tuning().symv_panel_cols > 0 ? tuning().symv_panel_cols : DEFAULT_PANEL_COLS;
    // 16-byte elements: one tile per wave keeps the kernel at three waves per SIMD
    int64_t ktw = tuning().symv_tiles_per_wave > 0 ? tuning().symv_tiles_per_wave
                                                   : (sizeof(T) == 16 ? 1 : DEFAULT_TILES_PER_WAVE);
    if (sizing) { C = 64; ktw = 1; }
    p.panel_cols = C;
    p.npanels = ceil_div(n, C);
    p.chunk_tiles = SY_NW * ktw;
    p.max_chunks = ceil_div(p.ntiles, p.chunk_tiles);
    p.rows_padded = partial_stride<T>(p.ntiles * TR);
    p.xpack_off = 0;
    p.wsn_off = round_up((size_t)n * sizeof(T), WS_ALIGN);
    p.wst_off = p.wsn_off + round_up((size_t)p.npanels * p.rows_padded * sizeof(T), WS_ALIGN);
    p.total_bytes = p.wst_off + round_up((size_t)p.npanels * p.max_chunks * C * sizeof(T), WS_ALIGN);
    return p;
}

namespace {
template <class T, bool HERM, bool LOWER, int CGS, int KTW>
void launch_main(const SymvArgs<T>& a, hipStream_t s) {
    const dim3 grid((unsigned)(ceil_div(a.plan.npanels, XCDS) * XCDS * a.plan.max_chunks));
    hipLaunchKernelGGL((symv_kernel<T, HERM, LOWER, SY_NC, CGS, KTW, SY_NW>), grid, dim3(SY_NW * WAVE), 0, s, a);
}
template <class T, bool HERM, bool LOWER> bool dispatch_main(const SymvArgs<T>& a, hipStream_t s) {
    const int cgs = (int)(a.plan.panel_cols / SY_NC), ktw = (int)(a.plan.chunk_tiles / SY_NW);
    if (cgs == 8 && ktw == 1) launch_main<T, HERM, LOWER, 8, 1>(a, s);
    else if (cgs == 8 && ktw == 2) launch_main<T, HERM, LOWER, 8, 2>(a, s);
    else if (cgs == 16 && ktw == 1) launch_main<T, HERM, LOWER, 16, 1>(a, s);
    else if (cgs == 16 && ktw == 2) launch_main<T, HERM, LOWER, 16, 2>(a, s);
    else return false;
    return true;
}
}  // namespace

template <class T> hipError_t launch_symv(const SymvArgs<T>& a, bool lower, hipStream_t s) {
    constexpr bool HERM = Traits<T>::cplx;
    const bool ok = lower ? dispatch_main<T, HERM, true>(a, s) : dispatch_main<T, HERM, false>(a, s);
    if (!ok) return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 rgrid((unsigned)ceil_div(a.n, RED_ROWS));
    const dim3 rblock(RED_ROWS, RED_PARTS);
    if (lower)
        hipLaunchKernelGGL((symv_reduce_kernel<T, true>), rgrid, rblock, 0, s, a, (int)a.plan.panel_cols);
    else
        hipLaunchKernelGGL((symv_reduce_kernel<T, false>), rgrid, rblock, 0, s, a, (int)a.plan.panel_cols);
    return hipGetLastError();
}

#define KMV_INSTANTIATE_SYMV(T)                                                       \
    template SymvPlan<T> plan_symv<T>(bool, int64_t, const void*, int64_t);           \
    template hipError_t launch_symv<T>(const SymvArgs<T>&, bool, hipStream_t);
KMV_INSTANTIATE_SYMV(float)
KMV_INSTANTIATE_SYMV(double)
KMV_INSTANTIATE_SYMV(cf32)
KMV_INSTANTIATE_SYMV(cf64)

}  // namespace kmv
