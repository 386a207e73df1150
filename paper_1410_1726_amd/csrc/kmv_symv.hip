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
// Kept: the dual use of each element, the register double buffer, blocks of
// the stored triangle as the unit of work.  Different, to fit wave64 and what
// was measured on the MI355X (small writes scattered through a read stream
// cost far more than their bytes; a workgroup that reads a few columns over
// several KiB of consecutive rows streams at full speed; each of the 8 XCDs
// has its own L2):
//  * lanes map to 16-byte row vectors, a wave streams 1 KiB of a column per
//    instruction;
//  * a workgroup owns a chunk of NW*KTW row tiles and walks HORIZONTALLY over
//    a chain of column panels (every Q-th panel that the chunk's rows touch),
//    each wave keeping the non-transposed row sums of its own KTW tiles in
//    registers for the whole chain: they are stored once per chain into a
//    workspace indexed [class][row], instead of once per block;
//  * inside a panel the workgroup sweeps groups of NC columns, so at any
//    moment it reads NC columns over NW consecutive KiB; the next group is in
//    flight (registers) while the current one is used, across panel borders;
//  * the transposed column sums are reduced across the wave once per column
//    group (DPP), meet the other waves' in LDS once per panel (one barrier per
//    panel, none inside) and go to a workspace indexed [panel][chunk][column];
//  * diagonal and edge tiles are handled in the same kernel and the same
//    prefetch pipeline by element loads that never touch the other triangle,
//    so the mirrored copy of Section 6.5 is never built;
//  * consecutive workgroup ids differ in the class, so every XCD sees all row
//    offsets (with a power-of-two leading dimension the lines of one row range
//    in all columns share few L2 sets), and long chains are dispatched first.
// A second kernel adds, in a fixed order, all row sums and column sums that
// belong to y_i and applies alpha and beta (no atomics anywhere).
#include "kmv_launch.hpp"

namespace kmv {

namespace {
constexpr int SY_NW = 4;    // waves per workgroup
// columns per column group (with two tiles per wave: 8 loads in flight per lane
// and buffer, three workgroups per compute unit)
template <class T> constexpr int sy_nc() { return 4; }
constexpr int DEFAULT_PANEL_COLS = 16;
constexpr int64_t TARGET_CHAINS = 2048;   // chains (workgroups) the class count aims at
constexpr int DEFAULT_TILES_PER_WAVE = 2;
constexpr int MAX_CLASSES = 256;
constexpr int RED_ROWS = 16, RED_PARTS = 16;
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
// first / one-past-last panel whose stored part touches the row tiles [tbeg, tend)
template <bool LOWER>
__host__ __device__ __forceinline__ void chunk_panels(int64_t tbeg, int64_t tend, int64_t C, int shift, int64_t TR,
                                                      int64_t npanels, int64_t& plo, int64_t& phi) {
    if (LOWER) {   // panels with tlo(p) < tend
        plo = 0;
        phi = (tend * TR - shift - 1) / C + 1;
        if (phi > npanels) phi = npanels;
    } else {       // panels with thi(p) > tbeg  <=>  (p+1)*C >= tbeg*TR - shift + 1
        const int64_t need = tbeg * TR - shift + 1;
        plo = need > 0 ? (need + C - 1) / C - 1 : 0;
        phi = npanels;
    }
}

template <class T, bool HERM, bool LOWER, int NC, int CGS, int KTW, int NW>
__global__ __launch_bounds__(NW * WAVE, 3) void symv_kernel(SymvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    constexpr int C = NC * CGS;
    constexpr int CT = NW * KTW;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int64_t n = a.n, lda = a.lda;
    const int shift = a.plan.shift;
    const int64_t ntiles = a.plan.ntiles;
    const T* __restrict__ x = a.x;

    // chain = (chunk k, class cls); long chains first: the bottom chunks for
    // 'L', the top chunks for 'U'
    const int64_t Q = a.plan.classes;
    const int64_t cls = (int64_t)blockIdx.x % Q, kord = (int64_t)blockIdx.x / Q;
    const int64_t k = LOWER ? (a.plan.nchunks - 1 - kord) : kord;
    const int64_t tbeg = k * CT;
    int64_t tend = tbeg + CT;
    if (tend > ntiles) tend = ntiles;
    int64_t plo, phi;
    chunk_panels<LOWER>(tbeg, tend, C, shift, TR, a.plan.npanels, plo, phi);
    const int64_t p0 = plo + ((cls - plo) % Q + Q) % Q;            // first panel of the class
    const int64_t np = p0 < phi ? (phi - p0 + Q - 1) / Q : 0;      // panels of this chain
    const int64_t units = np * CGS;

    // this wave's row tiles, their x segment and their row-sum accumulators
    int64_t tq[KTW], rq[KTW];
    bool inrange[KTW], rowfull[KTW];
    Vec<T> xi[KTW];
    T accN[KTW][VEC];
#pragma unroll
    for (int q = 0; q < KTW; ++q) {
        tq[q] = tbeg + w + (int64_t)NW * q;
        inrange[q] = tq[q] < tend;
        const int64_t r0 = tq[q] * TR - shift;
        rowfull[q] = inrange[q] && r0 >= 0 && r0 + TR <= n;
        rq[q] = r0 + (int64_t)lane * VEC;
        if (rowfull[q]) {
            xi[q] = load_cached(x + rq[q]);
        } else {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const int64_t row = rq[q] + v;
                const int64_t rc = row < 0 ? 0 : (row >= n ? n - 1 : row);
                xi[q].e[v] = select_of(inrange[q] && row >= 0 && row < n, x[rc], zero_of<T>());
            }
        }
#pragma unroll
        for (int v = 0; v < VEC; ++v) accN[q][v] = zero_of<T>();
    }

    __shared__ T tpart[2][NW][C];

    // per panel: which of this wave's tiles carry stored elements at all (valid)
    // and which are "fast": all rows exist, the panel is full width and every
    // (row, column) pair lies strictly inside the stored triangle
    auto tile_flags = [&](int64_t p, bool(&valid)[KTW], bool(&fast)[KTW]) {
        const int64_t J0 = p * C;
        int64_t tlo, thi;
        panel_tiles<LOWER>(J0, C, n, shift, TR, ntiles, tlo, thi);
        const bool ragged = (J0 + C > n);
#pragma unroll
        for (int q = 0; q < KTW; ++q) {
            const int64_t r0 = tq[q] * TR - shift;
            valid[q] = inrange[q] && tq[q] >= tlo && tq[q] < thi;
            fast[q] = valid[q] && rowfull[q] && !ragged && (LOWER ? (r0 > J0 + C - 1) : (r0 + TR - 1 < J0));
        }
    };

    // one unit of work = one column group (NC columns) of one panel over all KTW
    // tiles of the wave; the next unit's matrix vectors and x_j scalars are in
    // flight while the current one is being used
    Vec<T> b0[KTW][NC], b1[KTW][NC];
    T xj0[NC], xj1[NC];
    auto load_unit = [&](Vec<T>(&buf)[KTW][NC], T(&xjb)[NC], int64_t u) {
        const int64_t p = p0 + Q * (u / CGS);
        const int64_t jg = p * C + (u % CGS) * NC;
        bool valid[KTW], fast[KTW];
        tile_flags(p, valid, fast);
#pragma unroll
        for (int q = 0; q < KTW; ++q) {
            if (fast[q]) {
                const T* src = a.A + jg * lda + rq[q];
#pragma unroll
                for (int c = 0; c < NC; ++c) buf[q][c] = load_stream(src + (int64_t)c * lda);
            } else if (valid[q]) {
                // edge / diagonal tile: element loads into the same buffer; a pair
                // outside the stored triangle loads the (always stored) diagonal
                // element of its column instead and is skipped at use
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const int64_t row = rq[q] + v;
                    const bool rowok = row >= 0 && row < n;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int64_t j = jg + c;
                        const int64_t jc = j < n ? j : n - 1;
                        const bool ins = rowok && j < n && (LOWER ? row >= j : row <= j);
                        buf[q][c].e[v] = load_elem_stream(a.A + (ins ? row : jc) + jc * lda);
                    }
                }
            }
        }
#pragma unroll
        for (int c = 0; c < NC; ++c) xjb[c] = select_of(jg + c < n, x[jg + c < n ? jg + c : n - 1], zero_of<T>());
    };
    auto compute_unit = [&](const Vec<T>(&buf)[KTW][NC], const T(&xjb)[NC], int64_t u) {
        const int64_t pi = u / CGS;
        const int cg = (int)(u % CGS);
        const int64_t p = p0 + Q * pi;
        const int64_t jg = p * C + (int64_t)cg * NC;
        bool valid[KTW], fast[KTW];
        tile_flags(p, valid, fast);
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
                // edge / diagonal tile (element-loaded above): pairs outside the
                // stored triangle are skipped, the diagonal feeds only the row sum
                // and HEMV takes its real part
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    const int64_t row = rq[q] + v;
                    const bool rowok = row >= 0 && row < n;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int64_t j = jg + c;
                        const bool ins = rowok && j < n && (LOWER ? row >= j : row <= j);
                        const bool dia = (row == j);
                        const T av = buf[q][c].e[v];
                        const T an = select_of(HERM && dia, real_part_only(av), av);
                        T nn = accN[q][v], nt = accT[c];
                        fma_acc(nn, an, xjb[c]);
                        fma_op<HERM>(nt, av, xi[q].e[v]);
                        accN[q][v] = select_of(ins, nn, accN[q][v]);
                        accT[c] = select_of(ins && !dia, nt, accT[c]);
                    }
                }
            }
        }
        T(&tp)[NW][C] = tpart[pi & 1];
#pragma unroll
        for (int c = 0; c < NC; ++c) {
            const T s = wave_sum(accT[c]);
            if (lane == 0) tp[w][cg * NC + c] = s;
        }
        if (cg == CGS - 1) {
            // panel finished: the column sums of the NW waves meet in LDS and are
            // added in wave order.  tpart alternates between two copies, so one
            // barrier per panel is enough.
            __syncthreads();
            if (threadIdx.x < C) {
                const int c = threadIdx.x;
                T s = tp[0][c];
#pragma unroll
                for (int ww = 1; ww < NW; ++ww) s = add_of(s, tp[ww][c]);
                a.wst[(p * a.plan.nchunks + k) * C + c] = s;
            }
        }
    };

    if (units > 0) load_unit(b0, xj0, 0);
    for (int64_t u = 0; u < units; u += 2) {
        if (u + 1 < units) load_unit(b1, xj1, u + 1);
        compute_unit(b0, xj0, u);
        if (u + 1 < units) {
            if (u + 2 < units) load_unit(b0, xj0, u + 2);
            compute_unit(b1, xj1, u + 1);
        }
    }

    // row sums of the whole chain: one 16-byte store per lane and tile into
    // wsn[class][row slot] (zeros where the chain had nothing to add)
    T* __restrict__ wsn = a.wsn + cls * a.plan.rows_padded + shift;
#pragma unroll
    for (int q = 0; q < KTW; ++q) {
        if (inrange[q]) {
            Vec<T> o;
#pragma unroll
            for (int v = 0; v < VEC; ++v) o.e[v] = accN[q][v];
            store_vec_stream(wsn + rq[q], o);
        }
    }
}

// y_i = alpha * ( sum over classes of wsn[class][i] + sum over chunks of
// wst[panel(i)][chunk][i] ) + beta*y_i.  blockDim = (RED_ROWS, RED_PARTS): part g
// adds the classes g, g+RED_PARTS, ... and then the chunks kbeg+g, kbeg+g+
// RED_PARTS, ... in ascending order; the parts meet in LDS and are added in
// part order, so the result does not depend on scheduling.
template <class T, bool LOWER>
__global__ __launch_bounds__(RED_ROWS * RED_PARTS) void symv_reduce_kernel(SymvArgs<T> a) {
    constexpr int TR = tile_rows<T>();
    const int lx = threadIdx.x, g = threadIdx.y;
    const int64_t i = (int64_t)blockIdx.x * RED_ROWS + lx;
    const int shift = a.plan.shift;
    const int64_t C = a.plan.panel_cols;
    __shared__ T part[RED_PARTS][RED_ROWS];
    T s = zero_of<T>();
    if (i < a.n) {
        const T* __restrict__ wsn = a.wsn + i + shift;
#pragma unroll 4
        for (int64_t q = g; q < a.plan.classes; q += RED_PARTS) s = add_of(s, wsn[q * a.plan.rows_padded]);
        // chunks whose row tiles intersect the tile range of the panel of column i
        const int64_t pi = i / C;
        int64_t tlo, thi;
        panel_tiles<LOWER>(pi * C, C, a.n, shift, TR, a.plan.ntiles, tlo, thi);
        const int64_t kbeg = tlo / a.plan.chunk_tiles, kend = (thi - 1) / a.plan.chunk_tiles + 1;
        const T* __restrict__ wst = a.wst + pi * a.plan.nchunks * C + (i - pi * C);
#pragma unroll 4
        for (int64_t k = kbeg + g; k < kend; k += RED_PARTS) s = add_of(s, wst[k * C]);
    }
    part[g][lx] = s;
    __syncthreads();
    if (g == 0 && i < a.n) {
        T tot = part[0][lx];
#pragma unroll
        for (int gg = 1; gg < RED_PARTS; ++gg) tot = add_of(tot, part[gg][lx]);
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
    int64_t C = tuning().symv_panel_cols > 0 ? tuning().symv_panel_cols : DEFAULT_PANEL_COLS;
    // chunks of about 1024 rows (512 for 16-byte elements): one 256-row tile per wave in single precision
    int64_t ktw = tuning().symv_tiles_per_wave > 0 ? tuning().symv_tiles_per_wave
                                                   : (sizeof(T) == 4 ? 1 : DEFAULT_TILES_PER_WAVE);
    if (sizing) { C = 16; ktw = 1; }   // sizing takes the settings that need the most room
    p.panel_cols = C;
    p.npanels = ceil_div(n, C);
    p.chunk_tiles = SY_NW * ktw;
    p.nchunks = ceil_div(p.ntiles, p.chunk_tiles);
    // classes: a power of two between 32 and 128 that gives about TARGET_CHAINS
    // chains (measured: fewer chains leave compute units idle at the end, more
    // only add row-sum vectors), never more than there are panels
    int64_t Q = tuning().symv_classes;
    if (Q <= 0) {
        Q = 32;
        while (Q < 128 && Q * p.nchunks < TARGET_CHAINS) Q *= 2;
    }
    if (sizing) Q = MAX_CLASSES;
    else if (Q > p.npanels) Q = p.npanels;
    p.classes = Q;
    p.rows_padded = partial_stride<T>(p.ntiles * TR);
    p.xpack_off = 0;
    p.wsn_off = round_up((size_t)n * sizeof(T), WS_ALIGN);
    p.wst_off = p.wsn_off + round_up((size_t)Q * p.rows_padded * sizeof(T), WS_ALIGN);
    p.total_bytes = p.wst_off + round_up((size_t)p.npanels * p.nchunks * C * sizeof(T), WS_ALIGN);
    return p;
}

namespace {
template <class T, bool HERM, bool LOWER, int C, int KTW>
void launch_main(const SymvArgs<T>& a, hipStream_t s) {
    const dim3 grid((unsigned)(a.plan.nchunks * a.plan.classes));
    hipLaunchKernelGGL((symv_kernel<T, HERM, LOWER, sy_nc<T>(), C / sy_nc<T>(), KTW, SY_NW>), grid, dim3(SY_NW * WAVE),
                       0, s, a);
}
template <class T, bool HERM, bool LOWER> bool dispatch_main(const SymvArgs<T>& a, hipStream_t s) {
    const int cols = (int)a.plan.panel_cols, ktw = (int)(a.plan.chunk_tiles / SY_NW);
    if (cols == 16 && ktw == 1) launch_main<T, HERM, LOWER, 16, 1>(a, s);
    else if (cols == 16 && ktw == 2) launch_main<T, HERM, LOWER, 16, 2>(a, s);
    else if (cols == 32 && ktw == 1) launch_main<T, HERM, LOWER, 32, 1>(a, s);
    else if (cols == 32 && ktw == 2) launch_main<T, HERM, LOWER, 32, 2>(a, s);
    else if (cols == 64 && ktw == 1) launch_main<T, HERM, LOWER, 64, 1>(a, s);
    else if (cols == 64 && ktw == 2) launch_main<T, HERM, LOWER, 64, 2>(a, s);
    else if (cols == 128 && ktw == 1) launch_main<T, HERM, LOWER, 128, 1>(a, s);
    else if (cols == 128 && ktw == 2) launch_main<T, HERM, LOWER, 128, 2>(a, s);
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
        hipLaunchKernelGGL((symv_reduce_kernel<T, true>), rgrid, rblock, 0, s, a);
    else
        hipLaunchKernelGGL((symv_reduce_kernel<T, false>), rgrid, rblock, 0, s, a);
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
