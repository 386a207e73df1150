// GEMV kernels for gfx950: y <- alpha*op(A)*x + beta*y, A column major.
//
// The paper's two general kernels (Section 6.1, kernels 1 and 2; Algorithms
// "Non-transposed GEMV" and "Transposed GEMV") walk the matrix in blocks with
// a register double buffer (Section 6.3), reduce once at the end and add the
// result into y with atomics (Section 6.2).  What is kept here: the traversal
// directions, one reduction per workgroup at the very end, the prefetch of the
// next block into a second register buffer, and the balanced split of a block
// row / block column over several workgroups (Eqs. local_workload and
// starting_point).  What is different: lanes map to 16-byte row vectors so a
// wave64 streams 1 KiB of a column per instruction; partial results of
// different workgroups go to a workspace and are added in a fixed order by a
// second tiny kernel (no atomics, so results are reproducible and beta is
// applied in the same pass instead of a separate SCAL launch, Section 6.4);
// row tiles start on the 128-byte boundary below the first element and the
// leading slots are masked (Section 6.6) without a separate interface.
// Strided batches run the same kernels with the member in the grid's third dimension; members with short
// columns have a kernel of their own at the end of this file (one wave per member).
#include "kmv_launch.hpp"

namespace kmv {

// ------------------------------------------------------------------ GEMV-N --
// grid.x : blocks of NW*RT row tiles (one tile = 64*VEC rows); a wave owns RT
//          tiles that lie NW tiles apart, so that for every column the NW waves
//          of a workgroup read NW consecutive KiB, RT times
// grid.y : column splits; each workgroup walks its column range horizontally.
// Lanes own rows, so no cross-lane reduction is needed; x_j is wave uniform
// and comes through scalar loads.  A block = U columns x RT tiles of 16-byte
// row vectors plus the U x values, fetched one block ahead of its use.
// Edge tiles (rows before the first or after the last row) run the same
// pipeline with the lanes' load positions clamped into the column: the lanes
// outside compute sums of rows that do not exist, which are dropped.
// The workgroup's columns are c0, c0 + cs, ..., cw of them (cs > 1: the columns of one alignment class).
template <class T, int U, int RT, int NW, bool EDGE>
__device__ __forceinline__ void gemv_n_walk(const GemvArgs<T>& a, const int64_t (&r)[RT], int64_t c0, int64_t cw, int64_t cs,
                                            T (&acc)[RT][Traits<T>::VEC]) {
    constexpr int VEC = Traits<T>::VEC;
    const int64_t lda = a.lda;
    const T* __restrict__ x = a.x;
    const T* __restrict__ A = a.A;
    // edge tile: every lane loads its 16 bytes from a position clamped into the
    // column (no branch, same loads as an interior tile); at use the elements are
    // moved to where the lane's existing rows expect them
    int64_t rl[RT];
    int dsh[RT];
    int cut[RT];            // wave uniform: the tile is cut by the first or the last row (only those pay for the moves)
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        rl[t] = r[t];
        dsh[t] = 0;
        cut[t] = 0;
        if (EDGE) {
            rl[t] = r[t] < 0 ? 0 : (r[t] + VEC > a.m ? a.m - VEC : r[t]);
            dsh[t] = (int)(r[t] - rl[t]);
            const int64_t r0 = r[t] - (int64_t)(threadIdx.x & (WAVE - 1)) * VEC;
            cut[t] = __builtin_amdgcn_readfirstlane((int)(r0 < 0 || r0 + WAVE * VEC > a.m));
        }
    }
    Vec<T> b0[U][RT], b1[U][RT];
    T xb0[U], xb1[U];
    const int64_t cstride = cs * lda;
    auto load_blk = [&](Vec<T>(&buf)[U][RT], T(&xb)[U], int64_t j) {
        const T* q = A + j * lda;
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < RT; ++t) buf[u][t] = load_stream(q + (int64_t)u * cstride + rl[t]);
#pragma unroll
        for (int u = 0; u < U; ++u) xb[u] = x[j + u * cs];
    };
    auto compute_blk = [&](const Vec<T>(&buf)[U][RT], const T(&xb)[U]) {
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
            for (int t = 0; t < RT; ++t) {
                Vec<T> v = buf[u][t];
                if (EDGE && cut[t]) v = shift_elems(v, dsh[t]);
#pragma unroll
                for (int e = 0; e < VEC; ++e) fma_acc(acc[t][e], v.e[e], xb[u]);
            }
    };
    const int64_t nblk = cw / U;
    if (nblk > 0) load_blk(b0, xb0, c0);
    for (int64_t b = 0; b < nblk; b += 2) {
        const int64_t j = c0 + b * U * cs;
        if (b + 1 < nblk) load_blk(b1, xb1, j + U * cs);
        compute_blk(b0, xb0);
        if (b + 1 < nblk) {
            if (b + 2 < nblk) load_blk(b0, xb0, j + 2 * U * cs);
            compute_blk(b1, xb1);
        }
    }
    for (int64_t i = nblk * U; i < cw; ++i) {
        const int64_t j = c0 + i * cs;
        const T xj = x[j];
#pragma unroll
        for (int t = 0; t < RT; ++t) {
            Vec<T> v = load_stream(A + j * lda + rl[t]);
            if (EDGE && cut[t]) v = shift_elems(v, dsh[t]);
#pragma unroll
            for (int e = 0; e < VEC; ++e) fma_acc(acc[t][e], v.e[e], xj);
        }
    }
}

// fewer rows than one 16-byte vector: plain element loop (m <= 3)
template <class T, int RT>
__device__ __forceinline__ void gemv_n_few_rows(const GemvArgs<T>& a, const int64_t (&r)[RT], int64_t c0, int64_t cw,
                                                T (&acc)[RT][Traits<T>::VEC]) {
    constexpr int VEC = Traits<T>::VEC;
    for (int64_t j = c0; j < c0 + cw; ++j) {
        const T xj = a.x[j];
#pragma unroll
        for (int t = 0; t < RT; ++t)
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                int64_t row = r[t] + e;
                row = row < 0 ? 0 : (row >= a.m ? a.m - 1 : row);
                fma_acc(acc[t][e], a.A[row + j * a.lda], xj);
            }
    }
}

template <class T, int NW, int U, int RT, bool PTRS = false>
__global__ __launch_bounds__(NW * WAVE) void gemv_n_kernel(GemvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    // grid.x = column split (fastest: consecutive ids, i.e. different XCDs, share
    // the rows and differ in the columns), grid.y = block of row tiles
    const int64_t tbase = (int64_t)blockIdx.y * (NW * RT) + w;   // tiles tbase + NW*t, t < RT
    if (tbase >= a.plan.ntiles) return;
    select_member<PTRS>(a, blockIdx.z);   // member of a batch (strides all zero for a single product)

    int64_t cw, c0, cs = 1;
    int shift = a.plan.shift;
    int64_t ntiles = a.plan.ntiles, part_off = a.plan.part_off;
    if (a.plan.period > 1) {
        // columns of one alignment class: class, class + period, ...; the row tiles start on the
        // 128-byte boundary below the class's first element
        const int64_t P = a.plan.period, cls = (int64_t)blockIdx.x % P, q = (int64_t)blockIdx.x / P;
        const int64_t ncls = cls < a.n ? (a.n - cls + P - 1) / P : 0;
        int64_t k0;
        partition(ncls, a.plan.splits / P, q, cw, k0);
        c0 = cls + P * k0;
        cs = P;
        shift = (int)((uintptr_t)(a.A + cls * a.lda) % 128 / sizeof(T));
        ntiles = ceil_div(a.m + shift, (int64_t)TR);
        if (tbase >= ntiles) return;
    } else {
        partition(a.n, a.plan.splits, blockIdx.x, cw, c0);
    }
    int64_t r[RT];          // first row slot of this lane in each tile (may be outside [0, m))
    bool interior = true;   // all RT tiles fully inside the matrix (wave uniform)
#pragma unroll
    for (int t = 0; t < RT; ++t) {
        const int64_t r0 = (tbase + (int64_t)NW * t) * TR - shift;
        r[t] = r0 + (int64_t)lane * VEC;
        interior = interior && (r0 >= 0) && (r0 + TR <= a.m);
    }
    T acc[RT][VEC];
#pragma unroll
    for (int t = 0; t < RT; ++t)
#pragma unroll
        for (int v = 0; v < VEC; ++v) acc[t][v] = zero_of<T>();

    if (interior) gemv_n_walk<T, U, RT, NW, false>(a, r, c0, cw, cs, acc);
    else if (a.m >= VEC) gemv_n_walk<T, U, RT, NW, true>(a, r, c0, cw, cs, acc);
    else gemv_n_few_rows<T, RT>(a, r, c0, cw, acc);

#pragma unroll
    for (int t = 0; t < RT; ++t) {
        if (tbase + (int64_t)NW * t >= ntiles) continue;   // tile beyond the matrix: nothing to store
        if (a.plan.splits == 1) {
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                const int64_t row = r[t] + v;
                if (row >= 0 && row < a.m) {
                    T* yp = a.y + row * a.incy;
                    *yp = epilogue(scalar_of(a.alpha, a.alpha_dev), acc[t][v], scalar_of(a.beta, a.beta_dev), yp);
                }
            }
        } else {
            Vec<T> out;
#pragma unroll
            for (int v = 0; v < VEC; ++v) out.e[v] = acc[t][v];
            store_vec(a.partial + (int64_t)blockIdx.x * a.plan.part_stride + (r[t] + part_off), out);
        }
    }
}

// Short matrices (one or two row tiles in all): the NW waves of a workgroup would
// mostly idle in the kernel above, so here NW/tiles waves share a row tile and
// split the workgroup's column slice once more; their row sums meet in LDS and
// are added in wave order.  grid.x = column splits.
template <class T, int NW, int U>
__global__ __launch_bounds__(NW * WAVE) void gemv_n_short_kernel(GemvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int nt = (int)a.plan.ntiles;   // 1 or 2 (the launcher checks)
    const int ws = NW / nt;              // waves per row tile
    const int tile = w / ws, sub = w % ws;

    int64_t cw, c0, cws, c0s;
    partition(a.n, a.plan.splits, blockIdx.x, cw, c0);
    partition(cw, ws, sub, cws, c0s);
    int64_t r[1];
    const int64_t r0 = (int64_t)tile * TR - a.plan.shift;
    r[0] = r0 + (int64_t)lane * VEC;
    const bool interior = (r0 >= 0) && (r0 + TR <= a.m);
    T acc[1][VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[0][v] = zero_of<T>();
    if (interior) gemv_n_walk<T, U, 1, NW, false>(a, r, c0 + c0s, cws, 1, acc);
    else if (a.m >= VEC) gemv_n_walk<T, U, 1, NW, true>(a, r, c0 + c0s, cws, 1, acc);
    else gemv_n_few_rows<T, 1>(a, r, c0 + c0s, cws, acc);

    __shared__ T red[NW][TR];
#pragma unroll
    for (int v = 0; v < VEC; ++v) red[w][lane * VEC + v] = acc[0][v];
    __syncthreads();
    if (sub != 0) return;
    Vec<T> out;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        T sum = red[w][lane * VEC + v];
        for (int k = 1; k < ws; ++k) sum = add_of(sum, red[w + k][lane * VEC + v]);
        out.e[v] = sum;
    }
    if (a.plan.splits == 1) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            const int64_t row = r[0] + v;
            if (row >= 0 && row < a.m) {
                T* yp = a.y + row * a.incy;
                *yp = epilogue(scalar_of(a.alpha, a.alpha_dev), out.e[v], scalar_of(a.beta, a.beta_dev), yp);
            }
        }
    } else {
        store_vec(a.partial + (int64_t)blockIdx.x * a.plan.part_stride + (r[0] + a.plan.shift), out);
    }
}

// ------------------------------------------------------------------ GEMV-T --
// grid.x : groups of NC columns; grid.y : row splits.  The NW waves of a
// workgroup take row tiles round robin and walk down their columns; each lane
// keeps one accumulator per column; one wave reduction per column and one LDS
// step across the waves at the very end.
// WCOLS (short matrices, a few row tiles only): every wave owns NC columns of its
// own and walks all tiles of the split alone; nothing crosses waves.
// BANDS: the instance with the banded main loop below (it costs about 90 registers per lane, which the launches with
// little work per workgroup - row splits, small matrices - cannot spare: they keep the instance without it).
template <class T, bool CONJ, int NC, int NW_, bool WCOLS, bool PTRS = false, bool BANDS = false>
__global__ __launch_bounds__(NW_ * WAVE) void gemv_t_kernel(GemvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    constexpr int NW = WCOLS ? 1 : NW_;   // waves that share the tiles of a column group
    const int lane = threadIdx.x & (WAVE - 1);
    const int wv = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int w = WCOLS ? 0 : wv;
    select_member<PTRS>(a, blockIdx.z);   // member of a batch (strides all zero for a single product)
    const T* __restrict__ x = a.x;
    // A workgroup takes the column groups gx = blockIdx.x, blockIdx.x + gridDim.x, ...: one each in the usual launch,
    // several when the planner starts fewer workgroups than there are groups.
    const int64_t ngroups = (WCOLS || a.plan.t_groups <= 0) ? (int64_t)gridDim.x : a.plan.t_groups;
    for (int64_t gx = blockIdx.x; gx < ngroups; gx += gridDim.x) {
    int64_t j0 = WCOLS ? (gx * NW_ + wv) * NC : gx * NC;
    if (WCOLS && j0 >= a.n) return;   // a whole wave past the last column (no barrier in this form, one group per workgroup)
    int64_t ntiles = a.plan.ntiles;
    int shift = a.plan.shift;
    // the workgroup's columns are j0, j0 + js, ...; with alignment classes (period > 1) they are columns of
    // one class, and the row tiles start on the 128-byte boundary below that class's first element
    int64_t js = 1, jlast = a.n - 1;
    if (!WCOLS && a.plan.period > 1) {
        const int64_t P = a.plan.period, cls = gx % P;
        j0 = cls + P * (gx / P) * NC;
        js = P;
        jlast = cls < a.n ? cls + (a.n - 1 - cls) / P * P : 0;    // last column of the class (column 0 if it has none)
        shift = (int)((uintptr_t)(a.A + (cls < a.n ? cls : 0) * a.lda) % 128 / sizeof(T));
        ntiles = ceil_div(a.m + shift, (int64_t)TR);
    }

    int64_t tw, ts;
    partition(ntiles, a.plan.splits, blockIdx.y, tw, ts);

    // columns past n-1 are clamped: they read legitimate data that is dropped
    const T* __restrict__ col[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const int64_t j = (j0 + c * js < a.n) ? (j0 + c * js) : jlast;
        col[c] = a.A + j * a.lda;
    }
    T acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[c] = zero_of<T>();

    auto is_interior = [&](int64_t t) { return (t * TR - shift >= 0) && ((t + 1) * TR - shift <= a.m); };
    // edge tile: the same 16-byte loads as an interior tile, taken at a position clamped into the
    // column (all issued before the first use); at use the elements are moved to where the lane's
    // rows expect them and rows that do not exist are skipped.  Fewer rows than one vector: element
    // loads with the row index clamped.
    auto masked_tile = [&](int64_t t) {
        const int64_t r = t * TR - shift + (int64_t)lane * VEC;
        bool ok[VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) ok[v] = r + v >= 0 && r + v < a.m;
        if (a.m >= VEC) {     // wave uniform
            const int64_t rc = r < 0 ? 0 : (r + VEC > a.m ? a.m - VEC : r);
            const int dsh = (int)(r - rc);
            Vec<T> xv = load_cached(x + rc), av[NC];
#pragma unroll
            for (int c = 0; c < NC; ++c) av[c] = load_stream(col[c] + rc);
            xv = shift_elems(xv, dsh);
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const Vec<T> sv = shift_elems(av[c], dsh);
#pragma unroll
                for (int v = 0; v < VEC; ++v) {
                    T nacc = acc[c];
                    fma_op<CONJ>(nacc, sv.e[v], xv.e[v]);
                    acc[c] = select_of(ok[v], nacc, acc[c]);
                }
            }
            return;
        }
        T xv[VEC], av[NC][VEC];
#pragma unroll
        for (int v = 0; v < VEC; ++v) {
            int64_t row = r + v;
            row = row < 0 ? 0 : (row >= a.m ? a.m - 1 : row);
            xv[v] = x[row];
#pragma unroll
            for (int c = 0; c < NC; ++c) av[c][v] = load_elem_stream(col[c] + row);
        }
#pragma unroll
        for (int c = 0; c < NC; ++c)
#pragma unroll
            for (int v = 0; v < VEC; ++v) {
                T nacc = acc[c];
                fma_op<CONJ>(nacc, av[c][v], xv[v]);
                acc[c] = select_of(ok[v], nacc, acc[c]);
            }
    };

    // interior tiles [ilo, ihi) of this split; an edge tile at either end is done
    // by wave 0 / wave NW-1 on its own
    int64_t ilo = ts, ihi = ts + tw;
    const bool first_edge = tw > 0 && ilo == 0 && !is_interior(0);
    if (first_edge) ++ilo;
    const bool last_edge = ihi > ilo && ihi == ntiles && !is_interior(ntiles - 1);
    if (last_edge) --ihi;
    const int64_t ni = ihi - ilo;
    if (first_edge && w == 0) masked_tile(0);
    if (last_edge && w == NW - 1) masked_tile(ntiles - 1);

    // Bands first: while NW * RT interior tiles are left, wave w takes RT CONSECUTIVE tiles (w * RT ... of the band)
    // and walks the workgroup's columns CB at a time, x of its tiles in registers - every column is read in runs
    // of NW * RT KiB instead of one tile per wave and eight columns at once.  Two register buffers of RT x CB
    // vectors, the next block (or the next band's first, with its x) in flight while one is used.  The bands are
    // taken in an order rotated by the column group, as the tiles below.
    int64_t ilo_rest = ilo, ni_rest = ni;
    if constexpr (BANDS && !WCOLS) {
        constexpr int RT = 4, CB = 2, NBLK = NC / CB;
        static_assert(NC % CB == 0 && NBLK % 2 == 0, "an even number of blocks per band keeps the buffers' roles fixed");
        const int64_t band = (int64_t)NW * RT, nbands = ni / band;
        if (nbands > 0) {
            const int64_t brot = (gx * 37) % nbands;
            auto band_row = [&](int64_t b) {
                int64_t bi = b + brot;
                if (bi >= nbands) bi -= nbands;
                return (ilo + bi * band + (int64_t)w * RT) * TR - shift + (int64_t)lane * VEC;
            };
            Vec<T> xa[RT], xb[RT], b0[RT][CB], b1[RT][CB];
            auto load_x = [&](Vec<T>(&xv)[RT], int64_t r) {
#pragma unroll
                for (int t = 0; t < RT; ++t) xv[t] = load_cached(x + r + t * TR);
            };
            auto load_block = [&](Vec<T>(&buf)[RT][CB], int64_t r, int blk) {
#pragma unroll
                for (int cc = 0; cc < CB; ++cc)
#pragma unroll
                    for (int t = 0; t < RT; ++t) buf[t][cc] = load_stream(col[blk * CB + cc] + r + t * TR);
            };
            auto compute_block = [&](const Vec<T>(&buf)[RT][CB], const Vec<T>(&xv)[RT], int blk) {
#pragma unroll
                for (int cc = 0; cc < CB; ++cc)
#pragma unroll
                    for (int t = 0; t < RT; ++t)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) fma_op<CONJ>(acc[blk * CB + cc], buf[t][cc].e[v], xv[t].e[v]);
            };
            int64_t r = band_row(0);
            load_x(xa, r);
            load_block(b0, r, 0);
            for (int64_t b = 0; b < nbands; ++b) {
                const int64_t rn = b + 1 < nbands ? band_row(b + 1) : r;
#pragma unroll
                for (int blk = 0; blk < NBLK; blk += 2) {
                    load_block(b1, r, blk + 1);
                    compute_block(b0, xa, blk);
                    if (blk + 2 < NBLK) {
                        load_block(b0, r, blk + 2);
                    } else if (b + 1 < nbands) {
                        load_x(xb, rn);
                        load_block(b0, rn, 0);
                    }
                    compute_block(b1, xa, blk + 1);
                }
#pragma unroll
                for (int t = 0; t < RT; ++t) xa[t] = xb[t];
                r = rn;
            }
            ilo_rest = ilo + nbands * band;
            ni_rest = ni - nbands * band;
        }
    }

    // The waves take the interior tiles round robin, starting at a tile that
    // depends on the column group: workgroups that run at the same time then
    // sit at different row offsets (with a power-of-two leading dimension equal
    // row offsets of different columns share few L2 sets).  The rotation depends
    // only on the arguments, so results stay reproducible.
    const int64_t rot = (ni_rest > 0 && !WCOLS) ? (gx * 37) % ni_rest : 0;
    const int64_t cnt = ni_rest > w ? (ni_rest - w + NW - 1) / NW : 0;   // tiles of this wave
    {
        Vec<T> x0, x1, b0[NC], b1[NC];
        auto load_tile = [&](Vec<T>& xv, Vec<T>(&buf)[NC], int64_t k) {
            int64_t i = w + k * NW + rot;
            if (i >= ni_rest) i -= ni_rest;
            const int64_t r = (ilo_rest + i) * TR - shift + (int64_t)lane * VEC;
            xv = load_cached(x + r);
#pragma unroll
            for (int c = 0; c < NC; ++c) buf[c] = load_stream(col[c] + r);
        };
        auto compute_tile = [&](const Vec<T>& xv, const Vec<T>(&buf)[NC]) {
#pragma unroll
            for (int c = 0; c < NC; ++c)
#pragma unroll
                for (int v = 0; v < VEC; ++v) fma_op<CONJ>(acc[c], buf[c].e[v], xv.e[v]);
        };
        if (cnt > 0) load_tile(x0, b0, 0);
        for (int64_t k = 0; k < cnt; k += 2) {
            if (k + 1 < cnt) load_tile(x1, b1, k + 1);
            compute_tile(x0, b0);
            if (k + 1 < cnt) {
                if (k + 2 < cnt) load_tile(x0, b0, k + 2);
                compute_tile(x1, b1);
            }
        }
    }

    __shared__ T red[NW][NC];
    T mine = zero_of<T>();
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const T s = wave_sum(acc[c]);
        if (WCOLS) mine = select_of(lane == c, s, mine);
        else if (lane == 0) red[w][c] = s;
    }
    if (!WCOLS) __syncthreads();
    if (WCOLS ? lane < NC : threadIdx.x < NC) {
        const int c = WCOLS ? lane : threadIdx.x;
        const int64_t j = j0 + c * js;
        if (j < a.n) {
            T s = WCOLS ? mine : red[0][c];
            for (int ww = 1; ww < NW; ++ww) s = add_of(s, red[ww][c]);
            if (a.plan.splits == 1) {
                T* yp = a.y + j * a.incy;
                *yp = epilogue(scalar_of(a.alpha, a.alpha_dev), s, scalar_of(a.beta, a.beta_dev), yp);
            } else {
                a.partial[(int64_t)blockIdx.y * a.plan.part_stride + j] = s;
            }
        }
    }
    if (!WCOLS && gx + gridDim.x < ngroups) __syncthreads();   // red is written again for the next group
    }
}

// ------------------------------------------------------------- host side ----
namespace {
constexpr int GN_NW = 4;                // GEMV-N: waves per workgroup
constexpr int GN_LOADS = 8;             // GEMV-N: 16-byte loads per lane and prefetch block (columns x tiles)
constexpr int GN_WGS_PER_CU = 2;        // GEMV-N: workgroups per compute unit the column split aims at
constexpr int GT_NC = 8, GT_NW = 4;     // GEMV-T: columns per workgroup, waves per workgroup
constexpr int GT_BAND = GT_NW * 4;      // GEMV-T: row tiles of a band (four consecutive tiles per wave)
constexpr int64_t MAX_SPLITS = 256;
constexpr int64_t SHORT_T_TILES = 2;         // GEMV-T: up to this many row tiles every wave owns its columns
constexpr int64_t DEFAULT_WG_TARGET = 2048;   // about 8 workgroups per compute unit
constexpr int64_t DEFAULT_GN_ROW_TILES = 1;
}  // namespace

// Workgroups of gemv_n_kernel<T, ., ., rt> that one round should hold: compute
// units x min(occupancy, 2), queried once per instance.  A compute unit's share
// of the HBM bandwidth is capped, so the kernel is fastest when every compute
// unit holds the same number of equally long workgroups; measured with the split
// counts alternating in one process, two workgroups (8 waves with 8-16 loads in
// flight each) per compute unit beat the full occupancy of four by 1-12%, most
// below n = 8192 where fewer, longer workgroups also mean fewer partial sums.
template <class T> int64_t gemv_n_slots(int64_t rt) {
    static int64_t caches[MAX_CACHED_DEVICES][5] = {};
    const int di = cached_device_index();
    if (rt < 1 || rt > 4 || di < 0) return 0;
    int64_t(&cache)[5] = caches[di];
    if (cache[rt] == 0) {
        int dev = 0, cus = 0, nb = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess) {
            if (rt == 1) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, gemv_n_kernel<T, GN_NW, GN_LOADS, 1>, GN_NW * WAVE, 0);
            else if (rt == 2) e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, gemv_n_kernel<T, GN_NW, GN_LOADS / 2, 2>, GN_NW * WAVE, 0);
            else e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, gemv_n_kernel<T, GN_NW, GN_LOADS / 4, 4>, GN_NW * WAVE, 0);
        }
        cache[rt] = (e == hipSuccess && cus > 0 && nb > 0) ? (int64_t)cus * (nb < GN_WGS_PER_CU ? nb : GN_WGS_PER_CU) : -1;
        (void)hipGetLastError();
    }
    return cache[rt];
}

// compute units of the current device (0 when it cannot be asked)
inline int64_t device_cus() {
    static int64_t cache[MAX_CACHED_DEVICES] = {};
    const int di = cached_device_index();
    if (di < 0) return 0;
    if (cache[di] == 0) {
        int dev = 0, cus = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        cache[di] = (e == hipSuccess && cus > 0) ? cus : -1;
        (void)hipGetLastError();
    }
    return cache[di] > 0 ? cache[di] : 0;
}

// Column splits for `rb` row blocks: the largest count that still fits one
// resident round (rb*s <= slots), or two rounds when one round would leave
// more than a tenth of the slots empty and two rounds fill better.
inline int64_t choose_splits(int64_t rb, int64_t slots, int64_t cap) {
    if (slots <= 0) return 0;
    int64_t best = 1;
    double best_eff = 0.0;
    for (int rounds = 1; rounds <= 2; ++rounds) {
        int64_t s = rounds * slots / rb;
        if (s < 1) s = 1;
        if (s > cap) s = cap;
        const int64_t w = rb * s;
        const double eff = (double)w / (double)(ceil_div(w, slots) * slots);
        if (eff > best_eff + 0.1 || (rounds == 1)) { best = s; best_eff = eff; }
    }
    return best;
}

template <class T> GemvPlan<T> plan_gemv(bool notrans, int64_t m, int64_t n, const void* A, int64_t lda, bool classes) {
    constexpr int TR = tile_rows<T>();
    GemvPlan<T> p;
    p.row_tiles = 1;
    p.t_groups = 0;
    p.t_wgs = 0;
    const bool sizing = (A == nullptr);
    // the caller's tuning values, plus the measured settings of this size where the caller left the choice open
    const Tuning tn = sizing || !classes ? tuning() : tuned(notrans ? 'N' : 'T', prec_char<T>(), m, n, lda * (int64_t)sizeof(T));
    p.shift = sizing ? max_row_shift<T>() : row_shift<T>(A, lda);
    p.ntiles = ceil_div(m + p.shift, TR);
    // alignment classes: worth it when the columns are long and there are several workgroups' worth per class
    // (measured: a stream of 1 KiB loads that start 8 .. 64 bytes off a 128-byte boundary runs 4-9% slower,
    // nine lines per load instead of eight)
    p.period = 1;
    const uint64_t step = ((uint64_t)lda * sizeof(T)) % 128;
    if (classes && !sizing && step != 0 && tn.gemv_align_classes != 1) {
        uint64_t g = step, h = 128;
        while (h) { const uint64_t t = g % h; g = h; h = t; }
        const int64_t P = (int64_t)(128 / g);
        // by default for the transposed product only (SGEMV/DGEMV/CGEMV-T at n = 17001, lda = n: 6-7% faster; the
        // non-transposed kernel gains 0-3% at best, its split counts have to be multiples of the period)
        if (tn.gemv_align_classes == 2 || (!notrans && (double)m * sizeof(T) >= 16384.0 && n >= 64 * P)) {
            p.period = P;
            p.shift = max_row_shift<T>();
            p.ntiles = ceil_div(m + p.shift, TR);
        }
    }
    const int64_t target = tn.wg_target > 0 ? tn.wg_target : DEFAULT_WG_TARGET;
    int64_t s;
    const int64_t max_splits = MAX_SPLITS;
    p.short_form = 0;
    const int64_t short_mode = tn.gemv_short;   // 0 = automatic, 1 = never, 2 = whenever the kernels allow
    if (notrans && !sizing && short_mode != 1 && p.ntiles <= 2) {
        // one or two row tiles: NW/ntiles waves per tile split the columns once more
        p.short_form = 1;
        const int64_t ws = GN_NW / p.ntiles;
        int64_t cap = n / (GN_LOADS * ws) > 1 ? n / (GN_LOADS * ws) : 1;   // a block of columns per wave at least
        s = tn.gemv_n_splits > 0 ? tn.gemv_n_splits : (tn.wg_target > 0 ? tn.wg_target : 256);   // measured best
        if (s > cap) s = cap;
        p.part_stride = partial_stride<T>(p.ntiles * TR);
    } else if (!notrans && !sizing && short_mode != 1 && (p.ntiles <= SHORT_T_TILES || (short_mode == 2 && p.ntiles <= 64))) {
        // a few row tiles: every wave takes 8 columns of its own through all tiles, one launch
        p.short_form = 1;
        s = 1;
        p.part_stride = partial_stride<T>(n);
    } else if (notrans) {
        int64_t cap = n / 32 > 1 ? n / 32 : 1;   // at least 32 columns per split
        if (cap > MAX_SPLITS) cap = MAX_SPLITS;
        s = tn.gemv_n_splits;
        p.row_tiles = tn.gemv_n_row_tiles > 0 ? tn.gemv_n_row_tiles : DEFAULT_GN_ROW_TILES;
        if (tn.gemv_n_row_tiles <= 0 && s <= 0 && tn.wg_target <= 0 && !sizing) {
            // Large matrices: ONE workgroup per compute unit, each over 16 row tiles (four per wave, two
            // columns per prefetch block).  Measured with the settings alternating in one process this
            // is 3-7% faster than two workgroups per compute unit from about 256 MB of matrix on (the
            // read-bandwidth probe peaks at the same shape: one workgroup per compute unit, eight loads
            // in flight per lane), provided the workgroups fill nearly all compute units, their count is a
            // multiple of 8 (the number of XCDs that workgroup ids are dealt to) and the last block of 16
            // row tiles is not much shorter than the others (with one workgroup per compute unit nothing
            // fills in behind a short one; the 4-byte types lost 2-10% whenever it was not full).
            const int64_t cus = gemv_n_slots<T>(4) > 0 ? device_cus() : 0;
            const int64_t rb4 = ceil_div(p.ntiles, GN_NW * 4);
            int64_t step = 8;                      // s must be a multiple of 8 / gcd(rb4, 8)
            for (int64_t d = 8; d >= 1; d /= 2)
                if (rb4 % d == 0) { step = 8 / d; break; }
            int64_t s4 = cus > 0 && rb4 <= cus ? (cus / rb4) / step * step : 0;
            // With every column on the 128-byte grid the loads are whole lines and the memory pipeline saturates
            // before the compute units run out: THREE QUARTERS of them, each with a wider range of columns, stream
            // 1.5-3.5% faster than all of them (measured in s, d and z at n = 16384 ... 40960 with 128 to 256
            // workgroups: best at 176 to 208 of 256, DGEMV-N 32768 1202 -> 1176 us, SGEMV-N 16384 159 -> 152 us; below
            // 11/16 the time rises steeply).  Leading dimensions off the grid behave the other way round (unaligned
            // loads cost address cycles, 192 workgroups are 4-10% slower than 240-256) and keep the full round.
            const bool on_grid = (lda * (int64_t)sizeof(T)) % 128 == 0;
            if (on_grid && s4 >= 1) {
                const int64_t want = cus * 3 / 4;
                int64_t bestd = -1;
                for (int64_t st = step; rb4 * st <= cus; st += step) {
                    const int64_t wgs = rb4 * st, d = wgs > want ? wgs - want : want - wgs;
                    if (wgs * 16 >= cus * 11 && (bestd < 0 || d < bestd)) {
                        bestd = d;
                        s4 = st;
                    }
                }
            }
            if (s4 > cap) s4 = 0;
            const bool big = (double)m * (double)n * sizeof(T) >= 256.0 * 1024 * 1024;
            const bool rows_even = sizeof(T) == 4 ? p.ntiles % (GN_NW * 4) == 0 : p.ntiles * 100 >= rb4 * GN_NW * 4 * 85;
            // 4-byte elements on the grid whose first or last row tile is cut (a sub-block pointer, a ragged row
            // count): the waves that own the cut tiles pay four selects per load for every column, and with one
            // workgroup per compute unit the round waits for them (SGEMV-N on the 16383 x 16383 block at (1, 1) of a
            // 16384 x 16384 matrix: 173 us in this form, 160-164 us with two workgroups per compute unit; the wider
            // types lose nothing: 307 us either way).  They take the general rule below.
            const bool cut4 = sizeof(T) == 4 && on_grid && (p.shift != 0 || (m + p.shift) % TR != 0);
            if (p.period == 1 && big && rows_even && !cut4 && s4 >= 1 && rb4 * s4 * 100 >= cus * (on_grid ? 68 : 85)) {
                p.row_tiles = 4;
                s = s4;
            } else if (p.period == 1 && big && cus > 0 && !cut4) {
                // The same regime for the sizes that rule leaves out (ragged row counts, leading dimensions off
                // the 128-byte grid): still ONE workgroup per compute unit, with the tiles per wave that waste the
                // least of the single round - score = share of the compute units that get a workgroup x share of
                // a workgroup's tile slots that hold rows.  Measured at n = 17001, 20001, 30001 (lda = n) in s, d
                // and z against two workgroups per compute unit: 4-9% faster in eight cases of nine, equal in the
                // ninth; the 4-byte type does best with two tiles per wave, the others with four.
                double best = 0.0;
                for (int64_t rt = 4; rt >= 1; rt /= 2) {
                    const int64_t rbt = ceil_div(p.ntiles, GN_NW * rt);
                    if (rbt > cus || gemv_n_slots<T>(rt) <= 0) continue;
                    int64_t st = cus / rbt;
                    if (st > cap) st = cap;
                    const double fill = (double)(rbt * st) / (double)cus;
                    const double full = (double)p.ntiles / (double)(rbt * GN_NW * rt);
                    const double pref = sizeof(T) == 4 ? (rt == 2 ? 1.0 : 0.93)
                                                       : (rt == 4 ? 1.0 : (rt == 2 ? 0.98 : 0.95));
                    if (fill * full >= 0.80 && fill * full * pref > best) {
                        best = fill * full * pref;
                        p.row_tiles = (int)rt;
                        s = st;
                    }
                }
            }
        }
        // row blocks are the grid's second dimension (at most 65535): very tall matrices take more tiles per wave
        while (p.row_tiles < 4 && ceil_div(p.ntiles, GN_NW * p.row_tiles) > 65535) p.row_tiles *= 2;
        const int64_t rb = ceil_div(p.ntiles, GN_NW * p.row_tiles);
        if (s <= 0 && tn.wg_target <= 0 && !sizing) s = choose_splits(rb, gemv_n_slots<T>(p.row_tiles), cap);
        if (s <= 0) s = ceil_div(target, rb);
        if (s > cap) s = cap;
        if (p.period > 1) {     // every split lies in one class: a multiple of the period (n >= 64 columns per class)
            s = s / p.period * p.period;
            if (s < p.period) s = p.period;
            if (s > MAX_SPLITS) s = MAX_SPLITS / p.period * p.period;
        }
        p.part_stride = partial_stride<T>(p.ntiles * TR + TR);
    } else {
        const int64_t g = n > 0 ? ceil_div(n, GT_NC) : 1;
        // Row splits (and the second kernel that adds the pieces) pay only when the column groups
        // alone leave compute units idle AND a workgroup's 8 columns are long: a lone workgroup streams
        // at about 40 GB/s, the second launch costs 4-5 us.  Measured over shapes from 1024 x 1024 to
        // 65536 x 64 in three precisions: from 192 groups on a single launch is as fast or faster (by
        // up to 28% at n = 2048); below, splitting wins from about 6 us of work per workgroup on, and
        // then at least four splits (two are slower than either one or four).
        int64_t sa = 1;
        if (g < 192 && (double)m * GT_NC * sizeof(T) / 40e3 >= 6.0) {
            sa = ceil_div(512, g);
            if (sa < 4) sa = 4;
        }
        // From 192 groups on: while a group of columns holds less than about 600 KB, eight row splits (many short
        // workgroups that start and end at different times) beat one workgroup per group or per compute unit, whose
        // pipelines all fill and drain together: 8-19% in s for n = 5120 ... 11264, 3-8% up to 15360, 7-11% in d at
        // 3072 ... 7168, 6% in z at 3072 (sweep over n = 2048 ... 20480 in steps of 1024, splits 1 ... 16, with and
        // without the one-workgroup-per-compute-unit form).  Not when the column stride is 16 KB or a multiple of
        // 32 KB: the splits then start in the same memory channels and lose up to 25%, and the unsplit form is the
        // best there (odd multiples of 16 KB from 48 KB on behave like any other stride).
        const double group_bytes = (double)m * GT_NC * sizeof(T);
        const int64_t stride_bytes = lda * (int64_t)sizeof(T);
        if (g >= 192 && !sizing && stride_bytes != 16384 && stride_bytes % 32768 != 0 && group_bytes >= 96e3 && group_bytes < 600e3)
            sa = 8;
        s = tn.gemv_t_splits > 0 ? tn.gemv_t_splits
                                       : (tn.wg_target > 0 ? ceil_div(tn.wg_target, g) : sa);
        const int64_t cap = p.ntiles / (2 * GT_NW) > 1 ? p.ntiles / (2 * GT_NW) : 1;   // two tiles per wave at least
        if (s > cap) s = cap;
        p.part_stride = partial_stride<T>(n);
        p.t_groups = p.period * ceil_div(ceil_div(n > 0 ? n : 1, p.period), (int64_t)GT_NC);
        // One workgroup per compute unit, each taking every 256th group of columns, instead of one workgroup per
        // group: never slower, 3-7% faster around n = 6000 ... 8000, 1-3% up to 16384, below 1% beyond (s, d, c at
        // n = 6144 ... 49152; 192 workgroups, the best count of the non-transposed kernel, lose 1-4% here, 384 lose 6%).
        p.t_wgs = tn.gemv_t_wgs;
        if (p.t_wgs <= 0 && !sizing && s == 1) {
            const int64_t cus = device_cus();
            if (cus > 0 && p.t_groups >= 2 * cus) p.t_wgs = cus;
        }
    }
    if (s > max_splits) s = max_splits;
    if (s < 1) s = 1;
    if (p.short_form) {     // the kernels for short matrices take the columns as they come
        if (p.period > 1) {
            p.shift = 0;
            p.ntiles = ceil_div(m, TR);
        }
        p.period = 1;
    }
    p.splits = s;
    p.part_off = p.period > 1 ? max_row_shift<T>() : p.shift;
    const int64_t lenx = notrans ? n : m;
    p.xpack_off = 0;
    p.partial_off = round_up((size_t)lenx * sizeof(T), WS_ALIGN);
    const int64_t size_splits = sizing ? MAX_SPLITS : (s > 1 ? s : 0);
    p.total_bytes = p.partial_off + round_up((size_t)size_splits * p.part_stride * sizeof(T), WS_ALIGN);
    return p;
}

template <class T> hipError_t launch_gemv_n(const GemvArgs<T>& a, hipStream_t s, int64_t batch) {
    if (batch < 1 || batch > 65535 || (batch > 1 && (a.plan.splits != 1 || a.plan.short_form))) return hipErrorInvalidValue;
    if (a.plan.short_form) {
        if (a.plan.ntiles < 1 || a.plan.ntiles > 2) return hipErrorInvalidValue;
        hipLaunchKernelGGL((gemv_n_short_kernel<T, GN_NW, GN_LOADS>), dim3((unsigned)a.plan.splits), dim3(GN_NW * WAVE), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || a.plan.splits == 1) return e;
        return launch_reduce<T>(a.partial, a.plan.splits, a.plan.part_stride, a.plan.shift, a.m, a.alpha, a.beta, a.alpha_dev, a.beta_dev, a.y, a.incy, s);
    }
    const int64_t rt = a.plan.row_tiles;
    if (rt < 1 || ceil_div(a.plan.ntiles, GN_NW * rt) > 65535) return hipErrorInvalidValue;   // beyond the grid's second dimension
    const dim3 grid((unsigned)a.plan.splits, (unsigned)ceil_div(a.plan.ntiles, GN_NW * rt), (unsigned)batch);
    const dim3 block(GN_NW * WAVE);
    if (a.A_ptrs) {     // pointer-array batch: one instance (one row tile per wave, no column splits)
        if (rt != 1 || a.plan.splits != 1) return hipErrorInvalidValue;
        hipLaunchKernelGGL((gemv_n_kernel<T, GN_NW, GN_LOADS, 1, true>), grid, block, 0, s, a);
        return hipGetLastError();
    }
    if (rt == 1) hipLaunchKernelGGL((gemv_n_kernel<T, GN_NW, GN_LOADS, 1>), grid, block, 0, s, a);
    else if (rt == 2) hipLaunchKernelGGL((gemv_n_kernel<T, GN_NW, GN_LOADS / 2, 2>), grid, block, 0, s, a);
    else if (rt == 4) hipLaunchKernelGGL((gemv_n_kernel<T, GN_NW, GN_LOADS / 4, 4>), grid, block, 0, s, a);
    else return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.plan.splits == 1) return e;
    return launch_reduce<T>(a.partial, a.plan.splits, a.plan.part_stride, a.plan.part_off, a.m, a.alpha, a.beta, a.alpha_dev, a.beta_dev, a.y, a.incy, s);
}

template <class T> hipError_t launch_gemv_t(const GemvArgs<T>& a, bool conj, hipStream_t s, int64_t batch) {
    if (batch < 1 || batch > 65535 || (batch > 1 && a.plan.splits != 1)) return hipErrorInvalidValue;
    if (a.A_ptrs) {     // pointer-array batch: the instances without row splits
        if (a.plan.splits != 1) return hipErrorInvalidValue;
        const bool cj = conj && Traits<T>::cplx;
        if (a.plan.short_form) {
            const dim3 grid((unsigned)ceil_div(a.n, GT_NC * GT_NW), 1, (unsigned)batch);
            if (cj) hipLaunchKernelGGL((gemv_t_kernel<T, true, GT_NC, GT_NW, true, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
            else hipLaunchKernelGGL((gemv_t_kernel<T, false, GT_NC, GT_NW, true, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
        } else {
            const dim3 grid((unsigned)ceil_div(a.n, GT_NC), 1, (unsigned)batch);
            if (cj) hipLaunchKernelGGL((gemv_t_kernel<T, true, GT_NC, GT_NW, false, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
            else hipLaunchKernelGGL((gemv_t_kernel<T, false, GT_NC, GT_NW, false, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
        }
        return hipGetLastError();
    }
    if (a.plan.short_form) {
        const dim3 grid((unsigned)ceil_div(a.n, GT_NC * GT_NW), (unsigned)a.plan.splits, (unsigned)batch);
        if (conj && Traits<T>::cplx)
            hipLaunchKernelGGL((gemv_t_kernel<T, true, GT_NC, GT_NW, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
        else
            hipLaunchKernelGGL((gemv_t_kernel<T, false, GT_NC, GT_NW, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
    } else {
        // with alignment classes every class gets its own column groups
        const int64_t P = a.plan.period > 1 ? a.plan.period : 1;
        const int64_t groups = P * ceil_div(ceil_div(a.n, P), GT_NC);
        if (a.plan.t_groups > 0 && a.plan.t_groups != groups) return hipErrorInvalidValue;
        const int64_t wgs = a.plan.t_groups > 0 && a.plan.t_wgs > 0 && a.plan.t_wgs < groups ? a.plan.t_wgs : groups;
        const dim3 grid((unsigned)wgs, (unsigned)a.plan.splits, (unsigned)batch);
        // the banded instance when a split holds a band of tiles at least
        const bool bands = a.plan.ntiles / a.plan.splits >= GT_BAND;
        const bool cj = conj && Traits<T>::cplx;
        if (bands && cj) hipLaunchKernelGGL((gemv_t_kernel<T, true, GT_NC, GT_NW, false, false, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
        else if (bands) hipLaunchKernelGGL((gemv_t_kernel<T, false, GT_NC, GT_NW, false, false, true>), grid, dim3(GT_NW * WAVE), 0, s, a);
        else if (cj) hipLaunchKernelGGL((gemv_t_kernel<T, true, GT_NC, GT_NW, false>), grid, dim3(GT_NW * WAVE), 0, s, a);
        else hipLaunchKernelGGL((gemv_t_kernel<T, false, GT_NC, GT_NW, false>), grid, dim3(GT_NW * WAVE), 0, s, a);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || a.plan.splits == 1) return e;
    return launch_reduce<T>(a.partial, a.plan.splits, a.plan.part_stride, 0, a.n, a.alpha, a.beta, a.alpha_dev, a.beta_dev, a.y, a.incy, s);
}

// ---- strided batches of matrices at most one row tile tall: one WAVE per member --------------
// Below a row tile the general kernels leave most lanes of a wave idle and spend their time on the
// per-column instructions.  Here a member is one wave's work and the wave loads CPL = 64 / L columns at a
// time, L lanes (L * VEC >= m rows) on each: lane (sub, cl) = (lane % L, lane / L) owns rows sub*VEC ..
// sub*VEC+VEC-1 in the columns cl, cl + CPL, ...  'N': a_ij x_j goes into the lane's row sums, the lane
// groups are added at the end and group 0 writes y.  'T' / 'C': op(a_ij) x_i is summed over the L lanes of
// the column (DPP) and lane 0 of the group writes y_j.  No LDS, no barrier, loads three column groups ahead;
// a lane whose rows straddle the last row loads at m - VEC and moves the elements into place (needs m >= VEC).
constexpr int GTINY_NW = 4;   // members (waves) per workgroup
template <class T, int MODE, int L, bool PTRS>   // MODE 0: N, 1: T, 2: C
__global__ __launch_bounds__(GTINY_NW * WAVE) void gemv_tiny_kernel(GemvArgs<T> a, int batch) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int CPL = WAVE / L;
    constexpr int DEPTH = 4;
    const int lane = threadIdx.x & (WAVE - 1);
    const int member = (int)blockIdx.x * GTINY_NW + __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    if (member >= batch) return;     // the whole wave leaves; nothing below waits for another wave
    const int m = (int)a.m, n = (int)a.n;
    const int64_t lda = a.lda;
    select_member<PTRS>(a, member);
    const T* __restrict__ x = a.x;
    const T* __restrict__ A = a.A;
    T* y = a.y;
    const int sub = lane % L, cl = lane / L;
    const int r = sub * VEC;                               // first row of this lane
    const int rc = r + VEC <= m ? r : m - VEC;             // where its vector is loaded (m >= VEC)
    const T alpha = scalar_of(a.alpha, a.alpha_dev), beta = scalar_of(a.beta, a.beta_dev);
    T xr[VEC], acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        xr[e] = MODE == 0 ? zero_of<T>() : x[r + e < m ? r + e : 0];
        acc[e] = zero_of<T>();
    }
    const int ngroups = (n + CPL - 1) / CPL;
    auto column = [&](int g) {     // this lane's column of group g; past the end the last column (loaded, not used)
        const int j = g * CPL + cl;
        return j < n ? j : n - 1;
    };
    Vec<T> buf[DEPTH];
    T xj[DEPTH];
    auto load_group = [&](int d, int g) {
        const int j = column(g);
        buf[d] = load_stream(A + (int64_t)j * lda + rc);
        if (MODE == 0) xj[d] = x[j];
    };
    auto compute_group = [&](int d, int g) {
        const int j = g * CPL + cl;
        const bool valid = j < n;
        const Vec<T> sv = shift_elems(buf[d], r - rc);
        if (MODE == 0) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                T nt = acc[e];
                fma_acc(nt, sv.e[e], xj[d]);
                acc[e] = select_of(valid && r + e < m, nt, acc[e]);
            }
        } else {
            T t = zero_of<T>();
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                T tt = t;
                fma_op<MODE == 2>(tt, sv.e[e], xr[e]);
                t = select_of(r + e < m, tt, t);
            }
            const T cs = seg_sum<L>(t);
            if (valid && sub == 0) {
                T* yp = y + (int64_t)j * a.incy;
                *yp = epilogue(alpha, cs, beta, yp);
            }
        }
    };
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d) load_group(d, d);
    for (int g = 0; g < ngroups; g += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            load_group((d + DEPTH - 1) % DEPTH, g + d + DEPTH - 1);
            if (g + d < ngroups) compute_group(d, g + d);
        }
    }
    if (MODE == 0) {
        T sum[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) sum[e] = cross_sum<L>(acc[e]);
        if (cl != 0) return;
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            if (r + e >= m) continue;
            T* yp = y + (int64_t)(r + e) * a.incy;
            *yp = epilogue(alpha, sum[e], beta, yp);
        }
    }
}

template <class T, int MODE, bool PTRS>
void launch_gemv_tiny_mode(const GemvArgs<T>& a, hipStream_t s, int batch) {
    constexpr int VEC = Traits<T>::VEC;
    const dim3 grid((unsigned)ceil_div((int64_t)batch, (int64_t)GTINY_NW)), block(GTINY_NW * WAVE);
    if (a.m <= 8 * VEC) hipLaunchKernelGGL((gemv_tiny_kernel<T, MODE, 8, PTRS>), grid, block, 0, s, a, batch);
    else if (a.m <= 16 * VEC) hipLaunchKernelGGL((gemv_tiny_kernel<T, MODE, 16, PTRS>), grid, block, 0, s, a, batch);
    else if (a.m <= 32 * VEC) hipLaunchKernelGGL((gemv_tiny_kernel<T, MODE, 32, PTRS>), grid, block, 0, s, a, batch);
    else hipLaunchKernelGGL((gemv_tiny_kernel<T, MODE, 64, PTRS>), grid, block, 0, s, a, batch);
}
template <class T, bool PTRS>
void launch_gemv_tiny_ptrs(const GemvArgs<T>& a, int mode, hipStream_t s, int batch) {
    if (mode == 0) launch_gemv_tiny_mode<T, 0, PTRS>(a, s, batch);
    else if (mode == 2 && Traits<T>::cplx) launch_gemv_tiny_mode<T, 2, PTRS>(a, s, batch);
    else launch_gemv_tiny_mode<T, 1, PTRS>(a, s, batch);
}

// mode 0: N, 1: T, 2: C (complex T only).  Requires VEC <= m <= one row tile, n >= 1, batch <= 65535.
template <class T> hipError_t launch_gemv_tiny(const GemvArgs<T>& a, int mode, hipStream_t s, int64_t batch) {
    constexpr int VEC = Traits<T>::VEC;
    if (batch < 1 || batch > 65535 || a.m < VEC || a.m > WAVE * VEC || a.n < 1 || a.n > (int64_t)1 << 30) return hipErrorInvalidValue;
    if (a.A_ptrs) launch_gemv_tiny_ptrs<T, true>(a, mode, s, (int)batch);
    else launch_gemv_tiny_ptrs<T, false>(a, mode, s, (int)batch);
    return hipGetLastError();
}

#define KMV_INSTANTIATE_GEMV(T)                                                              \
    template GemvPlan<T> plan_gemv<T>(bool, int64_t, int64_t, const void*, int64_t, bool);         \
    template hipError_t launch_gemv_n<T>(const GemvArgs<T>&, hipStream_t, int64_t);          \
    template hipError_t launch_gemv_t<T>(const GemvArgs<T>&, bool, hipStream_t, int64_t);          \
    template hipError_t launch_gemv_tiny<T>(const GemvArgs<T>&, int, hipStream_t, int64_t);
KMV_INSTANTIATE_GEMV(float)
KMV_INSTANTIATE_GEMV(double)
KMV_INSTANTIATE_GEMV(cf32)
KMV_INSTANTIATE_GEMV(cf64)

}  // namespace kmv
