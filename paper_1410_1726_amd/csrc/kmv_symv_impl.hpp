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
// the stored triangle as the unit of work, the balanced partition of Section
// 6.2.  Two main kernels follow, each with its own description:
// symv_balanced_kernel (equal shares of the triangle's pieces for one resident
// round of workgroups) and symv_small_kernel (one launch, no workspace, for
// small matrices); strided batches of small matrices have symv_member_kernel
// (one workgroup per matrix) and symv_tiny_kernel (one wave per matrix).  What
// was measured on the MI355X and shaped them: lanes map to 16-byte row vectors,
// a wave streams 1 KiB of a column per instruction; small writes scattered
// through a read stream cost far more than their bytes, so row sums stay on
// chip for a whole share; each of the 8 XCDs has its own L2; the other
// triangle is never loaded, so the mirrored copy of Section 6.5 is never built.
// A second kernel adds, in a fixed order, all row sums and column sums that
// belong to y_i and applies alpha and beta (no atomics anywhere).
//
// This header holds the kernels and their host side as templates; the
// translation units kmv_symv_real.hip (s, d), kmv_symv_herm.hip (c, z
// Hermitian) and kmv_symv_csym.hip (c, z symmetric) instantiate them, so that
// the three groups compile side by side.
#pragma once
#include "kmv_launch.hpp"

namespace kmv {

namespace {
constexpr int SY_NW = 4;    // waves per workgroup
constexpr int RED_ROWS = 16, RED_PARTS = 16;
// final pass of the balanced kernel: rows per workgroup (a row group is read with one 128-byte access at least)
template <class T> constexpr int red_rows() { return sizeof(T) == 4 ? 32 : 16; }
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

// Groups of KT row tiles of the row chunk [tbeg, tend) that hold stored elements of panel p (C columns):
// [glo, ghi).  Inside a chunk's own panel range (chunk_panels) the range is never empty.
template <bool LOWER>
__host__ __device__ __forceinline__ void piece_groups(int p, int C, int n, int shift, int TR, int KT, int tbeg, int tend,
                                                      int& glo, int& ghi) {
    const int gk = (tend - tbeg + KT - 1) / KT;
    if (LOWER) {
        const int tlo = (p * C + shift) / TR;
        glo = tlo > tbeg ? (tlo - tbeg) / KT : 0;
        ghi = gk;
    } else {
        const int jend = p * C + C < n ? p * C + C : n;
        const int thi = (jend - 1 + shift) / TR + 1;
        glo = 0;
        ghi = thi < tend ? (thi - tbeg + KT - 1) / KT : gk;
    }
}

// Balanced form: the pieces (row chunk k, panel p) of the stored triangle are
// laid chunk by chunk on a work line, each with the weight of the row tiles it
// really holds plus a fixed part, and the line is dealt to the workgroups in
// equal contiguous shares by the partition of Section 6.2 (a piece goes to the
// share that holds its first unit).  The host computes where every share starts
// and passes the table in the kernel arguments, so a workgroup begins to load
// after two scalar reads.  The grid is exactly one resident round (compute
// units x occupancy): every workgroup starts at once, reads about the same
// number of bytes and ends at once, and at any moment the resident workgroups
// cover all row chunks, so the load on memory channels does not depend on the
// leading dimension.  A workgroup's share lies in one chunk, rarely two or more.
// Inside a piece wave w owns the columns [w*NC, (w+1)*NC) of the panel over the
// piece's stored groups of KT row tiles, visited in a per-wave rotated order so
// that the waves read different KiB of their columns at any moment.  The
// transposed column sums are private to the wave: one DPP reduction per column
// and panel, no barrier inside the walk, and the diagonal tiles' element-wise
// work is spread over all waves.  The row sums of a wave live in a wave-private
// LDS array (each lane touches only its own slots, no synchronisation) and meet
// the other waves' when the share leaves a chunk: one row-sum vector per
// (workgroup, chunk), stored at index workgroup + chunk.  x over the chunk's
// rows is staged in LDS; the x_j of a unit's columns travel with the unit's
// matrix vectors (one load, spread to the lanes' multiply-adds by readlane when
// the unit is used), so nothing between issuing a unit's loads and using the
// unit before it waits for memory.
template <class T, bool HERM, bool LOWER, int NC, int KT, int G, int NW>
__global__ __launch_bounds__(NW * WAVE, KT == 1 ? (G <= 8 ? 3 : (G <= 12 ? 2 : 1)) : 2) void symv_balanced_kernel(SymvArgs<T> a, SymvShares sh) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    constexpr int C = NC * NW;
    constexpr int CT = KT * G;
    constexpr int R = CT * TR;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    // row, column, tile and panel numbers are kept in 32 bits (the host uses this
    // kernel only while n + 2*CT*TR < 2^31); only addresses are 64-bit
    const int n = (int)a.n;
    const int64_t lda = a.lda;
    const int shift = a.plan.shift;
    const int ntiles = (int)a.plan.ntiles, nchunks = (int)a.plan.nchunks, npanels = (int)a.plan.npanels;
    const T* __restrict__ x = a.x;
    // long columns [jlo, jhi): at least VEC stored rows, so that any lane finds 16 stored bytes in them.  The
    // VEC - 1 short columns at the tip of the triangle (at most six elements) are left to the final pass.
    const int jlo = LOWER ? 0 : VEC - 1, jhi = LOWER ? n - VEC + 1 : n;

    // x over the chunk's rows (zeros outside [0, n)) and the row sums of each wave: static LDS up to 64 KB, the
    // tallest chunks take dynamic LDS (the launch passes balanced_lds_bytes)
    constexpr bool DYN_LDS = (size_t)(NW + 1) * R * sizeof(T) > 65536;
    extern __shared__ __align__(16) unsigned char dyn_lds[];
    __shared__ __align__(16) T xs_static[DYN_LDS ? 1 : R];
    __shared__ __align__(16) T rs_static[DYN_LDS ? 1 : NW][DYN_LDS ? 1 : R];
    T* const xs = DYN_LDS ? reinterpret_cast<T*>(dyn_lds) : xs_static;
    T(*const rs)[R] = DYN_LDS ? reinterpret_cast<T(*)[R]>(dyn_lds + (size_t)R * sizeof(T)) : reinterpret_cast<T(*)[R]>(&rs_static[0][0]);

    // this workgroup's share: from piece j0 of chunk k0 up to (not including) piece j1 of chunk k1
    const uint32_t e0 = sh.start[blockIdx.x], e1 = sh.start[blockIdx.x + 1];
    constexpr uint32_t PIECE_MASK = (1u << SHARE_PIECE_BITS) - 1;
    const int k0 = (int)(e0 >> SHARE_PIECE_BITS), j0 = (int)(e0 & PIECE_MASK);
    const int k1 = (int)(e1 >> SHARE_PIECE_BITS), j1 = (int)(e1 & PIECE_MASK);

    Vec<T> b0[KT][NC], b1[KT][NC];
    T xr0 = zero_of<T>(), xr1 = zero_of<T>();
    T accT[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) accT[c] = zero_of<T>();

    const int coff = (int)a.plan.chunk_off;
    for (int k = k0; k <= k1 && k < nchunks; ++k) {
        const int tbeg = k * CT - coff > 0 ? k * CT - coff : 0;
        const int tend = (k + 1) * CT - coff < ntiles ? (k + 1) * CT - coff : ntiles;
        int64_t plo64, phi64;
        chunk_panels<LOWER>(tbeg, tend, C, shift, TR, npanels, plo64, phi64);
        const int ja = k == k0 ? j0 : 0, jb = k == k1 ? j1 : (int)(phi64 - plo64);
        if (jb <= ja) continue;               // the share ends where this chunk begins
        const int pfirst = (int)plo64 + ja, npieces = jb - ja;
        const int row0 = tbeg * TR - shift;   // row of slot 0 of the chunk

        // row tiles of the chunk (numbered from 0) whose TR rows all exist: [tf_lo, tf_hi)
        const int tf_lo = row0 < 0 ? 1 : 0;
        const int tf_hi = (n - row0) / TR < tend - tbeg ? (n - row0) / TR : tend - tbeg;

        // Position of the share's walk through this chunk: piece pp, step ss of the piece's nu stored
        // groups [glo, glo + nu), at group gg (the waves start at different groups).  What depends on
        // the piece only is worked out once per piece: the wave's first column jg, its NC columns as
        // they are loaded (cj: a column that does not exist or is a short one stands in as the nearest
        // long column), the lane's address of row 0 of each (col), the lane's element of x, and the
        // tiles [fa, fb) in which every pair of the wave's columns is an ordinary off-diagonal element.
        struct Walk {
            int pp, ss, gg, glo, nu, fa, fb, ra, rb;
            bool longcols;   // the wave's NC columns all exist and are long ones
            int cj[NC];
            const T* col[NC];
            const T* xcol;
        };
        auto enter = [&](Walk& it) {
            const int p = pfirst + it.pp;
            int glo, ghi;
            piece_groups<LOWER>(p, C, n, shift, TR, KT, tbeg, tend, glo, ghi);
            it.glo = glo;
            it.nu = ghi - glo;
            int r = w;
#pragma unroll
            for (int i = 1; i < NW; ++i) r = r >= it.nu ? r - it.nu : r;
            it.gg = glo + r;
            it.ss = 0;
            const int jg = p * C + w * NC;
            it.longcols = jg >= jlo && jg + NC <= jhi;
            if (it.longcols) {
                // [ra, rb): tiles cut by the matrix's first or last row whose existing rows are all ordinary
                // off-diagonal elements of the wave's columns (the ragged last tile of the columns far above it
                // in lower storage, the shifted first tile of the columns far to its right in upper storage)
                if (LOWER) {
                    const int f = (jg + NC + shift + TR - 1) / TR - tbeg;   // first tile that starts at or below row jg + NC
                    it.fa = f > tf_lo ? f : tf_lo;
                    it.fb = tf_hi;
                    it.ra = f > tf_hi ? f : tf_hi;
                    it.rb = tend - tbeg;
                } else {
                    const int f = (jg + shift) / TR - tbeg;                 // tiles before f end above row jg
                    it.fa = tf_lo;
                    it.fb = f < tf_hi ? f : tf_hi;
                    it.ra = 0;
                    it.rb = f < tf_lo ? f : tf_lo;
                }
            } else {
                it.fa = it.fb = it.ra = it.rb = 0;
            }
#pragma unroll
            for (int c = 0; c < NC; ++c) {
                const int j = jg + c;
                it.cj[c] = j < jlo ? jlo : (j >= jhi ? jhi - 1 : j);
                it.col[c] = a.A + (int64_t)it.cj[c] * lda;
            }
            const int jx = jg + (lane & (NC - 1));
            it.xcol = x + (jx < jlo ? jlo : (jx >= jhi ? jhi - 1 : jx));
        };
        auto advance = [&](Walk& it) {
            if (it.pp >= npieces) return;   // the walk is over
            if (++it.ss == it.nu) {
                if (++it.pp < npieces) enter(it);
            } else if (++it.gg == it.glo + it.nu) {
                it.gg = it.glo;
            }
        };

        // One unit = the wave's NC columns of one panel over KT row tiles; the next unit's matrix vectors
        // and x_j are in flight while this one is used.  A unit is always 1 + KT*NC loads, whatever it
        // holds, so the number of loads in flight is known at every point of the walk: a lane whose VEC
        // rows are not all stored in the column (the diagonal crosses them, they lie beyond the matrix,
        // the tile lies on the other side of the diagonal) loads the nearest 16 bytes of the column's
        // stored part instead and moves the elements into place when the unit is used.  What the use
        // needs to know travels with the buffer: the first tile gt, the panel p, and flags (bit q: tile
        // q is fast; LAST: the piece ends with this unit; PAST: the walk is over, the loads are cheap
        // stand-ins that keep the pipeline's shape, every lane reading the first stored vector of its
        // column, and the use changes nothing).
        constexpr int F_WHOLE = 1 << 4, F_LAST = 1 << 8, F_PAST = 1 << 9, F_RAG = 1 << 12;
        struct Unit { int gt, p, fl; };
        Walk it;
        const int lane_row = lane * VEC;
        auto issue = [&](Vec<T>(&b)[KT][NC], T& xr, Unit& u) {
            const bool past = it.pp >= npieces;
            u.gt = it.gg * KT;
            u.p = pfirst + it.pp;
            u.fl = past ? F_PAST : (it.ss == it.nu - 1 ? F_LAST : 0);
            xr = *it.xcol;
#pragma unroll
            for (int q = 0; q < KT; ++q) {
                if (!past && u.gt + q >= it.fa && u.gt + q < it.fb) u.fl |= 1 << q;
                else if (!past && u.gt + q >= it.ra && u.gt + q < it.rb) u.fl |= F_RAG << q;
                else if (!past && it.longcols && u.gt + q >= tf_lo && u.gt + q < tf_hi) u.fl |= F_WHOLE << q;
                const int r = (past ? -(1 << 30) : row0 + (u.gt + q) * TR) + lane_row;
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const int slo = LOWER ? it.cj[c] : 0, top = LOWER ? n - VEC : it.cj[c] + 1 - VEC;
                    const int rc = max(min(r, top), slo);   // slo <= top: the column holds VEC stored rows
                    b[q][c] = load_stream(it.col[c] + rc);
                }
            }
            advance(it);
        };
        auto use = [&](const Vec<T>(&b)[KT][NC], const T& xr, const Unit& u) {
            const int jg = u.p * C + w * NC;
            T xjb[NC];   // wave-uniform
#pragma unroll
            for (int c = 0; c < NC; ++c) xjb[c] = read_lane(xr, c);
#pragma unroll
            for (int q = 0; q < KT; ++q) {
                const int slot = (u.gt + q) * TR + lane_row;
                Vec<T> xi, an;
                __builtin_memcpy(&xi, &xs[slot], sizeof(xi));
                __builtin_memcpy(&an, &rs[w][slot], sizeof(an));
                if (u.fl & (1 << q)) {
#pragma unroll
                    for (int c = 0; c < NC; ++c)
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            fma_acc(an.e[v], b[q][c].e[v], xjb[c]);
                            fma_op<HERM>(accT[c], b[q][c].e[v], xi.e[v]);
                        }
                } else if (u.fl & (F_RAG << q)) {
                    // the tile is cut by the first or the last row of the matrix and lies away from the diagonal:
                    // a lane whose vector was loaded at a clamped position moves its elements into place, rows
                    // that do not exist are skipped, everything else is an ordinary pair
                    const int r = row0 + slot;
                    const int rc = LOWER ? (r < n - VEC ? r : n - VEC) : (r > 0 ? r : 0);
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const Vec<T> sv = shift_elems(b[q][c], r - rc);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            const bool ins = LOWER ? r + v < n : r + v >= 0;
                            T nn = an.e[v], nt = accT[c];
                            fma_acc(nn, sv.e[v], xjb[c]);
                            fma_op<HERM>(nt, sv.e[v], xi.e[v]);
                            an.e[v] = select_of(ins, nn, an.e[v]);
                            accT[c] = select_of(ins, nt, accT[c]);
                        }
                    }
                } else if (u.fl & (F_WHOLE << q)) {
                    // the diagonal crosses the tile, all its rows and the wave's columns exist: a lane's vector
                    // is used whole when it lies strictly on the stored side of the column's diagonal element
                    // and not at all otherwise (the vector that holds the diagonal element belongs to the
                    // final pass), so nothing has to be moved or masked element by element
                    const int r = row0 + slot;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int j = jg + c;
                        const bool whole = LOWER ? r > j : r + VEC - 1 < j;
                        T nt = accT[c];
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            T nn = an.e[v];
                            fma_acc(nn, b[q][c].e[v], xjb[c]);
                            an.e[v] = select_of(whole, nn, an.e[v]);
                            fma_op<HERM>(nt, b[q][c].e[v], xi.e[v]);
                        }
                        accT[c] = select_of(whole, nt, accT[c]);
                    }
                } else {
                    // edge tiles (rows before the first or beyond the last one, short or missing columns):
                    // pairs outside the stored triangle are skipped, and so are the pairs whose row lies in
                    // the same aligned group of VEC rows as the column's diagonal element (final pass)
                    const int r = row0 + slot;
                    const bool past = (u.fl & F_PAST) != 0;
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const int j = jg + c;
                        const bool exists = !past && j >= jlo && j < jhi;
                        const int jc = j < jlo ? jlo : (j >= jhi ? jhi - 1 : j);
                        const int slo = LOWER ? jc : 0, shi = LOWER ? n : jc + 1;
                        const int rc = r < slo ? slo : (r > shi - VEC ? shi - VEC : r);
                        const Vec<T> sv = shift_elems(b[q][c], r - rc);
#pragma unroll
                        for (int v = 0; v < VEC; ++v) {
                            const int row = r + v;
                            const bool ins = exists && row >= slo && row < shi && (row + shift) / VEC != (j + shift) / VEC;
                            const T av = sv.e[v];
                            T nn = an.e[v], nt = accT[c];
                            fma_acc(nn, av, xjb[c]);
                            fma_op<HERM>(nt, av, xi.e[v]);
                            an.e[v] = select_of(ins, nn, an.e[v]);
                            accT[c] = select_of(ins, nt, accT[c]);
                        }
                    }
                }
                __builtin_memcpy(&rs[w][slot], &an, sizeof(an));
            }
            if (u.fl & F_LAST) {
                // piece finished: column sums of this wave's NC columns, lane c keeps column c
                T mine = zero_of<T>();
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const T sum = wave_sum(accT[c]);
                    mine = select_of(lane == c, sum, mine);
                    accT[c] = zero_of<T>();
                }
                if (lane < NC) a.wst[((int64_t)u.p * nchunks + k) * C + w * NC + lane] = mine;
            }
        };

        // the first matrix vectors are on their way while x is staged
        Unit u0, u1;
        it.pp = 0;
        enter(it);
        issue(b0, xr0, u0);
        for (int i = threadIdx.x; i < R; i += NW * WAVE) {
            const int row = row0 + i;
            const int rc = row < 0 ? 0 : (row >= n ? n - 1 : row);
            xs[i] = select_of(row >= 0 && row < n, x[rc], zero_of<T>());
        }
        {
            Vec<T> z;
#pragma unroll
            for (int v = 0; v < VEC; ++v) z.e[v] = zero_of<T>();
#pragma unroll
            for (int t = 0; t < CT; ++t) __builtin_memcpy(&rs[w][t * TR + lane_row], &z, sizeof(z));
        }
        __syncthreads();
        // Every pass of the loop issues two units' loads and uses two units, unconditionally, and the only
        // exit is at the bottom: no path through the loop holds fewer loads in flight than another, so the
        // waits in front of a unit's first use cover exactly the loads issued before it.
        do {
            issue(b1, xr1, u1);
            use(b0, xr0, u0);
            issue(b0, xr0, u0);
            use(b1, xr1, u1);
        } while (!(u0.fl & F_PAST));
        // the stand-in loads issued past the end are never used; waiting for them here (vmcnt(0), the other
        // counters left alone) tells the compiler that no load is in flight when the next chunk's walk starts
        __builtin_amdgcn_s_waitcnt(0x0F70);

        // leaving the chunk: the NW waves' row sums are added in wave order and
        // stored as row-sum vector number workgroup + chunk
        __syncthreads();
        T* __restrict__ wsn = a.wsn + ((int64_t)blockIdx.x + k) * a.plan.rows_padded;
        const int nvec = (int)(tend - tbeg) * WAVE;   // 16-byte row vectors of this chunk
        for (int vi = threadIdx.x; vi < nvec; vi += NW * WAVE) {
            Vec<T> sum;
            __builtin_memcpy(&sum, &rs[0][vi * VEC], sizeof(sum));
#pragma unroll
            for (int ww = 1; ww < NW; ++ww) {
                Vec<T> o;
                __builtin_memcpy(&o, &rs[ww][vi * VEC], sizeof(o));
#pragma unroll
                for (int v = 0; v < VEC; ++v) sum.e[v] = add_of(sum.e[v], o.e[v]);
            }
            store_vec_stream(wsn + (int64_t)vi * VEC, sum);
        }
        __syncthreads();   // before xs and rs are reused for the next chunk
    }
}

// Small matrices, one launch: a workgroup owns NC consecutive outputs y_j
// (j0 <= j < j0+NC) and forms the whole rows j of the symmetric matrix from the
// stored triangle: the part of row j that is stored as column j (a dot product
// down the column, conjugated for HEMV), the part that is stored as row j (NC
// consecutive elements of every column on the other side of the diagonal block,
// one column per lane) and the NC x NC diagonal block (one stored pair per lane,
// used for both of its outputs).  Every stored element is read twice, which is
// affordable while the triangle stays in cache, and there is no workspace and
// no second kernel: below a few thousand rows the two launches of the kernels
// above cost more than the traffic.
template <class T, bool HERM, bool LOWER, int NC, int NW, bool PTRS = false>
__global__ __launch_bounds__(NW * WAVE) void symv_small_kernel(SymvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    static_assert(NC * NC == WAVE && NC % VEC == 0, "one lane per pair of the diagonal block");
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int64_t n = a.n, lda = a.lda;
    const int shift = a.plan.shift;
    const int64_t j0 = (int64_t)blockIdx.x * NC;
    const int64_t jend = j0 + NC < n ? j0 + NC : n;   // one past the last existing output
    select_member<PTRS>(a, blockIdx.y);   // member of a batch (strides all zero for a single product)
    const T* __restrict__ x = a.x;
    const T* __restrict__ A = a.A;
    T acc[NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) acc[c] = zero_of<T>();

    // ---- stored as columns: rows below (lower) / above (upper) the diagonal block
    {
        const int64_t rlo = LOWER ? jend : 0, rhi = LOWER ? n : j0;   // rows [rlo, rhi)
        const T* __restrict__ col[NC];
#pragma unroll
        for (int c = 0; c < NC; ++c) col[c] = A + (j0 + c < n ? j0 + c : n - 1) * lda;
        if (rhi > rlo) {
            const int64_t tlo = (rlo + shift) / TR, thi = (rhi - 1 + shift) / TR + 1;
            for (int64_t t = tlo + w; t < thi; t += NW) {
                const int64_t r0 = t * TR - shift, r = r0 + (int64_t)lane * VEC;
                if (r0 >= rlo && r0 + TR <= rhi) {
                    const Vec<T> xv = load_cached(x + r);
#pragma unroll
                    for (int c = 0; c < NC; ++c) {
                        const Vec<T> v = load_cached(col[c] + r);
#pragma unroll
                        for (int e = 0; e < VEC; ++e) fma_op<HERM>(acc[c], v.e[e], xv.e[e]);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const int64_t row = r + e;
                        const bool ok = row >= rlo && row < rhi;
                        const int64_t rc = ok ? row : rlo;   // rlo is a stored row of every column of the group
                        const T xi = x[rc];
#pragma unroll
                        for (int c = 0; c < NC; ++c) {
                            T nt = acc[c];
                            fma_op<HERM>(nt, col[c][rc], xi);
                            acc[c] = select_of(ok, nt, acc[c]);
                        }
                    }
                }
            }
        }
    }
    // ---- stored as rows: columns left (lower) / right (upper) of the diagonal block,
    // one column per lane, NC consecutive rows of it
    {
        const int64_t ilo = LOWER ? 0 : jend, ihi = LOWER ? j0 : n;
        const bool whole = (j0 + NC <= n);   // all NC rows exist: 16-byte loads
        for (int64_t ib = ilo + (int64_t)w * WAVE; ib < ihi; ib += NW * WAVE) {
            const int64_t i = ib + lane;
            const bool ok = i < ihi;
            const int64_t ic = ok ? i : ihi - 1;
            const T xi = x[ic];
            const T* __restrict__ seg = A + j0 + ic * lda;
            if (whole) {
#pragma unroll
                for (int cv = 0; cv < NC / VEC; ++cv) {
                    const Vec<T> v = load_cached(seg + cv * VEC);
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        T nt = acc[cv * VEC + e];
                        fma_acc(nt, v.e[e], xi);
                        acc[cv * VEC + e] = select_of(ok, nt, acc[cv * VEC + e]);
                    }
                }
            } else {
#pragma unroll
                for (int c = 0; c < NC; ++c) {
                    const bool rok = j0 + c < n;
                    T nt = acc[c];
                    fma_acc(nt, seg[rok ? c : 0], xi);
                    acc[c] = select_of(rok && ok, nt, acc[c]);
                }
            }
        }
    }
    // ---- diagonal block: lane (r, c) holds the pair (j0+r, j0+c) if it is stored
    if (w == 0) {
        const int r = lane / NC, c = lane % NC;
        const int64_t row = j0 + r, colj = j0 + c;
        const bool stored = row < n && colj < n && (LOWER ? r >= c : r <= c);
        const T av = A[(stored ? row : j0) + (stored ? colj : j0) * lda];   // (j0, j0) is always stored
        const T xr = x[stored ? row : j0], xc = x[stored ? colj : j0];
        // a(row, col) * x_col goes to output row; off the diagonal its mirror image
        // op(a) * x_row goes to output col
        T to_row = zero_of<T>(), to_col = zero_of<T>();
        fma_acc(to_row, select_of(HERM && r == c, real_part_only(av), av), xc);
        fma_op<HERM>(to_col, av, xr);
#pragma unroll
        for (int k = 0; k < NC; ++k) {
            acc[k] = select_of(stored && r == k, add_of(acc[k], to_row), acc[k]);
            acc[k] = select_of(stored && c == k && r != c, add_of(acc[k], to_col), acc[k]);
        }
    }

    __shared__ T red[NW][NC];
#pragma unroll
    for (int c = 0; c < NC; ++c) {
        const T sum = wave_sum(acc[c]);
        if (lane == 0) red[w][c] = sum;
    }
    __syncthreads();
    if (threadIdx.x < NC && j0 + threadIdx.x < n) {
        const int c = threadIdx.x;
        T sum = red[0][c];
#pragma unroll
        for (int ww = 1; ww < NW; ++ww) sum = add_of(sum, red[ww][c]);
        T* yp = a.y + (j0 + c) * a.incy;
        *yp = epilogue(scalar_of(a.alpha, a.alpha_dev), sum, scalar_of(a.beta, a.beta_dev), yp);
    }
}

// Members of a batch, one workgroup per matrix (n <= MAXT row tiles): the whole product stays on one
// compute unit, so every stored element is loaded once and nothing crosses workgroups.  Wave w takes the
// columns j = w, w + NW, ... (a balanced share of the triangle).  Lanes own rows as everywhere else: for
// column j a lane loads the stored part of its rows, adds a_ij x_j to its row sums (registers, one set per
// wave) and collects op(a_ij) x_i for the column sum, which one wave reduction per column turns into the
// "transposed" part of y_j (LDS, each column written by exactly one wave).  At the end the waves add their
// row sums into one LDS vector in wave order and the epilogue runs.
// The loads of a column are issued without any branch, one to three columns ahead of the arithmetic: a tile that
// holds no stored row of the column loads one vector of the stored part (the same for all lanes), and a
// lane whose VEC rows straddle the diagonal or the last row loads its vector at the nearest position that
// lies inside the stored part and moves the elements into place afterwards, so the other triangle is never
// loaded here either.  That needs VEC stored rows in the column; the VEC - 1 columns at the short end of
// the triangle (at most 6 elements) are left to the epilogue, which adds them to the outputs they belong to.
template <class T, bool HERM, bool LOWER, int MAXT, int NW, bool PTRS>
__global__ __launch_bounds__(NW * WAVE) void symv_member_kernel(SymvArgs<T> a) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int TR = WAVE * VEC;
    const int lane = threadIdx.x & (WAVE - 1);
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    const int n = (int)a.n;
    const int64_t lda = a.lda;
    select_member<PTRS>(a, blockIdx.x);
    const T* __restrict__ x = a.x;
    const T* __restrict__ A = a.A;
    T* y = a.y;

    __shared__ T rowsum[MAXT * TR];   // N parts, all waves
    __shared__ T colsum[MAXT * TR];   // T parts, one writer per column

    T xr[MAXT][VEC], acc[MAXT][VEC];
#pragma unroll
    for (int t = 0; t < MAXT; ++t)
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            const int row = t * TR + lane * VEC + e;
            xr[t][e] = x[row < n ? row : 0];
            acc[t][e] = zero_of<T>();
        }

    // columns with at least VEC stored rows: [jlo, jhi)
    const int jlo = LOWER ? 0 : VEC - 1;
    const int jhi = LOWER ? n - VEC + 1 : n;
    if (jhi > jlo) {
        const int ncols = jhi - jlo;
        const int cnt = ncols > w ? (ncols - w + NW - 1) / NW : 0;   // columns of this wave
        // k-th column of this wave; past the end the last column of the range (loaded, not used)
        auto column = [&](int k) {
            const int j = jlo + w + k * NW;
            return j < jhi ? j : jhi - 1;
        };
        // position of the lane's vector in tile t of column j: the stored rows are [slo, shi)
        auto vec_row = [&](int t, int j) {
            const int slo = LOWER ? j : 0, shi = LOWER ? n : j + 1;
            const int tlo = slo / TR, thi = (shi - 1) / TR + 1;
            const int r = (t >= tlo && t < thi) ? t * TR + lane * VEC : slo;
            const int rc = r < slo ? slo : r;
            return rc > shi - VEC ? shi - VEC : rc;
        };
        // x_j travels with the column's buffer: fetched at compute time it would be a load in the critical path
        // of every column in the pointer-array instances, where x is not known to be read-only kernel input
        auto load_col = [&](Vec<T>(&buf)[MAXT], T& xj, int j) {
            const T* __restrict__ col = A + (int64_t)j * lda;
#pragma unroll
            for (int t = 0; t < MAXT; ++t) buf[t] = load_stream(col + vec_row(t, j));
            xj = x[j];
        };
        auto compute_col = [&](const Vec<T>(&buf)[MAXT], const T xj, int j) {
            const int slo = LOWER ? j : 0, shi = LOWER ? n : j + 1;
            const int tlo = slo / TR, thi = (shi - 1) / TR + 1;
            T tsum = zero_of<T>();
#pragma unroll
            for (int t = 0; t < MAXT; ++t) {
                if (t < tlo || t >= thi) continue;     // wave uniform
                const int r = t * TR + lane * VEC;
                if (t * TR >= slo && (t + 1) * TR <= shi - (LOWER ? 0 : 1) && (!LOWER || t * TR > j)) {
                    // every row of the tile is stored and none is the diagonal
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        fma_acc(acc[t][e], buf[t].e[e], xj);
                        fma_op<HERM>(tsum, buf[t].e[e], xr[t][e]);
                    }
                } else {
                    const Vec<T> sv = shift_elems(buf[t], r - vec_row(t, j));
#pragma unroll
                    for (int e = 0; e < VEC; ++e) {
                        const int row = r + e;
                        const bool stored = row >= slo && row < shi;
                        const bool dia = row == j;
                        const T av = sv.e[e];
                        // a_ij x_j for y_i (the diagonal element takes part here, as a real number for HEMV)
                        T nt = acc[t][e];
                        fma_acc(nt, select_of(HERM && dia, real_part_only(av), av), xj);
                        acc[t][e] = select_of(stored, nt, acc[t][e]);
                        // op(a_ij) x_i for y_j
                        T tt = tsum;
                        fma_op<HERM>(tt, av, xr[t][e]);
                        tsum = select_of(stored && !dia, tt, tsum);
                    }
                }
            }
            const T cs = wave_sum(tsum);
            if (lane == 0) colsum[j] = cs;
        };
        // DEPTH column buffers, DEPTH - 1 columns in flight while one is worked on (more for the
        // small members, whose columns are short; deeper settings measured the same or 1-4% slower)
        constexpr int DEPTH = MAXT == 1 ? 4 : (MAXT == 2 ? 3 : 2);
        Vec<T> b[DEPTH][MAXT];
        T xb[DEPTH];
#pragma unroll
        for (int d = 0; d < DEPTH - 1; ++d) load_col(b[d], xb[d], column(d));
        for (int k = 0; k < cnt; k += DEPTH) {
#pragma unroll
            for (int d = 0; d < DEPTH; ++d) {
                load_col(b[(d + DEPTH - 1) % DEPTH], xb[(d + DEPTH - 1) % DEPTH], column(k + d + DEPTH - 1));
                if (k + d < cnt) compute_col(b[d], xb[d], jlo + w + (k + d) * NW);
            }
        }
    }

    // row sums of the waves, added in wave order
    for (int ww = 0; ww < NW; ++ww) {
        if (w == ww) {
#pragma unroll
            for (int t = 0; t < MAXT; ++t)
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const int row = t * TR + lane * VEC + e;
                    if (row < n) rowsum[row] = ww == 0 ? acc[t][e] : add_of(rowsum[row], acc[t][e]);
                }
        }
        __syncthreads();
    }
    const T alpha = scalar_of(a.alpha, a.alpha_dev), beta = scalar_of(a.beta, a.beta_dev);
    // the short columns left out above: indices [clo, chi)
    const int clo = LOWER ? (jhi > 0 ? jhi : 0) : 0, chi = LOWER ? n : (jlo < n ? jlo : n);
    for (int i = threadIdx.x; i < n; i += NW * WAVE) {
        T sum = rowsum[i];
        if (i >= jlo && i < jhi) sum = add_of(sum, colsum[i]);
        if (VEC > 1 && i >= clo && i < chi) {
            for (int k = clo; k < chi; ++k) {
                const bool own = LOWER ? i >= k : i <= k;      // a_ik itself is stored (else a_ki)
                const T av = own ? A[i + (int64_t)k * lda] : A[k + (int64_t)i * lda];
                if (own) fma_acc(sum, select_of(HERM && i == k, real_part_only(av), av), x[k]);
                else fma_op<HERM>(sum, av, x[k]);
            }
        }
        T* yp = y + (int64_t)i * a.incy;
        *yp = epilogue(alpha, sum, beta, yp);
    }
}

// Members of a batch that are at most half a row tile tall (n <= 32 * VEC): one WAVE per matrix, and the wave
// loads CPL = 64 / L columns at a time, L lanes (L * VEC >= n rows) on each.  The per-column work of the kernel
// above (address arithmetic, masks for the diagonal, the reduction of the column sum) is what bounds it when a
// column is shorter than a wave's 1 KiB load; here it is shared by CPL columns.  Lane (sub, cl) = (lane % L,
// lane / L) owns rows sub*VEC .. sub*VEC+VEC-1 in the columns j = cl, cl + CPL, ...: it adds a_ij x_j to its
// row sums and collects op(a_ij) x_i, which a reduction over the L lanes of the column (DPP, plus one
// cross-lane move for L = 32) turns into the column sum; the lane that owns row j takes it into its row sums.
// At the end the row sums of the CPL lane groups are added (rotations inside the rows of 16 lanes, cross-lane
// moves between them) and the lanes of group 0 write y.  No LDS, no barrier; loads run three column groups
// ahead, clamped into the stored part as above, and the short columns at the end of the triangle go to the
// epilogue in the same way.
constexpr int TINY_NW = 4;   // members (waves) per workgroup

template <class T, bool HERM, bool LOWER, int L, bool PTRS>
__global__ __launch_bounds__(TINY_NW * WAVE) void symv_tiny_kernel(SymvArgs<T> a, int batch) {
    constexpr int VEC = Traits<T>::VEC;
    constexpr int CPL = WAVE / L;
    constexpr int DEPTH = 4;
    static_assert(L == 8 || L == 16 || L == 32 || L == 64, "lanes per column");
    const int lane = threadIdx.x & (WAVE - 1);
    const int member = (int)blockIdx.x * TINY_NW + __builtin_amdgcn_readfirstlane(threadIdx.x / WAVE);
    if (member >= batch) return;     // the whole wave leaves; nothing below waits for another wave
    const int n = (int)a.n;
    const int64_t lda = a.lda;
    select_member<PTRS>(a, member);
    const T* __restrict__ x = a.x;
    const T* __restrict__ A = a.A;
    T* y = a.y;
    const int sub = lane % L, cl = lane / L;
    const int r = sub * VEC;         // first row of this lane

    T xr[VEC], acc[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        xr[e] = x[r + e < n ? r + e : 0];
        acc[e] = zero_of<T>();
    }
    // columns with at least VEC stored rows: [jlo, jhi)
    const int jlo = LOWER ? 0 : VEC - 1;
    const int jhi = LOWER ? n - VEC + 1 : n;
    if (jhi > jlo) {
        const int ngroups = (jhi - jlo + CPL - 1) / CPL;
        // position of the lane's vector in column j: the stored rows are [slo, shi), at least VEC of them
        auto vec_row = [&](int j) {
            const int slo = LOWER ? j : 0, shi = LOWER ? n : j + 1;
            const int rc = r < slo ? slo : r;
            return rc > shi - VEC ? shi - VEC : rc;
        };
        auto column = [&](int g) {     // this lane's column of group g; past the end the last column (loaded, not used)
            const int j = jlo + g * CPL + cl;
            return j < jhi ? j : jhi - 1;
        };
        Vec<T> buf[DEPTH];
        T xj[DEPTH];
        auto load_group = [&](int d, int g) {
            const int j = column(g);
            buf[d] = load_stream(A + (int64_t)j * lda + vec_row(j));
            xj[d] = x[j];
        };
        auto compute_group = [&](int d, int g) {
            const int j = column(g);
            const bool valid = jlo + g * CPL + cl < jhi;
            const int slo = LOWER ? j : 0, shi = LOWER ? n : j + 1;
            const Vec<T> sv = shift_elems(buf[d], r - vec_row(j));
            T tsum = zero_of<T>();
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const int row = r + e;
                const bool stored = valid && row >= slo && row < shi;
                const bool dia = row == j;
                const T av = sv.e[e];
                T nt = acc[e];
                fma_acc(nt, select_of(HERM && dia, real_part_only(av), av), xj[d]);
                acc[e] = select_of(stored, nt, acc[e]);
                T tt = tsum;
                fma_op<HERM>(tt, av, xr[e]);
                tsum = select_of(stored && !dia, tt, tsum);
            }
            const T cs = seg_sum<L>(tsum);      // column sum of column j, in all L lanes of the column
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = select_of(valid && j == r + e, add_of(acc[e], cs), acc[e]);
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
    }
    // rows of the CPL lane groups added; group 0 finishes its rows
    T sum[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) sum[e] = cross_sum<L>(acc[e]);
    if (cl != 0) return;
    const T alpha = scalar_of(a.alpha, a.alpha_dev), beta = scalar_of(a.beta, a.beta_dev);
    const int clo = LOWER ? (jhi > 0 ? jhi : 0) : 0, chi = LOWER ? n : (jlo < n ? jlo : n);   // the short columns
#pragma unroll
    for (int e = 0; e < VEC; ++e) {
        const int i = r + e;
        if (i >= n) continue;
        T s = sum[e];
        if (VEC > 1 && i >= clo && i < chi) {
            for (int k = clo; k < chi; ++k) {
                const bool own = LOWER ? i >= k : i <= k;      // a_ik itself is stored (else a_ki)
                const T av = own ? A[i + (int64_t)k * lda] : A[k + (int64_t)i * lda];
                if (own) fma_acc(s, select_of(HERM && i == k, real_part_only(av), av), x[k]);
                else fma_op<HERM>(s, av, x[k]);
            }
        }
        T* yp = y + (int64_t)i * a.incy;
        *yp = epilogue(alpha, s, beta, yp);
    }
}

// y_i = alpha * ( sum over the workgroups whose share touches the chunk of row i of their row-sum
// vectors + sum over chunks of wst[panel(i)][chunk][i] + the pairs left to this pass ) + beta*y_i.
// blockDim = (RR, RP) with RR = 16 rows (32 for 4-byte elements, so that a row group is one 128-byte access) and
// RP = 256 / RR parts: part g adds the vectors g, g+RP, ... and then the chunks kbeg+g, kbeg+g+RP, ... in ascending
// order; the parts meet in LDS and are added in part order, so the result does not depend on scheduling.
template <class T, bool HERM, bool LOWER>
__global__ __launch_bounds__(256) void symv_reduce_kernel(SymvArgs<T> a, SymvOwners owners) {
    constexpr int TR = tile_rows<T>();
    constexpr int RR = red_rows<T>(), RP = 256 / RR;
    const int lx = threadIdx.x, g = threadIdx.y;
    const int64_t i = (int64_t)blockIdx.x * RR + lx;
    const int shift = a.plan.shift;
    const int64_t C = a.plan.panel_cols;
    __shared__ T part[RP][RR];
    T s = zero_of<T>();
    if (i < a.n) {
        {
            // row-sum vectors of the workgroups whose share touches the chunk of row i:
            // numbers ylo..yhi (from the host's table of shares), vector y + k each
            const int64_t CT = a.plan.chunk_tiles, slot = i + shift;
            const int64_t k = (slot + a.plan.chunk_off * TR) / (CT * TR);
            const int64_t tbeg = k * CT - a.plan.chunk_off > 0 ? k * CT - a.plan.chunk_off : 0;   // the chunk's first tile
            const int64_t ylo = owners.first[k], yhi = owners.last[k];
            const T* __restrict__ wsn = a.wsn + (slot - tbeg * TR);
#pragma unroll 4
            for (int64_t yy = ylo + g; yy <= yhi; yy += RP) s = add_of(s, wsn[(yy + k) * a.plan.rows_padded]);
        }
        // chunks whose row tiles intersect the tile range of the panel of column i
        const int64_t pi = i / C;
        int64_t tlo, thi;
        panel_tiles<LOWER>(pi * C, C, a.n, shift, TR, a.plan.ntiles, tlo, thi);
        const int64_t kbeg = (tlo + a.plan.chunk_off) / a.plan.chunk_tiles;
        const int64_t kend = (thi - 1 + a.plan.chunk_off) / a.plan.chunk_tiles + 1;
        const T* __restrict__ wst = a.wst + pi * a.plan.nchunks * C + (i - pi * C);
#pragma unroll 4
        for (int64_t k = kbeg + g; k < kend; k += RP) s = add_of(s, wst[k * C]);
        // The balanced kernel leaves two kinds of pairs to this pass: those whose row lies in the same aligned
        // group of VEC rows as the column's diagonal element (the groups of the lanes' 16-byte vectors: rows
        // m*VEC - shift ...), and the VEC - 1 columns at the tip of the triangle that hold fewer than VEC stored
        // rows.  Both are a handful of elements per output.
        constexpr int VEC = Traits<T>::VEC;
        if (g == 0) {
            auto add_pair = [&](int64_t k) {
                const bool own = LOWER ? i >= k : i <= k;      // a_ik itself is stored (else a_ki)
                const T av = own ? a.A[i + k * a.lda] : a.A[k + i * a.lda];
                if (own) fma_acc(s, select_of(HERM && i == k, real_part_only(av), av), a.x[k]);
                else fma_op<HERM>(s, av, a.x[k]);
            };
            const int64_t glo = (i + shift) / VEC * VEC - shift;
            const int64_t gbeg = glo > 0 ? glo : 0, gend = glo + VEC < a.n ? glo + VEC : a.n;
            for (int64_t k = gbeg; k < gend; ++k) add_pair(k);
            if (VEC > 1) {
                const int64_t clo = LOWER ? (a.n - VEC + 1 > 0 ? a.n - VEC + 1 : 0) : 0;
                const int64_t chi = LOWER ? a.n : (VEC - 1 < a.n ? VEC - 1 : a.n);
                if (i >= clo && i < chi)
                    for (int64_t k = clo; k < chi; ++k)
                        if (k < gbeg || k >= gend) add_pair(k);
            }
        }
    }
    part[g][lx] = s;
    __syncthreads();
    if (g == 0 && i < a.n) {
        T tot = part[0][lx];
#pragma unroll
        for (int gg = 1; gg < RP; ++gg) tot = add_of(tot, part[gg][lx]);
        T* yp = a.y + i * a.incy;
        *yp = epilogue(scalar_of(a.alpha, a.alpha_dev), tot, scalar_of(a.beta, a.beta_dev), yp);
    }
}

// ------------------------------------------------------------- host side ----
namespace {
constexpr int BAL_NC = 4;   // balanced kernel: columns per wave
constexpr int SMALL_NC = 8;            // small-matrix kernel: outputs per workgroup
// largest n the small-matrix kernel is chosen for (measured against the two-launch path at n = 1536 .. 3072 in
// steps of 128 .. 256, both triangles: it wins up to 2176 in s (10-15 us against 15-16), up to 2048 in d and c,
// up to about 1600 in z, and loses by 20-70% from 2560 on)
template <class T> constexpr int64_t small_n() { return sizeof(T) == 4 ? 2176 : (sizeof(T) == 16 ? 1664 : 2048); }
// Row tiles per unit (KT), chunk height and workgroups per compute unit, measured with the settings
// alternating in one process over n = 2560 .. 32768 in all four precisions: one tile per unit (4 matrix
// loads and one of x per lane and buffer) is never slower than two; ONE workgroup per compute unit is
// fastest from a few hundred megabytes of triangle on (the kernel's loads are pipelined by the wave itself,
// and more resident workgroups only lengthen the queues in front of the memory channels: DSYMV 16384
// 164 us against 176-178 us with two or three per compute unit), two below; chunks of 8 row tiles pay for
// real 8-byte elements from about n = 17400 (1-2%; not at 16384: -4%), for complex 8-byte elements from about 9000
// (2-5%; except where the column stride is a multiple of 32 KB, n = 12288 and 16384 with lda = n: there 8-tile chunks
// are 2-3% SLOWER than 4-tile ones and 12-tile chunks as fast or faster, while 11264, 13312, 15360 gain 1.5-4% from 8
// tiles and lose with 12 - the plan takes 12 tiles for such strides below 18432), for 16-byte elements from about n = 8400 (10% at 24576) - the complex types spend more on the column
// sums of a piece, which a taller piece amortises; 12 tiles
// (what 64 KB of static LDS hold) add 1-2.5% for 16-byte elements from about 10000, and 16 tiles (80 KB of dynamic
// LDS) another 0.7-4% from 16384 (ZHEMV 32768: 1314 -> 1271 us) and 1.7% for 8-byte elements at 40960; 4-byte elements
// gain 1-2.7% from 8 tiles from about n = 36000 on (and lose 3-4% at 32768); 4 tiles elsewhere.
template <class T> inline int default_unit_tiles(int64_t) { return 1; }
inline int wgs_per_cu(int kt) { return kt == 1 ? 3 : 2; }   // the most the kernel instances are built for
template <class T> inline int default_wgs_per_cu(int64_t n) {
    const double bytes = 0.5 * (double)n * (double)n * sizeof(T);
    return bytes >= (sizeof(T) == 16 ? 600e6 : 200e6) ? 1 : 2;
}
template <class T> inline int64_t default_tiles_per_wave(int64_t n) {
    if (sizeof(T) == 4) return n >= 36864 ? 2 : 1;
    if (sizeof(T) == 16) return n >= 16384 ? 4 : (n >= 10240 ? 3 : (n >= 8448 ? 2 : 1));
    return n >= 36864 ? 4 : (n >= (Traits<T>::cplx ? 9216 : 17408) ? 2 : 1);
}
// fixed part of a piece's weight on the work line, in row tiles (the column sums and their store, the
// change of panel): measured over s, d, c, z at n = 16384 and 32768 with the key symv_piece_fixed: three tiles' worth is
// never slower than one and 2-4% faster for SSYMV at 16384 and ZHEMV with tall chunks (whose pieces on the diagonal
// are the most lopsided); beyond that nothing changes
constexpr int DEFAULT_PIECE_FIXED = 3;
// what an edge tile costs on top of an ordinary one, in row tiles (tuning key symv_edge_weight)
// measured at n = 17001 (one ragged tile at the bottom of every column): one tile's worth for 8- and 16-byte
// elements, three for 4-byte ones (four elements per lane to move into place)
template <class T> constexpr int default_edge_weight() { return sizeof(T) == 4 ? 3 : 1; }
// compute units and min(occupancy, most workgroups wanted per compute unit), queried once per instance
// Dynamic LDS of an instance: 0 while its arrays fit the 64 KB of static LDS, else their size; such an instance
// is allowed the larger amount once per device (the symmetric and the Hermitian instance are different kernels).
template <class T, bool HERM, bool LOWER, int KT, int G> size_t balanced_dynamic_lds() {
    constexpr size_t bytes = (size_t)(SY_NW + 1) * KT * G * tile_rows<T>() * sizeof(T);
    if (bytes <= 65536) return 0;
    static bool allowed[MAX_CACHED_DEVICES] = {};
    const int di = cached_device_index();
    if (di < 0 || !allowed[di]) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&symv_balanced_kernel<T, HERM, LOWER, BAL_NC, KT, G, SY_NW>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
        (void)hipGetLastError();
        if (di >= 0) allowed[di] = true;
    }
    return bytes;
}
template <class T, bool LOWER, int KT, int G> int64_t balanced_slots_of() {
    constexpr bool HERM = Traits<T>::cplx;
    int dev = 0, cus = 0, nb = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    if (e == hipSuccess)
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, symv_balanced_kernel<T, HERM, LOWER, BAL_NC, KT, G, SY_NW>,
                                                         SY_NW * WAVE, balanced_dynamic_lds<T, HERM, LOWER, KT, G>());
    (void)hipGetLastError();
    if (e != hipSuccess || cus <= 0 || nb <= 0) return -1;
    return ((int64_t)cus << 8) | (nb < wgs_per_cu(KT) ? nb : wgs_per_cu(KT));   // compute units, workgroups that fit on one
}
template <class T> int64_t balanced_slots(bool lower, int ktw, int kt) {
    static int64_t cache[MAX_CACHED_DEVICES][2][5][3] = {};
    const int di = cached_device_index();
    if (ktw < 1 || ktw > 4 || kt < 1 || kt > 2 || (ktw >= 3 && kt != 1) || di < 0) return -1;
    int64_t& c = cache[di][lower ? 1 : 0][ktw][kt];
    if (c == 0) {
        if (lower) {
            if (ktw == 4) c = balanced_slots_of<T, true, 1, 4 * SY_NW>();
            else if (ktw == 3) c = balanced_slots_of<T, true, 1, 3 * SY_NW>();
            else if (kt == 1) c = ktw == 1 ? balanced_slots_of<T, true, 1, SY_NW>() : balanced_slots_of<T, true, 1, 2 * SY_NW>();
            else c = ktw == 1 ? balanced_slots_of<T, true, 2, SY_NW / 2>() : balanced_slots_of<T, true, 2, SY_NW>();
        } else {
            if (ktw == 4) c = balanced_slots_of<T, false, 1, 4 * SY_NW>();
            else if (ktw == 3) c = balanced_slots_of<T, false, 1, 3 * SY_NW>();
            else if (kt == 1) c = ktw == 1 ? balanced_slots_of<T, false, 1, SY_NW>() : balanced_slots_of<T, false, 1, 2 * SY_NW>();
            else c = ktw == 1 ? balanced_slots_of<T, false, 2, SY_NW / 2>() : balanced_slots_of<T, false, 2, SY_NW>();
        }
    }
    return c;
}
}  // namespace

// Walks the work line of the balanced kernel in runs of pieces of equal weight: f(chunk, first piece of
// the run inside the chunk, pieces in the run, weight of each).  Within a chunk the number of stored
// groups of a piece changes only where the diagonal crosses a group boundary, so a chunk has at most
// chunk_tiles / unit_tiles + 1 runs and the walk costs a few operations per run.
template <class T, class F>
inline void walk_work_line(bool lower, int64_t n, int shift, int ct, int kt, int fixed, int edge, F&& f) {
    constexpr int TR = tile_rows<T>();
    constexpr int C = BAL_NC * SY_NW;
    const int ntiles = (int)ceil_div(n + shift, TR), npanels = (int)ceil_div(n, C);
    const int coff = (int)symv_chunk_offset(lower, ntiles, ct, kt), nchunks = (int)ceil_div(ntiles + coff, ct);
    for (int k = 0; k < nchunks; ++k) {
        const int tbeg = k * ct - coff > 0 ? k * ct - coff : 0, tend = (k + 1) * ct - coff < ntiles ? (k + 1) * ct - coff : ntiles;
        int64_t plo, phi;
        if (lower) chunk_panels<true>(tbeg, tend, C, shift, TR, npanels, plo, phi);
        else chunk_panels<false>(tbeg, tend, C, shift, TR, npanels, plo, phi);
        // groups of the chunk that hold an edge tile (rows before row 0 or beyond row n - 1): their pairs are
        // masked and moved element by element, which costs `edge` row tiles' worth of time on top
        const int ge0 = (k == 0 && shift > 0) ? 0 : -1;
        const int ge1 = (tend == ntiles && (int64_t)ntiles * TR - shift > n) ? (tend - 1 - tbeg) / kt : -1;
        int64_t p = plo;
        while (p < phi) {
            int glo, ghi;
            int64_t q;   // first panel after p with another number of stored groups
            if (lower) {
                piece_groups<true>((int)p, C, (int)n, shift, TR, kt, tbeg, tend, glo, ghi);
                // one group fewer from the panel whose first column lies at or below row (tbeg + (glo + 1) kt) TR - shift
                q = ceil_div((int64_t)(tbeg + (glo + 1) * kt) * TR - shift, C);
            } else {
                piece_groups<false>((int)p, C, (int)n, shift, TR, kt, tbeg, tend, glo, ghi);
                // one group more from the panel whose last column lies at or beyond row (tbeg + ghi kt) TR - shift
                const int gk = (tend - tbeg + kt - 1) / kt;
                q = ghi >= gk ? phi : ceil_div((int64_t)(tbeg + ghi * kt) * TR - shift + 1, C) - 1;
            }
            if (q > phi) q = phi;
            if (q <= p) q = p + 1;   // cannot happen (see the two conditions above); keeps the walk finite regardless
            const int edges = (ge0 >= glo && ge0 < ghi ? 1 : 0) + (ge1 >= glo && ge1 < ghi && ge1 != ge0 ? 1 : 0);
            f(k, (int)(p - plo), (int)(q - p), (ghi - glo) * kt + fixed + edges * edge);
            p = q;
        }
    }
}

// The shares for one (shape, alignment, tuning): looked up in a small per-thread cache, else computed.
// `slots` = workgroups wanted (one resident round).  Every share holds at least one piece: the worker
// count is capped so that a share is at least as long as the heaviest piece.
template <class T>
inline const SymvBalanced* balanced_shares(bool lower, int64_t n, int shift, int ct, int kt, int64_t slots, int fixed, int edge) {
    constexpr int NCACHE = 8;
    thread_local SymvBalanced cache[NCACHE];
    thread_local int used = 0, next = 0;
    if (slots > SHARE_MAX_WORKERS) slots = SHARE_MAX_WORKERS;
    if (slots < 1) slots = 1;
    for (int i = 0; i < used; ++i) {
        const SymvBalanced& e = cache[i];
        if (e.n == n && e.shift == shift && e.lower == (int)lower && e.chunk_tiles == ct && e.unit_tiles == kt &&
            e.slots == (int)slots && e.fixed == fixed && e.edge == edge)
            return &e;
    }
    SymvBalanced& b = cache[next];
    next = (next + 1) % NCACHE;
    if (used < NCACHE) ++used;
    b.n = n; b.shift = shift; b.lower = lower; b.chunk_tiles = ct; b.unit_tiles = kt; b.slots = (int)slots; b.fixed = fixed; b.edge = edge;
    int64_t W = 0, pieces = 0;
    walk_work_line<T>(lower, n, shift, ct, kt, fixed, edge, [&](int, int, int cnt, int wt) {
        W += (int64_t)cnt * wt;
        pieces += cnt;
    });
    int64_t Y = slots;
    const int64_t wmax = ct + fixed + 2 * edge;
    if (Y > W / wmax) Y = W / wmax;
    if (Y > pieces) Y = pieces;
    if (Y < 1) Y = 1;
    b.work = W;
    b.workers = (int)Y;
    constexpr int TR = tile_rows<T>();
    const int64_t ntiles_all = ceil_div(n + shift, TR);
    const int nchunks = (int)ceil_div(ntiles_all + symv_chunk_offset(lower, ntiles_all, ct, kt), ct);
    // worker y starts at the first piece whose first unit lies at or after partition's starting point s(y)
    int64_t pos = 0, y = 0, wy, sy;
    partition(W, Y, 0, wy, sy);
    walk_work_line<T>(lower, n, shift, ct, kt, fixed, edge, [&](int k, int j, int cnt, int wt) {
        const int64_t last_start = pos + (int64_t)(cnt - 1) * wt;
        while (y < Y && sy <= last_start) {
            const int64_t idx = sy <= pos ? 0 : (sy - pos + wt - 1) / wt;
            b.shares.start[y] = ((uint32_t)k << SHARE_PIECE_BITS) | (uint32_t)(j + idx);
            ++y;
            if (y < Y) partition(W, Y, y, wy, sy);
        }
        pos += (int64_t)cnt * wt;
    });
    b.shares.start[Y] = (uint32_t)nchunks << SHARE_PIECE_BITS;
    for (int64_t i = Y + 1; i <= SHARE_MAX_WORKERS; ++i) b.shares.start[i] = b.shares.start[Y];
    // owners of every chunk's first and last piece
    for (int k = 0; k < SHARE_MAX_CHUNKS; ++k) { b.owners.first[k] = 0; b.owners.last[k] = 0; }
    constexpr uint32_t PIECE_MASK = (1u << SHARE_PIECE_BITS) - 1;
    for (int64_t yy = Y - 1; yy >= 0; --yy) {
        const uint32_t e0 = b.shares.start[yy], e1 = b.shares.start[yy + 1];
        const int ka = (int)(e0 >> SHARE_PIECE_BITS);
        const int kb = (e1 & PIECE_MASK) ? (int)(e1 >> SHARE_PIECE_BITS) : (int)(e1 >> SHARE_PIECE_BITS) - 1;
        for (int k = ka; k <= kb && k < SHARE_MAX_CHUNKS; ++k) b.owners.first[k] = (uint16_t)yy;
    }
    for (int64_t yy = 0; yy < Y; ++yy) {
        const uint32_t e0 = b.shares.start[yy], e1 = b.shares.start[yy + 1];
        const int ka = (int)(e0 >> SHARE_PIECE_BITS);
        const int kb = (e1 & PIECE_MASK) ? (int)(e1 >> SHARE_PIECE_BITS) : (int)(e1 >> SHARE_PIECE_BITS) - 1;
        for (int k = ka; k <= kb && k < SHARE_MAX_CHUNKS; ++k) b.owners.last[k] = (uint16_t)yy;
    }
    return &b;
}

template <class T>
const SymvBalanced* symv_shares(bool lower, int64_t n, int shift, int chunk_tiles, int unit_tiles, int64_t slots, int fixed,
                                int edge) {
    return balanced_shares<T>(lower, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge);
}

template <class T> SymvPlan<T> plan_symv(bool lower, int64_t n, const void* A, int64_t lda) {
    constexpr int TR = tile_rows<T>();
    constexpr int64_t C = BAL_NC * SY_NW;
    SymvPlan<T> p;
    const bool sizing = (A == nullptr);
    // the caller's tuning values, plus the measured settings of this size where the caller left the choice open
    const Tuning tn = sizing ? tuning() : tuned(lower ? 'L' : 'U', prec_char<T>(), n, n, lda * (int64_t)sizeof(T));
    p.shift = sizing ? max_row_shift<T>() : row_shift<T>(A, lda);
    p.ntiles = ceil_div(n + p.shift, TR);
    // main kernel: the one-launch kernel up to small_n, the balanced kernel beyond
    p.variant = (int)tn.symv_variant;
    if (p.variant <= 0) p.variant = n <= small_n<T>() ? 3 : 2;
    // the balanced kernel loads 16-byte vectors from columns with at least VEC stored rows: it needs some
    if (p.variant == 2 && n < 4 * Traits<T>::VEC) p.variant = 3;
    // chunk height in units of 4 row tiles
    int64_t ktw = tn.symv_tiles_per_wave;
    if (ktw <= 0) {
        ktw = default_tiles_per_wave<T>(n);
        if (Traits<T>::cplx && sizeof(T) == 8 && ktw == 2 && n < 18432 && (lda * (int64_t)sizeof(T)) % 32768 == 0) ktw = 3;
    }
    // the balanced kernel's tables hold SHARE_MAX_CHUNKS chunks (enough for every matrix that fits the device's
    // memory when the chunks are 8 to 16 tiles high)
    while (ktw < 4 && ceil_div(p.ntiles, SY_NW * ktw) > SHARE_MAX_CHUNKS) ++ktw;
    if (sizing) ktw = 1;   // sizing takes the settings that need the most room
    p.panel_cols = C;
    p.npanels = ceil_div(n, C);
    p.chunk_tiles = SY_NW * ktw;
    p.unit_tiles = tn.symv_unit_tiles > 0 ? (int)tn.symv_unit_tiles : default_unit_tiles<T>(n);
    if (ktw >= 3 || sizing || p.variant != 2) p.unit_tiles = 1;   // the 12- and 16-tile chunks exist with one-tile units only
    p.chunk_off = sizing ? 0 : symv_chunk_offset(lower, p.ntiles, p.chunk_tiles, p.unit_tiles);
    p.nchunks = sizing ? ceil_div(p.ntiles, p.chunk_tiles) + 1 : ceil_div(p.ntiles + p.chunk_off, p.chunk_tiles);
    p.work = 0;
    p.workers = 0;
    p.bal = nullptr;
    size_t wsn_bytes = 0;
    if (sizing) {
        // one row-sum vector of the chunk's height per workgroup and chunk; workgroups <= pieces <= chunks x
        // panels, for either chunk height
        p.rows_padded = partial_stride<T>(4 * SY_NW * TR);
        for (int64_t kw = 1; kw <= 4; ++kw) {
            const int64_t nc = ceil_div(p.ntiles, SY_NW * kw) + 1;   // the chunk grid may start before tile 0
            int64_t entries = nc * p.npanels < SHARE_MAX_WORKERS ? nc * p.npanels : SHARE_MAX_WORKERS;
            entries += nc + 1;
            const size_t bytes = (size_t)entries * partial_stride<T>(kw * SY_NW * TR) * sizeof(T);
            if (bytes > wsn_bytes) wsn_bytes = bytes;
        }
    } else if (p.variant == 2) {
        if (n > (int64_t)1 << 30 || p.nchunks > SHARE_MAX_CHUNKS) {
            p.variant = 0;   // beyond what the kernel's 32-bit row numbers and tables hold: the launch is refused
            p.total_bytes = 0;
            return p;
        }
        int64_t Y = tn.wg_target;
        if (Y <= 0) {
            // one resident round: compute units x workgroups per compute unit (never more than fit)
            const int64_t q = balanced_slots<T>(lower, (int)ktw, p.unit_tiles);
            const int64_t cus = q > 0 ? q >> 8 : 256, fit = q > 0 ? q & 255 : wgs_per_cu(p.unit_tiles);
            const int64_t want = default_wgs_per_cu<T>(n);
            Y = cus * (want < fit ? want : fit);
        }
        const int fixed = tn.symv_piece_fixed > 0 ? (int)tn.symv_piece_fixed - 1 : DEFAULT_PIECE_FIXED;
        const int edge = tn.symv_edge_weight > 0 ? (int)tn.symv_edge_weight - 1 : default_edge_weight<T>();
        p.bal = balanced_shares<T>(lower, n, p.shift, (int)p.chunk_tiles, p.unit_tiles, Y, fixed, edge);
        p.work = p.bal->work;
        p.workers = p.bal->workers;
        p.rows_padded = partial_stride<T>(p.chunk_tiles * TR);
        wsn_bytes = (size_t)(p.workers + p.nchunks) * p.rows_padded * sizeof(T);
    } else {
        p.rows_padded = 0;   // the one-launch kernels use no partial sums
    }
    p.xpack_off = 0;
    p.wsn_off = round_up((size_t)n * sizeof(T), WS_ALIGN);
    p.wst_off = p.wsn_off + round_up(wsn_bytes, WS_ALIGN);
    // column sums: one slot per column of every panel and chunk
    const size_t wst_bytes = (sizing || p.variant == 2) ? (size_t)p.npanels * C * p.nchunks * sizeof(T) : 0;
    p.total_bytes = p.wst_off + round_up(wst_bytes, WS_ALIGN);
    return p;
}

namespace {
template <class T, bool HERM, bool LOWER, int KT, int G>
void launch_balanced(const SymvArgs<T>& a, hipStream_t s) {
    const dim3 grid((unsigned)a.plan.workers);
    const size_t dyn = balanced_dynamic_lds<T, HERM, LOWER, KT, G>();
    hipLaunchKernelGGL((symv_balanced_kernel<T, HERM, LOWER, BAL_NC, KT, G, SY_NW>), grid, dim3(SY_NW * WAVE), dyn, s, a,
                       a.plan.bal->shares);
}
template <class T, bool HERM, bool LOWER> bool dispatch_main(const SymvArgs<T>& a, hipStream_t s) {
    const int cols = (int)a.plan.panel_cols, ktw = (int)(a.plan.chunk_tiles / SY_NW);
    if (a.plan.variant == 2) {
        const int kt = a.plan.unit_tiles;
        if (cols != BAL_NC * SY_NW || a.plan.workers < 1 || !a.plan.bal) return false;
        if (ktw == 1 && kt == 1) launch_balanced<T, HERM, LOWER, 1, SY_NW>(a, s);
        else if (ktw == 2 && kt == 1) launch_balanced<T, HERM, LOWER, 1, 2 * SY_NW>(a, s);
        else if (ktw == 1 && kt == 2) launch_balanced<T, HERM, LOWER, 2, SY_NW / 2>(a, s);
        else if (ktw == 2 && kt == 2) launch_balanced<T, HERM, LOWER, 2, SY_NW>(a, s);
        else if (ktw == 3 && kt == 1) launch_balanced<T, HERM, LOWER, 1, 3 * SY_NW>(a, s);
        else if (ktw == 4 && kt == 1) launch_balanced<T, HERM, LOWER, 1, 4 * SY_NW>(a, s);
        else return false;
        return true;
    }
    return false;
}
}  // namespace

namespace {
template <class T, bool HERM, int NW>
void launch_small(const SymvArgs<T>& a, bool lower, dim3 grid, hipStream_t s) {
    if (a.A_ptrs) {
        if (lower) hipLaunchKernelGGL((symv_small_kernel<T, HERM, true, SMALL_NC, NW, true>), grid, dim3(NW * WAVE), 0, s, a);
        else hipLaunchKernelGGL((symv_small_kernel<T, HERM, false, SMALL_NC, NW, true>), grid, dim3(NW * WAVE), 0, s, a);
        return;
    }
    if (lower) hipLaunchKernelGGL((symv_small_kernel<T, HERM, true, SMALL_NC, NW>), grid, dim3(NW * WAVE), 0, s, a);
    else hipLaunchKernelGGL((symv_small_kernel<T, HERM, false, SMALL_NC, NW>), grid, dim3(NW * WAVE), 0, s, a);
}
template <class T, bool HERM, int L, bool PTRS>
void launch_tiny_ptrs(const SymvArgs<T>& a, bool lower, dim3 grid, dim3 block, int batch, hipStream_t s) {
    if (lower) hipLaunchKernelGGL((symv_tiny_kernel<T, HERM, true, L, PTRS>), grid, block, 0, s, a, batch);
    else hipLaunchKernelGGL((symv_tiny_kernel<T, HERM, false, L, PTRS>), grid, block, 0, s, a, batch);
}
template <class T, bool HERM, int L>
void launch_tiny(const SymvArgs<T>& a, bool lower, dim3 grid, dim3 block, int batch, hipStream_t s) {
    if (a.A_ptrs) launch_tiny_ptrs<T, HERM, L, true>(a, lower, grid, block, batch, s);
    else launch_tiny_ptrs<T, HERM, L, false>(a, lower, grid, block, batch, s);
}
template <class T, bool HERM, int MAXT, int NW, bool PTRS>
void launch_member_ptrs(const SymvArgs<T>& a, bool lower, unsigned batch, hipStream_t s) {
    const dim3 grid(batch);
    if (lower) hipLaunchKernelGGL((symv_member_kernel<T, HERM, true, MAXT, NW, PTRS>), grid, dim3(NW * WAVE), 0, s, a);
    else hipLaunchKernelGGL((symv_member_kernel<T, HERM, false, MAXT, NW, PTRS>), grid, dim3(NW * WAVE), 0, s, a);
}
template <class T, bool HERM, int MAXT>
void launch_member(const SymvArgs<T>& a, bool lower, unsigned batch, hipStream_t s) {
    // eight waves from 2 KB per column on (measured on 1 GiB batches: 3-10% faster there, up to 45% for the
    // largest members, 3-10% slower below)
    const bool eight = tuning().symv_member_waves ? tuning().symv_member_waves == 8 : a.n * (int64_t)sizeof(T) >= 2048;
    if (a.A_ptrs) {
        if (eight) launch_member_ptrs<T, HERM, MAXT, 8, true>(a, lower, batch, s);
        else launch_member_ptrs<T, HERM, MAXT, 4, true>(a, lower, batch, s);
    } else {
        if (eight) launch_member_ptrs<T, HERM, MAXT, 8, false>(a, lower, batch, s);
        else launch_member_ptrs<T, HERM, MAXT, 4, false>(a, lower, batch, s);
    }
}
}  // namespace

// HERM: conjugate the mirrored triangle and take the real part of the diagonal
// (complex Hermitian); false for real symmetric and complex symmetric matrices.
template <class T, bool HERM>
hipError_t launch_symv_kind(const SymvArgs<T>& a, bool lower, hipStream_t s, int64_t batch) {
    static_assert(!HERM || Traits<T>::cplx, "Hermitian kernels exist for complex types only");
    if (batch < 1 || batch > 65535 || a.plan.variant < 2 || (batch > 1 && a.plan.variant < 3)) return hipErrorInvalidValue;
    if (a.plan.variant == 4) {   // members of a batch: one workgroup per matrix
        constexpr int VEC = Traits<T>::VEC;
        // One wave per member, several columns per load when they are short: measured on 1 GiB batches against
        // the workgroup-per-member kernel it is 1.5-3x faster up to half a row tile and 6-25% faster up to three
        // quarters of a tile for 8- and 16-byte elements (a whole tile for 16-byte ones), 3-10% slower beyond.
        constexpr int tiny_rows = sizeof(T) == 4 ? 32 * VEC : (sizeof(T) == 8 ? 48 * VEC : 64 * VEC);
        if (a.n <= tiny_rows && tuning().symv_member_waves != 4 && tuning().symv_member_waves != 8) {
            const dim3 grid((unsigned)ceil_div(batch, (int64_t)TINY_NW)), block(TINY_NW * WAVE);
            const int b = (int)batch;
            if (a.n <= 8 * VEC) launch_tiny<T, HERM, 8>(a, lower, grid, block, b, s);
            else if (a.n <= 16 * VEC) launch_tiny<T, HERM, 16>(a, lower, grid, block, b, s);
            else if (a.n <= 32 * VEC) launch_tiny<T, HERM, 32>(a, lower, grid, block, b, s);
            else if constexpr (tiny_rows > 32 * VEC) launch_tiny<T, HERM, 64>(a, lower, grid, block, b, s);
            return hipGetLastError();
        }
        const int64_t tiles = ceil_div(a.n, (int64_t)tile_rows<T>());
        constexpr int M = member_max_tiles<T>();
        if (tiles < 1 || tiles > M) return hipErrorInvalidValue;
        if (tiles <= 1) launch_member<T, HERM, 1>(a, lower, (unsigned)batch, s);
        else if (tiles <= 2) launch_member<T, HERM, 2>(a, lower, (unsigned)batch, s);
        else if (tiles <= 3) launch_member<T, HERM, (M < 3 ? M : 3)>(a, lower, (unsigned)batch, s);
        else if (tiles <= 4) launch_member<T, HERM, (M < 4 ? M : 4)>(a, lower, (unsigned)batch, s);
        else if (tiles <= 6) launch_member<T, HERM, (M < 6 ? M : 6)>(a, lower, (unsigned)batch, s);
        else launch_member<T, HERM, M>(a, lower, (unsigned)batch, s);
        return hipGetLastError();
    }
    if (a.plan.variant == 3) {   // one launch, no workspace
        const dim3 grid((unsigned)ceil_div(a.n, SMALL_NC), (unsigned)batch);
        // eight waves: 2-11% faster than four at n = 512 .. 2048 in every precision, sixteen no better
        const int64_t nw = tuning().symv_small_waves > 0 ? tuning().symv_small_waves : 8;
        if (nw == 16) launch_small<T, HERM, 16>(a, lower, grid, s);
        else if (nw == 8) launch_small<T, HERM, 8>(a, lower, grid, s);
        else launch_small<T, HERM, 4>(a, lower, grid, s);
        return hipGetLastError();
    }
    const bool ok = lower ? dispatch_main<T, HERM, true>(a, s) : dispatch_main<T, HERM, false>(a, s);
    if (!ok) return hipErrorInvalidValue;
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const dim3 rgrid((unsigned)ceil_div(a.n, (int64_t)red_rows<T>()));
    const dim3 rblock(red_rows<T>(), 256 / red_rows<T>());
    if (lower) hipLaunchKernelGGL((symv_reduce_kernel<T, HERM, true>), rgrid, rblock, 0, s, a, a.plan.bal->owners);
    else hipLaunchKernelGGL((symv_reduce_kernel<T, HERM, false>), rgrid, rblock, 0, s, a, a.plan.bal->owners);
    return hipGetLastError();
}

}  // namespace kmv
