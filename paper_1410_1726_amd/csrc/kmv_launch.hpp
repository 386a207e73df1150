// Host-side contracts between the C-ABI layer (kmv_api.hip) and the kernel
// translation units.  Plain structs of pointers and sizes; every launcher
// only enqueues kernels on the given stream and returns the HIP error code.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "kmv_common.hpp"

namespace kmv {

// Process-wide tuning values (0 = choose automatically).
struct Tuning {
    int64_t gemv_n_splits = 0;     // column splits of GEMV-N
    int64_t gemv_t_splits = 0;     // row splits of GEMV-T
    int64_t gemv_n_row_tiles = 0;  // GEMV-N row tiles per wave: 1, 2 or 4
    int64_t gemv_t_wgs = 0;        // GEMV-T: workgroups of the main kernel (each takes several column groups); 0 = planner
    int64_t gemv_short = 0;        // kernels for matrices of a few row tiles: 1 = never, 2 = whenever possible
    int64_t gemv_align_classes = 0;   // columns grouped by their alignment when lda is no multiple of 128 bytes: 1 = never, 2 = always
    int64_t symv_tiles_per_wave = 0;  // SYMV row-chunk height in units of 4 row tiles: 1 or 2
    int64_t symv_variant = 0;         // SYMV main kernel: 2 = balanced shares, 3 = one launch
    int64_t symv_unit_tiles = 0;      // balanced kernel: row tiles per prefetch unit (1 or 2)
    int64_t symv_piece_fixed = 0;     // balanced kernel: fixed part of a piece's weight on the work line, plus one
    int64_t symv_edge_weight = 0;     // balanced kernel: extra weight of a piece per edge tile it holds, plus one
    int64_t wg_target = 0;         // workgroups the heuristics aim for
    int64_t symv_member_rows = 0;     // batches: largest n for the one-workgroup-per-member kernel
    int64_t symv_member_waves = 0;    // batches: waves of that kernel's workgroup (4 or 8)
    int64_t symv_small_waves = 0;     // small-matrix kernel: waves per workgroup (4, 8 or 16)
    int64_t gemv_tiny_rows = 0;       // batches: one wave per member for m < this value (1 = never)
    int64_t tuned_table = 0;          // measured per-size settings: 1 = ignore them (the planners' rules alone)
};
Tuning& tuning();

// Measured per-size settings (Section 9: tuning parameters found by a coarse and a fine sweep, kept apart from the
// kernels).  The rows are written by the tuning tool (`tune table --save`) into kmv_tuned_table.inc and compiled
// in.  A row applies to the square products of its routine ('N', 'T' for both transposed forms, 'L', 'U') and
// precision whose size lies in [n_lo, n_hi) and whose leading dimension is a whole number of 128-byte lines (what
// the tool measures); a zero field leaves that choice to the planner's rule.  tuned() returns the caller's
// tuning values with the matching row filled into the keys the caller left at 0: an explicit key always wins.
struct TunedRow {
    char op, prec;
    int32_t n_lo, n_hi;
    int16_t gemv_n_splits, gemv_n_row_tiles, gemv_t_splits, symv_variant, symv_tiles_per_wave, symv_unit_tiles, wg_target;
};
Tuning tuned(char op, char prec, int64_t m, int64_t n, int64_t lda_bytes);
template <class T> constexpr char prec_char() {
    return sizeof(T) == 4 ? 's' : (sizeof(T) == 16 ? 'z' : (Traits<T>::cplx ? 'c' : 'd'));
}

// Index of the current device for the per-device caches of the planners
// (occupancy and compute-unit counts differ between devices), -1 if it cannot
// be found or lies beyond the cached range: the planners then use defaults.
constexpr int MAX_CACHED_DEVICES = 64;
inline int cached_device_index() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) {
        (void)hipGetLastError();
        return -1;
    }
    return (dev >= 0 && dev < MAX_CACHED_DEVICES) ? dev : -1;
}

constexpr int64_t WS_ALIGN = 256;
inline size_t round_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
// Distance (in elements) between consecutive partial vectors of `elems` elements:
// a whole number of 256-byte units, and an odd one, so that the vectors of
// different workgroups that hold the same rows do not all fall on one memory
// channel the way a power-of-two distance would make them.
template <class T> inline int64_t partial_stride(int64_t elems) {
    size_t units = round_up((size_t)elems * sizeof(T), 256) / 256;
    if (units % 2 == 0) ++units;
    return (int64_t)(units * 256 / sizeof(T));
}

// Row tiles start on the 128-byte boundary below the first element when every
// column has the same misalignment (lda*sizeof(T) multiple of 128); `shift` is
// the number of leading, masked element slots of tile 0 (Section 6.6: start at
// the aligned address and ignore the extra rows).
template <class T> inline int row_shift(const void* A, int64_t lda) {
    const uint64_t b = sizeof(T);
    if ((uint64_t)lda * b % 128 != 0) return 0;
    return (int)(((uint64_t)(uintptr_t)A % 128) / b);
}
template <class T> constexpr int max_row_shift() { return 128 / (int)sizeof(T) - 1; }

// ---------------------------------------------------------------- GEMV ----
template <class T> struct GemvPlan {
    int shift;            // masked leading slots of row tile 0
    int64_t ntiles;       // row tiles of tile_rows<T>() rows covering [-shift, m)
    int64_t splits;       // N: column splits; T: row splits
    int64_t row_tiles;    // N: row tiles per wave
    int short_form;       // kernels for matrices of a few row tiles (waves split columns instead of rows)
    // Alignment classes (Section 6.6 carried to leading dimensions that are no multiple of 128 bytes): the
    // misalignment of column j is (A + j*lda) mod 128, which repeats every `period` columns.  With period > 1
    // a workgroup takes columns of ONE class (j = class, class + period, ...), all equally aligned, and starts
    // its row tiles on THEIR 128-byte boundary (the kernel works the shift out from the class's first column);
    // shift and ntiles above then describe the class with the largest shift.  1 = all columns alike.
    int64_t period;
    int64_t t_groups;     // T: column groups of the main kernel (0: one per workgroup, as launched),
    int64_t t_wgs;        //    workgroups that share them (0 or >= t_groups: one group each)
    int64_t part_off;     // slot of row 0 in a partial vector of GEMV-N
    int64_t part_stride;  // elements between consecutive partial vectors
    size_t xpack_off, partial_off, total_bytes;   // workspace layout
};
// plan for a concrete call (A != nullptr) or the worst case over alignments
// (classes = false: never group the columns by alignment; the batched forms, whose members share one grid)
template <class T> GemvPlan<T> plan_gemv(bool notrans, int64_t m, int64_t n, const void* A, int64_t lda, bool classes = true);

template <class T> struct GemvArgs {
    int64_t m, n, lda;
    const T* A;
    const T* x;       // contiguous x (packed copy when incx != 1)
    T* y;             // element k of y is y[k*incy] (base already moved for incy < 0)
    int64_t incy;
    T alpha, beta;
    const T* alpha_dev = nullptr;   // non-null: alpha / beta are read from device memory by the epilogue
    const T* beta_dev = nullptr;
    // strided batches: workgroups with blockIdx.z = b work on A + b*batch_A, x + b*batch_x, y + b*batch_y
    // (elements); all zero for a single product
    int64_t batch_A = 0, batch_x = 0, batch_y = 0;
    // pointer-array batches (kernel instances with PTRS): member b works on A_ptrs[b], x_ptrs[b] and
    // y_ptrs[b] + y_shift (the shift moves the base for incy < 0); arrays of device pointers in device memory
    const T* const* A_ptrs = nullptr;
    const T* const* x_ptrs = nullptr;
    T* const* y_ptrs = nullptr;
    int64_t y_shift = 0;
    T* partial;       // [splits][part_stride]
    GemvPlan<T> plan;
};
// batch > 1: a strided batch in one launch (requires plan.splits == 1 and the general kernels)
template <class T> hipError_t launch_gemv_n(const GemvArgs<T>& a, hipStream_t s, int64_t batch = 1);
template <class T> hipError_t launch_gemv_t(const GemvArgs<T>& a, bool conj, hipStream_t s, int64_t batch = 1);
// strided batches of matrices with VEC <= m <= gemv_tiny_rows<T>(notrans): one wave per member, several columns per
// load (mode 0: N, 1: T, 2: C); uses none of the plan
template <class T> hipError_t launch_gemv_tiny(const GemvArgs<T>& a, int mode, hipStream_t s, int64_t batch);
// Largest m it is chosen for.  Measured on 1 GiB batches of square members against the general kernels: 'N' wins
// up to 256 bytes per column (384 for 4-byte elements: 1.1-3.6x), 'T' / 'C' up to half a row tile (a whole one for
// 16-byte elements: 1.1-4.8x); beyond, the general kernels are 2-25% faster.
template <class T> inline int64_t gemv_tiny_rows(bool notrans) {
    constexpr int64_t VEC = Traits<T>::VEC;
    const int64_t cap = 64 * VEC;
    if (tuning().gemv_tiny_rows > 0) return tuning().gemv_tiny_rows - 1 < cap ? tuning().gemv_tiny_rows - 1 : cap;
    if (notrans) return sizeof(T) == 4 ? 24 * VEC : 16 * VEC;
    return sizeof(T) == 16 ? 64 * VEC : 32 * VEC;
}

// ----------------------------------------------------------- SYMV/HEMV ----
// Shares of the balanced kernel's work line, computed on the host and handed to the kernels as arguments
// (Section 6.2 deals equal contiguous shares to the workers; here the shares are cut where pieces start and a
// piece weighs what it holds).  start[y] = (row chunk << SHARE_PIECE_BITS) | piece inside the chunk: the first
// piece of worker y; start[workers] = (number of chunks, 0).  first / last: the workers that hold the first and
// the last piece of a chunk, which is all the final pass needs to find the chunk's row-sum vectors.
constexpr int SHARE_MAX_WORKERS = 800;      // 3204 bytes of kernel arguments
constexpr int SHARE_PIECE_BITS = 20;
constexpr int SHARE_MAX_CHUNKS = 272;
struct SymvShares { uint32_t start[SHARE_MAX_WORKERS + 1]; };
struct SymvOwners { uint16_t first[SHARE_MAX_CHUNKS], last[SHARE_MAX_CHUNKS]; };
struct SymvBalanced {
    // what the table was computed for
    int64_t n;
    int shift, lower, chunk_tiles, unit_tiles, slots, fixed, edge;
    // the table
    int64_t work;     // length of the work line
    int workers;      // shares (workgroups of the main kernel)
    SymvShares shares;
    SymvOwners owners;
};

template <class T> struct SymvPlan {
    int shift;
    int variant;           // main kernel: 2 = balanced shares of pieces, 3 = one launch (4: batches, one workgroup per member; 0: refused)
    int unit_tiles;        // variant 2: row tiles per prefetch unit
    int64_t ntiles;        // row tiles covering [-shift, n)
    int64_t panel_cols;    // columns per panel
    int64_t npanels;       // column panels
    int64_t chunk_tiles;   // row tiles per row chunk
    int64_t chunk_off;     // row chunk k covers the row tiles [k*chunk_tiles - chunk_off, (k+1)*chunk_tiles - chunk_off)
    int64_t nchunks;       // row chunks
    int64_t rows_padded;   // distance between two row-sum vectors (>= chunk rows)
    int64_t work;          // variant 2: length of the work line (stored row tiles of all pieces plus a fixed part per piece)
    int64_t workers;       // variant 2: workgroups of the main kernel
    const SymvBalanced* bal;   // variant 2: the shares (host memory of the planner, valid until the thread's next few plans)
    size_t xpack_off, wsn_off, wst_off, total_bytes;
};
// Where the row chunks start.  The tiles rarely divide into whole chunks, and a short chunk is made of short pieces,
// for which the per-piece work (column sums, change of panel) and an edge tile weigh most.  It therefore goes
// where the triangle is narrow: lower storage starts with it (its rows hold the fewest stored columns), upper storage
// ends with it.  Returns the number of tiles by which the chunk grid starts before tile 0: a multiple of the unit's
// tiles, so that only the matrix's last chunk can end inside a unit (whose rows beyond n are masked anyway).
__host__ __device__ __forceinline__ int64_t symv_chunk_offset(bool lower, int64_t ntiles, int64_t chunk_tiles, int64_t unit_tiles) {
    const int64_t c = (chunk_tiles - ntiles % chunk_tiles) % chunk_tiles;
    return lower ? c - c % unit_tiles : 0;
}
template <class T> SymvPlan<T> plan_symv(bool lower, int64_t n, const void* A, int64_t lda);
// the table of shares for given settings (what plan_symv looks up for the balanced kernel; exported for tests)
template <class T>
const SymvBalanced* symv_shares(bool lower, int64_t n, int shift, int chunk_tiles, int unit_tiles, int64_t slots, int fixed,
                                int edge);

template <class T> struct SymvArgs {
    int64_t n, lda;
    const T* A;
    const T* x;       // contiguous
    T* y;
    int64_t incy;
    T alpha, beta;
    const T* alpha_dev = nullptr;   // non-null: alpha / beta are read from device memory by the epilogue
    const T* beta_dev = nullptr;
    // strided batches: workgroups with blockIdx.z = b work on A + b*batch_A, x + b*batch_x, y + b*batch_y
    // (elements); all zero for a single product
    int64_t batch_A = 0, batch_x = 0, batch_y = 0;
    const T* const* A_ptrs = nullptr;   // pointer-array batches, as in GemvArgs
    const T* const* x_ptrs = nullptr;
    T* const* y_ptrs = nullptr;
    int64_t y_shift = 0;
    T* wsn;           // row sums ("N part"): [workgroup + chunk][rows_padded]
    T* wst;           // [npanels][nchunks][panel_cols]  column sums ("T part")
    SymvPlan<T> plan;
};
// Operands of member b of a batch, inside a kernel: strided (base + b*stride; all strides zero for a single
// product) or, in the kernel instances for pointer-array batches, read from the arrays.
template <bool PTRS, class Args> __device__ __forceinline__ void select_member(Args& a, int64_t b) {
    if constexpr (PTRS) {
        a.A = a.A_ptrs[b];
        a.x = a.x_ptrs[b];
        a.y = a.y_ptrs[b] + a.y_shift;
    } else {
        a.A += b * a.batch_A;
        a.x += b * a.batch_x;
        a.y += b * a.batch_y;
    }
}
// HERM selects the Hermitian rule (conjugated mirror image, real diagonal); it exists for
// complex T only.  Each (T, HERM) pair is instantiated in exactly one translation unit.
// Row tiles of the largest matrix the one-workgroup-per-member kernel (plan.variant == 4, batches only)
// is compiled for: its row sums, x and two columns of matrix data live in registers (4 * MAXT vectors
// per lane), which allows 8 tiles (1024 rows of 8-byte elements, 512 of 16-byte ones; 1024 rows are
// 4 tiles of 4-byte elements).
template <class T> constexpr int member_max_tiles() { return 1024 / tile_rows<T>() < 8 ? 1024 / tile_rows<T>() : 8; }
// Largest n that kernel is chosen for (a member is streamed by a single compute unit).
template <class T> inline int64_t member_rows() {
    const int64_t cap = (int64_t)member_max_tiles<T>() * tile_rows<T>();
    const int64_t want = tuning().symv_member_rows > 0 ? tuning().symv_member_rows : cap;
    return want < cap ? want : cap;
}
// batch > 1: a strided batch in one launch (requires plan.variant == 3 or 4)
template <class T, bool HERM> hipError_t launch_symv_kind(const SymvArgs<T>& a, bool lower, hipStream_t s, int64_t batch);
template <class T>
inline hipError_t launch_symv(const SymvArgs<T>& a, bool lower, bool herm, hipStream_t s, int64_t batch = 1) {
    if constexpr (Traits<T>::cplx) {
        if (herm) return launch_symv_kind<T, true>(a, lower, s, batch);
    }
    return launch_symv_kind<T, false>(a, lower, s, batch);
}

// ------------------------------------------------------------ auxiliary ----
// dst[k] = element k of the strided vector src (base already moved for inc < 0)
template <class T> hipError_t launch_pack(const T* src, int64_t inc, int64_t len, T* dst, hipStream_t s);
// y[k*incy] = beta * y[k*incy]   (alpha == 0 path; beta == 0 stores zeros)
// (`batch` vectors, `stride` elements apart)
template <class T>
hipError_t launch_scal(int64_t len, T beta, T* y, int64_t incy, hipStream_t s, int64_t batch = 1, int64_t stride = 0);
// y <- beta*y for the members of a pointer-array batch (member b: y_ptrs[b] + shift)
template <class T>
hipError_t launch_scal_ptrs(int64_t len, T beta, T* const* y_ptrs, int64_t shift, int64_t incy, hipStream_t s, int64_t batch);
// y[k*incy] = alpha * sum_s partial[s*stride + off + k] + beta*y[k*incy], s ascending
template <class T> hipError_t launch_reduce(const T* partial, int64_t splits, int64_t stride, int64_t off,
                                            int64_t len, T alpha, T beta, const T* alpha_dev, const T* beta_dev, T* y,
                                            int64_t incy, hipStream_t s);

hipError_t launch_stream_probe(int kind, int64_t n, const double* a, double* b, double* c, double* sink, hipStream_t s);

}  // namespace kmv
