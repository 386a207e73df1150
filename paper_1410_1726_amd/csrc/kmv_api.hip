// C ABI of the kmv library: argument checks, quick returns, workspace layout
// and the choice of kernels.  Nothing here synchronises with the device or
// allocates memory; every call only enqueues kernels on the caller's stream.
// The routines follow the standard BLAS argument lists, as the paper's
// routines do (Section 5.2), with the stream of its "_async" variants.
#include <string.h>

#include <mutex>

#include "../../include/kmv.h"
#include "kmv_launch.hpp"

// Scratch memory of kmv_dsymv_static: partial sums and the packed x of one product, in place of the caller's
// workspace.  Every device the library runs on holds its own copy at its own address until the process ends.
// In host code the name is only a handle for hipGetSymbolAddress; the kernels get the looked-up address.
static __device__ __align__(256) unsigned char static_scratch[KMV_STATIC_SCRATCH_BYTES];

namespace kmv {

namespace {
std::mutex static_scratch_mutex;
void* static_scratch_ptr[MAX_CACHED_DEVICES] = {};
}  // namespace

Tuning& tuning() {
    static Tuning t;
    return t;
}

namespace {
const TunedRow TUNED_ROWS[] = {
#include "kmv_tuned_table.inc"
    {0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0},   // end mark
};
}  // namespace

Tuning tuned(char op, char prec, int64_t m, int64_t n, int64_t lda_bytes) {
    Tuning t = tuning();
    if (t.tuned_table == 1 || m != n || lda_bytes % 128 != 0) return t;
    for (const TunedRow* r = TUNED_ROWS; r->op; ++r) {
        if (r->op != op || r->prec != prec || n < r->n_lo || n >= r->n_hi) continue;
        if (op == 'N' && t.gemv_n_splits == 0 && t.gemv_n_row_tiles == 0 && t.wg_target == 0) {
            t.gemv_n_splits = r->gemv_n_splits;
            t.gemv_n_row_tiles = r->gemv_n_row_tiles;
        }
        if (op == 'T' && t.gemv_t_splits == 0 && t.wg_target == 0) t.gemv_t_splits = r->gemv_t_splits;
        if ((op == 'L' || op == 'U') && t.symv_variant == 0 && t.symv_tiles_per_wave == 0 && t.symv_unit_tiles == 0 &&
            t.wg_target == 0) {
            t.symv_variant = r->symv_variant;
            t.symv_tiles_per_wave = r->symv_tiles_per_wave;
            t.symv_unit_tiles = r->symv_unit_tiles;
            t.wg_target = r->wg_target;
        }
        break;
    }
    return t;
}

namespace {

inline int hip_code(hipError_t e) { return e == hipSuccess ? KMV_OK : KMV_ERR_HIP + (int)e; }

// first storage position of a strided vector (reference-BLAS rule for inc < 0)
template <class T> inline T* vec_base(T* v, int64_t len, int64_t inc) {
    return inc >= 0 ? v : v + (1 - len) * inc;
}

template <class T>
int gemv_entry(char trans, int64_t m, int64_t n, const T* alpha, const T* A, int64_t lda, const T* x, int64_t incx,
               const T* beta, T* y, int64_t incy, void* workspace, size_t workspace_bytes, void* stream,
               bool dev_scalars = false) {
    const bool notrans = (trans == 'N' || trans == 'n');
    const bool tr = (trans == 'T' || trans == 't');
    const bool ct = (trans == 'C' || trans == 'c');
    if (!notrans && !tr && !ct) return -1;
    if (m < 0) return -2;
    if (n < 0) return -3;
    if (lda < (m > 1 ? m : 1)) return -6;
    if (incx == 0) return -8;
    if (incy == 0) return -11;
    if (!alpha || !beta) return KMV_ERR_NULL;
    // scalars in device memory are not looked at here: the quick returns that depend on their
    // values do not apply, the epilogue kernels read them when they run
    const T al = dev_scalars ? zero_of<T>() : *alpha, be = dev_scalars ? zero_of<T>() : *beta;
    if (m == 0 || n == 0 || (!dev_scalars && is_zero(al) && is_one(be))) return KMV_OK;
    if (!A || !x || !y) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t leny = notrans ? m : n, lenx = notrans ? n : m;
    T* yb = vec_base(y, leny, incy);
    if (!dev_scalars && is_zero(al)) return hip_code(launch_scal<T>(leny, be, yb, incy, s));

    const GemvPlan<T> plan = plan_gemv<T>(notrans, m, n, A, lda);
    const bool need_ws = (incx != 1) || plan.splits > 1;
    if (need_ws && (!workspace || workspace_bytes < plan.total_bytes || ((uintptr_t)workspace % WS_ALIGN) != 0))
        return KMV_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    GemvArgs<T> a;
    a.m = m; a.n = n; a.lda = lda; a.A = A;
    a.y = yb; a.incy = incy; a.alpha = al; a.beta = be;
    if (dev_scalars) { a.alpha_dev = alpha; a.beta_dev = beta; }
    a.partial = plan.splits > 1 ? reinterpret_cast<T*>(ws + plan.partial_off) : nullptr;
    a.plan = plan;
    if (incx != 1) {
        T* xp = reinterpret_cast<T*>(ws + plan.xpack_off);
        hipError_t e = launch_pack<T>(vec_base(x, lenx, incx), incx, lenx, xp, s);
        if (e != hipSuccess) return hip_code(e);
        a.x = xp;
    } else {
        a.x = x;
    }
    return hip_code(notrans ? launch_gemv_n<T>(a, s) : launch_gemv_t<T>(a, ct, s));
}

template <class T>
int symv_entry(bool herm, char uplo, int64_t n, const T* alpha, const T* A, int64_t lda, const T* x, int64_t incx, const T* beta,
               T* y, int64_t incy, void* workspace, size_t workspace_bytes, void* stream, bool dev_scalars = false) {
    const bool lower = (uplo == 'L' || uplo == 'l');
    const bool upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (n < 0) return -2;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (incx == 0) return -7;
    if (incy == 0) return -10;
    if (!alpha || !beta) return KMV_ERR_NULL;
    const T al = dev_scalars ? zero_of<T>() : *alpha, be = dev_scalars ? zero_of<T>() : *beta;
    if (n == 0 || (!dev_scalars && is_zero(al) && is_one(be))) return KMV_OK;
    if (!A || !x || !y) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    T* yb = vec_base(y, n, incy);
    if (!dev_scalars && is_zero(al)) return hip_code(launch_scal<T>(n, be, yb, incy, s));

    const SymvPlan<T> plan = plan_symv<T>(lower, n, A, lda);
    if (plan.variant == 0) return KMV_ERR_HIP + (int)hipErrorInvalidValue;   // beyond what the kernels index
    // the one-launch kernel with a contiguous x touches no workspace
    const bool need_ws = plan.variant == 2 || incx != 1;
    if (need_ws && (!workspace || workspace_bytes < plan.total_bytes || ((uintptr_t)workspace % WS_ALIGN) != 0))
        return KMV_ERR_WORKSPACE;
    char* ws = static_cast<char*>(workspace);
    SymvArgs<T> a;
    a.n = n; a.lda = lda; a.A = A;
    a.y = yb; a.incy = incy; a.alpha = al; a.beta = be;
    if (dev_scalars) { a.alpha_dev = alpha; a.beta_dev = beta; }
    a.wsn = plan.variant == 2 ? reinterpret_cast<T*>(ws + plan.wsn_off) : nullptr;
    a.wst = plan.variant == 2 ? reinterpret_cast<T*>(ws + plan.wst_off) : nullptr;
    a.plan = plan;
    if (incx != 1) {
        T* xp = reinterpret_cast<T*>(ws + plan.xpack_off);
        hipError_t e = launch_pack<T>(vec_base(x, n, incx), incx, n, xp, s);
        if (e != hipSuccess) return hip_code(e);
        a.x = xp;
    } else {
        a.x = x;
    }
    return hip_code(launch_symv<T>(a, lower, herm, s));
}

// Sub-block calls that name the parent matrix (Section 6.6).  Logical elements off..len-1 of a
// strided parent vector start `off` increments further on when the increment is positive and
// at the same address when it is negative (the shorter vector ends where the parent's does).
template <class T> inline T* vec_from(T* v, int64_t off, int64_t inc) {
    return (v && inc > 0) ? v + off * inc : v;
}
template <class T>
int gemv_offset_entry(char trans, int64_t m, int64_t n, const T* alpha, const T* A, int64_t lda, const T* x,
                      int64_t incx, const T* beta, T* y, int64_t incy, int64_t offset_r, int64_t offset_c,
                      void* workspace, size_t workspace_bytes, void* stream) {
    const bool notrans = (trans == 'N' || trans == 'n');
    if (!notrans && trans != 'T' && trans != 't' && trans != 'C' && trans != 'c') return -1;
    if (m < 0) return -2;
    if (n < 0) return -3;
    if (lda < (m > 1 ? m : 1)) return -6;
    if (offset_r < 0 || offset_r > m) return -12;
    if (offset_c < 0 || offset_c > n) return -13;
    const int64_t offx = notrans ? offset_c : offset_r, offy = notrans ? offset_r : offset_c;
    return gemv_entry<T>(trans, m - offset_r, n - offset_c, alpha, A ? A + offset_r + offset_c * lda : A, lda,
                         vec_from(x, offx, incx), incx, beta, vec_from(y, offy, incy), incy, workspace,
                         workspace_bytes, stream);
}
template <class T>
int symv_offset_entry(bool herm, char uplo, int64_t n, const T* alpha, const T* A, int64_t lda, const T* x,
                      int64_t incx, const T* beta, T* y, int64_t incy, int64_t offset, void* workspace,
                      size_t workspace_bytes, void* stream) {
    if (uplo != 'L' && uplo != 'l' && uplo != 'U' && uplo != 'u') return -1;
    if (n < 0) return -2;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (offset < 0 || offset > n) return -11;
    return symv_entry<T>(herm, uplo, n - offset, alpha, A ? A + offset + offset * lda : A, lda,
                         vec_from(x, offset, incx), incx, beta, vec_from(y, offset, incy), incy, workspace,
                         workspace_bytes, stream);
}

// Strided batches: `batch` products of one shape, operand b at base + b*stride.  One launch per
// product type covers the whole batch (grid z / y = member), with the single-launch forms of the
// kernels (no column or row splits, small-matrix SYMV kernel), so no workspace is involved.
constexpr int64_t MAX_GRID_BATCH = 65535;

template <class T>
int gemv_batched_entry(char trans, int64_t m, int64_t n, const T* alpha, const T* A, int64_t lda, int64_t strideA,
                       const T* x, int64_t incx, int64_t stridex, const T* beta, T* y, int64_t incy, int64_t stridey,
                       int64_t batch, void* stream) {
    const bool notrans = (trans == 'N' || trans == 'n');
    const bool tr = (trans == 'T' || trans == 't');
    const bool ct = (trans == 'C' || trans == 'c');
    if (!notrans && !tr && !ct) return -1;
    if (m < 0) return -2;
    if (n < 0) return -3;
    if (lda < (m > 1 ? m : 1)) return -6;
    if (strideA < 0) return -7;
    if (incx != 1) return -9;              // a strided x would need packing space per member
    if (stridex < 0) return -10;
    if (incy == 0) return -13;
    const int64_t leny = notrans ? m : n;
    const int64_t exty = leny > 0 ? 1 + (leny - 1) * (incy < 0 ? -incy : incy) : 0;
    if (stridey < 0 || (batch > 1 && stridey < exty)) return -14;   // outputs of two members must not overlap
    if (batch < 0) return -15;
    if (!alpha || !beta) return KMV_ERR_NULL;
    const T al = *alpha, be = *beta;
    if (m == 0 || n == 0 || batch == 0 || (is_zero(al) && is_one(be))) return KMV_OK;
    if (!y || (!is_zero(al) && (!A || !x))) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    T* yb = vec_base(y, leny, incy);
    GemvArgs<T> a;
    a.m = m; a.n = n; a.lda = lda;
    a.incy = incy; a.alpha = al; a.beta = be;
    a.partial = nullptr;
    a.batch_A = strideA; a.batch_x = stridex; a.batch_y = stridey;
    for (int64_t b0 = 0; b0 < batch; b0 += MAX_GRID_BATCH) {
        const int64_t nb = batch - b0 < MAX_GRID_BATCH ? batch - b0 : MAX_GRID_BATCH;
        if (is_zero(al)) {   // y <- beta*y, A and x not referenced
            const hipError_t e = launch_scal<T>(leny, be, yb + b0 * stridey, incy, s, nb, stridey);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        a.A = A + b0 * strideA; a.x = x + b0 * stridex; a.y = yb + b0 * stridey;
        if (m >= Traits<T>::VEC && m <= gemv_tiny_rows<T>(notrans)) {   // short columns: one wave per member
            const hipError_t e = launch_gemv_tiny<T>(a, notrans ? 0 : (ct ? 2 : 1), s, nb);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        GemvPlan<T> plan = plan_gemv<T>(notrans, m, n, a.A, lda, false);
        // the members share one tile grid: keep the pointer's alignment shift only if every member has it
        if (nb > 1 && ((uint64_t)strideA * sizeof(T)) % 128 != 0) {
            plan.shift = 0;
            plan.ntiles = ceil_div(m, (int64_t)tile_rows<T>());
        }
        plan.splits = 1;
        // transposed products of one or two row tiles: every wave takes columns of its own
        plan.short_form = (!notrans && plan.ntiles <= 2) ? 1 : 0;
        plan.row_tiles = 1;
        a.plan = plan;
        const hipError_t e = notrans ? launch_gemv_n<T>(a, s, nb) : launch_gemv_t<T>(a, ct, s, nb);
        if (e != hipSuccess) return hip_code(e);
    }
    return KMV_OK;
}

template <class T>
int symv_batched_entry(bool herm, char uplo, int64_t n, const T* alpha, const T* A, int64_t lda, int64_t strideA,
                       const T* x, int64_t incx, int64_t stridex, const T* beta, T* y, int64_t incy, int64_t stridey,
                       int64_t batch, void* stream) {
    const bool lower = (uplo == 'L' || uplo == 'l');
    const bool upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (n < 0) return -2;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (strideA < 0) return -6;
    if (incx != 1) return -8;
    if (stridex < 0) return -9;
    if (incy == 0) return -12;
    const int64_t exty = n > 0 ? 1 + (n - 1) * (incy < 0 ? -incy : incy) : 0;
    if (stridey < 0 || (batch > 1 && stridey < exty)) return -13;
    if (batch < 0) return -14;
    if (!alpha || !beta) return KMV_ERR_NULL;
    const T al = *alpha, be = *beta;
    if (n == 0 || batch == 0 || (is_zero(al) && is_one(be))) return KMV_OK;
    if (!y || (!is_zero(al) && (!A || !x))) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    T* yb = vec_base(y, n, incy);
    SymvArgs<T> a;
    a.n = n; a.lda = lda;
    a.incy = incy; a.alpha = al; a.beta = be;
    a.wsn = nullptr; a.wst = nullptr;
    a.batch_A = strideA; a.batch_x = stridex; a.batch_y = stridey;
    for (int64_t b0 = 0; b0 < batch; b0 += MAX_GRID_BATCH) {
        const int64_t nb = batch - b0 < MAX_GRID_BATCH ? batch - b0 : MAX_GRID_BATCH;
        if (is_zero(al)) {
            const hipError_t e = launch_scal<T>(n, be, yb + b0 * stridey, incy, s, nb, stridey);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        a.A = A + b0 * strideA; a.x = x + b0 * stridex; a.y = yb + b0 * stridey;
        SymvPlan<T> plan = plan_symv<T>(lower, n, a.A, lda);
        if (nb > 1 && ((uint64_t)strideA * sizeof(T)) % 128 != 0) plan.shift = 0;
        // one workgroup per member for small members, else the one-launch kernel for small matrices with
        // the member in the grid's second dimension
        plan.variant = n <= member_rows<T>() ? 4 : 3;
        a.plan = plan;
        const hipError_t e = launch_symv<T>(a, lower, herm, s, nb);
        if (e != hipSuccess) return hip_code(e);
    }
    return KMV_OK;
}

// Pointer-array batches: member b uses A[b], x[b], y[b], arrays of device pointers in device memory (they are
// read by the kernels, never by the host).  The same single-launch kernels as for strided batches, in
// instances of their own that fetch the operand pointers from the arrays; the members' alignment is unknown,
// so the tile grids start at row 0.
inline const void* some_aligned_address() { return reinterpret_cast<const void*>(uintptr_t(WS_ALIGN)); }

template <class T>
int gemv_ptr_batched_entry(char trans, int64_t m, int64_t n, const T* alpha, const T* const* A, int64_t lda,
                           const T* const* x, int64_t incx, const T* beta, T* const* y, int64_t incy, int64_t batch,
                           void* stream) {
    const bool notrans = (trans == 'N' || trans == 'n');
    const bool tr = (trans == 'T' || trans == 't');
    const bool ct = (trans == 'C' || trans == 'c');
    if (!notrans && !tr && !ct) return -1;
    if (m < 0) return -2;
    if (n < 0) return -3;
    if (lda < (m > 1 ? m : 1)) return -6;
    if (incx != 1) return -8;
    if (incy == 0) return -11;
    if (batch < 0) return -12;
    if (!alpha || !beta) return KMV_ERR_NULL;
    const T al = *alpha, be = *beta;
    if (m == 0 || n == 0 || batch == 0 || (is_zero(al) && is_one(be))) return KMV_OK;
    if (!y || (!is_zero(al) && (!A || !x))) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const int64_t leny = notrans ? m : n;
    GemvArgs<T> a;
    a.m = m; a.n = n; a.lda = lda;
    a.A = nullptr; a.x = nullptr; a.y = nullptr;
    a.incy = incy; a.alpha = al; a.beta = be;
    a.partial = nullptr;
    a.y_shift = incy < 0 ? (1 - leny) * incy : 0;
    for (int64_t b0 = 0; b0 < batch; b0 += MAX_GRID_BATCH) {
        const int64_t nb = batch - b0 < MAX_GRID_BATCH ? batch - b0 : MAX_GRID_BATCH;
        if (is_zero(al)) {
            const hipError_t e = launch_scal_ptrs<T>(leny, be, y + b0, a.y_shift, incy, s, nb);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        a.A_ptrs = A + b0; a.x_ptrs = x + b0; a.y_ptrs = y + b0;
        if (m >= Traits<T>::VEC && m <= gemv_tiny_rows<T>(notrans)) {
            const hipError_t e = launch_gemv_tiny<T>(a, notrans ? 0 : (ct ? 2 : 1), s, nb);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        GemvPlan<T> plan = plan_gemv<T>(notrans, m, n, some_aligned_address(), lda, false);
        plan.shift = 0;
        plan.ntiles = ceil_div(m, (int64_t)tile_rows<T>());
        plan.splits = 1;
        plan.short_form = (!notrans && plan.ntiles <= 2) ? 1 : 0;
        plan.row_tiles = 1;
        a.plan = plan;
        const hipError_t e = notrans ? launch_gemv_n<T>(a, s, nb) : launch_gemv_t<T>(a, ct, s, nb);
        if (e != hipSuccess) return hip_code(e);
    }
    return KMV_OK;
}

template <class T>
int symv_ptr_batched_entry(bool herm, char uplo, int64_t n, const T* alpha, const T* const* A, int64_t lda,
                           const T* const* x, int64_t incx, const T* beta, T* const* y, int64_t incy, int64_t batch,
                           void* stream) {
    const bool lower = (uplo == 'L' || uplo == 'l');
    const bool upper = (uplo == 'U' || uplo == 'u');
    if (!lower && !upper) return -1;
    if (n < 0) return -2;
    if (lda < (n > 1 ? n : 1)) return -5;
    if (incx != 1) return -7;
    if (incy == 0) return -10;
    if (batch < 0) return -11;
    if (!alpha || !beta) return KMV_ERR_NULL;
    const T al = *alpha, be = *beta;
    if (n == 0 || batch == 0 || (is_zero(al) && is_one(be))) return KMV_OK;
    if (!y || (!is_zero(al) && (!A || !x))) return KMV_ERR_NULL;
    hipStream_t s = static_cast<hipStream_t>(stream);
    SymvArgs<T> a;
    a.n = n; a.lda = lda;
    a.A = nullptr; a.x = nullptr; a.y = nullptr;
    a.incy = incy; a.alpha = al; a.beta = be;
    a.wsn = nullptr; a.wst = nullptr;
    a.y_shift = incy < 0 ? (1 - n) * incy : 0;
    for (int64_t b0 = 0; b0 < batch; b0 += MAX_GRID_BATCH) {
        const int64_t nb = batch - b0 < MAX_GRID_BATCH ? batch - b0 : MAX_GRID_BATCH;
        if (is_zero(al)) {
            const hipError_t e = launch_scal_ptrs<T>(n, be, y + b0, a.y_shift, incy, s, nb);
            if (e != hipSuccess) return hip_code(e);
            continue;
        }
        a.A_ptrs = A + b0; a.x_ptrs = x + b0; a.y_ptrs = y + b0;
        SymvPlan<T> plan = plan_symv<T>(lower, n, some_aligned_address(), lda);
        plan.shift = 0;
        plan.variant = n <= member_rows<T>() ? 4 : 3;
        a.plan = plan;
        const hipError_t e = launch_symv<T>(a, lower, herm, s, nb);
        if (e != hipSuccess) return hip_code(e);
    }
    return KMV_OK;
}

template <class T> size_t gemv_ws(char trans, int64_t m, int64_t n) {
    const bool notrans = (trans == 'N' || trans == 'n');
    if (m <= 0 || n <= 0) return 0;   // an empty product returns before it would use a workspace
    return plan_gemv<T>(notrans, m, n, nullptr, 0).total_bytes;
}
template <class T> size_t symv_ws(char uplo, int64_t n) {
    if (n <= 0) return 0;
    return plan_symv<T>(uplo == 'L' || uplo == 'l', n, nullptr, 0).total_bytes;
}

struct Key { const char* name; int64_t Tuning::*field; int64_t lo, hi; };
const Key KEYS[] = {
    {"gemv_n_splits", &Tuning::gemv_n_splits, 0, 256},
    {"gemv_t_splits", &Tuning::gemv_t_splits, 0, 256},
    {"gemv_n_row_tiles", &Tuning::gemv_n_row_tiles, 0, 4},
    {"gemv_t_wgs", &Tuning::gemv_t_wgs, 0, 65535},
    {"gemv_short", &Tuning::gemv_short, 0, 2},
    {"gemv_align_classes", &Tuning::gemv_align_classes, 0, 2},
    {"symv_tiles_per_wave", &Tuning::symv_tiles_per_wave, 0, 4},
    {"symv_variant", &Tuning::symv_variant, 0, 3},
    {"symv_unit_tiles", &Tuning::symv_unit_tiles, 0, 2},
    {"symv_piece_fixed", &Tuning::symv_piece_fixed, 0, 17},
    {"symv_edge_weight", &Tuning::symv_edge_weight, 0, 17},
    {"wg_target", &Tuning::wg_target, 0, 1 << 20},
    {"symv_member_rows", &Tuning::symv_member_rows, 0, 1024},
    {"symv_member_waves", &Tuning::symv_member_waves, 0, 8},
    {"symv_small_waves", &Tuning::symv_small_waves, 0, 16},
    {"gemv_tiny_rows", &Tuning::gemv_tiny_rows, 0, 1024},
    {"tuned_table", &Tuning::tuned_table, 0, 1},
};

}  // namespace
}  // namespace kmv

using namespace kmv;

extern "C" {

int kmv_sgemv(char trans, int64_t m, int64_t n, const float* alpha, const float* A, int64_t lda, const float* x,
              int64_t incx, const float* beta, float* y, int64_t incy, void* ws, size_t wsb, void* stream) {
    return gemv_entry<float>(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, ws, wsb, stream);
}
int kmv_dgemv(char trans, int64_t m, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x,
              int64_t incx, const double* beta, double* y, int64_t incy, void* ws, size_t wsb, void* stream) {
    return gemv_entry<double>(trans, m, n, alpha, A, lda, x, incx, beta, y, incy, ws, wsb, stream);
}
int kmv_cgemv(char trans, int64_t m, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return gemv_entry<cf32>(trans, m, n, (const cf32*)alpha, (const cf32*)A, lda, (const cf32*)x, incx,
                            (const cf32*)beta, (cf32*)y, incy, ws, wsb, stream);
}
int kmv_zgemv(char trans, int64_t m, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return gemv_entry<cf64>(trans, m, n, (const cf64*)alpha, (const cf64*)A, lda, (const cf64*)x, incx,
                            (const cf64*)beta, (cf64*)y, incy, ws, wsb, stream);
}

int kmv_ssymv(char uplo, int64_t n, const float* alpha, const float* A, int64_t lda, const float* x, int64_t incx,
              const float* beta, float* y, int64_t incy, void* ws, size_t wsb, void* stream) {
    return symv_entry<float>(false, uplo, n, alpha, A, lda, x, incx, beta, y, incy, ws, wsb, stream);
}
int kmv_dsymv(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x, int64_t incx,
              const double* beta, double* y, int64_t incy, void* ws, size_t wsb, void* stream) {
    return symv_entry<double>(false, uplo, n, alpha, A, lda, x, incx, beta, y, incy, ws, wsb, stream);
}
int kmv_chemv(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return symv_entry<cf32>(true, uplo, n, (const cf32*)alpha, (const cf32*)A, lda, (const cf32*)x, incx, (const cf32*)beta,
                            (cf32*)y, incy, ws, wsb, stream);
}
int kmv_zhemv(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return symv_entry<cf64>(true, uplo, n, (const cf64*)alpha, (const cf64*)A, lda, (const cf64*)x, incx, (const cf64*)beta,
                            (cf64*)y, incy, ws, wsb, stream);
}
int kmv_csymv(char uplo, int64_t n, const kmv_complex64* alpha, const kmv_complex64* A, int64_t lda,
              const kmv_complex64* x, int64_t incx, const kmv_complex64* beta, kmv_complex64* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return symv_entry<cf32>(false, uplo, n, (const cf32*)alpha, (const cf32*)A, lda, (const cf32*)x, incx,
                            (const cf32*)beta, (cf32*)y, incy, ws, wsb, stream);
}
int kmv_zsymv(char uplo, int64_t n, const kmv_complex128* alpha, const kmv_complex128* A, int64_t lda,
              const kmv_complex128* x, int64_t incx, const kmv_complex128* beta, kmv_complex128* y, int64_t incy,
              void* ws, size_t wsb, void* stream) {
    return symv_entry<cf64>(false, uplo, n, (const cf64*)alpha, (const cf64*)A, lda, (const cf64*)x, incx,
                            (const cf64*)beta, (cf64*)y, incy, ws, wsb, stream);
}

#define KMV_GEMV_OFFSET(NAME, CT, T)                                                                              \
    int NAME(char trans, int64_t m, int64_t n, const CT* alpha, const CT* A, int64_t lda, const CT* x,            \
             int64_t incx, const CT* beta, CT* y, int64_t incy, int64_t offset_r, int64_t offset_c, void* ws,     \
             size_t wsb, void* stream) {                                                                          \
        return gemv_offset_entry<T>(trans, m, n, (const T*)alpha, (const T*)A, lda, (const T*)x, incx,            \
                                    (const T*)beta, (T*)y, incy, offset_r, offset_c, ws, wsb, stream);            \
    }
KMV_GEMV_OFFSET(kmv_sgemv_offset, float, float)
KMV_GEMV_OFFSET(kmv_dgemv_offset, double, double)
KMV_GEMV_OFFSET(kmv_cgemv_offset, kmv_complex64, cf32)
KMV_GEMV_OFFSET(kmv_zgemv_offset, kmv_complex128, cf64)
#undef KMV_GEMV_OFFSET

#define KMV_SYMV_OFFSET(NAME, CT, T, HERM)                                                                        \
    int NAME(char uplo, int64_t n, const CT* alpha, const CT* A, int64_t lda, const CT* x, int64_t incx,          \
             const CT* beta, CT* y, int64_t incy, int64_t offset, void* ws, size_t wsb, void* stream) {           \
        return symv_offset_entry<T>(HERM, uplo, n, (const T*)alpha, (const T*)A, lda, (const T*)x, incx,          \
                                    (const T*)beta, (T*)y, incy, offset, ws, wsb, stream);                        \
    }
KMV_SYMV_OFFSET(kmv_ssymv_offset, float, float, false)
KMV_SYMV_OFFSET(kmv_dsymv_offset, double, double, false)
KMV_SYMV_OFFSET(kmv_chemv_offset, kmv_complex64, cf32, true)
KMV_SYMV_OFFSET(kmv_zhemv_offset, kmv_complex128, cf64, true)
KMV_SYMV_OFFSET(kmv_csymv_offset, kmv_complex64, cf32, false)
KMV_SYMV_OFFSET(kmv_zsymv_offset, kmv_complex128, cf64, false)
#undef KMV_SYMV_OFFSET

// alpha and beta in device memory
#define KMV_GEMV_DEVSCALARS(NAME, CT, T)                                                                          \
    int NAME(char trans, int64_t m, int64_t n, const CT* alpha, const CT* A, int64_t lda, const CT* x,            \
             int64_t incx, const CT* beta, CT* y, int64_t incy, void* ws, size_t wsb, void* stream) {             \
        return gemv_entry<T>(trans, m, n, (const T*)alpha, (const T*)A, lda, (const T*)x, incx, (const T*)beta,   \
                             (T*)y, incy, ws, wsb, stream, true);                                                 \
    }
KMV_GEMV_DEVSCALARS(kmv_sgemv_devscalars, float, float)
KMV_GEMV_DEVSCALARS(kmv_dgemv_devscalars, double, double)
KMV_GEMV_DEVSCALARS(kmv_cgemv_devscalars, kmv_complex64, cf32)
KMV_GEMV_DEVSCALARS(kmv_zgemv_devscalars, kmv_complex128, cf64)
#undef KMV_GEMV_DEVSCALARS

#define KMV_SYMV_DEVSCALARS(NAME, CT, T, HERM)                                                                    \
    int NAME(char uplo, int64_t n, const CT* alpha, const CT* A, int64_t lda, const CT* x, int64_t incx,          \
             const CT* beta, CT* y, int64_t incy, void* ws, size_t wsb, void* stream) {                           \
        return symv_entry<T>(HERM, uplo, n, (const T*)alpha, (const T*)A, lda, (const T*)x, incx, (const T*)beta, \
                             (T*)y, incy, ws, wsb, stream, true);                                                 \
    }
KMV_SYMV_DEVSCALARS(kmv_ssymv_devscalars, float, float, false)
KMV_SYMV_DEVSCALARS(kmv_dsymv_devscalars, double, double, false)
KMV_SYMV_DEVSCALARS(kmv_chemv_devscalars, kmv_complex64, cf32, true)
KMV_SYMV_DEVSCALARS(kmv_zhemv_devscalars, kmv_complex128, cf64, true)
KMV_SYMV_DEVSCALARS(kmv_csymv_devscalars, kmv_complex64, cf32, false)
KMV_SYMV_DEVSCALARS(kmv_zsymv_devscalars, kmv_complex128, cf64, false)
#undef KMV_SYMV_DEVSCALARS

// strided batches
#define KMV_GEMV_BATCHED(NAME, CT, T)                                                                             \
    int NAME(char trans, int64_t m, int64_t n, const CT* alpha, const CT* A, int64_t lda, int64_t strideA,        \
             const CT* x, int64_t incx, int64_t stridex, const CT* beta, CT* y, int64_t incy, int64_t stridey,    \
             int64_t batch, void* stream) {                                                                       \
        return gemv_batched_entry<T>(trans, m, n, (const T*)alpha, (const T*)A, lda, strideA, (const T*)x, incx,  \
                                     stridex, (const T*)beta, (T*)y, incy, stridey, batch, stream);               \
    }
KMV_GEMV_BATCHED(kmv_sgemv_strided_batched, float, float)
KMV_GEMV_BATCHED(kmv_dgemv_strided_batched, double, double)
KMV_GEMV_BATCHED(kmv_cgemv_strided_batched, kmv_complex64, cf32)
KMV_GEMV_BATCHED(kmv_zgemv_strided_batched, kmv_complex128, cf64)
#undef KMV_GEMV_BATCHED

#define KMV_SYMV_BATCHED(NAME, CT, T, HERM)                                                                       \
    int NAME(char uplo, int64_t n, const CT* alpha, const CT* A, int64_t lda, int64_t strideA, const CT* x,       \
             int64_t incx, int64_t stridex, const CT* beta, CT* y, int64_t incy, int64_t stridey, int64_t batch,  \
             void* stream) {                                                                                      \
        return symv_batched_entry<T>(HERM, uplo, n, (const T*)alpha, (const T*)A, lda, strideA, (const T*)x,      \
                                     incx, stridex, (const T*)beta, (T*)y, incy, stridey, batch, stream);         \
    }
KMV_SYMV_BATCHED(kmv_ssymv_strided_batched, float, float, false)
KMV_SYMV_BATCHED(kmv_dsymv_strided_batched, double, double, false)
KMV_SYMV_BATCHED(kmv_chemv_strided_batched, kmv_complex64, cf32, true)
KMV_SYMV_BATCHED(kmv_zhemv_strided_batched, kmv_complex128, cf64, true)
KMV_SYMV_BATCHED(kmv_csymv_strided_batched, kmv_complex64, cf32, false)
KMV_SYMV_BATCHED(kmv_zsymv_strided_batched, kmv_complex128, cf64, false)
#undef KMV_SYMV_BATCHED

// pointer-array batches
#define KMV_GEMV_PTR_BATCHED(NAME, CT, T)                                                                         \
    int NAME(char trans, int64_t m, int64_t n, const CT* alpha, const CT* const* A, int64_t lda,                  \
             const CT* const* x, int64_t incx, const CT* beta, CT* const* y, int64_t incy, int64_t batch,         \
             void* stream) {                                                                                      \
        return gemv_ptr_batched_entry<T>(trans, m, n, (const T*)alpha, (const T* const*)A, lda,                   \
                                         (const T* const*)x, incx, (const T*)beta, (T* const*)y, incy, batch,     \
                                         stream);                                                                 \
    }
KMV_GEMV_PTR_BATCHED(kmv_sgemv_batched, float, float)
KMV_GEMV_PTR_BATCHED(kmv_dgemv_batched, double, double)
KMV_GEMV_PTR_BATCHED(kmv_cgemv_batched, kmv_complex64, cf32)
KMV_GEMV_PTR_BATCHED(kmv_zgemv_batched, kmv_complex128, cf64)
#undef KMV_GEMV_PTR_BATCHED

#define KMV_SYMV_PTR_BATCHED(NAME, CT, T, HERM)                                                                   \
    int NAME(char uplo, int64_t n, const CT* alpha, const CT* const* A, int64_t lda, const CT* const* x,          \
             int64_t incx, const CT* beta, CT* const* y, int64_t incy, int64_t batch, void* stream) {             \
        return symv_ptr_batched_entry<T>(HERM, uplo, n, (const T*)alpha, (const T* const*)A, lda,                 \
                                         (const T* const*)x, incx, (const T*)beta, (T* const*)y, incy, batch,     \
                                         stream);                                                                 \
    }
KMV_SYMV_PTR_BATCHED(kmv_ssymv_batched, float, float, false)
KMV_SYMV_PTR_BATCHED(kmv_dsymv_batched, double, double, false)
KMV_SYMV_PTR_BATCHED(kmv_chemv_batched, kmv_complex64, cf32, true)
KMV_SYMV_PTR_BATCHED(kmv_zhemv_batched, kmv_complex128, cf64, true)
KMV_SYMV_PTR_BATCHED(kmv_csymv_batched, kmv_complex64, cf32, false)
KMV_SYMV_PTR_BATCHED(kmv_zsymv_batched, kmv_complex128, cf64, false)
#undef KMV_SYMV_PTR_BATCHED

size_t kmv_gemv_workspace_bytes(char prec, char trans, int64_t m, int64_t n) {
    switch (prec) {
        case 's': return gemv_ws<float>(trans, m, n);
        case 'd': return gemv_ws<double>(trans, m, n);
        case 'c': return gemv_ws<cf32>(trans, m, n);
        case 'z': return gemv_ws<cf64>(trans, m, n);
    }
    return 0;
}
size_t kmv_symv_workspace_bytes(char prec, char uplo, int64_t n) {
    switch (prec) {
        case 's': return symv_ws<float>(uplo, n);
        case 'd': return symv_ws<double>(uplo, n);
        case 'c': return symv_ws<cf32>(uplo, n);
        case 'z': return symv_ws<cf64>(uplo, n);
    }
    return 0;
}

void kmv_partition(int64_t W, int64_t Y, int64_t y, int64_t* w, int64_t* s) {
    int64_t ww = 0, ss = 0;
    if (Y > 0 && y >= 0 && y < Y && W >= 0) partition(W, Y, y, ww, ss);
    if (w) *w = ww;
    if (s) *s = ss;
}

int kmv_stream_probe(int kind, int64_t n, const double* a, double* b, double* c, double* sink, void* stream) {
    if (kind < 0 || kind > 3 || n < 0) return -1;
    const bool reads = kind == 0 || kind == 3;
    if (!a || (reads && !sink) || (!reads && !b) || (kind == 2 && !c)) return KMV_ERR_NULL;
    return hip_code(launch_stream_probe(kind, n, a, b, c, sink, static_cast<hipStream_t>(stream)));
}

int kmv_set_tuning(const char* key, int64_t value) {
    if (!key) return -1;
    for (const Key& k : KEYS)
        if (strcmp(k.name, key) == 0) {
            if (value < k.lo || value > k.hi) return -1;
            if (k.field == &Tuning::gemv_n_row_tiles && value == 3) return -1;
            if (k.field == &Tuning::symv_member_waves && value != 0 && value != 4 && value != 8) return -1;
            if (k.field == &Tuning::symv_small_waves && value != 0 && value != 4 && value != 8 && value != 16) return -1;
            if (k.field == &Tuning::symv_variant && value == 1) return -1;
            tuning().*(k.field) = value;
            return 0;
        }
    return -1;
}
int64_t kmv_get_tuning(const char* key) {
    if (!key) return -1;
    for (const Key& k : KEYS)
        if (strcmp(k.name, key) == 0) return tuning().*(k.field);
    return -1;
}
const char* kmv_tuning_keys(void) { return "gemv_n_splits,gemv_t_splits,gemv_n_row_tiles,gemv_t_wgs,gemv_short,gemv_align_classes,symv_tiles_per_wave,symv_variant,symv_unit_tiles,symv_piece_fixed,symv_edge_weight,wg_target,symv_member_rows,symv_member_waves,symv_small_waves,gemv_tiny_rows,tuned_table"; }

int kmv_tuned_settings(char prec, char op, int64_t n, int64_t* values) {
    if (!values || n < 0 || !strchr("sdcz", prec) || prec == 0 || !strchr("NTLU", op) || op == 0) return -1;
    if (tuning().tuned_table == 1) return 0;
    for (const TunedRow* r = TUNED_ROWS; r->op; ++r)
        if (r->op == op && r->prec == prec && n >= r->n_lo && n < r->n_hi) {
            const int64_t v[7] = {r->gemv_n_splits, r->gemv_n_row_tiles, r->gemv_t_splits, r->symv_variant,
                                  r->symv_tiles_per_wave, r->symv_unit_tiles, r->wg_target};
            for (int i = 0; i < 7; ++i) values[i] = v[i];
            return 1;
        }
    return 0;
}

int kmv_symv_kernel_variant(char prec, char uplo, int64_t n, const void* A, int64_t lda) {
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if ((!lower && !upper) || n < 0 || lda < (n > 1 ? n : 1)) return 0;
    // a null A would ask the planner for the workspace bound instead of a launch plan
    const void* base = A ? A : reinterpret_cast<const void*>(uintptr_t(WS_ALIGN));
    switch (prec) {
        case 's': return plan_symv<float>(lower, n, base, lda).variant;
        case 'd': return plan_symv<double>(lower, n, base, lda).variant;
        case 'c': return plan_symv<cf32>(lower, n, base, lda).variant;
        case 'z': return plan_symv<cf64>(lower, n, base, lda).variant;
    }
    return 0;
}

int kmv_symv_shares(char prec, char uplo, int64_t n, int shift, int chunk_tiles, int unit_tiles, int64_t slots, int fixed,
                    int edge, uint32_t* start, uint16_t* first, uint16_t* last, int64_t* work) {
    const bool lower = (uplo == 'L' || uplo == 'l'), upper = (uplo == 'U' || uplo == 'u');
    if ((!lower && !upper) || n < 1 || n > ((int64_t)1 << 30) || shift < 0 || (chunk_tiles != 4 && chunk_tiles != 8 && chunk_tiles != 12 && chunk_tiles != 16) ||
        (unit_tiles != 1 && unit_tiles != 2) || slots < 1 || fixed < 0 || fixed > 16 || edge < 0 || edge > 16)
        return -1;
    const SymvBalanced* b = nullptr;
    int tr = 0;
    switch (prec) {
        case 's': tr = tile_rows<float>(); break;
        case 'd': tr = tile_rows<double>(); break;
        case 'c': tr = tile_rows<cf32>(); break;
        case 'z': tr = tile_rows<cf64>(); break;
        default: return -1;
    }
    if (shift >= tr || ceil_div(ceil_div(n + shift, tr), chunk_tiles) + 1 > SHARE_MAX_CHUNKS) return -1;
    switch (prec) {
        case 's': b = symv_shares<float>(lower, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge); break;
        case 'd': b = symv_shares<double>(lower, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge); break;
        case 'c': b = symv_shares<cf32>(lower, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge); break;
        case 'z': b = symv_shares<cf64>(lower, n, shift, chunk_tiles, unit_tiles, slots, fixed, edge); break;
    }
    if (!b) return -1;
    if (start) memcpy(start, b->shares.start, sizeof(uint32_t) * (size_t)(b->workers + 1));
    if (first) memcpy(first, b->owners.first, sizeof(b->owners.first));
    if (last) memcpy(last, b->owners.last, sizeof(b->owners.last));
    if (work) *work = b->work;
    return b->workers;
}

int kmv_dsymv_static(char uplo, int64_t n, const double* alpha, const double* A, int64_t lda, const double* x,
                     int64_t incx, const double* beta, double* y, int64_t incy, void* stream) {
    // the device address of this device's copy of the array, looked up once per device
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_code(e);
    if (dev < 0 || dev >= MAX_CACHED_DEVICES) return KMV_ERR_HIP + (int)hipErrorInvalidDevice;
    void* ptr = nullptr;
    {
        std::lock_guard<std::mutex> lock(static_scratch_mutex);
        if (!static_scratch_ptr[dev]) {
            void* p = nullptr;
            e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
            if (e != hipSuccess) return hip_code(e);
            if (!p) return KMV_ERR_HIP + (int)hipErrorInvalidSymbol;
            static_scratch_ptr[dev] = p;
        }
        ptr = static_scratch_ptr[dev];
    }
    // sizes whose partial sums do not fit the array are refused before anything is enqueued
    // (symv_entry compares the plan's need with the size given here)
    return symv_entry<double>(false, uplo, n, alpha, A, lda, x, incx, beta, y, incy, ptr, KMV_STATIC_SCRATCH_BYTES, stream);
}

const char* kmv_version(void) { return "kmv 0.1 (gfx950)"; }

}  // extern "C"
