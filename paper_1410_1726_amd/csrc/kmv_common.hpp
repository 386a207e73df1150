// Device-side building blocks shared by the kmv kernels (gfx950, wave64).
//
// Element types, 16-byte vector loads, fused multiply-adds for the four
// precisions, wave-level reductions and the balanced work partition of the
// paper's Section 6.2.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace kmv {

struct cf32 { float re, im; };
struct cf64 { double re, im; };

constexpr int WAVE = 64;

template <class T> struct Traits;
template <> struct Traits<float>  { typedef float real;  static constexpr int VEC = 4; static constexpr bool cplx = false; };
template <> struct Traits<double> { typedef double real; static constexpr int VEC = 2; static constexpr bool cplx = false; };
template <> struct Traits<cf32>   { typedef float real;  static constexpr int VEC = 2; static constexpr bool cplx = true; };
template <> struct Traits<cf64>   { typedef double real; static constexpr int VEC = 1; static constexpr bool cplx = true; };

// VEC consecutive column elements = 16 bytes = what one lane loads at a time;
// a wave covers TR = 64*VEC consecutive rows (1 KiB) per load instruction.
template <class T> struct Vec { T e[Traits<T>::VEC]; };
template <class T> constexpr int tile_rows() { return WAVE * Traits<T>::VEC; }

// ---- scalar helpers --------------------------------------------------------
template <class T> __host__ __device__ __forceinline__ T zero_of();
template <> __host__ __device__ __forceinline__ float zero_of<float>() { return 0.f; }
template <> __host__ __device__ __forceinline__ double zero_of<double>() { return 0.0; }
template <> __host__ __device__ __forceinline__ cf32 zero_of<cf32>() { return cf32{0.f, 0.f}; }
template <> __host__ __device__ __forceinline__ cf64 zero_of<cf64>() { return cf64{0.0, 0.0}; }

__host__ __device__ __forceinline__ bool is_zero(float v) { return v == 0.f; }
__host__ __device__ __forceinline__ bool is_zero(double v) { return v == 0.0; }
__host__ __device__ __forceinline__ bool is_zero(cf32 v) { return v.re == 0.f && v.im == 0.f; }
__host__ __device__ __forceinline__ bool is_zero(cf64 v) { return v.re == 0.0 && v.im == 0.0; }
__host__ __device__ __forceinline__ bool is_one(float v) { return v == 1.f; }
__host__ __device__ __forceinline__ bool is_one(double v) { return v == 1.0; }
__host__ __device__ __forceinline__ bool is_one(cf32 v) { return v.re == 1.f && v.im == 0.f; }
__host__ __device__ __forceinline__ bool is_one(cf64 v) { return v.re == 1.0 && v.im == 0.0; }

// acc += a * x
__device__ __forceinline__ void fma_acc(float& acc, float a, float x) { acc = fmaf(a, x, acc); }
__device__ __forceinline__ void fma_acc(double& acc, double a, double x) { acc = fma(a, x, acc); }
__device__ __forceinline__ void fma_acc(cf32& acc, cf32 a, cf32 x) {
    acc.re = fmaf(a.re, x.re, acc.re); acc.re = fmaf(-a.im, x.im, acc.re);
    acc.im = fmaf(a.re, x.im, acc.im); acc.im = fmaf(a.im, x.re, acc.im);
}
__device__ __forceinline__ void fma_acc(cf64& acc, cf64 a, cf64 x) {
    acc.re = fma(a.re, x.re, acc.re); acc.re = fma(-a.im, x.im, acc.re);
    acc.im = fma(a.re, x.im, acc.im); acc.im = fma(a.im, x.re, acc.im);
}
// acc += conj(a) * x
__device__ __forceinline__ void fma_acc_conj(float& acc, float a, float x) { acc = fmaf(a, x, acc); }
__device__ __forceinline__ void fma_acc_conj(double& acc, double a, double x) { acc = fma(a, x, acc); }
__device__ __forceinline__ void fma_acc_conj(cf32& acc, cf32 a, cf32 x) {
    acc.re = fmaf(a.re, x.re, acc.re); acc.re = fmaf(a.im, x.im, acc.re);
    acc.im = fmaf(a.re, x.im, acc.im); acc.im = fmaf(-a.im, x.re, acc.im);
}
__device__ __forceinline__ void fma_acc_conj(cf64& acc, cf64 a, cf64 x) {
    acc.re = fma(a.re, x.re, acc.re); acc.re = fma(a.im, x.im, acc.re);
    acc.im = fma(a.re, x.im, acc.im); acc.im = fma(-a.im, x.re, acc.im);
}
template <bool CONJ, class T> __device__ __forceinline__ void fma_op(T& acc, T a, T x) {
    if (CONJ) fma_acc_conj(acc, a, x); else fma_acc(acc, a, x);
}

__device__ __forceinline__ float add_of(float a, float b) { return a + b; }
__device__ __forceinline__ double add_of(double a, double b) { return a + b; }
__device__ __forceinline__ cf32 add_of(cf32 a, cf32 b) { return cf32{a.re + b.re, a.im + b.im}; }
__device__ __forceinline__ cf64 add_of(cf64 a, cf64 b) { return cf64{a.re + b.re, a.im + b.im}; }

__device__ __forceinline__ float mul_of(float a, float b) { return a * b; }
__device__ __forceinline__ double mul_of(double a, double b) { return a * b; }
__device__ __forceinline__ cf32 mul_of(cf32 a, cf32 b) { cf32 r = zero_of<cf32>(); fma_acc(r, a, b); return r; }
__device__ __forceinline__ cf64 mul_of(cf64 a, cf64 b) { cf64 r = zero_of<cf64>(); fma_acc(r, a, b); return r; }

// c ? a : b, member by member (keeps complex values in registers)
__device__ __forceinline__ float select_of(bool c, float a, float b) { return c ? a : b; }
__device__ __forceinline__ double select_of(bool c, double a, double b) { return c ? a : b; }
__device__ __forceinline__ cf32 select_of(bool c, cf32 a, cf32 b) { return cf32{c ? a.re : b.re, c ? a.im : b.im}; }
__device__ __forceinline__ cf64 select_of(bool c, cf64 a, cf64 b) { return cf64{c ? a.re : b.re, c ? a.im : b.im}; }

// HEMV uses only the real part of a diagonal element
__device__ __forceinline__ float real_part_only(float a) { return a; }
__device__ __forceinline__ double real_part_only(double a) { return a; }
__device__ __forceinline__ cf32 real_part_only(cf32 a) { return cf32{a.re, 0.f}; }
__device__ __forceinline__ cf64 real_part_only(cf64 a) { return cf64{a.re, 0.0}; }

// A scalar of the call: the value copied at enqueue time, or, when the caller keeps its scalars
// in device memory, the value found there when the kernel runs (a wave-uniform load).
template <class T> __device__ __forceinline__ T scalar_of(T value, const T* dev) { return dev ? *dev : value; }

// alpha*sum (+ beta*yold when beta != 0; yold is not read otherwise).  alpha == 0 can only arrive
// through a device-resident scalar (the host path returns earlier); the sum then does not count,
// whatever it holds.
template <class T> __device__ __forceinline__ T epilogue(T alpha, T sum, T beta, const T* yold) {
    T r = is_zero(alpha) ? zero_of<T>() : mul_of(alpha, sum);
    if (!is_zero(beta)) r = add_of(r, mul_of(beta, *yold));
    return r;
}

// ---- 16-byte loads -----------------------------------------------------------
// The vector type carries only 4-byte alignment: sub-block pointers and odd
// leading dimensions give columns that are merely element aligned, and global
// memory accepts such dwordx4 accesses.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef u32x4 u32x4_a4 __attribute__((aligned(4)));

// streaming load of matrix data (read once, never reused: non-temporal hint)
template <class T> __device__ __forceinline__ Vec<T> load_stream(const T* p) {
    u32x4 raw = __builtin_nontemporal_load(reinterpret_cast<const u32x4_a4*>(p));
    Vec<T> v;
    __builtin_memcpy(&v, &raw, 16);
    return v;
}
// cached load (vector operands that every workgroup re-reads from L2)
template <class T> __device__ __forceinline__ Vec<T> load_cached(const T* p) {
    u32x4 raw = *reinterpret_cast<const u32x4_a4*>(p);
    Vec<T> v;
    __builtin_memcpy(&v, &raw, 16);
    return v;
}
template <class T> __device__ __forceinline__ void store_vec(T* p, const Vec<T>& v) {
    u32x4 raw;
    __builtin_memcpy(&raw, &v, 16);
    *reinterpret_cast<u32x4_a4*>(p) = raw;
}
// streaming store (written once, read once by a later kernel)
template <class T> __device__ __forceinline__ void store_vec_stream(T* p, const Vec<T>& v) {
    u32x4 raw;
    __builtin_memcpy(&raw, &v, 16);
    __builtin_nontemporal_store(raw, reinterpret_cast<u32x4_a4*>(p));
}
template <class T> __device__ __forceinline__ T load_elem_stream(const T* p) {
    return __builtin_nontemporal_load(p);
}
template <> __device__ __forceinline__ cf32 load_elem_stream<cf32>(const cf32* p) {
    const float* q = reinterpret_cast<const float*>(p);
    return cf32{__builtin_nontemporal_load(q), __builtin_nontemporal_load(q + 1)};
}
template <> __device__ __forceinline__ cf64 load_elem_stream<cf64>(const cf64* p) {
    const double* q = reinterpret_cast<const double*>(p);
    return cf64{__builtin_nontemporal_load(q), __builtin_nontemporal_load(q + 1)};
}

// element e of the result = element e + d of v (lanes of an edge tile whose
// vector was loaded at a clamped position; elements that fall outside belong to
// rows that do not exist or are not stored, and may hold anything)
template <class T> __device__ __forceinline__ Vec<T> shift_elems(const Vec<T>& v, int d) {
    constexpr int VEC = Traits<T>::VEC;
    Vec<T> o = v;
#pragma unroll
    for (int e = 0; e < VEC; ++e)
#pragma unroll
        for (int k = 0; k < VEC; ++k) o.e[e] = select_of(e + d == k, v.e[k], o.e[e]);
    return o;
}

// ---- wave64 sum: DPP inside each row of 16 lanes, then the four row sums are
// read in lane order 0,16,32,48 and added left to right (a fixed order). The
// result is wave-uniform.
template <int CTRL> __device__ __forceinline__ int dpp_i32(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
template <int CTRL> __device__ __forceinline__ float dpp_move(float v) {
    return __builtin_bit_cast(float, dpp_i32<CTRL>(__builtin_bit_cast(int, v)));
}
template <int CTRL> __device__ __forceinline__ double dpp_move(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)dpp_i32<CTRL>((int)(uint32_t)u);
    const uint32_t hi = (uint32_t)dpp_i32<CTRL>((int)(uint32_t)(u >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ float read_lane(float v, int lane) {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), lane));
}
__device__ __forceinline__ double read_lane(double v, int lane) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)u, lane);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(u >> 32), lane);
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
__device__ __forceinline__ cf32 read_lane(cf32 v, int lane) { return cf32{read_lane(v.re, lane), read_lane(v.im, lane)}; }
__device__ __forceinline__ cf64 read_lane(cf64 v, int lane) { return cf64{read_lane(v.re, lane), read_lane(v.im, lane)}; }
template <class R> __device__ __forceinline__ R wave_sum_real(R v) {
    v += dpp_move<0xB1>(v);    // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);    // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);   // row_half_mirror
    v += dpp_move<0x140>(v);   // row_mirror: all 16 lanes of a row hold the row sum
    R s = read_lane(v, 0);
    s += read_lane(v, 16);
    s += read_lane(v, 32);
    s += read_lane(v, 48);
    return s;
}
__device__ __forceinline__ float wave_sum(float v) { return wave_sum_real(v); }
__device__ __forceinline__ double wave_sum(double v) { return wave_sum_real(v); }
__device__ __forceinline__ cf32 wave_sum(cf32 v) { return cf32{wave_sum_real(v.re), wave_sum_real(v.im)}; }
__device__ __forceinline__ cf64 wave_sum(cf64 v) { return cf64{wave_sum_real(v.re), wave_sum_real(v.im)}; }

// ---- sums over groups of lanes, for kernels that put several short columns on one wave: lane = cl * L + sub
// (L lanes per column, 64 / L columns side by side)
template <int M> __device__ __forceinline__ int xor_lane_i32(int v) {
    const int lane = (int)(threadIdx.x & (WAVE - 1));
    return __builtin_amdgcn_ds_bpermute((lane ^ M) << 2, v);
}
template <int M> __device__ __forceinline__ float xor_lane(float v) {
    return __builtin_bit_cast(float, xor_lane_i32<M>(__builtin_bit_cast(int, v)));
}
template <int M> __device__ __forceinline__ double xor_lane(double v) {
    const uint64_t u = __builtin_bit_cast(uint64_t, v);
    const uint32_t lo = (uint32_t)xor_lane_i32<M>((int)(uint32_t)u), hi = (uint32_t)xor_lane_i32<M>((int)(uint32_t)(u >> 32));
    return __builtin_bit_cast(double, ((uint64_t)hi << 32) | lo);
}
// sum over the aligned group of L consecutive lanes (L = 8 .. 64), the same value in each of them
template <int L, class R> __device__ __forceinline__ R seg_sum_real(R v) {
    v += dpp_move<0xB1>(v);                           // quad_perm [1,0,3,2]
    v += dpp_move<0x4E>(v);                           // quad_perm [2,3,0,1]
    v += dpp_move<0x141>(v);                          // row_half_mirror: 8 lanes
    if constexpr (L >= 16) v += dpp_move<0x140>(v);   // row_mirror: 16 lanes
    if constexpr (L >= 32) v += xor_lane<16>(v);
    if constexpr (L >= 64) v += xor_lane<32>(v);
    return v;
}
// sum over the 64 / L lanes that hold the same position in their group of L, the same value in each of them
template <int L, class R> __device__ __forceinline__ R cross_sum_real(R v) {
    if constexpr (L <= 8) v += dpp_move<0x128>(v);    // row_ror 8: the other group of 8 in the row
    if constexpr (L <= 16) v += xor_lane<16>(v);
    if constexpr (L <= 32) v += xor_lane<32>(v);
    return v;
}
template <int L> __device__ __forceinline__ float seg_sum(float v) { return seg_sum_real<L>(v); }
template <int L> __device__ __forceinline__ double seg_sum(double v) { return seg_sum_real<L>(v); }
template <int L> __device__ __forceinline__ cf32 seg_sum(cf32 v) { return cf32{seg_sum_real<L>(v.re), seg_sum_real<L>(v.im)}; }
template <int L> __device__ __forceinline__ cf64 seg_sum(cf64 v) { return cf64{seg_sum_real<L>(v.re), seg_sum_real<L>(v.im)}; }
template <int L> __device__ __forceinline__ float cross_sum(float v) { return cross_sum_real<L>(v); }
template <int L> __device__ __forceinline__ double cross_sum(double v) { return cross_sum_real<L>(v); }
template <int L> __device__ __forceinline__ cf32 cross_sum(cf32 v) { return cf32{cross_sum_real<L>(v.re), cross_sum_real<L>(v.im)}; }
template <int L> __device__ __forceinline__ cf64 cross_sum(cf64 v) { return cf64{cross_sum_real<L>(v.re), cross_sum_real<L>(v.im)}; }


// ---- balanced contiguous partition (Section 6.2, Eqs. local_workload and
// starting_point with W for the misprinted d): worker y of Y gets w items
// starting at s; shares differ by at most one and tile the range [0, W).
__host__ __device__ __forceinline__ void partition(int64_t W, int64_t Y, int64_t y, int64_t& w, int64_t& s) {
    const int64_t q = W / Y, r = W % Y;
    w = q + (y < r ? 1 : 0);
    s = y * q + (y < r ? y : r);
}

__host__ __device__ __forceinline__ int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace kmv
