// Small kernels around the matrix kernels: packing of a strided x, the scaling
// of y when alpha == 0 (the SCAL step of Section 6.4), the fixed-order sum of
// per-workgroup partial vectors with the alpha/beta epilogue (the replacement
// of the atomic accumulation of Section 6.2), and the STREAM-style bandwidth
// probe that Section 7 uses to define the sustained bandwidth of the roofline.
#include "kmv_launch.hpp"

namespace kmv {

template <class T> __global__ void pack_kernel(const T* __restrict__ src, int64_t inc, int64_t len, T* __restrict__ dst) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) dst[k] = src[k * inc];
}

template <class T> __global__ void scal_kernel(int64_t len, T beta, T* y, int64_t incy, int64_t stride) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) {
        T* yp = y + (int64_t)blockIdx.y * stride + k * incy;
        *yp = is_zero(beta) ? zero_of<T>() : mul_of(beta, *yp);
    }
}

// the same for the members of a pointer-array batch: member blockIdx.y scales y_ptrs[blockIdx.y] + shift
template <class T> __global__ void scal_ptrs_kernel(int64_t len, T beta, T* const* y_ptrs, int64_t shift, int64_t incy) {
    const int64_t k = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (k < len) {
        T* yp = y_ptrs[blockIdx.y] + shift + k * incy;
        *yp = is_zero(beta) ? zero_of<T>() : mul_of(beta, *yp);
    }
}

// blockDim = 256 = 32 outputs x 8 groups: group g adds the partial vectors
// g, g+8, ... in ascending order, the eight group sums meet in LDS and are
// added in group order, so the result does not depend on scheduling.
constexpr int RD_OUT = 32, RD_GRP = 8;
template <class T>
__global__ __launch_bounds__(RD_OUT * RD_GRP) void reduce_kernel(const T* __restrict__ partial, int64_t splits,
                                                                  int64_t stride, int64_t off, int64_t len, T alpha,
                                                                  T beta, const T* alpha_dev, const T* beta_dev,
                                                                  T* y, int64_t incy) {
    const int lx = threadIdx.x % RD_OUT, g = threadIdx.x / RD_OUT;
    const int64_t k = (int64_t)blockIdx.x * RD_OUT + lx;
    __shared__ T part[RD_GRP][RD_OUT];
    T s = zero_of<T>();
    if (k < len) {
        const T* p = partial + off + k;
#pragma unroll 4
        for (int64_t i = g; i < splits; i += RD_GRP) s = add_of(s, p[i * stride]);
    }
    part[g][lx] = s;
    __syncthreads();
    if (g == 0 && k < len) {
        T tot = part[0][lx];
#pragma unroll
        for (int gg = 1; gg < RD_GRP; ++gg) tot = add_of(tot, part[gg][lx]);
        T* yp = y + k * incy;
        *yp = epilogue(scalar_of(alpha, alpha_dev), tot, scalar_of(beta, beta_dev), yp);
    }
}

template <class T> hipError_t launch_pack(const T* src, int64_t inc, int64_t len, T* dst, hipStream_t s) {
    if (len <= 0) return hipSuccess;
    hipLaunchKernelGGL((pack_kernel<T>), dim3((unsigned)ceil_div(len, 256)), dim3(256), 0, s, src, inc, len, dst);
    return hipGetLastError();
}
template <class T>
hipError_t launch_scal(int64_t len, T beta, T* y, int64_t incy, hipStream_t s, int64_t batch, int64_t stride) {
    if (len <= 0 || batch <= 0) return hipSuccess;
    if (batch > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL((scal_kernel<T>), dim3((unsigned)ceil_div(len, 256), (unsigned)batch), dim3(256), 0, s, len, beta,
                       y, incy, stride);
    return hipGetLastError();
}
template <class T>
hipError_t launch_scal_ptrs(int64_t len, T beta, T* const* y_ptrs, int64_t shift, int64_t incy, hipStream_t s, int64_t batch) {
    if (len <= 0 || batch <= 0) return hipSuccess;
    if (batch > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL((scal_ptrs_kernel<T>), dim3((unsigned)ceil_div(len, 256), (unsigned)batch), dim3(256), 0, s, len, beta,
                       y_ptrs, shift, incy);
    return hipGetLastError();
}
template <class T>
hipError_t launch_reduce(const T* partial, int64_t splits, int64_t stride, int64_t off, int64_t len, T alpha, T beta,
                         const T* alpha_dev, const T* beta_dev, T* y, int64_t incy, hipStream_t s) {
    if (len <= 0) return hipSuccess;
    hipLaunchKernelGGL((reduce_kernel<T>), dim3((unsigned)ceil_div(len, RD_OUT)), dim3(RD_OUT * RD_GRP), 0, s, partial,
                       splits, stride, off, len, alpha, beta, alpha_dev, beta_dev, y, incy);
    return hipGetLastError();
}

#define KMV_INSTANTIATE_AUX(T)                                                                              \
    template hipError_t launch_pack<T>(const T*, int64_t, int64_t, T*, hipStream_t);                        \
    template hipError_t launch_scal<T>(int64_t, T, T*, int64_t, hipStream_t, int64_t, int64_t);             \
    template hipError_t launch_scal_ptrs<T>(int64_t, T, T* const*, int64_t, int64_t, hipStream_t, int64_t); \
    template hipError_t launch_reduce<T>(const T*, int64_t, int64_t, int64_t, int64_t, T, T, const T*, const T*, T*, \
                                         int64_t, hipStream_t);
KMV_INSTANTIATE_AUX(float)
KMV_INSTANTIATE_AUX(double)
KMV_INSTANTIATE_AUX(cf32)
KMV_INSTANTIATE_AUX(cf64)

// ------------------------------------------------------------- STREAM probe --
// Each lane moves 16-byte vectors; a workgroup of 256 lanes walks a contiguous
// slab so that every wave instruction covers 1 KiB, the same access shape as
// the matrix kernels.
namespace {
constexpr int PROBE_WG = 8192;
typedef double d2 __attribute__((ext_vector_type(2)));

__global__ __launch_bounds__(256) void probe_read(const d2* __restrict__ a, int64_t nvec, double* __restrict__ sink) {
    int64_t w, s;
    partition(ceil_div(nvec, 1024), gridDim.x, blockIdx.x, w, s);   // units of 1024 vectors = 16 KiB
    const int64_t beg = s * 1024, end = (s + w) * 1024 < nvec ? (s + w) * 1024 : nvec;
    d2 acc0 = {0, 0}, acc1 = {0, 0}, acc2 = {0, 0}, acc3 = {0, 0};
    int64_t i = beg + threadIdx.x;
    for (; i + 768 < end; i += 1024) {
        const d2 v0 = __builtin_nontemporal_load(a + i), v1 = __builtin_nontemporal_load(a + i + 256);
        const d2 v2 = __builtin_nontemporal_load(a + i + 512), v3 = __builtin_nontemporal_load(a + i + 768);
        acc0 += v0; acc1 += v1; acc2 += v2; acc3 += v3;
    }
    for (; i < end; i += 256) acc0 += __builtin_nontemporal_load(a + i);
    const d2 t = acc0 + acc1 + acc2 + acc3;
    double r = wave_sum(t.x + t.y);
    __shared__ double red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
// the same with 16 loads in flight per lane (two sets of 8, the next set issued before the current one is summed)
__global__ __launch_bounds__(256) void probe_read_deep(const d2* __restrict__ a, int64_t nvec, double* __restrict__ sink) {
    int64_t w, s;
    partition(ceil_div(nvec, 2048), gridDim.x, blockIdx.x, w, s);   // units of 2048 vectors = 32 KiB
    const int64_t beg = s * 2048, end = (s + w) * 2048 < nvec ? (s + w) * 2048 : nvec;
    d2 acc[8], b0[8], b1[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = d2{0, 0};
    int64_t i = beg + threadIdx.x;
    auto load = [&](d2(&buf)[8], int64_t at) {
#pragma unroll
        for (int u = 0; u < 8; ++u) buf[u] = __builtin_nontemporal_load(a + at + u * 256);
    };
    auto add = [&](const d2(&buf)[8]) {
#pragma unroll
        for (int u = 0; u < 8; ++u) acc[u] += buf[u];
    };
    const int64_t nfull = (end - beg) / 2048;     // whole blocks of 2048 vectors
    if (nfull > 0) load(b0, i);
    for (int64_t k = 0; k < nfull; k += 2) {
        if (k + 1 < nfull) load(b1, i + (k + 1) * 2048);
        add(b0);
        if (k + 1 < nfull) {
            if (k + 2 < nfull) load(b0, i + (k + 2) * 2048);
            add(b1);
        }
    }
    for (int64_t r = i + nfull * 2048; r < end; r += 256) acc[0] += __builtin_nontemporal_load(a + r);
    d2 t = acc[0];
#pragma unroll
    for (int u = 1; u < 8; ++u) t += acc[u];
    double r = wave_sum(t.x + t.y);
    __shared__ double red[4];
    if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = r;
    __syncthreads();
    if (threadIdx.x == 0) sink[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}
__global__ __launch_bounds__(256) void probe_copy(const d2* __restrict__ a, d2* __restrict__ b, int64_t nvec) {
    int64_t w, s;
    partition(ceil_div(nvec, 1024), gridDim.x, blockIdx.x, w, s);
    const int64_t beg = s * 1024, end = (s + w) * 1024 < nvec ? (s + w) * 1024 : nvec;
    int64_t i = beg + threadIdx.x;
    for (; i + 768 < end; i += 1024) {
        const d2 v0 = __builtin_nontemporal_load(a + i), v1 = __builtin_nontemporal_load(a + i + 256);
        const d2 v2 = __builtin_nontemporal_load(a + i + 512), v3 = __builtin_nontemporal_load(a + i + 768);
        __builtin_nontemporal_store(v0, b + i); __builtin_nontemporal_store(v1, b + i + 256);
        __builtin_nontemporal_store(v2, b + i + 512); __builtin_nontemporal_store(v3, b + i + 768);
    }
    for (; i < end; i += 256) __builtin_nontemporal_store(__builtin_nontemporal_load(a + i), b + i);
}
__global__ __launch_bounds__(256) void probe_triad(const d2* __restrict__ a, const d2* __restrict__ b, d2* __restrict__ c,
                                                   int64_t nvec, double sc) {
    int64_t w, s;
    partition(ceil_div(nvec, 1024), gridDim.x, blockIdx.x, w, s);
    const int64_t beg = s * 1024, end = (s + w) * 1024 < nvec ? (s + w) * 1024 : nvec;
    for (int64_t i = beg + threadIdx.x; i < end; i += 256) {
        const d2 va = __builtin_nontemporal_load(a + i), vb = __builtin_nontemporal_load(b + i);
        __builtin_nontemporal_store(va + sc * vb, c + i);
    }
}
}  // namespace

hipError_t launch_stream_probe(int kind, int64_t n, const double* a, double* b, double* c, double* sink, hipStream_t s) {
    const int64_t nvec = n / 2;   // whole 16-byte vectors only
    if (nvec <= 0) return hipSuccess;
    int64_t wg = ceil_div(nvec, 1024);
    if (wg > PROBE_WG) wg = PROBE_WG;
    if (kind == 3) {     // the read probe in the matrix kernels' best launch shape: few workgroups, deep prefetch
        const int64_t want = tuning().wg_target > 0 ? tuning().wg_target : 192;
        if (wg > want) wg = want;
        hipLaunchKernelGGL(probe_read_deep, dim3((unsigned)wg), dim3(256), 0, s, reinterpret_cast<const d2*>(a), nvec, sink);
        return hipGetLastError();
    }
    const dim3 grid((unsigned)wg), block(256);
    if (kind == 0)
        hipLaunchKernelGGL(probe_read, grid, block, 0, s, reinterpret_cast<const d2*>(a), nvec, sink);
    else if (kind == 1)
        hipLaunchKernelGGL(probe_copy, grid, block, 0, s, reinterpret_cast<const d2*>(a), reinterpret_cast<d2*>(b), nvec);
    else
        hipLaunchKernelGGL(probe_triad, grid, block, 0, s, reinterpret_cast<const d2*>(a), reinterpret_cast<const d2*>(b),
                           reinterpret_cast<d2*>(c), nvec, 3.0);
    return hipGetLastError();
}

}  // namespace kmv
