// Column reductions over the node axis and row fills.
//
//  * node mean       xbar = (1/n) sum_i x_i                       (App. A notation)
//  * consensus error ||X - 1 xbar^T||_F^2 = sum_c sum_i (x_ic - xbar_c)^2
//                    (the consensus distance of Sec. 4 / App. B)
//  * fill            every row <- one d-vector (Algorithm 1: all x_i^(0) equal)
//
// Both reductions read X exactly once (4 B per element).  The consensus error
// uses the shifted one-pass form with row 0 as the shift:
//     d_i = x_i - x_0 ;  sum_i (x_i - xbar)^2 = sum_i d_i^2 - (sum_i d_i)^2 / n
// with d_i formed in fp32 (exact or nearly so when rows are close) and both
// sums carried in fp64, so the subtraction never loses the small quantity the
// method is about.  Column results are reduced with a wavefront shuffle, an LDS
// step across waves and one partial per workgroup; a last single-workgroup
// kernel adds the partials in a fixed order (bitwise reproducible).
#include "gpga_internal.hpp"

namespace {

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;
}

template <typename T>
__device__ __forceinline__ T ld_stream(const T* p) {
    return __builtin_nontemporal_load(p);
}

struct d4 {
    double x, y, z, w;
};
__device__ __forceinline__ void acc_add(double& a, float v) { a += (double)v; }
__device__ __forceinline__ void acc_add(d4& a, v4f v) {
    a.x += (double)v.x;
    a.y += (double)v.y;
    a.z += (double)v.z;
    a.w += (double)v.w;
}
__device__ __forceinline__ void acc_sq(double& a, float v) { a += (double)v * (double)v; }
__device__ __forceinline__ void acc_sq(d4& a, v4f v) {
    a.x += (double)v.x * v.x;
    a.y += (double)v.y * v.y;
    a.z += (double)v.z * v.z;
    a.w += (double)v.w * v.w;
}
__device__ __forceinline__ float to_mean(double a, double inv_n) { return (float)(a * inv_n); }
__device__ __forceinline__ v4f to_mean(const d4& a, double inv_n) {
    v4f r;
    r.x = (float)(a.x * inv_n);
    r.y = (float)(a.y * inv_n);
    r.z = (float)(a.z * inv_n);
    r.w = (float)(a.w * inv_n);
    return r;
}
__device__ __forceinline__ double col_ss(double s1, double s2, double inv_n) {
    const double v = s2 - s1 * s1 * inv_n;
    return v > 0.0 ? v : 0.0;
}
__device__ __forceinline__ double col_ss(const d4& s1, const d4& s2, double inv_n) {
    return col_ss(s1.x, s2.x, inv_n) + col_ss(s1.y, s2.y, inv_n) + col_ss(s1.z, s2.z, inv_n) +
           col_ss(s1.w, s2.w, inv_n);
}

template <typename T>
struct AccOf;
template <>
struct AccOf<float> {
    typedef double type;
    __device__ static double zero() { return 0.0; }
};
template <>
struct AccOf<v4f> {
    typedef d4 type;
    __device__ static d4 zero() { return {0.0, 0.0, 0.0, 0.0}; }
};

constexpr int U = 4;

template <typename T>
__global__ void __launch_bounds__(256) k_col_mean(const float* __restrict__ x, int64_t ld,
                                                  int64_t col0, int64_t ncols, int32_t n,
                                                  float* __restrict__ xbar) {
    constexpr int V = sizeof(T) / sizeof(float);
    const int64_t col = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= ncols) return;
    const int64_t ldT = ld / V;
    const T* __restrict__ xp = reinterpret_cast<const T*>(x + col0) + col;
    typename AccOf<T>::type acc = AccOf<T>::zero();
    for (int base = 0; base < n; base += U) {
        T v[U];
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u < n) v[u] = ld_stream(xp + (int64_t)(base + u) * ldT);
#pragma unroll
        for (int u = 0; u < U; ++u)
            if (base + u < n) acc_add(acc, v[u]);
    }
    reinterpret_cast<T*>(xbar + col0)[col] = to_mean(acc, 1.0 / (double)n);
}

template <typename T>
__global__ void __launch_bounds__(256) k_consensus(const float* __restrict__ x, int64_t ld,
                                                   int64_t col0, int64_t ncols, int32_t n,
                                                   double* __restrict__ partials) {
    constexpr int V = sizeof(T) / sizeof(float);
    __shared__ double s_buf[4];
    const int64_t col = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    double ss = 0.0;
    if (col < ncols) {
        const int64_t ldT = ld / V;
        const T* __restrict__ xp = reinterpret_cast<const T*>(x + col0) + col;
        const T x0 = xp[0];
        typename AccOf<T>::type s1 = AccOf<T>::zero(), s2 = AccOf<T>::zero();
        for (int base = 1; base < n; base += U) {
            T v[U];
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u < n) v[u] = ld_stream(xp + (int64_t)(base + u) * ldT);
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (base + u < n) {
                    const T dlt = v[u] - x0;
                    acc_add(s1, dlt);
                    acc_sq(s2, dlt);
                }
        }
        ss = col_ss(s1, s2, 1.0 / (double)n);
    }
    ss = wave_sum(ss);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) s_buf[wave] = ss;
    __syncthreads();
    if (threadIdx.x == 0) partials[blockIdx.x] = (s_buf[0] + s_buf[1]) + (s_buf[2] + s_buf[3]);
}

// out[0] = sum of `count` partials, one workgroup, fixed order.
__global__ void __launch_bounds__(256) k_final_sum(const double* __restrict__ partials,
                                                   int64_t count, double* __restrict__ out) {
    __shared__ double s_buf[4];
    double acc = 0.0;
    for (int64_t t = threadIdx.x; t < count; t += blockDim.x) acc += partials[t];
    acc = wave_sum(acc);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) s_buf[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = (s_buf[0] + s_buf[1]) + (s_buf[2] + s_buf[3]);
}

// slot[0] = sqrt(sum of `count` partials), one workgroup, fixed order.
__global__ void __launch_bounds__(256) k_trace_store(const double* __restrict__ partials, int64_t count,
                                                     double* __restrict__ slot) {
    __shared__ double s_buf[4];
    double acc = 0.0;
    for (int64_t t = threadIdx.x; t < count; t += blockDim.x) acc += partials[t];
    acc = wave_sum(acc);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) s_buf[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) slot[0] = sqrt((s_buf[0] + s_buf[1]) + (s_buf[2] + s_buf[3]));
}

// out[0] = (1/count) sum v[i], one workgroup, fixed order.
__global__ void __launch_bounds__(256) k_mean_f32(const float* __restrict__ v, int64_t count,
                                                  double* __restrict__ out) {
    __shared__ double s_buf[4];
    double acc = 0.0;
    for (int64_t t = threadIdx.x; t < count; t += blockDim.x) acc += (double)v[t];
    acc = wave_sum(acc);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) s_buf[wave] = acc;
    __syncthreads();
    if (threadIdx.x == 0) out[0] = ((s_buf[0] + s_buf[1]) + (s_buf[2] + s_buf[3])) / (double)count;
}

template <typename T>
__global__ void __launch_bounds__(256) k_fill_rows(float* __restrict__ dst, int64_t ld,
                                                   int64_t col0, int64_t ncols, int32_t n,
                                                   const float* __restrict__ src) {
    constexpr int V = sizeof(T) / sizeof(float);
    const int64_t col = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (col >= ncols) return;
    const int64_t ldT = ld / V;
    const T v = src ? reinterpret_cast<const T*>(src + col0)[col] : T(0);
    T* __restrict__ dp = reinterpret_cast<T*>(dst + col0) + col;
    for (int row = 0; row < n; ++row) dp[(int64_t)row * ldT] = v;
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Plain streaming kernels used to measure what this chip's memory system delivers
// for reads, writes and copies (the context in which the fused step's rate is read).
// kind 0: read only (the sum keeps the loads alive), kind 1: write only, kind 2: copy
// src -> dst, kind 3: the fused step's arithmetic on flat arrays (read src, src2,
// inout; write inout, dst).  128-bit non-temporal accesses, consecutive lanes on
// consecutive 16-byte words; one word per lane, or grid-stride when the grid is capped.
template <int KIND>
__global__ void __launch_bounds__(256) k_probe_stream(const v4f* __restrict__ src, v4f* __restrict__ dst,
                                                      const v4f* __restrict__ src2, v4f* __restrict__ inout,
                                                      int64_t count, float* __restrict__ sink) {
    v4f acc = v4f(0);
    const int64_t stride = (int64_t)gridDim.x * blockDim.x;
#pragma unroll 4
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < count; t += stride) {
        if (KIND == 0) acc += ld_stream(src + t);
        if (KIND == 1) __builtin_nontemporal_store(v4f(1.0f), dst + t);
        if (KIND == 2) __builtin_nontemporal_store(ld_stream(src + t), dst + t);
        if (KIND == 3) {  // the fused step's mix without any row structure: 3 reads, 2 writes
            const v4f xv = ld_stream(src + t), mv = ld_stream(inout + t), gv = ld_stream(src2 + t);
            const v4f mom = 0.9f * mv + gv;
            __builtin_nontemporal_store(mom, inout + t);
            __builtin_nontemporal_store(xv - 0.1f * mom, dst + t);
        }
    }
    if (KIND == 0) {
        float v = acc.x + acc.y + acc.z + acc.w;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
        if ((threadIdx.x & (kWave - 1)) == 0 && v == 12345.678f) atomicAdd(sink, v);  // practically never taken
    }
}

}  // namespace

hipError_t launch_probe_stream(int kind, const float* src, float* dst, const float* src2, float* inout,
                               int64_t count16, float* sink, int64_t blocks, hipStream_t st) {
    const v4f* s = reinterpret_cast<const v4f*>(src);
    v4f* d = reinterpret_cast<v4f*>(dst);
    const v4f* s2 = reinterpret_cast<const v4f*>(src2);
    v4f* io = reinterpret_cast<v4f*>(inout);
    const dim3 grid((unsigned)blocks), block(256);
    if (kind == 0) hipLaunchKernelGGL((k_probe_stream<0>), grid, block, 0, st, s, d, s2, io, count16, sink);
    else if (kind == 1) hipLaunchKernelGGL((k_probe_stream<1>), grid, block, 0, st, s, d, s2, io, count16, sink);
    else if (kind == 2) hipLaunchKernelGGL((k_probe_stream<2>), grid, block, 0, st, s, d, s2, io, count16, sink);
    else hipLaunchKernelGGL((k_probe_stream<3>), grid, block, 0, st, s, d, s2, io, count16, sink);
    return hipGetLastError();
}

size_t consensus_partials_used(const gpga_ctx* c) {
    const bool vec = aligned16(c->x) && (c->ld % 4 == 0);
    const int64_t nv = vec ? c->d / 4 : 0;
    return (size_t)((nv + 255) / 256 + (c->d - nv * 4 + 255) / 256);
}

size_t consensus_partials_needed(const gpga_ctx* c) {
    // vector pass workgroups + scalar tail workgroup + 1 result slot
    return (size_t)((c->d / 4 + 255) / 256) + (size_t)((c->d + 255) / 256) + 2;
}

hipError_t launch_fill_rows(const gpga_ctx* c, float* dst, const float* src) {
    const bool vec = aligned16(dst) && (!src || aligned16(src)) && (c->ld % 4 == 0);
    const int64_t nv = vec ? c->d / 4 : 0;
    if (nv > 0) {
        hipLaunchKernelGGL((k_fill_rows<v4f>), dim3((unsigned)((nv + 255) / 256)), dim3(256), 0,
                           c->stream, dst, c->ld, (int64_t)0, nv, c->n, src);
    }
    const int64_t tail = c->d - nv * 4;
    if (tail > 0) {
        hipLaunchKernelGGL((k_fill_rows<float>), dim3((unsigned)((tail + 255) / 256)), dim3(256), 0,
                           c->stream, dst, c->ld, nv * 4, tail, c->n, src);
    }
    return hipGetLastError();
}

hipError_t launch_col_mean(const gpga_ctx* c, float* xbar) {
    const bool vec = aligned16(c->x) && aligned16(xbar) && (c->ld % 4 == 0);
    const int64_t nv = vec ? c->d / 4 : 0;
    if (nv > 0) {
        hipLaunchKernelGGL((k_col_mean<v4f>), dim3((unsigned)((nv + 255) / 256)), dim3(256), 0,
                           c->stream, c->x, c->ld, (int64_t)0, nv, c->n, xbar);
    }
    const int64_t tail = c->d - nv * 4;
    if (tail > 0) {
        hipLaunchKernelGGL((k_col_mean<float>), dim3((unsigned)((tail + 255) / 256)), dim3(256), 0,
                           c->stream, c->x, c->ld, nv * 4, tail, c->n, xbar);
    }
    return hipGetLastError();
}

// Per-workgroup partial sums of squared deviations of the live X into parts[0 ..] (room for
// `cap` doubles); *count receives their number.
static hipError_t launch_consensus_partials(const gpga_ctx* c, double* parts, size_t cap, int64_t* count) {
    *count = 0;
    const bool vec = aligned16(c->x) && (c->ld % 4 == 0);
    const int64_t nv = vec ? c->d / 4 : 0;
    const int64_t tail = c->d - nv * 4;
    const int64_t b1 = (nv + 255) / 256, b2 = (tail + 255) / 256;
    if ((size_t)(b1 + b2) > cap) return hipErrorOutOfMemory;
    if (b1 > 0) {
        hipLaunchKernelGGL((k_consensus<v4f>), dim3((unsigned)b1), dim3(256), 0, c->stream, c->x,
                           c->ld, (int64_t)0, nv, c->n, parts);
    }
    if (b2 > 0) {
        hipLaunchKernelGGL((k_consensus<float>), dim3((unsigned)b2), dim3(256), 0, c->stream, c->x,
                           c->ld, nv * 4, tail, c->n, parts + b1);
    }
    *count = b1 + b2;
    return hipGetLastError();
}

hipError_t launch_consensus_sq(gpga_ctx* c, size_t* partials_needed) {
    *partials_needed = consensus_partials_needed(c);
    int64_t count = 0;
    // slot 0 of the context's scratch holds the result of the synchronous entry point
    const hipError_t e = launch_consensus_partials(c, c->partials + 1, c->partials_cap - 1, &count);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(k_final_sum, dim3(1), dim3(256), 0, c->stream, c->partials + 1, count, c->partials);
    return hipGetLastError();
}

hipError_t launch_consensus_trace(gpga_ctx* c, double* slot) {
    return launch_consensus_distance(c, c->partials + 1, c->partials_cap - 1, slot);
}

hipError_t launch_consensus_distance(const gpga_ctx* c, double* scratch, size_t scratch_cap, double* slot) {
    int64_t count = 0;
    const hipError_t e = launch_consensus_partials(c, scratch, scratch_cap, &count);
    if (e != hipSuccess) return e;
    return launch_trace_store(c, scratch, count, slot);
}

hipError_t launch_trace_store(const gpga_ctx* c, const double* partials, int64_t count, double* slot) {
    hipLaunchKernelGGL(k_trace_store, dim3(1), dim3(256), 0, c->stream, partials, count, slot);
    return hipGetLastError();
}

hipError_t launch_mean_f32(const gpga_ctx* c, const float* v, int64_t count, double* out) {
    hipLaunchKernelGGL(k_mean_f32, dim3(1), dim3(256), 0, c->stream, v, count, out);
    return hipGetLastError();
}
