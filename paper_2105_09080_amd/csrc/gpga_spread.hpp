// Shifted one-pass sums behind the consensus distance ||X - 1 xbar^T||_F (Sec. 4 / App. B):
// per column, s1 = sum_i (x_i - ref) and s2 = sum_i (x_i - ref)^2 in fp64 for a reference
// value ref near the column's values; sum_i (x_i - mean)^2 = s2 - s1^2 / n.
// One instance covers the 4, 2 or 1 columns of a lane (16-, 8- or 4-byte lanes).
#pragma once

#include "gpga_internal.hpp"

__device__ __forceinline__ float spread_elem(const v4f& v, int j) { return v[j]; }
__device__ __forceinline__ float spread_elem(const v2f& v, int j) { return v[j]; }
__device__ __forceinline__ float spread_elem(const float& v, int) { return v; }

template <typename T>
struct ColumnSpread {
    static constexpr int V = sizeof(T) / sizeof(float);
    T ref;
    double s1[V], s2[V];
    __device__ __forceinline__ void reset(const T& r) {
        ref = r;
#pragma unroll
        for (int j = 0; j < V; ++j) s1[j] = s2[j] = 0.0;
    }
    __device__ __forceinline__ void add(const T& v) {  // branch-free: it sits in the pipelined loops
        const T dl = v - ref;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const double t = (double)spread_elem(dl, j);
            s1[j] += t;
            s2[j] += t * t;
        }
    }
    __device__ __forceinline__ double sum_sq(double inv_n) const {
        double r = 0.0;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            const double v = s2[j] - s1[j] * s1[j] * inv_n;
            r += v > 0.0 ? v : 0.0;
        }
        return r;
    }
    // Sums of several wavefronts that used the SAME ref meet in LDS: this lane's 2V sums go to
    // dst[j * 64] (s1) and dst[(V + j) * 64] (s2) ...
    __device__ __forceinline__ void store(double* dst) const {
#pragma unroll
        for (int j = 0; j < V; ++j) {
            dst[(size_t)j * 64] = s1[j];
            dst[(size_t)(V + j) * 64] = s2[j];
        }
    }
    // ... and one lane adds the `waves` records (stride 2V * 64 doubles, in wavefront order) and
    // finishes its columns: sum over them of sum_i (x_i - mean)^2.
    static __device__ __forceinline__ double finish(const double* src, int waves, double inv_n) {
        double r = 0.0;
#pragma unroll
        for (int j = 0; j < V; ++j) {
            double a = 0.0, b = 0.0;
            for (int w = 0; w < waves; ++w) {
                a += src[((size_t)w * 2 * V + j) * 64];
                b += src[((size_t)w * 2 * V + V + j) * 64];
            }
            const double v = b - a * a * inv_n;
            r += v > 0.0 ? v : 0.0;
        }
        return r;
    }
};
