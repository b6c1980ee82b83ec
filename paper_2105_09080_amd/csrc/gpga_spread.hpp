// Shifted one-pass sums behind the consensus distance ||X - 1 xbar^T||_F (Sec. 4 / App. B):
// per column, s1 = sum_i (x_i - ref) and s2 = sum_i (x_i - ref)^2 in fp64 for a reference
// value ref near the column's values; sum_i (x_i - mean)^2 = s2 - s1^2 / n.
#pragma once

#include "gpga_internal.hpp"

template <typename T>
struct ColumnSpread;
template <>
struct ColumnSpread<v4f> {
    v4f ref;
    double s1[4], s2[4];
    __device__ __forceinline__ void reset(const v4f& r) {
        ref = r;
#pragma unroll
        for (int j = 0; j < 4; ++j) s1[j] = s2[j] = 0.0;
    }
    __device__ __forceinline__ void add(const v4f& v) {  // branch-free: it sits in the pipelined loop
        const v4f dl = v - ref;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double t = (double)dl[j];
            s1[j] += t;
            s2[j] += t * t;
        }
    }
    __device__ __forceinline__ double sum_sq(double inv_n) const {
        double r = 0.0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const double v = s2[j] - s1[j] * s1[j] * inv_n;
            r += v > 0.0 ? v : 0.0;
        }
        return r;
    }
};
template <>
struct ColumnSpread<v2f> {  // as for float below
    __device__ __forceinline__ void reset(v2f) {}
    __device__ __forceinline__ void add(v2f) {}
    __device__ __forceinline__ double sum_sq(double) const { return 0.0; }
};
template <>
struct ColumnSpread<float> {  // never instantiated with tracing on; keeps the template uniform
    __device__ __forceinline__ void reset(float) {}
    __device__ __forceinline__ void add(float) {}
    __device__ __forceinline__ double sum_sq(double) const { return 0.0; }
};

