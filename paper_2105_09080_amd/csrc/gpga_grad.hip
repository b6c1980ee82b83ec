// Local stochastic gradients g_i = grad F_i(x_i; xi_i) for all n simulated nodes
// (Algorithm 1, line 1 of the loop).  Three families:
//
//  * synthetic    G[i][c] = sigma * N(seed, TAG_GRAD, i, k, c): a counter-addressed
//                 normal (Philox4x32-10 + Box-Muller) standing in for a network's
//                 backward pass.  Integer/ALU bound; one 128-bit store per lane.
//  * stored rows  least squares and logistic regression (Sec. 5.1 loss) on a
//                 materialised n x M x d array: a batched GEMV pair per node,
//                 (1) margins z_b = <row_b, x_i> -> per-sample coefficient,
//                 (2) g_i = sum_b coef_b * row_b.  Plain FMA, no matrix cores: each
//                 node has its own x_i, so there is no shared operand to tile.
//  * virtual rows logistic regression whose feature rows are regenerated from
//                 the counter RNG inside both passes (the array would not fit).
#include "gpga_internal.hpp"

namespace {

// ---------------------------------------------------------------- counter RNG

constexpr uint32_t kPhiloxM0 = 0xD2511F53u;
constexpr uint32_t kPhiloxM1 = 0xCD9E8D57u;
constexpr uint32_t kPhiloxW0 = 0x9E3779B9u;
constexpr uint32_t kPhiloxW1 = 0xBB67AE85u;

constexpr uint32_t TAG_GRAD = 1u;
constexpr uint32_t TAG_FEAT = 2u;
constexpr uint32_t TAG_MU = 3u;

struct u32x4 {
    uint32_t a, b, c, d;
};

// Philox4x32 with 10 rounds (Salmon et al., SC'11): two 32x32->64 multiplies per
// round, outputs permuted and xor-ed with the round key; key += Weyl constants.
__device__ __forceinline__ u32x4 philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                               uint32_t k0, uint32_t k1) {
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint64_t p0 = (uint64_t)kPhiloxM0 * c0, p1 = (uint64_t)kPhiloxM1 * c2;
        const uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        const uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        // three-input xor in one instruction (v_bitop3_b32, truth table 0x96 = a ^ b ^ c)
        const uint32_t n0 = __builtin_amdgcn_bitop3_b32(hi1, c1, k0, 0x96);
        const uint32_t n2 = __builtin_amdgcn_bitop3_b32(hi0, c3, k1, 0x96);
        c0 = n0;
        c1 = lo1;
        c2 = n2;
        c3 = lo0;
        k0 += kPhiloxW0;
        k1 += kPhiloxW1;
    }
    return {c0, c1, c2, c3};
}

// 32 random bits -> uniform in (0,1), exactly representable in fp32: u = ((r >> 9) + 0.5) * 2^-23.
// Built without an integer-to-float conversion: the 23 bits become the mantissa of a float in
// [1, 2) (one funnel shift puts the exponent 0x7F above them), and subtracting 1 - 2^-24 leaves
// (k + 0.5) * 2^-23 exactly (it has at most 24 significant bits, so the subtraction does not round).
__device__ __forceinline__ float uniform23(uint32_t r) {
    const uint32_t bits = __builtin_amdgcn_alignbit(0x7Fu, r, 9u);  // ({0x7F, r} >> 9) = 0x3F800000 | (r >> 9)
    return __uint_as_float(bits) - 0x1.fffffep-1f;
}

// Four standard normals for one column quad: Box-Muller on (u0,u1) and (u2,u3).
// The transcendental part uses the hardware units directly: v_log_f32 (log2),
// v_sqrt_f32, and v_sin_f32 / v_cos_f32, whose argument is in revolutions, so
// sin(2 pi u) is one instruction on u itself with no range reduction.  Measured
// over all 2^23 possible u: |sin|, |cos| error <= 1.3e-7, ln relative error
// <= 1.7e-7, radius error <= 4.9e-7 (radius <= 5.7).
__device__ __forceinline__ v4f normals4(uint32_t c4, uint32_t a, uint32_t b, uint32_t tag,
                                        uint32_t k0, uint32_t k1) {
    const u32x4 r = philox4x32_10(c4, a, b, tag, k0, k1);
    constexpr float kMinus2Ln2 = -1.3862943611198906f;  // -2 ln u = (-2 ln 2) log2 u
    const float ra = __builtin_amdgcn_sqrtf(kMinus2Ln2 * __builtin_amdgcn_logf(uniform23(r.a)));
    const float rb = __builtin_amdgcn_sqrtf(kMinus2Ln2 * __builtin_amdgcn_logf(uniform23(r.c)));
    const float ub = uniform23(r.b), ud = uniform23(r.d);
    v4f z;
    z.x = ra * __builtin_amdgcn_cosf(ub);
    z.y = ra * __builtin_amdgcn_sinf(ub);
    z.z = rb * __builtin_amdgcn_cosf(ud);
    z.w = rb * __builtin_amdgcn_sinf(ud);
    return z;
}

// ---------------------------------------------------------------- synthetic

__global__ void __launch_bounds__(256) k_synth_grad(float* __restrict__ g, int64_t ld, int64_t d,
                                                    uint32_t k0, uint32_t k1, uint32_t kiter,
                                                    float sigma, int vec_ok) {
    const int64_t c4 = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t c = c4 * 4;
    if (c >= d) return;
    const uint32_t i = blockIdx.y;
    const v4f z = sigma * normals4((uint32_t)c4, i, kiter, TAG_GRAD, k0, k1);
    float* row = g + (int64_t)i * ld;
    if (vec_ok && c + 3 < d) {
        __builtin_nontemporal_store(z, reinterpret_cast<v4f*>(row + c));
    } else {
        row[c] = z.x;
        if (c + 1 < d) row[c + 1] = z.y;
        if (c + 2 < d) row[c + 2] = z.z;
        if (c + 3 < d) row[c + 3] = z.w;
    }
}

// ---------------------------------------------------------------- reductions

__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;
}

// Sum over the workgroup; result valid in thread 0.
__device__ __forceinline__ double block_sum(double v, double* s_buf) {
    v = wave_sum(v);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x >> 6;
    if (lane == 0) s_buf[wave] = v;
    __syncthreads();
    double t = 0.0;
    if (threadIdx.x == 0)
        for (int w = 0; w < (int)(blockDim.x >> 6); ++w) t += s_buf[w];
    return t;
}

// Lane-shift reductions on the data-parallel-primitive path of the vector ALU (no LDS
// round trips): a 64-bit value moved as two 32-bit halves from the lane CTRL selects.
template <int CTRL>
__device__ __forceinline__ double dpp_f64(double v) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(u & 0xffffffffull), CTRL, 0xf, 0xf, true);
    const unsigned hi = (unsigned)__builtin_amdgcn_update_dpp(0, (int)(unsigned)(u >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
__device__ __forceinline__ double readlane_f64(double v, int src_lane) {
    const unsigned long long u = (unsigned long long)__double_as_longlong(v);
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u & 0xffffffffull), src_lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(u >> 32), src_lane);
    return __longlong_as_double((long long)(((unsigned long long)hi << 32) | lo));
}
// Sum over each aligned row of 16 lanes (shifts by 1, 2, 4, 8 within the row; a lane without
// a source adds 0); complete in the row's last lane.  Every lane of the wavefront must be active.
__device__ __forceinline__ double row16_sum_last(double v) {
    v += dpp_f64<0x111>(v);  // row_shr:1
    v += dpp_f64<0x112>(v);  // row_shr:2
    v += dpp_f64<0x114>(v);  // row_shr:4
    v += dpp_f64<0x118>(v);  // row_shr:8
    return v;
}
// Sum over each aligned group of G lanes, G = 16, 32 or 64 (uniform); complete in the group's
// last lane.  Every lane of the wavefront must be active.
__device__ __forceinline__ double group_sum_last(double v, int G) {
    v = row16_sum_last(v);
    if (G == 16) return v;
    const double r0 = readlane_f64(v, 15), r1 = readlane_f64(v, 31), r2 = readlane_f64(v, 47), r3 = readlane_f64(v, 63);
    if (G == 32) return (threadIdx.x & 32) ? r2 + r3 : r0 + r1;
    return (r0 + r1) + (r2 + r3);
}

// Per-sample coefficient and loss term from the margin z.
//   least squares: r = z - b          coef = r / B           loss = r^2 / (2B)
//   logistic     : t = y z            coef = -y s(-t) / B    loss = ln(1 + e^{-t}) / B
template <int KIND>
__device__ __forceinline__ void sample_terms(double z, float target, float invB, float* coef,
                                             float* loss) {
    if (KIND == PROB_LSQ) {
        const double r = z - (double)target;
        *coef = (float)(r * invB);
        *loss = (float)(0.5 * r * r * invB);
    } else {
        const double t = (double)target * z;
        const double e = exp(-fabs(t));               // in (0,1], never overflows
        const double sig = (t >= 0.0) ? e / (1.0 + e) : 1.0 / (1.0 + e);   // sigma(-t)
        *coef = (float)(-(double)target * sig * invB);
        *loss = (float)((fmax(-t, 0.0) + log1p(e)) * invB);
    }
}

// ---------------------------------------------------------------- stored rows

// Pass 1: one workgroup per (sample slot b, node i): z = <row, x_i> in fp64.
template <int KIND>
__global__ void __launch_bounds__(256) k_rows_margin(const float* __restrict__ feat,
                                                     const float* __restrict__ tgt,
                                                     const float* __restrict__ x, int64_t ld,
                                                     const int32_t* __restrict__ idx, int32_t B,
                                                     int32_t M, int64_t d, int vec_ok,
                                                     float* __restrict__ coef,
                                                     float* __restrict__ lossterm) {
    __shared__ double s_buf[4];
    const int b = blockIdx.x, i = blockIdx.y;
    const int32_t r = idx ? idx[(int64_t)i * B + b] : b;
    if (r < 0 || r >= M) {  // a sample index outside [0, M): no access, the node's gradient and loss become NaN
        if (threadIdx.x == 0) {
            coef[(int64_t)i * B + b] = __builtin_nanf("");
            lossterm[(int64_t)i * B + b] = __builtin_nanf("");
        }
        return;
    }
    const float* __restrict__ f = feat + ((int64_t)i * M + r) * d;
    const float* __restrict__ xi = x + (int64_t)i * ld;
    const float target = tgt[(int64_t)i * M + r];  // fetched with the row, not after the reduction
    double acc = 0.0;
    if (vec_ok) {
        const int64_t d4 = d >> 2;
        const v4f* f4 = reinterpret_cast<const v4f*>(f);
        const v4f* x4 = reinterpret_cast<const v4f*>(xi);
#pragma unroll 4
        for (int64_t c = threadIdx.x; c < d4; c += blockDim.x) {
            const v4f fv = f4[c], xv = x4[c];
            acc += (double)fv.x * xv.x + (double)fv.y * xv.y + (double)fv.z * xv.z +
                   (double)fv.w * xv.w;
        }
    } else {
        for (int64_t c = threadIdx.x; c < d; c += blockDim.x) acc += (double)f[c] * xi[c];
    }
    const double z = block_sum(acc, s_buf);
    if (threadIdx.x == 0) {
        float cf, ls;
        sample_terms<KIND>(z, target, 1.0f / (float)B, &cf, &ls);
        coef[(int64_t)i * B + b] = cf;
        lossterm[(int64_t)i * B + b] = ls;
    }
}

// Pass 1 for short rows (d <= 32): one thread per (node, sample slot); neighbouring threads
// read neighbouring rows, so a full-batch evaluation over many samples streams the
// feature array instead of spending a workgroup on every ten-element dot product.
template <int KIND>
__global__ void __launch_bounds__(256) k_rows_margin_short(const float* __restrict__ feat,
                                                           const float* __restrict__ tgt,
                                                           const float* __restrict__ x, int64_t ld,
                                                           const int32_t* __restrict__ idx, int32_t B,
                                                           int32_t M, int32_t d, int64_t pairs,
                                                           float* __restrict__ coef,
                                                           float* __restrict__ lossterm) {
    const int64_t p = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;  // i * B + b
    if (p >= pairs) return;
    const int64_t i = p / B;
    const int32_t r = idx ? idx[p] : (int32_t)(p - i * B);
    float cf = __builtin_nanf(""), ls = __builtin_nanf("");  // index outside [0, M): no access, NaN
    if (r >= 0 && r < M) {
        const float* __restrict__ f = feat + (i * M + r) * d;
        const float* __restrict__ xi = x + i * ld;
        double acc = 0.0;
        for (int c = 0; c < d; ++c) acc += (double)f[c] * xi[c];
        sample_terms<KIND>(acc, tgt[i * M + r], 1.0f / (float)B, &cf, &ls);
    }
    coef[p] = cf;
    lossterm[p] = ls;
}

// Pass 2: g = sum_b coef_b * row_b[c] for node i.  A workgroup of W wavefronts owns 64 column quads;
// the wavefronts share the samples (b = wave, wave + W, ...) and their fp64 partial sums meet in LDS in
// wavefront order, so a minibatch of 32 rows is four chains of eight dependent loads instead of one of 32
// and a small problem still fills the chip (cfg2: 1280 -> 5120 wavefronts, 15 -> 9 us).  W = 4
// wavefronts per workgroup, 16 for minibatches of 64 rows and more.
template <int W>
__global__ void __launch_bounds__(kWave* W) k_rows_accum(const float* __restrict__ feat,
                                                    const float* __restrict__ coef,
                                                    const int32_t* __restrict__ idx, int32_t B,
                                                    int32_t M, int64_t d, int vec_ok,
                                                    float* __restrict__ g, int64_t ld) {
    __shared__ double s_part[W - 1][4][kWave];
    const int i = blockIdx.y;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const float* __restrict__ fi = feat + (int64_t)i * M * d;
    const float* __restrict__ ci = coef + (int64_t)i * B;
    const int32_t* __restrict__ ii = idx ? idx + (int64_t)i * B : nullptr;
    float* __restrict__ gi = g + (int64_t)i * ld;
    const int64_t t = (int64_t)blockIdx.x * kWave + lane;          // column quad (vector path) or column
    const bool on = vec_ok ? t * 4 < d : t < d;
    double a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (on) {
        for (int b = wave; b < B; b += W) {
            int32_t r = ii ? ii[b] : b;
            if (r < 0 || r >= M) r = 0;  // its coefficient is NaN (set by the margin pass): row 0 is only a safe address
            const double cb = ci[b];
            if (vec_ok) {
                const v4f fv = reinterpret_cast<const v4f*>(fi + (int64_t)r * d)[t];
                a0 += cb * fv.x;
                a1 += cb * fv.y;
                a2 += cb * fv.z;
                a3 += cb * fv.w;
            } else {
                a0 += cb * fi[(int64_t)r * d + t];
            }
        }
    }
    if (wave > 0) {
        s_part[wave - 1][0][lane] = a0;
        s_part[wave - 1][1][lane] = a1;
        s_part[wave - 1][2][lane] = a2;
        s_part[wave - 1][3][lane] = a3;
    }
    __syncthreads();
    if (wave == 0 && on) {
#pragma unroll
        for (int w = 0; w < W - 1; ++w) {
            a0 += s_part[w][0][lane];
            a1 += s_part[w][1][lane];
            a2 += s_part[w][2][lane];
            a3 += s_part[w][3][lane];
        }
        if (vec_ok) {
            v4f out;
            out.x = (float)a0;
            out.y = (float)a1;
            out.z = (float)a2;
            out.w = (float)a3;
            __builtin_nontemporal_store(out, reinterpret_cast<v4f*>(gi) + t);
        } else {
            gi[t] = (float)a0;
        }
    }
}

// loss[i] = sum_b lossterm[i][b]  (terms already carry the 1/B)
__global__ void __launch_bounds__(256) k_loss_sum(const float* __restrict__ lossterm, int32_t B,
                                                  float* __restrict__ loss) {
    __shared__ double s_buf[4];
    const int i = blockIdx.x;
    double acc = 0.0;
    for (int b = threadIdx.x; b < B; b += blockDim.x) acc += lossterm[(int64_t)i * B + b];
    const double t = block_sum(acc, s_buf);
    if (threadIdx.x == 0) loss[i] = (float)t;
}

// ---------------------------------------------------------------- virtual rows

// Feature quad h_{i,m}[4c4 .. 4c4+3] = mu_i + zeta_{i,m}, rounded to fp32 like a
// stored feature would be.
__device__ __forceinline__ v4f virtual_quad(v4f mu, uint32_t c4, uint32_t i, uint32_t m,
                                            uint32_t k0, uint32_t k1) {
    return mu + normals4(c4, i, m, TAG_FEAT, k0, k1);
}

// Pass 1: grid (column chunks, node).  Each lane owns column quads and keeps B
// partial margins; the node shift mu_i is generated once per quad and reused for
// all B samples.  Partial margins are combined per workgroup and stored as
// zpart[i][b][chunk]; the coefficient kernel adds the chunks in a fixed order, so the
// result does not depend on the order in which workgroups finish.
template <int BMAX>
__global__ void __launch_bounds__(256) k_virtual_margin(const float* __restrict__ x, int64_t ld,
                                                        int64_t d, const int32_t* __restrict__ idx,
                                                        int32_t B, uint32_t k0, uint32_t k1,
                                                        float mu_sigma, int64_t quads_per_block,
                                                        double* __restrict__ zpart) {
    __shared__ double s_buf[4];
    const uint32_t i = blockIdx.y;
    const int64_t d4 = (d + 3) >> 2;
    const int64_t q_begin = (int64_t)blockIdx.x * quads_per_block;
    const int64_t q_end = (q_begin + quads_per_block < d4) ? q_begin + quads_per_block : d4;
    const float* __restrict__ xi = x + (int64_t)i * ld;
    double acc[BMAX];
#pragma unroll
    for (int b = 0; b < BMAX; ++b) acc[b] = 0.0;
    for (int64_t q = q_begin + threadIdx.x; q < q_end; q += blockDim.x) {
        const int64_t c = q * 4;
        v4f xv;
        xv.x = xi[c];
        xv.y = (c + 1 < d) ? xi[c + 1] : 0.f;
        xv.z = (c + 2 < d) ? xi[c + 2] : 0.f;
        xv.w = (c + 3 < d) ? xi[c + 3] : 0.f;
        const v4f mu = mu_sigma * normals4((uint32_t)q, i, 0u, TAG_MU, k0, k1);
#pragma unroll
        for (int b = 0; b < BMAX; ++b) {
            if (b < B) {
                const v4f h = virtual_quad(mu, (uint32_t)q, i, (uint32_t)idx[(int64_t)i * B + b], k0, k1);
                // the four products of a quad are summed in fp32 (three roundings of ~6e-8 relative to
                // the quad's own terms, random in sign over the d/4 quads of a margin), the quads in fp64:
                // 6 issue slots per sample where four conversions and four fp64 operations took 12
                const float t = h.x * xv.x + h.y * xv.y + h.z * xv.z + h.w * xv.w;
                acc[b] += (double)t;
            }
        }
    }
#pragma unroll
    for (int b = 0; b < BMAX; ++b) {
        if (b < B) {
            const double t = block_sum(acc[b], s_buf);
            if (threadIdx.x == 0) zpart[((int64_t)i * B + b) * gridDim.x + blockIdx.x] = t;
            __syncthreads();
        }
    }
}

__global__ void k_virtual_coef(const double* __restrict__ zpart, int32_t chunks, const float* __restrict__ y,
                               const int32_t* __restrict__ idx, int32_t B, int32_t M, int32_t n,
                               float* __restrict__ coef, float* __restrict__ lossterm) {
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= (int64_t)n * B) return;
    double z = 0.0;
    for (int32_t ch = 0; ch < chunks; ++ch) z += zpart[t * chunks + ch];
    const int i = (int)(t / B);
    float cf, ls;
    const int32_t r = idx[t];
    if (r < 0 || r >= M) {  // label index outside [0, M): no access, NaN marks the node's gradient and loss
        coef[t] = __builtin_nanf("");
        lossterm[t] = __builtin_nanf("");
        return;
    }
    sample_terms<PROB_LOGREG>(z, y[(int64_t)i * M + r], 1.0f / (float)B, &cf, &ls);
    coef[t] = cf;
    lossterm[t] = ls;
}

// Pass 2: one lane per column quad of node i, features regenerated.
template <int BMAX>
__global__ void __launch_bounds__(256) k_virtual_accum(const float* __restrict__ coef,
                                                       const int32_t* __restrict__ idx, int32_t B,
                                                       int64_t d, uint32_t k0, uint32_t k1,
                                                       float mu_sigma, int vec_ok,
                                                       float* __restrict__ g, int64_t ld) {
    const uint32_t i = blockIdx.y;
    const int64_t q = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t c = q * 4;
    if (c >= d) return;
    const v4f mu = mu_sigma * normals4((uint32_t)q, i, 0u, TAG_MU, k0, k1);
    // g = sum_b coef_b h_b over at most 32 samples of similar size: fp32 fused multiply-adds (error
    // <= 32 x 6e-8 of sum |coef_b h_b|, far inside 1e-5 of the row's scale).  A sample whose
    // coefficient is exactly zero adds exactly nothing and its features are not regenerated:
    // once the margins of a logistic problem are large, sigma(-y z) underflows to 0 for every
    // correctly classified sample.  (NaN coefficients, which mark invalid sample indices, are
    // not zero and poison the row as before.)  The coefficient is the same for the whole
    // workgroup, so the test is a scalar branch.
    v4f a = v4f(0.f);
#pragma unroll
    for (int b = 0; b < BMAX; ++b) {
        if (b < B) {
            const float cb = coef[(int64_t)i * B + b];
            if (cb != 0.f) {
                const v4f h = virtual_quad(mu, (uint32_t)q, i, (uint32_t)idx[(int64_t)i * B + b], k0, k1);
                a += cb * h;
            }
        }
    }
    const float a0 = a.x, a1 = a.y, a2 = a.z, a3 = a.w;
    float* row = g + (int64_t)i * ld;
    if (vec_ok && c + 3 < d) {
        v4f out;
        out.x = (float)a0;
        out.y = (float)a1;
        out.z = (float)a2;
        out.w = (float)a3;
        // streamed past the caches: the fused step that follows reads g once, and dirty lines left behind
        // here would be written back while that step is already being timed against its pacing clock
        __builtin_nontemporal_store(out, reinterpret_cast<v4f*>(row + c));
    } else {
        row[c] = (float)a0;
        if (c + 1 < d) row[c + 1] = (float)a1;
        if (c + 2 < d) row[c + 2] = (float)a2;
        if (c + 3 < d) row[c + 3] = (float)a3;
    }
}

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }


// ---------------------------------------------------------------- small problems: whole iterations in one workgroup

// When the n x d state and one minibatch of work fit in a single workgroup, T whole
// iterations of Algorithm 1 - stochastic gradients at the current rows, momentum and local
// update, gossip step or global average, and the consensus distance - run inside ONE launch
// with X, M and x^(k+1/2) held in LDS.  Such problems (the logistic simulation of Sec. 5.1:
// n <= 100 nodes, d = 10) are otherwise bound by the latency of three to five dependent
// kernel launches per iteration; here an iteration costs a few workgroup barriers and one
// dependent pair of global reads (sample index, then feature row).
// The arithmetic follows the large kernels: margins and gradient sums accumulate in fp64,
// state and x^(k+1/2) are fp32, the mean of a global average is one value broadcast to
// all rows.
struct SmallArgs {
    const float* x;  // n x ld, the iterates before the first iteration of this launch
    float* x_out;    // n x ld, receives the iterates after the last one (may be the same array)
    float* m;  // n x ld momentum buffers (unused when mu = 0)
    float* g;  // n x ld, receives the gradients of the last iteration
    int64_t ld;
    int32_t n, d;
    const float* feat;  // n x M x d
    const float* tgt;   // n x M
    int32_t M;
    const int32_t* idx;  // T x n x B sample indices, or NULL = every node's whole data set (B = M)
    int32_t B;
    int32_t topo;
    int64_t H, k0;
    int32_t T;
    float mu;
    const int32_t* wptr;  // W in compressed-row form for the sparse-W topologies
    const int32_t* wcol;
    const float* wval;
    double* trace;  // trace[k] = consensus distance after iteration k, for k < trace_cap
    int64_t trace_cap;
    float lr[kSmallRunMaxIters];  // step size of each iteration of this launch
};

template <int KIND, int MOM>
__global__ void __launch_bounds__(kSmallRunThreads) k_small_run(const SmallArgs a) {
    extern __shared__ __align__(16) unsigned char s_raw[];
    const int n = a.n, d = a.d, nd = n * d, B = a.B;
    double* __restrict__ sMean = reinterpret_cast<double*>(s_raw);  // d column means
    double* __restrict__ sRed = sMean + d;                          // two sets of one slot per wavefront
    double* __restrict__ sZ = sRed + 2 * (kSmallRunThreads / kWave);  // n x B margins
    float* __restrict__ sX = reinterpret_cast<float*>(sZ + n * a.B);
    float* __restrict__ sY = sX + nd;
    float* __restrict__ sM = sY + nd;               // MOM only
    float* __restrict__ sC = sM + (MOM ? nd : 0);   // n x B per-sample coefficients
    int32_t* __restrict__ sIdx = reinterpret_cast<int32_t*>(sC + n * B);  // n x B sample rows of the iteration
    const int G = d <= 16 ? 16 : d <= 32 ? 32 : kWave;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid >> 6, nw = blockDim.x >> 6;
    const float invB = 1.0f / (float)B;
    const float third = 1.0f / 3.0f;
    const double inv_n = 1.0 / (double)n;
    int tau = 0;
    while ((1LL << tau) < n) ++tau;
    if (tau < 1) tau = 1;

    for (int e = tid; e < nd; e += blockDim.x) {
        const int i = e / d, c = e - i * d;
        sX[e] = a.x[(int64_t)i * a.ld + c];
        if (MOM) sM[e] = a.m[(int64_t)i * a.ld + c];
    }
    __syncthreads();

    // column means of src (n x d in LDS) into sMean: one wavefront per column, lanes over rows
    auto column_means = [&](const float* src) {
        for (int c = wave; c < d; c += nw) {
            double s = 0.0;
            for (int i = lane; i < n; i += kWave) s += (double)src[i * d + c];
            s = group_sum_last(s, kWave);
            if (lane == 0) sMean[c] = s * inv_n;
        }
        __syncthreads();
    };

    // Short rows (d <= G) whose pairs fit a few passes are software-pipelined across iterations:
    // lane lg of group tid / G keeps, for pair p = tid / G + j * PP, the sample row, the label and
    // feature value number lg of the NEXT iteration in registers.
    const int npairs = n * B, PP = blockDim.x / G, lg = tid & (G - 1);
    const bool piped = d <= G && npairs <= kSmallRunPasses * PP;
    auto fetch_row = [&](int tt, int j) -> int32_t {  // validated sample row of pair j in iteration tt, or -1
        const int p = tid / G + j * PP;
        if (tt >= a.T || p >= npairs) return -1;
        const int32_t r = a.idx ? a.idx[(int64_t)tt * npairs + p] : p % B;
        return (r >= 0 && r < a.M) ? r : -1;
    };
    auto fetch_sample = [&](int j, int32_t r, float& f, float& y) {
        f = 0.f;
        y = 0.f;
        if (r >= 0) {
            const int i = (tid / G + j * PP) / B;
            if (lg < d) f = a.feat[((int64_t)i * a.M + r) * d + lg];
            y = a.tgt[(int64_t)i * a.M + r];
        }
    };
    // The coefficient of a sample needs a double-precision exponential: with one pass of lane
    // groups the group's last lane computes it on the spot; with several passes the margins
    // go to LDS first and one thread per pair computes them all at once.
    const bool one_pass = npairs <= PP;
    auto coefficient = [&](double z, float y, int32_t r) -> float {
        float cf = __builtin_nanf(""), ls;  // no valid sample: the node's gradient becomes NaN
        if (r >= 0) sample_terms<KIND>(z, y, invB, &cf, &ls);
        return cf;
    };
    auto coefficients_from_margins = [&]() {
        for (int p = tid; p < npairs; p += blockDim.x) sC[p] = coefficient(sZ[p], sC[p], sIdx[p]);
        __syncthreads();
    };
    int32_t rcur[kSmallRunPasses], rnext[kSmallRunPasses];
    float fcur[kSmallRunPasses], ycur[kSmallRunPasses];
    if (piped) {
#pragma unroll
        for (int j = 0; j < kSmallRunPasses; ++j) {
            rcur[j] = rnext[j] = -1;
            fcur[j] = ycur[j] = 0.f;
            if (j * PP >= npairs) continue;
            rcur[j] = fetch_row(0, j);
            fetch_sample(j, rcur[j], fcur[j], ycur[j]);
            rnext[j] = fetch_row(1, j);
        }
    }

    for (int t = 0; t < a.T; ++t) {
        const int64_t k = a.k0 + t;
        const float lr = a.lr[t];
        const int32_t* __restrict__ idx_t = a.idx ? a.idx + (int64_t)t * npairs : nullptr;

        if (piped) {
            // The rows, labels and feature values of this iteration were fetched during the one
            // before (they do not depend on x); only the products with the current x are left.
#pragma unroll
            for (int j = 0; j < kSmallRunPasses; ++j) {
                if (j * PP >= npairs) break;  // uniform: no pair left for this pass
                const int p = tid / G + j * PP;
                const bool have = p < npairs;
                const int i = have ? p / B : 0;
                double acc = (have && rcur[j] >= 0 && lg < d) ? (double)fcur[j] * sX[i * d + lg] : 0.0;
                acc = group_sum_last(acc, G);
                if (have && lg == G - 1) {
                    sIdx[p] = rcur[j];
                    if (one_pass) {
                        sC[p] = coefficient(acc, ycur[j], rcur[j]);
                    } else {  // margin and label now, the coefficient from one thread per pair below
                        sZ[p] = acc;
                        sC[p] = ycur[j];
                    }
                }
            }
            // fetch for the next iteration and the sample rows of the one after it
#pragma unroll
            for (int j = 0; j < kSmallRunPasses; ++j) {
                if (j * PP >= npairs) break;
                rcur[j] = rnext[j];
                fetch_sample(j, rcur[j], fcur[j], ycur[j]);
                rnext[j] = fetch_row(t + 2, j);
            }
            __syncthreads();
            if (!one_pass) coefficients_from_margins();
        } else {
            // sample rows of this iteration into LDS (-1 = index outside [0, M))
            for (int p = tid; p < npairs; p += blockDim.x) {
                const int32_t r = idx_t ? idx_t[p] : p % B;
                sIdx[p] = (r >= 0 && r < a.M) ? r : -1;
            }
            __syncthreads();

            // per-sample coefficients from the margins <h, x_i>: a group of G lanes per (node,
            // sample slot), G the power of two that covers d (16..64)
            for (int p0 = 0; p0 < npairs; p0 += PP) {
                const int p = p0 + tid / G;
                const bool have = p < npairs;
                const int i = have ? p / B : 0;
                const int32_t r = have ? sIdx[p] : -1;
                double acc = 0.0;
                if (r >= 0) {
                    const float* __restrict__ f = a.feat + ((int64_t)i * a.M + r) * d;
                    int c = lg;
                    for (; c + 3 * G < d; c += 4 * G) {  // four loads in flight
                        const float f0 = f[c], f1 = f[c + G], f2 = f[c + 2 * G], f3 = f[c + 3 * G];
                        acc += (double)f0 * sX[i * d + c] + (double)f1 * sX[i * d + c + G] +
                               (double)f2 * sX[i * d + c + 2 * G] + (double)f3 * sX[i * d + c + 3 * G];
                    }
                    for (; c < d; c += G) acc += (double)f[c] * sX[i * d + c];
                }
                acc = group_sum_last(acc, G);
                if (have && lg == G - 1) {
                    const float y = r >= 0 ? a.tgt[(int64_t)i * a.M + r] : 0.f;
                    if (one_pass) {
                        sC[p] = coefficient(acc, y, r);
                    } else {
                        sZ[p] = acc;
                        sC[p] = y;
                    }
                }
            }
            __syncthreads();
            if (!one_pass) coefficients_from_margins();
        }

        // gradient, momentum and local update, one element per thread and pass
        for (int e = tid; e < nd; e += blockDim.x) {
            const int i = e / d, c = e - i * d;
            double acc = 0.0;
            for (int b = 0; b < B; ++b) {
                int32_t r = sIdx[i * B + b];
                if (r < 0) r = 0;  // its coefficient is NaN: row 0 is only a safe address
                acc += (double)sC[i * B + b] * a.feat[((int64_t)i * a.M + r) * d + c];
            }
            const float gv = (float)acc;
            float mom = gv;
            if (MOM) {
                mom = a.mu * sM[e] + gv;
                sM[e] = mom;
            }
            sY[e] = MOM == 2 ? sX[e] - lr * (gv + a.mu * mom) : sX[e] - lr * mom;
            if (t == a.T - 1) a.g[(int64_t)i * a.ld + c] = gv;
        }
        __syncthreads();

        // gossip step or global average (Algorithm 1: the mean iff mod(k+1, H) = 0)
        const bool global = a.topo == GPGA_TOPO_FULL || (a.H > 0 && (k + 1) % a.H == 0);
        if (n > 1 && global) column_means(sY);
        const int S = (int)((1LL << (int)(k % tau)) % n);  // one-peer offset of this iteration
        for (int e = tid; e < nd; e += blockDim.x) {
            const int i = e / d, c = e - i * d;
            float v = sY[e];
            if (n > 1) {
                if (global) {
                    v = (float)sMean[c];
                } else if (a.topo == GPGA_TOPO_RING) {
                    const int im = i == 0 ? n - 1 : i - 1, ip = i == n - 1 ? 0 : i + 1;
                    v = (sY[im * d + c] + v + sY[ip * d + c]) * third;
                } else if (a.topo == GPGA_TOPO_EXPO1) {
                    if (S) v = (v + sY[((i + S) % n) * d + c]) * 0.5f;
                } else if (a.topo != GPGA_TOPO_NONE) {
                    float acc = 0.f;
                    for (int p = a.wptr[i]; p < a.wptr[i + 1]; ++p) acc += a.wval[p] * sY[a.wcol[p] * d + c];
                    v = acc;
                }
            }
            sX[e] = v;
        }
        __syncthreads();

        // consensus distance ||X - 1 xbar^T||_F of the new iterates (exactly 0 after an average):
        // a wavefront takes whole columns, lanes over the rows, so the column mean and the
        // squared deviations from it need no exchange with other wavefronts
        if (a.trace && k < a.trace_cap) {
            double part = 0.0;
            if (n > 1 && !global) {
                for (int c = wave; c < d; c += nw) {
                    double s1 = 0.0;
                    for (int i = lane; i < n; i += kWave) s1 += (double)sX[i * d + c];
                    const double mean = group_sum_last(s1, kWave) * inv_n;
                    for (int i = lane; i < n; i += kWave) {
                        const double dv = (double)sX[i * d + c] - mean;
                        part += dv * dv;
                    }
                }
            }
            part = group_sum_last(part, kWave);
            double* __restrict__ slots = sRed + (t & 1) * (kSmallRunThreads / kWave);  // the other half next time
            if (lane == 0) slots[wave] = part;
            __syncthreads();
            if (tid == 0) {
                double tot = 0.0;
                for (int w = 0; w < nw; ++w) tot += slots[w];
                a.trace[k] = sqrt(tot);
            }
        }
    }

    for (int e = tid; e < nd; e += blockDim.x) {
        const int i = e / d, c = e - i * d;
        a.x_out[(int64_t)i * a.ld + c] = sX[e];
        if (MOM) a.m[(int64_t)i * a.ld + c] = sM[e];
    }
}

size_t small_run_lds(const gpga_ctx* c, int32_t Beff) {
    const size_t nd = (size_t)c->n * (size_t)c->d;
    return ((size_t)c->d + 2 * (kSmallRunThreads / kWave) + (size_t)c->n * (size_t)Beff) * sizeof(double) +
           ((c->mu != 0.f ? 3 : 2) * nd + 2 * (size_t)c->n * (size_t)Beff) * sizeof(float);
}

}  // namespace

hipError_t launch_synth_grad(const gpga_ctx* c) {
    const int64_t d4 = (c->d + 3) / 4;
    dim3 grid((unsigned)((d4 + 255) / 256), (unsigned)c->n), block(256);
    const int vec_ok = aligned16(c->g) && (c->ld % 4 == 0);
    hipLaunchKernelGGL(k_synth_grad, grid, block, 0, c->stream, c->g, c->ld, c->d,
                       (uint32_t)(c->seed & 0xffffffffu), (uint32_t)(c->seed >> 32),
                       (uint32_t)(c->k & 0xffffffff), c->grad_sigma, vec_ok);
    return hipGetLastError();
}

hipError_t launch_rows_grad(const gpga_ctx* c, const int32_t* idx, int32_t B, float* loss_out) {
    const int32_t Beff = idx ? B : c->M;
    float* coef = c->coef;
    float* lossterm = c->coef + (size_t)c->n * Beff;
    const int vec_feat = aligned16(c->feat) && (c->d % 4 == 0);
    const int vec_x = vec_feat && aligned16(c->x) && (c->ld % 4 == 0);
    dim3 grid1((unsigned)Beff, (unsigned)c->n), block(256);
    const int64_t pairs = (int64_t)c->n * Beff;
    if (c->d <= 32 && (pairs + 255) / 256 <= 0x7fffffffLL) {
        const dim3 grid_short((unsigned)((pairs + 255) / 256));
        if (c->problem == PROB_LSQ) {
            hipLaunchKernelGGL((k_rows_margin_short<PROB_LSQ>), grid_short, block, 0, c->stream, c->feat, c->tgt,
                               c->x, c->ld, idx, Beff, c->M, (int32_t)c->d, pairs, coef, lossterm);
        } else {
            hipLaunchKernelGGL((k_rows_margin_short<PROB_LOGREG>), grid_short, block, 0, c->stream, c->feat, c->tgt,
                               c->x, c->ld, idx, Beff, c->M, (int32_t)c->d, pairs, coef, lossterm);
        }
    } else if (c->problem == PROB_LSQ) {
        hipLaunchKernelGGL((k_rows_margin<PROB_LSQ>), grid1, block, 0, c->stream, c->feat, c->tgt,
                           c->x, c->ld, idx, Beff, c->M, c->d, vec_x, coef, lossterm);
    } else {
        hipLaunchKernelGGL((k_rows_margin<PROB_LOGREG>), grid1, block, 0, c->stream, c->feat,
                           c->tgt, c->x, c->ld, idx, Beff, c->M, c->d, vec_x, coef, lossterm);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (loss_out) {
        hipLaunchKernelGGL(k_loss_sum, dim3((unsigned)c->n), block, 0, c->stream, lossterm, Beff,
                           loss_out);
        return hipGetLastError();
    }
    const int vec_g = vec_feat && aligned16(c->g) && (c->ld % 4 == 0);
    const int64_t cols = vec_g ? c->d / 4 : c->d;
    dim3 grid2((unsigned)((cols + kWave - 1) / kWave), (unsigned)c->n);
    if (Beff >= 64) {
        hipLaunchKernelGGL(k_rows_accum<16>, grid2, dim3(kWave * 16), 0, c->stream, c->feat, coef, idx, Beff, c->M,
                           c->d, vec_g, c->g, c->ld);
    } else {
        hipLaunchKernelGGL(k_rows_accum<4>, grid2, block, 0, c->stream, c->feat, coef, idx, Beff, c->M,
                           c->d, vec_g, c->g, c->ld);
    }
    return hipGetLastError();
}

// Column chunks per node of the margin pass: enough workgroups per node to fill the chip, at least
// 256 quads each, every chunk non-empty.
int64_t virtual_margin_chunks(const gpga_ctx* c) {
    const int64_t d4 = (c->d + 3) / 4;
    int64_t chunks = (4096 + c->n - 1) / c->n;
    const int64_t max_chunks = (d4 + 255) / 256;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    const int64_t qpb = (d4 + chunks - 1) / chunks;
    return (d4 + qpb - 1) / qpb;
}

hipError_t launch_virtual_grad(const gpga_ctx* c, const int32_t* idx, int32_t B, float* loss_out) {
    constexpr int BMAX = 32;
    if (B > BMAX) return hipErrorInvalidValue;
    float* coef = c->coef;
    float* lossterm = c->coef + (size_t)c->n * B;
    double* zpart = c->partials;  // n*B*chunks doubles, sized by the caller (n * B * virtual_margin_chunks)
    const uint32_t k0 = (uint32_t)(c->seed & 0xffffffffu), k1 = (uint32_t)(c->seed >> 32);
    const int64_t nb = (int64_t)c->n * B;
    const int64_t d4 = (c->d + 3) / 4;
    const int64_t chunks = virtual_margin_chunks(c);
    const int64_t qpb = (d4 + chunks - 1) / chunks;
    dim3 grid1((unsigned)chunks, (unsigned)c->n), block(256);
    hipLaunchKernelGGL((k_virtual_margin<BMAX>), grid1, block, 0, c->stream, c->x, c->ld, c->d, idx,
                       B, k0, k1, c->mu_sigma, qpb, zpart);
    hipLaunchKernelGGL(k_virtual_coef, dim3((unsigned)((nb + 255) / 256)), dim3(256), 0, c->stream,
                       zpart, (int32_t)chunks, c->tgt, idx, B, c->M, c->n, coef, lossterm);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    if (loss_out) {
        hipLaunchKernelGGL(k_loss_sum, dim3((unsigned)c->n), block, 0, c->stream, lossterm, B,
                           loss_out);
        return hipGetLastError();
    }
    const int vec_ok = aligned16(c->g) && (c->ld % 4 == 0);
    dim3 grid2((unsigned)((d4 + 255) / 256), (unsigned)c->n);
    hipLaunchKernelGGL((k_virtual_accum<BMAX>), grid2, block, 0, c->stream, coef, idx, B, c->d, k0,
                       k1, c->mu_sigma, vec_ok, c->g, c->ld);
    return hipGetLastError();
}

bool small_run_fits(const gpga_ctx* c, const int32_t* idx, int32_t B) {
    if (c->opt_small_run == 0 || c->aga) return false;
    if (c->problem != PROB_LSQ && c->problem != PROB_LOGREG) return false;
    if ((c->topo == GPGA_TOPO_GRID || c->topo == GPGA_TOPO_EXPO || c->topo == GPGA_TOPO_CUSTOM) && !c->csr_ready)
        return false;
    const int64_t Beff = idx ? B : c->M;
    if (Beff < 1 || Beff > 32 || c->d > 512 || c->n > 4096) return false;  // a thread walks a row / a batch: keep both short
    const int64_t nd = (int64_t)c->n * c->d, nb = (int64_t)c->n * Beff;
    // one workgroup does all the work of an iteration: keep it to a few hundred operations per thread
    if (nd > 8192 || nb > 4096 || nb * c->d > (1 << 17)) return false;
    return small_run_lds(c, (int32_t)Beff) <= 100 * 1024 && small_run_lds(c, (int32_t)Beff) <= (size_t)c->max_lds_block;
}

template <int KIND>
static hipError_t launch_small_kind(const gpga_ctx* c, const SmallArgs& a, size_t lds) {
    const dim3 grid(1), block(kSmallRunThreads);
    if (c->mu == 0.f) {
        hipLaunchKernelGGL((k_small_run<KIND, 0>), grid, block, lds, c->stream, a);
    } else if (!c->nesterov) {
        hipLaunchKernelGGL((k_small_run<KIND, 1>), grid, block, lds, c->stream, a);
    } else {
        hipLaunchKernelGGL((k_small_run<KIND, 2>), grid, block, lds, c->stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_small_run(const gpga_ctx* c, int32_t T, const int32_t* idx, int32_t B, const float* lr) {
    if (T < 1 || T > kSmallRunMaxIters) return hipErrorInvalidValue;
    SmallArgs a;
    a.x = c->x;
    a.x_out = (T % 2) ? c->x_new : c->x;  // where T separate steps would leave the live iterates
    a.m = c->m;
    a.g = c->g;
    a.ld = c->ld;
    a.n = c->n;
    a.d = (int32_t)c->d;
    a.feat = c->feat;
    a.tgt = c->tgt;
    a.M = c->M;
    a.idx = idx;
    a.B = idx ? B : c->M;
    a.topo = c->topo;
    a.H = c->H;
    a.k0 = c->k;
    a.T = T;
    a.mu = c->mu;
    a.wptr = c->csr_ptr_d;
    a.wcol = c->csr_col_d;
    a.wval = c->csr_val_d;
    a.trace = c->trace;
    a.trace_cap = c->trace_cap;
    for (int t = 0; t < T; ++t) a.lr[t] = lr[t];
    const size_t lds = small_run_lds(c, a.B);
    return c->problem == PROB_LSQ ? launch_small_kind<PROB_LSQ>(c, a, lds) : launch_small_kind<PROB_LOGREG>(c, a, lds);
}
