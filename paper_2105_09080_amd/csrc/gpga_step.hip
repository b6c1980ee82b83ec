// Fused Gossip-PGA step kernels for gfx950 (Algorithm 1, lines 2-6 of the
// paper's listing in Sec. 3; matrix form in App. A):
//
//     m_i <- mu*m_i + g_i ;  y_i = x_i - gamma*m_i              (local update)
//     Nesterov momentum (App. F.1):  y_i = x_i - gamma*(g_i + mu*m_i)
//     gossip :  x_new_i = sum_j w_ij y_j                         (W_k sparse)
//     global :  x_new_i = (1/n) sum_j y_j                        (every H-th step)
//
// The node axis (rows) is the only axis along which elements interact, so a
// lane owns one 128-bit column group (4 fp32 columns) and *walks down rows*.
// Lanes of a wavefront sit on consecutive column groups: every access of a wave
// is one fully coalesced 1 KiB row segment.  Each element of x, m, g is read
// from HBM exactly once per step and each element of m, x_new written once.
//
// Gossip ("walk") kernel.  Both graphs are stencils along cycles of the row
// permutation i -> (i + S) mod n:
//   ring      S = 1      one cycle of length n, taps (prev, cur, next)/3
//   one-peer  S = 2^s    gcd(S,n) cycles of length n/gcd, taps (cur, next)/2
//   W = I     -          n cycles of length 1, tap cur (also used, writing y over the old
//                        iterate, as the first pass of sparse-W steps with many rows)
// A "walker" is one wavefront walking a contiguous segment of one cycle with
// the last two y values kept in registers.  When a cycle is split over Q
// wavefronts of a workgroup (few columns, many rows) the first/last y of every
// segment are staged through LDS, so neighbour rows are never re-read from HBM.
// Large problems run as persistent launches paced against the chip's clock (see
// gpga_pace.hpp): every wavefront is then at the same row at the same time, a
// paced one-peer work item takes all cycles of its column tile in turn, and
// one-peer cycles of two rows have a kernel of their own whose batches are whole
// cycles (k_step_cycles).  A tracing variant also sums the squared deviations of
// what it stores from the column means (the consensus distance of the new X).
//
// Global-average kernel.  Small problems: rows are spread over (row lanes of a
// wave) x (waves of the workgroup); partial column sums are combined with a
// wavefront shuffle (xor butterfly) and then an LDS tree across waves.  Large
// problems: one lane sums its whole column while walking it, and the n copies
// of the mean are stored row by row while the wavefront already reads its next
// tile.  Every row gets the same bits of the mean, so the rows are bit-identical
// afterwards.
#include <type_traits>

#include "gpga_internal.hpp"
#include "gpga_pace.hpp"
#include "gpga_spread.hpp"

namespace {

#ifndef GPGA_NT_LOAD
#define GPGA_NT_LOAD 1
#endif
#ifndef GPGA_NT_STORE
#define GPGA_NT_STORE 1
#endif
template <typename T>
__device__ __forceinline__ T ld_stream(const T* p) {
#if GPGA_NT_LOAD
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}
template <typename T>
__device__ __forceinline__ void st_stream(T* p, T v) {
#if GPGA_NT_STORE
    __builtin_nontemporal_store(v, p);
#else
    *p = v;
#endif
}

__device__ __forceinline__ float shfl_xor_t(float v, int off) { return __shfl_xor(v, off, kWave); }
__device__ __forceinline__ v4f shfl_xor_t(v4f v, int off) {
    v4f r;
    r.x = __shfl_xor(v.x, off, kWave);
    r.y = __shfl_xor(v.y, off, kWave);
    r.z = __shfl_xor(v.z, off, kWave);
    r.w = __shfl_xor(v.w, off, kWave);
    return r;
}

// x^(k+1/2) from x, the gradient and the NEW momentum value (mom = g when there is no buffer).
template <int MOM, typename T>
__device__ __forceinline__ T half_step(const T& xv, const T& gv, const T& mom, float lr, float mu) {
    if (MOM == 2) return xv - lr * (gv + mu * mom);
    return xv - lr * mom;
}

// Running consensus sums of the values a lane stores into its column group of
// x_new (all n rows of it): shifted by a reference close to them (the old iterate of
// the first row, set by the caller before the first add), deviations
// formed in fp32 (exact or nearly so while rows are close), sums in fp64, so
// that sum_i (x_i - xbar)^2 = S2 - S1^2 / n keeps the small quantity.
constexpr int kMaxWaves = 8;
constexpr int kDefaultUnroll = 2;  // rows per batch; two batches are in flight (software pipeline)

struct WalkArgs {
    StepGeom ge;
    int32_t S;    // row stride of the permutation
    int32_t C;    // number of cycles
    int32_t L;    // cycle length
    int32_t Q;    // segments (wavefronts) per cycle
    int32_t tpb;  // column tiles per workgroup
    int32_t xcd;  // remap tile groups so that an XCD sees contiguous tiles
    int64_t gx;   // tile groups
    int64_t gy;   // walker groups; work items = gx * gy, tile group fastest
    int32_t cpi;  // cycles per work item (1, or all C cycles when the consensus sums ride along)
    double* spread_partials;  // TRACE kernels: one sum of squared deviations per workgroup
    PaceArgs pace;
};

// blockIdx.x -> logical tile-group index.  Hardware hands consecutive workgroup
// ids to the 8 XCDs round-robin; with the remap each XCD walks a contiguous
// range of column tiles (its own L2 and the fabric then see sequential
// streams).
__device__ __forceinline__ int64_t logical_block(int64_t bid, int64_t gx, int xcd) {
    if (!xcd) return bid;
    const int64_t per = gx >> 3;          // groups per XCD (floor)
    const int64_t main_part = per << 3;   // blocks covered by the regular part
    if (bid >= main_part) return bid;     // ragged tail keeps its identity
    return (bid & 7) * per + (bid >> 3);
}


// MOM: 0 = no momentum buffer, 1 = heavy-ball, 2 = Nesterov.
// TRACE: also sum (x_new - column mean)^2 over everything stored; requires that one
// walker covers whole columns (one cycle, one segment), which the launcher checks.
template <typename T, int MODE, int MOM, int U, bool TRACE = false>
__global__ void __launch_bounds__(kWave* kMaxWaves) k_step_walk(const WalkArgs a) {
    constexpr int V = sizeof(T) / sizeof(float);
    __shared__ T s_first[kMaxWaves][kWave];
    __shared__ T s_last[kMaxWaves][kWave];
    __shared__ double s_spread[kMaxWaves];
    ColumnSpread<T> spread;
    double spread_acc = 0.0;

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform -> SGPR
    const int waves = blockDim.x >> 6;
    const int wpb = waves / a.tpb;  // walkers per workgroup
    const int tile_l = wave / wpb;
    const int walk_l = wave - tile_l * wpb;
    const int n = a.ge.n;
    const int S = a.S;
    const int64_t ldT = a.ge.ld / V;  // row stride in units of T
    const float lr = a.ge.lr, mu = a.ge.mu;
    const float third = 1.0f / 3.0f;
    constexpr uint32_t kRowUnits = MOM ? 5u : 3u;  // 4-byte streams touched per row

    const PaceRun run = pace_begin(a.pace, lane);
    uint32_t units_done = 0;

    // Grid-stride over work items (walker group, tile group), tile group
    // fastest.  With a grid sized to the resident workgroups of the chip
    // (persistent launch) all wavefronts start the same rows together and,
    // paced, stay in step: at any moment the whole chip streams a few rows of
    // x, m, g over a wide contiguous column window instead of touching all n
    // rows of every array at once.
    const int64_t work = a.gx * a.gy;
    for (int64_t w = blockIdx.x; w < work; w += gridDim.x) {
        const int by = (int)(w / a.gx);
        const int64_t bx = w - (int64_t)by * a.gx;
        // cpi > 1 (tracing one-peer steps): this work item takes all cycles of its column tile one
        // after the other, so that the lane stores - and sums - whole columns
        for (int cc = 0; cc < a.cpi; ++cc) {
        const int walker = (by * a.cpi + cc) * wpb + walk_l;
        const bool walker_on = walker < a.C * a.Q;
        const int cyc = walker / a.Q;
        const int seg = walker - cyc * a.Q;
        const int p0 = (int)(((int64_t)seg * a.L) / a.Q);
        const int p1 = (int)(((int64_t)(seg + 1) * a.L) / a.Q);
        const int len = p1 - p0;
        const int row_first = (int)(((int64_t)cyc + (int64_t)p0 * S) % n);

        const int64_t tile = logical_block(bx, a.gx, a.xcd) * a.tpb + tile_l;
        const int64_t col = tile * kWave + lane;
        const bool on = walker_on && (col < a.ge.ncols);
        const int64_t coff = col;

        const T* __restrict__ xp = reinterpret_cast<const T*>(a.ge.x + a.ge.col0) + coff;
        const T* __restrict__ gp = reinterpret_cast<const T*>(a.ge.g + a.ge.col0) + coff;
        T* __restrict__ mp = MOM ? reinterpret_cast<T*>(a.ge.m + a.ge.col0) + coff : nullptr;
        T* __restrict__ xnp = reinterpret_cast<T*>(a.ge.x_new + a.ge.col0) + coff;
        auto put = [&](int rw, const T& v) {
            st_stream(xnp + (int64_t)rw * ldT, v);
            if (TRACE) spread.add(v);
        };

        T yf = T(0), ys = T(0), pp = T(0), pc = T(0);
        int row = row_first;
        int row_prev = row;

        // One row: issue its three loads / turn loaded values into y (and store m).
        auto load_row = [&](T& xv, T& mv, T& gv, int& rw) {
            rw = row;
            const int64_t off = (int64_t)row * ldT;
            xv = ld_stream(xp + off);
            if (MOM) mv = ld_stream(mp + off);
            gv = ld_stream(gp + off);
            row += S;
            if (row >= n) row -= n;
        };
        auto y_of = [&](const T& xv, const T& mv, const T& gv, int rw) -> T {
            T mom = gv;
            if (MOM) {
                mom = mu * mv + gv;
                st_stream(mp + (int64_t)rw * ldT, mom);
            }
            return half_step<MOM>(xv, gv, mom, lr, mu);
        };
        // Steady state (third row of the segment onwards): the new y completes the
        // stencil of the previous row.
        auto emit = [&](const T& y, int rw) {
            if (MODE == MODE_RING) put(row_prev, (pp + pc + y) * third);
            if (MODE == MODE_PEER) put(row_prev, (pc + y) * 0.5f);
            pp = pc;
            pc = y;
            row_prev = rw;
        };
        struct Batch {
            T xv[U], mv[U], gv[U];
            int rw[U];
        };
        auto load_full = [&](Batch& b) {
            pace_wait(run, units_done);
            units_done += U * kRowUnits;
#pragma unroll
            for (int u = 0; u < U; ++u) load_row(b.xv[u], b.mv[u], b.gv[u], b.rw[u]);
        };
        auto process_full = [&](const Batch& b) {
#pragma unroll
            for (int u = 0; u < U; ++u) emit(y_of(b.xv[u], b.mv[u], b.gv[u], b.rw[u]), b.rw[u]);
        };

        if (on) {
            // First two rows of the segment: they only start the stencil window.
            {
                T x0, m0, g0, x1, m1, g1;
                int r0 = 0, r1 = 0;
                pace_wait(run, units_done);
                units_done += (len >= 2 ? 2u : 1u) * kRowUnits;
                load_row(x0, m0, g0, r0);
                if (len >= 2) load_row(x1, m1, g1, r1);
                if (TRACE && cc == 0) spread.reset(x0);
                yf = y_of(x0, m0, g0, r0);
                if (MODE == MODE_SELF) st_stream(xnp + (int64_t)r0 * ldT, yf);
                // in place: over the old iterate, through a pointer derived from the one it was read with
                if (MODE == MODE_INPLACE) st_stream(const_cast<T*>(xp) + (int64_t)r0 * ldT, yf);
                pc = yf;
                row_prev = r0;
                if (len >= 2) {
                    ys = y_of(x1, m1, g1, r1);
                    if (MODE == MODE_PEER) put(r0, (yf + ys) * 0.5f);
                    if (MODE == MODE_SELF) st_stream(xnp + (int64_t)r1 * ldT, ys);
                    if (MODE == MODE_INPLACE) st_stream(const_cast<T*>(xp) + (int64_t)r1 * ldT, ys);
                    pp = yf;
                    pc = ys;
                    row_prev = r1;
                }
            }
            // Software-pipelined steady state over full batches of U rows.  The
            // loads of the next batch are issued BEFORE the stores of the current
            // one: a wavefront's memory operations retire in order, so a wait for
            // those loads never includes the slower write acknowledgements of the
            // stores behind them.  The hot loop is branch-free so that the wait
            // counts stay exact.
            const int rem = len > 2 ? len - 2 : 0;
            const int nfull = rem / U;
            const int tail = rem - nfull * U;
            Batch A, B;
            if (nfull >= 1) {
                load_full(A);
                int b = 0;
                for (; b + 3 <= nfull; b += 2) {
                    load_full(B);
                    __builtin_amdgcn_sched_barrier(0);  // keep the issue order: loads, then stores
                    process_full(A);
                    __builtin_amdgcn_sched_barrier(0);
                    load_full(A);
                    __builtin_amdgcn_sched_barrier(0);
                    process_full(B);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if (nfull - b == 2) {
                    load_full(B);
                    __builtin_amdgcn_sched_barrier(0);
                    process_full(A);
                    process_full(B);
                } else {
                    process_full(A);
                }
            }
            for (int t = 0; t < tail; ++t) {
                T xv, mv, gv;
                int rw;
                units_done += kRowUnits;
                load_row(xv, mv, gv, rw);
                emit(y_of(xv, mv, gv, rw), rw);
            }
        }
        if (MODE == MODE_SELF || MODE == MODE_INPLACE) continue;

        // Close the stencil at the two ends of the segment.  One walker per
        // cycle: the cycle closes on itself.  Q walkers per cycle: neighbours'
        // boundary y values come through LDS.
        T left = pc, right = yf;
        if (a.Q > 1) {
            s_first[wave][lane] = yf;
            s_last[wave][lane] = pc;
            __syncthreads();
            const int w0 = wave - seg;
            left = s_last[w0 + (seg + a.Q - 1) % a.Q][lane];
            right = s_first[w0 + (seg + 1) % a.Q][lane];
            __syncthreads();  // LDS is rewritten by the next tile group
        }
        if (on) {
            if (MODE == MODE_RING) {
                if (len == 1) {
                    put(row_first, (left + yf + right) * third);
                } else {
                    put(row_first, (left + yf + ys) * third);
                    put(row_prev, (pp + pc + right) * third);
                }
            } else {  // MODE_PEER: last row of the segment pairs with the next segment's first
                put(row_prev, (pc + right) * 0.5f);
            }
            if (TRACE && cc == a.cpi - 1) spread_acc += spread.sum_sq(1.0 / (double)n);
        }
        }  // cycles of this work item
    }
    const unsigned long long t_done = pace_now(a.pace);
    if (TRACE) {
        // one partial per workgroup, summed in a fixed order
        double v = spread_acc;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
        if (lane == 0) s_spread[wave] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w = 0; w < waves; ++w) t += s_spread[w];
            a.spread_partials[blockIdx.x] = t;
        }
    }
    pace_end(a.pace, run, units_done, lane, t_done);
}

// One-peer steps whose cycles are short (instantiated for L = 2, 4, 8 and 16 rows: offsets n/2 ... n/16).
// A lane streams the rows of its column group cycle after cycle - rows c, c+S, ..., c+(L-1)S of
// cycle c, then cycle c+1 - as ONE software pipeline: one row per batch, the loads of the next row
// (which may belong to the next cycle) issued ahead of this row's stores, two rows in flight
// throughout.  Only the stencil restarts at a cycle boundary: the first y of a cycle is kept to
// close it, (y_{L-1} + y_0) / 2, when its last row arrives.  The general walk kernel drains its
// pipeline at the end of every cycle; with 4-row cycles that exposed one memory latency per four
// rows and its wavefronts fell behind the pacing clock 5 % earlier than on long cycles.
// The body is unrolled over the L rows of a cycle, so the loop over cycles is branch-free.
struct CycleArgs {
    StepGeom ge;
    int32_t S;   // row offset of the peer
    int32_t C;   // number of cycles
    int64_t gx;  // tile groups (one column tile per wavefront)
    double* spread_partials;  // TRACE kernels: one sum of squared deviations per workgroup
    PaceArgs pace;
};

template <int MOM, int L, bool TRACE = false>
__global__ void __launch_bounds__(kWave* kMaxWaves) k_step_cycles(const CycleArgs a) {
    static_assert(L >= 2 && L % 2 == 0, "two row buffers alternate: a cycle has an even number of rows");
    typedef v4f T;
    __shared__ double s_spread[kMaxWaves];
    ColumnSpread<T> spread;
    double spread_acc = 0.0;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int waves = blockDim.x >> 6;
    const int n = a.ge.n;
    const int S = a.S;
    const int64_t ldT = a.ge.ld / 4;
    const float lr = a.ge.lr, mu = a.ge.mu;
    constexpr uint32_t kRowUnits = MOM ? 5u : 3u;
    const PaceRun run = pace_begin(a.pace, lane);
    uint32_t units_done = 0;

    for (int64_t w = blockIdx.x; w < a.gx; w += gridDim.x) {
        const int64_t col = (w * waves + wave) * kWave + lane;
        if (col >= a.ge.ncols) continue;
        if (TRACE) spread.reset(reinterpret_cast<const T*>(a.ge.x + a.ge.col0)[col]);  // row 0 of the old iterate
        const T* __restrict__ xp = reinterpret_cast<const T*>(a.ge.x + a.ge.col0) + col;
        const T* __restrict__ gp = reinterpret_cast<const T*>(a.ge.g + a.ge.col0) + col;
        T* __restrict__ mp = MOM ? reinterpret_cast<T*>(a.ge.m + a.ge.col0) + col : nullptr;
        T* __restrict__ xnp = reinterpret_cast<T*>(a.ge.x_new + a.ge.col0) + col;

        struct Row {
            T xv, mv, gv;
            int rw;
        };
        int next_row = 0;  // row the next load takes: walks cycle 0, then cycle 1, ...
        int next_pos = 0, next_cyc = 0;
        auto load_row = [&](Row& b) {
            pace_wait(run, units_done);
            units_done += kRowUnits;
            b.rw = next_row;
            const int64_t off = (int64_t)next_row * ldT;
            b.xv = ld_stream(xp + off);
            if (MOM) b.mv = ld_stream(mp + off);
            b.gv = ld_stream(gp + off);
            if (++next_pos == L) {  // on to the first row of the next cycle
                next_pos = 0;
                next_row = ++next_cyc;
            } else {
                next_row += S;
                if (next_row >= n) next_row -= n;
            }
        };
        T yf = T(0), pc = T(0);
        int row_prev = 0;
        auto process = [&](const Row& b, int pos) {  // pos is a compile-time constant at every call
            T mom = b.gv;
            if (MOM) {
                mom = mu * b.mv + b.gv;
                st_stream(mp + (int64_t)b.rw * ldT, mom);
            }
            const T y = half_step<MOM>(b.xv, b.gv, mom, lr, mu);
            if (pos == 0) {
                yf = y;
            } else {
                const T v = (pc + y) * 0.5f;
                st_stream(xnp + (int64_t)row_prev * ldT, v);
                if (TRACE) spread.add(v);
            }
            if (pos == L - 1) {
                const T v = (y + yf) * 0.5f;
                st_stream(xnp + (int64_t)b.rw * ldT, v);
                if (TRACE) spread.add(v);
            }
            pc = y;
            row_prev = b.rw;
        };
        Row A, B;
        load_row(A);
        for (int c = 0; c + 1 < a.C; ++c) {  // every cycle but the last: the load after its last row opens the next cycle
#pragma unroll
            for (int pos = 0; pos < L; pos += 2) {
                load_row(B);
                __builtin_amdgcn_sched_barrier(0);  // keep the issue order: loads, then stores
                process(A, pos);
                __builtin_amdgcn_sched_barrier(0);
                load_row(A);
                __builtin_amdgcn_sched_barrier(0);
                process(B, pos + 1);
                __builtin_amdgcn_sched_barrier(0);
            }
        }
#pragma unroll
        for (int pos = 0; pos < L; pos += 2) {  // the last cycle: nothing to load after its last row
            load_row(B);
            __builtin_amdgcn_sched_barrier(0);
            process(A, pos);
            __builtin_amdgcn_sched_barrier(0);
            if (pos + 2 < L) load_row(A);
            __builtin_amdgcn_sched_barrier(0);
            process(B, pos + 1);
            __builtin_amdgcn_sched_barrier(0);
        }
        if (TRACE) spread_acc += spread.sum_sq(1.0 / (double)n);
    }
    const unsigned long long t_done = pace_now(a.pace);
    if (TRACE) {
        double v = spread_acc;
#pragma unroll
        for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
        if (lane == 0) s_spread[wave] = v;
        __syncthreads();
        if (threadIdx.x == 0) {
            double t = 0.0;
            for (int w2 = 0; w2 < waves; ++w2) t += s_spread[w2];
            a.spread_partials[blockIdx.x] = t;
        }
    }
    pace_end(a.pace, run, units_done, lane, t_done);
}

struct GlobalArgs {
    StepGeom ge;
    int32_t RL;   // lanes of a wave spread over rows (1, 2, 4)
    int32_t tpb;  // column tiles per workgroup
    int32_t xcd;
    int64_t gx;
    float inv_n;
    PaceArgs pace;
};

template <typename T, int MOM, int U>
__global__ void __launch_bounds__(kWave* kMaxWaves) k_step_global(const GlobalArgs a) {
    constexpr int V = sizeof(T) / sizeof(float);
    __shared__ T s_part[kMaxWaves][kWave];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);  // wave-uniform -> SGPR
    const int waves = blockDim.x >> 6;
    const int wpb = waves / a.tpb;  // waves sharing one column tile
    const int tile_l = wave / wpb;
    const int wrow = wave - tile_l * wpb;
    const int CL = kWave / a.RL;  // column lanes per wave
    const int lane_c = lane & (CL - 1);
    const int lane_r = lane / CL;
    const int n = a.ge.n;
    const int RS = a.RL * wpb;            // row splitters per column
    const int r0 = wrow * a.RL + lane_r;  // this lane's first row
    const int64_t ldT = a.ge.ld / V;  // row stride in units of T
    const float lr = a.ge.lr, mu = a.ge.mu;
    constexpr uint32_t kReadUnits = MOM ? 4u : 2u;  // 4-byte streams per row in the read phase
    const PaceRun run = pace_begin(a.pace, lane);
    uint32_t units_done = 0;

    // deferred mean of the previous whole tile of this wavefront (see below)
    T prev_mean = T(0);
    T* prev_xnp = nullptr;
    bool have_prev = false;  // wave-uniform
    auto flush_prev = [&]() {
        for (int row = 0; row < n; row += U) {
            pace_wait(run, units_done);
            units_done += U;
#pragma unroll
            for (int u = 0; u < U; ++u)
                if (row + u < n) st_stream(prev_xnp + (int64_t)(row + u) * ldT, prev_mean);
        }
    };

    for (int64_t bx = blockIdx.x; bx < a.gx; bx += gridDim.x) {
        const int64_t tile = logical_block(bx, a.gx, a.xcd) * a.tpb + tile_l;
        const int64_t col = tile * CL + lane_c;
        const bool on = col < a.ge.ncols;
        const int64_t coff = col;

        const T* __restrict__ xp = reinterpret_cast<const T*>(a.ge.x + a.ge.col0) + coff;
        const T* __restrict__ gp = reinterpret_cast<const T*>(a.ge.g + a.ge.col0) + coff;
        T* __restrict__ mp = MOM ? reinterpret_cast<T*>(a.ge.m + a.ge.col0) + coff : nullptr;
        T* __restrict__ xnp = reinterpret_cast<T*>(a.ge.x_new + a.ge.col0) + coff;

        T sum = T(0);
        // One lane walks all n rows of its column group (large problems).  The n copies of
        // a tile's mean are not written in a burst of their own: they are DEFERRED and
        // stored row by row while the next tile of this wavefront is being read, so that
        // the chip sees the same steady 3-read : 2-write mix as in the gossip walk.  Only
        // whole tiles take this path (the ragged last tile falls through to the plain one).
        const bool whole_tile = (tile + 1) * CL <= a.ge.ncols;  // wave-uniform
        if (RS == 1 && whole_tile) {
            // Same software pipeline as the gossip walk: next batch's loads are issued
            // ahead of this batch's stores; branch-free hot loop.
            struct Batch {
                T xv[U], mv[U], gv[U];
            };
            auto rows_pass = [&](auto with_prev) {
                constexpr bool WP = decltype(with_prev)::value;
                constexpr uint32_t kUnits = kReadUnits + (WP ? 1u : 0u);
                int row = 0;
                auto load_full = [&](Batch& b) {
                    pace_wait(run, units_done);
                    units_done += U * kUnits;
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        const int64_t off = (int64_t)(row + u) * ldT;
                        b.xv[u] = ld_stream(xp + off);
                        if (MOM) b.mv[u] = ld_stream(mp + off);
                        b.gv[u] = ld_stream(gp + off);
                    }
                    row += U;
                };
                auto process_full = [&](const Batch& b, int first_row) {
                    T part = T(0);
#pragma unroll
                    for (int u = 0; u < U; ++u) {
                        T mom = b.gv[u];
                        if (MOM) {
                            mom = mu * b.mv[u] + b.gv[u];
                            st_stream(mp + (int64_t)(first_row + u) * ldT, mom);
                        }
                        if (WP) st_stream(prev_xnp + (int64_t)(first_row + u) * ldT, prev_mean);
                        part += half_step<MOM>(b.xv[u], b.gv[u], mom, lr, mu);
                    }
                    sum += part;
                };
                const int nfull = n / U;
                Batch A, B;
                int done = 0;
                if (nfull >= 1) {
                    load_full(A);
                    int b = 0;
                    for (; b + 3 <= nfull; b += 2) {
                        load_full(B);
                        __builtin_amdgcn_sched_barrier(0);
                        process_full(A, done);
                        __builtin_amdgcn_sched_barrier(0);
                        load_full(A);
                        __builtin_amdgcn_sched_barrier(0);
                        process_full(B, done + U);
                        __builtin_amdgcn_sched_barrier(0);
                        done += 2 * U;
                    }
                    if (nfull - b == 2) {
                        load_full(B);
                        __builtin_amdgcn_sched_barrier(0);
                        process_full(A, done);
                        process_full(B, done + U);
                        done += 2 * U;
                    } else {
                        process_full(A, done);
                        done += U;
                    }
                }
                for (; done < n; ++done) {
                    const int64_t off = (int64_t)done * ldT;
                    const T xv = ld_stream(xp + off);
                    const T gv = ld_stream(gp + off);
                    T mom = gv;
                    if (MOM) {
                        mom = mu * ld_stream(mp + off) + gv;
                        st_stream(mp + off, mom);
                    }
                    if (WP) st_stream(prev_xnp + off, prev_mean);
                    units_done += kUnits;
                    sum += half_step<MOM>(xv, gv, mom, lr, mu);
                }
            };
            if (have_prev) rows_pass(std::true_type{}); else rows_pass(std::false_type{});
            prev_mean = sum * a.inv_n;
            prev_xnp = xnp;
            have_prev = true;
            continue;
        }
        if (have_prev) {  // a tile that writes at once follows: nothing may stay deferred behind it
            flush_prev();
            have_prev = false;
        }
        if (on) {
            for (int base = r0; base < n; base += RS * U) {
                T xv[U], mv[U], gv[U];
                pace_wait(run, units_done);
                units_done += U * kReadUnits;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int row = base + u * RS;
                    if (row < n) {
                        const int64_t off = (int64_t)row * ldT;
                        xv[u] = ld_stream(xp + off);
                        if (MOM) mv[u] = ld_stream(mp + off);
                        gv[u] = ld_stream(gp + off);
                    }
                }
                T part = T(0);
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int row = base + u * RS;
                    if (row < n) {
                        T mom = gv[u];
                        if (MOM) {
                            mom = mu * mv[u] + gv[u];
                            st_stream(mp + (int64_t)row * ldT, mom);
                        }
                        part += half_step<MOM>(xv[u], gv[u], mom, lr, mu);
                    }
                }
                sum += part;
            }
        }
        // wavefront shuffle across the row lanes (xor butterfly: all lanes end equal)
        for (int off = CL; off < kWave; off <<= 1) sum += shfl_xor_t(sum, off);
        // LDS tree across the waves that share this column tile
        if (wpb > 1) {
            if (lane_r == 0) s_part[wave][lane_c] = sum;
            __syncthreads();
            const int w0 = tile_l * wpb;
            for (int stride = 1; stride < wpb; stride <<= 1) {
                if (lane_r == 0 && (wrow & (2 * stride - 1)) == 0 && wrow + stride < wpb)
                    s_part[wave][lane_c] += s_part[wave + stride][lane_c];
                __syncthreads();
            }
            sum = s_part[w0][lane_c];
            __syncthreads();  // LDS is rewritten by the next tile group
        }
        const T mean = sum * a.inv_n;
        if (on) {
            for (int base = r0; base < n; base += RS * U) {
                pace_wait(run, units_done);
                units_done += U;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    const int row = base + u * RS;
                    if (row < n) st_stream(xnp + (int64_t)row * ldT, mean);
                }
            }
        }
    }
    if (have_prev) flush_prev();
    pace_end(a.pace, run, units_done, lane, pace_now(a.pace));
}

int gcd_i(int a, int b) {
    while (b) {
        int t = a % b;
        a = b;
        b = t;
    }
    return a;
}
int pow2_floor(int v) {
    int p = 1;
    while (p * 2 <= v) p *= 2;
    return p;
}
int pow2_ceil(int v) {
    int p = 1;
    while (p < v) p *= 2;
    return p;
}

// Launch plan shared by both kernels: `work` work items; persistent launches
// use at most blocks_per_cu resident workgroups per compute unit (never more
// than the kernel's occupancy allows, so that every workgroup is resident and
// the paced wavefronts really run side by side).
struct LaunchPlan {
    int64_t work = 0;        // work items of a one-shot launch
    int bpc = 0;             // requested resident workgroups per CU (0 = one-shot launch)
    int num_cus = 0;
    int waves = 0;           // wavefronts per workgroup
    double pace_gbs = 0.0;   // 0 = free running, > 0 = paced at this rate, < 0 = paced at the rate the controller finds
    int pace_key = 0;        // which controller state the launch shares (PaceKey)
    double clock_hz = 1e8;
    int vec = 4;
    const gpga_ctx* ctx = nullptr;
    int64_t* blocks_out = nullptr;  // receives the number of workgroups launched
};

template <typename Args, typename Kernel>
hipError_t launch_planned(Kernel kernel, LaunchPlan plan, Args a, hipStream_t st) {
    const int threads = kWave * plan.waves;
    int64_t blocks = plan.work;
    pace_setup(nullptr, 0.0, 0, 0.0, 0, &a.pace);
    if (plan.bpc > 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, kernel, threads, 0) != hipSuccess || occ < 1) occ = 1;
        const int bpc = plan.bpc < occ ? plan.bpc : occ;
        const int64_t resident = (int64_t)plan.num_cus * bpc;
        if (resident < blocks) blocks = balanced_blocks(plan.work, resident);  // persistent: each workgroup strides over the work items
        // Pacing needs every workgroup of the launch to be resident at once, which
        // holds here: blocks <= CUs x workgroups per CU that fit.
        pace_setup(const_cast<gpga_ctx*>(plan.ctx), plan.pace_gbs, plan.pace_key, (double)blocks * plan.waves, plan.vec * 4, &a.pace);
    }
    if (blocks > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    if (plan.blocks_out) *plan.blocks_out = blocks;
    hipLaunchKernelGGL(kernel, dim3((unsigned)blocks), dim3(threads), 0, st, a);
    return hipGetLastError();
}

template <int MOM, int L>
hipError_t launch_cycles_traced(bool traced, const LaunchPlan& plan, const CycleArgs& a, hipStream_t st) {
    return traced ? launch_planned(k_step_cycles<MOM, L, true>, plan, a, st)
                  : launch_planned(k_step_cycles<MOM, L, false>, plan, a, st);
}
template <int MOM>
hipError_t launch_cycles_len(int L, bool traced, const LaunchPlan& plan, const CycleArgs& a, hipStream_t st) {
    if (L == 2) return launch_cycles_traced<MOM, 2>(traced, plan, a, st);
    if (L == 4) return launch_cycles_traced<MOM, 4>(traced, plan, a, st);
    if (L == 8) return launch_cycles_traced<MOM, 8>(traced, plan, a, st);
    return launch_cycles_traced<MOM, 16>(traced, plan, a, st);
}
hipError_t launch_cycles(int L, int mom, bool traced, const LaunchPlan& plan, const CycleArgs& a, hipStream_t st) {
    if (mom == 2) return launch_cycles_len<2>(L, traced, plan, a, st);
    return mom ? launch_cycles_len<1>(L, traced, plan, a, st) : launch_cycles_len<0>(L, traced, plan, a, st);
}

template <typename T, int MODE, int MOM>
hipError_t launch_walk_u(int U, const LaunchPlan& plan, hipStream_t st, const WalkArgs& a) {
    switch (U) {
        case 1: return launch_planned(k_step_walk<T, MODE, MOM, 1>, plan, a, st);
        case 2: return launch_planned(k_step_walk<T, MODE, MOM, 2>, plan, a, st);
        case 8: return launch_planned(k_step_walk<T, MODE, MOM, 8>, plan, a, st);
        default: return launch_planned(k_step_walk<T, MODE, MOM, 4>, plan, a, st);
    }
}

// Tracing variants exist for the default geometry only (128-bit lanes, 1 or 2 rows per batch).
template <int MOM>
hipError_t launch_walk_trace(int mode, int U, const LaunchPlan& plan, hipStream_t st, const WalkArgs& a) {
    if (mode == MODE_RING) {
        return U == 1 ? launch_planned(k_step_walk<v4f, MODE_RING, MOM, 1, true>, plan, a, st)
                      : launch_planned(k_step_walk<v4f, MODE_RING, MOM, 2, true>, plan, a, st);
    }
    return U == 1 ? launch_planned(k_step_walk<v4f, MODE_PEER, MOM, 1, true>, plan, a, st)
                  : launch_planned(k_step_walk<v4f, MODE_PEER, MOM, 2, true>, plan, a, st);
}

template <typename T, int MOM>
hipError_t launch_walk_mode(int mode, int U, const LaunchPlan& plan, hipStream_t st, const WalkArgs& a) {
    switch (mode) {
        case MODE_RING: return launch_walk_u<T, MODE_RING, MOM>(U, plan, st, a);
        case MODE_PEER: return launch_walk_u<T, MODE_PEER, MOM>(U, plan, st, a);
        case MODE_INPLACE: return launch_walk_u<T, MODE_INPLACE, MOM>(U, plan, st, a);
        default: return launch_walk_u<T, MODE_SELF, MOM>(U, plan, st, a);
    }
}

template <typename T, int MOM>
hipError_t launch_global_u(int U, const LaunchPlan& plan, hipStream_t st, const GlobalArgs& a) {
    switch (U) {
        case 1: return launch_planned(k_step_global<T, MOM, 1>, plan, a, st);
        case 2: return launch_planned(k_step_global<T, MOM, 2>, plan, a, st);
        case 8: return launch_planned(k_step_global<T, MOM, 8>, plan, a, st);
        default: return launch_planned(k_step_global<T, MOM, 4>, plan, a, st);
    }
}

// From this many whole-column walkers on (half of the 256 CUs x 16 resident
// wavefronts) the chip is kept busy with one wavefront per column tile walking
// all its rows, which is the shape the paced launch needs; below it the rows
// are split over lanes / wavefronts of a workgroup instead.
constexpr int64_t kPacedWaves = 2048;

// Default policy: large launches whose wavefronts each walk many rows run
// persistent and paced, at the rate the controller of their kind has found;
// everything else is a one-shot launch.
constexpr int kAutoBlocksPerCu = 4;

LaunchPlan make_plan(const gpga_ctx* c, int64_t work, int waves, int vec, bool walks_rows, int pace_key) {
    LaunchPlan p;
    p.work = work;
    p.num_cus = c->num_cus;
    p.waves = waves;
    p.vec = vec;
    p.ctx = c;
    p.clock_hz = c->clock_hz;
    p.pace_key = pace_key;
    const bool big = walks_rows && vec == 4 && (int64_t)c->n * c->d * 4 >= kPaceMinBytes;
    p.bpc = c->opt_blocks_per_cu < 0 ? (big ? kAutoBlocksPerCu : 0) : c->opt_blocks_per_cu;
    p.pace_gbs = c->opt_pace_gbs < 0 ? (big ? -1.0 : 0.0) : (double)c->opt_pace_gbs;
    if (!walks_rows) p.pace_gbs = 0.0;
    return p;
}

}  // namespace

hipError_t launch_step_walk(const gpga_ctx* c, const StepGeom& ge, int mode, int32_t S, int vec,
                            double* spread_partials, int64_t* spread_count) {
    if (spread_count) *spread_count = 0;
    if (ge.ncols <= 0) return hipSuccess;
    const int n = ge.n;
    WalkArgs a;
    a.ge = ge;
    if (mode == MODE_SELF || mode == MODE_INPLACE) {
        a.S = 0;
        a.C = n;
        a.L = 1;
    } else {
        a.S = S;
        a.C = gcd_i(S, n);
        a.L = n / a.C;
    }
    const int waves = c->opt_waves ? c->opt_waves : 4;
    const int64_t tiles = (ge.ncols + kWave - 1) / kWave;

    // One-peer steps over short cycles (2, 4, 8 or 16 rows) on large problems: the row-streaming kernel,
    // persistent and paced.
    if (mode == MODE_PEER && vec == 4 && (a.L == 2 || a.L == 4 || a.L == 8 || a.L == 16) && !c->opt_row_split &&
        c->opt_cycle_kernel != 0 && (tiles >= kPacedWaves || c->opt_cycle_kernel == 1)) {
        CycleArgs ca;
        ca.ge = ge;
        ca.S = S;
        ca.C = a.C;
        ca.gx = (tiles + waves - 1) / waves;
        LaunchPlan plan = make_plan(c, ca.gx, waves, vec, true,
                                    a.L == 2 ? PACE_CYCLES : a.L == 4 ? PACE_PEER_4 : a.L == 8 ? PACE_PEER_8 : PACE_PEER_16);
        if (c->opt_blocks_per_cu < 0 && plan.bpc == 0) plan.bpc = kAutoBlocksPerCu;  // forced on a small problem
        const int momk = c->mu != 0.f ? (c->nesterov ? 2 : 1) : 0;
        ca.spread_partials = nullptr;
        const bool traced = spread_partials && spread_count;  // every lane stores whole columns: the consensus sums ride along
        if (traced) {
            ca.spread_partials = spread_partials;
            plan.blocks_out = spread_count;
        }
        c->note_path(PATH_CYCLES, 16);
        return launch_cycles(a.L, momk, traced, plan, ca, c->stream);
    }

    c->note_path(PATH_WALK, vec * 4);
    int Q = 1;
    if (mode != MODE_SELF && mode != MODE_INPLACE) {
        if (c->opt_row_split) {
            Q = c->opt_row_split;
        } else if (tiles * a.C < kPacedWaves) {
            // too few column tiles to occupy the chip with one walker per cycle:
            // split each cycle over the wavefronts of a workgroup (LDS exchange)
            Q = pow2_floor(a.L / 4 > 0 ? a.L / 4 : 1);  // keep segments of >= 4 rows
        }
        if (Q > waves) Q = waves;
        if (Q > a.L) Q = pow2_floor(a.L);
    }
    a.Q = Q;
    // Walkers per workgroup.  One walker per cycle and plenty of tiles: give a
    // workgroup adjacent tiles of ONE cycle (wpb = 1), so that a launch works on
    // one cycle group at a time and few rows are open at once.  Otherwise pack
    // the walkers of a tile into one workgroup.
    int wpb = pow2_ceil((int)((int64_t)a.C * Q > waves ? waves : a.C * Q));
    if (wpb > waves) wpb = waves;
    if (Q == 1 && tiles >= kPacedWaves && !c->opt_row_split) wpb = 1;
    if (wpb < Q) wpb = Q;
    a.tpb = waves / wpb;
    const int64_t gx = (tiles + a.tpb - 1) / a.tpb;
    const int64_t gy = ((int64_t)a.C * Q + wpb - 1) / wpb;
    if (gx * gy > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.gx = gx;
    a.gy = gy;
    a.xcd = c->opt_xcd_swizzle;
    // pacing assumes every wavefront does the same work: one walker per cycle, equal segments
    const bool uniform = (Q == 1) && (((int64_t)a.C * Q) % wpb == 0);
    // cycles of 4 rows and more are paced (a work item then takes all cycles of its tile, below);
    // shorter ones keep few rows open in a one-shot launch anyway
    const int min_cycle = c->opt_pace_min_cycle > 0 ? c->opt_pace_min_cycle : 4;
    // short cycles sustain lower rates than long walks (measured on n = 64, d = 25.6M: 8 rows 5.97 TB/s,
    // 4 rows 5.78 TB/s, long walks 6.15 TB/s), so each class has a controller of its own
    const int pace_key = mode == MODE_RING ? PACE_RING
                         : mode != MODE_PEER ? PACE_SELF
                         : a.L <= 4 ? PACE_PEER_4 : a.L <= 8 ? PACE_PEER_8 : PACE_PEER_LONG;
    const LaunchPlan plan = make_plan(c, gx * gy, waves, vec, uniform && a.L >= min_cycle, pace_key);
    // paced wavefronts advance one row per batch (two rows in flight); free-running ones two
    const int U = c->opt_unroll ? c->opt_unroll : (plan.pace_gbs != 0.0 ? 1 : kDefaultUnroll);
    const int mom = c->mu != 0.f ? (c->nesterov ? 2 : 1) : 0;
    a.spread_partials = nullptr;
    a.cpi = 1;
    LaunchPlan lp = plan;
    // Paced launches with one cycle per workgroup: a work item takes ALL cycles of its column tile
    // in turn instead of one (measured 3.41 -> 3.33 ms on n = 1024, d = 1M); its lanes then store
    // whole columns, as they do when there is a single cycle.
    if (a.C > 1 && Q == 1 && wpb == 1 && plan.pace_gbs != 0.0 && plan.bpc > 0 && mode == MODE_PEER) {
        a.cpi = a.C;
        a.gy = 1;
        lp.work = a.gx;
    }
    const bool whole_columns = a.C == 1 || a.cpi == a.C;
    // the consensus sums can ride along when one walker stores whole columns
    if (spread_partials && spread_count && vec == 4 && Q == 1 && whole_columns && (U == 1 || U == 2) &&
        (mode == MODE_RING || mode == MODE_PEER)) {
        lp.blocks_out = spread_count;
        a.spread_partials = spread_partials;
        if (mom == 2) return launch_walk_trace<2>(mode, U, lp, c->stream, a);
        return mom ? launch_walk_trace<1>(mode, U, lp, c->stream, a) : launch_walk_trace<0>(mode, U, lp, c->stream, a);
    }
    if (vec == 4) {
        if (mom == 2) return launch_walk_mode<v4f, 2>(mode, U, lp, c->stream, a);
        return mom ? launch_walk_mode<v4f, 1>(mode, U, lp, c->stream, a)
                   : launch_walk_mode<v4f, 0>(mode, U, lp, c->stream, a);
    }
    if (mom == 2) return launch_walk_mode<float, 2>(mode, U, lp, c->stream, a);
    return mom ? launch_walk_mode<float, 1>(mode, U, lp, c->stream, a)
               : launch_walk_mode<float, 0>(mode, U, lp, c->stream, a);
}

hipError_t launch_step_global(const gpga_ctx* c, const StepGeom& ge, int vec) {
    if (ge.ncols <= 0) return hipSuccess;
    c->note_path(PATH_GLOBAL, vec * 4);
    const int n = ge.n;
    GlobalArgs a;
    a.ge = ge;
    a.inv_n = 1.0f / (float)n;
    const int waves = c->opt_waves ? c->opt_waves : 4;

    // Spread rows over lanes and waves only when columns alone cannot fill the chip.
    const int64_t tiles64 = (ge.ncols + kWave - 1) / kWave;
    int RL = 1, wpb = 1;
    if (c->opt_row_lanes) {
        RL = c->opt_row_lanes;
    } else if (tiles64 < kPacedWaves) {
        RL = 4;
    }
    while (RL > 1 && RL > n) RL >>= 1;
    if (c->opt_row_split) {
        wpb = c->opt_row_split;
    } else if (tiles64 < kPacedWaves) {
        wpb = pow2_floor(n / (4 * RL) > 0 ? n / (4 * RL) : 1);
    }
    if (wpb > waves) wpb = waves;
    while (wpb > 1 && RL * wpb > n) wpb >>= 1;
    a.RL = RL;
    a.tpb = waves / wpb;
    const int CL = kWave / RL;
    const int64_t tiles = (ge.ncols + CL - 1) / CL;
    const int64_t gx = (tiles + a.tpb - 1) / a.tpb;
    if (gx > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.gx = gx;
    a.xcd = c->opt_xcd_swizzle;
    const LaunchPlan plan = make_plan(c, gx, waves, vec, RL == 1 && wpb == 1 && n >= 8, PACE_GLOBAL);
    const int U = c->opt_unroll ? c->opt_unroll : (plan.pace_gbs != 0.0 ? 1 : 4);
    const int mom = c->mu != 0.f ? (c->nesterov ? 2 : 1) : 0;
    if (vec == 4) {
        if (mom == 2) return launch_global_u<v4f, 2>(U, plan, c->stream, a);
        return mom ? launch_global_u<v4f, 1>(U, plan, c->stream, a)
                   : launch_global_u<v4f, 0>(U, plan, c->stream, a);
    }
    if (mom == 2) return launch_global_u<float, 2>(U, plan, c->stream, a);
    return mom ? launch_global_u<float, 1>(U, plan, c->stream, a)
               : launch_global_u<float, 0>(U, plan, c->stream, a);
}
