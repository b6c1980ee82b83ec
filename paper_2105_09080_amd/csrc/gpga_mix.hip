// Gossip step with a general sparse weight matrix W (grid, static exponential
// graph, caller-supplied W), Algorithm 1 of the paper with the matrix form of
// App. A:   X_new = W (X - gamma * M'),   M' = mu*M + G.
//
// W is held in compressed-row form: row i lists the neighbours j in N_i and the
// weights w_ij (Sec. 3).  Mixing acts along the node axis only, so a column
// tile of ALL n rows is self-contained:
//
//  * fused tile kernel (the n x 64-lane tile fits in the 160 KiB of LDS a workgroup may
//    have): a workgroup of 8 or 16 wavefronts owns one column tile (64 lanes x 16 or 4
//    bytes; 8 on request).  Phase 1: the waves share the rows, read x, m, g once
//    (coalesced row segments), store the new m and put y = x^(k+1/2) into LDS.  Phase 2:
//    each wave produces its share of output rows as sum_j w_ij y_j from LDS and streams
//    them to x_new.  Every element of x, m, g is read from HBM once and m, x_new written
//    once (20 B per element), exactly like the ring / one-peer stencil kernels.
//  * sliding-window kernel (banded W: every neighbour within a fixed circular distance of
//    its node; any number of rows): the same traffic with only a window of y in LDS.
//  * two-pass path (anything else): pass 1 is the elementwise local update (the W = I
//    walk of the stencil kernel), which writes y over the old iterate x (dead once y
//    exists: that array is the target of the next step); pass 2 is the sparse product
//    x_new = W y with workgroups ordered so that all rows of a column tile run together
//    and re-reads of y hit the caches (28 B per element of HBM traffic when they do).
#include <type_traits>

#include "gpga_internal.hpp"
#include "gpga_pace.hpp"
#include "gpga_spread.hpp"

namespace {

template <typename T>
__device__ __forceinline__ T ld_stream(const T* p) {
    return __builtin_nontemporal_load(p);
}
template <typename T>
__device__ __forceinline__ void st_stream(T* p, T v) {
    __builtin_nontemporal_store(v, p);
}

// x^(k+1/2) from x, g and the new momentum value (MOM: 0 none, 1 heavy-ball, 2 Nesterov).
template <int MOM, typename T>
__device__ __forceinline__ T half_step(const T& xv, const T& gv, const T& mom, float lr, float mu) {
    if (MOM == 2) return xv - lr * (gv + mu * mom);
    return xv - lr * mom;
}

struct CsrDev {
    const int32_t* ptr;
    const int32_t* col;
    const float* val;
};

struct TileArgs {
    StepGeom ge;
    CsrDev w;
    int64_t tiles;  // column tiles; workgroups stride over them
    int32_t nnz;    // entries of W (the LDS copy needs the count)
    double* spread_partials;  // TRACE kernels: one sum of squared deviations per workgroup (nullptr: not wanted)
    PaceArgs pace;
};

constexpr int kTileWavesDefault = 4;
constexpr int kTileWavesMax = 16;
constexpr int kTileUnroll = 2;  // rows per wavefront and batch in phase 1: 1, 2, 4 and 8 measure within the spread between
                                // buffer placements of each other (5.2-5.9 TB/s on n = 64 and 128), 2 most often ahead
// Largest tile (n rows x 64 lanes) the whole-tile kernel stages: what the device grants one workgroup
// (160 KiB on gfx950) unless the "mix_tile_kb" option asks for less.
inline size_t tile_lds_cap(const gpga_ctx* c) {
    const size_t most = (size_t)c->max_lds_block;
    if (c->opt_mix_tile_kb <= 0) return most;
    const size_t want = (size_t)c->opt_mix_tile_kb * 1024;
    return want < most ? want : most;
}
constexpr size_t kTileCsrLdsBytes = 16 * 1024;  // largest W copied into LDS (two workgroups per CU still fit)

// LCSR: W is copied into LDS behind the tile once per workgroup and phase 2 reads it from
// there.  Vector memory operations of a wavefront retire in order, so a neighbour list
// fetched from global memory inside the output loop would make every output row wait for
// the stores of the rows before it; LDS reads are counted separately and leave the stores
// streaming.
// TRACE: the kernel also leaves, per workgroup, the sum over the columns of its tiles of
// sum_i (x_new[i] - column mean)^2: every wavefront keeps shifted fp64 sums of the rows it
// stores, the wavefronts' sums meet in LDS once the tile's y is no longer needed, and the
// workgroup adds up its tiles in the order it takes them.
template <typename T, int MOM, bool LCSR, bool TRACE>
__global__ void __launch_bounds__(kWave* kTileWavesMax) k_step_tile(const TileArgs a) {
    constexpr int V = sizeof(T) / sizeof(float);
    extern __shared__ __align__(16) unsigned char s_raw[];
    T* __restrict__ sy = reinterpret_cast<T*>(s_raw);  // [n][kWave]

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int kTileWaves = blockDim.x >> 6;
    const int n = a.ge.n;
    // LDS copy of W: row pointers (n + 1, padded to an even count), columns, weights
    int32_t* __restrict__ s_ptr = reinterpret_cast<int32_t*>(s_raw + (size_t)n * kWave * sizeof(T));
    int32_t* __restrict__ s_col = s_ptr + ((n + 2) & ~1);
    float* __restrict__ s_val = reinterpret_cast<float*>(s_col + a.nnz);
    if (LCSR) {  // visible to phase 2 through the barrier that ends the first phase 1
        for (int p = threadIdx.x; p <= n; p += blockDim.x) s_ptr[p] = a.w.ptr[p];
        for (int p = threadIdx.x; p < a.nnz; p += blockDim.x) {
            s_col[p] = a.w.col[p];
            s_val[p] = a.w.val[p];
        }
    }
    const int64_t ldT = a.ge.ld / V;
    const float lr = a.ge.lr, mu = a.ge.mu;
    constexpr uint32_t kLoadUnits = MOM ? 4u : 2u;  // 4-byte streams per row in phase 1 (reads + the m store)
    const PaceRun run = pace_begin(a.pace, lane);
    uint32_t units_done = 0;
    double wg_spread = 0.0;  // TRACE: lane 0 of wavefront 0 adds up the workgroup's tiles

    // Workgroups stride over the column tiles (one tile each in the default one-shot launch).
    // A paced launch has exactly the resident workgroups: they then read the same row group
    // of their tiles at the same time and later store the same output rows.
    for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
        const int64_t col = tile * kWave + lane;
        const bool on = col < a.ge.ncols;

        const T* __restrict__ xp = reinterpret_cast<const T*>(a.ge.x + a.ge.col0) + col;
        const T* __restrict__ gp = reinterpret_cast<const T*>(a.ge.g + a.ge.col0) + col;
        T* __restrict__ mp = MOM ? reinterpret_cast<T*>(a.ge.m + a.ge.col0) + col : nullptr;
        T* __restrict__ xnp = reinterpret_cast<T*>(a.ge.x_new + a.ge.col0) + col;

        // Phase 1: rows wave, wave + W, ... : local update, y into LDS.
        // Whole row groups of a whole tile first, in a loop of their own without lane or row
        // predicates: all the loads of a group are issued back to back before the first use,
        // and nothing makes them wait for the stores of the group before.
        int base = wave;
        if ((tile + 1) * kWave <= a.ge.ncols) {  // every lane has a column
            for (; base + (kTileUnroll - 1) * kTileWaves < n; base += kTileWaves * kTileUnroll) {
                T xv[kTileUnroll], mv[kTileUnroll], gv[kTileUnroll];
                pace_wait(run, units_done);
                units_done += kTileUnroll * kLoadUnits;
#pragma unroll
                for (int u = 0; u < kTileUnroll; ++u) {
                    const int64_t off = (int64_t)(base + u * kTileWaves) * ldT;
                    xv[u] = ld_stream(xp + off);
                    if (MOM) mv[u] = ld_stream(mp + off);
                    gv[u] = ld_stream(gp + off);
                }
#pragma unroll
                for (int u = 0; u < kTileUnroll; ++u) {
                    const int row = base + u * kTileWaves;
                    T mom = gv[u];
                    if (MOM) {
                        mom = mu * mv[u] + gv[u];
                        st_stream(mp + (int64_t)row * ldT, mom);
                    }
                    sy[row * kWave + lane] = half_step<MOM>(xv[u], gv[u], mom, lr, mu);
                }
            }
        }
        // Ragged row groups and the last, partial tile: predicated per row and per lane.
        for (; base < n; base += kTileWaves * kTileUnroll) {
            T xv[kTileUnroll], mv[kTileUnroll], gv[kTileUnroll];
            pace_wait(run, units_done);
            units_done += kTileUnroll * kLoadUnits;
#pragma unroll
            for (int u = 0; u < kTileUnroll; ++u) {
                const int row = base + u * kTileWaves;
                if (row < n && on) {
                    const int64_t off = (int64_t)row * ldT;
                    xv[u] = ld_stream(xp + off);
                    if (MOM) mv[u] = ld_stream(mp + off);
                    gv[u] = ld_stream(gp + off);
                }
            }
#pragma unroll
            for (int u = 0; u < kTileUnroll; ++u) {
                const int row = base + u * kTileWaves;
                if (row < n) {
                    T y = T(0);
                    if (on) {
                        T mom = gv[u];
                        if (MOM) {
                            mom = mu * mv[u] + gv[u];
                            st_stream(mp + (int64_t)row * ldT, mom);
                        }
                        y = half_step<MOM>(xv[u], gv[u], mom, lr, mu);
                    }
                    sy[row * kWave + lane] = y;
                }
            }
        }
        __syncthreads();
        // Phase 2: output rows wave, wave + W, ... from the staged y.  The (j, w_ij) list of
        // a row is fetched with one coalesced load (lane p holds entry p; the next row's list
        // is fetched while this row is being summed) and broadcast entry by entry with
        // readlane; taps are taken four at a time (padding taps have weight 0 and read row 0)
        // so that four LDS reads are in flight.  All lanes stay active: readlane must find
        // every source lane's registers written.
        auto fetch_list = [&](int i, int c0, int& cj, float& wv) {
            cj = 0;
            wv = 0.f;
            if (i < n) {
                const int p = (LCSR ? s_ptr[i] : a.w.ptr[i]) + c0 + lane;
                if (p < (LCSR ? s_ptr[i + 1] : a.w.ptr[i + 1])) {
                    cj = LCSR ? s_col[p] : a.w.col[p];
                    wv = LCSR ? s_val[p] : a.w.val[p];
                }
            }
        };
        int cj_next;
        float wv_next;
        fetch_list(wave, 0, cj_next, wv_next);
        ColumnSpread<T> spread;
        if (TRACE) spread.reset(sy[lane]);  // row 0 of y: a value near every x_new of the column
        for (int i = wave; i < n; i += kTileWaves) {
            const int cnt = LCSR ? __builtin_amdgcn_readfirstlane(s_ptr[i + 1] - s_ptr[i]) : a.w.ptr[i + 1] - a.w.ptr[i];
            int cj_l = cj_next;
            float wv_l = wv_next;
            fetch_list(i + kTileWaves, 0, cj_next, wv_next);
            T acc = T(0);
            for (int c0 = 0; c0 < cnt; c0 += kWave) {
                if (c0 > 0) fetch_list(i, c0, cj_l, wv_l);
                const int m = cnt - c0 < kWave ? cnt - c0 : kWave;
                for (int q = 0; q < m; q += 4) {
#pragma unroll
                    for (int t = 0; t < 4; ++t) {
                        const int cj = __builtin_amdgcn_readlane(cj_l, q + t);
                        const float wv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(wv_l), q + t));
                        acc += wv * sy[cj * kWave + lane];
                    }
                }
            }
            pace_wait(run, units_done);
            units_done += 1u;
            if (on) st_stream(xnp + (int64_t)i * ldT, acc);
            if (TRACE) spread.add(acc);  // lanes without a column hold zeros throughout
        }
        __syncthreads();  // the next tile's phase 1 overwrites the staged y
        if (TRACE) {
            // the wavefronts' sums meet in LDS ([wave][2V][lane] doubles over the y tile, which is
            // no longer needed); wavefront 0 adds them in wavefront order and finishes the columns
            double* __restrict__ sw = reinterpret_cast<double*>(s_raw);
            spread.store(sw + ((size_t)wave * 2 * V) * kWave + lane);
            __syncthreads();
            if (wave == 0) {
                double part = ColumnSpread<T>::finish(sw + lane, kTileWaves, 1.0 / (double)n);
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) part += __shfl_down(part, off, kWave);
                wg_spread += part;
            }
            __syncthreads();
        }
    }
    if (TRACE && a.spread_partials && threadIdx.x == 0) a.spread_partials[blockIdx.x] = wg_spread;
    pace_end(a.pace, run, units_done, lane, pace_now(a.pace));
}

// Banded W (every neighbour within circular distance `band` of its node: rings with more taps, the
// grid / torus, whose neighbours sit at distances 1 and the grid width): a sliding window instead
// of the whole column tile.  The wavefronts of a workgroup take the rows of their column tile in
// order, one row each per batch; y goes into a ring of 2*band + 2*waves rows in LDS, and output
// row i is formed as soon as row i + band has arrived.  Rows 0 .. 2*band-1 of y are also kept
// aside: the first `band` output rows wait for the last rows of the walk, and the last `band`
// output rows wrap round to the first.  Every element of x, m, g is read once and m, x_new
// written once (20 B per element) for any number of rows, LDS holds 4*band + 2*waves rows, and
// the whole chip works on the same few rows at a time (persistent, paced), where the tile kernel
// has every row of every array open at once.
// The neighbour list of an output row (offset and weight, entry p in lane p; a fixed number of
// entries per row, padded with weight 0, so that no row pointer has to be fetched first) travels
// with the row loads of its batch, a few batches ahead; rows may have at most 64 neighbours.
struct BandArgs {
    StepGeom ge;
    const int32_t* off;  // signed circular offsets j - i, K entries per row (padding: offset 0, weight 0)
    const float* val;
    int32_t K;
    int64_t tiles;
    int32_t band;
    int32_t ring_rows;   // 2*band + 2*waves
    double* spread_partials;  // TRACE kernels: one sum of squared deviations per workgroup (nullptr: not wanted)
    PaceArgs pace;
};

constexpr int kBandDepth = 4;    // row batches in flight per wavefront, the one being mixed included
constexpr int kBandTailMax = 8;  // tail output rows per wavefront: 2*band <= kBandTailMax * waves

// TRACE: as in the tile kernel, every wavefront keeps shifted fp64 sums of the rows it stores (all relative
// to y of row 0, which is kept aside anyway), they meet in LDS after the tile's last row, and the workgroup
// leaves the sum over its tiles.
template <typename T, int MOM, bool TRACE>
__global__ void __launch_bounds__(kWave* 8) k_step_band(const BandArgs a) {
    constexpr int V = sizeof(T) / sizeof(float);
    extern __shared__ __align__(16) unsigned char s_raw[];
    T* __restrict__ ring = reinterpret_cast<T*>(s_raw);            // [ring_rows][kWave]
    T* __restrict__ head = ring + (size_t)a.ring_rows * kWave;     // [2*band][kWave]: y of the first rows
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int NW = blockDim.x >> 6;
    const int n = a.ge.n, band = a.band, RB = a.ring_rows;
    const int64_t ldT = a.ge.ld / V;
    const float lr = a.ge.lr, mu = a.ge.mu;
    constexpr uint32_t kRowUnits = MOM ? 5u : 3u;
    const PaceRun run = pace_begin(a.pace, lane);
    uint32_t units_done = 0;
    const int nb = (n + NW - 1) / NW;  // batches of NW rows
    double wg_spread = 0.0;            // TRACE: lane 0 of wavefront 0 adds up the workgroup's tiles

    struct Row {
        T xv, mv, gv;
    };
    struct Taps {  // neighbour list of one output row: entry p in lane p
        int off;
        float val;
        int cnt;
    };

    for (int64_t tile = blockIdx.x; tile < a.tiles; tile += gridDim.x) {
        const int64_t col = tile * kWave + lane;
        const bool on = col < a.ge.ncols;
        const T* __restrict__ xp = reinterpret_cast<const T*>(a.ge.x + a.ge.col0) + col;
        const T* __restrict__ gp = reinterpret_cast<const T*>(a.ge.g + a.ge.col0) + col;
        T* __restrict__ mp = MOM ? reinterpret_cast<T*>(a.ge.m + a.ge.col0) + col : nullptr;
        T* __restrict__ xnp = reinterpret_cast<T*>(a.ge.x_new + a.ge.col0) + col;

        auto load_row = [&](Row& r, int row) {  // row is the same for the whole wavefront
            if (row < n && on) {
                const int64_t o = (int64_t)row * ldT;
                r.xv = ld_stream(xp + o);
                if (MOM) r.mv = ld_stream(mp + o);
                r.gv = ld_stream(gp + o);
            }
        };
        auto load_taps = [&](Taps& t, int i) {  // i uniform; rows outside [0, n) have no taps
            t.off = 0;
            t.val = 0.f;
            t.cnt = 0;
            if (i >= 0 && i < n) {
                t.cnt = a.K;
                if (lane < a.K) {
                    t.off = a.off[(int64_t)i * a.K + lane];
                    t.val = a.val[(int64_t)i * a.K + lane];
                }
            }
        };
        // sum_j w_ij y_j for output row i; `fetch(j)` returns y of (unwrapped) row i + offset
        auto mix = [&](const Taps& t, auto fetch) -> T {
            T acc = T(0);
            const int cnt = __builtin_amdgcn_readfirstlane(t.cnt);
            for (int q = 0; q < cnt; ++q) {
                const int dj = __builtin_amdgcn_readlane(t.off, q);
                const float wv = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(t.val), q));
                acc += wv * fetch(dj);
            }
            return acc;
        };

        // neighbour lists of this wavefront's tail rows (the last `band` and the first `band` output rows),
        // fetched before anything else of the tile
        Taps tail[kBandTailMax];
#pragma unroll
        for (int m = 0; m < kBandTailMax; ++m) {
            const int k = wave + m * NW;  // k < band: output row n - band + k;  band <= k < 2*band: output row k - band
            load_taps(tail[m], k < band ? n - band + k : (k < 2 * band ? k - band : -1));
        }

        // Rows and neighbour lists run kBandDepth - 1 batches ahead of the batch being mixed: a batch ends
        // in a workgroup barrier, and with a single batch of look-ahead every barrier exposed one memory
        // latency (measured: 2.8 us per batch whatever the pacing rate).  The buffers rotate through a loop
        // unrolled kBandDepth times, so every index is a constant.
        Row rows[kBandDepth];
        Taps taps[kBandDepth];
        ColumnSpread<T> spread;
        // HOT: nothing in the batch is conditional (whole tile, whole batches, every wavefront has an output
        // row whose window lies inside the walk).  Only then can the wait for a batch's data leave exactly the
        // younger loads and stores outstanding; a store under a condition makes that count uncertain and the
        // wait falls back to "everything", which empties the pipeline.
        auto fetch_batch = [&](auto hot, Row& r, Taps& tp, int t) {  // batch t: row t*NW + wave and the list of its output row
            constexpr bool HOT = decltype(hot)::value;
            if (HOT) {
                const int row = t * NW + wave;
                const int64_t e = (int64_t)(row - band) * a.K + (lane < a.K ? lane : 0);
                tp.off = a.off[e];
                tp.val = a.val[e];
                tp.cnt = a.K;
                pace_wait(run, units_done);
                units_done += kRowUnits;
                const int64_t o = (int64_t)row * ldT;
                r.xv = ld_stream(xp + o);
                if (MOM) r.mv = ld_stream(mp + o);
                r.gv = ld_stream(gp + o);
            } else if (t < nb) {
                load_taps(tp, t * NW + wave - band);
                pace_wait(run, units_done);
                units_done += kRowUnits;
                load_row(r, t * NW + wave);
            }
        };
        int sb = 0;  // ring slot of the first row of the current batch: (t * NW) mod RB
        auto batch = [&](auto hot, const Row& cur, const Taps& tp, Row& ahead_r, Taps& ahead_t, int t) {
            constexpr bool HOT = decltype(hot)::value;
            fetch_batch(hot, ahead_r, ahead_t, t + kBandDepth - 1);
            __builtin_amdgcn_sched_barrier(0);  // keep the issue order: loads, then stores
            const int row = t * NW + wave;
            if (HOT || row < n) {
                T y = T(0);
                if (HOT || on) {
                    T mom = cur.gv;
                    if (MOM) {
                        mom = mu * cur.mv + cur.gv;
                        st_stream(mp + (int64_t)row * ldT, mom);
                    }
                    y = half_step<MOM>(cur.xv, cur.gv, mom, lr, mu);
                }
                int slot = sb + wave;
                if (slot >= RB) slot -= RB;
                ring[slot * kWave + lane] = y;
                if (!HOT && row < 2 * band) head[row * kWave + lane] = y;
            }
            __syncthreads();  // rows < (t + 1) * NW are in the ring
            if (TRACE && !HOT && t == 0) spread.reset(head[lane]);  // y of row 0: no output row precedes this point
            const int i = row - band;  // this wavefront's output row: its window ends at row i + band = row
            if (HOT || (i >= band && row < n)) {
                const T acc = mix(tp, [&](int dj) -> T {
                    int slot = sb + wave - band + dj;  // in [-2*band, RB + NW)
                    if (slot < 0) slot += RB;
                    if (slot >= RB) slot -= RB;
                    return ring[slot * kWave + lane];
                });
                if (HOT || on) st_stream(xnp + (int64_t)i * ldT, acc);
                if (TRACE) spread.add(acc);  // lanes without a column hold zeros throughout
            }
            sb += NW;
            if (sb >= RB) sb -= RB;
        };
        const bool whole_tile = (tile + 1) * kWave <= a.ge.ncols;
        const int nb_full = n / NW;                        // batches whose rows all exist
        const int t_hot = (2 * band + NW - 1) / NW;        // from this batch on every wavefront has an output row
#pragma unroll
        for (int j = 0; j < kBandDepth - 1; ++j) fetch_batch(std::false_type{}, rows[j], taps[j], j);
        // all kBandDepth batches of a hot round, and the batches they fetch ahead, are whole and past the start
        auto is_hot = [&](int t0) { return whole_tile && t0 >= t_hot && t0 + 2 * kBandDepth - 2 < nb_full; };
        for (int t0 = 0; t0 < nb;) {
            if (is_hot(t0)) {
                // consecutive hot rounds form a loop of their own: its only other predecessor is itself, so the
                // outstanding loads and stores are known exactly at every wait from the second round on
                do {
#pragma unroll
                    for (int j = 0; j < kBandDepth; ++j)
                        batch(std::true_type{}, rows[j], taps[j], rows[(j + kBandDepth - 1) % kBandDepth],
                              taps[(j + kBandDepth - 1) % kBandDepth], t0 + j);
                    t0 += kBandDepth;
                } while (is_hot(t0));
            } else {
#pragma unroll
                for (int j = 0; j < kBandDepth; ++j) {
                    if (t0 + j >= nb) break;
                    batch(std::false_type{}, rows[j], taps[j], rows[(j + kBandDepth - 1) % kBandDepth],
                          taps[(j + kBandDepth - 1) % kBandDepth], t0 + j);
                }
                t0 += kBandDepth;
            }
        }
        // Tail: output rows n - band .. n - 1 wrap round to the first rows of y (kept aside), output rows
        // 0 .. band - 1 reach back to the last rows of the walk (still in the ring).
        const int sb_last = sb - NW;           // may be negative: slot of row (nb - 1) * NW, modulo RB
        const int row_last0 = (nb - 1) * NW;   // the row that slot belongs to
        auto ring_row = [&](int r) -> T {      // r in [n - 2*band, n)
            int slot = sb_last + (r - row_last0);
            while (slot < 0) slot += RB;
            if (slot >= RB) slot -= RB;
            return ring[slot * kWave + lane];
        };
#pragma unroll
        for (int m = 0; m < kBandTailMax; ++m) {
            const int k = wave + m * NW;
            if (k >= 2 * band) break;
            const int i = k < band ? n - band + k : k - band;
            const T acc = mix(tail[m], [&](int dj) -> T {
                const int j = i + dj;
                if (j >= n) return head[(j - n) * kWave + lane];
                if (j < 0) return ring_row(j + n);
                return k < band ? ring_row(j) : head[j * kWave + lane];
            });
            if (on) st_stream(xnp + (int64_t)i * ldT, acc);
            if (TRACE) spread.add(acc);
        }
        __syncthreads();  // the next tile overwrites the ring and the kept rows
        if (TRACE) {      // the wavefronts' sums meet where the ring was
            double* __restrict__ sw = reinterpret_cast<double*>(s_raw);
            spread.store(sw + ((size_t)wave * 2 * V) * kWave + lane);
            __syncthreads();
            if (wave == 0) {
                double part = ColumnSpread<T>::finish(sw + lane, NW, 1.0 / (double)n);
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) part += __shfl_down(part, off, kWave);
                wg_spread += part;
            }
            __syncthreads();
        }
    }
    if (TRACE && a.spread_partials && threadIdx.x == 0) a.spread_partials[blockIdx.x] = wg_spread;
    pace_end(a.pace, run, units_done, lane, pace_now(a.pace));
}

// Two-pass path, pass 2: x_new[i, :] = sum_j w_ij y[j, :].  One workgroup = 256 / LANES consecutive
// rows of one column tile of LANES lanes.  Workgroup ids are dealt to the 8 XCDs round-robin, each
// with its own L2; the id is remapped so that all rows of a tile run on ONE XCD, in row order: the
// y rows a tile needs are then fetched into that L2 once and re-read from it by the neighbouring
// rows.  That only works while the tile's y (n x LANES x lane bytes) is well below the 4 MiB of an
// L2, so tiles get narrower as n grows.
template <typename T, int LANES>
__global__ void __launch_bounds__(256) k_spmm_rows(const float* __restrict__ y, float* __restrict__ x_new,
                                                   int64_t ld, int64_t col0, int64_t ncols, int32_t n,
                                                   int64_t tiles, const CsrDev w) {
    constexpr int V = sizeof(T) / sizeof(float);
    constexpr int R = 256 / LANES;                   // rows per workgroup
    const int64_t ldT = ld / V;
    const int64_t bid = blockIdx.x;
    const int64_t ng = (n + R - 1) / R;              // row groups per tile
    const int64_t full = (tiles >> 3) << 3;          // tiles covered by whole groups of 8
    int64_t tile;
    int g;
    if (bid < full * ng) {
        const int64_t slot = bid >> 3;               // position within this XCD's queue
        tile = (slot / ng) * 8 + (bid & 7);
        g = (int)(slot % ng);
    } else {                                         // ragged tail: plain order
        const int64_t r = bid - full * ng;
        tile = full + r / ng;
        g = (int)(r % ng);
    }
    // a row per wavefront or more: the row index is uniform in a wavefront (scalar loads of the neighbour list)
    const int i = g * R + __builtin_amdgcn_readfirstlane((int)(threadIdx.x / LANES));
    const int64_t col = tile * LANES + (threadIdx.x % LANES);
    if (col >= ncols || i >= n) return;
    const T* __restrict__ yb = reinterpret_cast<const T*>(y + col0) + col;
    const int p0 = w.ptr[i], p1 = w.ptr[i + 1];
    T acc = T(0);
    for (int p = p0; p < p1; ++p) acc += w.val[p] * yb[(int64_t)w.col[p] * ldT];
    st_stream(reinterpret_cast<T*>(x_new + col0) + col + (int64_t)i * ldT, acc);
}

template <typename T, int LANES>
hipError_t launch_spmm(const gpga_ctx* c, const StepGeom& ge, const CsrDev& w) {
    const int64_t tiles = (ge.ncols + LANES - 1) / LANES;
    const int64_t ng = ((int64_t)ge.n + 256 / LANES - 1) / (256 / LANES);
    if (tiles * ng > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((k_spmm_rows<T, LANES>), dim3((unsigned)(tiles * ng)), dim3(256), 0, c->stream, ge.x, ge.x_new,
                       ge.ld, ge.col0, ge.ncols, ge.n, tiles, w);
    return hipGetLastError();
}

// Fused consensus sums: one partial per workgroup, if the context's partial-sum array (handed in one slot
// past its start) has room for them; otherwise the kernel keeps its sums to itself and the caller, who finds
// *spread_count still 0, takes the separate reduction pass.
inline bool spread_slots_fit(const gpga_ctx* c, int64_t blocks) { return blocks + 1 <= (int64_t)c->partials_cap; }

template <typename T, int MOM, bool LCSR, bool TRACE>
hipError_t launch_tile_mom(const gpga_ctx* c, TileArgs a, int waves, size_t lds, int64_t* spread_count) {
    const int threads = kWave * waves;
    int64_t blocks = a.tiles;
    pace_setup(nullptr, 0.0, 0, 0.0, 0, &a.pace);
    // Large problems: exactly the resident workgroups, striding over the tiles and paced at the rate the
    // controller of this kind of launch has found: all workgroups then read the same row group of their
    // tiles at the same time and later store the same output rows, so the chip alternates between a pure
    // read phase and a pure write phase over a few rows at a time.  Small problems, or pacing switched
    // off: one workgroup per tile.
    const bool big = (int64_t)c->n * c->d * 4 >= kPaceMinBytes && sizeof(T) >= 8;
    const double gbs = c->opt_pace_gbs > 0 ? (double)c->opt_pace_gbs : (c->opt_pace_gbs < 0 && big ? -1.0 : 0.0);
    const int want = c->opt_blocks_per_cu < 0 ? (gbs != 0.0 ? 32 : 0) : c->opt_blocks_per_cu;
    if (lds > 48 * 1024) {  // per instantiation and device: allow more than the default 64 KiB of dynamic LDS
        static bool attr_set[64] = {false};
        const int dev = c->device >= 0 && c->device < 64 ? c->device : 0;
        if (!attr_set[dev]) {
            const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_step_tile<T, MOM, LCSR, TRACE>),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->max_lds_block);
            if (e != hipSuccess) return e;
            attr_set[dev] = true;
        }
    }
    if (want > 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_step_tile<T, MOM, LCSR, TRACE>, threads, lds) != hipSuccess || occ < 1)
            occ = 1;
        const int64_t resident = (int64_t)c->num_cus * (want < occ ? want : occ);
        if (resident < blocks) blocks = balanced_blocks(a.tiles, resident);
        pace_setup(const_cast<gpga_ctx*>(c), gbs, PACE_TILE, (double)blocks * waves, (int)sizeof(T), &a.pace);
    }
    if (TRACE) {
        if (spread_count && a.spread_partials && spread_slots_fit(c, blocks)) *spread_count = blocks;
        else a.spread_partials = nullptr;
    }
    hipLaunchKernelGGL((k_step_tile<T, MOM, LCSR, TRACE>), dim3((unsigned)blocks), dim3(threads), lds, c->stream, a);
    return hipGetLastError();
}

template <typename T, bool TRACE>
hipError_t launch_tile_traced(const gpga_ctx* c, const TileArgs& a, int waves, size_t lds, bool lcsr, int mom,
                              int64_t* spread_count) {
    if (lcsr) {
        if (mom == 2) return launch_tile_mom<T, 2, true, TRACE>(c, a, waves, lds, spread_count);
        return mom == 1 ? launch_tile_mom<T, 1, true, TRACE>(c, a, waves, lds, spread_count)
                        : launch_tile_mom<T, 0, true, TRACE>(c, a, waves, lds, spread_count);
    }
    if (mom == 2) return launch_tile_mom<T, 2, false, TRACE>(c, a, waves, lds, spread_count);
    return mom == 1 ? launch_tile_mom<T, 1, false, TRACE>(c, a, waves, lds, spread_count)
                    : launch_tile_mom<T, 0, false, TRACE>(c, a, waves, lds, spread_count);
}

template <typename T>
hipError_t launch_tile(const gpga_ctx* c, const StepGeom& ge, const CsrDev& w, int mom,
                       double* spread_partials = nullptr, int64_t* spread_count = nullptr) {
    c->note_path(PATH_TILE, (int)sizeof(T));
    TileArgs a;
    a.ge = ge;
    a.w = w;
    a.tiles = (ge.ncols + kWave - 1) / kWave;
    a.spread_partials = nullptr;
    if (a.tiles > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    a.nnz = (int32_t)c->csr.col.size();
    const size_t tile_lds = (size_t)ge.n * kWave * sizeof(T);
    // W rides along in LDS when it is small and the device grants the workgroup the room
    const size_t csr_lds = ((((size_t)ge.n + 2) & ~(size_t)1) + 2 * (size_t)a.nnz) * sizeof(int32_t);
    const bool lcsr = c->opt_mix_csr_lds != 0 && csr_lds <= kTileCsrLdsBytes && tile_lds + csr_lds <= (size_t)c->max_lds_block;
    // measured on the n = 64, d = 25.6M shape: 8 or 16 wavefronts per workgroup stream
    // 5.2-6.0 TB/s, 4 wavefronts 4.8-5.1 TB/s (more rows are in flight while others mix).  A tile of
    // more than 64 KiB leaves room for one workgroup per compute unit, which then needs all 16
    // wavefronts (n = 256: 4.6 against 3.7 TB/s with 8, n = 512: 3.6 against 2.6).
    const int waves = c->opt_mix_waves ? c->opt_mix_waves
                                       : (tile_lds > 64 * 1024 || ge.n > 160 ? kTileWavesMax : (ge.n >= 32 ? 8 : kTileWavesDefault));
    size_t lds = tile_lds + (lcsr ? csr_lds : 0);
    if (spread_partials && spread_count) {
        // the consensus sums ride along: the wavefronts' sums meet in waves x 2V x 64 doubles of the tile's LDS
        const size_t meet = (size_t)waves * 2 * (sizeof(T) / sizeof(float)) * kWave * sizeof(double);
        if (meet <= tile_lds) {
            a.spread_partials = spread_partials;
            return launch_tile_traced<T, true>(c, a, waves, lds, lcsr, mom, spread_count);
        }
    }
    return launch_tile_traced<T, false>(c, a, waves, lds, lcsr, mom, nullptr);
}

template <typename T>
hipError_t launch_two_pass(const gpga_ctx* c, const StepGeom& ge, const CsrDev& w, int vec) {
    c->note_path(PATH_TWO_PASS, (int)sizeof(T));
    // pass 1: the W = I walk of the stencil kernel, storing y = x^(k+1/2) over the old iterate
    hipError_t e = launch_step_walk(c, ge, MODE_INPLACE, 0, vec);
    if (e != hipSuccess) return e;
    // tile width: y of all rows of a tile should take a fraction of an L2 (4 MiB)
    const size_t row_bytes = (size_t)ge.n * sizeof(T);
    const int lanes = c->opt_mix_spmm_lanes ? c->opt_mix_spmm_lanes : (row_bytes * 256 <= (1u << 20) ? 256 : row_bytes * 128 <= (1u << 20) ? 128 : 64);
    if (lanes == 256) return launch_spmm<T, 256>(c, ge, w);
    if (lanes == 128) return launch_spmm<T, 128>(c, ge, w);
    return launch_spmm<T, 64>(c, ge, w);
}

// Whether the banded kernel can take this W, and with which lane type: the ring of 2*band + 2*waves rows
// plus the 2*band kept rows must fit in LDS (at least two workgroups per compute unit), the window must
// not overlap itself (n >= 4*band), and the tail rows must fit the per-wavefront lists.
template <typename T, int MOM, bool TRACE>
hipError_t launch_band_mom(const gpga_ctx* c, BandArgs a, int waves, size_t lds, int64_t* spread_count) {
    const int threads = kWave * waves;
    int64_t blocks = a.tiles;
    pace_setup(nullptr, 0.0, 0, 0.0, 0, &a.pace);
    const bool big = (int64_t)c->n * c->d * 4 >= kPaceMinBytes;
    const double gbs = c->opt_pace_gbs > 0 ? (double)c->opt_pace_gbs : (c->opt_pace_gbs < 0 && big ? -1.0 : 0.0);
    const int want = c->opt_blocks_per_cu < 0 ? (big || gbs != 0.0 ? 32 : 0) : c->opt_blocks_per_cu;
    // per instantiation and device: allow more than the default 64 KiB of dynamic LDS (setting it twice is harmless)
    static bool attr_set[64] = {false};
    const int dev = c->device >= 0 && c->device < 64 ? c->device : 0;
    if (!attr_set[dev] && lds > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(&k_step_band<T, MOM, TRACE>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)c->max_lds_block);
        if (e != hipSuccess) return e;
        attr_set[dev] = true;
    }
    if (want > 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_step_band<T, MOM, TRACE>, threads, lds) != hipSuccess || occ < 1) occ = 1;
        const int64_t resident = (int64_t)c->num_cus * (want < occ ? want : occ);
        if (resident < blocks) blocks = balanced_blocks(a.tiles, resident);
        pace_setup(const_cast<gpga_ctx*>(c), gbs, PACE_BAND, (double)blocks * waves, (int)sizeof(T), &a.pace);
    }
    if (TRACE) {
        if (spread_count && a.spread_partials && spread_slots_fit(c, blocks)) *spread_count = blocks;
        else a.spread_partials = nullptr;
    }
    hipLaunchKernelGGL((k_step_band<T, MOM, TRACE>), dim3((unsigned)blocks), dim3(threads), lds, c->stream, a);
    return hipGetLastError();
}

template <typename T, bool TRACE>
hipError_t launch_band_traced(const gpga_ctx* c, const BandArgs& a, int waves, size_t lds, int mom, int64_t* spread_count) {
    if (mom == 2) return launch_band_mom<T, 2, TRACE>(c, a, waves, lds, spread_count);
    return mom == 1 ? launch_band_mom<T, 1, TRACE>(c, a, waves, lds, spread_count)
                    : launch_band_mom<T, 0, TRACE>(c, a, waves, lds, spread_count);
}

template <typename T>
hipError_t launch_band(const gpga_ctx* c, const StepGeom& ge, int mom, int waves, double* spread_partials,
                       int64_t* spread_count) {
    c->note_path(PATH_BAND, (int)sizeof(T));
    BandArgs a;
    a.ge = ge;
    a.off = c->csr_off_d;
    a.val = c->csr_ellval_d;
    a.K = c->csr_max_row;
    a.tiles = (ge.ncols + kWave - 1) / kWave;
    a.band = c->csr_band;
    a.ring_rows = 2 * c->csr_band + 2 * waves;
    a.spread_partials = nullptr;
    if (a.tiles > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    const size_t lds = (size_t)(a.ring_rows + 2 * c->csr_band) * kWave * sizeof(T);
    if (spread_partials && spread_count) {
        // the wavefronts' consensus sums meet in waves x 2V x 64 doubles where the ring was
        const size_t meet = (size_t)waves * 2 * (sizeof(T) / sizeof(float)) * kWave * sizeof(double);
        a.spread_partials = spread_partials;
        return launch_band_traced<T, true>(c, a, waves, lds < meet ? meet : lds, mom, spread_count);
    }
    return launch_band_traced<T, false>(c, a, waves, lds, mom, nullptr);
}

// 0 = W does not qualify, else the lane bytes (16, 8 or 4) the banded kernel would run with.
int band_lane_bytes(const gpga_ctx* c, int vec, int waves) {
    const int band = c->csr_band;
    if (band < 1 || c->csr_max_row > kWave || c->n < 4 * band || 2 * band > kBandTailMax * waves || !c->csr_off_d) return 0;
    const size_t rows = (size_t)(4 * band + 2 * waves);
    const size_t budget = (size_t)c->max_lds_block / 2;  // two workgroups per compute unit
    const int cap = vec == 4 ? (c->opt_mix_lane_bytes ? c->opt_mix_lane_bytes : 16) : 4;
    for (int bytes = cap; bytes >= 4; bytes /= 2)
        if (rows * kWave * (size_t)bytes <= budget) return bytes;
    return 0;
}

}  // namespace

hipError_t launch_step_csr(const gpga_ctx* c, const StepGeom& ge, int vec, double* spread_partials,
                           int64_t* spread_count) {
    if (spread_count) *spread_count = 0;
    if (ge.ncols <= 0) return hipSuccess;
    if (!c->csr_ready) return hipErrorInvalidValue;
    const CsrDev w{c->csr_ptr_d, c->csr_col_d, c->csr_val_d};
    const int mom = c->mu != 0.f ? (c->nesterov ? 2 : 1) : 0;
    const size_t n = (size_t)ge.n;
    const bool two_pass = c->opt_mix_two_pass == 1;
    const size_t lane_cap = c->opt_mix_lane_bytes ? (size_t)c->opt_mix_lane_bytes : 16;
    // Which kernel (rates measured on 1.6e9 elements, static exponential graph and grid, medians over
    // re-allocated buffers):
    //  * the whole tile with 16-byte lanes where it fits (n <= 160 with 160 KiB of LDS): n = 128 5.6-5.8 TB/s
    //    (8-byte lanes in 64 KiB 4.8, 4-byte lanes 5.4-5.6, the banded kernel 5.0); it also fuses the
    //    consensus trace;
    //  * banded W on more rows: the sliding-window kernel (grid, n = 256 / 512 / 1024: 5.7 / 5.2 / 5.8 TB/s;
    //    the whole tile with 4-byte lanes 5.3 / 4.0 / -);
    //  * any other W whose tile fits with 4-byte lanes (n <= 640): the whole tile, 16 wavefronts (static
    //    exponential graph, n = 256 / 512: 4.6 / 3.6 TB/s; 8-byte lanes are no faster; two passes 3.4 / 3.4);
    //  * else two passes.
    const bool big = (int64_t)c->n * c->d * 4 >= kPaceMinBytes;
    const size_t cap = tile_lds_cap(c);
    const bool wide_tile_fits = n * kWave * sizeof(v4f) <= cap && lane_cap >= 16 && vec == 4;
    const int band_waves = 8;
    const int band_bytes = (!two_pass && c->opt_mix_band != 0 && (c->opt_mix_band == 1 || (big && !wide_tile_fits)))
                               ? band_lane_bytes(c, vec, band_waves) : 0;
    if (band_bytes) {
        StepGeom g2 = ge;
        if (vec == 4 && band_bytes == 16) return launch_band<v4f>(c, ge, mom, band_waves, spread_partials, spread_count);
        if (vec == 4 && band_bytes == 8) {
            g2.ncols = ge.ncols * 2;
            return launch_band<v2f>(c, g2, mom, band_waves, spread_partials, spread_count);
        }
        if (vec == 4) g2.ncols = ge.ncols * 4;
        return launch_band<float>(c, g2, mom, band_waves, spread_partials, spread_count);
    }
    if (vec == 4) {
        // 16-byte aligned rows also satisfy the narrower lane types.  8-byte lanes only on request
        // ("mix_lane_bytes" = 8): they were the slowest of the three wherever two of them fit.
        StepGeom g2 = ge;
        if (!two_pass && lane_cap >= 16 && n * kWave * sizeof(v4f) <= cap)
            return launch_tile<v4f>(c, ge, w, mom, spread_partials, spread_count);
        if (!two_pass && lane_cap == 8 && n * kWave * sizeof(v2f) <= cap) {
            g2.ncols = ge.ncols * 2;
            return launch_tile<v2f>(c, g2, w, mom, spread_partials, spread_count);
        }
        if (!two_pass && n * kWave * sizeof(float) <= cap) {
            g2.ncols = ge.ncols * 4;
            return launch_tile<float>(c, g2, w, mom, spread_partials, spread_count);
        }
        return launch_two_pass<v4f>(c, ge, w, 4);
    }
    if (!two_pass && n * kWave * sizeof(float) <= cap) return launch_tile<float>(c, ge, w, mom, spread_partials, spread_count);
    return launch_two_pass<float>(c, ge, w, 1);
}
