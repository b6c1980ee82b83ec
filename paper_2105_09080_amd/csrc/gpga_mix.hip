// Gossip step with a general sparse weight matrix W (grid, static exponential
// graph, caller-supplied W), Algorithm 1 of the paper with the matrix form of
// App. A:   X_new = W (X - gamma * M'),   M' = mu*M + G.
//
// W is held in compressed-row form: row i lists the neighbours j in N_i and the
// weights w_ij (Sec. 3).  Mixing acts along the node axis only, so a column
// tile of ALL n rows is self-contained:
//
//  * fused tile kernel (n*tile bytes fit in 64 KiB of LDS): a workgroup of four
//    wavefronts owns one column tile (64 lanes x 16 / 8 / 4 bytes).  Phase 1: the
//    waves share the rows, read x, m, g once (coalesced row segments), store the
//    new m and put y = x^(k+1/2) into LDS.  Phase 2: each wave produces its share
//    of output rows as sum_j w_ij y_j from LDS and streams them to x_new.  Every
//    element of x, m, g is read from HBM once and m, x_new written once (20 B per
//    element), exactly like the ring / one-peer stencil kernels.
//  * two-pass path (more rows than LDS can hold): pass 1 is the elementwise local
//    update (the W = I walk of the stencil kernel), which writes y over the old
//    iterate x (dead once y exists: that array is the target of the next step);
//    pass 2 is the sparse product x_new = W y with workgroups ordered so that
//    all rows of a column tile run together and re-reads of y hit the caches
//    (28 B per element of HBM traffic when they do).
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
    double* spread_partials;  // TRACE kernels: one sum of squared deviations per column tile
    PaceArgs pace;
};

constexpr int kTileWavesDefault = 4;
constexpr int kTileWavesMax = 16;
constexpr int kTileUnroll = 4;
constexpr size_t kTileLdsBytes = 64 * 1024;
constexpr size_t kTileCsrLdsBytes = 16 * 1024;  // largest W copied into LDS (two workgroups per CU still fit)

// Per-lane spread sums of one wavefront to LDS (stride kWave doubles between the 8 values) ...
__device__ __forceinline__ void tile_spread_store(const ColumnSpread<v4f>& sp, double* dst) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        dst[(size_t)j * kWave] = sp.s1[j];
        dst[(size_t)(4 + j) * kWave] = sp.s2[j];
    }
}
__device__ __forceinline__ void tile_spread_store(const ColumnSpread<v2f>&, double*) {}
__device__ __forceinline__ void tile_spread_store(const ColumnSpread<float>&, double*) {}
// ... and this lane's four columns finished from the sums of all `waves` wavefronts.
template <typename T>
__device__ __forceinline__ double tile_spread_finish(const double* src, int waves, double inv_n) {
    double r = 0.0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        double s1 = 0.0, s2 = 0.0;
        for (int w = 0; w < waves; ++w) {
            s1 += src[((size_t)w * 8 + j) * kWave];
            s2 += src[((size_t)w * 8 + 4 + j) * kWave];
        }
        const double v = s2 - s1 * s1 * inv_n;
        r += v > 0.0 ? v : 0.0;
    }
    return r;
}

// LCSR: W is copied into LDS behind the tile once per workgroup and phase 2 reads it from
// there.  Vector memory operations of a wavefront retire in order, so a neighbour list
// fetched from global memory inside the output loop would make every output row wait for
// the stores of the rows before it; LDS reads are counted separately and leave the stores
// streaming.
// TRACE (16-byte lanes only): the kernel also leaves, per column tile, the sum over its columns
// of sum_i (x_new[i] - column mean)^2: every wavefront keeps shifted fp64 sums of the rows it
// stores, the wavefronts' sums meet in LDS once the tile's y is no longer needed.
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
            // the wavefronts' sums meet in LDS ([wave][8][lane] doubles over the y tile, which is
            // no longer needed); wavefront 0 adds them in wavefront order, finishes the columns
            // and leaves one partial for the tile
            double* __restrict__ sw = reinterpret_cast<double*>(s_raw);
            tile_spread_store(spread, sw + ((size_t)wave * 8) * kWave + lane);
            __syncthreads();
            if (wave == 0) {
                double part = tile_spread_finish<T>(sw + lane, kTileWaves, 1.0 / (double)n);
#pragma unroll
                for (int off = kWave / 2; off > 0; off >>= 1) part += __shfl_down(part, off, kWave);
                if (lane == 0) a.spread_partials[tile] = part;
            }
            __syncthreads();
        }
    }
    pace_end(a.pace, run, units_done, lane, pace_now(a.pace));
}

// Two-pass path, pass 2: x_new[i, :] = sum_j w_ij y[j, :].  One workgroup = one row of one
// column tile (256 lanes).  Workgroup ids are dealt to the 8 XCDs round-robin, each
// with its own L2; the id is remapped so that all rows of a tile run on ONE XCD, in
// row order: the y rows a tile needs are then fetched into that L2 once and re-read
// from it by the neighbouring rows.
template <typename T>
__global__ void __launch_bounds__(256) k_spmm_rows(const float* __restrict__ y, float* __restrict__ x_new,
                                                   int64_t ld, int64_t col0, int64_t ncols, int32_t n,
                                                   int64_t tiles, const CsrDev w) {
    constexpr int V = sizeof(T) / sizeof(float);
    const int64_t ldT = ld / V;
    const int64_t bid = blockIdx.x;
    const int64_t full = (tiles >> 3) << 3;          // tiles covered by whole groups of 8
    int64_t tile;
    int i;
    if (bid < full * n) {
        const int64_t slot = bid >> 3;               // position within this XCD's queue
        tile = (slot / n) * 8 + (bid & 7);
        i = (int)(slot % n);
    } else {                                         // ragged tail: plain order
        const int64_t r = bid - full * n;
        tile = full + r / n;
        i = (int)(r % n);
    }
    const int64_t col = tile * 256 + threadIdx.x;
    if (col >= ncols) return;
    const T* __restrict__ yb = reinterpret_cast<const T*>(y + col0) + col;
    const int p0 = w.ptr[i], p1 = w.ptr[i + 1];
    T acc = T(0);
    for (int p = p0; p < p1; ++p) acc += w.val[p] * yb[(int64_t)w.col[p] * ldT];
    st_stream(reinterpret_cast<T*>(x_new + col0) + col + (int64_t)i * ldT, acc);
}


template <typename T, int MOM, bool LCSR, bool TRACE>
hipError_t launch_tile_mom(const gpga_ctx* c, TileArgs a, int waves, size_t lds) {
    const int threads = kWave * waves;
    int64_t blocks = a.tiles;
    pace_setup(nullptr, 0.0, 0, 0.0, 0, &a.pace);
    // Default: one workgroup per tile.  On request ("pace_gbs" / "blocks_per_cu" options) exactly
    // the resident workgroups, striding over the tiles and paced.  Measured on the n = 64,
    // d = 25.6M shape the paced form is bimodal (5.0-5.1 TB/s at most targets, 5.5-5.7 TB/s at
    // isolated ones) against a steady 5.2-5.3 TB/s one-shot, so it is not the default.
    const double gbs = c->opt_pace_gbs > 0 ? (double)c->opt_pace_gbs : 0.0;
    const int want = c->opt_blocks_per_cu < 0 ? (gbs > 0.0 ? 32 : 0) : c->opt_blocks_per_cu;
    if (want > 0) {
        int occ = 0;
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, k_step_tile<T, MOM, LCSR, TRACE>, threads, lds) != hipSuccess || occ < 1)
            occ = 1;
        const int64_t resident = (int64_t)c->num_cus * (want < occ ? want : occ);
        if (resident < blocks) blocks = resident;
        pace_setup(const_cast<gpga_ctx*>(c), gbs, PACE_TILE, (double)blocks * waves, (int)sizeof(T), &a.pace);
    }
    hipLaunchKernelGGL((k_step_tile<T, MOM, LCSR, TRACE>), dim3((unsigned)blocks), dim3(threads), lds, c->stream, a);
    return hipGetLastError();
}

template <typename T, bool TRACE>
hipError_t launch_tile_traced(const gpga_ctx* c, const TileArgs& a, int waves, size_t lds, bool lcsr, int mom) {
    if (lcsr) {
        if (mom == 2) return launch_tile_mom<T, 2, true, TRACE>(c, a, waves, lds);
        return mom == 1 ? launch_tile_mom<T, 1, true, TRACE>(c, a, waves, lds) : launch_tile_mom<T, 0, true, TRACE>(c, a, waves, lds);
    }
    if (mom == 2) return launch_tile_mom<T, 2, false, TRACE>(c, a, waves, lds);
    return mom == 1 ? launch_tile_mom<T, 1, false, TRACE>(c, a, waves, lds) : launch_tile_mom<T, 0, false, TRACE>(c, a, waves, lds);
}

template <typename T>
hipError_t launch_tile(const gpga_ctx* c, const StepGeom& ge, const CsrDev& w, int mom,
                       double* spread_partials = nullptr, int64_t* spread_count = nullptr) {
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
    // 5.2-6.0 TB/s, 4 wavefronts 4.8-5.1 TB/s (more rows are in flight while others mix)
    const int waves = c->opt_mix_waves ? c->opt_mix_waves : (ge.n >= 32 ? 8 : kTileWavesDefault);
    size_t lds = tile_lds + (lcsr ? csr_lds : 0);
    if constexpr (std::is_same<T, v4f>::value) if (spread_partials && spread_count) {
        // the consensus sums ride along: the wavefronts' sums need waves x 8 x 64 doubles of LDS
        const size_t meet = (size_t)waves * 8 * kWave * sizeof(double);
        size_t tile_part = tile_lds < meet ? meet : tile_lds;
        if (tile_part + (lcsr ? csr_lds : 0) <= (size_t)c->max_lds_block && tile_part == tile_lds) {
            a.spread_partials = spread_partials;
            *spread_count = a.tiles;
            return launch_tile_traced<T, true>(c, a, waves, lds, lcsr, mom);
        }
    }
    return launch_tile_traced<T, false>(c, a, waves, lds, lcsr, mom);
}

template <typename T>
hipError_t launch_two_pass(const gpga_ctx* c, const StepGeom& ge, const CsrDev& w, int vec) {
    // pass 1: the W = I walk of the stencil kernel, storing y = x^(k+1/2) over the old iterate
    hipError_t e = launch_step_walk(c, ge, MODE_INPLACE, 0, vec);
    if (e != hipSuccess) return e;
    const int64_t tiles = (ge.ncols + 255) / 256;
    if (tiles * ge.n > 0x7fffffffLL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL((k_spmm_rows<T>), dim3((unsigned)(tiles * ge.n)), dim3(256), 0, c->stream, ge.x, ge.x_new,
                       ge.ld, ge.col0, ge.ncols, ge.n, tiles, w);
    return hipGetLastError();
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
    if (vec == 4) {
        // widest lane type whose n x 64-lane tile fits in LDS (16-byte aligned rows also
        // satisfy the narrower types)
        StepGeom g2 = ge;
        if (!two_pass && lane_cap >= 16 && n * kWave * sizeof(v4f) <= kTileLdsBytes)
            return launch_tile<v4f>(c, ge, w, mom, spread_partials, spread_count);
        if (!two_pass && lane_cap >= 8 && n * kWave * sizeof(v2f) <= kTileLdsBytes) {
            g2.ncols = ge.ncols * 2;
            return launch_tile<v2f>(c, g2, w, mom);
        }
        if (!two_pass && n * kWave * sizeof(float) <= kTileLdsBytes) {
            g2.ncols = ge.ncols * 4;
            return launch_tile<float>(c, g2, w, mom);
        }
        return launch_two_pass<v4f>(c, ge, w, 4);
    }
    if (!two_pass && n * kWave * sizeof(float) <= kTileLdsBytes) return launch_tile<float>(c, ge, w, mom);
    return launch_two_pass<float>(c, ge, w, 1);
}
