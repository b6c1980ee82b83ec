// Internal declarations shared by the translation units of libgpga.
// Host-side context, launch descriptors and the launcher entry points of each
// kernel family.  Nothing here is part of the public ABI (include/gpga.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "gpga.h"

typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v2f __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;  // gfx950 wavefront width

enum GpgaProblem : int { PROB_NONE = 0, PROB_LSQ, PROB_LOGREG, PROB_LOGREG_VIRTUAL, PROB_SYNTH };

// Mixing stencil along a walk over rows.
enum StencilMode : int {
    MODE_RING = 0,  // (prev + cur + next) / 3
    MODE_PEER = 1,  // (cur + next) / 2
    MODE_SELF = 2,  // cur
    MODE_INPLACE = 3  // cur, stored over the old iterate it was computed from (x_new and g untouched)
};

// A sparse mixing matrix W in compressed-row form: row i lists the nodes j whose
// iterates node i mixes (w_ij > 0) and their weights.
struct HostCsr {
    std::vector<int32_t> ptr;  // n + 1
    std::vector<int32_t> col;
    std::vector<float> val;
};

constexpr int kSmallRunThreads = 1024;   // workgroup of the single-workgroup trajectory kernel
constexpr int kSmallRunPasses = 4;     // (node, sample) pairs a lane group keeps in registers for the next iteration
constexpr int kSmallRunMaxIters = 256;   // iterations per launch (their step sizes travel in the kernel arguments)

enum LrSchedule : int { SCHED_NONE = 0, SCHED_STEP, SCHED_MILESTONES, SCHED_POLY };
constexpr int kMaxMilestones = 16;

struct PaceState;  // gpga_pace.hpp

// Arrays of at least this many bytes (n x d x 4) run the fused step as paced persistent launches.  Measured on
// the ring walk with n = 64: 281 MB (0.3 ms) 4.1 TB/s paced against 4.9 one-shot, 563 MB equal, 1.1 GB 5.3
// against 4.9: a paced launch ends about 100 us after its plan whatever its length.
constexpr int64_t kPaceMinBytes = 512ll << 20;

enum StepPath : int { PATH_NONE = 0, PATH_WALK = 1, PATH_CYCLES = 2, PATH_GLOBAL = 3, PATH_TILE = 4, PATH_BAND = 5,
                      PATH_TWO_PASS = 6, PATH_SMALL_RUN = 7 };

struct gpga_ctx {
    void note_path(int path, int lane_bytes) const {
        if (last_path == PATH_NONE) {
            last_path = path;
            last_lane_bytes = lane_bytes;
        }
    }
    int32_t n = 0;
    int64_t d = 0;
    int32_t topo = 0;
    int64_t H = 0;
    float lr = 0.f, mu = 0.f;
    bool nesterov = false;  // x^(k+1/2) = x - lr*(g + mu*m) instead of x - lr*m
    int64_t k = 0;
    int device = 0;

    // bound buffers (borrowed)
    float* x = nullptr;      // live iterates
    float* x_new = nullptr;  // target of the next step
    const float* x_first = nullptr;  // the array bound as x (tells the two directions of the ping-pong apart)
    float* m = nullptr;
    float* g = nullptr;
    int64_t ld = 0;
    hipStream_t stream = nullptr;
    bool bound = false;

    // attached problem (borrowed data)
    int problem = PROB_NONE;
    const float* feat = nullptr;  // A or features, n x M x d
    const float* tgt = nullptr;   // b or labels, n x M
    int32_t M = 0;
    uint64_t seed = 0;
    float grad_sigma = 0.f;  // sqrt(grad_var)
    float mu_sigma = 0.f;    // sqrt(mu_var)

    // library-owned scratch
    float* coef = nullptr;  // n x B per-sample coefficients / margins
    size_t coef_cap = 0;    // in floats
    double* partials = nullptr;
    size_t partials_cap = 0;  // in doubles
    double* host_scalar = nullptr;  // pinned, 1 double

    // launch geometry overrides (0 = automatic)
    int opt_unroll = 0;
    int opt_waves = 0;
    int opt_row_split = 0;
    int opt_row_lanes = 0;
    int opt_xcd_swizzle = 0;
    int opt_mix_lane_bytes = 0;  // sparse-W tile kernel: widest lane type allowed (0 = automatic, 4, 8, 16)
    // what the most recent step ran as (gpga_query "step_path" ...): written by the launchers
    mutable int last_path = 0;        // StepPath; the vector pass of a step decides, a scalar tail pass does not overwrite it
    mutable int last_paced = 0;       // 1 = that launch was paced
    mutable int last_lane_bytes = 0;  // bytes per lane of that launch (16, 8, 4)
    int last_trace_fused = 0;         // 1 = the step kernel itself produced the consensus sums of the trace entry
    int opt_mix_spmm_lanes = 0;  // two-pass sparse W, pass 2: lanes per column tile (0 = automatic, 64, 128, 256)
    int opt_mix_tile_kb = 0;     // sparse-W tile kernel: largest tile in KiB of LDS (0 = automatic)
    int opt_mix_waves = 0;       // sparse-W tile kernel: wavefronts per workgroup (0 = automatic, 2, 4, 8, 16)
    int opt_mix_two_pass = 0;  // 1 = sparse-W steps always take the two-pass path
    int opt_mix_band = -1;     // sliding-window kernel for banded W: -1 = automatic (large problems), 0 = never, 1 = whenever W qualifies
    int opt_mix_csr_lds = 1;   // 0 = the tile kernel reads W from global memory even when it fits in LDS
    int opt_small_run = 1;     // 0 = gpga_run never takes the single-workgroup path for small problems
    int opt_blocks_per_cu = -1;  // -1 = automatic, 0 = one workgroup per tile group, k = persistent
    int num_cus = 256;
    int max_lds_block = 64 * 1024;  // LDS bytes one workgroup may ask for on this device
    int opt_pace_gbs = -1;   // target GB/s of paced persistent launches: -1 = automatic, 0 = off
    int opt_cycle_kernel = -1;   // row-streaming kernel for one-peer cycles of 2 .. 16 rows: -1 automatic, 0 never, 1 always
    int opt_pace_min_cycle = 0;  // shortest row cycle that is paced (0 = automatic)
    double clock_hz = 1e8;   // rate of the constant chip clock read by the pacing code
    PaceState* pace_states = nullptr;  // kPaceKeys controller states in device memory, library-owned

    // sparse mixing matrix of the grid / static exponential / custom graphs
    HostCsr csr;                 // host copy (also used by the beta estimate)
    int32_t* csr_ptr_d = nullptr;  // device copies, library-owned
    int32_t* csr_col_d = nullptr;
    float* csr_val_d = nullptr;
    int32_t* csr_off_d = nullptr;  // band kernel: signed circular offsets j - i (|offset| <= csr_band), csr_max_row per row
    float* csr_ellval_d = nullptr; // band kernel: the weights in the same padded layout (padding has weight 0)
    int32_t csr_band = 0;          // largest circular distance between a node and a neighbour: W is banded (mod n) with this half width
    int32_t csr_max_row = 0;       // most entries in one row
    bool csr_ready = false;

    // step-size schedule gamma_k (evaluated on the host in double, stored as float)
    int sched = SCHED_NONE;
    double sched_base = 0.0, sched_factor = 1.0, sched_start = 0.0, sched_power = 1.0;
    int64_t sched_period = 1, sched_warmup = 0, sched_total = 0;
    int sched_count = 0;
    int64_t sched_milestones[kMaxMilestones] = {0};

    // consensus trace (borrowed device array)
    double* trace = nullptr;
    int64_t trace_cap = 0;

    // adaptive averaging period (Algorithm 2)
    bool aga = false;
    int64_t aga_H_init = 0, aga_warmup = 0, aga_H_max = 0, aga_C = 0;
    double aga_F_init = 0.0;
    float* aga_loss = nullptr;  // n minibatch losses (library-owned; used by gpga_run)
    size_t aga_loss_cap = 0;

    char err[256] = {0};
};

// Description of one fused step launch over columns [col0, col0 + ncols*V).
struct StepGeom {
    const float* x;
    float* x_new;
    float* m;
    const float* g;
    int64_t ld;     // floats
    int64_t col0;   // first column of this pass (floats)
    int64_t ncols;  // columns of this pass in units of the vector type
    int32_t n;
    float lr, mu;
};

// ---- launchers (each returns hipSuccess or the launch error) ----------------

// Gossip step: stencil `mode` along cycles of the row permutation i -> (i+S) mod n.
// If spread_partials / spread_count are given and one walker stores whole columns, the
// kernel also writes one partial sum of squared deviations from the column means of
// x_new per workgroup and *spread_count receives their number (0 = not produced).
hipError_t launch_step_walk(const gpga_ctx* c, const StepGeom& ge, int mode, int32_t S, int vec,
                            double* spread_partials = nullptr, int64_t* spread_count = nullptr);
// Global-average step.
hipError_t launch_step_global(const gpga_ctx* c, const StepGeom& ge, int vec);

// Gossip step with a sparse W in CSR form (c->csr_*_d): one fused kernel with the
// column tile of all n rows staged in LDS when it fits, else local update into
// the g buffer followed by a sparse product.
// With spread_partials / spread_count (as for launch_step_walk) the fused kernel also leaves one
// partial sum of squared deviations per column tile when it runs with 16-byte lanes.
hipError_t launch_step_csr(const gpga_ctx* c, const StepGeom& ge, int vec, double* spread_partials = nullptr,
                           int64_t* spread_count = nullptr);

// Host-side graph construction and analysis.
void build_ring_csr(int32_t n, HostCsr* out);
void build_one_peer_csr(int32_t n, int32_t shift, HostCsr* out);
void build_grid_csr(int32_t n, HostCsr* out);
void build_static_expo_csr(int32_t n, HostCsr* out);
// Copies a caller's CSR arrays after range checks on the row pointers; nullptr, or what is wrong.
const char* copy_csr(int32_t n, const int64_t* row_ptr, const int32_t* col, const float* val, HostCsr* out);
// Checks shape, index range, non-negativity and row / column sums (|sum - 1| <= tol).
// Returns nullptr when W is acceptable, else a static description of the defect.
const char* validate_csr(int32_t n, const HostCsr& w, double tol);
// beta = ||W - (1/n) 1 1^T||_2 (Assumption 3) by Lanczos iteration on W^T W restricted
// to the complement of the all-ones vector.
double mixing_beta(int32_t n, const HostCsr& w);

// Gradients.
hipError_t launch_synth_grad(const gpga_ctx* c);
hipError_t launch_rows_grad(const gpga_ctx* c, const int32_t* idx, int32_t B, float* loss_out);
hipError_t launch_virtual_grad(const gpga_ctx* c, const int32_t* idx, int32_t B, float* loss_out);
// Small problems: T <= kSmallRunMaxIters whole iterations (stored-feature gradients, update,
// mix or average, consensus trace) in one single-workgroup launch; the final iterates go to the
// array T separate steps would leave them in (c->x for even T, c->x_new for odd T: the caller
// swaps the roles), g is left holding the last gradients; lr[t] is the step size of iteration c->k + t.
// small_run_fits tells whether the context's problem and sizes qualify.
bool small_run_fits(const gpga_ctx* c, const int32_t* idx, int32_t B);
hipError_t launch_small_run(const gpga_ctx* c, int32_t T, const int32_t* idx, int32_t B, const float* lr);
// Column chunks per node of the virtual-feature margin pass; it needs n * B * chunks doubles in c->partials.
int64_t virtual_margin_chunks(const gpga_ctx* c);

// Reductions and fills.
hipError_t launch_fill_rows(const gpga_ctx* c, float* dst, const float* row_or_null);
hipError_t launch_col_mean(const gpga_ctx* c, float* xbar);
// Sum of squared deviations into c->partials[0] (device double).
hipError_t launch_consensus_sq(gpga_ctx* c, size_t* partials_needed);
size_t consensus_partials_needed(const gpga_ctx* c);
// Partials the reduction pass over the bound X really writes (depends on its alignment).
size_t consensus_partials_used(const gpga_ctx* c);
// slot[0] = consensus distance of the live X (reduction pass + one final kernel).
hipError_t launch_consensus_trace(gpga_ctx* c, double* slot);
// The same with the per-workgroup partials in caller-chosen scratch (scratch_cap doubles, at least
// consensus_partials_needed(c) - 1): slot[0] = ||X - 1 xbar^T||_F.  hipErrorOutOfMemory if too small.
hipError_t launch_consensus_distance(const gpga_ctx* c, double* scratch, size_t scratch_cap, double* slot);
// Entries of the static scratch array behind gpga_consensus_error_static and its per-device address.
size_t static_scratch_doubles();
hipError_t static_scratch_for_device(int device, double** ptr_out);
// slot[0] = sqrt(sum of `count` partials) (count = 0 stores 0): one entry of the consensus trace.
hipError_t launch_trace_store(const gpga_ctx* c, const double* partials, int64_t count, double* slot);
// Streaming probe over count16 16-byte words (kind 0 read, 1 write, 2 copy, 3 three reads : two writes).
hipError_t launch_probe_stream(int kind, const float* src, float* dst, const float* src2, float* inout,
                               int64_t count16, float* sink, int64_t blocks, hipStream_t st);
// out[0] = mean of count floats (one workgroup, fp64 accumulation).
hipError_t launch_mean_f32(const gpga_ctx* c, const float* v, int64_t count, double* out);
