// Deadline pacing of persistent launches, shared by the fused step kernels, and the
// controller that finds the pacing rate by itself.
//
// Measured on this chip: a 3-read / 2-write stream mix runs at 6.3-6.5 TB/s when the
// whole chip streams one row of each array at a time, and drops to the 5.1-5.2 TB/s of a
// scattered copy once >= 32 different rows are open at once - which is what free-running
// walkers drift into, since each is at a different row of its own tile.  Pacing keeps
// them together without exchanging data: all wavefronts share one start time t0 (the
// first wavefront to arrive publishes the chip's constant-rate clock with a
// compare-and-swap) and a wavefront issues the loads of a row batch no earlier than
// t0 + (stream rows it has issued so far) * unit, where unit is the time the whole launch
// needs for one stream row at the pacing rate.  A late wavefront never waits; every wait
// ends at its deadline (the clock always advances) and is also capped by a poll count, so
// the grid always drains.
//
// The rate.  Below the rate the memory system sustains for a kernel's access pattern the
// launch is simply rate-limited and every wavefront ends within a few microseconds of its
// last deadline; above it the wavefronts fall behind, drift apart and the launch slows
// down.  The fastest rate at which the wavefronts still keep up is the optimum, and it
// differs between kernels, shapes and machines.  Every launch therefore measures how late
// its slowest wavefront ended (one atomic maximum per wavefront that ended late), and the
// last workgroup to leave turns that into the rate of the NEXT launch of the same kind:
// climb while launches keep up, bisect between the last rate that kept up and the first
// that did not, then hold a little below the edge and probe upwards again now and then.
// All of it lives in a PaceState in device memory: nothing depends on host-side launch
// counters, so a captured graph replays paced (and keeps adapting) like eager launches.
// The state resets itself - the last workgroup to leave clears the start time - so the
// next launch on the stream finds it clean.  Launches that share a PaceState must not
// overlap (a context enqueues on one stream).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gpga_internal.hpp"

constexpr double kPaceInitGbs = 6000.0;          // first rate of a controller (it climbs from there)
constexpr double kPaceMaxGbs = 7900.0;           // the controller never asks for more than this
// A launch that keeps up ends 40-65 us after the last deadline of its slowest wavefront (the
// queueing latency of the last row batch, measured on every kind of launch at every rate below
// its edge, fluctuating up to ~110 us at the edge); past the edge the figure grows by
// 50-100 us per percent of rate, faster than the planned duration shrinks.
constexpr double kPaceLateFloorSeconds = 100e-6;

// Rates are in bytes per clock count x 16 ("fp"); the clock is the chip's constant-rate
// counter (s_memrealtime, 100 MHz), so 6 TB/s is 60000 bytes per count = 960000 fp.
struct PaceState {             // 128 bytes (a cache line of its own), device memory owned by the context, zero-initialised
    unsigned long long t0;     // start time of the launch in flight; 0 between launches
    uint32_t left;             // workgroups of the launch in flight that have finished
    uint32_t late_max;         // largest lateness (clock counts) among its wavefronts so far
    uint32_t rate_fp;          // rate of the next launch; 0 = controller not started
    uint32_t lo_fp;            // last rate at which a launch kept up (0 = none known)
    uint32_t hi_fp;            // lowest recent rate at which a launch fell behind (0 = none known)
    uint32_t hold;             // launches left before the controller probes upwards again
    uint32_t launches;         // statistics: paced launches, and those that fell behind
    uint32_t late_launches;
    uint32_t last_rate_fp;     // the most recent launch: its rate, the lateness of its slowest
    uint32_t last_late;        //   wavefront and the planned duration, in clock counts
    uint32_t last_plan;
    uint32_t last_elapsed;     // t0 to the moment the last workgroup left
    uint16_t streak;           // consecutive launches that kept up while climbing (the climb step doubles with it)
    uint16_t hold_len;         // launches the next hold lasts: 16, doubling (to 128) each time a search ends where it began
    uint32_t history;          // one bit per recent launch, newest lowest: 1 = it fell behind
    uint32_t last_hold_fp;     // the rate the most recent hold began at
    uint32_t reserved[15];
};
static_assert(sizeof(PaceState) == 128, "PaceState is one 128-byte line");

enum PaceKey : int {           // launches of one kind share a PaceState ...
    PACE_GLOBAL = 0, PACE_RING, PACE_PEER_LONG, PACE_PEER_8, PACE_PEER_4, PACE_CYCLES, PACE_SELF, PACE_TILE, PACE_PEER_16, PACE_BAND,
    kPaceKinds = 16,
    // ... per direction of the x / x_new ping-pong: which of the two bound arrays a step reads and which it
    // writes changes the rate the memory system sustains (by up to 8 % for some placements of the arrays),
    // and steps alternate between the two directions
    kPaceKeys = 2 * kPaceKinds
};

struct PaceArgs {
    PaceState* st;             // nullptr = pacing off
    uint32_t unit_bytes;       // bytes the whole launch moves per 4-byte stream row (wavefronts x 64 x lane bytes)
    uint32_t rate_fixed_fp;    // > 0: pace at exactly this rate, controller off
    uint32_t rate_init_fp;     // controller: first rate, and the range it may move in
    uint32_t rate_min_fp, rate_max_fp;
    uint32_t late_floor;       // clock counts a wavefront may end after its last deadline and still count as keeping up
};

struct PaceRun {
    unsigned long long t0;
    uint32_t unit_fp;          // clock counts x 256 per stream row of the whole launch; 0 = off
    uint32_t rate_fp;
};

__device__ __forceinline__ unsigned long long pace_uniform64(unsigned long long v) {
    // readfirstlane returns a signed int: go through unsigned before widening
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(v >> 32));
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(v & 0xffffffffull));
    return ((unsigned long long)hi << 32) | (unsigned long long)lo;
}

__device__ __forceinline__ PaceRun pace_begin(const PaceArgs& p, int lane) {
    PaceRun r;
    r.t0 = 0ull;
    r.unit_fp = 0u;
    r.rate_fp = 0u;
    if (!p.st) return r;
    // the rate was left by the last workgroup of the previous launch of this kind (stream order)
    uint32_t rate = p.rate_fixed_fp;
    if (!rate) rate = __hip_atomic_load(&p.st->rate_fp, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    if (!rate) rate = p.rate_init_fp;
    rate = (uint32_t)__builtin_amdgcn_readfirstlane((int)rate);
    r.rate_fp = rate;
    unsigned long long unit = ((unsigned long long)p.unit_bytes << 12) / rate;  // x 16 (fp rate) x 256
    if (unit < 1ull) unit = 1ull;
    if (unit > 0xffffffffull) unit = 0xffffffffull;
    r.unit_fp = (uint32_t)unit;
    const unsigned long long mine = __builtin_amdgcn_s_memrealtime();
    unsigned long long seen = 0;
    if (lane == 0) {
        seen = atomicCAS(&p.st->t0, 0ull, mine);
        if (seen == 0ull) seen = mine;
    }
    r.t0 = pace_uniform64(seen);
    return r;
}

__device__ __forceinline__ void pace_wait(const PaceRun& r, uint32_t units_done) {
    if (!r.unit_fp) return;
    const unsigned long long deadline = r.t0 + (((unsigned long long)units_done * r.unit_fp) >> 8);
    for (int guard = 0; guard < (1 << 14); ++guard) {
        if (__builtin_amdgcn_s_memrealtime() >= deadline) break;
        __builtin_amdgcn_s_sleep(2);
    }
}

// The controller: state after a launch at rate r whose slowest wavefront ended `late` clock
// counts after its last deadline, of `plan` planned.  Runs in one thread.
// A rate counts as too fast only when two launches in a row fell behind at it.
//   searching (hold == 0): climb from the last rate that kept up (by 0.4 % of the rate twice, then
//     doubling with every launch in a row that keeps up, at most 1.6 %) until a rate is too fast, then
//     bisect between the two until they are 0.4 % apart, and hold the lower one;
//   holding (hold > 0): stay; if the rate has become too fast move down by half the fraction
//     the launch fell behind (at least 0.4 %, at most 6 %: past the edge a launch falls behind by
//     one to two times the excess); when the hold runs out search upwards again.
//   A hold lasts 16 launches at first and twice as long each time the search after it ends
//     within 0.4 % of where it began (at most 128); a search that ends elsewhere, or a rate that
//     became too fast, starts again at 16.  So a settled rate is probed rarely and a moved edge
//     (other buffers, another direction of the ping-pong, a busier machine) is followed quickly.
// (Also compiled for the host: the CPU test suite runs it against a model of a launch.)
__host__ __device__ __forceinline__ void pace_controller(const PaceArgs& p, uint32_t r, uint32_t late, uint32_t plan) {
    PaceState* st = p.st;
    const bool behind = late > p.late_floor + (plan >> 8);  // later than the usual tail + 0.4 % of the launch
    uint32_t lo = st->lo_fp, hi = st->hi_fp, hold = st->hold, streak = st->streak;
    uint32_t hold_len = st->hold_len ? st->hold_len : 16u;
    const uint32_t hist = ((st->history << 1) | (behind ? 1u : 0u)) & 7u;  // the last three launches
    uint32_t next = r;
    if (behind) st->late_launches += 1u;
    if (behind && !(hist & 2u)) {
        // the first late launch in a row decides nothing (one launch in ten is late at a rate that
        // otherwise keeps up, and the two directions of the x / x_new ping-pong differ): look again
        st->history = hist;
        return;
    }
    // a search has ended at rate `at`: hold it, the longer the more often searches end where they began
    auto begin_hold = [&](uint32_t at) {
        const uint32_t ref = st->last_hold_fp;
        const bool same = ref != 0u && (at > ref ? at - ref : ref - at) <= (ref >> 8);
        hold_len = same ? (hold_len < 64u ? hold_len * 2u : 128u) : 16u;
        hold = hold_len;
        st->last_hold_fp = at;
    };
    if (hold > 0u) {
        if (behind) {  // two late launches in a row while holding: the edge has moved down
            unsigned long long f = plan ? ((unsigned long long)(late - p.late_floor) << 9) / plan : 0ull;  // x 1024, halved
            if (f < 4ull) f = 4ull;
            if (f > 61ull) f = 61ull;
            next = r - (uint32_t)(((unsigned long long)r * f) >> 10);
            hi = r;
            lo = next;
            hold_len = 16u;
            hold = hold_len;
            st->last_hold_fp = next;
        } else {
            hold -= 1u;
            if (hold == 0u) {  // search upwards again from here
                lo = r;
                hi = 0u;
                streak = 0u;
            }
        }
    } else if (behind) {
        streak = 0u;
        if (lo != 0u && lo < r) {
            hi = r;  // the edge lies between the last rate that kept up and this one
            if (hi - lo > (lo >> 8)) {
                next = lo + ((hi - lo) >> 1);
            } else {
                next = lo;
                begin_hold(lo);
            }
        } else {
            // no lower rate known to keep up (first launches, or the edge has moved down): step down by
            // the fraction the launch fell behind, at least 0.8 %, at most 6 %
            unsigned long long f = plan ? ((unsigned long long)late << 10) / plan : 0ull;  // x 1024
            if (f < 8ull) f = 8ull;
            if (f > 61ull) f = 61ull;
            next = r - (uint32_t)(((unsigned long long)r * f) >> 10);
            hi = r;
            lo = 0u;
        }
    } else {
        lo = r;
        if (hi != 0u && hi <= r) hi = 0u;  // kept up at a rate that once was too fast: forget that edge
        if (hi == 0u) {
            next = r + ((r >> 8) << (streak < 2u ? 0u : streak < 4u ? streak - 1u : 2u));
            streak += 1u;
        } else if (hi - lo > (lo >> 8)) {
            next = lo + ((hi - lo) >> 1);
        } else {
            begin_hold(r);  // bracketed to 0.4 %: hold the rate that kept up
        }
    }
    if (next < p.rate_min_fp) next = p.rate_min_fp;
    if (next > p.rate_max_fp) next = p.rate_max_fp;
    st->lo_fp = lo;
    st->hi_fp = hi;
    st->hold = hold;
    st->streak = (uint16_t)(streak < 0xffffu ? streak : 0xffffu);
    st->hold_len = (uint16_t)hold_len;
    st->history = next != r ? 0u : hist;  // a new rate starts with a clean record
#if defined(__HIP_DEVICE_COMPILE__)
    __hip_atomic_store(&st->rate_fp, next, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
#else
    st->rate_fp = next;
#endif
}

// The moment a wavefront has issued its last row: to be taken right after its work loop, before
// any workgroup barrier (a wavefront without work would otherwise report its siblings' time).
__device__ __forceinline__ unsigned long long pace_now(const PaceArgs& p) {
    return p.st ? __builtin_amdgcn_s_memrealtime() : 0ull;
}

// End of a paced kernel: every wavefront reports how far behind its last deadline it ended
// (`now` from pace_now), the last workgroup to leave runs the controller and clears the
// launch's state.  Must be reached by every thread of every workgroup (it contains a
// workgroup barrier).
__device__ __forceinline__ void pace_end(const PaceArgs& p, const PaceRun& r, uint32_t units_done, int lane,
                                         unsigned long long now) {
    if (!p.st) return;
    const unsigned long long plan64 = ((unsigned long long)units_done * r.unit_fp) >> 8;
    const unsigned long long deadline = r.t0 + plan64;
    if (lane == 0 && now > deadline) {
        const unsigned long long late = now - deadline;
        atomicMax(&p.st->late_max, late > 0xffffffffull ? 0xffffffffu : (uint32_t)late);
    }
    __syncthreads();  // all wavefronts of this workgroup have read the start time and reported
    if (threadIdx.x == 0) {
        __threadfence();
        const uint32_t done = atomicAdd(&p.st->left, 1u);
        if (done == gridDim.x - 1u) {
            __threadfence();
            const uint32_t late = atomicExch(&p.st->late_max, 0u);
            const uint32_t plan = plan64 > 0xffffffffull ? 0xffffffffu : (uint32_t)plan64;
            const unsigned long long el = __builtin_amdgcn_s_memrealtime() - r.t0;
            p.st->launches += 1u;
            p.st->last_rate_fp = r.rate_fp;
            p.st->last_late = late;
            p.st->last_plan = plan;
            p.st->last_elapsed = el > 0xffffffffull ? 0xffffffffu : (uint32_t)el;
            if (!p.rate_fixed_fp) pace_controller(p, r.rate_fp, late, plan);
            __threadfence();
            atomicExch(&p.st->left, 0u);
            atomicExch(&p.st->t0, 0ull);
        }
    }
}

// Host side: how many workgroups a persistent launch of `work` items gets when `resident` fit on the chip.
// A paced launch lasts as long as its busiest workgroup and a round lasts the same however many
// workgroups take part in it, so the items are dealt in whole rounds: with 25000 items and 1024
// resident workgroups, 1000 workgroups of 25 items each keep the whole launch busy to the end, where
// 1024 would leave 600 of them idle during the last of 25 rounds.  Fewer workgroups stream a little
// slower (measured on the ring walk: 97 % of the full rate with three quarters of the wavefronts, 89 %
// with half), which never outweighs a partly empty round: 1563 items on 1024 workgroups run as 782 x 2
// (2 x 0.76 / 0.97 = 1.57 full rounds' worth of time) rather than 1024 x 2 (2 rounds).
inline int64_t balanced_blocks(int64_t work, int64_t resident) {
    if (resident <= 0 || work <= resident) return work;
    const int64_t rounds = (work + resident - 1) / resident;
    return (work + rounds - 1) / rounds;
}

// Host side: pacing arguments of one launch whose `wavefronts` resident wavefronts each move
// 64 lanes x lane_bytes per stream row.  gbs > 0 paces at exactly that rate (GB/s); gbs < 0 lets
// the controller of PaceState `key` choose; gbs == 0, or a context without pacing state, or a
// geometry that does not fit the fixed-point fields leaves pacing off.
inline double pace_fp_per_gbs(const gpga_ctx* c) { return 1e9 / c->clock_hz * 16.0; }

inline void pace_setup(gpga_ctx* c, double gbs, int key, double wavefronts, int lane_bytes, PaceArgs* p) {
    p->st = nullptr;
    p->unit_bytes = 0;
    p->rate_fixed_fp = p->rate_init_fp = p->rate_min_fp = p->rate_max_fp = 0;
    p->late_floor = 0;
    if (gbs == 0.0 || !c || !c->pace_states || key < 0 || key >= kPaceKinds) return;
    const double bytes = wavefronts * 64.0 * lane_bytes;
    if (!(bytes >= 1.0 && bytes < 4.0e9)) return;
    const double fp = pace_fp_per_gbs(c);
    const double lo = 1000.0 * fp, hi = 16000.0 * fp;
    if (!(hi < 4.0e9)) return;
    p->st = c->pace_states + 2 * key + (c->x == c->x_first ? 0 : 1);
    p->unit_bytes = (uint32_t)bytes;
    p->rate_fixed_fp = gbs > 0.0 ? (uint32_t)(gbs * fp) : 0u;
    p->rate_init_fp = (uint32_t)(kPaceInitGbs * fp);
    p->rate_min_fp = (uint32_t)lo;
    p->rate_max_fp = (uint32_t)(kPaceMaxGbs * fp);
    p->late_floor = (uint32_t)(kPaceLateFloorSeconds * c->clock_hz);
    c->last_paced = 1;
}
