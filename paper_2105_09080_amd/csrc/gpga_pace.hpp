// Deadline pacing of persistent launches, shared by the fused step kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gpga_internal.hpp"

// Pacing of a persistent launch (see pace_begin / pace_wait below).
struct PaceArgs {
    unsigned long long* slots;  // 64 start-time words, one per launch sequence number mod 64
    uint32_t seq;               // launch sequence number
    uint32_t unit_fp;           // clock counts (x 256) per 4-byte stream row of the whole launch; 0 = off
};


// Deadline pacing of a persistent launch.  Measured on this chip: a 3-read /
// 2-write stream mix runs at 6.3-6.5 TB/s when the whole chip streams one row
// of each array at a time, and drops to the 5.1-5.2 TB/s of a scattered copy
// once >= 32 different rows are open at once - which is what free-running
// walkers drift into, since each is at a different row of its own tile.
// Pacing keeps them together without exchanging data: all wavefronts share
// one start time t0 (the first workgroup to arrive publishes the chip's
// constant-rate clock with a compare-and-swap) and a wavefront issues the
// loads of a row batch no earlier than t0 + (stream rows it has issued so
// far) * unit, where unit is the time the whole launch needs for one stream
// row at the target rate.  A late wavefront never waits; every wait ends at its
// deadline (the clock always advances) and is also capped by a poll count, so
// the grid always drains.
__device__ __forceinline__ unsigned long long pace_begin(const PaceArgs& p, int lane, bool first_thread) {
    if (!p.unit_fp) return 0ull;
    if (first_thread) p.slots[(p.seq + 32u) & 63u] = 0ull;  // recycle a slot for a later launch
    const unsigned long long mine = __builtin_amdgcn_s_memrealtime();
    unsigned long long seen = 0;
    if (lane == 0) {
        seen = atomicCAS(p.slots + (p.seq & 63u), 0ull, mine);
        if (seen == 0ull) seen = mine;
    }
    // readfirstlane returns a signed int: go through unsigned before widening
    const unsigned hi = (unsigned)__builtin_amdgcn_readfirstlane((int)(seen >> 32));
    const unsigned lo = (unsigned)__builtin_amdgcn_readfirstlane((int)(seen & 0xffffffffull));
    const unsigned long long t0v = ((unsigned long long)hi << 32) | (unsigned long long)lo;
    return t0v;
}
__device__ __forceinline__ void pace_wait(const PaceArgs& p, unsigned long long t0, uint32_t units_done) {
    if (!p.unit_fp) return;
    const unsigned long long deadline = t0 + (((unsigned long long)units_done * p.unit_fp) >> 8);
    for (int guard = 0; guard < (1 << 14); ++guard) {
        if (__builtin_amdgcn_s_memrealtime() >= deadline) break;
        __builtin_amdgcn_s_sleep(2);
    }
}

// Host side: pacing arguments of one launch whose `wavefronts` resident wavefronts each move
// 64 lanes x lane_bytes per stream row, at the target rate gbs (GB/s).  Leaves pacing off
// (unit_fp = 0) when the rate is 0, the context has no start-time words, or the unit
// does not fit its fixed-point field.
inline void pace_setup(gpga_ctx* c, double gbs, double wavefronts, int lane_bytes, PaceArgs* p) {
    p->unit_fp = 0;
    p->slots = nullptr;
    p->seq = 0;
    if (!(gbs > 0.0) || !c || !c->pace_slots) return;
    // time (clock counts x 256) for the whole launch to move one stream row
    const double bytes = wavefronts * 64.0 * lane_bytes;
    const double fp = bytes / (gbs * 1e9) * c->clock_hz * 256.0;
    if (fp >= 1.0 && fp < 4.0e9) {
        p->unit_fp = (uint32_t)fp;
        p->slots = c->pace_slots;
        p->seq = c->pace_seq++;
    }
}
