// Shared device-side definitions of the gfx950 FastSGD codec: workspace records, wave64 helpers,
// the decoupled look-back scan, exact float64 -> float32 conversions on bit patterns.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fastsgd.h"

namespace fsgd {

typedef uint32_t u32;
typedef uint64_t u64;
typedef int64_t i64;

constexpr u32 kWave = 64;
constexpr u32 kThreads = 256;                 // workgroup size of every streaming kernel
constexpr u32 kWaves = kThreads / kWave;
constexpr u32 kTile = 4096;                   // elements per tile: 4 float4 per thread
constexpr u32 kHeaderBytes = 64;
constexpr u32 kMagic = 0x44475346u;           // "FSGD"
constexpr u32 kVersion = 1;
constexpr u32 kBins = 16;                     // exponent bins of the exact abs-sum (16 exponents each)
constexpr u32 kMaxKB = 4096;
constexpr u32 kSpinLimit = 1u << 20;          // bounded wait of the look-back scan

// Host-built description of one gradient (segment) of a call.
struct SegInfo {
    u64 elem_begin;     // first element, counted from the 16-byte-aligned base of the arrays
    u64 elem_count;
    u64 tile_begin;     // first tile of this segment in the call's tile numbering
    double base;
    u32 tau, flag_bits, block_keys, pad;
};

// Device-computed state of one segment.
struct SegState {
    double sum;         // Algorithm 1 line 1
    u32 thr_bits;       // bit pattern of the early-stop threshold (Algorithm 1 line 2); 0xFFFFFFFF = keep nothing
    u32 pad0;
    u64 rank_begin;     // global rank of the segment's first survivor
    u64 d;              // survivors
    u64 item_begin;     // first work item (key block) of the segment
    u64 stream_begin;   // byte offset of the segment's stream in the output
    u32 nb;             // key blocks
    u32 pad[3];
    u32 B[128];         // B[c-1] = bit pattern of the boundary of code c
};

// Per key block, filled by the key encoder, consumed by the finaliser.
struct BlockInfo { u32 preKey, M, payload_bits, size8; };

// A returning atomic on one address costs about 11 ns on this part and they serialise, so one ticket
// counter per tile would cap a pass at ~90 M tiles/s.  Tiles are therefore dealt from kLanesOfTickets
// counters on separate cache lines: counter c hands out tiles c, c + 8, c + 16, ...; wave c of every
// workgroup draws from counter c.  Any resident workgroup owns a wave for every counter, so the lowest
// unpublished tile is always either in work or about to be drawn by a wave that is not waiting:
// the look-back cannot deadlock, whatever part of the grid is resident.
constexpr u32 kTicketLanes = 8;
constexpr u32 kTicketStride = 32;             // u32 words between counters (128 bytes)

struct Ctrl {
    u32 ticket_val[kTicketLanes * kTicketStride];
    u32 ticket_key[kTicketLanes * kTicketStride];
    u32 status;         // first device-detected fastsgd_status
    u32 done_key;       // key-encoder work items finished
    u64 total_items;
    u64 total_d;
    u64 pad[5];
};
static_assert(sizeof(Ctrl) == 2 * kTicketLanes * kTicketStride * 4 + 64, "control block layout");

struct EncodePlan {     // host-computed carve-up of the workspace
    u64 n_tiles, max_items, total_n;
    u32 n_segments, n_slots;
    u64 off_ctrl, off_gbins, off_tdesc, off_idesc, zero_end, zero_end_batch;   // [off_ctrl, zero_end*) is cleared per call
    u64 off_seginfo, off_segstate, off_binfo, off_ckeys, off_codes, total;
};

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() { return threadIdx.x & 63u; }
__device__ __forceinline__ u32 wave_id() { return threadIdx.x >> 6; }

__device__ __forceinline__ u32 wave_incl_scan(u32 x) {
#pragma unroll
    for (u32 d = 1; d < 64; d <<= 1) {
        u32 y = __shfl_up(x, d, 64);
        if (lane_id() >= d) x += y;
    }
    return x;
}
__device__ __forceinline__ u64 wave_incl_scan64(u64 x) {
#pragma unroll
    for (u32 d = 1; d < 64; d <<= 1) {
        u64 y = __shfl_up((unsigned long long)x, d, 64);
        if (lane_id() >= d) x += y;
    }
    return x;
}
__device__ __forceinline__ u64 wave_sum64(u64 x) {
#pragma unroll
    for (u32 d = 32; d >= 1; d >>= 1) x += __shfl_xor((unsigned long long)x, d, 64);
    return x;
}
__device__ __forceinline__ u32 wave_max(u32 x) {
#pragma unroll
    for (u32 d = 32; d >= 1; d >>= 1) { u32 y = __shfl_xor(x, d, 64); x = x > y ? x : y; }
    return x;
}

// Exclusive scan of one u32 per thread over the 256-thread workgroup; *total receives the sum.
// `scratch` holds kWaves + 1 words.  Contains two barriers.
__device__ __forceinline__ u32 block_excl_scan(u32 x, u32* scratch, u32* total) {
    u32 incl = wave_incl_scan(x);
    if (lane_id() == 63) scratch[wave_id()] = incl;
    __syncthreads();
    u32 base = 0, tot = 0;
#pragma unroll
    for (u32 w = 0; w < kWaves; ++w) {
        u32 t = scratch[w];
        if (w < wave_id()) base += t;
        tot += t;
    }
    __syncthreads();
    *total = tot;
    return base + incl - x;
}

// ---------------------------------------------------------------------------------------------
// Decoupled look-back over descriptors {status:2, value:62}.  Items are numbered by a ticket taken
// when a workgroup starts on them, so every predecessor of a waiting item is already running and
// publishes its aggregate without waiting on anyone.  Called by all 64 lanes of ONE wave; returns
// the exclusive prefix of item `idx` to every lane.  The wait is bounded: on giving up *gave_up is
// set (the caller reports FASTSGD_ERR_DEVICE) and a prefix is still published, so no successor
// can wait forever.
constexpr u64 kDescAgg = 1ull << 62, kDescPrefix = 2ull << 62, kDescMask = (1ull << 62) - 1;

__device__ __forceinline__ u64 desc_load(const u64* p) {
    return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void desc_store(u64* p, u64 v) {
    __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ u64 lookback_exclusive(u64* desc, u64 idx, u64 aggregate, u32* gave_up) {
    const u32 lane = lane_id();
    if (idx == 0) {
        if (lane == 0) desc_store(&desc[0], kDescPrefix | aggregate);
        return 0;
    }
    if (lane == 0) desc_store(&desc[idx], kDescAgg | aggregate);
    u64 excl = 0;
    i64 top = (i64)idx - 1;
    u32 spins = 0;
    for (;;) {
        i64 j = top - (i64)lane;
        u64 w = (j >= 0) ? desc_load(&desc[j]) : kDescPrefix;      // virtual prefix 0 before item 0
        u32 st = (u32)(w >> 62);
        u64 none = __ballot(st == 0);
        u64 pref = __ballot(st == 2);
        u32 first_none = none ? (u32)__builtin_ctzll(none) : 64u;
        u32 first_pref = pref ? (u32)__builtin_ctzll(pref) : 64u;
        if (first_none < first_pref) {                             // a needed descriptor is not there yet
            if (++spins > kSpinLimit) { *gave_up = 1; break; }
            __builtin_amdgcn_s_sleep(2);
            continue;
        }
        u32 last = first_pref < 64u ? first_pref : 63u;
        excl += wave_sum64(lane <= last ? (w & kDescMask) : 0ull);
        if (first_pref < 64u) break;
        top -= 64;
    }
    if (lane == 0) desc_store(&desc[idx], kDescPrefix | ((excl + aggregate) & kDescMask));
    return excl;
}

// ---------------------------------------------------------------------------------------------
// binary64 -> binary32 bit pattern of a positive, finite, normal double, rounding either to
// nearest-even or towards +infinity.  Integer arithmetic only, so the result does not depend on
// the float mode the kernel runs in.
__device__ __forceinline__ u32 f64_to_f32_bits(double t, bool round_up) {
    u64 u = (u64)__double_as_longlong(t);
    int e = (int)((u >> 52) & 0x7FF);
    u64 man = (u & ((1ull << 52) - 1)) | (1ull << 52);
    int E = e - 1023;
    if (E > 127) return 0x7F800000u;
    if (E >= -126) {
        u64 q = man >> 29, rem = man & ((1ull << 29) - 1);
        if (round_up ? (rem != 0) : (rem > (1ull << 28) || (rem == (1ull << 28) && (q & 1)))) ++q;
        return (u32)(((u64)(E + 127) << 23) + (q - (1ull << 23)));   // a carry lands in the exponent
    }
    int s = -97 - E;                        // shift that leaves units of 2^-149; s >= 30
    if (s >= 64) return round_up ? 1u : 0u;  // below half of the smallest denormal
    u64 q = man >> s, rem = man & ((1ull << s) - 1), half = 1ull << (s - 1);
    if (round_up ? (rem != 0) : (rem > half || (rem == half && (q & 1)))) ++q;
    return (u32)q;
}

// P[c] = fl64(P[c-1] * b), t_c = fl64(sum / P[c]): the real boundary sum / b^c of Eq. 3 in binary64.
// One thread walks the chain into `P` (129 doubles, shared memory); callers then divide in parallel.
__device__ __forceinline__ void power_chain(double base, u32 tau, double* P) {
    double p = 1.0;
    P[0] = 1.0;
    for (u32 c = 1; c <= tau; ++c) { p = p * base; P[c] = p; }
}

__device__ __forceinline__ u32 find_segment(const SegInfo* segs, u32 n_segments, u64 tile) {
    u32 lo = 0, hi = n_segments;            // last segment with tile_begin <= tile that is not empty of tiles
    while (hi - lo > 1) {
        u32 mid = (lo + hi) >> 1;
        if (segs[mid].tile_begin <= tile) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ void set_status(Ctrl* ctrl, u32 code) { atomicCAS(&ctrl->status, 0u, code); }

}  // namespace fsgd
