// Shared device-side definitions of the gfx950 FastSGD codec: workspace records, wave64 helpers,
// exact float64 -> float32 conversions on bit patterns.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/fastsgd.h"
#include "../../include/fastsgd_profile.h"

namespace fsgd {

typedef uint32_t u32;
typedef uint64_t u64;
typedef int64_t i64;

constexpr u32 kWave = 64;
constexpr u32 kThreads = 256;                 // workgroup size of the streaming kernels
constexpr u32 kWaves = kThreads / kWave;
constexpr u32 kRow = 256;                     // elements of one row: a float4 per lane of a wave
constexpr u32 kTile = 4096;                   // elements of one abs-sum tile: 4 rows per wave of the workgroup
constexpr u32 kValRows = 8;                   // rows a wave of the value pass loads at a time
constexpr u32 kValTile = kRow * kValRows;     // 2048 elements
constexpr u32 kHeaderBytes = 64;
constexpr u32 kMagic = 0x44475346u;           // "FSGD"
constexpr u32 kVersion = 1;
constexpr u32 kBins = 16;                     // exponent bins of the exact abs-sum (16 exponents each)
constexpr u32 kMaxKB = 4096;
constexpr u32 kMaxTau = 256;                  // Section 3.2 recommends 128 (a token of one byte); above it a token takes 9 bits
constexpr u32 kChunkTarget = 4096;            // chunks a call's elements are cut into (one per wave of the value pass)
constexpr u32 kMaxSegChunks = kChunkTarget;   // no segment has more chunks than this
constexpr u32 kGranule = 32;                  // values that share one bound of the first pass: the unit the second pass fetches by
constexpr u32 kGranLanes = kGranule / 4;      // lanes (a float4 each) that hold one granule of a row
constexpr u32 kRowGranules = kRow / kGranule; // bounds per row
constexpr u32 kMaxChunkRows = (65536 / kRowGranules - 1) / kValRows * kValRows;   // a granule's index inside its chunk fits 16 bits
constexpr u32 kMaxGroups = 2048;              // groups of key blocks whose sizes are added up by atomics
constexpr u32 kSub = 1024;                    // keys of a key block a wave handles at a time (16 rows of 64)
constexpr u32 kLaneKeys = kSub / 64;          // ... 16 consecutive keys per lane

// Host-built description of one gradient (segment) of a call.
struct SegInfo {
    u64 elem_begin;     // first element, counted from the 16-byte-aligned base of the arrays
    u64 elem_count;
    double base;
    u32 tile_begin;     // first tile of the segment in the abs-sum pass
    u32 chunk_begin;    // first chunk of the segment in the value pass
    u32 tau, flag_bits, block_keys;
    u32 row_begin;      // first row of the segment in the call's row numbering (row maxima)
};
static_assert(sizeof(SegInfo) == 48, "segment record layout");

// Device-computed state of one segment.
struct SegState {
    double sum;         // Algorithm 1 line 1
    u32 thr_bits;       // bit pattern of the early-stop threshold (Algorithm 1 line 2); 0xFFFFFFFF = keep nothing
    u32 nb;             // key blocks (batch calls; a single gradient derives it from the survivor count)
    u64 d;              // survivors
    u64 item_begin;     // first work item (key block) of the segment
    u64 unit_begin;     // first work unit (kWaves key blocks of one segment) of the segment
    float lg_sum;       // log2(sum) and 1 / log2(b) in binary32: the value pass's first guess of a code,
    float inv_lg_base;  //   (lg_sum - log2|v|) * inv_lg_base ~ log_b(sum / |v|)
    u32 B[kMaxTau];     // B[c-1] = bit pattern of the boundary of code c
};

// A survivor's code in the scratch array between the value pass and the key encoder: code-1 with the sign
// on top, in a byte while every tau of the call is at most 128, in 16 bits otherwise.
template <bool WIDE> struct ScratchCode { typedef uint8_t type; };
template <> struct ScratchCode<true> { typedef uint16_t type; };

// Per key block (work item), filled by k_measure_keys, consumed by k_pack_keys.
//   span8: 8-byte words the item adds to the output: its two planes and, for the first item of a
//   segment, the segment's header, value plane and directory.
struct BlockInfo { u32 preKey, M, payload_bits, span8; };

struct Ctrl {
    u32 status;         // first device-detected fastsgd_status
    u32 reserved;
    u64 total_items;    // batch calls: work items / units of the key encoder
    u64 total_units;
    u64 pad[5];
};
static_assert(sizeof(Ctrl) == 64, "control block layout");

struct EncodePlan {     // host-computed carve-up of the workspace
    u64 max_chunks, max_items, total_n, max_slots, max_rows;
    u32 n_segments, n_slots;
    u64 off_ctrl, off_gsum, zero_end, off_gbins, zero_end_batch;   // [off_ctrl, zero_end*) is cleared per call
    u64 off_rowmax, off_ccount, off_binfo, off_seginfo, off_segstate, off_skeys, off_scodes;
    u64 total_narrow, total;      // bytes needed if every tau is at most 128 (a byte per code) / in any case
};

// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ u32 lane_id() { return threadIdx.x & 63u; }
__device__ __forceinline__ u32 wave_id() { return threadIdx.x >> 6; }
__device__ __forceinline__ u32 uniform(u32 x) { return (u32)__builtin_amdgcn_readfirstlane((int)x); }
__device__ __forceinline__ u64 uniform64(u64 x) {
    return (u64)uniform((u32)x) | ((u64)uniform((u32)(x >> 32)) << 32);
}

// Cross-lane moves by data-parallel primitives (no trip through the LDS crossbar).  `old` is what a
// lane gets when its source lane does not exist or its row is masked out.
template <int CTRL, int ROW_MASK = 0xF>
__device__ __forceinline__ u32 dpp_mov(u32 old, u32 x) {
    return (u32)__builtin_amdgcn_update_dpp((int)old, (int)x, CTRL, ROW_MASK, 0xF, false);
}
constexpr int kDppRowShr1 = 0x111, kDppRowShr2 = 0x112, kDppRowShr4 = 0x114, kDppRowShr8 = 0x118;
constexpr int kDppRowBcast15 = 0x142, kDppRowBcast31 = 0x143, kDppWaveShr1 = 0x138;

// value of lane - 1 (lane 0 gets `first`)
__device__ __forceinline__ u32 lane_above(u32 x, u32 first) { return dpp_mov<kDppWaveShr1>(first, x); }
__device__ __forceinline__ u32 read_lane(u32 x, u32 lane) { return (u32)__builtin_amdgcn_readlane((int)x, (int)lane); }

__device__ __forceinline__ u32 wave_incl_scan(u32 x) {
    x += dpp_mov<kDppRowShr1>(0u, x);
    x += dpp_mov<kDppRowShr2>(0u, x);
    x += dpp_mov<kDppRowShr4>(0u, x);
    x += dpp_mov<kDppRowShr8>(0u, x);                 // inclusive inside each row of 16 lanes
    x += dpp_mov<kDppRowBcast15, 0xA>(0u, x);         // rows 1 and 3 add the total of the row before
    x += dpp_mov<kDppRowBcast31, 0xC>(0u, x);         // rows 2 and 3 add the total of rows 0-1
    return x;
}
__device__ __forceinline__ u64 wave_incl_scan64(u64 x) {
#define FSGD_STEP64(CTRL, MASK)                                                                   \
    {                                                                                              \
        const u32 lo = dpp_mov<CTRL, MASK>(0u, (u32)x), hi = dpp_mov<CTRL, MASK>(0u, (u32)(x >> 32)); \
        x += (u64)lo | ((u64)hi << 32);                                                            \
    }
    FSGD_STEP64(kDppRowShr1, 0xF) FSGD_STEP64(kDppRowShr2, 0xF) FSGD_STEP64(kDppRowShr4, 0xF)
    FSGD_STEP64(kDppRowShr8, 0xF) FSGD_STEP64(kDppRowBcast15, 0xA) FSGD_STEP64(kDppRowBcast31, 0xC)
#undef FSGD_STEP64
    return x;
}
__device__ __forceinline__ u32 wave_sum(u32 x) { return read_lane(wave_incl_scan(x), 63); }
__device__ __forceinline__ u64 wave_sum64(u64 x) {
    const u64 s = wave_incl_scan64(x);
    return (u64)read_lane((u32)s, 63) | ((u64)read_lane((u32)(s >> 32), 63) << 32);
}
__device__ __forceinline__ u32 wave_max(u32 x) {
    u32 y;
    y = dpp_mov<kDppRowShr1>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr2>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr4>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr8>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowBcast15, 0xA>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowBcast31, 0xC>(0u, x); x = x > y ? x : y;
    return read_lane(x, 63);
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
// One thread walks the chain into `P` (kMaxTau + 1 doubles, shared memory); callers then divide in parallel.
__device__ __forceinline__ void power_chain(double base, u32 tau, double* P) {
    double p = 1.0;
    P[0] = 1.0;
    for (u32 c = 1; c <= tau; ++c) { p = p * base; P[c] = p; }
}

// Largest index i in [0, n) with value(i) <= x, for a non-decreasing value() with value(0) <= x and an
// x that is the same in all lanes: the wave probes 64 evenly spaced entries per round, so 4096
// entries take two memory round trips instead of twelve.
template <class Value>
__device__ __forceinline__ u32 wave_upper_index(u32 n, u64 x, Value value) {
    u32 lo = 0, hi = n;
    while (hi - lo > 1) {
        const u32 step = (hi - lo + 63u) / 64u;
        const u32 idx = lo + lane_id() * step;
        const bool p = idx < hi && value(idx) <= x;
        const u32 c = (u32)__popcll(__ballot(p));          // >= 1: lane 0 probes lo
        lo = uniform(lo + (c - 1u) * step);
        hi = lo + step < hi ? lo + step : hi;
    }
    return lo;
}

// Last segment whose first tile / chunk is <= the given one (segments without any share their
// successor's value).
__device__ __forceinline__ u32 find_tile_segment(const SegInfo* segs, u32 n_segments, u32 tile) {
    return wave_upper_index(n_segments, tile, [&](u32 i) { return segs[i].tile_begin; });
}
__device__ __forceinline__ u32 find_chunk_segment(const SegInfo* segs, u32 n_segments, u32 chunk) {
    return wave_upper_index(n_segments, chunk, [&](u32 i) { return segs[i].chunk_begin; });
}

// 16 bytes of a large array that is streamed through once per pass: a non-temporal load, which tells the
// caches not to keep the line (the first value pass ran 12 % faster for it: nothing of a 496 MB array that is
// read from end to end is still cached when the next pass comes, so keeping it only costs).
typedef u32 u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_stream16(const void* p) {
    const u32x4 q = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
    return make_uint4(q.x, q.y, q.z, q.w);
}

// Orders a wave's shared-memory accesses: what its lanes wrote before is visible to all of them after.
__device__ __forceinline__ void wave_lds_sync() {
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__device__ __forceinline__ void set_status(Ctrl* ctrl, u32 code) { atomicCAS(&ctrl->status, 0u, code); }

__device__ __forceinline__ u64 align8(u64 x) { return (x + 7) & ~7ull; }

// Section 3.2: after the filter a code (stored as code-1) takes ceil(log2 tau) bits, one more for the
// sign; 8 bits for tau in 65..128.
__device__ __forceinline__ u32 code_width(u32 tau) { return 1u + (32u - (u32)__clz((int)(tau - 1u))); }
// Bytes of the value plane: d tokens of `width` bits, zero-padded to 64-bit words.
__device__ __forceinline__ u64 value_plane_bytes(u64 d, u32 width) { return 8ull * ((d * width + 63ull) >> 6); }
constexpr int kBufferWord3 = 0x00020000;   // fourth word of a gfx9 raw buffer descriptor: 32-bit data format
constexpr u32 kCodeWords = 32u * 8u;   // 32-bit words of 1024 tokens of at most 8 bits (nine-bit tokens take 288 of the 512)

// Level lengths of Algorithm 2's length flag for a block with maximal length M and l flag bits:
// level i (1..2^l) holds ceil(i*M / 2^l) bits; a delta of `need` significant bits takes the
// smallest level that holds it, i = floor((need-1) * 2^l / M) + 1 (level 1 for need = 0).
// The division is by the block's M (<= 32) of a number below 1024, done as a multiplication by
// ceil(2^16 / M), which is exact in that range.
__device__ __forceinline__ u32 level_magic(u32 M) { return (65536u + M - 1u) / M; }
__device__ __forceinline__ u32 level_of(u32 need, u32 l, u32 magic) {
    return need ? ((((need - 1u) << l) * magic) >> 16) + 1u : 1u;
}
__device__ __forceinline__ u32 level_len(u32 level, u32 M, u32 l) { return (level * M + (1u << l) - 1u) >> l; }

}  // namespace fsgd
