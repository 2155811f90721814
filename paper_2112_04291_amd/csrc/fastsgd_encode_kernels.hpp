// Encoder kernels of the gfx950 FastSGD codec (Algorithms 1 and 2 of arXiv 2112.04291).
//
//   k_init           batch calls: clears the per-call control words, stores the segment table
//   k_abs_sum        Algorithm 1 line 1: exact sum of |v| per segment (integer accumulation)
//   k_tables         Algorithm 1 line 2 + Eq. 3 as a boundary table sum / b^c, c = 1..tau
//   k_encode_values  Algorithm 1 lines 4-10: threshold test, code, sign, compaction of survivors
//   k_plan_segments  per segment: scan of the chunk counts, survivors d, key blocks
//   k_number_segments  batch calls: work-item numbering over the segments
//   k_measure_keys   Algorithm 2, first loop, per key block: deltas, maxDelta -> M, size of the block
//   k_pack_keys      Algorithm 2, second loop: length flags, bit packing; directory, headers, value planes
#pragma once
#include "fastsgd_device.hpp"

namespace fsgd {

// ---------------------------------------------------------------------------------------------
constexpr u32 kSegBatch = 80;            // segment records per launch: 3840 bytes of the 4 KB a launch can carry
struct SegBatch { SegInfo seg[kSegBatch]; };   // passed by value: the segment table needs no host->device copy

__global__ void k_init(u64* zero_begin, u64 zero_words, SegInfo* segs, SegBatch batch, u32 first, u32 count) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (; i < zero_words; i += stride) zero_begin[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x < count) segs[first + threadIdx.x] = batch.seg[threadIdx.x];
}

__global__ void k_store_segments(SegInfo* segs, SegBatch batch, u32 first, u32 count) {
    if (threadIdx.x < count) segs[first + threadIdx.x] = batch.seg[threadIdx.x];
}

// Rows (of 256 elements) of a segment, counted from its first element rounded down to a multiple of 4.
__device__ __forceinline__ u64 segment_rows(const SegInfo& s) {
    return s.elem_count ? (s.elem_begin + s.elem_count - (s.elem_begin & ~3ull) + kRow - 1) / kRow : 0ull;
}

// ---------------------------------------------------------------------------------------------
// Tile geometry of the abs-sum pass.  A segment's tiles start at its first element rounded down to
// a multiple of 4 (so float4 loads stay aligned); thread (wave w, lane) holds, for r = 0..3, the
// four elements  tile0 + w*1024 + r*256 + lane*4 + {0,1,2,3}.
struct TileGeom {
    u64 tile0;      // element index of the tile's first slot
    u64 lo, hi;     // valid element range [lo, hi) of the segment
    bool full;
};
__device__ __forceinline__ TileGeom tile_geom(const SegInfo& s, u64 tile) {
    TileGeom g;
    g.tile0 = (s.elem_begin & ~3ull) + (tile - s.tile_begin) * kTile;
    g.lo = s.elem_begin;
    g.hi = s.elem_begin + s.elem_count;
    g.full = (g.tile0 >= g.lo) && (g.tile0 + kTile <= g.hi);
    return g;
}
// keep: the tile is among the last ones the pass reads, which the second value pass reads first (it walks
// the array from its end): an ordinary load, so that the caches hold on to it; everything else streams.
__device__ __forceinline__ void load_tile(const float* __restrict__ values, const TileGeom& g, u32 bits[4][4], bool keep = false) {
    const u32 slot0 = wave_id() * 1024u + lane_id() * 4u;
    if (g.full && keep) {
#pragma unroll
        for (u32 r = 0; r < 4; ++r) {
            const uint4 q = *reinterpret_cast<const uint4*>(values + g.tile0 + slot0 + r * 256u);
            bits[r][0] = q.x; bits[r][1] = q.y; bits[r][2] = q.z; bits[r][3] = q.w;
        }
    } else if (g.full) {
#pragma unroll
        for (u32 r = 0; r < 4; ++r) {
            const uint4 q = load_stream16(values + g.tile0 + slot0 + r * 256u);
            bits[r][0] = q.x; bits[r][1] = q.y; bits[r][2] = q.z; bits[r][3] = q.w;
        }
    } else {
#pragma unroll
        for (u32 r = 0; r < 4; ++r)
#pragma unroll
            for (u32 c = 0; c < 4; ++c) {
                u64 e = g.tile0 + slot0 + r * 256u + c;
                bits[r][c] = (e >= g.lo && e < g.hi) ? __float_as_uint(values[e]) : 0u;
            }
    }
}

// ---------------------------------------------------------------------------------------------
// Exact abs-sum.  |v| = m * 2^(e1-150) with m the 24-bit significand and e1 = max(exponent, 1).
// Exponents are grouped 16 to a bin; inside bin k the element adds m << (e1 & 15) (< 2^39) to a
// 64-bit integer.  Integer addition is associative, so any partition of the work gives the same
// bins, and the sum can be rounded exactly once.  Every lane owns a private row of bins in shared
// memory (one 64-bit add per element, no conflicts, no atomics between lanes); a workgroup folds
// its lanes into (low-half sum, high-half sum) pairs.
//
// Records of kBinWords u64: words 2k, 2k+1 = low/high half sums of bin k, word 32 = non-finite flag.
// A segment's n_slots records are stored word-major (word w of slot i at [w * n_slots + i]) so that
// the kernel that adds them up reads consecutive addresses.
//   single gradient : every workgroup stores its one record in slot blockIdx.x (plain stores, so
//                     nothing has to be cleared beforehand), and the launch also clears the control
//                     words and counters the later kernels rely on;
//   batch           : a workgroup owns a contiguous run of tiles and adds a record to one of n_slots
//                     copies of the segment's record each time it leaves a segment (atomics on
//                     memory k_init cleared).
constexpr u32 kBinWords = 2 * kBins + 2;
#ifndef FSGD_KEEP_MB
#define FSGD_KEEP_MB 160
#endif
constexpr u64 kKeepTiles = (u64)FSGD_KEEP_MB * 64;     // 16 KB a tile: what the first value pass leaves in the caches

template <bool SINGLE>
__device__ __forceinline__ void flush_bins(u64 (*bins)[kThreads], u64* rec, u32 n_slots, u32 maxa) {
    __syncthreads();
    const u32 t = threadIdx.x;
    const u32 bin = t >> 4, part = t & 15u;          // 16 threads per bin, 16 lanes each
    u64 lo = 0, hi = 0;
#pragma unroll
    for (u32 k = 0; k < 16; ++k) {
        u64 x = bins[bin][part * 16u + k];
        lo += x & 0xFFFFFFFFull;
        hi += x >> 32;
    }
#pragma unroll
    for (u32 d = 8; d >= 1; d >>= 1) {
        lo += __shfl_xor((unsigned long long)lo, d, 16);
        hi += __shfl_xor((unsigned long long)hi, d, 16);
    }
    const bool bad = __syncthreads_or(maxa >= 0x7F800000u);
    const u64 ns = n_slots;
    if (SINGLE) {
        if (part == 0) { rec[(2 * bin) * ns] = lo; rec[(2 * bin + 1) * ns] = hi; }
        if (t == 0) { rec[(2 * kBins) * ns] = bad ? 1u : 0u; rec[(2 * kBins + 1) * ns] = 0; }
    } else {
        if (part == 0) {
            if (lo) atomicAdd((unsigned long long*)&rec[(2 * bin) * ns], (unsigned long long)lo);
            if (hi) atomicAdd((unsigned long long*)&rec[(2 * bin + 1) * ns], (unsigned long long)hi);
        }
        if (bad && t == 0) atomicOr((unsigned long long*)&rec[(2 * kBins) * ns], 1ull);
#pragma unroll
        for (u32 b = 0; b < kBins; ++b) bins[b][t] = 0;
        __syncthreads();
    }
}

// Also stores, for each of the wave's four rows of the tile that exist (row index below row_end), the
// largest |v| of each granule of the row (kGranule values: the float4s of kGranLanes neighbouring lanes):
// the upper 16 bits of its bit pattern, rounded up, so that the stored bound is never below the true
// maximum.  The second pass skips every granule whose bound is below the threshold.  rowmax points at
// the bounds of the tile's first row; trow0 is that row's index.
// With `stage` set the bounds of the wave's four rows (16 words) go there, in shared memory, instead of
// to rowmax (the caller writes them out many tiles at a time).
__device__ __forceinline__ void accumulate_tile(const u32 bits[4][4], u64 (*bins)[kThreads], u32& maxa,
                                                uint16_t* __restrict__ rowmax, u64 trow0, u64 row_end,
                                                u32* stage = nullptr) {
    const u32 t = threadIdx.x;
#pragma unroll
    for (u32 r = 0; r < 4; ++r) {
        u32 m = bits[r][0] & 0x7FFFFFFFu;
#pragma unroll
        for (u32 c = 1; c < 4; ++c) { const u32 a = bits[r][c] & 0x7FFFFFFFu; m = a > m ? a : m; }
        maxa = m > maxa ? m : maxa;
        u32 y;                                              // maximum over the kGranLanes lanes up to this one
        y = dpp_mov<kDppRowShr1>(0u, m); m = m > y ? m : y;
        y = dpp_mov<kDppRowShr2>(0u, m); m = m > y ? m : y;
        y = dpp_mov<kDppRowShr4>(0u, m); m = m > y ? m : y;
        const u32 wr = wave_id() * 4u + r;
        if (kGranLanes == 16) {
            y = dpp_mov<kDppRowShr8>(0u, m); m = m > y ? m : y;
            if ((lane_id() & 15u) == 15u && trow0 + wr < row_end)
                rowmax[wr * kRowGranules + (lane_id() >> 4)] = (uint16_t)((m + 0xFFFFu) >> 16);   // m < 2^31: no overflow
        } else {
            // lanes 7 and 15 of every 16 hold a bound each: lane 15 stores the pair as one word
            const u32 b16 = (m + 0xFFFFu) >> 16;
            y = dpp_mov<kDppRowShr8>(0u, b16);
            if (stage) {
                if ((lane_id() & 15u) == 15u) stage[r * (kRowGranules / 2u) + (lane_id() >> 4)] = y | (b16 << 16);
            } else if ((lane_id() & 15u) == 15u && trow0 + wr < row_end) {
                reinterpret_cast<u32*>(rowmax)[wr * (kRowGranules / 2u) + (lane_id() >> 4)] = y | (b16 << 16);
            }
        }
    }
#pragma unroll
    for (u32 r = 0; r < 4; ++r)
#pragma unroll
        for (u32 c = 0; c < 4; ++c) {
            const u32 a = bits[r][c] & 0x7FFFFFFFu;
            const u32 e = a >> 23;
            const u32 e1 = e ? e : 1u;
            const u32 m = a - ((e1 - 1u) << 23);          // significand with its leading one (none for denormals)
            const u64 val = (u64)m << (e1 & 15u);
            // a NaN/Inf lands in bin 15 as garbage; the record's flag makes the whole sum void
            atomicAdd((unsigned long long*)&bins[e1 >> 4][t], (unsigned long long)val);
        }
}

constexpr u32 kWaveTileWords = 4 * kRowGranules / 2;   // 32-bit words of bounds a wave produces per tile (four rows)
constexpr u32 kBoundStage = 16;                         // tiles whose bounds a workgroup collects before writing them
static_assert(kWaves * kWaveTileWords * 4 == 256 && kBoundStage * 16 == kThreads, "one 16-byte part per thread when the bounds leave");

template <bool SINGLE>
__global__ void __launch_bounds__(kThreads)
k_abs_sum(const float* __restrict__ values, const SegInfo* __restrict__ segs, u32 n_segments, u64 n_tiles,
          u64* gbins, u32 n_slots, u64* zero_begin, u64 zero_words, SegInfo single_seg, SegInfo* seg_store,
          uint16_t* __restrict__ rowmax) {
    __shared__ u64 bins[kBins][kThreads];
    __shared__ __attribute__((aligned(16))) u32 s_bounds[SINGLE ? kBoundStage : 1][kWaves * kWaveTileWords];
    const u32 t = threadIdx.x;
#pragma unroll
    for (u32 b = 0; b < kBins; ++b) bins[b][t] = 0;
    if (SINGLE) {
        for (u64 i = (u64)blockIdx.x * kThreads + t; i < zero_words; i += (u64)gridDim.x * kThreads) zero_begin[i] = 0;
        if (blockIdx.x == 0 && t == 0) seg_store[0] = single_seg;
    }
    __syncthreads();
    u32 maxa = 0;
    const u64 G = gridDim.x;
    const u64 per_wg = (n_tiles + G - 1) / G;
    if (SINGLE) {
        // The bounds of the workgroup's tiles (256 bytes a tile) wait in shared memory and leave
        // kBoundStage tiles at a time, in one store instruction: single words written between the loads
        // of a streaming read cost far more than their bytes.  (Rows behind the last row of the array get
        // bounds too, of zero; the bounds array has room for a whole last tile.)
        const TileGeom g0 = tile_geom(single_seg, 0);
        const u64 row_end = segment_rows(single_seg);
        u64 it0 = 0;                                          // iteration of the first tile waiting
        u32 waiting = 0;
        auto write_bounds = [&]() {
            __syncthreads();
            const u32 piece = t >> 4, part = t & 15u;         // a tile's bounds: sixteen 16-byte parts
            if (piece < waiting) {
                const u64 tile = (it0 + piece) * G + blockIdx.x;
                uint4* dst = reinterpret_cast<uint4*>(rowmax + tile * (kRowGranules * kTile / kRow));
                dst[part] = reinterpret_cast<const uint4*>(s_bounds[piece])[part];
            }
            __syncthreads();
            it0 += waiting;
            waiting = 0;
        };
        for (u64 it = 0; it < per_wg; ++it) {
            const u64 tile = it * G + blockIdx.x;             // neighbours in time are neighbours in memory
            if (tile >= n_tiles) break;
            TileGeom g = g0;
            g.tile0 += tile * kTile;
            g.full = (g.tile0 >= g.lo) && (g.tile0 + kTile <= g.hi);
            u32 bits[4][4];
            load_tile(values, g, bits, tile + kKeepTiles >= n_tiles);
            accumulate_tile(bits, bins, maxa, rowmax, tile * (kTile / kRow), row_end, s_bounds[waiting] + wave_id() * kWaveTileWords);
            if (++waiting == kBoundStage) write_bounds();
        }
        if (waiting) write_bounds();
        flush_bins<true>(bins, gbins + blockIdx.x, n_slots, maxa);
    } else {
        u32 cur_seg = 0xFFFFFFFFu;
        const u64 t_begin = blockIdx.x * per_wg;
        const u64 t_end = (t_begin + per_wg < n_tiles) ? t_begin + per_wg : n_tiles;
        SegInfo info = single_seg;                            // (overwritten before use)
        u64 seg_tile_end = 0, seg_rows = 0;                   // first tile behind the segment in hand, its rows
        for (u64 tile = t_begin; tile < t_end; ++tile) {
            if (tile >= seg_tile_end) {                       // the segment is looked up only when a tile leaves it
                const u32 seg = find_tile_segment(segs, n_segments, (u32)tile);
                if (cur_seg != 0xFFFFFFFFu) {
                    flush_bins<false>(bins, gbins + (u64)cur_seg * n_slots * kBinWords + blockIdx.x % n_slots, n_slots, maxa);
                    maxa = 0;
                }
                cur_seg = seg;
                info = segs[seg];
                seg_rows = segment_rows(info);
                seg_tile_end = info.tile_begin + (seg_rows * kRow + kTile - 1) / kTile;
            }
            const TileGeom g = tile_geom(info, tile);
            u32 bits[4][4];
            load_tile(values, g, bits);
            const u64 trow0 = (tile - info.tile_begin) * (kTile / kRow);
            accumulate_tile(bits, bins, maxa, rowmax + (u64)kRowGranules * (info.row_begin + trow0), trow0, seg_rows);
        }
        if (cur_seg != 0xFFFFFFFFu)
            flush_bins<false>(bins, gbins + (u64)cur_seg * n_slots * kBinWords + blockIdx.x % n_slots, n_slots, maxa);
    }
}

// ---------------------------------------------------------------------------------------------
// One workgroup per segment: add up the segment's records, fold the bins into a 384-bit integer
// counting units of 2^-150, round once to binary64 (nearest, ties to even), then the boundary table.
// The fold runs on 32-bit digits: bin word w (a sum below 2^60 at bit position 16*(w/2) + 32*(w%2))
// is split over three digits and added by shared-memory atomics; one thread then propagates the
// carries.  A second wave walks the power chain b^c meanwhile.
constexpr u32 kTableThreads = 1024;
constexpr u32 kDigits = 12;

__global__ void __launch_bounds__(kTableThreads)
k_tables(const SegInfo* __restrict__ segs, SegState* __restrict__ states, const u64* __restrict__ gbins,
         u32 n_slots, Ctrl* ctrl) {
    __shared__ u64 s_tot[kBinWords];
    __shared__ unsigned long long s_dig[kDigits];
    __shared__ double s_P[kMaxTau + 1];
    __shared__ double s_sum;
    __shared__ u32 s_bad;
    const u32 seg = blockIdx.x, t = threadIdx.x;
    const SegInfo info = segs[seg];
    SegState* st = &states[seg];
    if (t < kDigits) s_dig[t] = 0;
    if (t == 0) s_bad = 0;
    {
        // wave v adds up words v, v + 16, v + 32 over all slots: 16 coalesced loads per lane in flight,
        // a sum inside the lane, one reduction across the wave per word
        const u64* g = gbins + (u64)seg * n_slots * kBinWords;
        const u32 lane = lane_id();
        for (u32 w = wave_id(); w < kBinWords; w += kTableThreads / 64) {
            const u64* gw = g + (u64)w * n_slots;
            u64 acc = 0;
            for (u32 base = 0; base < n_slots; base += 1024) {
                u64 x[16];
#pragma unroll
                for (u32 j = 0; j < 16; ++j) {
                    const u32 sl = base + j * 64u + lane;
                    x[j] = gw[sl < n_slots ? sl : n_slots - 1];
                }
#pragma unroll
                for (u32 j = 0; j < 16; ++j) acc += (base + j * 64u + lane < n_slots) ? x[j] : 0ull;
            }
            const u64 tot = wave_sum64(acc);
            if (lane == 63) s_tot[w] = tot;
        }
    }
    __syncthreads();
    if (t == 64) power_chain(info.base, info.tau, s_P);
    if (t < kBinWords) {
        const u64 x = s_tot[t];
        if (t < 2 * kBins) {
            const u32 bitpos = 16u * (t >> 1) + 32u * (t & 1u);
            const u32 q = bitpos >> 5, sh = bitpos & 31u;         // sh is 0 or 16
            const u64 lo = x << sh, hi = sh ? (x >> (64u - sh)) : 0ull;
            if (lo & 0xFFFFFFFFull) atomicAdd(&s_dig[q], (unsigned long long)(lo & 0xFFFFFFFFull));
            if (lo >> 32) atomicAdd(&s_dig[q + 1], (unsigned long long)(lo >> 32));
            if (hi) atomicAdd(&s_dig[q + 2], (unsigned long long)hi);
        } else if (t == 2 * kBins && x != 0) {
            s_bad = 1;
        }
    }
    __syncthreads();
    if (t == 0) {
        u64 L[6];
        u64 carry = 0;
#pragma unroll
        for (u32 i = 0; i < kDigits; i += 2) {
            const u64 v0 = s_dig[i] + carry;
            const u64 v1 = s_dig[i + 1] + (v0 >> 32);
            carry = v1 >> 32;
            L[i >> 1] = (v0 & 0xFFFFFFFFull) | (v1 << 32);
        }
        int hi_i = -1;
#pragma unroll
        for (int i = 0; i < 6; ++i) if (L[i]) hi_i = i;
        double sum = 0.0;
        if (hi_i >= 0) {
            u64 hi = 0, lo = 0;
            bool below = false;                       // any set bit in limbs under `lo`
#pragma unroll
            for (int i = 0; i < 6; ++i) {
                if (i == hi_i) hi = L[i];
                if (i + 1 == hi_i) lo = L[i];
                if (i + 1 < hi_i && L[i]) below = true;
            }
            const u32 s = 63u - (u32)__builtin_clzll(hi);       // top bit inside its limb
            const int top = hi_i * 64 + (int)s;
            // 64-bit window whose most significant bit is the sum's leading one
            const u64 W = (s == 63u) ? hi : ((hi << (63u - s)) | (lo >> (s + 1u)));
            const bool lost = below || (s != 63u && (lo & ((1ull << (s + 1u)) - 1ull)) != 0);
            u64 q = W >> 11;                                    // 53 significant bits
            const bool guard = (W >> 10) & 1ull;
            const bool sticky = (W & 0x3FFull) != 0 || lost;
            if (guard && (sticky || (q & 1ull))) ++q;           // q = 2^53 carries into the exponent below
            const u64 bits = ((u64)(top - 150 + 1023) << 52) + (q - (1ull << 52));
            sum = __longlong_as_double((long long)bits);
        }
        const bool bad = s_bad != 0;
        if (bad) set_status(ctrl, FASTSGD_ERR_NONFINITE);
        st->sum = bad ? 0.0 : sum;
        s_sum = bad ? 0.0 : sum;
        // for the value pass's first guess of a code, ceil(log_b(sum / |v|)) in binary32
        st->lg_sum = (sum > 0.0 && !bad) ? (float)log2(sum) : 0.0f;
        st->inv_lg_base = (float)(1.0 / log2(info.base));
    }
    __syncthreads();
    const double sum = s_sum;
    if (t >= 1 && t <= info.tau) {
        u32 b = 0xFFFFFFFFu;
        if (sum > 0.0) b = f64_to_f32_bits(sum / s_P[t], true);
        st->B[t - 1] = b;
        if (t == info.tau) st->thr_bits = b;
    }
}

// ---------------------------------------------------------------------------------------------
// Second pass over the values (Algorithm 1 lines 4-10).  No wave depends on another.  The elements of
// a call are cut into chunks of R rows (a row = 256 elements, a float4 per lane); every WAVE owns one
// chunk:
//   the bounds the first pass left behind, one per granule (32 elements = 128 bytes, the share of 8
//   lanes), tell which granules can hold a survivor at all (the early-stop test of Algorithm 1 line 5
//   applied to a whole granule); only those are read, and they are read as one ascending stream: a batch
//   is eight rows of 256 elements, each made of the next eight granules of the stream wherever they sit,
//   so that every lane fetches something useful however few granules are in play -> per row, keep
//   test |v| >= threshold as four wave-wide masks -> survivors are staged in the wave's slice of shared
//   memory in element order (mask popcounts + mbcnt) -> once a round of 256 waits there, densely over
//   the staged survivors only and in whole rounds: key fetch, code by binary search in the boundary
//   table -> code and key appended to the CHUNK'S OWN SLOT of the scratch arrays (the chunk's first
//   element index + rank in the chunk).  The key fetches are issued right behind the loads of the next
//   batch and used two rows later, so the two round trips overlap.
// The chunk's survivor count goes to ccount[chunk].  Global ranks are never materialised: k_plan_segments
// turns the (at most 4096) chunk counts of a segment into their scan and the key encoder gathers through
// that scan.
constexpr u32 kStage = 1024;             // staged survivors per wave (a ring of 8-byte entries)
constexpr u32 kRing = 512;               // ring of granules per wave: under a batch left over plus 256 from a top-up
constexpr u32 kValWaves = 4;             // waves per workgroup of the value encoder (they never synchronise)
constexpr u32 kGather = 4;               // survivors a lane handles per round of a flush: four CONSECUTIVE ones
static_assert((kRing & (kRing - 1)) == 0 && kRing >= kRowGranules * kValRows - 1 + 4 * 64, "ring: a short batch plus 256 granules");
static_assert(kMaxChunkRows * kRowGranules <= 65536 && kMaxChunkRows % kValRows == 0 && kRowGranules % 4 == 0,
              "ring entries are 16 bits; bounds come in groups of four");
constexpr u32 kRound = 64 * kGather;     // survivors per round of a flush
static_assert((kStage & (kStage - 1)) == 0 && kStage % kRound == 0 && kStage >= 2 * kRow + kRound,
              "stage: a power of two, whole rounds, a forced flush sends at least one");
static_assert(4 * kMaxTau + 8 * kStage + 2 * kRing <= 10240, "shared memory for sixteen waves per compute unit");
#ifndef FSGD_DENSE_ROWS
#define FSGD_DENSE_ROWS 2
#endif
static_assert(FSGD_DENSE_ROWS * kRow + kRound <= kStage, "a batch of rows on top of what a flush leaves");
constexpr u32 kDenseNum = 3, kDenseDen = 4;   // a chunk is walked row by row if this share of its granules can hold a survivor

// |v| >= threshold as a float compare with the |x| source modifier: for non-negative finite floats
// (denormals are preserved in this build) it orders exactly like the unsigned compare of the bit
// patterns, and a NaN threshold (bit pattern 0xFFFFFFFF = keep nothing) compares false.
__device__ __forceinline__ bool keeps(u32 value_bits, float threshold) {
    return __builtin_fabsf(__uint_as_float(value_bits)) >= threshold;
}

__device__ __forceinline__ u32 lanes_below(u64 mask, u32 add) {
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, add));
}

struct Chunk {           // wave-uniform description of the chunk a wave owns
    u32 seg, nrows;
    u32 row0;            // index of the chunk's first row in the call's row numbering
    u64 e0;              // element index of the chunk's first slot
    u64 slot0;           // scratch entry of the chunk's first survivor
    u64 lo, hi;          // valid elements [lo, hi) of the segment
};

// Scratch entry of the first slot of a segment's chunk j.  Segment s is shifted by 4*s entries so
// that the rounding-down of its first element can never reach into its predecessor's entries.
__device__ __forceinline__ u64 chunk_slot0(const SegInfo& s, u32 seg, u32 j, u32 R) {
    return (s.elem_begin & ~3ull) + (u64)j * R * kRow + 4ull * seg;
}

__device__ __forceinline__ Chunk chunk_geom(const SegInfo* __restrict__ segs, u32 n_segments, u32 chunk, u32 R) {
    Chunk c;
    c.seg = (n_segments == 1) ? 0u : find_chunk_segment(segs, n_segments, chunk);
    const SegInfo s = segs[c.seg];
    const u32 j = chunk - s.chunk_begin;
    const u64 rows = segment_rows(s), r0 = (u64)j * R;
    c.nrows = (u32)(rows - r0 < R ? rows - r0 : R);
    c.row0 = s.row_begin + (u32)r0;
    c.e0 = (s.elem_begin & ~3ull) + r0 * kRow;
    c.slot0 = chunk_slot0(s, c.seg, j, R);
    c.lo = s.elem_begin;
    c.hi = s.elem_begin + s.elem_count;
    return c;
}

// What a wave of the value pass knows about its chunk and its call (wave-uniform unless said otherwise).
struct ValueCtx {
    Chunk ck;
    u32 lane;                          // (per lane)
    const u32* s_B;                    // shared memory: [c - 1] = boundary of code c
    uint2* s_ent;                      // shared memory: staged survivors (value bits, tag), a ring of kStage
    uint16_t* s_ring;                  // shared memory: granules still to be read
    u32 thr, tau;
    float thr_f, lg_sum, inv_lg_base;
    const u32* keys;                   // the call's key array (nullptr: keys are the indices) ...
    const float* values;               // ... and value array, both counted from the aligned base
    const u32* ckeys;                  // the chunk's first key / value
    const float* cvals;
    u32 key0;                          // key of the chunk's first element where keys are the indices
    const uint2* crmax;                // the chunk's granule bounds, in groups of four
    u32 nwords;                        // ... and how many groups
    u32* skeys;
    void* scodes;
};

// which of the four bounds of a group reach the threshold (unsigned compare of bit patterns: the same
// order as the float compare, and nothing passes the keep-nothing threshold)
__device__ __forceinline__ u32 live_bits(uint2 x, u32 thr) {
    return ((x.x << 16) >= thr ? 1u : 0u) | ((x.x & 0xFFFF0000u) >= thr ? 2u : 0u) |
           ((x.y << 16) >= thr ? 4u : 0u) | ((x.y & 0xFFFF0000u) >= thr ? 8u : 0u);
}

// One chunk of the second value pass; returns the number of its survivors (in the scratch arrays when the
// function returns).
//
// Survivors wait in a ring of (value bits, tag) entries in the wave's shared memory, in element order; the
// tag is the survivor's key where that is known when it is staged (BY_ROWS, or IMPLICIT: no key array) and
// its element offset in the chunk otherwise (its key is then fetched when it leaves).  They leave in rounds
// of 256, four consecutive ones to a lane: code by a first guess from the binary logarithm of |v| checked
// against the boundary table (two probes; a binary search over the table where the probes do not bracket the
// value), the lane's four codes in one store, its four keys in another.
//
// BY_ROWS: most granules of the chunk can hold a survivor, so the chunk is read row by row, keys alongside the
// values, everything coalesced.  Otherwise granule by granule: only the granules that can hold a survivor, as
// one ascending stream.
// WIDE: some segment of the call has tau > 128; then every survivor's scratch code takes 16 bits (sign
// in bit 15) instead of 8 (sign in bit 7), and the boundary table has up to 256 entries.
template <bool WIDE, bool BY_ROWS, bool IMPLICIT>
__device__ __forceinline__ u32 encode_chunk(const ValueCtx& cx) {
    typedef typename ScratchCode<WIDE>::type CodeT;
    constexpr bool TAG_IS_KEY = BY_ROWS || IMPLICIT;
    CodeT* __restrict__ scodes = static_cast<CodeT*>(cx.scodes);
    u32* __restrict__ skeys = cx.skeys;
    const Chunk& ck = cx.ck;
    const u32 lane = cx.lane, thr = cx.thr, tau = cx.tau;
    const float thr_f = cx.thr_f, lg_sum = cx.lg_sum, inv_lg_base = cx.inv_lg_base;
    const u32* s_B = cx.s_B;
    uint2* s_ent = cx.s_ent;
    const u32* ckeys = cx.ckeys;
    const float* cvals = cx.cvals;
    const u32 key0 = cx.key0;
    u32 cbase = 0;                           // survivors of the chunk already in the scratch arrays
    u32 staged = 0;                          // survivors waiting in shared memory
    u32 first = 0;                           // ring position of the oldest staged survivor (a multiple of kRound)

    // A round of (up to) kRound staged survivors -> scratch arrays.  begin() issues the key fetches of the round
    // that leaves (only where the tags are element offsets), complete() turns values into codes and stores
    // codes and keys.  Where keys have to be fetched the wave stages the next two rows between the two, whose
    // loads were issued before the key fetches: the key fetches arrive right behind them instead of being
    // waited for on their own.  While the chunk goes on only whole rounds leave.
    u32 pending = 0;                         // staged survivors that are leaving (at most kRound)
    u32 pk0 = 0, pk1 = 0, pk2 = 0, pk3 = 0;  // its keys, where they had to be fetched
    auto begin = [&](u32 n_out) {
        wave_lds_sync();
        if (!TAG_IS_KEY) {
            const uint4* e4 = reinterpret_cast<const uint4*>(s_ent + first) + 2u * lane;
            const uint4 x = e4[0], y = e4[1];
            const u32 j = kGather * lane;
            pk0 = (j + 0u < n_out) ? ckeys[x.y] : 0u;
            pk1 = (j + 1u < n_out) ? ckeys[x.w] : 0u;
            pk2 = (j + 2u < n_out) ? ckeys[y.y] : 0u;
            pk3 = (j + 3u < n_out) ? ckeys[y.w] : 0u;
        }
        pending = n_out;
    };
    // the lane's four survivors of the round that leaves: how many of them exist, their codes (sign on top of
    // code - 1, as the scratch array holds them) and keys
    auto round_codes = [&](u32 n_out, u32& have, u32 (&cd)[kGather], u32 (&key)[kGather]) {
        const uint4* e4 = reinterpret_cast<const uint4*>(s_ent + first) + 2u * lane;
        const uint4 x = e4[0], y = e4[1];
        const u32 vb[kGather] = {x.x, x.z, y.x, y.z};
        key[0] = TAG_IS_KEY ? x.y : pk0; key[1] = TAG_IS_KEY ? x.w : pk1;
        key[2] = TAG_IS_KEY ? y.y : pk2; key[3] = TAG_IS_KEY ? y.w : pk3;
        const u32 j = kGather * lane;
        have = j >= n_out ? 0u : (n_out - j < kGather ? n_out - j : kGather);
        // codes: a first guess ceil(log_b(sum / |v|)) in binary32, good to a small fraction of a code, checked
        // against the table (B[c-1] > a >= B[c] settles it); entries beyond the staged ones hold stale bits,
        // they get the threshold's code and are not stored
        bool settled = true;
#pragma unroll
        for (u32 k = 0; k < kGather; ++k) {
            const u32 a = k < have ? (vb[k] & 0x7FFFFFFFu) : thr;
            const float g = (lg_sum - __log2f(__uint_as_float(a))) * inv_lg_base;
            int ci = (int)__builtin_ceilf(g);
            ci = ci < 1 ? 1 : (ci > (int)tau ? (int)tau : ci);
            const u32 c = (u32)ci;
            const u32 below = s_B[c - 1u], above = s_B[c >= 2u ? c - 2u : 0u];
            settled = settled & (a >= below) & (c == 1u || a < above);
            cd[k] = c;
        }
        if (__builtin_expect(__any(!settled), 0)) {
            // somewhere the guess was off (a value next to a boundary, a base next to 1, a denormal): the
            // smallest code c in [1, tau] with a >= B[c] by binary search (B non-increasing, a >= B[tau])
#pragma unroll
            for (u32 k = 0; k < kGather; ++k) {
                const u32 a = k < have ? (vb[k] & 0x7FFFFFFFu) : thr;
                u32 lo = 1, hi = tau;
                while (lo < hi) {
                    const u32 mid = (lo + hi) >> 1;
                    if (a >= s_B[mid - 1]) hi = mid; else lo = mid + 1;
                }
                cd[k] = lo;
                __builtin_amdgcn_sched_barrier(0);        // one search at a time
            }
        }
#pragma unroll
        for (u32 k = 0; k < kGather; ++k) cd[k] = ((vb[k] >> 31) << (WIDE ? 15 : 7)) | (cd[k] - 1u);
    };
    auto round_done = [&](u32 n_out) {
        wave_lds_sync();
        cbase += n_out;
        staged -= n_out;
        first = (first + n_out) & (kStage - 1u);
    };
    auto complete = [&]() {
        const u64 slot = ck.slot0 + cbase;
        u32 have, cd[kGather], key[kGather];
        round_codes(pending, have, cd, key);
        const u32 j = kGather * lane;
        CodeT* cdst = scodes + slot + j;
        u32* kdst = skeys + slot + j;
        if (have == kGather) {
            if (WIDE) *reinterpret_cast<uint2*>(cdst) = make_uint2(cd[0] | (cd[1] << 16), cd[2] | (cd[3] << 16));
            else *reinterpret_cast<u32*>(cdst) = cd[0] | (cd[1] << 8) | (cd[2] << 16) | (cd[3] << 24);
            *reinterpret_cast<uint4*>(kdst) = make_uint4(key[0], key[1], key[2], key[3]);
        } else {
#pragma unroll
            for (u32 k = 0; k < kGather; ++k)
                if (k < have) { cdst[k] = (CodeT)cd[k]; kdst[k] = key[k]; }
        }
        round_done(pending);
        pending = 0;
    };

    // one row of four values per lane: masks, and staging if anything survives
    auto stage_row = [&](const u32 (&row)[4], const u32 (&tag)[4]) {
        u64 m[4];
#pragma unroll
        for (u32 c = 0; c < 4; ++c) m[c] = __ballot(keeps(row[c], thr_f));
        if ((m[0] | m[1] | m[2] | m[3]) == 0) return;
        u32 pos = lanes_below(m[3], lanes_below(m[2], lanes_below(m[1], lanes_below(m[0], first + staged))));
#pragma unroll
        for (u32 c = 0; c < 4; ++c)
            if (keeps(row[c], thr_f)) {
                s_ent[pos & (kStage - 1u)] = make_uint2(row[c], tag[c]);
                ++pos;
            }
        staged += (u32)__popcll(m[0]) + (u32)__popcll(m[1]) + (u32)__popcll(m[2]) + (u32)__popcll(m[3]);
    };
    // whole rounds leave at once: under a round stays, so two more rows always fit (kStage = 4 rows)
    auto flush_rounds = [&]() {
        while (staged >= kRound) {
            begin(kRound);
            complete();
        }
    };

    if constexpr (BY_ROWS) {
        // ---- row by row: row r = elements 256 r + 4 lane .. + 3 of the chunk.  Rows that lie wholly inside
        // the segment (all but, at most, the chunk's first and last) are fetched through buffer descriptors
        // that end with the last of them, so that a batch reaching beyond reads zeros -- which never survive --
        // without a branch; kDenseRows rows are staged while the next kDenseRows are on their way.
        constexpr u32 kDenseRows = FSGD_DENSE_ROWS;
        const u32 nrows = ck.nrows;
        auto row_inside = [&](u32 r) { const u64 e = ck.e0 + (u64)r * kRow; return e >= ck.lo && e + kRow <= ck.hi; };
        // a row cut by the segment's ends: element by element
        auto cut_row = [&](u32 r) {
            u32 vrow[4], tag[4];
#pragma unroll
            for (u32 c = 0; c < 4; ++c) {
                const u32 elem = r * kRow + lane * 4u + c;
                const u64 ee = ck.e0 + elem;
                const bool in = ee >= ck.lo && ee < ck.hi;
                vrow[c] = in ? __float_as_uint(cx.values[ee]) : 0u;       // zero never survives
                tag[c] = IMPLICIT ? key0 + elem : (in ? cx.keys[ee] : 0u);
            }
            stage_row(vrow, tag);
            flush_rounds();
        };
        const u32 rb = row_inside(0) ? 0u : 1u;                               // first and ...
        const u32 re = (nrows > rb && !row_inside(nrows - 1u)) ? nrows - 1u : nrows;   // ... one past the last whole row
        if (rb) cut_row(0);
        if (re > rb) {
            const u32 nfull = re - rb;
            const __amdgpu_buffer_rsrc_t vrs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<float*>(cvals + rb * kRow), 0, (int)(nfull * kRow * 4u), kBufferWord3);
            const __amdgpu_buffer_rsrc_t krs = __builtin_amdgcn_make_buffer_rsrc(
                const_cast<u32*>(IMPLICIT ? reinterpret_cast<const u32*>(cvals) : ckeys + rb * kRow), 0, (int)(nfull * kRow * 4u), kBufferWord3);
            constexpr int kNt = 2;                                             // non-temporal: read once
            u32 va[kDenseRows][4], ka[kDenseRows][4], vb2[kDenseRows][4], kb2[kDenseRows][4];
            auto load_batch = [&](u32 (&v)[kDenseRows][4], u32 (&k)[kDenseRows][4], u32 r) {      // rows rb + r ..
#pragma unroll
                for (u32 s = 0; s < kDenseRows; ++s) {
                    const u32x4 q = __builtin_amdgcn_raw_buffer_load_b128(vrs, (int)(lane * 16u), (int)((r + s) * kRow * 4u), kNt);
                    v[s][0] = q.x; v[s][1] = q.y; v[s][2] = q.z; v[s][3] = q.w;
                    if (!IMPLICIT) {
                        const u32x4 kq = __builtin_amdgcn_raw_buffer_load_b128(krs, (int)(lane * 16u), (int)((r + s) * kRow * 4u), kNt);
                        k[s][0] = kq.x; k[s][1] = kq.y; k[s][2] = kq.z; k[s][3] = kq.w;
                    }
                }
            };
            auto stage_batch = [&](const u32 (&v)[kDenseRows][4], const u32 (&k)[kDenseRows][4], u32 r) {
#pragma unroll
                for (u32 s = 0; s < kDenseRows; ++s) {
                    if (IMPLICIT) {
                        const u32 t0 = key0 + (rb + r + s) * kRow + lane * 4u;
                        const u32 tag[4] = {t0, t0 + 1u, t0 + 2u, t0 + 3u};
                        stage_row(v[s], tag);
                    } else {
                        stage_row(v[s], k[s]);
                    }
                }
            };
            // A whole round leaves, if one is waiting, between the request for the next rows and the wait for
            // the rows in hand.  Its two stores are issued in any case, through buffer descriptors over the
            // chunk's scratch entries, with an offset beyond the descriptor's end when no round leaves (the
            // hardware drops such a store): a wave's loads and stores complete in the order issued, and the
            // compiler counts how many may still be out when it waits for a load; stores that exist on one
            // path only would make every such wait also wait for loads that were only just issued.
            const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
                scodes + ck.slot0, 0, (int)(nrows * kRow * (u32)sizeof(CodeT)), kBufferWord3);
            const __amdgpu_buffer_rsrc_t srs = __builtin_amdgcn_make_buffer_rsrc(
                skeys + ck.slot0, 0, (int)(nrows * kRow * 4u), kBufferWord3);
            constexpr int kDropped = 0x40000000;                       // an offset no chunk reaches
            auto round_leaves = [&]() {
                const bool go = staged >= kRound;
                const u32 at = cbase;
                u32 cd[kGather] = {0u, 0u, 0u, 0u}, key[kGather] = {0u, 0u, 0u, 0u};
                if (go) {
                    u32 have;
                    wave_lds_sync();
                    round_codes(kRound, have, cd, key);
                    round_done(kRound);
                }
                u32x4 kq;
                kq.x = key[0]; kq.y = key[1]; kq.z = key[2]; kq.w = key[3];
                if (WIDE) {
                    typedef u32 u32x2 __attribute__((ext_vector_type(2)));
                    u32x2 cq;
                    cq.x = cd[0] | (cd[1] << 16); cq.y = cd[2] | (cd[3] << 16);
                    __builtin_amdgcn_raw_buffer_store_b64(cq, crs, (int)(lane * 8u), go ? (int)(at * 2u) : kDropped, 0);
                } else {
                    __builtin_amdgcn_raw_buffer_store_b32(cd[0] | (cd[1] << 8) | (cd[2] << 16) | (cd[3] << 24), crs,
                                                          (int)(lane * 4u), go ? (int)at : kDropped, 0);
                }
                __builtin_amdgcn_raw_buffer_store_b128(kq, srs, (int)(lane * 16u), go ? (int)(at * 4u) : kDropped, 0);
            };
            load_batch(va, ka, 0);
            for (u32 r = 0; r < nfull; r += 2u * kDenseRows) {
                load_batch(vb2, kb2, r + kDenseRows);
                round_leaves();
                while (staged >= kRound) round_leaves();               // (more than half of the values survive)
                stage_batch(va, ka, r);
                load_batch(va, ka, r + 2u * kDenseRows);
                round_leaves();
                while (staged >= kRound) round_leaves();
                stage_batch(vb2, kb2, r + kDenseRows);
            }
            flush_rounds();
        }
        if (re < nrows) cut_row(nrows - 1u);
    } else {
        // ---- granule by granule.  The unit of the fetch is the granule: a batch is eight "virtual rows" of
        // kRowGranules granules that can hold a survivor, taken in ascending order from wherever they sit, so
        // that every lane fetches something useful however few granules are in play.
        // One virtual row: lanes kGranLanes g .. kGranLanes (g + 1) - 1 fetch the g-th of its granules; `elem`
        // is the chunk-relative element offset of the lane's first element.  Granules cut by the segment's ends
        // are fetched element by element; elements outside [lo, hi) become zero, which never survives.
        uint16_t* s_ring = cx.s_ring;
        const uint2* crmax = cx.crmax;
        const u32 nwords = cx.nwords;
        auto load_granules = [&](bool on, u32 elem, u32 (&row)[4]) {
            const u64 e = ck.e0 + elem;
            const bool inside = e >= ck.lo && e + 4u <= ck.hi;
            uint4 q = make_uint4(0u, 0u, 0u, 0u);
            if (__all(inside || !on)) {
                if (on) q = *reinterpret_cast<const uint4*>(cvals + elem);
                row[0] = q.x; row[1] = q.y; row[2] = q.z; row[3] = q.w;
            } else {
#pragma unroll
                for (u32 c = 0; c < 4; ++c) {
                    const u64 ee = e + c;
                    row[c] = (on && ee >= ck.lo && ee < ck.hi) ? __float_as_uint(cx.values[ee]) : 0u;
                }
            }
        };
        auto stage_granules = [&](const u32 (&row)[4], u32 elem) {
            const u32 t0 = IMPLICIT ? key0 + elem : elem;
            const u32 tag[4] = {t0, t0 + 1u, t0 + 2u, t0 + 3u};
            stage_row(row, tag);
        };
        // after every two rows of the granule stream; `loads_issued`: the next batch's loads have just been issued
        auto flush_step = [&](bool loads_issued) {
            if (pending) complete();
            while (staged > kStage - 2 * kRow) {                   // no room for two more rows: at once
                begin(kRound);
                complete();
            }
            if (loads_issued && staged >= kRound) begin(kRound);
        };

        // The granules (kGranule values, the share of kGranLanes lanes) that can hold a survivor form one
        // ascending stream over the chunk, kept in a ring in shared memory (entry = index of the granule inside
        // the chunk).  The ring is topped up 256 granules at a time: lane j compares four bounds, those of the
        // granules 4 (scanned + j) .. + 3, with the threshold.  The bounds of the 256 granules after those are
        // fetched meanwhile.
        uint2 xnext = crmax[lane < nwords ? lane : nwords - 1u];
        u32 scanned = 0;                          // groups of four bounds whose granules are in the ring or behind it
        u32 head = 0, tail = 0;                   // granules taken from / put into the ring since the start
        auto refill = [&]() {
            const uint2 x = xnext;
            const u32 word = scanned + lane;
            scanned += 64u;
            if (scanned < nwords) {
                const u32 wn = scanned + lane;
                xnext = crmax[wn < nwords ? wn : nwords - 1u];
            }
            u32 qb = live_bits(x, thr);
            if (word >= nwords) qb = 0;
            const u32 mine = (u32)__popc(qb);
            const u32 incl = wave_incl_scan(mine);
            u32 at = tail + incl - mine;
#pragma unroll
            for (u32 q = 0; q < 4; ++q)
                if ((qb >> q) & 1u) s_ring[(at++) & (kRing - 1u)] = (uint16_t)((word << 2) | q);
            tail += read_lane(incl, 63);
        };
        // A batch is eight rows of 256 elements in flight, each put together from the next kRowGranules
        // granules of the stream (lanes kGranLanes k .. kGranLanes (k + 1) - 1 take the k-th of them).
        constexpr u32 kBatch = kRowGranules * kValRows;
        auto take = [&](u32 (&elem)[kValRows], u32 (&on)[kValRows]) -> u32 {
            if (tail - head < kBatch && scanned < nwords) {
                do refill(); while (tail - head < kBatch && scanned < nwords);
                wave_lds_sync();
            }
            const u32 left = tail - head;
            const u32 nq = left < kBatch ? left : kBatch;
#pragma unroll
            for (u32 slot = 0; slot < kValRows; ++slot) {
                const u32 i = kRowGranules * slot + lane / kGranLanes;
                on[slot] = i < nq ? 1u : 0u;
                const u32 e = on[slot] ? s_ring[(head + i) & (kRing - 1u)] : 0u;
                elem[slot] = e * kGranule + (lane & (kGranLanes - 1u)) * 4u;
            }
            head += nq;
            return (nq + kRowGranules - 1u) / kRowGranules;
        };
        u32 bits[kValRows][4], elem[kValRows], on[kValRows];
        u32 nr = take(elem, on);
#pragma unroll
        for (u32 slot = 0; slot < kValRows; ++slot) if (slot < nr) load_granules(on[slot] != 0, elem[slot], bits[slot]);
        while (nr) {
#pragma unroll
            for (u32 pair = 0; pair < kValRows / 2; ++pair) {
#pragma unroll
                for (u32 slot = 2 * pair; slot < 2 * pair + 2; ++slot) if (slot < nr) stage_granules(bits[slot], elem[slot]);
                if (pair + 1 == kValRows / 2) {
                    // the registers are free: start on the next rows before finishing these
                    nr = take(elem, on);
#pragma unroll
                    for (u32 slot = 0; slot < kValRows; ++slot)
                        if (slot < nr) load_granules(on[slot] != 0, elem[slot], bits[slot]);
                }
                flush_step(pair + 1 == kValRows / 2);
            }
        }
    }
    if (pending) complete();
    while (staged) {
        begin(staged < kRound ? staged : kRound);
        complete();
    }
    return cbase;
}

// Second pass over the values, one wave per chunk (see encode_chunk).
template <bool WIDE>
__global__ void __launch_bounds__(kValWaves * kWave) __attribute__((amdgpu_waves_per_eu(4, 8)))
k_encode_values(const u32* __restrict__ keys, const float* __restrict__ values,
                const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
                u32 n_chunks, u32 R, const uint16_t* __restrict__ rowmax, u32* __restrict__ ccount,
                u32* __restrict__ skeys, void* __restrict__ scodes_any) {
    constexpr u32 kTable = WIDE ? kMaxTau : 128u;
    __shared__ u32 s_Ball[kValWaves][kTable];               // [c - 1] = boundary of code c
    __shared__ __attribute__((aligned(16))) uint2 s_entall[kValWaves][kStage];
    __shared__ uint16_t s_ringall[kValWaves][kRing];        // granules still to be read, in ascending order
    const u32 lane = lane_id();
    const u32 w = uniform(wave_id());
    u32* s_B = s_Ball[w];
    // (chunks from the array's end to its beginning: the end is what the first pass read last)
    const u32 chunk_raw = blockIdx.x * kValWaves + w;
    if (chunk_raw >= n_chunks) return;
    const u32 chunk = n_chunks - 1u - chunk_raw;
    ValueCtx cx;
    cx.ck = chunk_geom(segs, n_segments, chunk, R);
    const SegState* st = &states[cx.ck.seg];
    cx.lane = lane;
    cx.s_B = s_B;
    cx.s_ent = s_entall[w];
    cx.s_ring = s_ringall[w];
    cx.thr = uniform(st->thr_bits);
    cx.tau = segs[cx.ck.seg].tau;
    cx.thr_f = __uint_as_float(cx.thr);
    cx.lg_sum = st->lg_sum;
    cx.inv_lg_base = st->inv_lg_base;
#pragma unroll
    for (u32 k = 0; k < kTable / 64u; ++k) s_B[lane + 64u * k] = st->B[lane + 64u * k];
    cx.keys = keys;
    cx.values = values;
    cx.ckeys = keys + cx.ck.e0;
    cx.cvals = values + cx.ck.e0;
    cx.key0 = (u32)(cx.ck.e0 - cx.ck.lo);                   // (wraps for the up to three slots before the segment)
    // bounds in groups of four (16 bits each): kRowGranules / 4 such groups per row
    cx.crmax = reinterpret_cast<const uint2*>(rowmax) + (u64)cx.ck.row0 * (kRowGranules / 4u);
    cx.nwords = cx.ck.nrows * (kRowGranules / 4u);
    cx.skeys = skeys;
    cx.scodes = scodes_any;
    const bool implicit = keys == nullptr;                  // dense gradient: the key is the index in the segment
    // How the chunk is read: row by row if at least kDenseNum / kDenseDen of its granules can hold a
    // survivor (that needs the keys 16-byte aligned like the values, or no key array at all).
    bool by_rows = false;
    if (implicit || (((uintptr_t)cx.ckeys & 15u) == 0)) {
        u32 live = 0;
        for (u32 i = lane; i < cx.nwords; i += 64u) live += (u32)__popc(live_bits(cx.crmax[i], cx.thr));
        live = wave_sum(live);
        by_rows = live * kDenseDen >= cx.nwords * 4u * kDenseNum;
    }
    wave_lds_sync();
    u32 count;
    if (by_rows) count = implicit ? encode_chunk<WIDE, true, true>(cx) : encode_chunk<WIDE, true, false>(cx);
    else count = implicit ? encode_chunk<WIDE, false, true>(cx) : encode_chunk<WIDE, false, false>(cx);
    if (lane == 0) ccount[chunk] = count;
}

// ---------------------------------------------------------------------------------------------
// One workgroup per segment turns the segment's chunk counts, in place, into their exclusive scan
// P[j] = survivors of the segment in its chunks before j (the table through which the key encoder
// finds rank r: chunk j with P[j] <= r < P[j+1]), and notes the segment's survivors d and key blocks.
// Batch calls then number the key encoder's work (k_number_segments): a work item is one key block (a
// segment without survivors still has one item, which carries its header); a work unit is kWaves
// consecutive items of one segment, the share of one workgroup iteration.
__global__ void __launch_bounds__(kThreads)
k_plan_segments(const SegInfo* __restrict__ segs, SegState* __restrict__ states, u32 n_segments, u32 R,
                u32* __restrict__ ccount, Ctrl* ctrl) {
    __shared__ u32 s_scan[kWaves + 1];
    const u32 t = threadIdx.x;
    {
        constexpr u32 PER = kMaxSegChunks / kThreads;
        const u32 seg = blockIdx.x;
        const SegInfo info = segs[seg];
        const u32 nch = info.elem_count ? (u32)((segment_rows(info) + R - 1) / R) : 0u;
        u32* P = ccount + info.chunk_begin;
        u32 v[PER], sum = 0;
#pragma unroll
        for (u32 k = 0; k < PER; ++k) {                 // no condition on the loads: all in flight at once
            const u32 j = t * PER + k;
            const u32 x = nch ? P[j < nch ? j : 0u] : 0u;
            v[k] = (j < nch) ? x : 0u;
        }
#pragma unroll
        for (u32 k = 0; k < PER; ++k) sum += v[k];
        u32 total;
        u32 run = block_excl_scan(sum, s_scan, &total);
#pragma unroll
        for (u32 k = 0; k < PER; ++k) {
            const u32 j = t * PER + k;
            if (j < nch) P[j] = run;
            run += v[k];
        }
        if (t == 0) {
            const u32 nb = (u32)(((u64)total + info.block_keys - 1) / info.block_keys);
            states[seg].d = total;
            states[seg].nb = nb;
            if (gridDim.x == 1) {                       // a single gradient: nothing to number
                states[seg].item_begin = 0;
                states[seg].unit_begin = 0;
                ctrl->total_items = nb ? nb : 1u;
                ctrl->total_units = ((nb ? nb : 1u) + kWaves - 1) / kWaves;
            }
        }
    }
}

// Batch calls: numbers the key encoder's work over the segments (one workgroup; a launch of its own, so
// that the per-segment workgroups of k_plan_segments need no fence and no counter).
__global__ void __launch_bounds__(kThreads)
k_number_segments(SegState* __restrict__ states, u32 n_segments, Ctrl* ctrl) {
    __shared__ u64 s_wave[2][kWaves];
    __shared__ u64 s_carry[2];
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    if (t < 2) s_carry[t] = 0;
    __syncthreads();
    for (u32 s0 = 0; s0 < n_segments; s0 += kThreads) {
        const u32 s = s0 + t;
        u64 items = 0, units = 0;
        if (s < n_segments) {
            const u32 nb = states[s].nb;
            items = nb ? nb : 1u;
            units = (items + kWaves - 1) / kWaves;
        }
        const u64 ii = wave_incl_scan64(items), iu = wave_incl_scan64(units);
        if (lane == 63) { s_wave[0][w] = ii; s_wave[1][w] = iu; }
        __syncthreads();
        u64 bi = s_carry[0], bu = s_carry[1], ti = 0, tu = 0;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            const u64 a = s_wave[0][k], b = s_wave[1][k];
            if (k < w) { bi += a; bu += b; }
            ti += a; tu += b;
        }
        if (s < n_segments) {
            states[s].item_begin = bi + ii - items;
            states[s].unit_begin = bu + iu - units;
        }
        __syncthreads();
        if (t == 0) { s_carry[0] += ti; s_carry[1] += tu; }
        __syncthreads();
    }
    if (t == 0) { ctrl->total_items = s_carry[0]; ctrl->total_units = s_carry[1]; }
}

// ---------------------------------------------------------------------------------------------
// Algorithm 2 on one block of surviving keys per WAVE, in two launches:
//   k_measure_keys  first loop of Algorithm 2 (deltas, maxDelta -> M), the size of the block's planes,
//                   and the sum of those sizes per group of 2^g_shift blocks (atomics);
//   k_pack_keys     byte offset of the block (scan of the group sums in shared memory + the sizes of
//                   the blocks before it in its group), second loop (length flags, bit packing),
//                   directory entry, header, value plane.
// Both fetch a block's keys through the scan P of the segment's chunk counts (left in place of the
// counts by k_plan_segments; 16 KB at most, so it stays in the L2): rank r of the segment lives in the
// chunk j with P[j] <= r < P[j+1], at entry chunk_slot0(j) + (r - P[j]) of the scratch arrays.
// A wave takes the block 1024 keys at a time; lane `lane` holds, for row k = 0..15, key 64*k + lane.
struct KeyUnit {        // workgroup-uniform
    u32 seg, KB, l, nb, blk0, cb, nch;
    u64 d, item_begin;
};

__device__ __forceinline__ u32 find_unit_segment(const SegState* states, u32 n_segments, u64 unit) {
    return wave_upper_index(n_segments, unit, [&](u32 i) { return states[i].unit_begin; });
}

__device__ __forceinline__ u32 segment_chunks(const SegInfo& s, u32 R) {
    return s.elem_count ? (u32)((segment_rows(s) + R - 1) / R) : 0u;
}

// `seg0` is the segment record of a single-gradient call (a kernel argument, so no load is needed).
// d0 / nb0: survivors and key blocks of segment 0, read once per kernel.
__device__ __forceinline__ KeyUnit key_unit(const SegInfo& seg0, const SegInfo* __restrict__ segs,
                                            const SegState* __restrict__ states, u32 n_segments, u32 R,
                                            u64 unit, u64 d0, u32 nb0, SegInfo* info_out) {
    KeyUnit ku;
    if (n_segments == 1) {
        *info_out = seg0;
        ku.seg = 0;
        ku.KB = seg0.block_keys;
        ku.d = d0;
        ku.nb = nb0;
        ku.item_begin = 0;
        ku.blk0 = (u32)unit * kWaves;
    } else {
        ku.seg = find_unit_segment(states, n_segments, unit);
        *info_out = segs[ku.seg];
        ku.KB = info_out->block_keys;
        ku.d = states[ku.seg].d;
        ku.nb = states[ku.seg].nb;
        ku.item_begin = states[ku.seg].item_begin;
        ku.blk0 = (u32)(unit - states[ku.seg].unit_begin) * kWaves;
    }
    ku.l = info_out->flag_bits;
    ku.cb = info_out->chunk_begin;
    ku.nch = segment_chunks(*info_out, R);
    return ku;
}

// In-place exclusive scan of arr[0..n) in shared memory by the whole workgroup, arr[n] = total;
// n <= PER * kThreads.  Starts and ends with a barrier.
template <typename T, u32 PER>
__device__ __forceinline__ void lds_excl_scan(T* arr, u32 n, T* scratch) {
    const u32 t = threadIdx.x;
    __syncthreads();
    T v[PER], sum = 0;
#pragma unroll
    for (u32 k = 0; k < PER; ++k) {
        const u32 j = t * PER + k;
        v[k] = j < n ? arr[j] : (T)0;
        sum += v[k];
    }
    // wave scan + workgroup combine
    T incl;
    if constexpr (sizeof(T) == 8) incl = wave_incl_scan64(sum); else incl = wave_incl_scan(sum);
    if (lane_id() == 63) scratch[wave_id()] = incl;
    __syncthreads();
    T base = 0, tot = 0;
#pragma unroll
    for (u32 w = 0; w < kWaves; ++w) {
        const T x = scratch[w];
        if (w < wave_id()) base += x;
        tot += x;
    }
    T run = base + incl - sum;
#pragma unroll
    for (u32 k = 0; k < PER; ++k) {
        const u32 j = t * PER + k;
        if (j < n) arr[j] = run;
        run += v[k];
    }
    if (t == 0) arr[n] = tot;
    __syncthreads();
}

// Chunk search: for a rank r that is the same in all lanes, the largest j in [0, nch) with P[j] <= r
// (P[0] = 0 <= r), and P[j] with it.  `coarse` is the wave's copy of every 64th entry of P in shared
// memory (load_coarse), so one memory round trip suffices: the wave reads the 64 entries behind the last
// coarse hit.  Done for three ranks at once (ra <= rb <= rc), with the three fetches in flight together.
__device__ __forceinline__ void find_chunks3(const u32* P, const u32* coarse, u32 nch, u32 ra, u32 rb, u32 rc, u32 lane,
                                             u32 (&j)[3], u32 (&pj)[3]) {
    const u32 cv = coarse[lane];
    const u32 r[3] = {ra, rb, rc};
    u32 c[3], v[3];
#pragma unroll
    for (u32 k = 0; k < 3; ++k) {
        c[k] = (u32)__popcll(__ballot(cv <= r[k])) - 1u;
        const u32 i2 = c[k] * 64u + lane;
        v[k] = i2 < nch ? P[i2] : 0xFFFFFFFFu;
    }
#pragma unroll
    for (u32 k = 0; k < 3; ++k) {
        const u32 c2 = (u32)__popcll(__ballot(v[k] <= r[k])) - 1u;
        pj[k] = read_lane(v[k], uniform(c2));
        j[k] = uniform(c[k] * 64u + c2);
    }
}

// Every 64th entry of the chunk scan P of a segment (0xFFFFFFFF beyond its nch chunks) into 64 words of
// the wave's shared memory.
__device__ __forceinline__ void load_coarse(const u32* P, u32 nch, u32 lane, u32* coarse) {
    wave_lds_sync();
    coarse[lane] = lane * 64u < nch ? P[lane * 64u] : 0xFFFFFFFFu;
    wave_lds_sync();
}

__device__ __forceinline__ u32 wave_incl_scan_max(u32 x) {
    u32 y;
    y = dpp_mov<kDppRowShr1>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr2>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr4>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowShr8>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowBcast15, 0xA>(0u, x); x = x > y ? x : y;
    y = dpp_mov<kDppRowBcast31, 0xC>(0u, x); x = x > y ? x : y;
    return x;
}

constexpr u32 kKeyRows = kSub / 64;   // rows of 64 keys a wave handles at a time

// Scratch entries, relative to the segment's chunk 0 (below 2^32: a gradient has fewer elements), of
// the n <= 1024 keys with segment ranks r0 + 64*q + lane, q = 0..15 (entries beyond n must not be
// used).  jlo / jhi are the chunks of the first / last of these ranks.  If the run crosses chunks,
// every chunk that starts inside it leaves its number at its first rank in `mark` (1024 words of the
// wave's shared memory, clobbered), and a running maximum spreads the numbers over the ranks.
__device__ __forceinline__ void find_entries(const u32* P, u32 stride, u32 jlo, u32 pjlo, u32 jhi, u32 r0, u32 n,
                                             u32 lane, u32* mark, u32 (&ent)[kKeyRows]) {
    if (jlo == jhi) {
        const u32 base = jlo * stride - pjlo;               // pjlo = P[jlo]
#pragma unroll
        for (u32 q = 0; q < kKeyRows; ++q) ent[q] = base + r0 + q * 64u + lane;
        return;
    }
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) mark[q * 64u + lane] = 0;
    wave_lds_sync();
    for (u32 j = jlo + 1u + lane; j <= jhi; j += 64u) atomicMax(&mark[P[j] - r0], j);   // r0 < P[j] <= r0 + n - 1
    wave_lds_sync();
    u32 m[kKeyRows];
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) m[q] = mark[q * 64u + lane];
    u32 carry = jlo;
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) {
        u32 j = wave_incl_scan_max(m[q]);
        j = j > carry ? j : carry;
        carry = read_lane(j, 63);
        m[q] = j;
    }
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) {
        const u32 j = (q * 64u < n) ? m[q] : jlo;
        ent[q] = j * stride + (r0 + q * 64u + lane - P[j]);
    }
    wave_lds_sync();
}

// Keys r0 .. r0 + n - 1 of a segment (n <= 1024), fetched row-wise (row q, lane: key 64*q + lane, so the
// fetches are coalesced wherever the ranks are contiguous in the scratch array) and handed to the lanes
// 16 CONSECUTIVE keys each through `buf` (1024 words of the wave's shared memory, 16-byte aligned,
// clobbered): kb[k] = key 16*lane + k (0 beyond n).  ent[q] keeps the scratch entry of key 64*q + lane.
__device__ __forceinline__ void gather_blocked(const u32* P, const u32* coarse, u32 nch, u32 stride,
                                               const u32* __restrict__ seg_keys, u32 r0, u32 n, u32 lane, u32* buf,
                                               u32 (&ent)[kKeyRows], u32 (&kb)[kLaneKeys], u32* prekey) {
    // chunks of the key before the run (if there is one and the caller wants it), of its first and of its last key
    u32 j[3], pj[3];
    const bool want_pre = prekey != nullptr && r0 != 0;
    find_chunks3(P, coarse, nch, want_pre ? r0 - 1u : r0, r0, r0 + n - 1u, lane, j, pj);
    u32 pre = 0;
    if (want_pre) pre = seg_keys[j[0] * stride + (r0 - 1u - pj[0])];
    const u32 jlo = j[1], pjlo = pj[1], jhi = j[2];
    find_entries(P, stride, jlo, pjlo, jhi, r0, n, lane, buf, ent);
    u32 key[kKeyRows];
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) key[q] = (q * 64u + lane < n) ? seg_keys[ent[q]] : 0u;
#pragma unroll
    for (u32 q = 0; q < kKeyRows; ++q) buf[q * 64u + lane] = key[q];
    wave_lds_sync();
    const uint4* b4 = reinterpret_cast<const uint4*>(buf) + lane * 4u;
#pragma unroll
    for (u32 j = 0; j < 4; ++j) {
        const uint4 x = b4[j];
        kb[4 * j] = x.x; kb[4 * j + 1] = x.y; kb[4 * j + 2] = x.z; kb[4 * j + 3] = x.w;
    }
    wave_lds_sync();
    if (prekey) *prekey = uniform(pre);
}

// Deltas of the lane's 16 keys (Eq. 4): dl[k] = kb[k] - key before it; `carry` is the key before the
// round on entry and the round's last key on return.  Keys that do not increase set bits in `unsorted`
// (the very first key of a segment may be 0, i.e. equal to its imaginary predecessor).
template <bool FULL>
__device__ __forceinline__ void lane_deltas(const u32 (&kb)[kLaneKeys], u32 r0, u32 n, u32 lane, u32& carry,
                                            u32 (&dl)[kLaneKeys], u64& unsorted) {
    // last valid key of the lane: for lanes that end beyond n, the round's last key
    const u32 nl = FULL ? kLaneKeys : (lane * kLaneKeys >= n ? 0u : (n - lane * kLaneKeys < kLaneKeys ? n - lane * kLaneKeys : kLaneKeys));
    u32 lastkey = kb[kLaneKeys - 1];
    if (!FULL) {
        lastkey = 0;
#pragma unroll
        for (u32 k = 0; k < kLaneKeys; ++k) if (k < nl) lastkey = kb[k];
    }
    u32 prev = lane_above(lastkey, carry);
#pragma unroll
    for (u32 k = 0; k < kLaneKeys; ++k) {
        const bool valid = FULL || k < nl;
        dl[k] = valid ? kb[k] - prev : 0u;
        u64 m = __ballot(valid && kb[k] <= prev);
        if (k == 0 && r0 == 0) m &= ~1ull;                    // rank 0 of the segment
        unsorted |= m;
        if (valid) prev = kb[k];
    }
    const u32 last_lane = (n - 1u) / kLaneKeys;
    carry = read_lane(lastkey, uniform(last_lane));
}

// BIG: some segment of the call has key blocks of more than 1024 keys, whose deltas' bit lengths then
// wait in shared memory for the block's M; otherwise they stay in registers.
template <bool BIG>
__global__ void __launch_bounds__(kThreads)
k_measure_keys(SegInfo seg0, const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
               u32 R, const u32* __restrict__ ccount, const u32* __restrict__ skeys, BlockInfo* __restrict__ binfo,
               unsigned long long* __restrict__ gsum, u32 g_shift, Ctrl* ctrl) {
    __shared__ __attribute__((aligned(16))) u32 s_bufall[kWaves][kSub];
    __shared__ __attribute__((aligned(16))) uint8_t s_needall[kWaves][BIG ? kMaxKB : 16];   // bit lengths of a big block's deltas
    __shared__ u32 s_lutall[kWaves][33];
    __shared__ u32 s_coarseall[kWaves][64];
    __shared__ u32 s_span[2][kWaves];                        // sizes of the unit's blocks, by parity of the round
    u32 lane = lane_id();
    const u32 w = uniform(wave_id());
    uint8_t* s_need = s_needall[w];
    u32* s_buf = s_bufall[w];
    u32* s_lut = s_lutall[w];
    u32* s_coarse = s_coarseall[w];
    const u64 total_units = ctrl->total_units;
    u32 coarse_seg = 0xFFFFFFFFu;                           // segment whose scan s_coarse samples
    const u64 d0 = states[0].d;
    const u32 nb0 = states[0].nb;
    // The sizes of a unit's (up to) kWaves blocks are added to the group sums by one thread of the
    // workgroup: an atomic per block would queue 64 deep on every sum (each takes a trip to the L2).
    u32 round = 0;
    for (u64 unit = blockIdx.x; unit < total_units; unit += gridDim.x, ++round) {
        // the lane number as a value of this unit: keeps the many addresses derived from it from being computed
        // once and held in registers across the whole kernel
        asm volatile("" : "+v"(lane));
        SegInfo info;
        const KeyUnit ku = key_unit(seg0, segs, states, n_segments, R, unit, d0, nb0, &info);
        const u32* P = ccount + ku.cb;                      // the segment's chunk scan
        const u32 blk = ku.blk0 + w;
        // the wave's block: its record, and the words it adds to the output (0: no block for this wave)
        auto measure_block = [&]() -> u32 {
        if (blk >= (ku.nb ? ku.nb : 1u)) return 0u;
        if (ku.seg != coarse_seg && ku.nb) { load_coarse(P, ku.nch, lane, s_coarse); coarse_seg = ku.seg; }
        const u64 item = ku.item_begin + blk;
        const u32 head8 = (u32)((kHeaderBytes + value_plane_bytes(ku.d, code_width(info.tau)) + 16ull * ku.nb) >> 3);   // first item of a segment
        if (ku.nb == 0) {                                   // a segment without survivors: its header only
            if (lane == 0) {
                BlockInfo bi; bi.preKey = 0; bi.M = 0; bi.payload_bits = 0; bi.span8 = head8;
                binfo[item] = bi;
            }
            return head8;
        }
        const u32 first = uniform(blk * ku.KB);
        const u32 cnt = uniform((u32)((ku.d - first < ku.KB) ? ku.d - first : ku.KB));
        const u32 nsub = (cnt + kSub - 1) / kSub;
        const u32 stride = R * kRow;
        const u32* seg_keys = skeys + chunk_slot0(info, ku.seg, 0, R);
        u32 preKey = 0;                                     // the key before the block (none for the segment's first block)
        // first loop of Algorithm 2: deltas and the longest of them (M = bit length of maxDelta)
        u64 unsorted = 0;
        u32 carry = 0, mxneed = 0;
        u32 packed[4] = {0, 0, 0, 0};
        for (u32 sub = 0; sub < nsub; ++sub) {
            const u32 n = cnt - sub * kSub < kSub ? cnt - sub * kSub : kSub;
            const u32 r0 = first + sub * kSub;
            u32 ent[kKeyRows], kb[kLaneKeys], dl[kLaneKeys];
            gather_blocked(P, s_coarse, ku.nch, stride, seg_keys, r0, n, lane, s_buf, ent, kb, sub == 0 ? &preKey : nullptr);
            if (sub == 0) carry = preKey;
            if (n == kSub) lane_deltas<true>(kb, r0, n, lane, carry, dl, unsorted);
            else lane_deltas<false>(kb, r0, n, lane, carry, dl, unsorted);
#pragma unroll
            for (u32 j = 0; j < 4; ++j) {
                u32 x = 0;
#pragma unroll
                for (u32 bb = 0; bb < 4; ++bb) {
                    const u32 need = 32u - __clz(dl[4 * j + bb]);      // __clz(0) = 32
                    mxneed = need > mxneed ? need : mxneed;
                    x |= need << (8u * bb);
                }
                packed[j] = x;
            }
            if (BIG) reinterpret_cast<uint4*>(s_need + sub * kSub)[lane] = make_uint4(packed[0], packed[1], packed[2], packed[3]);
        }
        mxneed = wave_max(mxneed);
        if (unsorted && lane == 0) set_status(ctrl, FASTSGD_ERR_UNSORTED_KEYS);
        const u32 M = mxneed ? mxneed : 1u;
        // payload bits: every key takes the length of the smallest level that holds its delta
        const u32 magic = level_magic(M), l = ku.l;
        if (lane <= 32) s_lut[lane] = level_len(level_of(lane, l, magic), M, l);     // length by bit length
        wave_lds_sync();
        u32 bits = 0;
        if (BIG) {
            for (u32 i = lane; i < cnt; i += 64) bits += s_lut[s_need[i]];
        } else {
            // one round: the bit lengths are still in registers (keys beyond cnt have none)
#pragma unroll
            for (u32 k = 0; k < kLaneKeys; ++k)
                if (lane * kLaneKeys + k < cnt) bits += s_lut[(packed[k >> 2] >> (8u * (k & 3u))) & 0xFFu];
        }
        bits = wave_sum(bits);
        wave_lds_sync();
        const u32 span8 = ((cnt * l + 63u) >> 6) + ((bits + 63u) >> 6) + (blk == 0 ? head8 : 0u);
        if (lane == 0) {
            BlockInfo bi;
            bi.preKey = preKey; bi.M = M; bi.payload_bits = bits; bi.span8 = span8;
            binfo[item] = bi;
        }
        return span8;
        };
        const u32 span8 = measure_block();
        if (lane == 0) s_span[round & 1u][w] = span8;
        __syncthreads();
        if (threadIdx.x == 0) {
            // the unit's items are consecutive: they fall into one group of sums or two
            const u64 item0 = ku.item_begin + ku.blk0, g0 = item0 >> g_shift;
            unsigned long long a = 0, b = 0;
#pragma unroll
            for (u32 k = 0; k < kWaves; ++k) {
                const u32 x = s_span[round & 1u][k];
                if (((item0 + k) >> g_shift) == g0) a += x; else b += x;
            }
            if (a) atomicAdd(&gsum[g0], a);
            if (b) atomicAdd(&gsum[g0 + 1], b);
        }
    }
}


// Offset (in 8-byte words) at which work item `item` starts adding to the output: the groups before
// its group (s_G, scanned) plus the items before it inside the group.  All lanes of the wave call it
// with the same item.
__device__ __forceinline__ u64 item_offset8(const u64* s_G, const BlockInfo* __restrict__ binfo, u32 g_shift, u64 item,
                                            u32 lane) {
    const u64 g = item >> g_shift;
    u64 acc = 0;
    for (u64 i = (g << g_shift) + lane; i < item; i += 64) acc += binfo[i].span8;
    return s_G[g] + wave_sum64(acc);
}

template <bool WIDE>
__global__ void __launch_bounds__(kThreads)
k_pack_keys(SegInfo seg0, const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
            u32 R, const u32* __restrict__ ccount, const u32* __restrict__ skeys,
            const void* __restrict__ scodes_any, const BlockInfo* __restrict__ binfo,
            const unsigned long long* __restrict__ gsum, u32 g_shift, uint8_t* __restrict__ out, u64 out_capacity,
            u64* out_offsets, u32 single, u32* out_status, const Ctrl* ctrl) {
    typedef typename ScratchCode<WIDE>::type CodeT;
    const CodeT* __restrict__ scodes = static_cast<const CodeT*>(scodes_any);
    __shared__ u64 s_G[kMaxGroups + 1];
    __shared__ u64 s_scan64[kWaves + 1];
    __shared__ __attribute__((aligned(16))) u32 s_payall[kWaves][kSub + 4];
    __shared__ u32 s_flgall[kWaves][kSub * 5 / 32 + 2];
    __shared__ u32 s_lutall[kWaves][33];
    __shared__ u32 s_coarseall[kWaves][64];
    const u32 t = threadIdx.x, w = uniform(wave_id());
    u32 lane = lane_id();
    u32* s_pay = s_payall[w];
    u32* s_flg = s_flgall[w];
    u32* s_lut = s_lutall[w];
    u32* s_coarse = s_coarseall[w];
    u32 coarse_seg = 0xFFFFFFFFu;                           // segment whose scan s_coarse samples
    const u64 total_items = ctrl->total_items, total_units = ctrl->total_units;
    if (blockIdx.x != 0 && blockIdx.x >= total_units) return;     // nothing to pack and nothing to report
    // byte offsets of the groups of work items
    const u32 ngroups = (u32)((total_items + (1ull << g_shift) - 1) >> g_shift);
    for (u32 i = t; i < ngroups; i += kThreads) s_G[i] = gsum[i];
    lds_excl_scan<u64, kMaxGroups / kThreads>(s_G, ngroups, s_scan64);
    const u64 total_bytes = 8ull * s_G[ngroups];
    u32 status = ctrl->status;
    if (status == 0 && total_bytes > out_capacity) status = FASTSGD_ERR_BUFFER_TOO_SMALL;
    const bool ok = (status == 0);

    if (blockIdx.x == 0) {          // length and status of the whole call
        if (single) {
            if (t == 0) out_offsets[0] = ok ? total_bytes : 0;
        } else {
            if (t == 0) out_offsets[n_segments] = ok ? total_bytes : 0;
            if (!ok) for (u32 s = t; s < n_segments; s += kThreads) out_offsets[s] = 0;
        }
        if (t == 0) *out_status = status;
    }
    if (!ok) return;                // nothing is written into a buffer that cannot hold the result

    for (u32 i = lane; i < kSub * 5 / 32 + 2; i += 64) s_flg[i] = 0;
    u64 sbeg8 = 0;
    u32 cur_seg = 0xFFFFFFFFu;
    const u64 d0 = states[0].d;
    const u32 nb0 = states[0].nb;
    for (u64 unit = blockIdx.x; unit < total_units; unit += gridDim.x) {
        asm volatile("" : "+v"(lane));      // (as in k_measure_keys: nothing derived from the lane number is kept across units)
        SegInfo info;
        const KeyUnit ku = key_unit(seg0, segs, states, n_segments, R, unit, d0, nb0, &info);
        const u32* P = ccount + ku.cb;                      // the segment's chunk scan
        if (ku.seg != cur_seg) {
            cur_seg = ku.seg;
            sbeg8 = (n_segments == 1) ? 0ull : item_offset8(s_G, binfo, g_shift, ku.item_begin, lane);
        }
        const u32 blk = ku.blk0 + w;
        const u32 nitems = ku.nb ? ku.nb : 1u;
        if (blk >= nitems) continue;
        const u64 item = ku.item_begin + blk;
        const u64 sbeg = 8ull * sbeg8;
        const u32 cwid = uniform(code_width(info.tau));               // bits of a value token
        const u64 dir_off = sbeg + kHeaderBytes + value_plane_bytes(ku.d, cwid);
        const u64 blocks_off = dir_off + 16ull * ku.nb;
        if (blk == 0) {
            const u64 send8 = item_offset8(s_G, binfo, g_shift, ku.item_begin + nitems, lane);
            if (lane == 0) {
                u64* h = reinterpret_cast<u64*>(out + sbeg);
                h[0] = (u64)kMagic | ((u64)kVersion << 32) | ((u64)info.flag_bits << 40) | ((u64)info.tau << 48);
                h[1] = (u64)info.block_keys | ((u64)ku.nb << 32);
                h[2] = (u64)__double_as_longlong(info.base);
                h[3] = (u64)__double_as_longlong(states[ku.seg].sum);
                h[4] = info.elem_count;
                h[5] = ku.d;
                h[6] = 8ull * (send8 - sbeg8);
                h[7] = 0;
                if (!single) out_offsets[ku.seg] = sbeg;
            }
            // zero padding between the value plane and the directory
            if (cwid == 8) {
                if (lane < 8 && ku.d + lane < align8(ku.d)) out[sbeg + kHeaderBytes + ku.d + lane] = 0;
            } else {
                // the last block writes whole 32-bit words; an odd number of them leaves one word of padding
                const u64 dw = (ku.d * cwid + 31ull) >> 5;
                if (lane == 0 && (dw & 1ull)) reinterpret_cast<u32*>(out + sbeg + kHeaderBytes)[dw] = 0;
            }
        }
        if (ku.nb == 0) continue;                                      // a segment without survivors
        if (ku.seg != coarse_seg) { load_coarse(P, ku.nch, lane, s_coarse); coarse_seg = ku.seg; }
        const BlockInfo bi = binfo[item];
        const u32 M = uniform(bi.M), l = ku.l, magic = level_magic(M);
        const u32 first = uniform(blk * ku.KB);
        const u32 cnt = uniform((u32)((ku.d - first < ku.KB) ? ku.d - first : ku.KB));
        const u32 nsub = (cnt + kSub - 1) / kSub;
        const u32 fwords = (cnt * l + 63u) >> 6;                       // 64-bit words of the flags plane
        const u64 start = (blk == 0) ? blocks_off : 8ull * item_offset8(s_G, binfo, g_shift, item, lane);
        if (lane == 0) {
            u64* e = reinterpret_cast<u64*>(out + dir_off + 16ull * blk);
            e[0] = (u64)(u32)((start - blocks_off) >> 3) | ((u64)bi.preKey << 32);
            e[1] = (u64)M | ((u64)bi.payload_bits << 32);
        }
        u32* fdst = reinterpret_cast<u32*>(out + start);               // flags plane, 32-bit words
        u32* pdst = fdst + 2u * fwords;                                // payload plane
        uint8_t* vdst = out + sbeg + kHeaderBytes + first;             // the block's part of the value plane (bytes)
        u32* vdst32 = reinterpret_cast<u32*>(out + sbeg + kHeaderBytes) + (first >> 5) * cwid;   // (narrower tokens)

        // second loop of Algorithm 2, 1024 keys at a time, 16 consecutive keys per lane
        const u32 stride = R * kRow;
        const u64 seg_slot0 = chunk_slot0(info, ku.seg, 0, R);
        const u32* seg_keys = skeys + seg_slot0;
        const CodeT* seg_codes = scodes + seg_slot0;
        // level and length by significant bits of the delta: lut[need] = (level - 1) | length << 8
        if (lane <= 32) {
            const u32 level = level_of(lane, l, magic);
            s_lut[lane] = (level - 1u) | (level_len(level, M, l) << 8);
        }
        u32 carry = uniform(bi.preKey);
        u32 wbits = 0;               // payload bits of this block waiting in `wword` from the previous round
        u32 wword = 0;
        u32 pw = 0;                  // payload words already written
        u64 unsorted = 0;
        uint8_t* s_flgb = reinterpret_cast<uint8_t*>(s_flg);
        for (u32 sub = 0; sub < nsub; ++sub) {
            const u32 n = cnt - sub * kSub < kSub ? cnt - sub * kSub : kSub;
            const u32 r0 = first + sub * kSub;
            u32 ent[kKeyRows], kb[kLaneKeys], dl[kLaneKeys], code[kKeyRows];
            gather_blocked(P, s_coarse, ku.nch, stride, seg_keys, r0, n, lane, s_pay, ent, kb, nullptr);    // borrows the payload window
#pragma unroll
            for (u32 q = 0; q < kKeyRows; ++q) code[q] = (q * 64u + lane < n) ? seg_codes[ent[q]] : 0u;
            if (cwid == 8) {
                // the survivors' code bytes go into the value plane 16 to a lane (single bytes cost several
                // times their share of a store): turned round in the (still unused) payload window
                uint8_t* s_b = reinterpret_cast<uint8_t*>(s_pay);
#pragma unroll
                for (u32 q = 0; q < kKeyRows; ++q) {
                    const u32 byte = WIDE ? ((code[q] >> 8) & 0x80u) | (code[q] & 0x7Fu) : code[q];
                    s_b[q * 64u + lane] = (uint8_t)byte;
                }
                wave_lds_sync();
                const uint4 c16 = reinterpret_cast<const uint4*>(s_pay)[lane];
                uint8_t* vrow = vdst + sub * kSub + 16u * lane;          // (8-byte aligned: streams and blocks are)
                if (16u * lane + 16u <= n) {
                    reinterpret_cast<uint2*>(vrow)[0] = make_uint2(c16.x, c16.y);
                    reinterpret_cast<uint2*>(vrow)[1] = make_uint2(c16.z, c16.w);
                } else if (16u * lane < n) {                             // the round's last, partial sixteen
                    const u32 cw4[4] = {c16.x, c16.y, c16.z, c16.w};
#pragma unroll
                    for (u32 k = 0; k < 16; ++k)
                        if (16u * lane + k < n) vrow[k] = (uint8_t)(cw4[k >> 2] >> (8u * (k & 3u)));
                }
                wave_lds_sync();
            } else {
                // tokens of cwid bits (sign on top of code-1), token i of the round at bit i * cwid:
                // assembled in the (still unused) payload window, stored as whole words
                CodeT* s_c = reinterpret_cast<CodeT*>(s_pay);            // the round's scratch codes
                u32* s_t = s_pay + kSub * sizeof(CodeT) / 4;             // the token words
                const u32 nw = (n * cwid + 31u) >> 5;
#pragma unroll
                for (u32 q = 0; q < kKeyRows; ++q) s_c[q * 64u + lane] = (CodeT)code[q];
                for (u32 i = lane; i < nw + 1u; i += 64) s_t[i] = 0;
                wave_lds_sync();
#pragma unroll 1
                for (u32 i = lane; i < n; i += 64) {
                    const u32 b = s_c[i];
                    const u32 tok = ((b >> (WIDE ? 15 : 7)) << (cwid - 1u)) | (b & (WIDE ? 0xFFu : 0x7Fu));
                    const u32 bit = i * cwid;
                    const u64 pv = (u64)tok << (bit & 31u);
                    atomicOr(&s_t[bit >> 5], (u32)pv);
                    if ((u32)(pv >> 32)) atomicOr(&s_t[(bit >> 5) + 1u], (u32)(pv >> 32));
                }
                wave_lds_sync();
                for (u32 i = lane; i < nw; i += 64) vdst32[sub * 32u * cwid + i] = s_t[i];
                wave_lds_sync();
            }
            // the payload window: word 0 carries the bits left over from the previous round
            for (u32 i = lane; i < kSub + 2; i += 64) s_pay[i] = (i == 0) ? wword : 0u;
            if (n == kSub) lane_deltas<true>(kb, r0, n, lane, carry, dl, unsorted);
            else lane_deltas<false>(kb, r0, n, lane, carry, dl, unsorted);
            // levels, lengths; the lane's 16 flags as a string of 16*l bits
            u32 len[kLaneKeys];
            u64 fstr[2] = {0, 0};
            u32 lanebits = 0;
#pragma unroll
            for (u32 k = 0; k < kLaneKeys; ++k) {
                const u32 e = s_lut[32u - __clz(dl[k])];
                const bool valid = lane * kLaneKeys + k < n;
                len[k] = valid ? e >> 8 : 0u;
                fstr[k >> 3] |= (u64)(valid ? e & 0xFFu : 0u) << ((k & 7u) * l);
                lanebits += len[k];
            }
            // 8 flags are l bytes: the lane's two halves go to bytes (2*lane + half) * l of the plane
#pragma unroll
            for (u32 half = 0; half < 2; ++half)
#pragma unroll
                for (u32 bb = 0; bb < 5; ++bb)
                    if (bb < l) s_flgb[(2u * lane + half) * l + bb] = (uint8_t)(fstr[half] >> (8u * bb));
            wave_lds_sync();
            const u32 incl = wave_incl_scan(lanebits);
            u32 bp = wbits + incl - lanebits;
#pragma unroll
            for (u32 k = 0; k < kLaneKeys; ++k) {
                const u64 pv = (u64)dl[k] << (bp & 31u);
                if (len[k]) {
                    atomicOr(&s_pay[bp >> 5], (u32)pv);
                    atomicOr(&s_pay[(bp >> 5) + 1], (u32)(pv >> 32));
                }
                bp += len[k];
            }
            const u32 roundend = wbits + read_lane(incl, 63);
            wave_lds_sync();
            const bool last = (sub + 1 == nsub);
            // flags of this round: whole 32-bit words (1024*l bits per full round)
            {
                const u32 nfw = (n * l + 31u) >> 5, f0 = sub * 32u * l;
                for (u32 i = lane; i < nfw; i += 64) { fdst[f0 + i] = s_flg[i]; s_flg[i] = 0; }
                if (last && ((f0 + nfw) & 1u) && lane == 0) fdst[f0 + nfw] = 0;      // pad to a 64-bit word
            }
            // payload: the full words; the partial last word waits for the next round
            {
                const u32 full = roundend >> 5, rest = roundend & 31u;
                const u32 nw = (last && rest) ? full + 1u : full;
                for (u32 i = lane; i < nw; i += 64) pdst[pw + i] = s_pay[i];
                if (last) {
                    if (((pw + nw) & 1u) && lane == 0) pdst[pw + nw] = 0;
                } else {
                    wword = uniform(s_pay[full]);
                    pw += full;
                    wbits = rest;
                }
            }
            wave_lds_sync();
        }
    }
}

}  // namespace fsgd
