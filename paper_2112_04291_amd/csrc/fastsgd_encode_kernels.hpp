// Encoder kernels of the gfx950 FastSGD codec (Algorithms 1 and 2 of arXiv 2112.04291).
//
//   k_init           clears the per-call control words and scan descriptors, stores the segment table
//   k_abs_sum        Algorithm 1 line 1: exact sum of |v| per segment (integer accumulation)
//   k_tables         Algorithm 1 line 2 + Eq. 3 as a boundary table sum / b^c, c = 1..tau
//   k_encode_values  Algorithm 1 lines 4-10: threshold test, code, sign, compaction of survivors
//   k_plan_keys      tile counts -> global ranks; per segment: survivors d, key blocks, work items
//   k_measure_keys   Algorithm 2, first loop, per key block: deltas, maxDelta -> M, size of the block
//   k_scan_items     byte offsets of the key blocks
//   k_pack_keys      Algorithm 2, second loop: length flags, bit packing; directory, headers, value planes
#pragma once
#include "fastsgd_device.hpp"

namespace fsgd {

// ---------------------------------------------------------------------------------------------
struct SegBatch { SegInfo seg[48]; };   // passed by value: the segment table needs no host->device copy

__global__ void k_init(u64* zero_begin, u64 zero_words, SegInfo* segs, SegBatch batch, u32 first, u32 count) {
    u64 i = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    u64 stride = (u64)gridDim.x * blockDim.x;
    for (; i < zero_words; i += stride) zero_begin[i] = 0;
    if (blockIdx.x == 0 && threadIdx.x < count) segs[first + threadIdx.x] = batch.seg[threadIdx.x];
}

__global__ void k_store_segments(SegInfo* segs, SegBatch batch, u32 first, u32 count) {
    if (threadIdx.x < count) segs[first + threadIdx.x] = batch.seg[threadIdx.x];
}

// ---------------------------------------------------------------------------------------------
// Tile geometry shared by the two passes over the values.  A segment's tiles start at its first
// element rounded down to a multiple of 4 (so float4 loads stay aligned); thread (wave w, lane)
// holds, for r = 0..3, the four elements  tile0 + w*1024 + r*256 + lane*4 + {0,1,2,3}.
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
__device__ __forceinline__ void load_tile(const float* __restrict__ values, const TileGeom& g, u32 bits[4][4]) {
    const u32 slot0 = wave_id() * 1024u + lane_id() * 4u;
    if (g.full) {
#pragma unroll
        for (u32 r = 0; r < 4; ++r) {
            const uint4 q = *reinterpret_cast<const uint4*>(values + g.tile0 + slot0 + r * 256u);
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
//   single gradient : every workgroup stores its one record at gbins[blockIdx.x] (plain stores, so
//                     nothing has to be cleared beforehand), and the launch also clears the scan
//                     descriptors and control words the later kernels rely on;
//   batch           : a workgroup owns a contiguous run of tiles and adds a record to one of n_slots
//                     copies of the segment's record each time it leaves a segment (atomics on
//                     memory k_init cleared).
constexpr u32 kBinWords = 2 * kBins + 2;

template <bool SINGLE>
__device__ __forceinline__ void flush_bins(u64 (*bins)[kThreads], u64* rec, u32 maxa) {
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
    if (SINGLE) {
        if (part == 0) { rec[2 * bin] = lo; rec[2 * bin + 1] = hi; }
        if (t == 0) { rec[2 * kBins] = bad ? 1u : 0u; rec[2 * kBins + 1] = 0; }
    } else {
        if (part == 0) {
            if (lo) atomicAdd((unsigned long long*)&rec[2 * bin], (unsigned long long)lo);
            if (hi) atomicAdd((unsigned long long*)&rec[2 * bin + 1], (unsigned long long)hi);
        }
        if (bad && t == 0) atomicOr((unsigned long long*)&rec[2 * kBins], 1ull);
#pragma unroll
        for (u32 b = 0; b < kBins; ++b) bins[b][t] = 0;
        __syncthreads();
    }
}

__device__ __forceinline__ void accumulate_tile(const u32 bits[4][4], u64 (*bins)[kThreads], u32& maxa) {
    const u32 t = threadIdx.x;
#pragma unroll
    for (u32 r = 0; r < 4; ++r)
#pragma unroll
        for (u32 c = 0; c < 4; ++c) {
            const u32 a = bits[r][c] & 0x7FFFFFFFu;
            maxa = a > maxa ? a : maxa;
            const u32 e = a >> 23;
            const u32 e1 = e ? e : 1u;
            const u32 m = a - ((e1 - 1u) << 23);          // significand with its leading one (none for denormals)
            const u64 val = (u64)m << (e1 & 15u);
            // a NaN/Inf lands in bin 15 as garbage; the record's flag makes the whole sum void
            atomicAdd((unsigned long long*)&bins[e1 >> 4][t], (unsigned long long)val);
        }
}

template <bool SINGLE>
__global__ void __launch_bounds__(kThreads)
k_abs_sum(const float* __restrict__ values, const SegInfo* __restrict__ segs, u32 n_segments, u64 n_tiles,
          u64* gbins, u32 n_slots, u64* zero_begin, u64 zero_words, SegInfo single_seg, SegInfo* seg_store) {
    __shared__ u64 bins[kBins][kThreads];
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
        const TileGeom g0 = tile_geom(single_seg, 0);
        for (u64 it = 0; it < per_wg; ++it) {
            const u64 tile = it * G + blockIdx.x;             // neighbours in time are neighbours in memory
            if (tile >= n_tiles) break;
            TileGeom g = g0;
            g.tile0 += tile * kTile;
            g.full = (g.tile0 >= g.lo) && (g.tile0 + kTile <= g.hi);
            u32 bits[4][4];
            load_tile(values, g, bits);
            accumulate_tile(bits, bins, maxa);
        }
        flush_bins<true>(bins, gbins + (u64)blockIdx.x * kBinWords, maxa);
    } else {
        u32 cur_seg = 0xFFFFFFFFu;
        const u64 t_begin = blockIdx.x * per_wg;
        const u64 t_end = (t_begin + per_wg < n_tiles) ? t_begin + per_wg : n_tiles;
        for (u64 tile = t_begin; tile < t_end; ++tile) {
            const u32 seg = find_segment(segs, n_segments, tile);
            if (seg != cur_seg) {
                if (cur_seg != 0xFFFFFFFFu) {
                    flush_bins<false>(bins, gbins + ((u64)cur_seg * n_slots + blockIdx.x % n_slots) * kBinWords, maxa);
                    maxa = 0;
                }
                cur_seg = seg;
            }
            const TileGeom g = tile_geom(segs[seg], tile);
            u32 bits[4][4];
            load_tile(values, g, bits);
            accumulate_tile(bits, bins, maxa);
        }
        if (cur_seg != 0xFFFFFFFFu)
            flush_bins<false>(bins, gbins + ((u64)cur_seg * n_slots + blockIdx.x % n_slots) * kBinWords, maxa);
    }
}

// ---------------------------------------------------------------------------------------------
// One workgroup per segment: add up the segment's records, fold the bins into a 384-bit integer
// counting units of 2^-150, round once to binary64 (nearest, ties to even), then the boundary table.
constexpr u32 kTableThreads = 1024;

__device__ __forceinline__ void wide_add(u64 (&L)[6], u64 x, u32 bitpos) {   // bitpos is a compile-time constant after unrolling
    const u32 i = bitpos >> 6, sh = bitpos & 63u;
    u64 parts[2] = {x << sh, sh ? (x >> (64u - sh)) : 0ull};
    u64 carry = 0;
#pragma unroll
    for (u32 j = 0; j < 6; ++j) {
        if (j >= i) {
            const u64 add = (j - i < 2) ? parts[j - i] : 0ull;
            const u64 s1 = L[j] + add;
            const u64 c1 = s1 < add ? 1ull : 0ull;
            const u64 s2 = s1 + carry;
            const u64 c2 = s2 < carry ? 1ull : 0ull;
            L[j] = s2;
            carry = c1 + c2;
        }
    }
}

__global__ void __launch_bounds__(kTableThreads)
k_tables(const SegInfo* __restrict__ segs, SegState* __restrict__ states, const u64* __restrict__ gbins,
         u32 n_slots, Ctrl* ctrl) {
    __shared__ u64 s_part[kTableThreads / 64][64];
    __shared__ double s_P[129];
    __shared__ double s_sum;
    const u32 seg = blockIdx.x, t = threadIdx.x;
    const SegInfo info = segs[seg];
    SegState* st = &states[seg];
    {
        // thread (group, word) adds up word `word` of records group, group+16, ...; 64 loads in flight
        const u32 word = t & 63u, group = t >> 6;
        constexpr u32 kGroups = kTableThreads / 64;
        u64 acc[4] = {0, 0, 0, 0};
        if (word < kBinWords) {
            const u64* g = gbins + (u64)seg * n_slots * kBinWords + word;
            for (u32 base = group; base < n_slots; base += kGroups * 64) {
#pragma unroll
                for (u32 j = 0; j < 64; ++j) {
                    const u32 sl = base + kGroups * j;
                    if (sl < n_slots) acc[j & 3] += g[(u64)sl * kBinWords];
                }
            }
        }
        s_part[group][word] = (acc[0] + acc[1]) + (acc[2] + acc[3]);
    }
    __syncthreads();
    if (t == 0) {
        u64 rec[kBinWords];
#pragma unroll
        for (u32 w = 0; w < kBinWords; ++w) {
            u64 x = 0;
#pragma unroll
            for (u32 g = 0; g < kTableThreads / 64; ++g) x += s_part[g][w];
            rec[w] = x;
        }
        // bin k holds lo + hi * 2^32 in units of 2^(16k - 150)
        u64 L[6] = {0, 0, 0, 0, 0, 0};
#pragma unroll
        for (u32 k = 0; k < kBins; ++k) {
            wide_add(L, rec[2 * k], 16u * k);
            wide_add(L, rec[2 * k + 1], 16u * k + 32u);
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
        const bool bad = rec[2 * kBins] != 0;
        if (bad) set_status(ctrl, FASTSGD_ERR_NONFINITE);
        st->sum = bad ? 0.0 : sum;
        s_sum = bad ? 0.0 : sum;
        power_chain(info.base, info.tau, s_P);
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
// Second pass over the values (Algorithm 1 lines 4-10).  A pure streaming pass: no tile depends on
// another.  Every WAVE walks its own tiles of 4096 elements (tile = wave + k * waves):
//   16 float4 loads per lane -> keep test |v| >= threshold -> survivors staged in the wave's slice of
//   shared memory at their rank inside the tile (ballot + mbcnt) -> densely over the staged survivors
//   only: code by binary search in the boundary table, key fetch -> code byte and key written to the
//   TILE'S OWN SLOT of the scratch arrays (entry tile*4096 + rank in tile) -> survivor count of the tile.
// Global ranks are fixed afterwards by a scan over the 4-byte tile counts (k_plan_keys); the key
// encoder gathers through that scan.  This keeps look-back chains and ticket counters -- dependent
// memory round trips that cost microseconds each while the memory system is saturated -- out of the
// one kernel that has to run at memory speed.
// Lane `lane` holds, for row r = 0..15, elements tile0 + r*256 + lane*4 + {0..3}.
constexpr u32 kRows = kTile / 256;       // 16 float4 rows per wave tile
constexpr u32 kStage = 1024;             // staged survivors per wave and round (4 rows can never exceed it)
constexpr u32 kValWaves = 4;             // waves per workgroup of the value encoder (they never synchronise)
constexpr u32 kGather = 8;               // key fetches a lane keeps in flight

// |v| >= threshold as a float compare with the |x| source modifier: for non-negative finite floats
// (denormals are preserved in this build) it orders exactly like the unsigned compare of the bit
// patterns, and a NaN threshold (bit pattern 0xFFFFFFFF = keep nothing) compares false.
__device__ __forceinline__ bool keeps(u32 value_bits, float threshold) {
    return __builtin_fabsf(__uint_as_float(value_bits)) >= threshold;
}

__device__ __forceinline__ u32 lanes_below(u64 mask) {
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
}

struct WaveTile {        // wave-uniform description of the tile a wave holds
    u64 tile;            // tile number (>= n_tiles: none)
    u64 tile0;           // element index of its first slot
    u32 seg;
    u32 lo_off, hi_off;  // slots [lo_off, hi_off) belong to the segment
};

__device__ __forceinline__ WaveTile describe_tile(const SegInfo* segs, u32 n_segments, u64 n_tiles, u64 tile) {
    WaveTile wt;
    wt.tile = tile; wt.tile0 = 0; wt.seg = 0; wt.lo_off = 0; wt.hi_off = 0;
    if (tile < n_tiles) {
        wt.seg = (n_segments == 1) ? 0u : find_segment(segs, n_segments, tile);
        const TileGeom g = tile_geom(segs[wt.seg], tile);
        wt.tile0 = g.tile0;
        wt.lo_off = g.lo > g.tile0 ? (u32)(g.lo - g.tile0) : 0u;
        wt.hi_off = g.hi - g.tile0 < kTile ? (u32)(g.hi - g.tile0) : kTile;
    }
    return wt;
}

__device__ __forceinline__ bool is_full(const WaveTile& wt) { return wt.lo_off == 0 && wt.hi_off == kTile; }

// A tile that lies wholly inside its segment: 16 coalesced float4 loads per lane.
__device__ __forceinline__ void load_full_tile(const float* __restrict__ values, const WaveTile& wt, u32 lane,
                                               u32 (&bits)[kRows][4]) {
    const uint4* src = reinterpret_cast<const uint4*>(values + wt.tile0) + lane;
#pragma unroll
    for (u32 r = 0; r < kRows; ++r) {
        const uint4 q = src[r * 64u];
        bits[r][0] = q.x; bits[r][1] = q.y; bits[r][2] = q.z; bits[r][3] = q.w;
    }
}

// A tile cut by a segment boundary (at most two per segment): slots outside the segment become zero,
// which never survives.  Goes through the wave's staging buffer in rolled loops so that this rare path
// costs no registers; the buffer must be free when it is called.
__device__ __forceinline__ void load_partial_tile(const float* __restrict__ values, const WaveTile& wt, u32 lane,
                                                  u32* stage, u32 (&bits)[kRows][4]) {
    const float* tvals = values + wt.tile0;
#pragma unroll
    for (u32 q = 0; q < kRows / 4; ++q) {
        __builtin_amdgcn_wave_barrier();
#pragma unroll 1
        for (u32 i = 0; i < 16; ++i) {
            const u32 off = q * 1024u + i * 64u + lane;
            stage[i * 64u + lane] = (off >= wt.lo_off && off < wt.hi_off) ? __float_as_uint(tvals[off]) : 0u;
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (u32 rr = 0; rr < 4; ++rr)
#pragma unroll
            for (u32 c = 0; c < 4; ++c) bits[4 * q + rr][c] = stage[rr * 256u + lane * 4u + c];
    }
    __builtin_amdgcn_wave_barrier();
}

// The loop is software-pipelined: once a tile's survivors sit in shared memory its registers are free,
// so the loads of the next tile are issued BEFORE the key fetches and stores of this one, and both
// waits collapse into one memory round trip per tile.
__global__ void __launch_bounds__(kValWaves * kWave) __attribute__((amdgpu_waves_per_eu(4, 8)))
k_encode_values(const u32* __restrict__ keys, const float* __restrict__ values,
                const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
                u64 n_tiles, u32* __restrict__ tcount, u32* __restrict__ skeys, uint8_t* __restrict__ scodes) {
    __shared__ u32 s_Ball[kValWaves][128];
    __shared__ u32 s_valall[kValWaves][kStage];
    __shared__ uint16_t s_idxall[kValWaves][kStage];
    const u32 lane = lane_id();
    const u32 w = (u32)__builtin_amdgcn_readfirstlane((int)wave_id());   // tell the compiler it is wave-uniform
    u32* s_B = s_Ball[w];
    u32* s_val = s_valall[w];
    uint16_t* s_idx = s_idxall[w];
    const u64 stride = (u64)gridDim.x * kValWaves;
    u32 cur_seg = 0xFFFFFFFFu, thr = 0xFFFFFFFFu, tau = 1;

    u32 bits[kRows][4];
    WaveTile cur = describe_tile(segs, n_segments, n_tiles, (u64)blockIdx.x * kValWaves + w);
    if (cur.tile >= n_tiles) return;
    if (is_full(cur)) load_full_tile(values, cur, lane, bits);
    else load_partial_tile(values, cur, lane, s_val, bits);

    for (;;) {
        if (cur.seg != cur_seg) {
            cur_seg = cur.seg;
            thr = states[cur_seg].thr_bits;
            tau = segs[cur_seg].tau;
            s_B[lane] = states[cur_seg].B[lane];
            s_B[lane + 64] = states[cur_seg].B[lane + 64];
        }
        // survivors of the tile: per-lane count, then one wave reduction
        const float thr_f = __uint_as_float(thr);
        u32 mine = 0;
#pragma unroll
        for (u32 r = 0; r < kRows; ++r)
#pragma unroll
            for (u32 c = 0; c < 4; ++c) mine += keeps(bits[r][c], thr_f) ? 1u : 0u;
#pragma unroll
        for (u32 d = 32; d >= 1; d >>= 1) mine += __shfl_xor(mine, d, 64);
        const u32 total = (u32)__builtin_amdgcn_readfirstlane((int)mine);

        float thr_s = thr_f;
        asm volatile("" : "+s"(thr_s));     // an opaque copy: the compare masks of the count pass stay dead
        // one row: stage its survivors behind `staged` earlier ones; returns the new count
        auto stage_row = [&](const u32 (&row)[4], u32 r, u32 staged) -> u32 {
            u64 m[4];
            u32 below = 0, rowcnt = 0;
#pragma unroll
            for (u32 c = 0; c < 4; ++c) {
                m[c] = __ballot(keeps(row[c], thr_s));
                below += lanes_below(m[c]);
                rowcnt += (u32)__popcll(m[c]);
            }
            u32 pos = staged + below;
#pragma unroll
            for (u32 c = 0; c < 4; ++c)
                if (keeps(row[c], thr_s)) {
                    s_val[pos] = row[c];
                    s_idx[pos] = (uint16_t)(r * 256u + lane * 4u + c);
                    ++pos;
                }
            return staged + rowcnt;
        };
        // staged survivors [0, cnt) of tile `wt` go to entries slot0 + j of the tile's slot
        auto write_staged = [&](const WaveTile& wt, u32 cnt, u64 slot0) {
            const u32* tkeys = keys + wt.tile0;
            __builtin_amdgcn_wave_barrier();
            for (u32 j0 = 0; j0 < cnt; j0 += 64u * kGather) {
                u32 key[kGather];
#pragma unroll
                for (u32 k = 0; k < kGather; ++k) {               // all key fetches of the chunk first
                    const u32 j = j0 + k * 64u + lane;
                    key[k] = (j < cnt) ? tkeys[s_idx[j]] : 0u;
                }
#pragma unroll
                for (u32 k = 0; k < kGather; ++k) {
                    const u32 j = j0 + k * 64u + lane;
                    if (j < cnt) {
                        const u32 vb = s_val[j];
                        const u32 a = vb & 0x7FFFFFFFu;
                        // smallest code c in [1, tau] with a >= B[c]  (B non-increasing, a >= B[tau])
                        u32 lo = 1, hi = tau;
                        while (lo < hi) {
                            const u32 mid = (lo + hi) >> 1;
                            if (a >= s_B[mid - 1]) hi = mid; else lo = mid + 1;
                        }
                        scodes[slot0 + j] = (uint8_t)(((vb >> 31) << 7) | (lo - 1));
                        skeys[slot0 + j] = key[k];
                    }
                    __builtin_amdgcn_sched_barrier(0);            // one search at a time: keeps registers low
                }
            }
            __builtin_amdgcn_wave_barrier();
        };

        const WaveTile done = cur;
        const u64 slot0 = done.tile * kTile;
        const bool fits = total <= kStage;
        if (fits) {
            if (total) {
                u32 staged = 0;
#pragma unroll
                for (u32 r = 0; r < kRows; ++r) staged = stage_row(bits[r], r, staged);
            }
        } else {
            // more than a quarter of the tile survives (far from the sparse regime this codec is for):
            // no staging, every lane codes and writes its own survivors
            const u32* tkeys = keys + done.tile0;
            u32 emitted = 0;
#pragma unroll
            for (u32 r = 0; r < kRows; ++r) {
                u64 m[4];
                u32 below = 0, rowcnt = 0;
#pragma unroll
                for (u32 c = 0; c < 4; ++c) {
                    m[c] = __ballot(keeps(bits[r][c], thr_s));
                    below += lanes_below(m[c]);
                    rowcnt += (u32)__popcll(m[c]);
                }
                u32 pos = emitted + below;
#pragma unroll
                for (u32 c = 0; c < 4; ++c)
                    if (keeps(bits[r][c], thr_s)) {
                        const u32 vb = bits[r][c], a = vb & 0x7FFFFFFFu;
                        u32 lo = 1, hi = tau;
                        while (lo < hi) {
                            const u32 mid = (lo + hi) >> 1;
                            if (a >= s_B[mid - 1]) hi = mid; else lo = mid + 1;
                        }
                        scodes[slot0 + pos] = (uint8_t)(((vb >> 31) << 7) | (lo - 1));
                        skeys[slot0 + pos] = tkeys[r * 256u + lane * 4u + c];
                        ++pos;
                    }
                emitted += rowcnt;
                __builtin_amdgcn_sched_barrier(0);
            }
        }
        // the registers are free: start on the next tile before finishing this one
        cur = describe_tile(segs, n_segments, n_tiles, done.tile + stride);
        const bool early = cur.tile < n_tiles && is_full(cur);
        if (early) load_full_tile(values, cur, lane, bits);
        if (fits && total) write_staged(done, total, slot0);
        if (lane == 0) tcount[done.tile] = total;
        if (cur.tile < n_tiles && !early) load_partial_tile(values, cur, lane, s_val, bits);
        if (cur.tile >= n_tiles) break;
    }
}

// ---------------------------------------------------------------------------------------------
// One workgroup turns the tile counts into global ranks and plans the key encoder:
//   A  inclusive scan of the tile counts -> tprefix
//   B  per segment: first rank, survivors d, key blocks, work-item numbering (one item per key block,
//      and one for a segment without any)
//   C  for every key block the tile that holds its first key and the tile that holds the key before it
constexpr u32 kPlanThreads = 1024;

__global__ void __launch_bounds__(kPlanThreads)
k_plan_keys(const SegInfo* __restrict__ segs, SegState* __restrict__ states, u32 n_segments, u64 n_tiles,
            const u32* __restrict__ tcount, u64* __restrict__ tprefix, u32* __restrict__ block_tile,
            u32* __restrict__ block_prev_tile, Ctrl* ctrl) {
    __shared__ u64 s_wave[kPlanThreads / 64];
    __shared__ u64 s_carry;
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    constexpr u32 kW = kPlanThreads / 64;

    auto block_scan = [&](u64 x, u64* total) -> u64 {       // exclusive scan over the workgroup
        const u64 incl = wave_incl_scan64(x);
        if (lane == 63) s_wave[w] = incl;
        __syncthreads();
        u64 base = 0, tot = 0;
        for (u32 k = 0; k < kW; ++k) { const u64 v = s_wave[k]; if (k < w) base += v; tot += v; }
        __syncthreads();
        *total = tot;
        return base + incl - x;
    };

    // A: every thread owns a run of consecutive tiles
    const u64 per = (n_tiles + kPlanThreads - 1) / kPlanThreads;
    const u64 a = (u64)t * per < n_tiles ? (u64)t * per : n_tiles;
    const u64 b = a + per < n_tiles ? a + per : n_tiles;
    u64 mine = 0;
    for (u64 i = a; i < b; ++i) mine += tcount[i];
    u64 total_d;
    u64 run = block_scan(mine, &total_d);
    for (u64 i = a; i < b; ++i) { run += tcount[i]; tprefix[i] = run; }
    __syncthreads();

    // B
    if (t == 0) s_carry = 0;
    __syncthreads();
    for (u32 s0 = 0; s0 < n_segments; s0 += kPlanThreads) {
        const u32 s = s0 + t;
        u64 items = 0;
        if (s < n_segments) {
            const u64 tb = segs[s].tile_begin;
            const u64 te = (s + 1 < n_segments) ? segs[s + 1].tile_begin : n_tiles;
            const u64 rb = tb ? tprefix[tb - 1] : 0;
            const u64 re = te ? tprefix[te - 1] : 0;
            const u64 d = re - rb;
            const u32 KB = segs[s].block_keys;
            const u32 nb = (u32)((d + KB - 1) / KB);
            states[s].rank_begin = rb;
            states[s].d = d;
            states[s].nb = nb;
            items = nb ? nb : 1u;
        }
        u64 total;
        const u64 ex = block_scan(items, &total);
        if (s < n_segments) states[s].item_begin = s_carry + ex;
        __syncthreads();
        if (t == 0) s_carry += total;
        __syncthreads();
    }
    if (t == 0) { ctrl->total_items = s_carry; ctrl->total_d = total_d; }

    // C: tile i holds the segment-relative ranks [lo, hi); it owns block starts b*KB in that range
    // (block_tile) and the ranks b*KB - 1 in that range (block_prev_tile)
    for (u64 i = t; i < n_tiles; i += kPlanThreads) {
        const u32 s = (n_segments == 1) ? 0u : find_segment(segs, n_segments, i);
        const u64 rb = states[s].rank_begin, ib = states[s].item_begin;
        const u64 KB = segs[s].block_keys;
        const u64 lo = (i ? tprefix[i - 1] : 0) - rb, hi = tprefix[i] - rb;
        if (hi > lo) {
            for (u64 blk = (lo + KB - 1) / KB; blk * KB < hi; ++blk) block_tile[ib + blk] = (u32)i;
            const u64 nb = states[s].nb;
            for (u64 blk = (lo + KB) / KB; blk * KB - 1 < hi && blk < nb; ++blk) block_prev_tile[ib + blk] = (u32)i;
        }
    }
}

__device__ __forceinline__ u32 find_item_segment(const SegState* states, u32 n_segments, u64 item) {
    u32 lo = 0, hi = n_segments;
    while (hi - lo > 1) {
        u32 mid = (lo + hi) >> 1;
        if (states[mid].item_begin <= item) lo = mid; else hi = mid;
    }
    return lo;
}

__device__ __forceinline__ u64 align8(u64 x) { return (x + 7) & ~7ull; }

// ---------------------------------------------------------------------------------------------
// Algorithm 2 on one block of surviving keys per work item, in two launches with a scan between:
//   k_measure_keys  first loop of Algorithm 2 (deltas, maxDelta -> M) and the size of the block's planes
//   k_scan_items    byte offset of every block (exclusive scan over the items)
//   k_pack_keys     second loop (length flags, bit packing), directory entry, header, value plane
// Both key kernels fetch a block's keys through the tile scan: rank r lives in the tile T with
// tprefix[T-1] <= r < tprefix[T], at entry T*4096 + (r - tprefix[T-1]) of the scratch arrays.
struct BlockGeom {
    u32 seg, blk, cnt, KB, l, nb;
    u64 d, first, grank;       // survivors of the segment; rank of the block's first key in the segment / globally
};

__device__ __forceinline__ BlockGeom block_geom(const SegInfo* segs, const SegState* states, u32 n_segments, u64 item) {
    BlockGeom g;
    g.seg = (n_segments == 1) ? 0u : find_item_segment(states, n_segments, item);
    const SegState* st = &states[g.seg];
    g.KB = segs[g.seg].block_keys; g.l = segs[g.seg].flag_bits;
    g.d = st->d; g.nb = st->nb;
    g.blk = (u32)(item - st->item_begin);
    g.first = (u64)g.blk * g.KB;
    g.cnt = g.nb ? (u32)((g.d - g.first < g.KB) ? g.d - g.first : g.KB) : 0u;
    g.grank = st->rank_begin + g.first;
    return g;
}

constexpr u32 kSlice = 1024;     // tile prefixes staged per round of the gather

// Fills s_keys[1 + i] (and, if codes_dst is given, codes_dst[i]) for the block's keys i = 0..cnt-1 and
// s_keys[0] with the key before the block (0 for a segment's first block).  All threads call it.
__device__ __forceinline__ void gather_block(const BlockGeom& g, u64 item, u64 n_tiles,
                                             const u64* __restrict__ tprefix, const u32* __restrict__ block_tile,
                                             const u32* __restrict__ block_prev_tile,
                                             const u32* __restrict__ skeys, const uint8_t* __restrict__ scodes,
                                             u32* s_keys, u64* s_pre, uint8_t* codes_dst) {
    const u32 t = threadIdx.x;
    if (g.cnt == 0) { if (t == 0) s_keys[0] = 0; __syncthreads(); return; }
    if (t == 0) {
        u32 pk = 0;
        if (g.first != 0) {
            const u64 T = block_prev_tile[item], r = g.grank - 1;
            pk = skeys[T * kTile + (r - (T ? tprefix[T - 1] : 0))];
        }
        s_keys[0] = pk;
    }
    const u64 r_end = g.grank + g.cnt;
    u64 T0 = block_tile[item];
    u32 len = 32;                 // a dense block spans a few tiles; a sparse one gets full slices afterwards
    for (;;) {
        // entry j = prefix BEFORE tile T0 + j, j = 0..len
        for (u32 j = t; j <= len; j += kThreads) {
            const u64 T = T0 + j;
            s_pre[j] = (T == 0) ? 0 : (T - 1 < n_tiles ? tprefix[T - 1] : ~0ull);
        }
        __syncthreads();
        const u64 covered = s_pre[len];                       // ranks below this are inside the slice
        for (u32 i = t; i < g.cnt; i += kThreads) {
            const u64 r = g.grank + i;
            if (r >= s_pre[0] && r < covered) {
                u32 lo = 0, hi = len - 1;                     // largest j with s_pre[j] <= r
                while (lo < hi) {
                    const u32 mid = (lo + hi + 1) >> 1;
                    if (s_pre[mid] <= r) lo = mid; else hi = mid - 1;
                }
                const u64 e = (T0 + lo) * kTile + (r - s_pre[lo]);
                s_keys[1 + i] = skeys[e];
                if (codes_dst) codes_dst[i] = scodes[e];
            }
        }
        __syncthreads();
        if (covered >= r_end) break;
        T0 += len;
        len = kSlice;
    }
}

__global__ void __launch_bounds__(kThreads)
k_measure_keys(const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments, u64 n_tiles,
               const u64* __restrict__ tprefix, const u32* __restrict__ block_tile,
               const u32* __restrict__ block_prev_tile, const u32* __restrict__ skeys,
               BlockInfo* __restrict__ binfo, Ctrl* ctrl) {
    __shared__ u32 s_keys[kMaxKB + 1];
    __shared__ u64 s_pre[kSlice + 1];
    __shared__ u32 s_red[kWaves], s_bits[kWaves];
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    const u64 total_items = ctrl->total_items;
    for (u64 item = blockIdx.x; item < total_items; item += gridDim.x) {
        const BlockGeom g = block_geom(segs, states, n_segments, item);
        gather_block(g, item, n_tiles, tprefix, block_tile, block_prev_tile, skeys, nullptr, s_keys, s_pre, nullptr);
        // first loop of Algorithm 2: deltas and their maximum
        u32 mx = 0;
        bool unsorted = false;
        for (u32 i = t; i < g.cnt; i += kThreads) {
            const u32 prev = s_keys[i], cur = s_keys[i + 1];
            unsorted |= (cur < prev) || (cur == prev && (g.first + i) != 0);
            const u32 dk = cur - prev;
            mx = dk > mx ? dk : mx;
        }
        mx = wave_max(mx);
        if (lane == 0) s_red[w] = mx;
        if (__any(unsorted) && lane == 0) set_status(ctrl, FASTSGD_ERR_UNSORTED_KEYS);
        __syncthreads();
        mx = s_red[0];
#pragma unroll
        for (u32 k = 1; k < kWaves; ++k) mx = s_red[k] > mx ? s_red[k] : mx;
        u32 M = 32u - __clz(mx);      // __clz(0) = 32
        if (M < 1) M = 1;
        // payload bits: every key takes the length of the smallest level that holds its delta
        u32 bits = 0;
        for (u32 i = t; i < g.cnt; i += kThreads) {
            const u32 need = 32u - __clz(s_keys[i + 1] - s_keys[i]);
            const u32 level = need ? (((need - 1u) << g.l) / M + 1u) : 1u;
            bits += (level * M + (1u << g.l) - 1u) >> g.l;
        }
#pragma unroll
        for (u32 d = 32; d >= 1; d >>= 1) bits += __shfl_xor(bits, d, 64);
        if (lane == 0) s_bits[w] = bits;
        __syncthreads();
        if (t == 0) {
            u32 pb = 0;
#pragma unroll
            for (u32 k = 0; k < kWaves; ++k) pb += s_bits[k];
            BlockInfo bi;
            bi.preKey = s_keys[0]; bi.M = M; bi.payload_bits = pb;
            bi.size8 = ((g.cnt * g.l + 63u) >> 6) + ((pb + 63u) >> 6);
            binfo[item] = bi;
        }
        __syncthreads();
    }
}

// Inclusive scan over the work items of the bytes each adds to the output: its key block, plus -- for
// the first item of a segment -- the segment's header, value plane and directory.
__global__ void __launch_bounds__(kPlanThreads)
k_scan_items(const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
             const BlockInfo* __restrict__ binfo, u64* __restrict__ ioff, const Ctrl* ctrl) {
    __shared__ u64 s_wave[kPlanThreads / 64];
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    constexpr u32 kW = kPlanThreads / 64;
    const u64 n = ctrl->total_items;
    const u64 per = (n + kPlanThreads - 1) / kPlanThreads;
    const u64 a = (u64)t * per < n ? (u64)t * per : n;
    const u64 b = a + per < n ? a + per : n;
    auto bytes_of = [&](u64 item) -> u64 {
        const u32 s = (n_segments == 1) ? 0u : find_item_segment(states, n_segments, item);
        u64 x = 8ull * binfo[item].size8;
        if (item == states[s].item_begin) x += kHeaderBytes + align8(states[s].d) + 16ull * states[s].nb;
        return x;
    };
    u64 mine = 0;
    for (u64 i = a; i < b; ++i) mine += bytes_of(i);
    const u64 incl = wave_incl_scan64(mine);
    if (lane == 63) s_wave[w] = incl;
    __syncthreads();
    u64 run = incl - mine;
    for (u32 k = 0; k < kW; ++k) if (k < w) run += s_wave[k];
    for (u64 i = a; i < b; ++i) { run += bytes_of(i); ioff[i] = run; }
}

__global__ void __launch_bounds__(kThreads)
k_pack_keys(const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments, u64 n_tiles,
            const u64* __restrict__ tprefix, const u32* __restrict__ block_tile,
            const u32* __restrict__ block_prev_tile, const u32* __restrict__ skeys,
            const uint8_t* __restrict__ scodes, const BlockInfo* __restrict__ binfo, const u64* __restrict__ ioff,
            uint8_t* __restrict__ out, u64 out_capacity, u64* out_offsets, u32 single, u32* out_status,
            const Ctrl* ctrl) {
    __shared__ u32 s_keys[kMaxKB + 1];
    __shared__ u64 s_pre[kSlice + 1];
    __shared__ u32 s_flags[kMaxKB * 5 / 32 + 2];
    __shared__ u32 s_pay[kMaxKB + 2];
    __shared__ u32 s_scan[kWaves + 1];
    __shared__ uint8_t s_codes[kMaxKB];
    const u32 t = threadIdx.x;
    const u64 total_items = ctrl->total_items;
    const u64 total_bytes = total_items ? ioff[total_items - 1] : 0;
    u32 status = ctrl->status;
    if (status == 0 && total_bytes > out_capacity) status = FASTSGD_ERR_BUFFER_TOO_SMALL;
    const bool ok = (status == 0);

    if (blockIdx.x == 0) {          // lengths and status of the whole call
        if (single) {
            if (t == 0) out_offsets[0] = ok ? total_bytes : 0;
        } else {
            for (u32 s = t; s <= n_segments; s += kThreads) {
                u64 off = 0;
                if (ok) {
                    if (s == n_segments) off = total_bytes;
                    else { const u64 ib = states[s].item_begin; off = ib ? ioff[ib - 1] : 0; }
                }
                out_offsets[s] = off;
            }
        }
        if (t == 0) *out_status = status;
    }
    if (!ok) return;                // nothing is written into a buffer that cannot hold the result

    for (u64 item = blockIdx.x; item < total_items; item += gridDim.x) {
        const BlockGeom g = block_geom(segs, states, n_segments, item);
        const SegInfo info = segs[g.seg];
        const u64 ib = states[g.seg].item_begin;
        const u64 sbeg = ib ? ioff[ib - 1] : 0;                        // stream start of the segment
        const u64 send = ioff[ib + (g.nb ? g.nb : 1u) - 1];            // and its end
        const u64 dir_off = sbeg + kHeaderBytes + align8(g.d);
        const u64 blocks_off = dir_off + 16ull * g.nb;
        if (g.blk == 0) {
            if (t == 0) {
                u64* h = reinterpret_cast<u64*>(out + sbeg);
                h[0] = (u64)kMagic | ((u64)kVersion << 32) | ((u64)info.flag_bits << 40) | ((u64)info.tau << 48);
                h[1] = (u64)info.block_keys | ((u64)g.nb << 32);
                h[2] = (u64)__double_as_longlong(info.base);
                h[3] = (u64)__double_as_longlong(states[g.seg].sum);
                h[4] = info.elem_count;
                h[5] = g.d;
                h[6] = send - sbeg;
                h[7] = 0;
            }
            // zero padding between the value plane and the directory
            if (t < 8 && g.d + t < align8(g.d)) out[sbeg + kHeaderBytes + g.d + t] = 0;
        }
        if (g.cnt == 0) continue;                                      // a segment without survivors
        const BlockInfo bi = binfo[item];
        const u32 M = bi.M, l = g.l, cnt = g.cnt;
        const u32 fwords = (cnt * l + 63u) >> 6, pwords = (bi.payload_bits + 63u) >> 6;
        const u64 start = ioff[item] - 8ull * bi.size8;                // this block's planes
        if (t == 0) {
            u64* e = reinterpret_cast<u64*>(out + dir_off + 16ull * g.blk);
            e[0] = (u64)(u32)((start - blocks_off) >> 3) | ((u64)bi.preKey << 32);
            e[1] = (u64)M | ((u64)bi.payload_bits << 32);
        }
        for (u32 i = t; i < 2 * fwords + 2; i += kThreads) s_flags[i] = 0;
        for (u32 i = t; i < 2 * pwords + 2; i += kThreads) s_pay[i] = 0;
        gather_block(g, item, n_tiles, tprefix, block_tile, block_prev_tile, skeys, scodes, s_keys, s_pre, s_codes);

        // value plane of the block's survivors
        {
            uint8_t* vdst = out + sbeg + kHeaderBytes + g.first;
            for (u32 i = t; i < cnt; i += kThreads) vdst[i] = s_codes[i];
        }
        // second loop of Algorithm 2: thread t owns keys [t*per, (t+1)*per)
        const u32 per = g.KB / kThreads;
        u32 len[16], lvl[16], delta[16], mybits = 0;
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            len[k] = 0; lvl[k] = 0; delta[k] = 0;
            if (k < per && i < cnt) {
                delta[k] = s_keys[i + 1] - s_keys[i];
                const u32 need = 32u - __clz(delta[k]);
                const u32 level = need ? (((need - 1u) << l) / M + 1u) : 1u;
                lvl[k] = level - 1u;
                len[k] = (level * M + (1u << l) - 1u) >> l;
                mybits += len[k];
            }
        }
        u32 payload_bits;
        u32 bitpos = block_excl_scan(mybits, s_scan, &payload_bits);
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            if (k < per && i < cnt) {
                const u32 fpos = i * l;
                const u64 fv = (u64)lvl[k] << (fpos & 31u);
                atomicOr(&s_flags[fpos >> 5], (u32)fv);
                if (fv >> 32) atomicOr(&s_flags[(fpos >> 5) + 1], (u32)(fv >> 32));
                const u64 pv = (u64)delta[k] << (bitpos & 31u);
                if ((u32)pv) atomicOr(&s_pay[bitpos >> 5], (u32)pv);
                if (pv >> 32) atomicOr(&s_pay[(bitpos >> 5) + 1], (u32)(pv >> 32));
                bitpos += len[k];
            }
        }
        __syncthreads();
        u64* dst = reinterpret_cast<u64*>(out + start);
        for (u32 i = t; i < fwords; i += kThreads) dst[i] = (u64)s_flags[2 * i] | ((u64)s_flags[2 * i + 1] << 32);
        for (u32 i = t; i < pwords; i += kThreads) dst[fwords + i] = (u64)s_pay[2 * i] | ((u64)s_pay[2 * i + 1] << 32);
        __syncthreads();
    }
}

}  // namespace fsgd
