// Encoder kernels of the gfx950 FastSGD codec (Algorithms 1 and 2 of arXiv 2112.04291).
//
//   k_init           clears the per-call control words and scan descriptors, stores the segment table
//   k_abs_sum        Algorithm 1 line 1: exact sum of |v| per segment (integer accumulation)
//   k_tables         Algorithm 1 line 2 + Eq. 3 as a boundary table sum / b^c, c = 1..tau
//   k_encode_values  Algorithm 1 lines 4-10: threshold test, code, sign, compaction of survivors
//   k_plan_keys      per segment: survivors d, key blocks, work-item numbering
//   k_encode_keys    Algorithm 2 per key block: deltas, M, length flags, bit packing
//   k_finalize       directory, headers, (segmented) value planes, lengths and status
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
// Second pass over the values (Algorithm 1 lines 4-10).  Every WAVE works on its own tiles of 4096
// elements and never waits for another wave of its workgroup, so memory latency of one wave hides
// behind the arithmetic of the others:
//   ticket -> 16 float4 loads per lane -> keep test |v| >= threshold (unsigned compare of bit
//   patterns, 64 ballots) -> survivor count -> decoupled look-back gives the tile's first global rank
//   -> survivors are staged in the wave's slice of shared memory at their rank inside the tile
//   (ballot + mbcnt) -> densely over the staged survivors only: code by binary search in the boundary
//   table, key fetch, code byte and key written at the global rank.
// Lane `lane` holds, for row r = 0..15, elements tile0 + r*256 + lane*4 + {0..3}.
constexpr u32 kRows = kTile / 256;       // 16 float4 rows per wave tile
constexpr u32 kStage = 1024;             // staged survivors per wave and round (4 rows can never exceed it)

// |v| >= threshold as a float compare with the |x| source modifier: for non-negative finite floats
// (denormals are preserved in this build) it orders exactly like the unsigned compare of the bit
// patterns, and a NaN threshold (bit pattern 0xFFFFFFFF = keep nothing) compares false.
__device__ __forceinline__ bool keeps(u32 value_bits, float threshold) {
    return __builtin_fabsf(__uint_as_float(value_bits)) >= threshold;
}

__device__ __forceinline__ u32 lanes_below(u64 mask) {
    return __builtin_amdgcn_mbcnt_hi((u32)(mask >> 32), __builtin_amdgcn_mbcnt_lo((u32)mask, 0u));
}

__global__ void __launch_bounds__(kTicketLanes * kWave) __attribute__((amdgpu_waves_per_eu(4, 8)))
k_encode_values(const u32* __restrict__ keys, const float* __restrict__ values,
                const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
                u64 n_tiles, u64* tdesc, u32* __restrict__ ckeys, uint8_t* __restrict__ codes,
                u64 codes_capacity, u64 ckeys_capacity, Ctrl* ctrl) {
    __shared__ u32 s_Ball[kTicketLanes][128];
    __shared__ u32 s_valall[kTicketLanes][kStage];
    __shared__ uint16_t s_idxall[kTicketLanes][kStage];
    const u32 lane = lane_id();
    const u32 w = (u32)__builtin_amdgcn_readfirstlane((int)wave_id());   // tell the compiler it is wave-uniform
    u32* s_B = s_Ball[w];
    u32* s_val = s_valall[w];
    uint16_t* s_idx = s_idxall[w];
    u32 cur_seg = 0xFFFFFFFFu, thr = 0xFFFFFFFFu, tau = 1;

    for (;;) {
        u32 ticket = 0;
        if (lane == 0) ticket = atomicAdd(&ctrl->ticket_val[w * kTicketStride], 1u);
        const u64 tile = (u64)(u32)__builtin_amdgcn_readfirstlane((int)ticket) * kTicketLanes + w;
        if (tile >= n_tiles) break;
        const u32 seg = (n_segments == 1) ? 0u : find_segment(segs, n_segments, tile);
        if (seg != cur_seg) {
            cur_seg = seg;
            thr = states[seg].thr_bits;
            tau = segs[seg].tau;
            s_B[lane] = states[seg].B[lane];
            s_B[lane + 64] = states[seg].B[lane + 64];
        }
        const TileGeom g = tile_geom(segs[seg], tile);
        const float* tvals = values + g.tile0;
        u32 bits[kRows][4];
        if (g.full) {
            const uint4* src = reinterpret_cast<const uint4*>(tvals) + lane;
#pragma unroll
            for (u32 r = 0; r < kRows; ++r) {
                const uint4 q = src[r * 64u];
                bits[r][0] = q.x; bits[r][1] = q.y; bits[r][2] = q.z; bits[r][3] = q.w;
            }
        } else {
            // slots [lo_off, hi_off) of the tile belong to the segment; others read a clamped (valid)
            // address and are replaced by zero, which never survives
            const u32 lo_off = g.lo > g.tile0 ? (u32)(g.lo - g.tile0) : 0u;
            const u32 hi_off = g.hi - g.tile0 < kTile ? (u32)(g.hi - g.tile0) : kTile;
#pragma unroll
            for (u32 r = 0; r < kRows; ++r) {
#pragma unroll
                for (u32 c = 0; c < 4; ++c) {
                    const u32 off = r * 256u + lane * 4u + c;
                    const u32 cl = off < lo_off ? lo_off : (off >= hi_off ? hi_off - 1u : off);
                    const u32 x = __float_as_uint(tvals[cl]);
                    bits[r][c] = (cl == off) ? x : 0u;
                }
                __builtin_amdgcn_sched_barrier(0);      // rare path: keep its address arithmetic row-local
            }
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
        u32 gave_up = 0;
        const u64 base = lookback_exclusive(tdesc, tile, total, &gave_up);
        if (gave_up && lane == 0) set_status(ctrl, FASTSGD_ERR_DEVICE);
        if (total == 0) continue;

        const u32* tkeys = keys + g.tile0;
        // one row: stage its survivors behind `staged` earlier ones; returns the new count
        float thr_s = thr_f;
        asm volatile("" : "+s"(thr_s));     // an opaque copy: the compare masks of the count pass stay dead
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
        // the staged survivors [0, cnt) have global ranks base + rank_off + j
        auto write_staged = [&](u32 cnt, u32 rank_off) {
            __builtin_amdgcn_wave_barrier();
            for (u32 j = lane; j < cnt; j += 64u) {
                const u32 vb = s_val[j];
                const u32 a = vb & 0x7FFFFFFFu;
                // smallest code c in [1, tau] with a >= B[c]  (B non-increasing, a >= B[tau])
                u32 lo = 1, hi = tau;
                while (lo < hi) {
                    const u32 mid = (lo + hi) >> 1;
                    if (a >= s_B[mid - 1]) hi = mid; else lo = mid + 1;
                }
                const u32 key = tkeys[s_idx[j]];
                const u64 rank = base + rank_off + j;
                if (rank < codes_capacity) codes[rank] = (uint8_t)(((vb >> 31) << 7) | (lo - 1));
                else set_status(ctrl, FASTSGD_ERR_BUFFER_TOO_SMALL);
                if (rank < ckeys_capacity) ckeys[rank] = key;
            }
            __builtin_amdgcn_wave_barrier();
        };
        if (total <= kStage) {
            u32 staged = 0;
#pragma unroll
            for (u32 r = 0; r < kRows; ++r) staged = stage_row(bits[r], r, staged);
            write_staged(total, 0);
        } else {
            u32 done = 0;
#pragma unroll
            for (u32 q = 0; q < kRows / 4; ++q) {
                u32 staged = 0;
#pragma unroll
                for (u32 rr = 0; rr < 4; ++rr) staged = stage_row(bits[4 * q + rr], 4 * q + rr, staged);
                write_staged(staged, done);
                done += staged;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// After the value pass every tile descriptor holds an inclusive prefix, so a segment's survivors are
// the difference of two of them.  Work items: one per key block, and one for a segment without any.
__global__ void __launch_bounds__(kThreads)
k_plan_keys(const SegInfo* __restrict__ segs, SegState* __restrict__ states, u32 n_segments, u64 n_tiles,
            const u64* __restrict__ tdesc, Ctrl* ctrl) {
    __shared__ u32 s_scan[kWaves + 1];
    __shared__ u64 s_carry;
    const u32 t = threadIdx.x;
    if (t == 0) s_carry = 0;
    __syncthreads();
    for (u32 s0 = 0; s0 < n_segments; s0 += kThreads) {
        const u32 s = s0 + t;
        u32 items = 0;
        if (s < n_segments) {
            const u64 tb = segs[s].tile_begin;
            const u64 te = (s + 1 < n_segments) ? segs[s + 1].tile_begin : n_tiles;
            const u64 rb = tb ? (tdesc[tb - 1] & kDescMask) : 0;
            const u64 re = te ? (tdesc[te - 1] & kDescMask) : 0;
            const u64 d = re - rb;
            const u32 KB = segs[s].block_keys;
            const u32 nb = (u32)((d + KB - 1) / KB);
            states[s].rank_begin = rb;
            states[s].d = d;
            states[s].nb = nb;
            items = nb ? nb : 1u;
        }
        u32 total;
        const u32 ex = block_excl_scan(items, s_scan, &total);
        if (s < n_segments) states[s].item_begin = s_carry + ex;
        __syncthreads();
        if (t == 0) s_carry += total;
        __syncthreads();
    }
    if (t == 0) {
        ctrl->total_items = s_carry;
        ctrl->total_d = n_tiles ? (tdesc[n_tiles - 1] & kDescMask) : 0;
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
// Algorithm 2 on one block of surviving keys per work item.  The block's planes are assembled in
// shared memory (zeroed, then OR-ed in at scanned bit offsets) and written out as 64-bit words at the
// byte offset a second look-back scan assigns.  The first item of a segment also accounts for the
// segment's header, value plane and directory in that scan.
__global__ void __launch_bounds__(kThreads)
k_encode_keys(const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
              const u32* __restrict__ ckeys, u64* idesc, BlockInfo* __restrict__ binfo,
              uint8_t* __restrict__ out, u64 out_capacity, Ctrl* ctrl) {
    __shared__ u32 s_keys[kMaxKB + 1];
    __shared__ u32 s_flags[kMaxKB * 5 / 32 + 2];
    __shared__ u32 s_pay[kMaxKB + 2];
    __shared__ u32 s_scan[kWaves + 1];
    __shared__ u32 s_red[kWaves];
    __shared__ u64 s_base;
    __shared__ u32 s_item_lo;
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    const u64 total_items = ctrl->total_items;

    for (;;) {
        if (t == 0) s_item_lo = atomicAdd(&ctrl->ticket_key[0], 1u);   // items < 2^32
        __syncthreads();
        const u64 item = s_item_lo;
        if (item >= total_items) break;
        const u32 seg = (n_segments == 1) ? 0u : find_item_segment(states, n_segments, item);
        const SegState* st = &states[seg];
        const u32 KB = segs[seg].block_keys, l = segs[seg].flag_bits;
        const u64 d = st->d;
        const u32 nb = st->nb;
        const u32 blk = (u32)(item - st->item_begin);
        const u64 first = (u64)blk * KB;                      // rank inside the segment
        const u32 cnt = nb ? (u32)((d - first < KB) ? d - first : KB) : 0u;
        const u64 grank = st->rank_begin + first;             // global rank of the block's first key
        const u32 per = KB / kThreads;                        // keys per thread: 1..16

        // keys of the block, preceded by preKey
        for (u32 i = t; i < cnt; i += kThreads) s_keys[i + 1] = ckeys[grank + i];
        if (t == 0) s_keys[0] = (first == 0) ? 0u : ckeys[grank - 1];
        for (u32 i = t; i < sizeof(s_flags) / 4; i += kThreads) s_flags[i] = 0;
        for (u32 i = t; i < sizeof(s_pay) / 4; i += kThreads) s_pay[i] = 0;
        __syncthreads();

        // first loop of Algorithm 2: deltas and their maximum
        u32 delta[16];
        u32 mx = 0;
        bool unsorted = false;
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            delta[k] = 0;
            if (k < per && i < cnt) {
                const u32 prev = s_keys[i], cur = s_keys[i + 1];
                delta[k] = cur - prev;
                unsorted |= (cur < prev) || (cur == prev && (first + i) != 0);
                mx = delta[k] > mx ? delta[k] : mx;
            }
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

        // second loop: level (smallest length that holds the delta) and its length
        u32 len[16], lvl[16], mybits = 0;
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            len[k] = 0; lvl[k] = 0;
            if (k < per && i < cnt) {
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
        const u32 fwords = (cnt * l + 63u) >> 6, pwords = (payload_bits + 63u) >> 6;   // 64-bit words
        const u32 size8 = fwords + pwords;
        const u64 fixed = (blk == 0) ? (kHeaderBytes + align8(d) + 16ull * nb) : 0ull;
        if (w == 0) {
            u32 gave_up = 0;
            const u64 base = lookback_exclusive(idesc, item, 8ull * size8 + fixed, &gave_up);
            if (lane == 0) {
                s_base = base;
                if (gave_up) set_status(ctrl, FASTSGD_ERR_DEVICE);
                BlockInfo bi;
                bi.preKey = s_keys[0]; bi.M = M; bi.payload_bits = payload_bits; bi.size8 = size8;
                binfo[item] = bi;
            }
        }
        __syncthreads();
        const u64 start = s_base + fixed;                     // byte offset of this block's planes
        if (start + 8ull * size8 <= out_capacity) {
            u64* dst = reinterpret_cast<u64*>(out + start);
            for (u32 i = t; i < fwords; i += kThreads)
                dst[i] = (u64)s_flags[2 * i] | ((u64)s_flags[2 * i + 1] << 32);
            for (u32 i = t; i < pwords; i += kThreads)
                dst[fwords + i] = (u64)s_pay[2 * i] | ((u64)s_pay[2 * i + 1] << 32);
        } else if (t == 0) {
            set_status(ctrl, FASTSGD_ERR_BUFFER_TOO_SMALL);
        }
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------------------------
// Everything that needs the resolved byte offsets: directory entries, headers, value planes of a
// segmented call (the single-gradient call wrote them in place), lengths and status.
__global__ void __launch_bounds__(kThreads)
k_finalize(const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
           const u64* __restrict__ idesc, const BlockInfo* __restrict__ binfo,
           const uint8_t* __restrict__ codes_scratch, uint8_t* __restrict__ out, u64 out_capacity,
           u64* out_offsets /* n_segments+1, or a single length if single */, u32 single,
           u32* out_status, Ctrl* ctrl) {
    const u32 t = threadIdx.x;
    const u64 total_items = ctrl->total_items;
    const u64 total_bytes = total_items ? (idesc[total_items - 1] & kDescMask) : 0;
    u32 status = ctrl->status;
    if (status == 0 && total_bytes > out_capacity) status = FASTSGD_ERR_BUFFER_TOO_SMALL;
    const bool ok = (status == 0);

    for (u64 item = blockIdx.x; item < total_items; item += gridDim.x) {
        const u32 seg = (n_segments == 1) ? 0u : find_item_segment(states, n_segments, item);
        const SegState* st = &states[seg];
        const SegInfo info = segs[seg];
        const u64 ib = st->item_begin;
        const u64 sbeg = ib ? (idesc[ib - 1] & kDescMask) : 0;            // stream start of the segment
        const u64 d = st->d;
        const u32 nb = st->nb;
        const u32 blk = (u32)(item - ib);
        const u64 dir_off = sbeg + kHeaderBytes + align8(d);
        const u64 blocks_off = dir_off + 16ull * nb;
        const u64 incl = idesc[item] & kDescMask;
        const u64 send = idesc[ib + (nb ? nb : 1u) - 1] & kDescMask;      // stream end
        if (!ok) continue;
        if (nb) {
            const BlockInfo bi = binfo[item];
            const u64 start = incl - 8ull * bi.size8;
            if (t == 0) {
                u64* e = reinterpret_cast<u64*>(out + dir_off + 16ull * blk);
                e[0] = (u64)(u32)((start - blocks_off) >> 3) | ((u64)bi.preKey << 32);
                e[1] = (u64)bi.M | ((u64)bi.payload_bits << 32);
            }
            if (!single) {
                const u32 KB = info.block_keys;
                const u64 first = (u64)blk * KB;
                const u32 cnt = (u32)((d - first < KB) ? d - first : KB);
                const uint8_t* src = codes_scratch + st->rank_begin + first;
                uint8_t* dst = out + sbeg + kHeaderBytes + first;
                for (u32 i = t; i < cnt; i += kThreads) dst[i] = src[i];
            }
        }
        if (blk == 0) {
            if (t == 0) {
                u64* h = reinterpret_cast<u64*>(out + sbeg);
                h[0] = (u64)kMagic | ((u64)kVersion << 32) | ((u64)info.flag_bits << 40) | ((u64)info.tau << 48);
                h[1] = (u64)info.block_keys | ((u64)nb << 32);
                h[2] = (u64)__double_as_longlong(info.base);
                h[3] = (u64)__double_as_longlong(st->sum);
                h[4] = info.elem_count;
                h[5] = d;
                h[6] = send - sbeg;
                h[7] = 0;
            }
            // zero padding between the value plane and the directory
            if (t < 8 && d + t < align8(d)) out[sbeg + kHeaderBytes + d + t] = 0;
        }
    }
    if (blockIdx.x == 0) {
        if (single) {
            if (t == 0) out_offsets[0] = ok ? total_bytes : 0;
        } else {
            for (u32 s = t; s <= n_segments; s += kThreads) {
                u64 off = 0;
                if (ok) {
                    if (s == n_segments) off = total_bytes;
                    else { const u64 ib = states[s].item_begin; off = ib ? (idesc[ib - 1] & kDescMask) : 0; }
                }
                out_offsets[s] = off;
            }
        }
        if (t == 0) *out_status = status;
    }
}

}  // namespace fsgd
