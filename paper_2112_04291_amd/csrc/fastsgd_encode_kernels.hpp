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
// its lanes into (low-half sum, high-half sum) pairs and adds them to one of `n_slots` copies of
// the segment's global bins.
__device__ __forceinline__ void flush_bins(u64 (*bins)[kThreads], u64* gbins_seg, u32 n_slots, u32 maxa,
                                           SegState* st) {
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
    if (part == 0) {
        u64* g = gbins_seg + (u64)(blockIdx.x % n_slots) * (2 * kBins) + 2 * bin;
        if (lo) atomicAdd((unsigned long long*)&g[0], (unsigned long long)lo);
        if (hi) atomicAdd((unsigned long long*)&g[1], (unsigned long long)hi);
    }
    if (__any(maxa >= 0x7F800000u) && lane_id() == 0) atomicOr(&st->nonfinite, 1u);
    __syncthreads();
#pragma unroll
    for (u32 b = 0; b < kBins; ++b) bins[b][t] = 0;
    __syncthreads();
}

__global__ void __launch_bounds__(kThreads)
k_abs_sum(const float* __restrict__ values, const SegInfo* __restrict__ segs, SegState* __restrict__ states,
          u32 n_segments, u64 n_tiles, u32 tiles_per_chunk, u64* gbins, u32 n_slots, Ctrl* ctrl) {
    __shared__ u64 bins[kBins][kThreads];
    __shared__ u32 s_chunk;
    const u32 t = threadIdx.x;
#pragma unroll
    for (u32 b = 0; b < kBins; ++b) bins[b][t] = 0;
    __syncthreads();

    u32 cur_seg = 0xFFFFFFFFu, maxa = 0;
    const u64 n_chunks = (n_tiles + tiles_per_chunk - 1) / tiles_per_chunk;
    for (;;) {
        if (t == 0) s_chunk = atomicAdd(&ctrl->ticket_sum, 1u);
        __syncthreads();
        const u64 chunk = s_chunk;
        __syncthreads();
        if (chunk >= n_chunks) break;
        const u64 t_begin = chunk * tiles_per_chunk;
        const u64 t_end = (t_begin + tiles_per_chunk < n_tiles) ? t_begin + tiles_per_chunk : n_tiles;
        for (u64 tile = t_begin; tile < t_end; ++tile) {
            const u32 seg = (n_segments == 1) ? 0u : find_segment(segs, n_segments, tile);
            if (seg != cur_seg) {
                if (cur_seg != 0xFFFFFFFFu) {
                    flush_bins(bins, gbins + (u64)cur_seg * n_slots * (2 * kBins), n_slots, maxa, &states[cur_seg]);
                    maxa = 0;
                }
                cur_seg = seg;
            }
            const TileGeom g = tile_geom(segs[seg], tile);
            u32 bits[4][4];
            load_tile(values, g, bits);
#pragma unroll
            for (u32 r = 0; r < 4; ++r)
#pragma unroll
                for (u32 c = 0; c < 4; ++c) {
                    const u32 a = bits[r][c] & 0x7FFFFFFFu;
                    maxa = a > maxa ? a : maxa;
                    const u32 e = a >> 23;
                    const u32 m = (a & 0x7FFFFFu) | (e ? 0x800000u : 0u);
                    const u32 e1 = e ? e : 1u;
                    const u64 val = (u64)m << (e1 & 15u);
                    if (e != 255u)     // NaN/Inf: reported through maxa, kept out of the bins
                        atomicAdd((unsigned long long*)&bins[e1 >> 4][t], (unsigned long long)val);
                }
        }
    }
    if (cur_seg != 0xFFFFFFFFu)
        flush_bins(bins, gbins + (u64)cur_seg * n_slots * (2 * kBins), n_slots, maxa, &states[cur_seg]);
}

// ---------------------------------------------------------------------------------------------
// One workgroup (one wave) per segment: fold the bins into a wide integer counting units of 2^-150,
// round once to binary64 (nearest, ties to even), then the boundary table.
__global__ void __launch_bounds__(kThreads)
k_tables(const SegInfo* __restrict__ segs, SegState* __restrict__ states, const u64* __restrict__ gbins,
         u32 n_slots, Ctrl* ctrl) {
    __shared__ u64 s_part[2 * kBins];
    __shared__ u32 s_limb[16];
    __shared__ double s_P[129];
    __shared__ double s_sum;
    const u32 seg = blockIdx.x, t = threadIdx.x;
    const SegInfo info = segs[seg];
    SegState* st = &states[seg];
    if (t < 2 * kBins) {
        const u64* g = gbins + (u64)seg * n_slots * (2 * kBins);
        u64 x = 0;
        for (u32 s = 0; s < n_slots; ++s) x += g[(u64)s * (2 * kBins) + t];
        s_part[t] = x;
    }
    if (t < 16) s_limb[t] = 0;
    __syncthreads();
    if (t == 0) {
        // bin k holds lo + hi * 2^32 in units of 2^(16k - 150)
        for (u32 k = 0; k < kBins; ++k)
            for (u32 h = 0; h < 2; ++h) {
                const u64 x = s_part[2 * k + h];
                const u32 bitpos = 16u * k + 32u * h;
                // add the two 32-bit halves of x, each shifted by bitpos % 32, at limb bitpos / 32
                for (u32 half = 0; half < 2; ++half) {
                    u64 piece = ((x >> (32 * half)) & 0xFFFFFFFFull) << (bitpos & 31u);
                    u32 li = (bitpos >> 5) + half;
                    while (piece) {
                        u64 s = (u64)s_limb[li] + (piece & 0xFFFFFFFFull);
                        s_limb[li] = (u32)s;
                        piece = (piece >> 32) + (s >> 32);
                        ++li;
                    }
                }
            }
        int top = -1;
        for (int li = 15; li >= 0; --li)
            if (s_limb[li]) { top = li * 32 + 31 - __builtin_clz(s_limb[li]); break; }
        double sum = 0.0;
        if (top >= 0) {
            u64 q = 0;
            const int lo = top - 52;
            for (int b = top; b >= lo && b >= 0; --b) q = (q << 1) | ((s_limb[b >> 5] >> (b & 31)) & 1u);
            if (lo > 0) {
                const u32 guard = (s_limb[(lo - 1) >> 5] >> ((lo - 1) & 31)) & 1u;
                u32 sticky = 0;
                for (int b = lo - 2; b >= 0 && !sticky; --b) sticky = (s_limb[b >> 5] >> (b & 31)) & 1u;
                if (guard && (sticky || (q & 1))) ++q;
            } else {
                q <<= (52 - top);            // fewer than 53 bits: exact, left-align the significand
            }
            // value = q * 2^(max(lo,0) - 150) with q in [2^52, 2^53]; q = 2^53 carries into the exponent
            const u64 bits = ((u64)(top - 150 + 1023) << 52) + (q - (1ull << 52));
            sum = __longlong_as_double((long long)bits);
        }
        const bool bad = st->nonfinite != 0;
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
// Second pass over the values: keep |v| >= threshold (one unsigned compare on bit patterns), rank
// the survivors in element order (wave scans inside the tile, decoupled look-back across tiles),
// then -- densely over the survivors only -- find the code by binary search in the boundary table,
// fetch the key, and write code byte and key at the survivor's global rank.
__global__ void __launch_bounds__(kThreads)
k_encode_values(const u32* __restrict__ keys, const float* __restrict__ values,
                const SegInfo* __restrict__ segs, const SegState* __restrict__ states, u32 n_segments,
                u64 n_tiles, u64* tdesc, u32* __restrict__ ckeys, uint8_t* __restrict__ codes,
                u64 codes_capacity, u64 ckeys_capacity, Ctrl* ctrl) {
    __shared__ u32 s_B[128];
    __shared__ u32 s_val[kTile];
    __shared__ uint16_t s_idx[kTile];
    __shared__ u32 s_wtot[kWaves];
    __shared__ u64 s_base;
    __shared__ u32 s_tile;
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    u32 cur_seg = 0xFFFFFFFFu, thr = 0xFFFFFFFFu, tau = 1;

    for (;;) {
        if (t == 0) s_tile = atomicAdd(&ctrl->ticket_val, 1u);
        __syncthreads();
        const u64 tile = s_tile;
        if (tile >= n_tiles) break;
        const u32 seg = (n_segments == 1) ? 0u : find_segment(segs, n_segments, tile);
        if (seg != cur_seg) {
            cur_seg = seg;
            thr = states[seg].thr_bits;
            tau = segs[seg].tau;
            if (t < 128) s_B[t] = states[seg].B[t];
        }
        const TileGeom g = tile_geom(segs[seg], tile);
        u32 bits[4][4];
        load_tile(values, g, bits);

        u32 kb[4], cnt[4];
#pragma unroll
        for (u32 r = 0; r < 4; ++r) {
            u32 m = 0;
#pragma unroll
            for (u32 c = 0; c < 4; ++c) m |= ((bits[r][c] & 0x7FFFFFFFu) >= thr ? 1u : 0u) << c;
            kb[r] = m;
            cnt[r] = __popc(m);
        }
        // wave-level ranks: two packed 16-bit scans cover the four rows
        const u32 p01 = cnt[0] | (cnt[1] << 16), p23 = cnt[2] | (cnt[3] << 16);
        const u32 i01 = wave_incl_scan(p01), i23 = wave_incl_scan(p23);
        const u32 t01 = __shfl(i01, 63, 64), t23 = __shfl(i23, 63, 64);
        u32 rowbase[4], excl[4];
        rowbase[0] = 0;
        rowbase[1] = t01 & 0xFFFFu;
        rowbase[2] = rowbase[1] + (t01 >> 16);
        rowbase[3] = rowbase[2] + (t23 & 0xFFFFu);
        const u32 wave_total = rowbase[3] + (t23 >> 16);
        excl[0] = (i01 & 0xFFFFu) - cnt[0];
        excl[1] = (i01 >> 16) - cnt[1];
        excl[2] = (i23 & 0xFFFFu) - cnt[2];
        excl[3] = (i23 >> 16) - cnt[3];
        if (lane == 0) s_wtot[w] = wave_total;
        __syncthreads();
        u32 wave_base = 0, tile_total = 0;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            const u32 x = s_wtot[k];
            if (k < w) wave_base += x;
            tile_total += x;
        }
        if (w == 0) {
            u32 gave_up = 0;
            const u64 base = lookback_exclusive(tdesc, tile, tile_total, &gave_up);
            if (lane == 0) {
                s_base = base;
                if (gave_up) set_status(ctrl, FASTSGD_ERR_DEVICE);
            }
        }
        // stage survivors (value bits + slot in the tile) at their rank inside the tile
#pragma unroll
        for (u32 r = 0; r < 4; ++r) {
            u32 pos = wave_base + rowbase[r] + excl[r];
#pragma unroll
            for (u32 c = 0; c < 4; ++c)
                if (kb[r] >> c & 1u) {
                    s_val[pos] = bits[r][c];
                    s_idx[pos] = (uint16_t)(w * 1024u + r * 256u + lane * 4u + c);
                    ++pos;
                }
        }
        __syncthreads();
        const u64 base = s_base;
        for (u32 j = t; j < tile_total; j += kThreads) {
            const u32 vb = s_val[j];
            const u32 a = vb & 0x7FFFFFFFu;
            // smallest code c in [1, tau] with a >= B[c]  (B non-increasing, a >= B[tau])
            u32 lo = 1, hi = tau;
            while (lo < hi) {
                const u32 mid = (lo + hi) >> 1;
                if (a >= s_B[mid - 1]) hi = mid; else lo = mid + 1;
            }
            const u32 key = keys[g.tile0 + s_idx[j]];
            const u64 rank = base + j;
            if (rank < codes_capacity) codes[rank] = (uint8_t)(((vb >> 31) << 7) | (lo - 1));
            else set_status(ctrl, FASTSGD_ERR_BUFFER_TOO_SMALL);
            if (rank < ckeys_capacity) ckeys[rank] = key;
        }
        __syncthreads();
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
        if (t == 0) s_item_lo = atomicAdd(&ctrl->ticket_key, 1u);   // items < 2^32
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
