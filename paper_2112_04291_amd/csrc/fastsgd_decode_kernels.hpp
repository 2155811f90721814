// Decoder kernels of the gfx950 FastSGD codec (Section 3.1 of arXiv 2112.04291, decoder phases 1-4).
//
//   k_decode_setup   per stream: validate the header, rebuild the table of decoded magnitudes
//                    sum / b^c (phases 3-4 evaluated once per code)
//   k_decode_plan    pair offsets and work-item numbering over the streams of a batch
//   k_decode         per key block: flags -> lengths -> bit offsets -> deltas (phase 1),
//                    prefix sum + preKey -> keys (phase 2), code byte -> value (phases 3-4)
#pragma once
#include "fastsgd_device.hpp"

namespace fsgd {

struct DecSeg {
    u64 stream_begin;   // byte offset of the stream in the buffer
    u64 d, pair_begin, item_begin;
    u64 dir_off, blocks_off, total_words;   // absolute byte offsets; words of all key blocks
    u32 nb, l, tau, KB;
    u32 ok, pad[3];
    u32 V[128];         // V[c-1] = bit pattern of the decoded magnitude of code c
};

struct DecCtrl {
    u32 status, pad;
    u64 total_items, total_pairs;
};

__device__ __forceinline__ void dec_fail(DecCtrl* ctrl, u32 code, u32* out_status, u64* out_counts, u32 n_counts) {
    if (atomicCAS(&ctrl->status, 0u, code) == 0u) *out_status = code;
    for (u32 i = 0; i < n_counts; ++i) out_counts[i] = 0;
}

__device__ __forceinline__ void plan_streams(DecSeg* segs, u32 n_segments, u64 capacity, DecCtrl* ctrl,
                                             u64* out_counts, u32 single, u32* out_status) {
    // serial over streams: a batch has at most a few thousand
    u64 pairs = 0, items = 0;
    bool ok = (ctrl->status == 0);
    for (u32 s = 0; s < n_segments; ++s) {
        segs[s].pair_begin = pairs;
        segs[s].item_begin = items;
        pairs += segs[s].d;
        items += segs[s].nb;
    }
    u32 status = ctrl->status;
    if (ok && pairs > capacity) { status = FASTSGD_ERR_BUFFER_TOO_SMALL; ctrl->status = status; ok = false; }
    ctrl->total_items = ok ? items : 0;
    ctrl->total_pairs = ok ? pairs : 0;
    if (single) out_counts[0] = ok ? pairs : 0;
    else {
        for (u32 s = 0; s < n_segments; ++s) out_counts[s] = ok ? segs[s].pair_begin : 0;
        out_counts[n_segments] = ok ? pairs : 0;
    }
    *out_status = status;
}

__global__ void __launch_bounds__(128)
k_decode_setup(const uint8_t* __restrict__ streams, u64 total_bytes, const u64* __restrict__ stream_offsets,
               u32 n_segments, DecSeg* segs, DecCtrl* ctrl, u64 capacity, u64* out_counts, u32* out_status) {
    // launched with one workgroup per stream; for a batch k_decode_clear has reset ctrl beforehand
    __shared__ double s_P[129];
    __shared__ double s_sum;
    __shared__ u32 s_ok, s_tau;
    const u32 seg = blockIdx.x, t = threadIdx.x;
    DecSeg* ds = &segs[seg];
    if (t == 0) {
        if (n_segments == 1) ctrl->status = 0;
        const u64 begin = stream_offsets ? stream_offsets[seg] : 0;
        const u64 end = stream_offsets ? stream_offsets[seg + 1] : total_bytes;
        bool ok = (begin <= end) && (end <= total_bytes) && ((begin & 7) == 0) && (end - begin >= kHeaderBytes);
        u32 l = 0, tau = 1, KB = 256, nb = 0;
        u64 d = 0, dir_off = 0, blocks_off = 0, total_words = 0;
        double base = 2.0, sum = 0.0;
        if (ok) {
            const u64* h = reinterpret_cast<const u64*>(streams + begin);
            const u64 h0 = h[0], h1 = h[1];
            l = (u32)(h0 >> 40) & 0xFF; tau = (u32)(h0 >> 48) & 0xFF; KB = (u32)h1; nb = (u32)(h1 >> 32);
            base = __longlong_as_double((long long)h[2]);
            sum = __longlong_as_double((long long)h[3]);
            const u64 n = h[4], total = h[6];
            d = h[5];
            ok = ((u32)h0 == kMagic) && (((h0 >> 32) & 0xFF) == kVersion) && ((h0 >> 56) == 0);
            ok = ok && l >= 1 && l <= 5 && tau >= 1 && tau <= 128;
            ok = ok && KB >= 256 && KB <= kMaxKB && (KB & (KB - 1)) == 0;
            ok = ok && (base >= 1.0 + 1.0 / 1048576.0) && (base <= 16.0);
            ok = ok && (sum >= 0.0) && (sum < __longlong_as_double(0x7FF0000000000000ll));
            ok = ok && n <= 4294967296ull && d <= n;
            if (ok) {
                ok = (u64)nb == (d + KB - 1) / KB;
                dir_off = kHeaderBytes + ((d + 7) & ~7ull);
                blocks_off = dir_off + 16ull * nb;
                ok = ok && total <= end - begin && total >= blocks_off && (total & 7) == 0;
                total_words = ok ? (total - blocks_off) >> 3 : 0;
                dir_off += begin; blocks_off += begin;
            }
        }
        if (!ok) { d = 0; nb = 0; tau = 1; }
        ds->stream_begin = begin; ds->d = d; ds->nb = nb; ds->l = l; ds->tau = tau; ds->KB = KB;
        ds->dir_off = dir_off; ds->blocks_off = blocks_off; ds->total_words = total_words; ds->ok = ok;
        if (!ok) atomicCAS(&ctrl->status, 0u, (u32)FASTSGD_ERR_CORRUPT_STREAM);
        s_ok = ok; s_tau = tau; s_sum = sum;
        if (ok) power_chain(base, tau, s_P);
    }
    __syncthreads();
    if (s_ok && t < s_tau) {            // thread t owns code c = t + 1
        const double sum = s_sum;
        ds->V[t] = (sum > 0.0) ? f64_to_f32_bits(sum / s_P[t + 1], false) : 0u;
    }
    if (n_segments == 1) {           // a single stream needs no separate planning launch
        __syncthreads();
        if (t == 0) plan_streams(segs, 1, capacity, ctrl, out_counts, stream_offsets == nullptr, out_status);
    }
}

__global__ void k_decode_clear(DecCtrl* ctrl) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { ctrl->status = 0; ctrl->total_items = 0; ctrl->total_pairs = 0; }
}

__global__ void k_decode_plan(DecSeg* segs, u32 n_segments, u64 capacity, DecCtrl* ctrl, u64* out_counts,
                              u32* out_status) {
    if (threadIdx.x == 0 && blockIdx.x == 0) plan_streams(segs, n_segments, capacity, ctrl, out_counts, 0, out_status);
}

__device__ __forceinline__ u32 find_dec_segment(const DecSeg* segs, u32 n_segments, u64 item) {
    u32 lo = 0, hi = n_segments;
    while (hi - lo > 1) {
        u32 mid = (lo + hi) >> 1;
        if (segs[mid].item_begin <= item) lo = mid; else hi = mid;
    }
    return lo;
}

__global__ void __launch_bounds__(kThreads)
k_decode(const uint8_t* __restrict__ streams, const DecSeg* __restrict__ segs, u32 n_segments, DecCtrl* ctrl,
         u32* __restrict__ keys_out, float* __restrict__ values_out, u64* out_counts, u32 n_counts,
         u32* out_status) {
    __shared__ u32 s_flags[kMaxKB * 5 / 32 + 2];
    __shared__ u32 s_pay[kMaxKB + 2];
    __shared__ u32 s_V[128];
    __shared__ u32 s_scan[kWaves + 1];
    __shared__ u64 s_scan64[kWaves];
    __shared__ u32 s_bad;
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    const u64 total_items = ctrl->total_items;
    u32 cur_seg = 0xFFFFFFFFu;

    for (u64 item = blockIdx.x; item < total_items; item += gridDim.x) {
        const u32 seg = (n_segments == 1) ? 0u : find_dec_segment(segs, n_segments, item);
        const DecSeg* ds = &segs[seg];
        const u32 KB = ds->KB, l = ds->l, tau = ds->tau, nb = ds->nb;
        const u64 d = ds->d;
        const u32 blk = (u32)(item - ds->item_begin);
        const u64 first = (u64)blk * KB;
        const u32 cnt = (u32)((d - first < KB) ? d - first : KB);
        const u32 per = KB / kThreads;
        if (seg != cur_seg) {
            __syncthreads();
            if (t < 128) s_V[t] = ds->V[t];
            cur_seg = seg;
        }
        if (t == 0) s_bad = 0;

        // directory entry, checked against its neighbour
        const u32* dir = reinterpret_cast<const u32*>(streams + ds->dir_off + 16ull * blk);
        const u32 off8 = dir[0], preKey = dir[1], M = dir[2], pbits = dir[3];
        const u64 next_off8 = (blk + 1 < nb) ? (u64)dir[4] : ds->total_words;
        const u32 fwords = (cnt * l + 63u) >> 6, pwords = (pbits + 63u) >> 6;
        bool bad = (M < 1 || M > 32) || (pbits > cnt * 32u) || ((u64)off8 + fwords + pwords != next_off8) ||
                   ((u64)off8 + fwords + pwords > ds->total_words) || (blk == 0 && (off8 != 0 || preKey != 0));
        __syncthreads();
        if (!bad) {
            const u64* src = reinterpret_cast<const u64*>(streams + ds->blocks_off + 8ull * off8);
            for (u32 i = t; i < fwords; i += kThreads) {
                const u64 x = src[i];
                s_flags[2 * i] = (u32)x; s_flags[2 * i + 1] = (u32)(x >> 32);
            }
            for (u32 i = t; i < pwords; i += kThreads) {
                const u64 x = src[fwords + i];
                s_pay[2 * i] = (u32)x; s_pay[2 * i + 1] = (u32)(x >> 32);
            }
            if (t < 2) { s_flags[2 * fwords + t] = 0; s_pay[2 * pwords + t] = 0; }   // window reads run one word over
        }
        __syncthreads();

        // phase 1: lengths from the flags, bit offsets by a scan
        u32 len[16], mybits = 0;
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            len[k] = 0;
            if (!bad && k < per && i < cnt) {
                const u32 fpos = i * l;
                const u64 win = (u64)s_flags[fpos >> 5] | ((u64)s_flags[(fpos >> 5) + 1] << 32);
                const u32 level = ((u32)(win >> (fpos & 31u)) & ((1u << l) - 1u)) + 1u;
                len[k] = (level * M + (1u << l) - 1u) >> l;
                mybits += len[k];
            }
        }
        u32 total_bits;
        u32 bitpos = block_excl_scan(mybits, s_scan, &total_bits);
        bad = bad || (total_bits != pbits);

        // deltas and their running sum inside the thread
        u64 run = 0;
        u64 local[16];
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            local[k] = 0;
            if (!bad && k < per && i < cnt) {
                const u64 win = (u64)s_pay[bitpos >> 5] | ((u64)s_pay[(bitpos >> 5) + 1] << 32);
                const u32 mask = len[k] >= 32u ? 0xFFFFFFFFu : ((1u << len[k]) - 1u);
                run += (u32)(win >> (bitpos & 31u)) & mask;
                local[k] = run;
                bitpos += len[k];
            }
        }
        // phase 2: prefix sum across the workgroup, plus preKey
        const u64 incl = wave_incl_scan64(run);
        if (lane == 63) s_scan64[w] = incl;
        __syncthreads();
        u64 before = preKey, block_sum = 0;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            if (k < w) before += s_scan64[k];
            block_sum += s_scan64[k];
        }
        before += incl - run;
        const u64 last_key = (u64)preKey + block_sum;
        bad = bad || (last_key > 0xFFFFFFFFull) || (blk + 1 < nb && (u32)last_key != dir[5]);

        // phases 3-4 and the writes
        const u64 out0 = ds->pair_begin + first;
        const uint8_t* codes = streams + ds->stream_begin + kHeaderBytes + first;
        bool badcode = false;
#pragma unroll
        for (u32 k = 0; k < 16; ++k) {
            const u32 i = t * per + k;
            if (!bad && k < per && i < cnt) {
                const u32 byte = codes[i];
                const u32 c = (byte & 0x7Fu) + 1u;
                if (c > tau) badcode = true;
                else {
                    keys_out[out0 + i] = (u32)(before + local[k]);
                    values_out[out0 + i] = __uint_as_float(s_V[c - 1] | ((byte >> 7) << 31));
                }
            }
        }
        if (bad || badcode) s_bad = 1;
        __syncthreads();
        if (s_bad && t == 0) dec_fail(ctrl, FASTSGD_ERR_CORRUPT_STREAM, out_status, out_counts, n_counts);
        __syncthreads();
    }
}

}  // namespace fsgd
