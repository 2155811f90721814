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

// One key block per WAVE, 1024 keys at a time; lane `lane` holds, for row q = 0..15, key 64*q + lane.
// Per round the wave fetches the round's flag words, the payload words the round can reach (its start
// is known from the rounds before, its end is bounded by M bits per key) and the code bytes in one
// go, parks flags and payload in its slice of shared memory, and then per row: flag -> level ->
// length, a scan of the lengths -> bit offsets, a 64-bit window at that offset -> delta, a scan of the
// deltas on top of the key before the row -> keys (phase 2), code byte -> magnitude table -> value
// (phases 3-4).  The waves of a workgroup never synchronise.
__global__ void __launch_bounds__(kThreads)
k_decode(const uint8_t* __restrict__ streams, const DecSeg* __restrict__ segs, u32 n_segments, DecCtrl* ctrl,
         u32* __restrict__ keys_out, float* __restrict__ values_out, u64* out_counts, u32 n_counts,
         u32* out_status) {
    __shared__ u32 s_payall[kWaves][kSub + 2];
    __shared__ u32 s_flgall[kWaves][kSub * 5 / 32 + 2];
    __shared__ u32 s_Vall[kWaves][128];
    const u32 lane = lane_id(), w = uniform(wave_id());
    u32* s_pay = s_payall[w];
    u32* s_flg = s_flgall[w];
    u32* s_V = s_Vall[w];
    const u64 total_items = ctrl->total_items;
    u32 cur_seg = 0xFFFFFFFFu;

    for (u64 item = (u64)blockIdx.x * kWaves + w; item < total_items; item += (u64)gridDim.x * kWaves) {
        const u32 seg = (n_segments == 1) ? 0u : uniform(find_dec_segment(segs, n_segments, item));
        const DecSeg* ds = &segs[seg];
        const u32 KB = uniform(ds->KB), l = uniform(ds->l), tau = uniform(ds->tau), nb = uniform(ds->nb);
        const u64 d = ds->d;
        const u32 blk = uniform((u32)(item - ds->item_begin));
        const u32 first = blk * KB;
        const u32 cnt = uniform((u32)((d - first < KB) ? d - first : KB));
        const u32 nsub = (cnt + kSub - 1) / kSub;
        if (seg != cur_seg) {
            wave_lds_sync();
            s_V[lane] = ds->V[lane];
            s_V[lane + 64] = ds->V[lane + 64];
            cur_seg = seg;
            wave_lds_sync();
        }
        // directory entry of the block and of the next one, checked against each other
        const u32* dir = reinterpret_cast<const u32*>(streams + ds->dir_off + 16ull * blk);
        const bool has_next = blk + 1 < nb;
        const u32 dword = (lane < 4 || (lane < 8 && has_next)) ? dir[lane] : 0u;
        const u32 off8 = read_lane(dword, 0), preKey = read_lane(dword, 1), M = read_lane(dword, 2);
        const u32 pbits = read_lane(dword, 3), next_off8_dir = read_lane(dword, 4), next_pre = read_lane(dword, 5);
        const u64 total_words = ds->total_words;
        const u64 next_off8 = has_next ? (u64)next_off8_dir : total_words;
        const u32 fwords = (cnt * l + 63u) >> 6, pwords = (pbits + 63u) >> 6;
        bool bad = (M < 1 || M > 32) || (pbits > cnt * 32u) || ((u64)off8 + fwords + pwords != next_off8) ||
                   ((u64)off8 + fwords + pwords > total_words) || (blk == 0 && (off8 != 0 || preKey != 0));
        if (!bad) {
            const u32* fsrc = reinterpret_cast<const u32*>(streams + ds->blocks_off + 8ull * off8);   // flags plane
            const u32* psrc = fsrc + 2u * fwords;                                                    // payload plane
            const u32 pw_total = 2u * pwords;
            const uint8_t* codes = streams + ds->stream_begin + kHeaderBytes + first;
            const u64 out0 = ds->pair_begin + first;
            u32 pbit = 0;                  // payload bits consumed by the rounds before
            u32 carry = preKey;            // key before the row in hand
            bool wrapped = false, badcode = false;
            for (u32 sub = 0; sub < nsub; ++sub) {
                const u32 n = cnt - sub * kSub < kSub ? cnt - sub * kSub : kSub;
                const u32 nfw = (n * l + 31u) >> 5, f0 = sub * 32u * l;
                const u32 pw0 = pbit >> 5, wbits = pbit & 31u;
                u32 npw = ((wbits + n * M + 31u) >> 5) + 1u;           // words this round can reach (+1: windows)
                if (npw > kSub + 2) npw = kSub + 2;
                // all fetches of the round first
                u32 fw[3], pwd[17], code[kKeyRows];
#pragma unroll
                for (u32 k = 0; k < 3; ++k) { const u32 i = k * 64u + lane; fw[k] = fsrc[f0 + (i < nfw ? i : 0u)]; }
#pragma unroll
                for (u32 k = 0; k < 17; ++k) {
                    const u32 i = k * 64u + lane;
                    pwd[k] = (k * 64u < npw && pw_total) ? psrc[(pw0 + i < pw_total) ? pw0 + i : pw_total - 1u] : 0u;
                }
#pragma unroll
                for (u32 q = 0; q < kKeyRows; ++q) code[q] = (q * 64u + lane < n) ? codes[sub * kSub + q * 64u + lane] : 0u;
#pragma unroll
                for (u32 k = 0; k < 3; ++k) { const u32 i = k * 64u + lane; if (i < nfw + 1u) s_flg[i] = (i < nfw) ? fw[k] : 0u; }
#pragma unroll
                for (u32 k = 0; k < 17; ++k) {
                    const u32 i = k * 64u + lane;
                    if (k * 64u < npw && i < npw) s_pay[i] = (pw0 + i < pw_total) ? pwd[k] : 0u;
                }
                wave_lds_sync();
                u32 rowbase = wbits;
#pragma unroll
                for (u32 q = 0; q < kKeyRows; ++q) {
                    const u32 i = q * 64u + lane;
                    if (q * 64u < n) {
                        u32 len = 0;
                        if (i < n) {
                            const u32 fpos = i * l;
                            const u64 win = (u64)s_flg[fpos >> 5] | ((u64)s_flg[(fpos >> 5) + 1] << 32);
                            const u32 level = ((u32)(win >> (fpos & 31u)) & ((1u << l) - 1u)) + 1u;
                            len = level_len(level, M, l);
                        }
                        const u32 incl = wave_incl_scan(len);
                        u32 delta = 0;
                        if (i < n) {
                            const u32 bitpos = rowbase + incl - len;
                            const u64 win = (u64)s_pay[bitpos >> 5] | ((u64)s_pay[(bitpos >> 5) + 1] << 32);
                            const u32 mask = len >= 32u ? 0xFFFFFFFFu : ((1u << len) - 1u);
                            delta = (u32)(win >> (bitpos & 31u)) & mask;
                        }
                        rowbase += read_lane(incl, 63);
                        const u32 key = carry + wave_incl_scan(delta);          // modulo 2^32 ...
                        const u32 prev = lane_above(key, carry);
                        if (i < n) {
                            wrapped |= key < prev;                              // ... so a wrap shows as a step down
                            const u32 byte = code[q];
                            const u32 c = (byte & 0x7Fu) + 1u;
                            if (c > tau) badcode = true;
                            else {
                                keys_out[out0 + sub * kSub + i] = key;
                                values_out[out0 + sub * kSub + i] = __uint_as_float(s_V[c - 1] | ((byte >> 7) << 31));
                            }
                        }
                        const u32 last_lane = (n - q * 64u) < 64u ? (n - q * 64u - 1u) : 63u;
                        carry = read_lane(key, uniform(last_lane));
                    }
                }
                pbit = rowbase - wbits + pbit;
                if (pbit > pbits) { bad = true; break; }        // the lengths overrun the payload plane
                wave_lds_sync();
            }
            bad = bad || (pbit != pbits) || __any(wrapped) || __any(badcode) || (has_next && carry != next_pre);
        }
        if (bad && lane == 0) dec_fail(ctrl, FASTSGD_ERR_CORRUPT_STREAM, out_status, out_counts, n_counts);
    }
}

}  // namespace fsgd
