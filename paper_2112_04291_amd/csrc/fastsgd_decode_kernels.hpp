// Decoder kernels of the gfx950 FastSGD codec (Section 3.1 of arXiv 2112.04291, decoder phases 1-4).
//
//   k_decode_setup   batches, per stream: validate the header, rebuild the table of decoded magnitudes
//                    sum / b^c (phases 3-4 evaluated once per code)
//   k_decode_plan    pair offsets and work-item numbering over the streams of a batch
//   k_decode         per key block: flags -> lengths -> bit offsets -> deltas (phase 1),
//                    prefix sum + preKey -> keys (phase 2), code byte -> value (phases 3-4).
//                    A single stream needs no other launch: every wave checks the header and rebuilds
//                    the magnitude table itself, and the last workgroup to finish reports the outcome.
#pragma once
#include "fastsgd_device.hpp"

namespace fsgd {

struct DecSeg {
    u64 stream_begin;   // byte offset of the stream in the buffer
    u64 d, pair_begin, item_begin;
    u64 dir_off, blocks_off, total_words;   // absolute byte offsets; words of all key blocks
    u32 nb, l, tau, KB;
    u32 ok, pad[3];
    u32 V[kMaxTau];     // V[c-1] = bit pattern of the decoded magnitude of code c
};

struct DecCtrl {
    u32 status, pad;
    u64 total_items, total_pairs;
};

// Completion count of a single-stream launch (which has no setup kernel and no kernel after it): the
// workgroups that have key blocks to decode count themselves in when their waves are through, and the one
// that completes the count reports the launch's outcome.  Atomics on one address are served one after the
// other, a few nanoseconds each, so the count is kept in kDoneGroups words on cache lines of their own
// (workgroup b counts in group b mod kDoneGroups) and one word on top that counts the completed groups.
// All words must be zero when a launch begins and are zero again when it ends: the counters wrap (atomicInc)
// and the last workgroup takes the failure word away, so they need clearing only once, before the
// workspace's first use.  Batch launches never touch them.
constexpr u32 kDoneGroups = 16;
struct DecDone {
    u32 fail;                    // the gravest failure the waves of the launch found (a fastsgd_status), 0 = none
    u32 top;                     // groups that have completed
    u32 pad[30];
    u32 group[kDoneGroups][32];  // [g][0]: workgroups of group g that have finished
};
constexpr u64 kDecDoneOffset = 128;       // in the decoder workspace
constexpr u64 kDecSegOffset = 4096;       // the per-stream records of a batch start here
static_assert(kDecDoneOffset + sizeof(DecDone) <= kDecSegOffset && sizeof(DecCtrl) <= kDecDoneOffset, "decoder workspace layout");

// What a stream's header says, checked; byte offsets are relative to the start of the stream.
struct DecHead {
    u64 d, dir_off, blocks_off, total_words;
    u32 nb, l, tau, KB;
    double base, sum;
};

// Parses and checks the 64-byte header at `h` of a stream that may use up to `avail` bytes.
__device__ __forceinline__ bool parse_header(const u64* __restrict__ h, u64 avail, DecHead& hd) {
    const u64 h0 = h[0], h1 = h[1];
    hd.l = (u32)(h0 >> 40) & 0xFF; hd.tau = (u32)(h0 >> 48); hd.KB = (u32)h1; hd.nb = (u32)(h1 >> 32);
    hd.base = __longlong_as_double((long long)h[2]);
    hd.sum = __longlong_as_double((long long)h[3]);
    const u64 n = h[4], total = h[6];
    hd.d = h[5];
    const u32 l = hd.l, tau = hd.tau, KB = hd.KB;
    bool ok = ((u32)h0 == kMagic) && (((h0 >> 32) & 0xFF) == kVersion);
    ok = ok && l >= 1 && l <= 5 && tau >= 1 && tau <= kMaxTau;
    ok = ok && KB >= 256 && KB <= kMaxKB && (KB & (KB - 1)) == 0;
    ok = ok && (hd.base >= 1.0 + 1.0 / 1048576.0) && (hd.base <= (tau > 128 ? 4.0 : 16.0));
    ok = ok && (hd.sum >= 0.0) && (hd.sum < __longlong_as_double(0x7FF0000000000000ll));
    ok = ok && n <= 4294967296ull && hd.d <= n;
    hd.dir_off = 0; hd.blocks_off = 0; hd.total_words = 0;
    if (ok) {
        ok = (u64)hd.nb == (hd.d + KB - 1) / KB;
        hd.dir_off = kHeaderBytes + value_plane_bytes(hd.d, code_width(tau));
        hd.blocks_off = hd.dir_off + 16ull * hd.nb;
        ok = ok && total <= avail && total >= hd.blocks_off && (total & 7) == 0;
        hd.total_words = ok ? (total - hd.blocks_off) >> 3 : 0;
    }
    return ok;
}

// A failure found while decoding.  If waves find different ones, the larger code stays: a corrupt stream
// outranks a buffer that is too small.
__device__ __forceinline__ void dec_fail(DecCtrl* ctrl, u32 code, u32* out_status, u64* out_counts, u32 n_counts) {
    atomicMax(&ctrl->status, code);
    atomicMax(out_status, code);
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

__global__ void __launch_bounds__(kMaxTau)
k_decode_setup(const uint8_t* __restrict__ streams, u64 total_bytes, const u64* __restrict__ stream_offsets,
               u32 plan_inline, DecSeg* segs, DecCtrl* ctrl, u64 capacity, u64* out_counts, u32* out_status) {
    // launched with one workgroup per stream; for a batch k_decode_clear has reset ctrl beforehand
    __shared__ double s_P[kMaxTau + 1];
    __shared__ double s_sum;
    __shared__ u32 s_ok, s_tau;
    const u32 seg = blockIdx.x, t = threadIdx.x;
    DecSeg* ds = &segs[seg];
    if (t == 0) {
        if (plan_inline) ctrl->status = 0;
        const u64 begin = stream_offsets ? stream_offsets[seg] : 0;
        const u64 end = stream_offsets ? stream_offsets[seg + 1] : total_bytes;
        bool ok = (begin <= end) && (end <= total_bytes) && ((begin & 7) == 0) && (end - begin >= kHeaderBytes);
        u32 l = 0, tau = 1, KB = 256, nb = 0;
        u64 d = 0, dir_off = 0, blocks_off = 0, total_words = 0;
        double base = 2.0, sum = 0.0;
        if (ok) {
            DecHead hd;
            ok = parse_header(reinterpret_cast<const u64*>(streams + begin), end - begin, hd);
            l = hd.l; tau = hd.tau; KB = hd.KB; nb = hd.nb; d = hd.d; base = hd.base; sum = hd.sum;
            dir_off = hd.dir_off + begin; blocks_off = hd.blocks_off + begin; total_words = hd.total_words;
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
    if (plan_inline) {               // a single stream needs no separate planning launch
        __syncthreads();
        if (t == 0) plan_streams(segs, 1, capacity, ctrl, out_counts, stream_offsets == nullptr, out_status);
    }
}

__global__ void k_decode_clear(DecCtrl* ctrl) {
    if (threadIdx.x == 0 && blockIdx.x == 0) { ctrl->status = 0; ctrl->total_items = 0; ctrl->total_pairs = 0; }
}

// Batch: pair offsets and work-item numbering over the streams, one workgroup scanning 256 streams
// at a time.
__global__ void __launch_bounds__(kThreads)
k_decode_plan(DecSeg* segs, u32 n_segments, u64 capacity, DecCtrl* ctrl, u64* out_counts, u32* out_status,
              u64* total_out) {
    __shared__ u64 s_wave[2][kWaves];
    __shared__ u64 s_carry[2];
    const u32 t = threadIdx.x, lane = lane_id(), w = wave_id();
    if (t < 2) s_carry[t] = 0;
    __syncthreads();
    for (u32 s0 = 0; s0 < n_segments; s0 += kThreads) {
        const u32 s = s0 + t;
        const u64 d = s < n_segments ? segs[s].d : 0, nb = s < n_segments ? segs[s].nb : 0;
        const u64 id = wave_incl_scan64(d), ib = wave_incl_scan64(nb);
        if (lane == 63) { s_wave[0][w] = id; s_wave[1][w] = ib; }
        __syncthreads();
        u64 bd = s_carry[0], bb = s_carry[1], td = 0, tb = 0;
#pragma unroll
        for (u32 k = 0; k < kWaves; ++k) {
            const u64 a = s_wave[0][k], b = s_wave[1][k];
            if (k < w) { bd += a; bb += b; }
            td += a; tb += b;
        }
        if (s < n_segments) {
            segs[s].pair_begin = bd + id - d;
            segs[s].item_begin = bb + ib - nb;
        }
        __syncthreads();
        if (t == 0) { s_carry[0] += td; s_carry[1] += tb; }
        __syncthreads();
    }
    const u64 pairs = s_carry[0], items = s_carry[1];
    u32 status = ctrl->status;
    __syncthreads();
    bool ok = (status == 0);
    if (ok && pairs > capacity) { status = FASTSGD_ERR_BUFFER_TOO_SMALL; ok = false; }
    for (u32 s = t; s < n_segments; s += kThreads) out_counts[s] = ok ? segs[s].pair_begin : 0;
    if (t == 0) {
        ctrl->status = status;
        ctrl->total_items = ok ? items : 0;
        ctrl->total_pairs = ok ? pairs : 0;
        out_counts[n_segments] = ok ? pairs : 0;
        if (total_out) *total_out = ok ? pairs : 0;
        *out_status = status;
    }
}

// Stream that work item `item` belongs to: the last one whose first item is not beyond it.
__device__ __forceinline__ u32 find_dec_segment(const DecSeg* segs, u32 n_segments, u64 item) {
    return wave_upper_index(n_segments, item, [&](u32 i) { return segs[i].item_begin; });
}

// One key block per WAVE, 1024 keys at a time, each lane owning 16 CONSECUTIVE keys of the round, so
// that the running sums inside a lane are plain additions and only one scan across the wave is needed
// for the lengths and one for the deltas:
//   the round's flag words, the payload words it can reach (its start is known from the rounds before,
//   its end is bounded by M bits per key) and the lane's 16 code bytes are fetched in one go; flags and
//   payload are parked in the wave's slice of shared memory -> per key: flag -> level -> length;
//   lengths summed up inside the lane, scanned across the wave -> bit offsets; a 64-bit window at that
//   offset -> delta; deltas summed up inside the lane, scanned across the wave on top of the key before
//   the round -> keys (phase 2); code byte -> magnitude table -> value (phases 3-4).  Keys and values
//   go through shared memory once more so that the stores to the output arrays are coalesced.
// The waves of a workgroup never synchronise.

// a * b + c for a, b below 2^24, in one full-rate instruction (a plain 32-bit multiply runs at a quarter
// of the rate and the compiler does not know the operands are small); b must be wave-uniform.
__device__ __forceinline__ u32 mad24(u32 a, u32 b, u32 c) {
    u32 r;
    asm("v_mad_u32_u24 %0, %1, %2, %3" : "=v"(r) : "v"(a), "s"(b), "v"(c));
    return r;
}

// What a decode launch does with the pairs: store them, add every value to dense[key] (Section 2.1,
// aggregation), or apply the Adam step of Section 4.1 at every key.
enum : int { kStore = 0, kAccum = 1, kAdam = 2, kHand = 3 };   // kHand: hand the pairs back to the caller, 16 consecutive ones per lane

// Adam state and hyper-parameters (Section 4.1); theta is passed as the dense array.
struct AdamArgs {
    float* m;
    float* v;
    float eta, beta1, one_minus_beta1, beta2, one_minus_beta2, eps;
};

// FULL: the round has all 1024 keys (no key-index tests).  MODE kAccum / kAdam: instead of storing the
// pairs, update the dense arrays at every key (keys are unique inside a stream, so plain
// read-modify-write is enough); a key >= dense_len sets too_big.  stream_start: the round begins with the
// stream's first key, the only one whose delta may be 0 (Eq. 4 is taken over distinct ascending keys).
// Returns false if the stream is corrupt.
template <bool FULL, int MODE>
__device__ __forceinline__ bool decode_round(const u32* __restrict__ fsrc_round, const u32* __restrict__ psrc,
                                             u32 pw_total, const uint8_t* __restrict__ codes_round, u32 n, u32 l,
                                             u32 M, u32 tau, u32 cwid, u32 pbits, u32& pbit, u32& carry, u32 lane,
                                             u32* s_pay, u32* s_flg, u32* s_cod, const u32* s_V, u32* __restrict__ keys_dst,
                                             float* __restrict__ values_dst, float* __restrict__ dense, u64 dense_len,
                                             const AdamArgs& adam, bool& too_big, bool stream_start,
                                             u32 (&out_keys)[kLaneKeys], u32 (&out_vals)[kLaneKeys]) {
    const u32 nfw = (n * l + 31u) >> 5;
    const u32 pw0 = pbit >> 5, wbits = pbit & 31u;
    u32 npw = ((wbits + n * M + 31u) >> 5) + 1u;           // words this round can reach (+1: windows)
    if (npw > kSub + 2) npw = kSub + 2;
    // all fetches of the round first; flags and payload through buffer descriptors that end with the
    // words the round may use, so that lanes beyond them read 0 without a test
    u32 fw[3], pwd[17];
    const u32 pw_left = pw_total > pw0 ? pw_total - pw0 : 0u;
    const __amdgpu_buffer_rsrc_t frs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u32*>(fsrc_round), 0, (int)uniform(nfw * 4u), kBufferWord3);
    const __amdgpu_buffer_rsrc_t prs = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<u32*>(psrc + uniform(pw0)), 0, (int)uniform((pw_left < npw ? pw_left : npw) * 4u), kBufferWord3);
#pragma unroll
    for (u32 k = 0; k < 3; ++k) fw[k] = __builtin_amdgcn_raw_buffer_load_b32(frs, (int)(lane * 4u + k * 256u), 0, 0);
#pragma unroll
    for (u32 k = 0; k < 17; ++k)
        pwd[k] = (k * 64u < npw) ? __builtin_amdgcn_raw_buffer_load_b32(prs, (int)(lane * 4u + k * 256u), 0, 0) : 0u;
    u32 cw[4];                                             // the lane's 16 code bytes
    if (cwid != 8) {
        // narrower tokens are widened further down, once the other fetches are parked
    } else if (FULL) {
        const uint2* c2 = reinterpret_cast<const uint2*>(codes_round) + 2u * lane;   // 8-byte aligned
        const uint2 a = c2[0], b = c2[1];
        cw[0] = a.x; cw[1] = a.y; cw[2] = b.x; cw[3] = b.y;
    } else {
        // through a descriptor that ends with the round's last word of bytes (the plane is padded to 64 bits):
        // words beyond it read 0, the bytes of the last word beyond n are masked away
        const __amdgpu_buffer_rsrc_t crs = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<uint8_t*>(codes_round), 0, (int)uniform((n + 3u) & ~3u), kBufferWord3);
#pragma unroll
        for (u32 j = 0; j < 4; ++j) {
            const u32 i0 = lane * kLaneKeys + j * 4u;
            u32 x = __builtin_amdgcn_raw_buffer_load_b32(crs, (int)i0, 0, 0);
            const u32 left = n > i0 ? n - i0 : 0u;          // bytes of the round from here on
            if (left < 4u) x &= (1u << (8u * left)) - 1u;
            cw[j] = x;
        }
    }
#pragma unroll
    for (u32 k = 0; k < 3; ++k) s_flg[k * 64u + lane] = fw[k];                     // (zeros behind the round's flags)
#pragma unroll
    for (u32 k = 0; k < 17; ++k)
        if (k * 64u < npw) s_pay[k * 64u + lane] = pwd[k];                         // (zeros behind the payload)
    wave_lds_sync();
    if (MODE != kHand && cwid != 8) {
        // token i of the round sits at bit i * cwid of the round's words; narrow ones are widened to the
        // byte form (sign in bit 7, code-1 below) through shared memory
        const u32* cwords = reinterpret_cast<const u32*>(codes_round);
        uint8_t* s_codb = reinterpret_cast<uint8_t*>(s_cod + kCodeWords);
        const u32 ncw = (n * cwid + 31u) >> 5;
        for (u32 i = lane; i < ncw + 1u; i += 64) s_cod[i] = (i < ncw) ? cwords[i] : 0u;
        wave_lds_sync();
        if (cwid < 8) {
            const u32 tmask = (1u << cwid) - 1u, cmask = tmask >> 1;
#pragma unroll 1
            for (u32 i = lane; i < kSub; i += 64) {
                u32 byte = 0;
                if (i < n) {
                    const u32 pos = i * cwid, wa = pos >> 5;
                    const u32 tok = __builtin_amdgcn_alignbit(s_cod[wa + 1u], s_cod[wa], pos & 31u) & tmask;
                    byte = ((tok >> (cwid - 1u)) << 7) | (tok & cmask);
                }
                s_codb[i] = (uint8_t)byte;
            }
            wave_lds_sync();
            const uint4 q = reinterpret_cast<const uint4*>(s_codb)[lane];
            cw[0] = q.x; cw[1] = q.y; cw[2] = q.z; cw[3] = q.w;
        }
        // (nine-bit tokens stay where they are until the values are looked up)
    }

    // flags -> lengths: 8 flags at a time out of a 64-bit window of the lane's flag bits
    const u32 lmask = (1u << l) - 1u, lenc = M + lmask;     // length = (flag * M + M + 2^l - 1) >> l
    const u32 Mu = uniform(M);
    u32 len[kLaneKeys];
#pragma unroll
    for (u32 half = 0; half < 2; ++half) {
        const u32 fb = (lane * kLaneKeys + half * 8u) * l, wi = fb >> 5;
        const u32 w0 = s_flg[wi], w1 = s_flg[wi + 1], w2 = s_flg[wi + 2];
        u64 fwin = (u64)__builtin_amdgcn_alignbit(w1, w0, fb & 31u) |
                   ((u64)__builtin_amdgcn_alignbit(w2, w1, fb & 31u) << 32);
#pragma unroll
        for (u32 k = 0; k < 8; ++k) {
            const u32 flag = (u32)fwin & lmask;
            fwin >>= l;
            u32 ln = mad24(flag, Mu, lenc) >> l;
            if (!FULL && lane * kLaneKeys + half * 8u + k >= n) ln = 0;
            len[half * 8u + k] = ln;
        }
    }
    u32 lanebits = 0;
#pragma unroll
    for (u32 k = 0; k < kLaneKeys; ++k) lanebits += len[k];
    const u32 incl = wave_incl_scan(lanebits);
    const u32 roundbits = read_lane(incl, 63);
    if (pbit + roundbits > pbits) return false;             // the lengths overrun the payload plane
    // deltas and their running sum inside the lane
    u32 bp = wbits + incl - lanebits;
    u32 kp[kLaneKeys];
    u32 acc = 0;
    bool ovf = false;                                       // a key beyond 32 bits, or one that repeats its predecessor
#pragma unroll
    for (u32 k = 0; k < kLaneKeys; ++k) {
        const u32 wa = bp >> 5;
        const u32 x = __builtin_amdgcn_alignbit(s_pay[wa + 1], s_pay[wa], bp & 31u);
        u32 dl = x & (0xFFFFFFFFu >> ((32u - len[k]) & 31u));
        if (!FULL && len[k] == 0) dl = 0;                   // (a real key has a length of at least 1)
        bp += len[k];
        const u32 nx = acc + dl;
        // the running sum must grow: it does not if it wraps (only a long delta can do that) or if the delta
        // is 0, i.e. the key repeats its predecessor -- which only the stream's very first key may do
        // (keys beyond n have no length and no delta)
        if (k == 0) ovf |= dl == 0 && (FULL || len[k] != 0) && !(stream_start && lane == 0);
        else ovf |= nx <= acc && (FULL || len[k] != 0);
        acc = nx;
        kp[k] = acc;
    }
    const u64 incl64 = wave_incl_scan64((u64)acc);
    const u64 kbase = (u64)carry + incl64 - acc;            // key before the lane's first key
    // the lane's keys do not decrease, so the last one tells whether any of them leaves 32 bits
    ovf |= ((kbase + acc) >> 32) != 0 && (FULL || lane * kLaneKeys < n);
#pragma unroll
    for (u32 k = 0; k < kLaneKeys; ++k) kp[k] = (u32)kbase + kp[k];
    // values: the code byte (sign in bit 7) indexes a table of signed values; a code >= tau shows as a
    // carry into bit 7 of (code-1) + (128 - tau), tested four bytes at a time
    bool badcode = false;
    u32 vb[kLaneKeys];
    if (MODE == kHand && cwid != 8) {
        // (this form keeps its shared memory small: the lane's tokens come straight from the token words, two
        // cached loads a token)
        const u32* cwords = reinterpret_cast<const u32*>(codes_round);
        const u32 ncw = (n * cwid + 31u) >> 5, tmask = (1u << cwid) - 1u, cmask = tmask >> 1;
#pragma unroll
        for (u32 k = 0; k < kLaneKeys; ++k) {
            const u32 i = lane * kLaneKeys + k, pos = i * cwid, wa = pos >> 5;
            const u32 w0 = wa < ncw ? cwords[wa] : 0u, w1 = wa + 1u < ncw ? cwords[wa + 1u] : 0u;
            u32 tok = __builtin_amdgcn_alignbit(w1, w0, pos & 31u) & tmask;
            if (!FULL && i >= n) tok = 0;
            const u32 c1 = tok & cmask, sign = tok >> (cwid - 1u);
            badcode |= c1 >= tau;
            vb[k] = cwid < 8 ? s_V[(sign << 7) | c1] : (s_V[c1 & 0xFFu] | (sign << 31));
        }
    } else if (cwid <= 8) {
        const u32 over = (128u - tau) * 0x01010101u;
        u32 badbits = 0;
#pragma unroll
        for (u32 j = 0; j < 4; ++j) badbits |= ((cw[j] & 0x7F7F7F7Fu) + over) & 0x80808080u;
        badcode = badbits != 0;                             // (bytes beyond n are 0: code 1, never beyond tau)
#pragma unroll
        for (u32 k = 0; k < kLaneKeys; ++k) vb[k] = s_V[(cw[k >> 2] >> (8u * (k & 3u))) & 0xFFu];
    }
    if (MODE == kHand) {
        // the caller takes the pairs as they are, 16 consecutive ones per lane (those beyond n repeat the last key,
        // their values mean nothing: the caller knows n)
#pragma unroll
        for (u32 k = 0; k < kLaneKeys; ++k) { out_keys[k] = kp[k]; out_vals[k] = vb[k]; }
        carry = read_lane(kp[kLaneKeys - 1], 63);           // (keys beyond n add nothing: the last lane ends on the round's last key)
        pbit += roundbits;
        wave_lds_sync();
        return !(__any(ovf) || __any(badcode));
    }
    // Lane-major -> row-major through shared memory (row q, lane: pair 64 * q + lane), so that stores to
    // the output arrays are coalesced and updates of the dense arrays touch neighbouring addresses in one
    // instruction.  A lane's 16 words sit 20 words apart (word i at i + 4 * (i / 16)), which spreads the
    // 16-byte writes over all banks.
    wave_lds_sync();
    uint4* t4 = reinterpret_cast<uint4*>(s_pay) + lane * 5u;
    const u32 rowpos = lane + 4u * (lane >> 4);            // position of word 64 * q + lane: rowpos + 80 * q
    u32 kr[kLaneKeys], vr[kLaneKeys];
#pragma unroll
    for (u32 j = 0; j < 4; ++j) t4[j] = make_uint4(kp[4 * j], kp[4 * j + 1], kp[4 * j + 2], kp[4 * j + 3]);
    wave_lds_sync();
#pragma unroll
    for (u32 q = 0; q < kLaneKeys; ++q) kr[q] = s_pay[rowpos + 80u * q];
    carry = s_pay[(n - 1u) + 4u * ((n - 1u) >> 4)];          // last key of the round (same in all lanes)
    if (MODE == kStore) {
#pragma unroll
        for (u32 q = 0; q < kLaneKeys; ++q) {
            const u32 i = q * 64u + lane;
            if (FULL || i < n) __builtin_nontemporal_store(kr[q], &keys_dst[i]);    // written once, not read again here
        }
    }
    wave_lds_sync();
    // nine-bit tokens (tau in 129..256) are taken row-wise straight from the round's token words: token i
    // at bit 9 i; code-1 in the low eight bits indexes the 256 magnitudes, bit 8 is the sign
    auto wide_value = [&](u32 i) -> u32 {
        const u32 pos = i * 9u, wa = pos >> 5;
        u32 tok = __builtin_amdgcn_alignbit(s_cod[wa + 1u], s_cod[wa], pos & 31u) & 0x1FFu;
        if (!FULL && i >= n) tok = 0;
        badcode |= (tok & 0xFFu) >= tau;
        return s_V[tok & 0xFFu] | ((tok >> 8) << 31);
    };
    if (MODE == kStore && cwid > 8) {
        // (a loop that stays a loop: the common case keeps its registers)
#pragma unroll 1
        for (u32 q = 0; q < kLaneKeys; ++q) {
            const u32 i = q * 64u + lane;
            const u32 x = wide_value(i);
            if (FULL || i < n) __builtin_nontemporal_store(__uint_as_float(x), &values_dst[i]);
        }
        pbit += roundbits;
        return !(__any(ovf) || __any(badcode));
    }
    if (cwid <= 8) {
#pragma unroll
        for (u32 j = 0; j < 4; ++j) t4[j] = make_uint4(vb[4 * j], vb[4 * j + 1], vb[4 * j + 2], vb[4 * j + 3]);
        wave_lds_sync();
#pragma unroll
        for (u32 q = 0; q < kLaneKeys; ++q) vr[q] = s_pay[rowpos + 80u * q];
        wave_lds_sync();
    } else if (MODE != kStore) {
#pragma unroll
        for (u32 q = 0; q < kLaneKeys; ++q) vr[q] = wide_value(q * 64u + lane);
    }
    if (MODE == kStore) {
#pragma unroll
        for (u32 q = 0; q < kLaneKeys; ++q) {
            const u32 i = q * 64u + lane;
            if (FULL || i < n) __builtin_nontemporal_store(__uint_as_float(vr[q]), &values_dst[i]);
        }
    } else {
        // all sixteen reads are issued before the first write: the keys of a valid stream are distinct,
        // and a stream that is not valid leaves unspecified arrays anyway
        bool big = false;
        float cur[kLaneKeys];
        bool on[kLaneKeys];
#pragma unroll
        for (u32 q = 0; q < kLaneKeys; ++q) {
            const bool have = FULL || q * 64u + lane < n;
            on[q] = have && kr[q] < dense_len;
            big |= have && !on[q];
            cur[q] = on[q] ? dense[kr[q]] : 0.0f;
        }
        if (MODE == kAccum) {
#pragma unroll
            for (u32 q = 0; q < kLaneKeys; ++q)
                if (on[q]) dense[kr[q]] = cur[q] + __uint_as_float(vr[q]);
        } else {
            // m = b1 m + (1 - b1) g;  v = b2 v + (1 - b2) g^2;  theta -= eta m / sqrt(v + eps)
            float mo[kLaneKeys], vo[kLaneKeys];
#pragma unroll
            for (u32 q = 0; q < kLaneKeys; ++q) {
                mo[q] = on[q] ? adam.m[kr[q]] : 0.0f;
                vo[q] = on[q] ? adam.v[kr[q]] : 0.0f;
            }
#pragma unroll
            for (u32 q = 0; q < kLaneKeys; ++q) {
                if (on[q]) {
                    const float g = __uint_as_float(vr[q]);
                    const float mt = adam.beta1 * mo[q] + adam.one_minus_beta1 * g;
                    const float vt = adam.beta2 * vo[q] + adam.one_minus_beta2 * g * g;
                    adam.m[kr[q]] = mt;
                    adam.v[kr[q]] = vt;
                    dense[kr[q]] = cur[q] - adam.eta * mt / __fsqrt_rn(vt + adam.eps);
                }
            }
        }
        too_big |= __any(big);
    }
    pbit += roundbits;
    return !(__any(ovf) || __any(badcode));
}

// MODE kAccum: the launch handles the key blocks of stream `only` alone and updates the dense array (one
// launch per stream, so that the updates happen stream after stream).
// INLINE: one stream and no other launch.  Every wave reads the 64-byte header and reaches the same verdict
// on it; the workgroup rebuilds the table of decoded magnitudes sum / b^c (phases 3-4 evaluated once per
// code): one thread walks the tau multiplications of b^c -- a chain of dependent binary64 operations that
// takes microseconds, which is why such a launch uses few, large workgroups (WAVES = 16: one chain per
// compute unit) -- then 256 threads divide, one code each.  A wave that finds its block corrupt leaves the
// code in done->fail (the larger code stays); every workgroup that has key blocks counts itself in `done` when its
// waves are through, and the one that completes the count writes *out_status and out_counts[0] and leaves
// the control words zero for the next launch (workgroups without key blocks leave at once; a launch with
// nothing to decode is reported by workgroup 0 alone).
template <int MODE, bool INLINE, u32 WAVES>
__global__ void __launch_bounds__(WAVES * kWave) __attribute__((amdgpu_waves_per_eu(MODE == kStore ? 4 : 2, 8)))
k_decode(const uint8_t* __restrict__ streams, u64 stream_bytes, u64 capacity, const DecSeg* __restrict__ segs,
         u32 n_segments, DecCtrl* ctrl, DecDone* done, u32* __restrict__ keys_out, float* __restrict__ values_out, u64* out_counts,
         u32 n_counts, u32* out_status, float* __restrict__ dense, u64 dense_len, u32 only, AdamArgs adam) {
    static_assert(!INLINE || WAVES >= 4, "256 threads divide for the 256 codes");
    __shared__ __attribute__((aligned(16))) u32 s_payall[WAVES][20 * 64];     // payload window (17 rows of 64 words); output staging (1280 words)
    __shared__ u32 s_flgall[WAVES][3 * 64];                                    // flags of a round (160 words at most)
    __shared__ u32 s_Vall[INLINE ? 1 : WAVES][256];                            // value by code byte (bit 7: sign); one stream: one table
    __shared__ __attribute__((aligned(16))) u32 s_codall[WAVES][2 * kCodeWords];   // token words, then widened bytes
    const u32 lane = lane_id(), w = uniform(wave_id());
    u32* s_pay = s_payall[w];
    u32* s_flg = s_flgall[w];
    u32* s_V = s_Vall[INLINE ? 0 : w];
    u32* s_cod = s_codall[w];
    u64 item_lo = 0, item_hi = 0;
    u32 cur_seg = 0xFFFFFFFFu;
    DecHead hd = {};                // the stream in hand (wave-uniform)
    u64 stream_begin = 0, pair_begin = 0, seg_item_begin = 0;
    u32 head_status = 0;            // INLINE: what the header alone says
    u32 n_work = 1;                 // INLINE: workgroups that have key blocks (and report through the count)
    u32 dir_first = 0;              // INLINE: the wave's first directory entry, fetched before the table is built
    if (INLINE) {
        bool ok = stream_bytes >= kHeaderBytes;
        if (ok) ok = parse_header(reinterpret_cast<const u64*>(streams), stream_bytes, hd);
        if (!ok) head_status = FASTSGD_ERR_CORRUPT_STREAM;
        else if (hd.d > capacity) head_status = FASTSGD_ERR_BUFFER_TOO_SMALL;
        head_status = uniform(head_status);
        if (head_status == 0 && hd.nb) {
            const u32 units = (hd.nb + WAVES - 1u) / WAVES;
            n_work = units < gridDim.x ? units : gridDim.x;
        }
        if (blockIdx.x >= n_work) return;                    // nothing to decode and nothing to report
        if (head_status == 0 && hd.nb) {
            item_hi = hd.nb;
            const u32 blk0 = blockIdx.x * WAVES + w;
            if (blk0 < hd.nb && (lane < 4 || (lane < 8 && blk0 + 1 < hd.nb)))
                dir_first = reinterpret_cast<const u32*>(streams + hd.dir_off + 16ull * blk0)[lane];
            // magnitudes of the codes: P[c] = fl64(P[c-1] * b) walked by one thread into wave 0's (still
            // unused) payload window, then thread t divides for code t + 1
            double* P = reinterpret_cast<double*>(s_payall[0]);
            if (threadIdx.x == 0) power_chain(hd.base, hd.tau, P);
            __syncthreads();
            const u32 t = threadIdx.x;
            u32 m = 0;
            if (t < hd.tau && hd.sum > 0.0) m = f64_to_f32_bits(hd.sum / P[t + 1u], false);
            __syncthreads();
            // tau <= 128: indexed by the code byte, magnitudes below, the same with the sign set above;
            // beyond that: the 256 magnitudes, the sign is added from the token's top bit
            if (hd.tau > 128u) {
                if (t < 256u) s_V[t] = m;
            } else if (t < 128u) {
                s_V[t] = m;
                s_V[t + 128u] = m | 0x80000000u;
            }
            cur_seg = 0;
            __syncthreads();
        }
    } else {
        item_hi = ctrl->total_items;
        if (MODE != kStore && item_hi) { item_lo = segs[only].item_begin; item_hi = item_lo + segs[only].nb; }
    }

    const u64 item_first = item_lo + (u64)blockIdx.x * WAVES + w;
    for (u64 item = item_first; item < item_hi; item += (u64)gridDim.x * WAVES) {
        const u32 seg = (INLINE || n_segments == 1) ? 0u : (MODE != kStore ? only : uniform(find_dec_segment(segs, n_segments, item)));
        if (!INLINE && seg != cur_seg) {
            const DecSeg* ds = &segs[seg];
            hd.KB = uniform(ds->KB); hd.l = uniform(ds->l); hd.tau = uniform(ds->tau); hd.nb = uniform(ds->nb);
            hd.d = uniform64(ds->d);
            hd.dir_off = uniform64(ds->dir_off); hd.blocks_off = uniform64(ds->blocks_off);   // (absolute in a batch)
            hd.total_words = uniform64(ds->total_words);
            stream_begin = uniform64(ds->stream_begin); pair_begin = uniform64(ds->pair_begin);
            seg_item_begin = uniform64(ds->item_begin);
            wave_lds_sync();
            // tau <= 128: indexed by the code byte, magnitudes below, the same with the sign set above;
            // beyond that: the 256 magnitudes, the sign is added from the token's top bit
            const bool wide = hd.tau > 128u;
            const u32 m0 = ds->V[lane], m1 = ds->V[lane + 64];
            const u32 m2 = ds->V[lane + (wide ? 128u : 0u)], m3 = ds->V[lane + (wide ? 192u : 64u)];
            s_V[lane] = m0;
            s_V[lane + 64] = m1;
            s_V[lane + 128] = wide ? m2 : m2 | 0x80000000u;
            s_V[lane + 192] = wide ? m3 : m3 | 0x80000000u;
            cur_seg = seg;
            wave_lds_sync();
        }
        const u32 KB = hd.KB, l = hd.l, tau = hd.tau, nb = hd.nb;
        const u64 d = hd.d;
        const u32 blk = uniform((u32)(item - seg_item_begin));
        const u32 first = blk * KB;
        const u32 cnt = uniform((u32)((d - first < KB) ? d - first : KB));
        const u32 nsub = (cnt + kSub - 1) / kSub;
        // directory entry of the block and of the next one, checked against each other
        const u32* dir = reinterpret_cast<const u32*>(streams + hd.dir_off + 16ull * blk);
        const bool has_next = blk + 1 < nb;
        u32 dword;
        if (INLINE && item == item_first) dword = dir_first;
        else dword = (lane < 4 || (lane < 8 && has_next)) ? dir[lane] : 0u;
        const u32 off8 = read_lane(dword, 0), preKey = read_lane(dword, 1), M = read_lane(dword, 2);
        const u32 pbits = read_lane(dword, 3), next_off8_dir = read_lane(dword, 4), next_pre = read_lane(dword, 5);
        const u64 total_words = hd.total_words;
        const u64 next_off8 = has_next ? (u64)next_off8_dir : total_words;
        const u32 fwords = (cnt * l + 63u) >> 6, pwords = (pbits + 63u) >> 6;
        bool bad = (M < 1 || M > 32) || (pbits > cnt * 32u) || ((u64)off8 + fwords + pwords != next_off8) ||
                   ((u64)off8 + fwords + pwords > total_words) || (blk == 0 && (off8 != 0 || preKey != 0));
        bool too_big = false;
        if (!bad) {
            const u32* fsrc = reinterpret_cast<const u32*>(streams + uniform64(hd.blocks_off + 8ull * off8));   // flags plane
            const u32* psrc = fsrc + 2u * fwords;                                                              // payload plane
            const u32 pw_total = 2u * pwords;
            const u32 cwid = uniform(code_width(tau));                 // bits of a value token
            const uint8_t* codes = streams + uniform64(stream_begin + kHeaderBytes + (u64)(first >> 3) * cwid);
            const u64 out0 = uniform64(pair_begin + first);
            u32 pbit = 0;                  // payload bits consumed by the rounds before
            u32 carry = preKey;            // key before the round in hand
            bool ok = true;
            for (u32 sub = 0; sub < nsub && ok; ++sub) {
                const u32 n = cnt - sub * kSub < kSub ? cnt - sub * kSub : kSub;
                // the lane number as a value of this round: keeps the dozens of shared-memory addresses derived
                // from it from being computed once and held in registers across the whole kernel
                u32 lane_r = lane;
                asm volatile("" : "+v"(lane_r));
                u32* kd = MODE != kStore ? nullptr : keys_out + out0 + sub * kSub;
                float* vd = MODE != kStore ? nullptr : values_out + out0 + sub * kSub;
                const bool stream_start = (blk == 0 && sub == 0);       // the round holds the stream's first key
                u32 unused_k[kLaneKeys], unused_v[kLaneKeys];
                if (n == kSub)
                    ok = decode_round<true, MODE>(fsrc + sub * 32u * l, psrc, pw_total, codes + sub * (kSub / 8u) * cwid, n, l, M,
                                                   tau, cwid, pbits, pbit, carry, lane_r, s_pay, s_flg, s_cod, s_V, kd, vd, dense, dense_len,
                                                   adam, too_big, stream_start, unused_k, unused_v);
                else
                    ok = decode_round<false, MODE>(fsrc + sub * 32u * l, psrc, pw_total, codes + sub * (kSub / 8u) * cwid, n, l, M,
                                                    tau, cwid, pbits, pbit, carry, lane_r, s_pay, s_flg, s_cod, s_V, kd, vd, dense, dense_len,
                                                    adam, too_big, stream_start, unused_k, unused_v);
            }
            bad = !ok || (pbit != pbits) || (has_next && carry != next_pre);
        }
        if ((bad || too_big) && lane == 0) {
            const u32 code = bad ? FASTSGD_ERR_CORRUPT_STREAM : FASTSGD_ERR_BUFFER_TOO_SMALL;
            if (INLINE) atomicMax(&done->fail, code);
            else dec_fail(ctrl, code, out_status, out_counts, n_counts);
        }
    }
    if (INLINE) {
        // (the barrier also waits for the memory operations of every wave of the workgroup, so a failure
        // word is in place before the workgroup counts itself)
        __syncthreads();
        if (threadIdx.x == 0) {
            const u32 n_groups = n_work < kDoneGroups ? n_work : kDoneGroups;
            const u32 g = blockIdx.x % kDoneGroups;
            const u32 members = (n_work - g + kDoneGroups - 1u) / kDoneGroups;        // workgroups b < n_work with b mod 16 = g
            if (atomicInc(&done->group[g][0], members - 1u) == members - 1u &&        // (wraps to 0 with the last one)
                atomicInc(&done->top, n_groups - 1u) == n_groups - 1u) {
                const u32 fail = atomicExch(&done->fail, 0u);
                const u32 status = head_status ? head_status : fail;
                *out_status = status;
                out_counts[0] = status ? 0ull : hd.d;
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
// Decode-and-aggregate in one pass over the dense vector (Section 2.1: the workers' gradients are decoded
// and added up).  For gradients that keep more than a few in a thousand of their entries, adding stream after
// stream moves the whole dense vector through the memory system once per stream; here it moves once per
// group of kTileStreams streams.
//
// A workgroup owns a run of consecutive tiles of TILE keys and holds one tile at a time in shared memory
// (the next one is on its way into registers meanwhile).  Wave w walks the key blocks of the group's w-th
// stream in order, one round of up to 1024 pairs at a time, and keeps the round in registers (16 consecutive
// pairs per lane) until the tile that holds its last key has come -- so a round that straddles tiles is
// decoded once.  Binary32 addition is not associative, so for every key the streams are added in the given
// order: every stream publishes a front, the key below which it has added everything it holds for the tile,
// and a wave adds a key only once the fronts of all streams before its own have passed it (keys are
// distinct inside a stream, so an addition is a plain read-add-write of shared memory).  A wave that has to
// wait decodes its stream's next round meanwhile, into a second set of registers, so that the streams
// decode side by side although they add one after the other.  The waves meet at a barrier only where a
// tile is written back and the next one comes in.
// A workgroup starts each stream at the block that holds the first key of its run (found by a search of the
// block directory's preKeys, which the launch checks to be strictly increasing so that every block is met
// by some workgroup) and decodes that block from its beginning, keys below the run being skipped.
// The workgroup that owns the last tile goes on to the end of every stream: what is left there has keys
// beyond the dense vector (FASTSGD_ERR_BUFFER_TOO_SMALL) unless it is corrupt, which is reported first.
constexpr u32 kTileStreams = 8;
constexpr u32 kMinAdd = 2048;             // keys of a tile a wave waits for before it adds a part of its round
constexpr u32 kFrontSpins = 1u << 22;     // polls of the other streams' fronts before a wait is given up (seconds)

// Largest index i in [0, n) with pre(i) <= x, or 0 (the wave probes 64 entries per round trip).  Stays inside
// [0, n) whatever the entries hold.
template <class Value>
__device__ __forceinline__ u32 dir_upper_index(u32 n, u32 x, Value pre) {
    u32 lo = 0, hi = n;
    while (hi - lo > 1) {
        const u32 step = (hi - lo + 63u) / 64u;
        const u32 idx = lo + lane_id() * step;
        const bool p = idx < hi && pre(idx) <= x;
        const u32 c = (u32)__popcll(__ballot(p));
        lo = uniform(lo + (c ? c - 1u : 0u) * step);           // (c <= lanes with idx < hi, so lo stays below hi)
        hi = lo + step < hi ? lo + step : hi;
    }
    return lo;
}

template <u32 TILE>
__global__ void __launch_bounds__(kTileStreams * kWave) __attribute__((amdgpu_waves_per_eu(2, 2)))
k_accumulate_tiles(const uint8_t* __restrict__ streams, const DecSeg* __restrict__ segs, u32 seg0, u32 n_here,
                   DecCtrl* ctrl, u64* out_count, u32* out_status, float* __restrict__ dense, u64 dense_len,
                   u32 tiles_per_group) {
    static_assert(TILE % (kTileStreams * kWave * 4) == 0, "whole 16-byte pieces for every thread");
    constexpr u32 kPieces = TILE / (kTileStreams * kWave * 4);
    __shared__ __attribute__((aligned(16))) float s_tile[TILE + kWave];      // (the last 64: a place to write for lanes with nothing to add)
    __shared__ __attribute__((aligned(16))) u32 s_payall[kTileStreams][17 * 64];      // payload window of a round
    __shared__ u32 s_flgall[kTileStreams][3 * 64];
    __shared__ u32 s_Vall[kTileStreams][256];
    __shared__ u32 s_front[kTileStreams];
    __shared__ u32 s_go;
    const u32 lane = lane_id(), w = uniform(wave_id()), t = threadIdx.x;
    if (t == 0) s_go = (ctrl->status == 0);          // (one reading for the whole workgroup: others may fail meanwhile)
    __syncthreads();
    if (!s_go) return;

    // the block directories must rise: preKey of a block is the last key of the one before
    for (u32 s = 0; s < n_here; ++s) {
        const DecSeg* ds = &segs[seg0 + s];
        const u32 nb = ds->nb;
        const u32* dir = reinterpret_cast<const u32*>(streams + ds->dir_off);
        bool falls = false;
        for (u64 b = (u64)blockIdx.x * blockDim.x + t; b + 1 < nb; b += (u64)gridDim.x * blockDim.x)
            falls |= dir[4 * (b + 1) + 1] <= dir[4 * b + 1];
        if (falls) dec_fail(ctrl, FASTSGD_ERR_CORRUPT_STREAM, out_status, out_count, 1);
    }

    const u64 n_tiles = (dense_len + TILE - 1) / TILE;
    const u64 t_begin = (u64)blockIdx.x * tiles_per_group;
    u64 t_end = t_begin + tiles_per_group;
    if (t_end > n_tiles) t_end = n_tiles;
    if (t_begin >= n_tiles) return;

    u32* s_pay = s_payall[w];
    u32* s_flg = s_flgall[w];
    u32* s_V = s_Vall[w];
    u32* s_cod = nullptr;                // (rounds handed back never stage their tokens)
    const bool mine = w < n_here;
    DecHead hd = {};
    u64 stream_begin = 0;
    if (mine) {
        const DecSeg* ds = &segs[seg0 + w];
        hd.KB = uniform(ds->KB); hd.l = uniform(ds->l); hd.tau = uniform(ds->tau); hd.nb = uniform(ds->nb);
        hd.d = uniform64(ds->d);
        hd.dir_off = uniform64(ds->dir_off); hd.blocks_off = uniform64(ds->blocks_off);
        hd.total_words = uniform64(ds->total_words);
        stream_begin = uniform64(ds->stream_begin);
        const bool wide = hd.tau > 128u;
        const u32 m0 = ds->V[lane], m1 = ds->V[lane + 64];
        const u32 m2 = ds->V[lane + (wide ? 128u : 0u)], m3 = ds->V[lane + (wide ? 192u : 64u)];
        s_V[lane] = m0;
        s_V[lane + 64] = m1;
        s_V[lane + 128] = wide ? m2 : m2 | 0x80000000u;
        s_V[lane + 192] = wide ? m3 : m3 | 0x80000000u;
        wave_lds_sync();
    }
    const u32 KB = hd.KB, l = hd.l, tau = hd.tau, nb = hd.nb;
    const u32 cwid = uniform(code_width(tau ? tau : 1u));
    const u32* dirs = reinterpret_cast<const u32*>(streams + hd.dir_off);

    // the wave's place in its stream
    bool ended = !mine || nb == 0;       // no round left to decode
    bool have = false;                   // the registers hold a round (it may reach into tiles to come)
    bool ahead = false;                  // ... and the one after it, decoded while the wave had to wait
    u32 kp[kLaneKeys], vb[kLaneKeys];    // the round in hand, 16 consecutive pairs per lane
    u32 kq[kLaneKeys], vq[kLaneKeys];    // the round ahead
#pragma unroll
    for (u32 k = 0; k < kLaneKeys; ++k) { kp[k] = 0; vb[k] = 0; kq[k] = 0; vq[k] = 0; }
    u32 n_cur = 0, last = 0;             // pairs of the round in hand, its last key
    u32 n_ahead = 0, last_ahead = 0;
    u32 blk = 0, sub = 0, nsub = 0, cnt = 0;
    u32 M = 1, pbits = 0, pbit = 0, carry = 0, next_pre = 0, pw_total = 0;
    bool has_next = false;
    const u32* fsrc = nullptr;
    const u32* psrc = nullptr;
    const uint8_t* codes = nullptr;
    if (!ended && t_begin) {
        const u32 r0 = (u32)(t_begin * TILE) - 1u;            // the block whose preKey is the last one below the run
        blk = uniform(dir_upper_index(nb, r0, [&](u32 i) { return dirs[4 * i + 1]; }));
    }
    // (What one lane could do alone -- report a failure, publish a front -- is done by all lanes alike: a branch
    // on the lane number in the middle of these loops makes the compiler treat the loops' own, wave-wide
    // conditions as if they differed between lanes, and it then runs them under lane masks.)
    auto stop = [&](u32 code) {
        dec_fail(ctrl, code, out_status, out_count, 1);
        ended = true;
        have = false;
        ahead = false;
    };
    // decodes the stream's next round into the registers of the round ahead (written without early ways out:
    // the loops around it keep a single exit each, which the compiler turns into plain branches)
    auto decode_next = [&]() {
        bool good = true;
        if (sub == nsub) {               // open block blk
            const u32* dir = dirs + 4ull * blk;
            has_next = blk + 1 < nb;
            const u32 dword = dir[has_next ? (lane & 7u) : (lane & 3u)];
            const u32 off8 = read_lane(dword, 0), preKey = read_lane(dword, 1);
            M = read_lane(dword, 2); pbits = read_lane(dword, 3);
            const u32 next_off8_dir = read_lane(dword, 4);
            next_pre = read_lane(dword, 5);
            const u32 first = blk * KB;
            cnt = uniform((u32)((hd.d - first < KB) ? hd.d - first : KB));
            const u64 next_off8 = has_next ? (u64)next_off8_dir : hd.total_words;
            const u32 fwords = (cnt * l + 63u) >> 6, pwords = (pbits + 63u) >> 6;
            good = !((M < 1 || M > 32) || (pbits > cnt * 32u) || ((u64)off8 + fwords + pwords != next_off8) ||
                     ((u64)off8 + fwords + pwords > hd.total_words) || (blk == 0 && (off8 != 0 || preKey != 0)));
            if (good) {
                fsrc = reinterpret_cast<const u32*>(streams + uniform64(hd.blocks_off + 8ull * off8));
                psrc = fsrc + 2u * fwords;
                pw_total = 2u * pwords;
                codes = streams + uniform64(stream_begin + kHeaderBytes + (u64)(first >> 3) * cwid);
                pbit = 0;
                carry = preKey;
                sub = 0;
                nsub = (cnt + kSub - 1) / kSub;
            }
        }
        if (good) {
            const u32 n = cnt - sub * kSub < kSub ? cnt - sub * kSub : kSub;
            u32 lane_r = lane;
            asm volatile("" : "+v"(lane_r));
            const bool stream_start = (blk == 0 && sub == 0);
            bool unused = false;
            if (n == kSub)
                good = decode_round<true, kHand>(fsrc + sub * 32u * l, psrc, pw_total, codes + sub * (kSub / 8u) * cwid, n, l, M, tau,
                                                 cwid, pbits, pbit, carry, lane_r, s_pay, s_flg, s_cod, s_V, nullptr, nullptr, nullptr,
                                                 0, AdamArgs(), unused, stream_start, kq, vq);
            else
                good = decode_round<false, kHand>(fsrc + sub * 32u * l, psrc, pw_total, codes + sub * (kSub / 8u) * cwid, n, l, M, tau,
                                                  cwid, pbits, pbit, carry, lane_r, s_pay, s_flg, s_cod, s_V, nullptr, nullptr, nullptr,
                                                  0, AdamArgs(), unused, stream_start, kq, vq);
            if (good) {
                ++sub;
                ahead = true;
                n_ahead = n;
                last_ahead = carry;
                if (sub == nsub) {
                    good = pbit == pbits && (!has_next || carry == next_pre);
                    ++blk;
                    if (blk == nb) ended = true;
                }
            }
        }
        if (!good) stop(FASTSGD_ERR_CORRUPT_STREAM);
        // (everything the loops branch on is the same in all lanes; said again, so that the branches are scalar)
        ahead = uniform((u32)ahead) != 0u;
        ended = uniform((u32)ended) != 0u;
        have = uniform((u32)have) != 0u;
        n_ahead = uniform(n_ahead);
        last_ahead = uniform(last_ahead);
        sub = uniform(sub); nsub = uniform(nsub); blk = uniform(blk);
        pbit = uniform(pbit); carry = uniform(carry);
    };

    const bool last_group = t_end == n_tiles;
    bool big = false;                    // the stream holds keys beyond the dense vector
    float4 q[kPieces];                   // a whole tile on its way from memory, a 16-byte piece per thread and step
    bool fetched = false;
#pragma unroll
    for (u32 j = 0; j < kPieces; ++j) q[j] = make_float4(0.f, 0.f, 0.f, 0.f);
    u64 tile = t_begin;
    u64 k0 = 0;                          // first key of the tile in shared memory
    u32 klen = 0;                        // its keys
    u32 my_front = 0;                    // the stream has added its keys below k0 + my_front
    // Tile in: 16 bytes per lane (the launch requires a 16-byte aligned vector).  A whole tile was fetched into
    // registers while the tile before it was at work (the run's first one: just now).
    auto enter = [&]() {
        k0 = tile * TILE;
        klen = (u32)(dense_len - k0 < TILE ? dense_len - k0 : TILE);
        float* dtile = dense + k0;
        if (klen == TILE) {
            if (!fetched) {
#pragma unroll
                for (u32 j = 0; j < kPieces; ++j) q[j] = reinterpret_cast<const float4*>(dtile)[t + j * kTileStreams * kWave];
                // (all of them under way before the first one is used: otherwise the compiler waits for each)
#pragma unroll
                for (u32 j = 0; j + 1 < kPieces; j += 2)
                    asm volatile("" : "+v"(q[j].x), "+v"(q[j].y), "+v"(q[j].z), "+v"(q[j].w), "+v"(q[j + 1].x), "+v"(q[j + 1].y),
                                      "+v"(q[j + 1].z), "+v"(q[j + 1].w));
            }
#pragma unroll
            for (u32 j = 0; j < kPieces; ++j) reinterpret_cast<float4*>(s_tile)[t + j * kTileStreams * kWave] = q[j];
        } else {
            for (u32 i = t * 4u; i < TILE; i += kTileStreams * kWave * 4u) {
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (i + 4u <= klen) v = *reinterpret_cast<const float4*>(dtile + i);
                else {
                    if (i < klen) v.x = dtile[i];
                    if (i + 1u < klen) v.y = dtile[i + 1u];
                    if (i + 2u < klen) v.z = dtile[i + 2u];
                }
                *reinterpret_cast<float4*>(&s_tile[i]) = v;
            }
        }
        // the next tile, if it is a whole one: on its way while this one is at work
        fetched = tile + 1 < t_end && dense_len - (k0 + TILE) >= TILE;
        if (fetched) {
#pragma unroll
            for (u32 j = 0; j < kPieces; ++j) q[j] = reinterpret_cast<const float4*>(dtile + TILE)[t + j * kTileStreams * kWave];
        }
        my_front = 0;
        s_front[w] = mine ? 0u : klen;
        __syncthreads();
    };
    // Tile out, once every stream is through with it.
    auto leave = [&]() {
        if (mine) {
            __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
            __hip_atomic_store(&s_front[w], klen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
            // while other streams are still at work on the tile: the round after the one in hand
            if (!ahead && !ended) {
                const u32 f = __hip_atomic_load(&s_front[lane & (kTileStreams - 1u)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                if (__any(lane < n_here && f < klen)) decode_next();
            }
        }
        __syncthreads();
        float* dtile = dense + k0;
        if (klen == TILE) {
#pragma unroll
            for (u32 j = 0; j < kPieces; ++j)
                reinterpret_cast<float4*>(dtile)[t + j * kTileStreams * kWave] = reinterpret_cast<const float4*>(s_tile)[t + j * kTileStreams * kWave];
        } else {
            for (u32 i = t * 4u; i < TILE; i += kTileStreams * kWave * 4u) {
                const float4 v = *reinterpret_cast<const float4*>(&s_tile[i]);
                if (i + 4u <= klen) *reinterpret_cast<float4*>(dtile + i) = v;
                else {
                    if (i < klen) dtile[i] = v.x;
                    if (i + 1u < klen) dtile[i + 1u] = v.y;
                    if (i + 2u < klen) dtile[i + 2u] = v.z;
                }
            }
        }
        __syncthreads();
        ++tile;
    };

    // Round after round (the round decoder appears once in the code: it is long, and the waves of a workgroup
    // are all at different places of the kernel and share one instruction cache); inside, the tiles the
    // round reaches.  Every wave passes the same barriers, two per tile, whatever its stream holds.
    // s_front[s]: stream s has added all its keys below k0 + s_front[s].  A wave adds a key only once the
    // fronts of all streams before its own have passed it; the first stream never waits, so the waits end.
    enter();
    bool tiles_left = true, run = true;
    u32 spins = 0;
    while (run) {
        // A block the wave has opened is decoded to its end even behind the run's last tile (its last round
        // carries the checks of the whole block, and the next workgroup may start behind it).  Behind the
        // vector's last tile the same goes for the rest of every stream: what is left there lies beyond the dense
        // vector, unless it is corrupt, which outranks that.
        if (!ahead && !ended && (tiles_left || last_group || sub != nsub)) decode_next();
        have = ahead;
        if (ahead) {
#pragma unroll
            for (u32 k = 0; k < kLaneKeys; ++k) { kp[k] = kq[k]; vb[k] = vq[k]; }
            n_cur = n_ahead;
            last = last_ahead;
            ahead = false;
        }
        if (!tiles_left) {
            run = have;
            big = big || (have && last_group);
        } else {
            bool more = true;            // the round (or the end of the stream) still has tiles to go through
            while (more) {
                const u64 past = (u64)last + 1u;                           // first key the round does not hold
                const u32 hi = uniform((have && past > k0) ? (u32)(past - k0 < klen ? past - k0 : klen) : 0u);
                while (have && my_front < hi) {
                    u32 lim = hi;
                    if (w) {
                        // the fronts of the streams before this one (lanes 0..w-1 read one each)
                        u32 f = __hip_atomic_load(&s_front[lane & (kTileStreams - 1u)], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                        f = lane < w ? f : klen;
#pragma unroll
                        for (u32 j = 0; j < kTileStreams - 1; ++j) {
                            const u32 fj = read_lane(f, j);
                            lim = fj < lim ? fj : lim;
                        }
                    }
                    lim = uniform(lim);
                    if (lim <= my_front && spins > kFrontSpins) {
                        // (only ends a wait that cannot end by itself, which has never been seen: the launch then
                        // reports a device failure instead of hanging)
                        dec_fail(ctrl, FASTSGD_ERR_DEVICE, out_status, out_count, 1);
                        lim = hi;
                    }
                    // (a pass over the wave's pairs costs the same for one key as for a thousand: short ranges wait
                    // until they have grown or the streams before have passed the round's end)
                    if (lim >= hi || lim >= my_front + kMinAdd) {
                        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
                        // The round's keys in [my_front, lim) of the tile: sixteen reads, sixteen additions, sixteen
                        // writes, without a branch -- a key outside the range takes the lane's own entry behind the
                        // tile instead, which nobody reads.
                        const u32 base = (u32)k0, width = lim - my_front;
                        const u32 mine_n = n_cur > lane * kLaneKeys ? n_cur - lane * kLaneKeys : 0u;   // the lane's pairs
                        u32 at[kLaneKeys];
                        float cur[kLaneKeys];
#pragma unroll
                        for (u32 k = 0; k < kLaneKeys; ++k) {
                            const u32 idx = kp[k] - base;                     // (keys below the tile wrap to far beyond it)
                            at[k] = (idx - my_front < width && k < mine_n) ? idx : TILE + lane;
                            cur[k] = s_tile[at[k]];
                        }
#pragma unroll
                        for (u32 k = 0; k < kLaneKeys; ++k) s_tile[at[k]] = cur[k] + __uint_as_float(vb[k]);
                        my_front = lim;
                        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
                        __hip_atomic_store(&s_front[w], my_front, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                    } else if (!ahead && !ended) {
                        // nothing to add yet: time to decode the round after this one
                        decode_next();
                        have = ahead || !ended;                                // (corrupt: reported, nothing more to add)
                    } else {
                        ++spins;
                        __builtin_amdgcn_s_sleep(2);
                    }
                }
                if (have && past < k0 + klen) more = false;                    // nothing of the round lies behind this tile
                else {
                    // the stream is through with this tile
                    leave();
                    if (tile == t_end) { tiles_left = false; more = false; }
                    else enter();
                }
            }
            if (!tiles_left) {
                big = have && (u64)last >= dense_len;
                run = have;
            }
        }
    }
    if (last_group && big && lane == 0) dec_fail(ctrl, FASTSGD_ERR_BUFFER_TOO_SMALL, out_status, out_count, 1);
}

}  // namespace fsgd
