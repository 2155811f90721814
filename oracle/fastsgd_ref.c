/*
 * fastsgd_ref.c -- plain, sequential CPU oracle for the FastSGD gradient codec.
 *
 * TEST INFRASTRUCTURE ONLY.  This file exists to check the HIP library, to be
 * timed as a CPU baseline, and to write stored expected values.  Nothing in the
 * product path may call it, and it shares no code, header, table or constant
 * generator with the HIP sources: every constant below is this file's own copy.
 *
 * What it follows (FastSGD, arXiv 2112.04291):
 *   - Algorithm 1 (GV-Encoder): sum of absolute values, early-stop threshold
 *     tau_e = sum / b^tau, then for every surviving value the reciprocal mapper
 *     (Eq. 2), the logarithm quantization L = ceil(log_b R) (Eq. 3), the
 *     threshold filter L <= tau (Phase 3) and the sign (end of Section 3.2).
 *   - Algorithm 2 (GK-Encoder): delta keys (Eq. 4), maximal binary length M,
 *     length flag of l bits selecting one of 2^l lengths (Phase 5), one token
 *     (flag, binary delta) per surviving key.
 *   - Decoder phases 1-4 (Section 3.1): split tokens by their flags, prefix-sum
 *     the deltas, scale the integers back up (b^L), divide sum by that.
 *
 * Where the paper leaves a detail open this file takes one fixed reading; each
 * is marked "Reading:" below.
 *
 * Pins (tests/test_oracle_*.py): the abs-sum equals Python's math.fsum; codes
 * equal ceil(log_b(sum/|v|)) evaluated with exact rationals; the Fig. 2 and
 * Fig. 3 worked examples; closed-form sizes of Section 3.4; a pure-Python token
 * parser reads back every stream.  No function here is "parity unpinned"
 * except the byte layout of the container, which the paper does not define and
 * which is pinned only by that independent parser.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---- interface values (kept numerically equal to the product's, by contract) ---- */
enum {
    REF_OK = 0,
    REF_ERR_INVALID_ARG = 1,
    REF_ERR_BUFFER_TOO_SMALL = 2,
    REF_ERR_NONFINITE = 3,
    REF_ERR_UNSORTED_KEYS = 4,
    REF_ERR_CORRUPT_STREAM = 5
};

typedef struct {
    double base;         /* b  */
    uint32_t tau;        /* threshold on the integer code, 1..256 */
    uint32_t flag_bits;  /* l, 1..5 */
    uint32_t block_keys; /* surviving keys per key block, power of two in [256, 4096] */
    uint32_t reserved;   /* must be 0 */
} ref_params;

#define REF_HEADER_BYTES 64u
#define REF_MAGIC 0x44475346u /* "FSGD" little-endian */
#define REF_VERSION 1u
#define REF_MAX_TAU 256u /* Section 3.2 recommends 128; up to 256 a token is 9 bits */

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint64_t f64_bits(double f) { uint64_t u; memcpy(&u, &f, 8); return u; }
static double bits_f64(uint64_t u) { double f; memcpy(&f, &u, 8); return f; }

static int params_ok(const ref_params *p) {
    if (!p) return 0;
    if (!(p->base >= 1.0 + 1.0 / 1048576.0) || !(p->base <= 16.0)) return 0;
    if (p->tau < 1 || p->tau > REF_MAX_TAU) return 0;
    if (p->tau > 128 && !(p->base <= 4.0)) return 0; /* b^tau <= 2^512: sum / b^c stays a normal binary64 */
    if (p->flag_bits < 1 || p->flag_bits > 5) return 0;
    if (p->block_keys < 256 || p->block_keys > 4096) return 0;
    if (p->block_keys & (p->block_keys - 1)) return 0;
    if (p->reserved != 0) return 0;
    return 1;
}

/* ------------------------------------------------------------------------- *
 * Algorithm 1, line 1:  sum = sum_i |v_i|.
 * Reading: the real-number sum, rounded once to binary64 (nearest, ties to
 * even).  Every finite binary32 is an integer multiple of 2^-149, so the sum is
 * held exactly in a wide unsigned integer counting units of 2^-149.
 * Returns 1 if a NaN or infinity is present (sum then undefined), else 0.
 * ------------------------------------------------------------------------- */
#define WIDE_LIMBS 12 /* 384 bits: 2^24 * 2^253 * 2^32 elements < 2^310 */

int fastsgd_ref_abs_sum(const float *v, uint64_t n, double *sum_out) {
    uint32_t acc[WIDE_LIMBS];
    memset(acc, 0, sizeof acc);
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t a = f32_bits(v[i]) & 0x7FFFFFFFu;
        uint32_t e = a >> 23, frac = a & 0x7FFFFFu;
        if (e == 255) return 1;
        /* |v| = m * 2^shift units of 2^-149 */
        uint32_t m = e ? (frac | 0x800000u) : frac;
        uint32_t shift = e ? e - 1 : 0;
        uint64_t x = (uint64_t)m << (shift % 32);
        uint32_t li = shift / 32;
        uint64_t carry = x;
        while (carry) { /* add `carry` at limb li and ripple */
            uint64_t t = (uint64_t)acc[li] + (carry & 0xFFFFFFFFu);
            acc[li] = (uint32_t)t;
            carry = (carry >> 32) + (t >> 32);
            ++li;
        }
    }
    /* highest set bit */
    int top = -1;
    for (int li = WIDE_LIMBS - 1; li >= 0 && top < 0; --li)
        if (acc[li])
            for (int b = 31; b >= 0; --b)
                if (acc[li] >> b & 1) { top = li * 32 + b; break; }
    if (top < 0) { *sum_out = 0.0; return 0; }
    /* collect the 53 leading bits, then guard and sticky */
    uint64_t q = 0;
    int lo = top - 52; /* index of the mantissa's last bit; may be negative */
    for (int b = top; b >= lo && b >= 0; --b)
        q = (q << 1) | (acc[b / 32] >> (b % 32) & 1);
    if (lo <= 0) { /* fits in 53 bits: exact */
        *sum_out = ldexp((double)q, -149);
        return 0;
    }
    int guard = (int)(acc[(lo - 1) / 32] >> ((lo - 1) % 32) & 1);
    int sticky = 0;
    for (int b = lo - 2; b >= 0 && !sticky; --b)
        sticky = (int)(acc[b / 32] >> (b % 32) & 1);
    if (guard && (sticky || (q & 1))) ++q; /* q may become 2^53: still exact as a double */
    *sum_out = ldexp((double)q, lo - 149);
    return 0;
}

/* ------------------------------------------------------------------------- *
 * Algorithm 1, line 2 and Eq. 3, evaluated once per code instead of once per
 * element.  L(v) <= c  <=>  log_b(sum/|v|) <= c  <=>  |v| >= sum / b^c, so the
 * code of a value is decided by comparing |v| with the boundaries sum / b^c.
 * Reading: P[0] = 1, P[c] = fl64(P[c-1] * b);  t_c = fl64(sum / P[c]);
 *   boundary  B[c] = smallest binary32 >= t_c (rounded up, so that a kept value
 *   is never below the real boundary);
 *   decoded magnitude V[c] = binary32 nearest t_c  (so |decoded| <= |original|,
 *   the under-estimate the ceiling in Eq. 3 is there for).
 * B[tau] is the early-stop threshold tau_e.  Arrays are indexed 1..tau; entry 0
 * is unused and set to 0.
 * ------------------------------------------------------------------------- */
void fastsgd_ref_tables(double sum, double base, uint32_t tau,
                        uint32_t *B_bits /* [tau + 1] */, uint32_t *V_bits /* [tau + 1] */) {
    double P = 1.0;
    B_bits[0] = 0; V_bits[0] = 0;
    for (uint32_t c = 1; c <= tau; ++c) {
        P = P * base;
        double t = sum / P;
        float nearest = (float)t;          /* round to nearest even */
        float up = nearest;
        if ((double)up < t) up = nextafterf(up, INFINITY);
        B_bits[c] = f32_bits(up);
        V_bits[c] = f32_bits(nearest);
    }
}

/* Phase 1-3 for one value that passed the early-stop test: the integer code.
 * Reading: L = 0 is only possible when one element carries the whole sum; it is
 * stored as 1, so codes are 1..tau and code-1 takes ceil(log2 tau) bits. */
static uint32_t code_of(uint32_t abs_bits, const uint32_t *B_bits, uint32_t tau) {
    uint32_t c = 1;
    for (uint32_t cp = 1; cp < tau; ++cp)
        if (abs_bits < B_bits[cp]) ++c; /* |v| < sum/b^cp  =>  L > cp */
    return c;
}

static uint32_t bitlen32(uint32_t x) { uint32_t n = 0; while (x) { ++n; x >>= 1; } return n; }

/* Phase 5: length of level i (1..2^l) when the longest delta needs M bits.
 * Reading: the paper's M/4, M/2, 3M/4, M generalised to ceil(i*M / 2^l). */
static uint32_t level_len(uint32_t i, uint32_t M, uint32_t l) {
    return (i * M + (1u << l) - 1) >> l;
}

/* getLengthFlag of Algorithm 2: the smallest level whose length holds delta. */
static uint32_t length_level(uint32_t delta, uint32_t M, uint32_t l) {
    uint32_t need = bitlen32(delta);
    for (uint32_t i = 1; i <= (1u << l); ++i)
        if (need <= level_len(i, M, l)) return i;
    return 1u << l; /* unreachable: level 2^l has length M >= need */
}

/* LSB-first bit writer over a zero-initialised byte buffer. */
static void put_bits(uint8_t *buf, uint64_t bitpos, uint32_t value, uint32_t nbits) {
    for (uint32_t k = 0; k < nbits; ++k)
        if (value >> k & 1) buf[(bitpos + k) >> 3] |= (uint8_t)(1u << ((bitpos + k) & 7));
}
static uint32_t get_bits(const uint8_t *buf, uint64_t bitpos, uint32_t nbits) {
    uint32_t v = 0;
    for (uint32_t k = 0; k < nbits; ++k)
        v |= (uint32_t)(buf[(bitpos + k) >> 3] >> ((bitpos + k) & 7) & 1) << k;
    return v;
}

static void put_u32(uint8_t *p, uint32_t x) { for (int k = 0; k < 4; ++k) p[k] = (uint8_t)(x >> (8 * k)); }
static void put_u64(uint8_t *p, uint64_t x) { for (int k = 0; k < 8; ++k) p[k] = (uint8_t)(x >> (8 * k)); }
static uint32_t get_u32(const uint8_t *p) { uint32_t x = 0; for (int k = 0; k < 4; ++k) x |= (uint32_t)p[k] << (8 * k); return x; }
static uint64_t get_u64(const uint8_t *p) { uint64_t x = 0; for (int k = 0; k < 8; ++k) x |= (uint64_t)p[k] << (8 * k); return x; }

static uint64_t words64(uint64_t bits) { return (bits + 63) / 64; }

/* Section 3.2, after the threshold filter: the codes 1..tau need ceil(log2 tau) bits (stored as
 * code-1), one more bit carries the sign: 8 bits for the recommended tau = 128, 9 above it. */
static uint32_t code_width(uint32_t tau) {
    uint32_t q = 0;
    while (((uint32_t)1 << q) < tau) ++q;
    return 1 + q;
}
/* bytes of the value plane of d survivors: d tokens of code_width bits, zero-padded to 8 bytes */
static uint64_t value_plane_bytes(uint64_t d, uint32_t tau) { return 8 * words64(d * code_width(tau)); }

/* Worst case: every element survives and every token takes l + 32 bits. */
uint64_t fastsgd_ref_compressed_size(uint64_t n, const ref_params *p) {
    if (!params_ok(p)) return 0;
    uint64_t KB = p->block_keys, nb = (n + KB - 1) / KB;
    uint64_t per_block = 8 * (words64(KB * p->flag_bits) + words64(KB * 32));
    return REF_HEADER_BYTES + value_plane_bytes(n, p->tau) + 16 * nb + nb * per_block;
}

/* ------------------------------------------------------------------------- *
 * Encoder = Algorithm 1 followed by Algorithm 2 on the surviving keys.
 *
 * Container (the paper fixes none; Reading): little-endian,
 *   [0,64)   header: magic, version u8, l u8, tau u16, block_keys u32,
 *            n_blocks u32, b f64, sum f64, n u64, d u64, total_bytes u64, 0 u64
 *   value plane: one token of w = 1 + ceil(log2 tau) bits per survivor (Section 3.2), token j at
 *            bit j*w counted LSB first: low w-1 bits = code-1, top bit = sign; for tau in 65..128
 *            that is one byte per survivor, bit7 = sign, bits0-6 = code-1; for tau in 129..256 nine bits
 *   zero padding to a multiple of 8 bytes
 *   block directory: n_blocks x {off8 u32, preKey u32, M u32, payload_bits u32}
 *   key blocks, back to back, each a flags plane (cnt*l bits) and a payload
 *            plane (payload_bits bits), both zero-padded to 64-bit words.
 * Reading: Algorithm 2 is applied per block of block_keys survivors with preKey
 * carried in (with one block it is the paper's algorithm unchanged), and the
 * tokens of a block are stored planar: all flags, then all binary deltas, in key
 * order -- the same bits as the paper's flag||delta concatenation, permuted.
 * Reading: M = max(1, bit length of maxDelta) (the paper's ceil(log2 maxDelta)
 * is one short for powers of two and undefined below 2).
 * ------------------------------------------------------------------------- */
int fastsgd_ref_compress(const uint32_t *keys, const float *values, uint64_t n,
                         const ref_params *p, uint8_t *out, uint64_t out_capacity,
                         uint64_t *out_bytes) {
    if (out_bytes) *out_bytes = 0;
    if (!params_ok(p) || !out || !out_bytes || (n && (!keys || !values))) return REF_ERR_INVALID_ARG;
    if (n > 4294967296ull) return REF_ERR_INVALID_ARG;
    if (out_capacity < REF_HEADER_BYTES) return REF_ERR_BUFFER_TOO_SMALL;
    const uint32_t tau = p->tau, l = p->flag_bits, KB = p->block_keys;

    /* Algorithm 1 line 1 */
    double sum;
    if (fastsgd_ref_abs_sum(values, n, &sum)) return REF_ERR_NONFINITE;

    /* line 2 (and the boundaries of all other codes) */
    uint32_t B_bits[REF_MAX_TAU + 1], V_bits[REF_MAX_TAU + 1];
    fastsgd_ref_tables(sum, p->base, tau, B_bits, V_bits);
    const uint32_t tau_e = B_bits[tau];

    /* lines 3-10: Result = codes of survivors, in key order */
    const uint32_t w = code_width(tau);
    uint64_t d = 0;
    uint32_t *skeys = (uint32_t *)malloc((n ? n : 1) * sizeof(uint32_t));
    uint16_t *token = (uint16_t *)malloc((n ? n : 1) * sizeof(uint16_t));
    if (!skeys || !token) { free(skeys); free(token); return REF_ERR_INVALID_ARG; }
    if (sum > 0.0) {
        for (uint64_t j = 0; j < n; ++j) {
            uint32_t bits = f32_bits(values[j]);
            uint32_t a = bits & 0x7FFFFFFFu;
            if (a >= tau_e) { /* |v_j| >= tau_e */
                uint32_t c = code_of(a, B_bits, tau);
                token[d] = (uint16_t)((bits >> 31) << (w - 1) | (c - 1));
                skeys[d] = keys[j];
                ++d;
            }
        }
    }
    uint64_t nb = (d + KB - 1) / KB;
    uint64_t dir_off = REF_HEADER_BYTES + value_plane_bytes(d, tau);
    uint64_t blocks_off = dir_off + 16 * nb;
    if (blocks_off > out_capacity) { free(skeys); free(token); return REF_ERR_BUFFER_TOO_SMALL; }
    memset(out + REF_HEADER_BYTES, 0, dir_off - REF_HEADER_BYTES);
    for (uint64_t j = 0; j < d; ++j) put_bits(out + REF_HEADER_BYTES, j * w, token[j], w);
    free(token);

    /* Algorithm 2 on the d surviving keys, block by block */
    uint64_t off8 = 0; /* running block offset in 8-byte units */
    uint32_t *delta = (uint32_t *)malloc(KB * sizeof(uint32_t));
    uint32_t preKey = 0;
    for (uint64_t blk = 0; blk < nb; ++blk) {
        uint64_t first = blk * KB;
        uint32_t cnt = (uint32_t)((d - first < KB) ? d - first : KB);
        uint32_t blockPre = preKey, maxDelta = 0;
        for (uint32_t i = 0; i < cnt; ++i) { /* first loop of Algorithm 2 */
            uint32_t k = skeys[first + i];
            if (k < preKey || (k == preKey && first + i != 0)) { free(delta); free(skeys); return REF_ERR_UNSORTED_KEYS; }
            delta[i] = k - preKey;
            preKey = k;
            if (maxDelta < delta[i]) maxDelta = delta[i];
        }
        uint32_t M = bitlen32(maxDelta);
        if (M < 1) M = 1;
        uint64_t payload_bits = 0;
        for (uint32_t i = 0; i < cnt; ++i) payload_bits += level_len(length_level(delta[i], M, l), M, l);
        uint64_t fwords = words64((uint64_t)cnt * l), pwords = words64(payload_bits);
        uint64_t start = blocks_off + 8 * off8, size = 8 * (fwords + pwords);
        if (start + size > out_capacity) { free(delta); free(skeys); return REF_ERR_BUFFER_TOO_SMALL; }
        memset(out + start, 0, size);
        uint64_t pbit = 0;
        for (uint32_t i = 0; i < cnt; ++i) { /* second loop of Algorithm 2 */
            uint32_t level = length_level(delta[i], M, l);
            uint32_t len = level_len(level, M, l);
            put_bits(out + start, (uint64_t)i * l, level - 1, l);
            put_bits(out + start + 8 * fwords, pbit, delta[i], len);
            pbit += len;
        }
        uint8_t *e = out + dir_off + 16 * blk;
        put_u32(e, (uint32_t)off8); put_u32(e + 4, blockPre); put_u32(e + 8, M); put_u32(e + 12, (uint32_t)payload_bits);
        off8 += fwords + pwords;
    }
    free(delta);
    free(skeys);

    uint64_t total = blocks_off + 8 * off8;
    uint8_t *h = out;
    memset(h, 0, REF_HEADER_BYTES);
    put_u32(h, REF_MAGIC);
    h[4] = REF_VERSION; h[5] = (uint8_t)l; h[6] = (uint8_t)(tau & 0xFF); h[7] = (uint8_t)(tau >> 8);
    put_u32(h + 8, KB); put_u32(h + 12, (uint32_t)nb);
    put_u64(h + 16, f64_bits(p->base)); put_u64(h + 24, f64_bits(sum));
    put_u64(h + 32, n); put_u64(h + 40, d); put_u64(h + 48, total);
    *out_bytes = total;
    return REF_OK;
}

/* ------------------------------------------------------------------------- *
 * Decoder, phases 1-4 of Section 3.1.
 * phase 1: tokens are told apart by their flags; phase 2: keys = running sum of
 * deltas; phase 3: b^L; phase 4: value = +-sum / b^L (taken from V[] above).
 * ------------------------------------------------------------------------- */
int fastsgd_ref_decompress(const uint8_t *stream, uint64_t stream_bytes,
                           uint32_t *keys_out, float *values_out, uint64_t capacity,
                           uint64_t *count_out) {
    if (count_out) *count_out = 0;
    if (!stream || !count_out) return REF_ERR_INVALID_ARG;
    if (stream_bytes < REF_HEADER_BYTES) return REF_ERR_CORRUPT_STREAM;
    const uint8_t *h = stream;
    if (get_u32(h) != REF_MAGIC || h[4] != REF_VERSION) return REF_ERR_CORRUPT_STREAM;
    ref_params p;
    p.flag_bits = h[5]; p.tau = h[6] | (uint32_t)h[7] << 8; p.block_keys = get_u32(h + 8); p.reserved = 0;
    p.base = bits_f64(get_u64(h + 16));
    if (!params_ok(&p)) return REF_ERR_CORRUPT_STREAM;
    uint64_t nb = get_u32(h + 12);
    double sum = bits_f64(get_u64(h + 24));
    uint64_t n = get_u64(h + 32), d = get_u64(h + 40), total = get_u64(h + 48);
    const uint32_t l = p.flag_bits, KB = p.block_keys, tau = p.tau;
    if (!(sum >= 0.0) || isinf(sum)) return REF_ERR_CORRUPT_STREAM;
    if (n > 4294967296ull || d > n) return REF_ERR_CORRUPT_STREAM;
    if (nb != (d + KB - 1) / KB) return REF_ERR_CORRUPT_STREAM;
    const uint32_t w = code_width(tau);
    uint64_t dir_off = REF_HEADER_BYTES + value_plane_bytes(d, tau), blocks_off = dir_off + 16 * nb;
    if (total > stream_bytes || total < blocks_off || (total & 7)) return REF_ERR_CORRUPT_STREAM;
    if (d > capacity) return REF_ERR_BUFFER_TOO_SMALL;
    if (d && (!keys_out || !values_out)) return REF_ERR_INVALID_ARG;

    uint32_t B_bits[REF_MAX_TAU + 1], V_bits[REF_MAX_TAU + 1];
    fastsgd_ref_tables(sum, p.base, tau, B_bits, V_bits);

    /* phases 3-4 */
    for (uint64_t j = 0; j < d; ++j) {
        uint32_t token = get_bits(stream + REF_HEADER_BYTES, j * w, w);
        uint32_t c = (token & (((uint32_t)1 << (w - 1)) - 1)) + 1;
        if (c > tau) return REF_ERR_CORRUPT_STREAM;
        values_out[j] = bits_f32(V_bits[c] | (token >> (w - 1)) << 31);
    }

    /* phases 1-2 */
    uint64_t total_words = (total - blocks_off) / 8, expect_off8 = 0;
    uint32_t prev_last = 0;
    for (uint64_t blk = 0; blk < nb; ++blk) {
        const uint8_t *e = stream + dir_off + 16 * blk;
        uint64_t off8 = get_u32(e);
        uint32_t preKey = get_u32(e + 4), M = get_u32(e + 8);
        uint64_t payload_bits = get_u32(e + 12);
        uint64_t first = blk * KB;
        uint32_t cnt = (uint32_t)((d - first < KB) ? d - first : KB);
        uint64_t fwords = words64((uint64_t)cnt * l), pwords = words64(payload_bits);
        if (M < 1 || M > 32) return REF_ERR_CORRUPT_STREAM;
        if (off8 != expect_off8 || off8 + fwords + pwords > total_words) return REF_ERR_CORRUPT_STREAM;
        if (preKey != prev_last) return REF_ERR_CORRUPT_STREAM;
        const uint8_t *fl = stream + blocks_off + 8 * off8, *pl = fl + 8 * fwords;
        uint64_t pbit = 0, key = preKey;
        for (uint32_t i = 0; i < cnt; ++i) {
            uint32_t level = get_bits(fl, (uint64_t)i * l, l) + 1;
            uint32_t len = level_len(level, M, l);
            if (pbit + len > payload_bits) return REF_ERR_CORRUPT_STREAM;
            uint32_t delta = get_bits(pl, pbit, len);
            /* Eq. 4 is taken over distinct ascending keys: only the very first delta of a gradient can be 0 */
            if (delta == 0 && first + i != 0) return REF_ERR_CORRUPT_STREAM;
            key += delta;
            pbit += len;
            if (key > 0xFFFFFFFFull) return REF_ERR_CORRUPT_STREAM;
            keys_out[first + i] = (uint32_t)key;
        }
        if (pbit != payload_bits) return REF_ERR_CORRUPT_STREAM;
        prev_last = (uint32_t)key;
        expect_off8 = off8 + fwords + pwords;
    }
    if (expect_off8 != total_words) return REF_ERR_CORRUPT_STREAM;
    *count_out = d;
    return REF_OK;
}

/* ------------------------------------------------------------------------- *
 * Several independent gradients in one call (a per-layer batch): gradient s is
 * elements [seg_offsets[s], seg_offsets[s+1]) with its own parameters; each is
 * encoded exactly as above into its own stream, streams are laid back to back,
 * and out_offsets[s] .. out_offsets[s+1] delimit stream s.
 * ------------------------------------------------------------------------- */
int fastsgd_ref_compress_segmented(const uint32_t *keys, const float *values,
                                   const uint64_t *seg_offsets, uint32_t n_segments,
                                   const ref_params *params, uint32_t params_stride,
                                   uint8_t *out, uint64_t out_capacity, uint64_t *out_offsets) {
    if (!seg_offsets || !params || !out || !out_offsets) return REF_ERR_INVALID_ARG;
    uint64_t pos = 0;
    out_offsets[0] = 0;
    for (uint32_t s = 0; s < n_segments; ++s) {
        if (seg_offsets[s + 1] < seg_offsets[s]) return REF_ERR_INVALID_ARG;
        uint64_t o = seg_offsets[s], cnt = seg_offsets[s + 1] - o, bytes = 0;
        const ref_params *p = &params[params_stride ? (uint64_t)s * params_stride : 0];
        int rc = fastsgd_ref_compress(keys + o, values + o, cnt, p, out + pos,
                                      out_capacity > pos ? out_capacity - pos : 0, &bytes);
        if (rc != REF_OK) return rc;
        pos += bytes;
        out_offsets[s + 1] = pos;
    }
    return REF_OK;
}

int fastsgd_ref_decompress_segmented(const uint8_t *streams, const uint64_t *stream_offsets,
                                     uint32_t n_segments, uint32_t *keys_out, float *values_out,
                                     uint64_t capacity, uint64_t *pair_offsets) {
    if (!streams || !stream_offsets || !pair_offsets) return REF_ERR_INVALID_ARG;
    uint64_t pos = 0;
    pair_offsets[0] = 0;
    for (uint32_t s = 0; s < n_segments; ++s) {
        if (stream_offsets[s + 1] < stream_offsets[s]) return REF_ERR_INVALID_ARG;
        uint64_t cnt = 0;
        int rc = fastsgd_ref_decompress(streams + stream_offsets[s],
                                        stream_offsets[s + 1] - stream_offsets[s],
                                        keys_out + pos, values_out + pos,
                                        capacity > pos ? capacity - pos : 0, &cnt);
        if (rc != REF_OK) return rc;
        pos += cnt;
        pair_offsets[s + 1] = pos;
    }
    return REF_OK;
}

/* ------------------------------------------------------------------------- *
 * Decoder followed by the aggregation the decoded gradients are for (Section
 * 2.1, Fig. 1: every worker's gradient is decoded and the gradients are added
 * up before the model update): dense[k] += v for every decoded pair (k, v),
 * stream after stream in the given order, every addition a binary32 addition.
 * Reading: the paper does not say in which order or precision the workers'
 * gradients are added; stream order and binary32 make the result reproducible
 * (keys are unique inside a stream, so the order inside a stream is immaterial).
 * A key >= dense_len is REF_ERR_BUFFER_TOO_SMALL.  On any error dense[] holds a
 * partial sum.
 * ------------------------------------------------------------------------- */
int fastsgd_ref_decompress_accumulate(const uint8_t *streams, const uint64_t *stream_offsets,
                                      uint32_t n_streams, float *dense, uint64_t dense_len,
                                      uint64_t *count_out) {
    if (count_out) *count_out = 0;
    if (!streams || !stream_offsets || !count_out || (dense_len && !dense)) return REF_ERR_INVALID_ARG;
    uint64_t total = 0;
    for (uint32_t s = 0; s < n_streams; ++s) {
        if (stream_offsets[s + 1] < stream_offsets[s]) return REF_ERR_INVALID_ARG;
        const uint8_t *st = streams + stream_offsets[s];
        uint64_t bytes = stream_offsets[s + 1] - stream_offsets[s];
        uint64_t d = bytes >= REF_HEADER_BYTES ? get_u64(st + 40) : 0;
        if (d > 8 * bytes) return REF_ERR_CORRUPT_STREAM;      /* every pair costs more than one bit */
        uint32_t *k = (uint32_t *)malloc((d + 1) * sizeof(uint32_t));
        float *v = (float *)malloc((d + 1) * sizeof(float));
        if (!k || !v) { free(k); free(v); return REF_ERR_INVALID_ARG; }
        uint64_t cnt = 0;
        int rc = fastsgd_ref_decompress(st, bytes, k, v, d, &cnt);
        for (uint64_t j = 0; rc == REF_OK && j < cnt; ++j) {
            if (k[j] >= dense_len) rc = REF_ERR_BUFFER_TOO_SMALL;
            else dense[k[j]] = dense[k[j]] + v[j];
        }
        free(k); free(v);
        if (rc != REF_OK) return rc;
        total += cnt;
    }
    *count_out = total;
    return REF_OK;
}

/* ------------------------------------------------------------------------- *
 * Decoder followed by the model update of Section 4.1 (Adam SGD), applied at
 * the decoded keys only: for every decoded pair (k, g)
 *     m[k]     = beta1 * m[k] + (1 - beta1) * g
 *     v[k]     = beta2 * v[k] + (1 - beta2) * g * g
 *     theta[k] = theta[k] - eta * m[k] / sqrt(v[k] + eps)
 * with the new m[k], v[k] on the right of the third line.  Readings: the two
 * equations of Section 4.1 are taken as printed, i.e. eps is under the square
 * root and there is no bias correction; coordinates whose gradient did not
 * survive the filter are not touched (their g is not known to the receiver).
 * The three arrays hold binary32; the arithmetic here is binary64 on the stored
 * values, each result rounded to binary32 when it is stored.
 * A key >= dim is REF_ERR_BUFFER_TOO_SMALL (arrays then partly updated).
 * ------------------------------------------------------------------------- */
int fastsgd_ref_decompress_adam(const uint8_t *stream, uint64_t bytes, float *theta, float *m, float *v,
                                uint64_t dim, double eta, double beta1, double beta2, double eps,
                                uint64_t *count_out) {
    if (count_out) *count_out = 0;
    if (!stream || !count_out || (dim && (!theta || !m || !v))) return REF_ERR_INVALID_ARG;
    uint64_t d = bytes >= REF_HEADER_BYTES ? get_u64(stream + 40) : 0;
    if (d > 8 * bytes) return REF_ERR_CORRUPT_STREAM;          /* every pair costs more than one bit */
    uint32_t *k = (uint32_t *)malloc((d + 1) * sizeof(uint32_t));
    float *g = (float *)malloc((d + 1) * sizeof(float));
    if (!k || !g) { free(k); free(g); return REF_ERR_INVALID_ARG; }
    uint64_t cnt = 0;
    int rc = fastsgd_ref_decompress(stream, bytes, k, g, d, &cnt);
    for (uint64_t j = 0; rc == REF_OK && j < cnt; ++j) {
        if (k[j] >= dim) { rc = REF_ERR_BUFFER_TOO_SMALL; break; }
        const uint32_t i = k[j];
        const double gj = (double)g[j];
        const double mt = beta1 * (double)m[i] + (1.0 - beta1) * gj;
        const double vt = beta2 * (double)v[i] + (1.0 - beta2) * gj * gj;
        m[i] = (float)mt;
        v[i] = (float)vt;
        theta[i] = (float)((double)theta[i] - eta * (double)m[i] / sqrt((double)v[i] + eps));
    }
    free(k); free(g);
    if (rc != REF_OK) return rc;
    *count_out = cnt;
    return REF_OK;
}

/* ------------------------------------------------------------------------- *
 * Debug view for the Fig. 3 worked example: Algorithm 2 literally (one global M,
 * no blocks), each token rendered the way the paper prints it: the flag as l
 * binary digits, then the delta as `len` binary digits, most significant first,
 * tokens separated by a space.  Returns M, or 0 if text_capacity is too small.
 * ------------------------------------------------------------------------- */
uint32_t fastsgd_ref_key_tokens_text(const uint32_t *keys, uint32_t d, uint32_t l,
                                     char *text, uint64_t text_capacity) {
    uint32_t preKey = 0, maxDelta = 0;
    for (uint32_t j = 0; j < d; ++j) {
        uint32_t dk = keys[j] - preKey;
        preKey = keys[j];
        if (maxDelta < dk) maxDelta = dk;
    }
    uint32_t M = bitlen32(maxDelta);
    if (M < 1) M = 1;
    uint64_t pos = 0;
    preKey = 0;
    for (uint32_t j = 0; j < d; ++j) {
        uint32_t dk = keys[j] - preKey;
        preKey = keys[j];
        uint32_t level = length_level(dk, M, l), len = level_len(level, M, l);
        if (pos + l + len + 2 > text_capacity) return 0;
        for (int k = (int)l - 1; k >= 0; --k) text[pos++] = ((level - 1) >> k & 1) ? '1' : '0';
        for (int k = (int)len - 1; k >= 0; --k) text[pos++] = (dk >> k & 1) ? '1' : '0';
        text[pos++] = (j + 1 < d) ? ' ' : '\0';
    }
    if (d == 0) { if (text_capacity < 1) return 0; text[0] = '\0'; }
    return M;
}
