/*
 * Sanitizer driver for the CPU oracle (test infrastructure): built together with oracle/fastsgd_ref.c under
 * AddressSanitizer and UndefinedBehaviorSanitizer and run on the CPU.  It encodes seeded gradients, then feeds
 * the decoders every single-bit flip of the header, a few thousand flips elsewhere in the stream, truncations
 * and wrong capacities.  Any verdict is fine; an out-of-bounds access, an overflowing shift or a misaligned load
 * makes the sanitizers abort, which is what the test looks for.
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct { double base; uint32_t tau, flag_bits, block_keys, reserved; } ref_params;
uint64_t fastsgd_ref_compressed_size(uint64_t n, const ref_params *p);
int fastsgd_ref_compress(const uint32_t *keys, const float *values, uint64_t n, const ref_params *p, uint8_t *out,
                         uint64_t out_capacity, uint64_t *out_bytes);
int fastsgd_ref_decompress(const uint8_t *stream, uint64_t stream_bytes, uint32_t *keys_out, float *values_out,
                           uint64_t capacity, uint64_t *count_out);
int fastsgd_ref_decompress_accumulate(const uint8_t *streams, const uint64_t *stream_offsets, uint32_t n_streams,
                                      float *dense, uint64_t dense_len, uint64_t *count_out);
int fastsgd_ref_decompress_adam(const uint8_t *stream, uint64_t bytes, float *theta, float *m, float *v, uint64_t dim,
                                double eta, double beta1, double beta2, double eps, uint64_t *count_out);

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd(void) { rng_state ^= rng_state << 13; rng_state ^= rng_state >> 7; rng_state ^= rng_state << 17; return rng_state; }

static long run_case(uint32_t n, uint32_t tau, uint32_t l, uint32_t kb, double base, uint32_t max_gap) {
    ref_params p = {base, tau, l, kb, 0};
    uint32_t *keys = malloc((n + 1) * sizeof *keys);
    float *vals = malloc((n + 1) * sizeof *vals);
    uint64_t k = rnd() % 7;
    for (uint32_t i = 0; i < n; ++i) {
        keys[i] = (uint32_t)k;
        k += 1 + rnd() % max_gap;
        vals[i] = (float)((double)(rnd() % 2000001) / 1e6 - 1.0) * (float)(1.0 / (1 + rnd() % 1000));
    }
    uint64_t cap = fastsgd_ref_compressed_size(n, &p), bytes = 0;
    uint8_t *st = malloc(cap + 8), *bad = malloc(cap + 8);
    if (fastsgd_ref_compress(keys, vals, n, &p, st, cap, &bytes) != 0) { printf("compress failed\n"); exit(2); }
    uint32_t *ko = malloc((n + 1) * sizeof *ko);
    float *vo = malloc((n + 1) * sizeof *vo);
    uint64_t cnt = 0;
    if (fastsgd_ref_decompress(st, bytes, ko, vo, n, &cnt) != 0) { printf("round trip failed\n"); exit(2); }
    const uint64_t dim = k + 1;
    float *dense = calloc(dim, sizeof *dense), *m = calloc(dim, sizeof *m), *v = calloc(dim, sizeof *v);
    long runs = 0;
    for (uint64_t trial = 0; trial < 512 + 3000; ++trial) {
        memcpy(bad, st, bytes);
        uint64_t bit = trial < 512 ? trial : rnd() % (8 * bytes);      /* every header bit, then anywhere */
        if (bit >= 8 * bytes) continue;
        bad[bit >> 3] ^= (uint8_t)(1u << (bit & 7));
        uint64_t give = (trial % 5 == 4) ? rnd() % (bytes + 1) : bytes;  /* sometimes truncated */
        uint64_t capn = (trial % 7 == 6) ? rnd() % (n + 1) : n;           /* sometimes too small */
        /* an exact-size copy, so that a read past the given length is a read past the allocation */
        uint8_t *exact = malloc(give ? give : 1);
        memcpy(exact, bad, give);
        fastsgd_ref_decompress(exact, give, ko, vo, capn, &cnt);
        if (trial % 4 == 0) {
            uint64_t offs[2] = {0, give};
            fastsgd_ref_decompress_accumulate(exact, offs, 1, dense, (trial % 8) ? dim : dim / 2, &cnt);
            fastsgd_ref_decompress_adam(exact, give, dense, m, v, (trial % 8) ? dim : dim / 2, 0.01, 0.9, 0.999, 1e-8, &cnt);
        }
        free(exact);
        ++runs;
    }
    free(keys); free(vals); free(st); free(bad); free(ko); free(vo); free(dense); free(m); free(v);
    return runs;
}

int main(void) {
    long runs = 0;
    runs += run_case(3000, 128, 2, 256, 1.05, 40);
    runs += run_case(5000, 200, 3, 1024, 1.03, 3);
    runs += run_case(700, 5, 1, 256, 1.9, 1u << 22);
    runs += run_case(9000, 64, 5, 4096, 1.08, 1000);
    runs += run_case(1, 128, 2, 1024, 1.1, 2);
    printf("sanitized runs: %ld\n", runs);
    return 0;
}
