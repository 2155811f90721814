"""Do the pins bite?  Each case plants one plausible mistake in a copy of the oracle's C source (a dropped
term, a comparison off by one, a rounding in the wrong direction, swapped operands), builds it, and runs the
pins against the broken build: at least one of them must fail.  Runs on the CPU only; the mistakes touch
arithmetic and comparisons, never addressing."""
import os
import subprocess

import pytest

from oracle import ref
from tests import test_oracle_adam as TA
from tests import test_oracle_aggregate as TG
from tests import test_oracle_keys as TK
from tests import test_oracle_values as TV

SRC = os.path.join(os.path.dirname(ref.__file__), "fastsgd_ref.c")

VALUE_PINS = [lambda: TV.test_abs_sum_equals_fsum_wide_exponents(0),
              TV.test_abs_sum_rounds_ties_to_even_and_sticky,
              TV.test_abs_sum_many_equal_values_carry_chain,
              lambda: TV.test_tables_against_exact_rationals(100.25, 1.1, 128),
              TV.test_fig2_worked_example,
              lambda: TV.test_codes_match_exact_rational_log(0, 1.1, 128),
              TV.test_kept_set_is_threshold_test,
              TV.test_single_element_code_clamped_to_one,
              lambda: TV.test_decode_underestimates_within_one_base_step(0, 1.1),
              TV.test_values_exactly_on_below_and_above_bucket_boundaries,
              lambda: TV.test_codes_take_one_plus_ceil_log2_tau_bits(33)]
WIDE_PINS = [TV.test_tables_for_256_codes_in_closed_form_down_to_the_smallest_binary32,
             lambda: TV.test_codes_above_128_match_exact_rational_log(20, 1.1, 200, 30, 1.0),
             lambda: TV.test_a_threshold_above_128_only_adds_survivors(200),
             TV.test_parameter_limits_above_128]
KEY_PINS = [TK.test_fig3_worked_example,
            lambda: TK.test_flag_is_smallest_level_that_fits(2, 0),
            lambda: TK.test_flag_is_smallest_level_that_fits(3, 1),
            TK.test_M_for_powers_of_two_and_small_deltas,
            lambda: TK.test_block_boundaries_carry_prekey(257),
            lambda: TK.test_size_constant_gap(8),
            lambda: TK.test_round_trip_keys_lossless(0, 256, 2),
            TK.test_unsorted_or_duplicate_surviving_keys_are_rejected]
DECODE_PINS = [lambda: TV.test_decode_underestimates_within_one_base_step(0, 1.1),
               TV.test_decoded_magnitude_stays_in_its_own_bucket,
               lambda: TK.test_round_trip_keys_lossless(0, 256, 2),
               lambda: TK.test_block_boundaries_carry_prekey(257),
               TK.test_corrupt_streams_are_rejected,
               TK.test_a_stream_that_repeats_a_key_is_rejected,
               TK.test_segmented_equals_independent_streams]
SIZE_PINS = [lambda: TK.test_size_bound_is_reached_by_a_block_of_longest_tokens(256),
             lambda: TK.test_size_bound_is_reached_by_a_block_of_longest_tokens(1024),
             TK.test_size_bound_term_by_term_over_a_grid]
AFTER_PINS = [lambda: TG.test_aggregate_equals_scatter_adds_in_stream_order(2),
              lambda: TG.test_aggregate_equals_scatter_adds_in_stream_order(5),
              TA.test_first_step_from_zero_state_closed_form,
              TA.test_sign_step_when_eps_is_zero,
              TA.test_betas_are_not_swapped_and_second_moment_uses_the_square,
              TA.test_repeated_steps_follow_the_geometric_closed_form]

# (name, text in the source, what it becomes, pins that must notice)
MUTANTS = [
    ("sum: hidden bit of normal values dropped", "uint32_t m = e ? (frac | 0x800000u) : frac;",
     "uint32_t m = frac;", VALUE_PINS),
    ("sum: carries between limbs dropped", "carry = (carry >> 32) + (t >> 32);", "carry = (carry >> 32);", VALUE_PINS),
    ("sum: ties rounded up instead of to even", "if (guard && (sticky || (q & 1))) ++q;", "if (guard) ++q;", VALUE_PINS),
    ("sum: truncated instead of rounded", "if (guard && (sticky || (q & 1))) ++q;", ";", VALUE_PINS),
    ("table: boundary rounded to nearest instead of up", "if ((double)up < t) up = nextafterf(up, INFINITY);", ";", VALUE_PINS),
    ("table: decoded magnitude rounded up", "V_bits[c] = f32_bits(nearest);", "V_bits[c] = f32_bits(up);", VALUE_PINS),
    ("table: b^c one step late", "        P = P * base;\n        double t = sum / P;", "        double t = sum / P;\n        P = P * base;", VALUE_PINS),
    ("code: a value on a boundary falls into the next bucket", "if (abs_bits < B_bits[cp]) ++c;", "if (abs_bits <= B_bits[cp]) ++c;", VALUE_PINS),
    ("code: counted from zero", "    uint32_t c = 1;\n    for (uint32_t cp = 1; cp < tau; ++cp)", "    uint32_t c = 0;\n    for (uint32_t cp = 1; cp < tau; ++cp)", VALUE_PINS),
    ("filter: a value on the threshold is dropped", "if (a >= tau_e) { /* |v_j| >= tau_e */", "if (a > tau_e) { /* |v_j| >= tau_e */", VALUE_PINS),
    ("sign lost", "token[d] = (uint16_t)((bits >> 31) << (w - 1) | (c - 1));", "token[d] = (uint16_t)(c - 1);", VALUE_PINS),
    ("tau above 128: token cut to a byte", "token[d] = (uint16_t)((bits >> 31) << (w - 1) | (c - 1));",
     "token[d] = (uint8_t)((bits >> 31) << (w - 1) | (c - 1));", WIDE_PINS),
    ("tau above 128: high byte of tau left out of the header", "h[7] = (uint8_t)(tau >> 8);", "h[7] = 0;", WIDE_PINS),
    ("tau above 128: header read as one byte", "p.tau = h[6] | (uint32_t)h[7] << 8;", "p.tau = h[6];", WIDE_PINS),
    ("tau above 128: any base allowed", "if (p->tau > 128 && !(p->base <= 4.0)) return 0;", ";", WIDE_PINS),
    ("tau above 128: limit one too low", "if (p->tau < 1 || p->tau > REF_MAX_TAU) return 0;",
     "if (p->tau < 1 || p->tau >= REF_MAX_TAU) return 0;", WIDE_PINS),
    ("token one bit too wide", "    return 1 + q;", "    return 2 + q;", VALUE_PINS),
    ("level length rounded down", "return (i * M + (1u << l) - 1) >> l;", "return (i * M) >> l;", KEY_PINS),
    ("level chosen one too high", "if (need <= level_len(i, M, l)) return i;", "if (need < level_len(i, M, l)) return i;", KEY_PINS),
    ("M = bit length of maxDelta - 1 (the ceil(log2) of the listing)", "        uint32_t M = bitlen32(maxDelta);\n        if (M < 1) M = 1;\n        uint64_t payload_bits = 0;",
     "        uint32_t M = bitlen32(maxDelta ? maxDelta - 1 : 0);\n        if (M < 1) M = 1;\n        uint64_t payload_bits = 0;", KEY_PINS),
    ("preKey not carried into the next block", "uint32_t blockPre = preKey, maxDelta = 0;", "uint32_t blockPre = preKey, maxDelta = 0; if (blk) preKey = 0;", KEY_PINS),
    ("equal neighbouring keys accepted", "if (k < preKey || (k == preKey && first + i != 0))", "if (k < preKey)", KEY_PINS),
    ("decoder: sign ignored", "values_out[j] = bits_f32(V_bits[c] | (token >> (w - 1)) << 31);",
     "values_out[j] = bits_f32(V_bits[c]);", DECODE_PINS),
    ("decoder: magnitude of the neighbouring code", "uint32_t c = (token & (((uint32_t)1 << (w - 1)) - 1)) + 1;",
     "uint32_t c = (token & (((uint32_t)1 << (w - 1)) - 1)) + 2;", DECODE_PINS),
    ("decoder: deltas not summed up", "key += delta;", "key = delta;", DECODE_PINS),
    ("decoder: a repeated key tolerated", "if (delta == 0 && first + i != 0) return REF_ERR_CORRUPT_STREAM;", ";", DECODE_PINS),
    ("decoder: block does not start from its preKey", "uint64_t pbit = 0, key = preKey;", "uint64_t pbit = 0, key = 0;", DECODE_PINS),
    ("decoder: directory chain not checked", "if (preKey != prev_last) return REF_ERR_CORRUPT_STREAM;", ";", DECODE_PINS),
    ("decoder: unused payload bits tolerated", "if (pbit != payload_bits) return REF_ERR_CORRUPT_STREAM;", ";", DECODE_PINS),
    ("size bound: directory entries left out", "return REF_HEADER_BYTES + value_plane_bytes(n, p->tau) + 16 * nb + nb * per_block;",
     "return REF_HEADER_BYTES + value_plane_bytes(n, p->tau) + nb * per_block;", SIZE_PINS),
    ("size bound: longest binary delta taken as 31 bits", "words64(KB * 32));", "words64(KB * 31));", SIZE_PINS),
    ("size bound: flags plane left out", "uint64_t per_block = 8 * (words64(KB * p->flag_bits) + words64(KB * 32));",
     "uint64_t per_block = 8 * words64(KB * 32);", SIZE_PINS),
    ("size bound: value tokens counted as bytes whatever tau is", "static uint64_t value_plane_bytes(uint64_t d, uint32_t tau) { return 8 * words64(d * code_width(tau)); }",
     "static uint64_t value_plane_bytes(uint64_t d, uint32_t tau) { (void)tau; return 8 * words64(d * 8); }", WIDE_PINS + SIZE_PINS),
    ("aggregate: streams taken from the last to the first", "const uint8_t *st = streams + stream_offsets[s];\n        uint64_t bytes = stream_offsets[s + 1] - stream_offsets[s];\n        uint64_t d = bytes >= REF_HEADER_BYTES ? get_u64(st + 40) : 0;\n        if (d > 8 * bytes) return REF_ERR_CORRUPT_STREAM;      /* every pair costs more than one bit */\n        uint32_t *k",
     "const uint32_t sr = n_streams - 1 - s;\n        const uint8_t *st = streams + stream_offsets[sr];\n        uint64_t bytes = stream_offsets[sr + 1] - stream_offsets[sr];\n        uint64_t d = bytes >= REF_HEADER_BYTES ? get_u64(st + 40) : 0;\n        if (d > 8 * bytes) return REF_ERR_CORRUPT_STREAM;\n        uint32_t *k", AFTER_PINS),
    ("aggregate overwrites instead of adding", "else dense[k[j]] = dense[k[j]] + v[j];", "else dense[k[j]] = v[j];", AFTER_PINS),
    ("Adam: betas swapped", "const double mt = beta1 * (double)m[i] + (1.0 - beta1) * gj;", "const double mt = beta2 * (double)m[i] + (1.0 - beta2) * gj;", AFTER_PINS),
    ("Adam: second moment without the square", "(1.0 - beta2) * gj * gj;", "(1.0 - beta2) * gj;", AFTER_PINS),
    ("Adam: eps outside the root", "/ sqrt((double)v[i] + eps));", "/ (sqrt((double)v[i]) + eps));", AFTER_PINS),
    ("Adam: step added instead of subtracted", "(double)theta[i] - eta * (double)m[i]", "(double)theta[i] + eta * (double)m[i]", AFTER_PINS),
]


@pytest.fixture
def broken_oracle(tmp_path):
    keep = ref._lib

    def build(old, new):
        text = open(SRC).read()
        assert text.count(old) == 1, f"the source no longer holds exactly one {old!r}"
        src = tmp_path / "mutant.c"
        lib = tmp_path / "libmutant.so"
        src.write_text(text.replace(old, new))
        subprocess.run(["gcc", "-std=c99", "-O1", "-ffp-contract=off", "-fno-fast-math", "-w", "-shared", "-fPIC",
                        "-o", str(lib), str(src), "-lm"], check=True)
        ref._lib = ref.load(str(lib))

    yield build
    ref._lib = keep


@pytest.mark.parametrize("name,old,new,pins", MUTANTS, ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_fails_a_pin(broken_oracle, name, old, new, pins):
    ref.lib()                                   # the sound build is loaded (and kept aside by the fixture)
    broken_oracle(old, new)
    caught = []
    for pin in pins:
        try:
            pin()
        except Exception:                       # an assertion, or the independent parser running off a plane
            caught.append(pin)
            break
    assert caught, f"no pin noticed: {name}"


def test_the_sound_oracle_passes_the_same_pins():
    for pin in VALUE_PINS + WIDE_PINS + KEY_PINS + DECODE_PINS + SIZE_PINS + AFTER_PINS:
        pin()
