"""Pins for the key side of the CPU oracle (Algorithm 2, Eq. 4, Phases 4-5, decoder phases 1-2),
the container, the error paths and the segmented form."""
import math
import os
import struct

import numpy as np
import pytest

from oracle import ref
from tests.streamparse import bitlen, level_len, parse, with_zero_delta
from tests.test_oracle_values import golden

BIG = np.float32(1.0)   # with b = 1.1, tau = 128 every equal-magnitude value survives while n < ~2e5


def all_survive(keys, p=None):
    keys = np.asarray(keys, dtype=np.uint32)
    p = p or ref.params(1.1, 128, 2, 1024)
    rc, st = ref.compress(keys, np.full(keys.size, BIG, np.float32), p)
    assert rc == ref.OK
    return st, parse(st)


# ----------------------------------------------------------------------------- worked example
def test_fig3_worked_example():
    g = golden("fig3_keys.txt")
    l = int(g["flag_bits"])
    keys = [5, 237, 300, 310, 500, 575, 578]          # deltas 5, 232, 63, 10, 190, 75, 3
    deltas = np.diff([0] + keys)
    assert deltas.max() == int(g["max_delta"]) and keys[-1] == int(g["last_key"])
    M, text = ref.key_tokens_text(keys, l)
    assert M == int(g["M"])
    toks = text.split(" ")
    assert toks[-1] == g["last_token"]                 # flag 00 then binary 11
    # the four flags cover [0,4) [4,16) [16,64) [64,256)
    uppers = [int(x) for x in g["range_upper_bounds"].split()]
    assert [1 << level_len(i, M, l) for i in range(1, 5)] == uppers
    for tok, dk in zip(toks, deltas):
        level = int(tok[:l], 2) + 1
        assert uppers[level - 1] > dk and (level == 1 or uppers[level - 2] <= dk)
        assert int(tok[l:], 2) == dk and len(tok) == l + level_len(level, M, l)
    # the container stores the same tokens (planar), one block
    st, info = all_survive(keys)
    assert info["keys"] == keys
    assert [(t[0], t[1], t[2]) for t in info["tokens"]] == \
        [(int(t[:l], 2) + 1, len(t) - l, int(t[l:], 2)) for t in toks]


# ----------------------------------------------------------------------------- token rules
@pytest.mark.parametrize("l", [1, 2, 3, 4, 5])
@pytest.mark.parametrize("seed", [0, 1])
def test_flag_is_smallest_level_that_fits(l, seed):
    rng = np.random.default_rng(seed * 10 + l)
    gaps = np.concatenate([rng.integers(1, 6, 500), rng.integers(1, 3000, 300), rng.integers(1, 2 ** 20, 50)])
    rng.shuffle(gaps)
    keys = np.cumsum(gaps) - 1
    st, info = all_survive(keys, ref.params(1.1, 128, l, 256))
    assert info["keys"] == list(keys)
    for level, ln, delta, M in info["tokens"]:
        assert bitlen(delta) <= ln == level_len(level, M, l)
        assert level == 1 or bitlen(delta) > level_len(level - 1, M, l)   # no smaller level fits


def test_M_for_powers_of_two_and_small_deltas():
    for delta, M in [(1, 1), (2, 2), (255, 8), (256, 9), (2 ** 31, 32), (2 ** 32 - 2, 32)]:
        st, info = all_survive([0, delta])
        assert info["tokens"][1][3] == M and info["keys"] == [0, delta]
    st, info = all_survive([0])                       # only delta 0: M = 1, level 1
    assert info["tokens"] == [(1, 1, 0, 1)]


@pytest.mark.parametrize("d", [1, 255, 256, 257, 512, 1000])
def test_block_boundaries_carry_prekey(d):
    rng = np.random.default_rng(d)
    keys = np.cumsum(rng.integers(1, 50, d))
    st, info = all_survive(keys, ref.params(1.1, 128, 2, 256))
    assert info["nb"] == -(-d // 256) and info["keys"] == list(keys)
    rc, k2, v2 = ref.decompress(st)
    assert rc == ref.OK and np.array_equal(k2, keys)


# ----------------------------------------------------------------------------- sizes (Section 3.4)
def key_bits(info):
    return sum(t[1] for t in info["tokens"]) + info["l"] * info["d"]


@pytest.mark.parametrize("l", [1, 2, 3])
def test_size_dense_all_survive(l):
    d = 5000
    st, info = all_survive(np.arange(d) + 1, ref.params(1.1, 128, l, 1024))
    assert key_bits(info) == d * (l + 1)              # every delta is 1: M = 1


@pytest.mark.parametrize("gap", [3, 8, 100, 1000])
def test_size_constant_gap(gap):
    d = 3000
    st, info = all_survive(np.arange(1, d + 1) * gap)
    assert key_bits(info) == d * (2 + bitlen(gap))
    # value plane: d bytes (Section 3.4), plus framing
    nb = info["nb"]
    words = sum(-(-min(1024, d - b * 1024) * 2 // 64) for b in range(nb)) + \
        sum(-(-sum(t[1] for t in info["tokens"][b * 1024:(b + 1) * 1024]) // 64) for b in range(nb))
    assert info["total"] == 64 + ((d + 7) & ~7) + 16 * nb + 8 * words


def test_size_uniform_gaps_close_to_paper_model():
    """Section 3.4: with evenly spread keys a delta costs about ceil(log2(D_m/d)) + l bits."""
    rng = np.random.default_rng(3)
    Dm, d, l = 10_000_000, 20_000, 2
    keys = np.sort(rng.choice(Dm, d, replace=False))
    st, info = all_survive(keys, ref.params(1.1, 128, l, 1024))
    per_key = key_bits(info) / d
    model = math.ceil(math.log2(Dm / d)) + l
    assert model - 1.5 <= per_key <= model + 1.5
    total_bits_model = 8 * d + d * model
    assert 0.85 * total_bits_model <= 8 * info["total"] <= 1.25 * total_bits_model
    assert info["total"] <= ref.compressed_size(d, ref.params(1.1, 128, l, 1024))


# ----------------------------------------------------------------------------- the size bound
def worst_case_bytes(n, tau, l, KB):
    """The bound of the container description, term by term: header, n value tokens of 1 + ceil(log2 tau)
    bits padded to 64-bit words, one 16-byte directory entry per block, and per block a flags plane of
    KB*l bits and a payload plane of KB*32 bits, each padded to 64-bit words."""
    w = 1 + (tau - 1).bit_length()
    nb = -(-n // KB)
    return 64 + 8 * (-(-(n * w) // 64)) + 16 * nb + nb * 8 * (-(-(KB * l) // 64) + -(-(KB * 32) // 64))


@pytest.mark.parametrize("KB", [256, 1024, 4096])
def test_size_bound_is_reached_by_a_block_of_longest_tokens(KB):
    """One full block, every element kept, l = 1: the first delta is 2^31 (M = 32, levels of 16 and 32 bits),
    every other delta is 2^16 and so takes the 32-bit level: every token costs l + 32 bits, which is the
    worst case the bound is made of.  The stream the encoder writes must fill the bound to the byte."""
    keys = (1 << 31) + (np.arange(KB, dtype=np.uint64) << 16)
    p = ref.params(1.1, 128, 1, KB)
    st, info = all_survive(keys, p)
    assert info["d"] == KB and info["nb"] == 1
    assert all(t[1] == 32 and t[3] == 32 for t in info["tokens"])
    assert info["total"] == len(st) == ref.compressed_size(KB, p) == worst_case_bytes(KB, 128, 1, KB)
    # one element more opens a second block: the bound grows by a whole worst-case block
    assert ref.compressed_size(KB + 1, p) == worst_case_bytes(KB + 1, 128, 1, KB) > info["total"] + 16 + 4 * KB


def test_size_bound_term_by_term_over_a_grid():
    for tau in (1, 2, 3, 64, 65, 128, 129, 200, 256):
        for l in (1, 2, 3, 4, 5):
            for KB in (256, 512, 1024, 2048, 4096):
                for n in (0, 1, 7, 8, 9, KB - 1, KB, KB + 1, 3 * KB, 3 * KB + 5, 1_000_003):
                    base = 1.1 if tau <= 128 else 1.05
                    assert ref.compressed_size(n, ref.params(base, tau, l, KB)) == worst_case_bytes(n, tau, l, KB), \
                        (n, tau, l, KB)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_no_stream_exceeds_the_size_bound(seed):
    """Keys drawn to make long tokens (large, uneven gaps), small blocks, every l."""
    rng = np.random.default_rng(seed)
    for l in (1, 2, 3, 4, 5):
        d = int(rng.integers(1, 2000))
        keys = np.sort(rng.choice(2 ** 32 - 1, d, replace=False))
        p = ref.params(1.1, 128, l, 256)
        st, info = all_survive(keys, p)
        assert info["d"] == d and len(st) <= ref.compressed_size(d, p)


# ----------------------------------------------------------------------------- round trip + errors
@pytest.mark.parametrize("seed,kb,l", [(0, 256, 2), (1, 1024, 1), (2, 4096, 5), (3, 512, 3)])
def test_round_trip_keys_lossless(seed, kb, l):
    rng = np.random.default_rng(seed)
    n = 30000
    keys = np.sort(rng.choice(2 ** 32 - 1, n, replace=False)).astype(np.uint32)
    v = rng.laplace(0, 1e-3, n).astype(np.float32)
    rc, st = ref.compress(keys, v, ref.params(1.09, 128, l, kb))
    assert rc == ref.OK
    info = parse(st)
    rc, k2, v2 = ref.decompress(st)
    assert rc == ref.OK and list(k2) == info["keys"] and 0 < info["d"] < n
    B, V = ref.tables(info["S"], 1.09, 128)
    keep = np.abs(v).view(np.uint32) >= B[128]
    assert np.array_equal(k2, keys[keep])              # decoded keys are the surviving keys, exactly


def test_unsorted_or_duplicate_surviving_keys_are_rejected():
    p = ref.params()
    v = np.full(4, BIG, np.float32)
    assert ref.compress([0, 5, 3, 9], v, p)[0] == ref.ERR_UNSORTED_KEYS
    assert ref.compress([1, 5, 5, 9], v, p)[0] == ref.ERR_UNSORTED_KEYS
    assert ref.compress([0, 5, 6, 9], v, p)[0] == ref.OK


def test_invalid_params_and_capacity():
    k, v = np.arange(100), np.full(100, BIG, np.float32)
    for bad in [ref.params(1.0), ref.params(17.0), ref.params(tau=0), ref.params(tau=257), ref.params(4.5, 129),
                ref.params(flag_bits=0), ref.params(flag_bits=6), ref.params(block_keys=128),
                ref.params(block_keys=1000), ref.params(block_keys=8192), ref.params(base=float("nan"))]:
        assert ref.compress(k, v, bad)[0] == ref.ERR_INVALID_ARG
    p = ref.params()
    rc, st = ref.compress(k, v, p)
    assert rc == ref.OK
    for cap in (0, 63, 64, 100, st.size - 1):
        assert ref.compress(k, v, p, capacity=cap)[0] == ref.ERR_BUFFER_TOO_SMALL
    assert ref.compress(k, v, p, capacity=st.size)[0] == ref.OK
    assert ref.decompress(st, capacity=99)[0] == ref.ERR_BUFFER_TOO_SMALL


def test_corrupt_streams_are_rejected():
    rng = np.random.default_rng(9)
    keys = np.cumsum(rng.integers(1, 100, 2000)).astype(np.uint32)
    rc, st = ref.compress(keys, np.full(2000, BIG, np.float32), ref.params(1.1, 100, 2, 256))
    assert rc == ref.OK and ref.decompress(st)[0] == ref.OK
    info = parse(st)
    dir_off = 64 + ((info["d"] + 7) & ~7)

    def broken(mut):
        s = st.copy()
        mut(s)
        return ref.decompress(s, capacity=4096)[0]

    def poke32(off, val):
        return lambda s: s.__setitem__(slice(off, off + 4), np.frombuffer(struct.pack("<I", val), np.uint8))

    def poke64(off, val):
        return lambda s: s.__setitem__(slice(off, off + 8), np.frombuffer(struct.pack("<Q", val), np.uint8))

    assert broken(lambda s: s.__setitem__(0, 0x58)) == ref.ERR_CORRUPT_STREAM          # magic
    assert broken(lambda s: s.__setitem__(4, 9)) == ref.ERR_CORRUPT_STREAM             # version
    assert broken(lambda s: s.__setitem__(5, 7)) == ref.ERR_CORRUPT_STREAM             # l
    assert broken(lambda s: s.__setitem__(6, 200)) == ref.ERR_CORRUPT_STREAM           # tau
    assert broken(poke32(8, 300)) == ref.ERR_CORRUPT_STREAM                            # block_keys
    assert broken(poke32(12, info["nb"] + 1)) == ref.ERR_CORRUPT_STREAM                # n_blocks
    assert broken(poke64(40, info["d"] + 1)) == ref.ERR_CORRUPT_STREAM                 # d vs directory
    assert broken(poke64(40, info["n"] + 1)) == ref.ERR_CORRUPT_STREAM                 # d > n
    assert broken(poke64(48, info["total"] + 8)) == ref.ERR_CORRUPT_STREAM             # total > bytes given
    assert broken(lambda s: s.__setitem__(64 + 5, 120)) == ref.ERR_CORRUPT_STREAM      # code > tau
    assert broken(poke32(dir_off + 16, 12345)) == ref.ERR_CORRUPT_STREAM               # block offset
    assert broken(poke32(dir_off + 16 + 4, 1)) == ref.ERR_CORRUPT_STREAM               # preKey chain
    assert broken(poke32(dir_off + 8, 33)) == ref.ERR_CORRUPT_STREAM                   # M
    assert broken(poke32(dir_off + 12, 17)) == ref.ERR_CORRUPT_STREAM                  # payload bits
    # a payload length one bit too long or too short that still rounds to the same number of words: only
    # the count of consumed bits can tell
    pbits0 = struct.unpack_from("<I", st, dir_off + 12)[0]
    assert pbits0 % 64 not in (0, 1)
    assert broken(poke32(dir_off + 12, pbits0 + 1)) == ref.ERR_CORRUPT_STREAM
    assert broken(poke32(dir_off + 12, pbits0 - 1)) == ref.ERR_CORRUPT_STREAM
    assert ref.decompress(st[:63])[0] == ref.ERR_CORRUPT_STREAM
    assert ref.decompress(st[:-8], capacity=4096)[0] == ref.ERR_CORRUPT_STREAM


def test_a_stream_that_repeats_a_key_is_rejected():
    """Eq. 4 is taken over the distinct, ascending keys of one gradient: a delta of 0 can only be the very first
    (key 0).  A stream whose tokens say otherwise is not one an encoder wrote."""
    keys = np.array([0, 3, 7, 20, 21, 300, 301, 5000], np.uint32)
    st, info = all_survive(keys, ref.params(1.1, 128, 2, 256))
    assert info["tokens"][0][2] == 0 and ref.decompress(st)[0] == ref.OK          # key 0: delta 0 at rank 0 is fine
    for rank in (1, 2, 4, 7):
        bad = with_zero_delta(st, rank)
        assert not np.array_equal(bad, st)
        assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM, rank
    # across a block boundary: first key of the second block equal to the last of the first
    keys = np.cumsum(np.full(300, 5)).astype(np.uint32)
    st, info = all_survive(keys, ref.params(1.1, 128, 2, 256))
    bad = with_zero_delta(st, 256)
    assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM      # (here the preKey chain notices as well)
    assert ref.decompress(with_zero_delta(st, 255))[0] == ref.ERR_CORRUPT_STREAM


# ----------------------------------------------------------------------------- segmented batch
def test_segmented_equals_independent_streams():
    rng = np.random.default_rng(21)
    sizes = [0, 1, 700, 5000, 3, 0, 2500]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = np.concatenate([rng.laplace(0, 10.0 ** -(i % 5 + 1), s) for i, s in enumerate(sizes)]).astype(np.float32)
    plist = [ref.params(1.04 + 0.01 * i, 128 - i, 1 + i % 3, 256 << (i % 3)) for i in range(len(sizes))]
    rc, blob, so = ref.compress_segmented(keys, vals, offs, plist)
    assert rc == ref.OK and so[0] == 0 and so[-1] == blob.size
    pos = 0
    for i, s in enumerate(sizes):
        a, b = int(offs[i]), int(offs[i + 1])
        rc1, st1 = ref.compress(keys[a:b], vals[a:b], plist[i])
        assert rc1 == ref.OK
        assert np.array_equal(blob[int(so[i]):int(so[i + 1])], st1)      # each stream stands alone
        assert int(so[i]) % 8 == 0
    cap = sum(sizes)
    rc, k2, v2, po = ref.decompress_segmented(blob, so, cap)
    assert rc == ref.OK
    for i in range(len(sizes)):
        rc1, k1, v1 = ref.decompress(blob[int(so[i]):int(so[i + 1])])
        assert np.array_equal(k2[int(po[i]):int(po[i + 1])], k1)
        assert np.array_equal(v2[int(po[i]):int(po[i + 1])], v1)
    # shared parameters
    rc, blob2, so2 = ref.compress_segmented(keys, vals, offs, plist[0])
    assert rc == ref.OK and parse(blob2[int(so2[3]):int(so2[4])])["tau"] == 128


def test_bits_per_key_against_flag_size_has_an_interior_minimum():
    # Table 6 (Section 4.2): on clustered keys the size per key first falls and then rises with l, smallest
    # at l = 2.  Synthetic stand-in for the paper's dataset: Zipf(1.2) gaps, 10 % of the pairs survive.
    from paper_2112_04291_amd import workloads as W
    w = W.config3(nnz=200_000, dim=2_000_000)
    b = W.solve_base(w.values, 0.1)
    bits = []
    for l in range(1, 6):
        rc, st = ref.compress(w.keys, w.values, ref.params(b, 128, l, 1024))
        assert rc == ref.OK
        d = int(st[40:48].view("<u8")[0])
        bits.append(8.0 * (st.size - 64 - ((d + 7) & ~7)) / d)
    assert bits[1] == min(bits)
    assert bits[0] > bits[1] < bits[2] < bits[3] < bits[4]
    assert all(x < 32.0 for x in bits)
