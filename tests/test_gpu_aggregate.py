"""GPU parity of decode-and-aggregate against the oracle: bit-identical dense sums (the additions happen
stream after stream on both sides), same status on errors."""
import numpy as np
import pytest

from oracle import ref
from tests.test_oracle_aggregate import worker_streams

pytestmark = pytest.mark.gpu


def hip_accumulate(blob, offs, dense, shift=0):
    """`shift`: the dense vector starts that many elements into its allocation (1: not 16-byte aligned)."""
    import torch
    from paper_2112_04291_amd import binding as B
    n = len(offs) - 1
    s = np.ascontiguousarray(blob, dtype=np.uint8)
    dev = torch.from_numpy(np.concatenate([s, np.zeros((-s.size) % 8 + 8, np.uint8)])).cuda()
    so = torch.from_numpy(np.ascontiguousarray(offs, dtype=np.uint64).view(np.int64)).cuda()
    dd = torch.from_numpy(np.concatenate([np.zeros(shift, np.float32), dense])).cuda()[shift:]
    count = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(n)
    rc = B.decompress_accumulate(dev, s.size, so, n, dd, count, status, ws)
    torch.cuda.synchronize()
    return rc, int(status[0]), int(count[0]), dd.cpu().numpy()


@pytest.mark.parametrize("n_workers,dim,nnz,keep", [(1, 100_000, 20_000, 0.5), (3, 400_000, 150_000, 0.3),
                                                    (8, 2_000_000, 300_000, 0.05), (2, 5_000, 5_000, 1.0),
                                                    (48, 500_000, 40_000, 0.2), (4, 4_000_000, 20_000, 0.5)])
def test_aggregate_matches_oracle_bit_for_bit(n_workers, dim, nnz, keep):
    from paper_2112_04291_amd import binding as B
    blob, offs, pairs = worker_streams(n_workers, dim, nnz, keep, 300 + n_workers)
    rng = np.random.default_rng(5)
    dense0 = rng.standard_normal(dim).astype(np.float32) * np.float32(1e-3)
    want = dense0.copy()
    rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
    assert rc_ref == ref.OK
    rc, status, cnt, got = hip_accumulate(blob, offs, dense0)
    assert rc == B.OK and status == 0 and cnt == cnt_ref
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_aggregate_into_a_vector_that_is_not_16_byte_aligned():
    """Such a vector is added to stream after stream, whatever the streams hold (the one-pass form moves 16-byte
    pieces of it)."""
    from paper_2112_04291_amd import binding as B
    blob, offs, pairs = worker_streams(3, 300_001, 120_000, 0.6, 17)
    rng = np.random.default_rng(9)
    dense0 = rng.standard_normal(300_001).astype(np.float32) * np.float32(1e-3)
    want = dense0.copy()
    rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
    assert rc_ref == ref.OK
    for shift in (1, 2, 3):
        rc, status, cnt, got = hip_accumulate(blob, offs, dense0, shift=shift)
        assert rc == B.OK and status == 0 and cnt == cnt_ref
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


def test_aggregate_errors_match_oracle():
    from paper_2112_04291_amd import binding as B
    blob, offs, pairs = worker_streams(3, 50_000, 10_000, 0.5, 11)
    top = max(int(k.max()) for k, _ in pairs)
    short = np.zeros(top, np.float32)
    assert ref.decompress_accumulate(blob, offs, short.copy())[0] == ref.ERR_BUFFER_TOO_SMALL
    rc, status, cnt, _ = hip_accumulate(blob, offs, short)
    assert rc == B.OK and status == B.ERR_BUFFER_TOO_SMALL and cnt == 0
    bad = blob.copy()
    bad[int(offs[2]) + 4] ^= 0x7                     # version byte of the third stream
    assert ref.decompress_accumulate(bad, offs, np.zeros(top + 1, np.float32))[0] == ref.ERR_CORRUPT_STREAM
    rc, status, cnt, _ = hip_accumulate(bad, offs, np.zeros(top + 1, np.float32))
    assert rc == B.OK and status == B.ERR_CORRUPT_STREAM and cnt == 0


def test_aggregate_rejects_a_stream_that_repeats_a_key():
    from paper_2112_04291_amd import binding as B
    from tests.streamparse import with_zero_delta
    blob, offs, pairs = worker_streams(3, 50_000, 10_000, 0.5, 12)
    top = max(int(k.max()) for k, _ in pairs)
    second = blob[int(offs[1]):int(offs[2])]
    for rank in (1, 700, pairs[1][0].size - 1):
        bad = blob.copy()
        bad[int(offs[1]):int(offs[2])] = with_zero_delta(second, rank)
        assert ref.decompress_accumulate(bad, offs, np.zeros(top + 1, np.float32))[0] == ref.ERR_CORRUPT_STREAM
        rc, status, cnt, _ = hip_accumulate(bad, offs, np.zeros(top + 1, np.float32))
        assert rc == B.OK and status == B.ERR_CORRUPT_STREAM and cnt == 0, rank


def test_aggregate_of_streams_with_narrow_and_nine_bit_tokens():
    from paper_2112_04291_amd import binding as B
    from paper_2112_04291_amd import workloads as W
    rng = np.random.default_rng(8)
    dim, blobs, offs = 300_000, [], [0]
    for tau in (16, 128, 5, 200, 256):
        keys = np.sort(rng.choice(dim, 60_000, replace=False)).astype(np.uint32)
        vals = (rng.laplace(0.0, 1e-3, keys.size) * np.exp(rng.uniform(-8, 0, keys.size))).astype(np.float32)
        vals[::5000] *= np.float32(1e3)
        rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, 0.4, tau), tau, 2, 512))
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
    blob, offs = np.concatenate(blobs), np.array(offs, np.uint64)
    want = np.zeros(dim, np.float32)
    rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
    assert rc_ref == ref.OK and cnt_ref > 100
    rc, status, cnt, got = hip_accumulate(blob, offs, np.zeros(dim, np.float32))
    assert rc == B.OK and status == 0 and cnt == cnt_ref
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))


# --- dense gradients: the library adds them in one pass over the dense vector (groups of eight streams, a
# tile of 16384 keys at a time, runs of tiles per workgroup); the cases below are sized so that this form is
# the one that runs (the streams' bytes, times ten, reach the vector's length per group of eight), with
# vectors that end inside a tile and inside a 16-byte piece, blocks of one to four rounds, partial groups

def dense_streams(n_workers, dim, nnz, keep, kb, seed, taus=(128,)):
    from paper_2112_04291_amd import workloads as W
    rng = np.random.default_rng(seed)
    blobs, offs = [], [0]
    for wkr in range(n_workers):
        keys = np.sort(rng.choice(dim, nnz, replace=False)).astype(np.uint32)
        vals = rng.laplace(0.0, 1e-3 * (wkr + 1), nnz).astype(np.float32)
        tau = taus[wkr % len(taus)]
        rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, keep, tau), tau, 1 + wkr % 4, kb))
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
    blob, offs = np.concatenate(blobs), np.array(offs, np.uint64)
    assert 10 * blob.size >= dim * (-(-n_workers // 8)) and n_workers >= 2      # (the library's own test for this form)
    return blob, offs


def check_against_oracle(blob, offs, dense0):
    from paper_2112_04291_amd import binding as B
    want = dense0.copy()
    rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
    rc, status, cnt, got = hip_accumulate(blob, offs, dense0)
    assert rc == B.OK and status == rc_ref
    if rc_ref == ref.OK:
        assert cnt == cnt_ref
        assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
    else:
        assert cnt == 0
    return rc_ref


@pytest.mark.parametrize("n_workers,dim,nnz,keep,kb", [(9, 200_003, 120_000, 0.5, 1024), (4, 150_001, 100_000, 0.9, 4096),
                                                       (8, 70_000, 60_000, 1.0, 1024), (3, 3 * 16384, 30_000, 0.6, 2048),
                                                       (2, 16_385, 9_000, 0.7, 1024), (17, 1_000_000, 400_000, 0.25, 1024),
                                                       (5, 2_000_002, 1_500_000, 0.8, 1024)])
def test_aggregate_in_one_pass_matches_oracle_bit_for_bit(n_workers, dim, nnz, keep, kb):
    blob, offs = dense_streams(n_workers, dim, nnz, keep, kb, 900 + n_workers, taus=(128, 16, 200))
    rng = np.random.default_rng(6)
    dense0 = rng.standard_normal(dim).astype(np.float32) * np.float32(1e-3)
    assert check_against_oracle(blob, offs, dense0) == ref.OK


def test_aggregate_in_one_pass_reports_keys_beyond_the_vector():
    blob, offs = dense_streams(3, 300_000, 200_000, 0.8, 1024, 21)
    for short in (299_000, 150_000, 20_000, 1):            # the last: every key but key 0 lies beyond
        assert check_against_oracle(blob, offs, np.zeros(short, np.float32)) == ref.ERR_BUFFER_TOO_SMALL


def test_aggregate_in_one_pass_rejects_damaged_streams():
    import struct
    from tests.streamparse import parse
    blob, offs = dense_streams(3, 120_000, 60_000, 0.9, 2048, 22)
    a, b = int(offs[1]), int(offs[2])
    info = parse(blob[a:b])
    dir_off = 64 + 8 * (-(-(info["d"] * info["w"]) // 64))
    assert info["nb"] >= 8
    cases = []
    for blk in (1, info["nb"] // 2, info["nb"] - 1):
        bad = blob.copy()                                  # a directory whose preKeys do not rise
        pre = struct.unpack_from("<I", bad, a + dir_off + 16 * blk + 4)[0]
        struct.pack_into("<I", bad, a + dir_off + 16 * blk + 4, struct.unpack_from("<I", bad, a + dir_off + 16 * (blk - 1) + 4)[0])
        cases.append(bad)
        bad = blob.copy()                                  # a preKey that is off by one
        struct.pack_into("<I", bad, a + dir_off + 16 * blk + 4, pre + 1)
        cases.append(bad)
        bad = blob.copy()                                  # payload bits of the block one short
        pb = struct.unpack_from("<I", bad, a + dir_off + 16 * blk + 12)[0]
        struct.pack_into("<I", bad, a + dir_off + 16 * blk + 12, pb - 1)
        cases.append(bad)
    bad = blob.copy()
    bad[a + 64] |= 0x7F                                    # a code beyond tau... or not: the oracle says which
    cases.append(bad)
    for rank in (1, 3000, info["d"] - 1):
        from tests.streamparse import with_zero_delta
        bad = blob.copy()
        bad[a:b] = with_zero_delta(blob[a:b], rank)
        cases.append(bad)
    n_bad = 0
    for bad in cases:
        n_bad += check_against_oracle(bad, offs, np.zeros(120_000, np.float32)) == ref.ERR_CORRUPT_STREAM
    assert n_bad >= len(cases) - 1
    # damaged behind the end of a vector that is too short as well: corrupt is what is reported (the first
    # stream here: the oracle stops at the first stream that fails, the library reports the gravest failure)
    first = parse(blob[:int(offs[1])])
    dir0 = 64 + 8 * (-(-(first["d"] * first["w"]) // 64))
    bad = blob.copy()
    struct.pack_into("<I", bad, dir0 + 16 * (first["nb"] - 1) + 12, 0)
    assert check_against_oracle(bad, offs, np.zeros(60_000, np.float32)) == ref.ERR_CORRUPT_STREAM


def test_aggregate_in_one_pass_of_uneven_streams():
    """Streams that are empty, that end early, that start late, that hold a single pair: every wave still passes
    every tile."""
    from paper_2112_04291_amd import workloads as W
    rng = np.random.default_rng(31)
    dim = 200_000
    spans = [(0, dim), (0, 0), (150_000, dim), (0, 30_000), (99_999, 100_000), (0, dim), (60_000, 61_000)]
    blobs, offs = [], [0]
    for lo, hi in spans:
        keys = np.arange(lo, hi, dtype=np.uint32)
        keys = keys[rng.random(keys.size) < 0.7]
        vals = rng.laplace(0.0, 1e-3, keys.size).astype(np.float32)
        base = W.solve_base(vals, 0.9) if keys.size else 1.5
        rc, st = ref.compress(keys, vals, ref.params(base, 128, 2, 1024))
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
    blob, offs = np.concatenate(blobs), np.array(offs, np.uint64)
    assert 10 * blob.size >= dim
    dense0 = rng.standard_normal(dim).astype(np.float32)
    assert check_against_oracle(blob, offs, dense0) == ref.OK


def test_aggregate_in_one_pass_keeps_denormal_sums():
    """Gradients so small that the sums are denormal: added as binary32 denormals, not flushed."""
    from paper_2112_04291_amd import workloads as W
    rng = np.random.default_rng(32)
    dim = 100_000
    blobs, offs = [], [0]
    for wkr in range(4):
        keys = np.sort(rng.choice(dim, 60_000, replace=False)).astype(np.uint32)
        vals = (rng.laplace(0.0, 1.0, keys.size) * 1e-41).astype(np.float32)
        assert np.count_nonzero(vals) > 50_000 and np.abs(vals).max() < 1.2e-38
        rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, 0.9), 128, 2, 1024))
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
    blob, offs = np.concatenate(blobs), np.array(offs, np.uint64)
    assert 10 * blob.size >= dim
    want = np.zeros(dim, np.float32)
    assert ref.decompress_accumulate(blob, offs, want)[0] == ref.OK
    tiny = np.abs(want[want != 0])
    assert tiny.size > 50_000 and tiny.max() < 1.2e-38           # the sums are denormal
    assert check_against_oracle(blob, offs, np.zeros(dim, np.float32)) == ref.OK
