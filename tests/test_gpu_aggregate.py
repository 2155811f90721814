"""GPU parity of decode-and-aggregate against the oracle: bit-identical dense sums (the additions happen
stream after stream on both sides), same status on errors."""
import numpy as np
import pytest

from oracle import ref
from tests.test_oracle_aggregate import worker_streams

pytestmark = pytest.mark.gpu


def hip_accumulate(blob, offs, dense):
    import torch
    from paper_2112_04291_amd import binding as B
    n = len(offs) - 1
    s = np.ascontiguousarray(blob, dtype=np.uint8)
    dev = torch.from_numpy(np.concatenate([s, np.zeros((-s.size) % 8 + 8, np.uint8)])).cuda()
    so = torch.from_numpy(np.ascontiguousarray(offs, dtype=np.uint64).view(np.int64)).cuda()
    dd = torch.from_numpy(dense.copy()).cuda()
    count = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(n)
    rc = B.decompress_accumulate(dev, s.size, so, n, dd, count, status, ws)
    torch.cuda.synchronize()
    return rc, int(status[0]), int(count[0]), dd.cpu().numpy()


@pytest.mark.parametrize("n_workers,dim,nnz,keep", [(1, 100_000, 20_000, 0.5), (3, 400_000, 150_000, 0.3),
                                                    (8, 2_000_000, 300_000, 0.05), (2, 5_000, 5_000, 1.0),
                                                    (48, 500_000, 40_000, 0.2)])
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
