"""Pins for the oracle's decode-and-aggregate (Section 2.1 / Fig. 1: decoded gradients of all workers are
added up): against numpy's own scatter-adds of the separately decoded pairs, stream by stream."""
import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W


def worker_streams(n_workers, dim, nnz, keep, seed):
    rng = np.random.default_rng(seed)
    blobs, offs, pairs = [], [0], []
    for wkr in range(n_workers):
        keys = np.sort(rng.choice(dim, nnz, replace=False)).astype(np.uint32)
        vals = rng.laplace(0.0, 1e-3 * (wkr + 1), nnz).astype(np.float32)
        rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, keep), 128, 2, 256))
        assert rc == ref.OK
        rc, k, v = ref.decompress(st)
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
        pairs.append((k, v))
    return np.concatenate(blobs), np.array(offs, np.uint64), pairs


@pytest.mark.parametrize("n_workers", [1, 2, 5])
def test_aggregate_equals_scatter_adds_in_stream_order(n_workers):
    dim = 200_000
    blob, offs, pairs = worker_streams(n_workers, dim, 30_000, 0.3, 100 + n_workers)
    dense = np.full(dim, 0.125, np.float32)
    expect = dense.copy()
    for k, v in pairs:                              # keys are unique inside a stream: a plain fancy-index add
        assert np.all(np.diff(k.astype(np.int64)) > 0)
        expect[k] = expect[k] + v                   # binary32 additions, stream after stream
    rc, cnt = ref.decompress_accumulate(blob, offs, dense)
    assert rc == ref.OK and cnt == sum(k.size for k, _ in pairs)
    assert np.array_equal(dense.view(np.uint32), expect.view(np.uint32))
    untouched = np.ones(dim, bool)
    for k, _ in pairs:
        untouched[k] = False
    assert np.all(dense[untouched] == np.float32(0.125))


def test_aggregate_order_matters_only_in_the_last_bits_and_sum_is_conserved():
    dim = 50_000
    blob, offs, pairs = worker_streams(4, dim, 20_000, 0.5, 7)
    dense = np.zeros(dim, np.float32)
    rc, cnt = ref.decompress_accumulate(blob, offs, dense)
    assert rc == ref.OK
    total = sum(float(v.astype(np.float64).sum()) for _, v in pairs)
    assert abs(float(dense.astype(np.float64).sum()) - total) <= 1e-6 * sum(float(np.abs(v).sum()) for _, v in pairs)


def test_aggregate_rejects_keys_beyond_the_dense_array_and_corrupt_streams():
    blob, offs, pairs = worker_streams(2, 10_000, 2_000, 0.5, 9)
    top = max(int(k.max()) for k, _ in pairs)
    dense = np.zeros(top, np.float32)               # one short
    assert ref.decompress_accumulate(blob, offs, dense)[0] == ref.ERR_BUFFER_TOO_SMALL
    dense = np.zeros(top + 1, np.float32)
    assert ref.decompress_accumulate(blob, offs, dense)[0] == ref.OK
    bad = blob.copy()
    bad[int(offs[1])] ^= 0xFF                       # magic of the second stream
    assert ref.decompress_accumulate(bad, offs, np.zeros(top + 1, np.float32))[0] == ref.ERR_CORRUPT_STREAM
    assert ref.decompress_accumulate(blob[:0], np.array([0], np.uint64), dense) == (ref.OK, 0)
