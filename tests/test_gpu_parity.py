"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Bar: the compressed stream is byte-identical; decoded keys are identical; decoded values are
within 1e-6 relative of the oracle's decode (in practice identical bit patterns)."""
import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W

pytestmark = pytest.mark.gpu

REL_TOL = 1e-6


def _gpu():
    import torch
    from paper_2112_04291_amd import binding as B
    from tests import gpu_util as G
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch, B, G


def check_round_trip(keys, values, base, tau=128, l=2, kb=1024, expect_status=0):
    torch, B, G = _gpu()
    keys = np.ascontiguousarray(keys, dtype=np.uint32)
    values = np.ascontiguousarray(values, dtype=np.float32)
    rc_ref, st_ref = ref.compress(keys, values, ref.params(base, tau, l, kb))
    rc, status, st, _ = G.hip_compress(keys, values, B.params(base, tau, l, kb))
    assert rc == B.OK
    assert status == rc_ref == expect_status, (status, rc_ref)
    if expect_status != 0:
        assert st.size == 0
        return None
    assert st.size == st_ref.size, (st.size, st_ref.size)
    if not np.array_equal(st, st_ref):
        bad = np.flatnonzero(st != st_ref)
        raise AssertionError(f"stream differs at {bad.size} bytes, first at {bad[:8]} of {st.size}; "
                             f"header hip={st[:64].tolist()} ref={st_ref[:64].tolist()}")
    d = int(st_ref[40:48].view("<u8")[0])
    rc_ref, k_ref, v_ref = ref.decompress(st_ref)
    rc, status, k, v = G.hip_decompress(st_ref, capacity=d)
    assert rc == B.OK and status == 0 and rc_ref == 0
    assert np.array_equal(k, k_ref)
    assert v.size == v_ref.size
    if d:
        assert np.all(np.abs(v.astype(np.float64) - v_ref.astype(np.float64)) <= REL_TOL * np.abs(v_ref.astype(np.float64)))
        assert np.array_equal(np.signbit(v), np.signbit(v_ref))
    return st


@pytest.mark.parametrize("n", [0, 1, 3, 255, 4095, 4096, 4097, 10_000, 70_001])
def test_small_sizes_and_ragged_tails(n):
    w = W.small_mixture(100 + n, n)
    b = W.solve_base(w.values, 0.2) if n else 1.1
    check_round_trip(w.keys, w.values, b)


@pytest.mark.parametrize("keep", [1.0, 0.5, 0.1, 0.01, 0.001])
def test_survival_fractions(keep):
    w = W.small_mixture(7, 300_000)
    check_round_trip(w.keys, w.values, W.solve_base(w.values, keep))


@pytest.mark.parametrize("tau,l,kb", [(128, 1, 256), (128, 3, 512), (100, 4, 2048), (64, 5, 4096), (1, 2, 1024),
                                      (17, 2, 256)])
def test_parameter_grid(tau, l, kb):
    w = W.small_mixture(11, 200_000)
    check_round_trip(w.keys, w.values, W.solve_base(w.values, 0.3, tau), tau, l, kb)


def test_config1_tiny_sparse_gradient():
    w = W.config1()
    st = check_round_trip(w.keys, w.values, W.solve_base(w.values, 0.10))
    d = int(st[40:48].view("<u8")[0])
    assert 0.09 * w.values.size <= d <= 0.11 * w.values.size
    # the paper's own defaults (b = 1.1) with a smaller tau that keeps about a tenth
    check_round_trip(w.keys, w.values, 1.1, tau=112)


def test_all_survive_and_none_survive():
    n = 50_000
    keys = np.arange(n, dtype=np.uint32) * 3
    check_round_trip(keys, np.full(n, 1.0, np.float32), 1.1)                 # everything kept, dense codes
    vals = np.full(n, 1e-3, np.float32)
    check_round_trip(keys, vals, 1.0 + 2.0 ** -19)                           # b^tau ~ 1: nothing reaches sum
    check_round_trip(keys, np.zeros(n, np.float32), 1.1)                     # all-zero gradient: d = 0
    one = np.zeros(n, np.float32)
    one[12345] = -2.5
    check_round_trip(keys, one, 1.1)                                         # one element is the whole sum


def test_wide_exponent_range_exact_sum():
    rng = np.random.default_rng(5)
    n = 123_457
    e = rng.integers(0, 255, n).astype(np.uint32)
    m = rng.integers(0, 1 << 23, n).astype(np.uint32)
    s = rng.integers(0, 2, n).astype(np.uint32)
    vals = ((s << 31) | (e << 23) | m).view(np.float32)
    keys = np.sort(rng.choice(2 ** 32 - 1, n, replace=False)).astype(np.uint32)
    check_round_trip(keys, vals, 1.9)
    check_round_trip(keys, vals, 16.0, tau=128, l=5, kb=256)
    # denormals only
    dn = rng.integers(1, 1 << 23, 20_000).astype(np.uint32).view(np.float32)
    check_round_trip(np.arange(20_000), dn, 1.07)


@pytest.mark.parametrize("badval", [np.nan, np.inf, -np.inf])
def test_nonfinite_input_is_reported(badval):
    w = W.small_mixture(3, 20_000)
    v = w.values.copy()
    v[17_123] = badval
    check_round_trip(w.keys, v, 1.1, expect_status=ref.ERR_NONFINITE)


def test_unsorted_surviving_keys_are_reported():
    n = 10_000
    keys = np.arange(n, dtype=np.uint32)
    keys[5000], keys[5001] = keys[5001], keys[5000]
    check_round_trip(keys, np.full(n, 1.0, np.float32), 1.1, expect_status=ref.ERR_UNSORTED_KEYS)
    keys = np.arange(n, dtype=np.uint32)
    keys[77] = keys[76]
    check_round_trip(keys, np.full(n, 1.0, np.float32), 1.1, expect_status=ref.ERR_UNSORTED_KEYS)


def test_which_status_wins_when_several_conditions_hold():
    """Non-finite input before keys out of order before a buffer too small; the sequential oracle reports
    whichever of the last two it meets first, so its verdict is only required to be one of them."""
    torch, B, G = _gpu()
    rng = np.random.default_rng(3)
    n = 20_000
    keys = np.cumsum(rng.integers(1, 9, n)).astype(np.uint32)
    vals = rng.laplace(0, 1e-3, n).astype(np.float32)
    p, rp = B.params(16.0), ref.params(16.0)                    # b^tau is huge: everything survives
    swapped = keys.copy()
    swapped[[15_000, 15_001]] = swapped[[15_001, 15_000]]
    small = 64 + 4096                                           # holds the header, not the stream
    rc, status, st, _ = G.hip_compress(swapped, vals, p, out_capacity=small)
    assert rc == B.OK and status == B.ERR_UNSORTED_KEYS and st.size == 0
    assert ref.compress(swapped, vals, rp, capacity=small)[0] in (ref.ERR_UNSORTED_KEYS, ref.ERR_BUFFER_TOO_SMALL)
    bad = vals.copy()
    bad[7] = np.inf
    rc, status, st, _ = G.hip_compress(swapped, bad, p, out_capacity=small)
    assert rc == B.OK and status == B.ERR_NONFINITE and st.size == 0
    assert ref.compress(swapped, bad, rp, capacity=small)[0] == ref.ERR_NONFINITE
    rc, status, st, _ = G.hip_compress(keys, vals, p, out_capacity=small)
    assert rc == B.OK and status == B.ERR_BUFFER_TOO_SMALL and st.size == 0
    assert ref.compress(keys, vals, rp, capacity=small)[0] == ref.ERR_BUFFER_TOO_SMALL


def test_output_capacity_is_respected():
    torch, B, G = _gpu()
    w = W.small_mixture(21, 100_000)
    b = W.solve_base(w.values, 0.5)
    rc_ref, st_ref = ref.compress(w.keys, w.values, ref.params(b))
    for cap in [64, 64 + 1000, st_ref.size - 8, st_ref.size]:
        bufs = B.Buffers(w.values.size, B.params(b), out_capacity=st_ref.size + 4096)
        guard = bufs.out_bytes_view()
        guard.fill_(0xAB)
        bufs.out_capacity = cap
        rc, status, st, _ = G.hip_compress(w.keys, w.values, B.params(b), bufs=bufs)
        assert rc == B.OK
        after = guard.cpu().numpy()
        assert np.all(after[cap:] == 0xAB), "wrote past the stated capacity"
        if cap >= st_ref.size:
            assert status == 0 and np.array_equal(st, st_ref)
        else:
            assert status == B.ERR_BUFFER_TOO_SMALL and st.size == 0
    assert G.hip_compress(w.keys, w.values, B.params(b), out_capacity=32)[0] == B.ERR_BUFFER_TOO_SMALL


def test_unaligned_input_pointers():
    torch, B, G = _gpu()
    w = W.small_mixture(31, 50_001)
    b = W.solve_base(w.values, 0.3)
    for shift in (1, 2, 3):
        keys, vals = w.keys[shift:], w.values[shift:]
        rc_ref, st_ref = ref.compress(keys, vals, ref.params(b))
        k = G.to_dev_u32(w.keys)[shift:]
        v = G.to_dev_f32(w.values)[shift:]
        bufs = B.Buffers(vals.size, B.params(b))
        rc = B.compress(k, v, B.params(b), bufs.out, bufs.out_offsets, bufs.status, bufs.workspace, n=vals.size,
                        out_capacity=bufs.out_capacity)
        torch.cuda.synchronize()
        assert rc == B.OK and int(bufs.status[0]) == 0
        nbytes = int(bufs.out_offsets[0])
        assert np.array_equal(bufs.out_bytes_view()[:nbytes].cpu().numpy(), st_ref)


def test_repeated_calls_are_deterministic_and_reuse_workspace():
    torch, B, G = _gpu()
    w = W.small_mixture(41, 400_000)
    b = W.solve_base(w.values, 0.05)
    bufs = B.Buffers(w.values.size, B.params(b))
    first = None
    for it in range(10):
        rc, status, st, _ = G.hip_compress(w.keys, w.values, B.params(b), bufs=bufs)
        assert rc == B.OK and status == 0
        if first is None:
            first = st
            assert np.array_equal(st, ref.compress(w.keys, w.values, ref.params(b))[1])
        else:
            assert np.array_equal(st, first)


def test_corrupt_streams_are_rejected_on_device():
    torch, B, G = _gpu()
    import struct
    rng = np.random.default_rng(9)
    keys = np.cumsum(rng.integers(1, 100, 2000)).astype(np.uint32)
    rc, st = ref.compress(keys, np.full(2000, 1.0, np.float32), ref.params(1.1, 100, 2, 256))
    assert rc == 0
    d = 2000
    dir_off = 64 + ((d + 7) & ~7)

    def run(mut, cap=4096):
        s = st.copy()
        mut(s)
        rc_ref = ref.decompress(s, capacity=cap)[0]
        rc, status, k, v = G.hip_decompress(s, capacity=cap)
        assert rc == B.OK
        assert status == rc_ref, (status, rc_ref)
        if status != 0:
            assert k.size == 0
        return status

    def poke(off, fmt, val):
        return lambda s: s.__setitem__(slice(off, off + struct.calcsize(fmt)), np.frombuffer(struct.pack(fmt, val), np.uint8))

    assert run(lambda s: None) == 0
    for mut in [poke(0, "<B", 0x58), poke(4, "<B", 9), poke(5, "<B", 7), poke(6, "<B", 200), poke(8, "<I", 300),
                poke(12, "<I", 9), poke(40, "<Q", d + 1), poke(40, "<Q", 10 ** 12), poke(48, "<Q", st.size + 8),
                poke(64 + 5, "<B", 120), poke(dir_off + 16, "<I", 12345), poke(dir_off + 16, "<I", 0xFFFFFFF0),
                poke(dir_off + 16 + 4, "<I", 1), poke(dir_off + 8, "<I", 33), poke(dir_off + 12, "<I", 17),
                poke(dir_off + 12, "<I", 0xFFFFFFFF)]:
        assert run(mut) == B.ERR_CORRUPT_STREAM
    # a payload length off by one bit that still rounds to the same number of words
    pbits0 = struct.unpack_from("<I", st, dir_off + 12)[0]
    assert pbits0 % 64 not in (0, 1)
    assert run(poke(dir_off + 12, "<I", pbits0 + 1)) == B.ERR_CORRUPT_STREAM
    assert run(poke(dir_off + 12, "<I", pbits0 - 1)) == B.ERR_CORRUPT_STREAM
    assert run(lambda s: None, cap=1999) == B.ERR_BUFFER_TOO_SMALL
    rc, status, k, v = G.hip_decompress(st[:48], capacity=10)
    assert status == B.ERR_CORRUPT_STREAM


def test_a_stream_that_repeats_a_key_is_rejected_on_device():
    """A delta of 0 anywhere but at the stream's first key (Eq. 4 is over distinct keys): same verdict as
    the oracle, at the first key of a lane, inside a lane, at a round's and a block's first key."""
    torch, B, G = _gpu()
    from tests.streamparse import with_zero_delta
    rng = np.random.default_rng(77)
    keys = np.concatenate([[0], np.cumsum(rng.integers(1, 60, 5000))]).astype(np.uint32)
    rc, st = ref.compress(keys, np.full(keys.size, 1.0, np.float32), ref.params(1.1, 128, 2, 2048))
    assert rc == 0 and ref.decompress(st)[0] == ref.OK
    rc, status, k, v = G.hip_decompress(st, capacity=keys.size)
    assert status == 0 and np.array_equal(k, keys)          # key 0 first: a delta of 0 at rank 0 is fine
    for rank in (1, 15, 16, 17, 1023, 1024, 2047, 2048, 2049, 4999, 5000):
        bad = with_zero_delta(st, rank)
        assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM
        rc, status, k, v = G.hip_decompress(bad, capacity=keys.size)
        assert rc == B.OK and status == B.ERR_CORRUPT_STREAM and k.size == 0, rank


def test_decoder_workspace_is_left_clear_after_every_call():
    """The decoder's control words are cleared once and must come back clear from every call, also from one
    that fails: good, corrupt, too small, good again on ONE workspace, every verdict the oracle's."""
    torch, B, G = _gpu()
    from tests.streamparse import with_zero_delta
    rng = np.random.default_rng(5)
    n = 300_000
    keys = np.cumsum(rng.integers(1, 9, n)).astype(np.uint32)
    vals = rng.laplace(0, 1e-3, n).astype(np.float32)
    rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, 0.3, 100), 100))
    assert rc == 0
    rc_ref, k_ref, v_ref = ref.decompress(st)
    d = k_ref.size
    bad = st.copy()
    bad[64 + 16 * (d // 32)] |= 0x7F                          # code 128 > tau = 100 in the middle of the value plane
    assert ref.decompress(bad)[0] == ref.ERR_CORRUPT_STREAM
    ws = B.decoder_workspace(1)
    keys_out = torch.empty(d, dtype=torch.int32, device="cuda")
    vals_out = torch.empty(d, dtype=torch.float32, device="cuda")
    count = torch.zeros(2, dtype=torch.int64, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")

    def run(stream, cap):
        dev = torch.from_numpy(np.concatenate([stream, np.zeros((-stream.size) % 8 + 8, np.uint8)])).cuda()
        count.fill_(-1)
        status.fill_(-1)
        assert B.decompress(dev, stream.size, keys_out, vals_out, count, status, ws, capacity=cap) == B.OK
        torch.cuda.synchronize()
        return int(status[0]), int(count[0])

    for _ in range(2):
        assert run(st, d) == (0, d)
        assert np.array_equal(keys_out.cpu().numpy().view(np.uint32), k_ref)
        assert run(bad, d) == (B.ERR_CORRUPT_STREAM, 0)
        assert run(st, d - 1) == (B.ERR_BUFFER_TOO_SMALL, 0)
        assert run(st[:40], d) == (B.ERR_CORRUPT_STREAM, 0)
        assert run(with_zero_delta(st, d - 1), d) == (B.ERR_CORRUPT_STREAM, 0)
    assert run(st, d) == (0, d)
    assert not ws[:512].any()                                 # the 4096 bytes of control words


def test_values_on_bucket_boundaries_and_granule_bounds():
    """Elements exactly on, one ulp below and one ulp above every boundary (exact powers of two by
    construction), scattered so that many granules (32 values, the unit the value pass skips by) hold a single borderline element: the row-skip
    bounds and the boundary table must agree with the oracle to the last bit."""
    from tests.test_oracle_values import boundary_gradient
    keys, vals, codes, kept = boundary_gradient(10)
    st = check_round_trip(keys, vals, 2.0, tau=10, l=2, kb=256)
    d = int(st[40:48].view("<u8")[0])
    assert d == int(kept.sum())
    # sparse variant: the borderline elements far apart, everything else far below the threshold
    rng = np.random.default_rng(8)
    n = 600_000
    v = np.zeros(n, np.float32)
    pos = np.sort(rng.choice(n, vals.size, replace=False))
    v[pos] = vals
    check_round_trip(np.arange(n, dtype=np.uint32), v, 2.0, tau=10, l=3, kb=1024)


def _spikes(n, pos, seed):
    """Background far below any threshold, survivors of magnitude about one at `pos`."""
    rng = np.random.default_rng(seed)
    v = (rng.uniform(1e-9, 1e-8, n) * rng.choice([-1.0, 1.0], n)).astype(np.float32)
    pos = np.unique(np.asarray(pos, dtype=np.int64))
    pos = pos[(pos >= 0) & (pos < n)]
    v[pos] = (rng.uniform(0.5, 2.0, pos.size) * rng.choice([-1.0, 1.0], pos.size)).astype(np.float32)
    return v, pos


@pytest.mark.parametrize("pattern", ["same_quarter_of_every_row", "every_17th_quarter", "ends_only", "one_row_in_300",
                                     "quarter_edges", "dense_island_in_a_desert", "last_quarter_only",
                                     "same_eighth_of_every_row", "eighth_edges", "every_other_eighth"])
def test_survivors_clustered_in_few_fetch_units(pattern):
    """Placements of the survivors chosen against the units the value pass fetches by (32 and 64 elements): the
    units it reads are few, far apart, unevenly spread over the rows, or all of them for a stretch;
    the array is ragged and several chunks long."""
    n = 1_500_003
    q = np.arange((n + 63) // 64, dtype=np.int64)
    if pattern == "same_quarter_of_every_row":
        pos = (q[q % 4 == 2] * 64)[:, None] + np.array([0, 31, 63])
    elif pattern == "every_17th_quarter":
        pos = q[::17] * 64 + (q[::17] * 7) % 64
    elif pattern == "ends_only":
        pos = np.array([0, n - 1])
    elif pattern == "one_row_in_300":
        pos = (np.arange(0, n // 256, 300)[:, None] * 256 + np.arange(256)[None, :])
    elif pattern == "quarter_edges":
        pos = np.concatenate([q * 64 + 63, q * 64])[:: 5]
    elif pattern == "dense_island_in_a_desert":
        pos = np.concatenate([np.arange(700_001, 760_007), [5], [n - 2]])
    elif pattern == "same_eighth_of_every_row":
        e = np.arange((n + 31) // 32, dtype=np.int64)
        pos = (e[e % 8 == 5] * 32)[:, None] + np.array([0, 17, 31])
    elif pattern == "eighth_edges":
        e = np.arange((n + 31) // 32, dtype=np.int64)
        pos = np.concatenate([e * 32 + 31, e * 32])[:: 7]
    elif pattern == "every_other_eighth":
        e = np.arange(0, (n + 31) // 32, 2, dtype=np.int64)
        pos = e * 32 + (e * 5) % 32
    else:
        pos = np.arange(n - (n % 64), n)
    v, pos = _spikes(n, np.ravel(pos), 31)
    b = W.solve_base(v, pos.size / n)
    st = check_round_trip(np.arange(n, dtype=np.uint32), v, b, kb=512)
    assert int(st[40:48].view("<u8")[0]) == pos.size


def test_workspace_and_buffers_reused_across_sizes():
    """The same workspace serves a large call, then a small one, then an empty one, then a large one
    again: nothing of an earlier call may leak into a later one."""
    torch, B, G = _gpu()
    big = W.small_mixture(51, 700_000)
    small = W.small_mixture(52, 3_000)
    p_big = B.params(W.solve_base(big.values, 0.2))
    bufs = B.Buffers(big.values.size, p_big)
    for w, keep in ((big, 0.2), (small, 0.5), (W.small_mixture(53, 0), 0.5), (big, 0.01), (small, 1.0)):
        b = W.solve_base(w.values, keep) if w.values.size else 1.1
        rc_ref, st_ref = ref.compress(w.keys, w.values, ref.params(b))
        rc, status, st, _ = G.hip_compress(w.keys, w.values, B.params(b), bufs=bufs)
        assert rc == B.OK and status == rc_ref == 0
        assert np.array_equal(st, st_ref)


def test_workspace_sized_for_one_byte_codes():
    """A caller that announces thresholds of at most 128 passes a workspace with a byte of scratch per code: every
    element may survive, nothing is written behind the workspace, and a call with a larger threshold is refused."""
    torch, B, G = _gpu()
    rng = np.random.default_rng(61)
    n = 300_000
    vals = rng.laplace(0.0, 1e-3, n).astype(np.float32)
    vals[np.abs(vals) < 1e-7] = np.float32(1e-7)
    w = W.Workload("all_survive", np.arange(n, dtype=np.uint32), vals, n)
    for tau, fits in ((128, True), (40, True), (129, False), (256, False)):
        b = min(W.solve_base(w.values, 1.0, tau), 4.0 if tau > 128 else 16.0)
        p = B.params(b, tau)
        bufs = B.Buffers(n, p)
        words = B.workspace_size(n, 1, p.block_keys, max_tau=128) // 8
        assert B.workspace_size(n, 1, p.block_keys, max_tau=128) % 8 == 0
        whole = torch.full((words + 512,), 0x5A5A5A5A5A5A5A5A, dtype=torch.int64, device="cuda")
        bufs.workspace = whole[:words]
        rc, status, st, _ = G.hip_compress(w.keys, w.values, p, bufs=bufs)
        if fits:
            rc_ref, st_ref = ref.compress(w.keys, w.values, ref.params(b, tau))
            assert rc == B.OK and status == rc_ref == 0 and np.array_equal(st, st_ref)
            assert int(st[40:48].view("<u8")[0]) > 0.9 * n            # (nearly) every element survived
        else:
            assert rc == B.ERR_BUFFER_TOO_SMALL
        assert bool((whole[words:] == 0x5A5A5A5A5A5A5A5A).all())


def test_many_rounds_per_block_and_mixed_block_sizes():
    """Blocks of 2048 and 4096 keys take several rounds of 1024 per wave; dense keys, all survive."""
    n = 50_000
    keys = np.cumsum(np.random.default_rng(4).integers(1, 70_000, n)).astype(np.uint32)
    vals = np.full(n, 0.25, np.float32)
    for kb, l in ((2048, 1), (4096, 5), (4096, 2)):
        check_round_trip(keys, vals, 1.2, tau=128, l=l, kb=kb)


@pytest.mark.parametrize("seed", range(40))
def test_random_shapes_and_parameters(seed):
    """Seeded sweep over sizes (ragged tails of every kind), survival fractions, key gap structures and
    codec parameters: stream bytes, keys and decoded values against the oracle."""
    _random_case(seed, [1, 2, 7, 64, 100, 127, 128])


@pytest.mark.parametrize("seed", range(100, 120))
def test_random_shapes_and_parameters_with_thresholds_above_128(seed):
    _random_case(seed, [129, 130, 160, 200, 255, 256])


def _random_case(seed, taus):
    rng = np.random.default_rng(1000 + seed)
    n = int(rng.choice([0, 1, 2, 63, 64, 65, 1023, 1025, 5000, 65_537, 200_003, 300_000]))
    if seed % 3 == 0:
        n = int(rng.integers(1, 400_000))
    tau = int(rng.choice(taus))
    l = int(rng.integers(1, 6))
    kb = int(rng.choice([256, 512, 1024, 2048, 4096]))
    keep = float(rng.choice([1.0, 0.9, 0.5, 0.1, 0.02, 0.001]))
    scale = 10.0 ** rng.integers(-30, 20)
    kind = seed % 4
    if kind == 0:
        vals = rng.laplace(0.0, scale, n)
    elif kind == 1:
        vals = rng.standard_normal(n) * scale * np.where(rng.random(n) < 0.05, 100.0, 1.0)
    elif kind == 2:
        vals = np.where(rng.random(n) < 0.3, 0.0, rng.standard_normal(n) * scale)     # many exact zeros
    else:
        vals = rng.choice(np.array([1.0, -1.0, 0.5, 3.0, 1e-3]), n) * scale             # many equal magnitudes
    vals = vals.astype(np.float32)
    gap_kind = seed % 5
    if gap_kind == 0:
        keys = np.arange(n, dtype=np.uint64)
    elif gap_kind == 1:
        keys = np.cumsum(rng.integers(1, 50, n)).astype(np.uint64)
    elif gap_kind == 2:
        keys = np.cumsum(rng.integers(1, max(2, (2 ** 32 - 2) // max(n, 1)), n)).astype(np.uint64)   # up to 2^32
    elif gap_kind == 3:
        keys = np.cumsum(np.where(rng.random(n) < 0.01, rng.integers(1, 5000, n), 1)).astype(np.uint64)
    else:
        keys = np.cumsum(2 ** rng.integers(0, 12, n)).astype(np.uint64)               # powers of two
    assert n == 0 or keys[-1] < 2 ** 32
    b = W.solve_base(vals, keep, tau) if n and np.any(vals != 0) else 1.1
    if tau > 128:
        b = min(b, 4.0)
    check_round_trip(keys.astype(np.uint32), vals, b, tau, l, kb)


@pytest.mark.parametrize("tau,l,kb,n,keep", [(128, 3, 1024, 3500, 0.8), (200, 2, 256, 3000, 0.9), (5, 1, 256, 4000, 0.5)])
def test_random_bit_flips_in_a_stream_decode_like_the_oracle(tau, l, kb, n, keep):
    """Every single-bit corruption is either rejected by both decoders or decodes to the same pairs in
    both (a flipped payload bit may still be a consistent stream): every bit of the header, and a few
    hundred bits of the planes and the directory; one-byte, nine-bit and four-bit value tokens."""
    torch, B, G = _gpu()
    rng = np.random.default_rng(77 + tau)
    keys = np.cumsum(rng.integers(1, 3000, n)).astype(np.uint32)
    vals = (rng.laplace(0, 1.0, n) * np.exp(rng.uniform(-8, 0, n))).astype(np.float32)
    if tau <= 5:
        vals[::50] *= np.float32(1e4)
    rc, st = ref.compress(keys, vals, ref.params(min(W.solve_base(vals, keep, tau), 4.0 if tau > 128 else 16.0), tau, l, kb))
    assert rc == 0
    d = int(st[40:48].view("<u8")[0])
    assert d > 1000                                   # several blocks, the last one partial
    positions = np.concatenate([np.arange(64 * 8), rng.integers(64 * 8, st.size * 8, 300)])
    for pos in positions:
        s = st.copy()
        s[int(pos) >> 3] ^= np.uint8(1 << (int(pos) & 7))
        rc_ref, k_ref, v_ref = ref.decompress(s, capacity=d + 8)
        rc, status, k, v = G.hip_decompress(s, capacity=d + 8)
        assert rc == B.OK
        assert status == rc_ref, (int(pos), status, rc_ref)
        if status == 0:
            assert np.array_equal(k, k_ref) and np.array_equal(v.view(np.uint32), v_ref.view(np.uint32)), int(pos)
        else:
            assert k.size == 0


@pytest.mark.parametrize("n,keep", [(1, 1.0), (255, 0.5), (4097, 0.3), (300_001, 0.05), (2_000_003, 0.002)])
def test_no_key_array_means_keys_are_the_indices(n, keep):
    # a dense gradient handed over without keys encodes like the explicit keys 0..n-1
    torch, B, G = _gpu()
    rng = np.random.default_rng(n)
    vals = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    p = ref.params(W.solve_base(vals, keep), 128, 2, 1024)
    rc_ref, want = ref.compress(np.arange(n, dtype=np.uint32), vals, p)
    assert rc_ref == ref.OK
    rc, status, got, _ = G.hip_compress(None, vals, B.params(p.base, 128, 2, 1024))
    assert rc == B.OK and status == 0
    assert np.array_equal(got, want)


@pytest.mark.parametrize("tau", [1, 2, 3, 5, 16, 33, 64])
@pytest.mark.parametrize("n,kb", [(700, 256), (150_001, 1024), (400_003, 4096)])
def test_narrow_value_tokens(tau, n, kb):
    # tau <= 64: value tokens of 1 + ceil(log2 tau) < 8 bits (Section 3.2), bit-packed; sizes span
    # several blocks, rounds of 1024 inside a block, and ragged tails
    rng = np.random.default_rng(tau * 1000 + kb)
    keys = np.sort(rng.choice(4 * n, n, replace=False)).astype(np.uint32)
    vals = rng.laplace(0.0, 1e-3, n).astype(np.float32)
    vals[::n // 10] *= np.float32(1e4)           # a few dominant values: something survives even for tau = 1
    st = check_round_trip(keys, vals, W.solve_base(vals, 0.6, tau), tau, 2, kb)
    assert int(st[40:48].view("<u8")[0]) >= 1


def _wide_range_values(rng, n):
    """Magnitudes over five orders of magnitude, so that codes far beyond 128 are in use."""
    return (rng.laplace(0.0, 1e-2, n) * np.exp(rng.uniform(-12.0, 0.0, n))).astype(np.float32)


@pytest.mark.parametrize("tau", [129, 200, 256])
@pytest.mark.parametrize("n,kb", [(700, 256), (150_001, 1024), (400_003, 4096)])
def test_thresholds_above_128_take_nine_bit_tokens(tau, n, kb):
    # tau in 129..256 (Section 3.2: ceil(log2 tau) bits for the code, one for the sign): several blocks,
    # several rounds of 1024 per block, ragged tails
    from tests.streamparse import parse
    rng = np.random.default_rng(tau * 1000 + kb)
    keys = np.sort(rng.choice(4 * n, n, replace=False)).astype(np.uint32)
    vals = _wide_range_values(rng, n)
    st = check_round_trip(keys, vals, W.solve_base(vals, 0.7, tau), tau, 2, kb)
    info = parse(st) if n < 1000 else None
    assert int(st[6]) | int(st[7]) << 8 == tau
    if info:
        assert info["w"] == 9 and max(info["code"]) > 128


def test_thresholds_above_128_without_key_array_and_with_the_papers_base():
    # the paper's b = 1.1 keeps 10 % of a large dense gradient only with tau near 160
    torch, B, G = _gpu()
    rng = np.random.default_rng(200)
    n = 3_000_017
    vals = (rng.standard_normal(n) * np.where(rng.random(n) < 0.1, 1e-3, 1e-5)).astype(np.float32)
    rc_ref, want = ref.compress(np.arange(n, dtype=np.uint32), vals, ref.params(1.1, 162, 2, 1024))
    assert rc_ref == ref.OK
    d = int(want[40:48].view("<u8")[0])
    assert 0.05 * n < d < 0.15 * n
    rc, status, got, _ = G.hip_compress(None, vals, B.params(1.1, 162, 2, 1024))
    assert rc == B.OK and status == 0
    assert np.array_equal(got, want)
    rc_ref, k_ref, v_ref = ref.decompress(want)
    rc, status, k, v = G.hip_decompress(want, capacity=d)
    assert rc == B.OK and status == 0
    assert np.array_equal(k, k_ref) and np.array_equal(v.view(np.uint32), v_ref.view(np.uint32))


def test_nine_bit_codes_beyond_tau_and_bad_limits_are_rejected():
    torch, B, G = _gpu()
    rng = np.random.default_rng(9)
    n = 5000
    keys = np.arange(n, dtype=np.uint32) * 3
    vals = _wide_range_values(rng, n)
    rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, 0.9, 200), 200, 2, 256))
    assert rc == ref.OK
    d = int(st[40:48].view("<u8")[0])
    assert d > 3000

    def both(s):
        rc_ref, k_ref, v_ref = ref.decompress(s, capacity=d)
        rc, status, k, v = G.hip_decompress(s, capacity=d)
        assert rc == B.OK and status == rc_ref, (status, rc_ref)
        return status

    # token j sits at bit 9 j: set the code-1 field of a token in the first round, in a later round of the
    # first block... to 200 (code 201 > tau) and to 199 (code 200 = tau: fine)
    for j in (0, 7, 1023, 1024, 2500, d - 1):
        for field, expect in ((200, B.ERR_CORRUPT_STREAM), (199, B.OK), (255, B.ERR_CORRUPT_STREAM)):
            s = st.copy()
            bit = 9 * j
            word = int.from_bytes(s[64 + (bit >> 3):64 + (bit >> 3) + 4].tobytes(), "little")
            word = (word & ~(0xFF << (bit & 7))) | (field << (bit & 7))
            s[64 + (bit >> 3):64 + (bit >> 3) + 4] = np.frombuffer(word.to_bytes(4, "little"), np.uint8)
            assert both(s) == expect, (j, field)
    # header: tau = 257, tau = 0, and a base above 4 with tau above 128
    for lo, hi in ((1, 1), (0, 0)):
        s = st.copy(); s[6], s[7] = lo, hi
        assert both(s) == B.ERR_CORRUPT_STREAM
    s = st.copy(); s[16:24] = np.frombuffer(np.float64(4.5).tobytes(), np.uint8)
    assert both(s) == B.ERR_CORRUPT_STREAM
    # host side: the same limits
    rc, status, got, _ = G.hip_compress(keys, vals, B.params(1.1, 257))
    assert rc == B.ERR_INVALID_ARG
    rc, status, got, _ = G.hip_compress(keys, vals, B.params(4.5, 129))
    assert rc == B.ERR_INVALID_ARG


def test_keys_that_span_the_whole_32_bit_range_and_streams_that_leave_it():
    """Deltas of 28 to 32 bits (a lane's running sum can wrap) up to the key 2^32 - 1, and corrupted
    copies whose keys would pass 2^32: same verdict as the oracle."""
    torch, B, G = _gpu()
    rng = np.random.default_rng(31)
    # 15 steps of 2^28 - 1, then small steps, ending exactly at 2^32 - 1
    big = np.full(15, (1 << 28) - 1, np.uint64)
    small = rng.integers(1, 50, 1500).astype(np.uint64)
    keys = np.cumsum(np.concatenate([np.array([7], np.uint64), big, small]))
    keys = np.concatenate([keys, np.array([(1 << 32) - 1], np.uint64)])
    assert keys[-2] < keys[-1]
    vals = rng.laplace(0, 1.0, keys.size).astype(np.float32)
    st = check_round_trip(keys.astype(np.uint32), vals, 16.0, tau=128, l=2, kb=256)   # everything survives
    d = int(st[40:48].view("<u8")[0])
    assert d == keys.size
    # one key of 2^32 - 1 alone (M = 32), and a first key of 0
    check_round_trip(np.array([(1 << 32) - 1], np.uint32), np.array([1.0], np.float32), 1.1)
    check_round_trip(np.array([0, (1 << 32) - 1], np.uint32), np.array([1.0, -2.0], np.float32), 1.1)
    # flip bits in the key planes of the long stream: most flips push a key past 2^32 or break the chain
    dir_off = 64 + ((d + 7) & ~7)
    blocks_off = dir_off + 16 * ((d + 255) // 256)
    seen = set()
    for pos in rng.integers(blocks_off * 8, st.size * 8, 60):
        s = st.copy()
        s[int(pos) >> 3] ^= np.uint8(1 << (int(pos) & 7))
        rc_ref, k_ref, v_ref = ref.decompress(s, capacity=d)
        rc, status, k, v = G.hip_decompress(s, capacity=d)
        assert rc == B.OK and status == rc_ref, (int(pos), status, rc_ref)
        seen.add(status)
        if status == 0:
            assert np.array_equal(k, k_ref)
    assert B.ERR_CORRUPT_STREAM in seen
