"""GPU parity for the segmented batch (many independent gradients in one call) against the oracle."""
import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W

pytestmark = pytest.mark.gpu


def _gpu():
    import torch
    from paper_2112_04291_amd import binding as B
    from tests import gpu_util as G
    assert torch.cuda.is_available()
    return torch, B, G


def check_segmented(keys, vals, offs, ref_plist, hip_plist):
    torch, B, G = _gpu()
    rc_ref, blob_ref, so_ref = ref.compress_segmented(keys, vals, offs, ref_plist)
    assert rc_ref == ref.OK
    rc, status, blob, so = G.hip_compress_segmented(keys, vals, offs, hip_plist)
    assert rc == B.OK and status == 0, (rc, status)
    assert np.array_equal(so, so_ref), (so[:8], so_ref[:8])
    if not np.array_equal(blob, blob_ref):
        bad = np.flatnonzero(blob != blob_ref)
        seg = int(np.searchsorted(so_ref, bad[0], side="right") - 1)
        raise AssertionError(f"{bad.size} bytes differ, first at {bad[0]} (segment {seg}, offset {bad[0] - int(so_ref[seg])})")
    cap = int(sum(int(blob_ref[int(o) + 40:int(o) + 48].view("<u8")[0]) for o in so_ref[:-1]))
    rc_ref, k_ref, v_ref, po_ref = ref.decompress_segmented(blob_ref, so_ref, cap)
    rc, status, k, v, po = G.hip_decompress_segmented(blob_ref, so_ref, cap)
    assert rc == B.OK and status == 0 and rc_ref == ref.OK
    assert np.array_equal(po, po_ref) and np.array_equal(k, k_ref)
    assert np.array_equal(v.view(np.uint32), v_ref.view(np.uint32))
    # every stream of the batch is decodable on its own
    nseg = len(so_ref) - 1
    for i in sorted({0, nseg // 2, nseg - 1}):
        a, b = int(so_ref[i]), int(so_ref[i + 1])
        rc1, st1, k1, v1 = G.hip_decompress(blob_ref[a:b], capacity=int(po_ref[i + 1] - po_ref[i]))
        assert rc1 == B.OK and st1 == 0
        assert np.array_equal(k1, k_ref[int(po_ref[i]):int(po_ref[i + 1])])
    return blob


def test_small_batch_with_empty_and_tiny_segments():
    torch, B, G = _gpu()
    rng = np.random.default_rng(21)
    sizes = [0, 1, 700, 5000, 3, 0, 2500, 4096, 4097, 12289, 0]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = np.concatenate([rng.laplace(0, 10.0 ** -(i % 5 + 1), s) for i, s in enumerate(sizes)]).astype(np.float32)
    args = [(1.04 + 0.01 * i, 128 - i, 1 + i % 3, 256 << (i % 3)) for i in range(len(sizes))]
    check_segmented(keys, vals, offs, [ref.params(*a) for a in args], [B.params(*a) for a in args])
    check_segmented(keys, vals, offs, ref.params(1.07), B.params(1.07))      # shared parameters


def test_single_segment_batch_matches_plain_call():
    torch, B, G = _gpu()
    w = W.small_mixture(5, 100_000)
    b = W.solve_base(w.values, 0.1)
    blob = check_segmented(w.keys, w.values, np.array([0, w.values.size], np.uint64), ref.params(b), B.params(b))
    rc, status, st, _ = G.hip_compress(w.keys, w.values, B.params(b))
    assert np.array_equal(blob, st)


def test_config5_scaled_down():
    """160 tensors, log-uniform sizes, per-tensor Laplace scale, per-tensor base keeping about 1%."""
    torch, B, G = _gpu()
    w = W.config5(lo=256, hi=262_144, total_range=(3_500_000, 4_000_000))
    offs = w.seg_offsets
    bases = [W.solve_base(w.values[int(offs[i]):int(offs[i + 1])], 0.01) for i in range(len(offs) - 1)]
    blob = check_segmented(w.keys, w.values, offs, [ref.params(b) for b in bases], [B.params(b) for b in bases])
    ratio = 8.0 * w.values.size / blob.size
    assert ratio > 50


def test_batch_with_a_nonfinite_segment_fails_as_a_whole():
    torch, B, G = _gpu()
    rng = np.random.default_rng(3)
    sizes = [5000, 6000, 7000]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = rng.laplace(0, 1e-3, sum(sizes)).astype(np.float32)
    vals[5000 + 17] = np.inf
    rc, status, blob, so = G.hip_compress_segmented(keys, vals, offs, B.params(1.1))
    assert rc == B.OK and status == B.ERR_NONFINITE and blob.size == 0 and np.all(so == 0)
    assert ref.compress_segmented(keys, vals, offs, ref.params(1.1))[0] == ref.ERR_NONFINITE


def test_batch_without_key_array_uses_the_indices_inside_each_segment():
    torch, B, G = _gpu()
    rng = np.random.default_rng(33)
    sizes = [0, 1, 700, 5000, 3, 70_001, 4096, 4097, 250_003]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = np.concatenate([rng.laplace(0, 10.0 ** -(i % 4 + 1), s) for i, s in enumerate(sizes)]).astype(np.float32)
    bases = [W.solve_base(vals[int(offs[i]):int(offs[i + 1])], 0.05) if sizes[i] > 100 else 1.1 for i in range(len(sizes))]
    rc_ref, blob_ref, so_ref = ref.compress_segmented(keys, vals, offs, [ref.params(b) for b in bases])
    assert rc_ref == ref.OK
    rc, status, blob, so = G.hip_compress_segmented(None, vals, offs, [B.params(b) for b in bases])
    assert rc == B.OK and status == 0
    assert np.array_equal(so, so_ref) and np.array_equal(blob, blob_ref)


def test_batch_with_mixed_token_widths():
    # segments with tau from 1 to 128 in one call: value tokens of 1 to 8 bits side by side
    torch, B, G = _gpu()
    rng = np.random.default_rng(44)
    taus = [128, 64, 5, 1, 33, 16, 2, 100, 3]
    sizes = [5000, 70_001, 4097, 300, 12289, 250_003, 1, 0, 9000]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = np.concatenate([rng.laplace(0, 1e-3, s) for s in sizes]).astype(np.float32)
    args = []
    for i, (tau, s) in enumerate(zip(taus, sizes)):
        seg = vals[int(offs[i]):int(offs[i + 1])]
        if s > 20:
            seg[::max(s // 7, 1)] *= np.float32(3e3)
        args.append((W.solve_base(seg, 0.4, tau) if s > 20 else 1.3, tau, 1 + i % 4, 256 << (i % 4)))
    check_segmented(keys, vals, offs, [ref.params(*a) for a in args], [B.params(*a) for a in args])


def test_batch_whose_survivors_sit_at_the_segment_ends():
    # segments of odd lengths (so that they start anywhere inside a row); the survivors are the first and
    # the last elements of each segment and a lone one in the middle of the long ones: the units (32 values) the
    # value pass reads are the ones that segment boundaries cut
    torch, B, G = _gpu()
    rng = np.random.default_rng(77)
    sizes = [1, 2, 63, 64, 65, 255, 257, 1021, 30_011, 3, 100_003, 511, 0, 7, 250_001, 129]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = (rng.uniform(1e-9, 1e-8, int(offs[-1])) * rng.choice([-1.0, 1.0], int(offs[-1]))).astype(np.float32)
    args = []
    for i, s in enumerate(sizes):
        seg = vals[int(offs[i]):int(offs[i + 1])]
        pos = sorted({0, min(1, s - 1), s - 1, s // 2} & set(range(s))) if s > 1000 else sorted({0, s - 1} & set(range(s)))
        for j in pos:
            seg[j] = np.float32(rng.uniform(0.5, 2.0) * rng.choice([-1.0, 1.0]))
        args.append((W.solve_base(seg, len(pos) / s) if s else 1.1, 128, 1 + i % 3, 256))
    check_segmented(keys, vals, offs, [ref.params(*a) for a in args], [B.params(*a) for a in args])
    # the placement did what it was meant to: exactly the planted elements survive
    rc, blob, so = ref.compress_segmented(keys, vals, offs, [ref.params(*a) for a in args])
    kept = [int(blob[int(o) + 40:int(o) + 48].view("<u8")[0]) for o in so[:-1]]
    assert kept == [min(s, 4 if s > 1000 else 2) for s in sizes]


def test_batch_with_thresholds_on_both_sides_of_128():
    # one segment with tau > 128 makes the whole call keep 16-bit scratch codes: the byte-token and the
    # narrow-token segments next to it must come out unchanged
    torch, B, G = _gpu()
    rng = np.random.default_rng(45)
    taus = [128, 200, 5, 256, 64, 129, 100, 33]
    sizes = [5000, 70_001, 4097, 30_000, 12289, 250_003, 1, 9000]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    keys = np.concatenate([np.arange(s, dtype=np.uint32) for s in sizes])
    vals = np.concatenate([rng.laplace(0, 1e-3, s) * np.exp(rng.uniform(-10, 0, s)) for s in sizes]).astype(np.float32)
    args = []
    for i, (tau, s) in enumerate(zip(taus, sizes)):
        seg = vals[int(offs[i]):int(offs[i + 1])]
        args.append((W.solve_base(seg, 0.5, tau) if s > 20 else 1.3, tau, 1 + i % 4, 256 << (i % 4)))
    blob = check_segmented(keys, vals, offs, [ref.params(*a) for a in args], [B.params(*a) for a in args])
    # the tau <= 128 segments alone, in a call of their own (byte scratch codes): the same streams
    rc_ref, blob_all, so = ref.compress_segmented(keys, vals, offs, [ref.params(*a) for a in args])
    for i in (0, 2, 4):
        a, b = int(offs[i]), int(offs[i + 1])
        rc, status, st, _ = G.hip_compress(keys[a:b], vals[a:b], B.params(*args[i]))
        assert rc == B.OK and status == 0
        assert np.array_equal(st, blob_all[int(so[i]):int(so[i + 1])])


@pytest.mark.parametrize("seed", range(16))
def test_random_batches(seed):
    """Seeded sweep over batches: number and sizes of the segments (empty, tiny, ragged, several chunks long),
    survival fractions, per-segment parameters on both sides of tau = 128, with and without a key array."""
    torch, B, G = _gpu()
    rng = np.random.default_rng(7000 + seed)
    nseg = int(rng.choice([1, 2, 3, 17, 80, 81, 200]))
    kinds = rng.integers(0, 5, nseg)
    sizes = np.where(kinds == 0, 0, np.where(kinds == 1, rng.integers(1, 70, nseg),
                     np.where(kinds == 2, rng.integers(200, 5000, nseg), rng.integers(5000, 120_000, nseg))))
    if seed % 4 == 0:
        sizes[int(rng.integers(0, nseg))] = int(rng.integers(600_000, 1_500_000))
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    n = int(offs[-1])
    implicit = seed % 3 == 0
    gaps = rng.integers(1, 40, n).astype(np.uint64)
    keys = np.empty(n, np.uint32)
    scales = 10.0 ** rng.uniform(-8, 2, nseg)
    vals = np.empty(n, np.float32)
    wide = seed % 2 == 1
    args = []
    for i in range(nseg):
        a, b = int(offs[i]), int(offs[i + 1])
        keys[a:b] = np.arange(b - a) if implicit else np.cumsum(gaps[a:b]) - 1
        v = rng.laplace(0.0, scales[i], b - a) * np.exp(rng.uniform(-6, 0, b - a))
        if b - a > 10 and rng.random() < 0.3:
            v[rng.random(b - a) < 0.5] = 0.0
        vals[a:b] = v.astype(np.float32)
        tau = int(rng.choice([129, 160, 256, 128, 64, 5] if wide else [128, 128, 100, 64, 7, 1]))
        keep = float(rng.choice([1.0, 0.5, 0.1, 0.01]))
        seg = vals[a:b]
        base = W.solve_base(seg, keep, tau) if b > a and np.any(seg != 0) else 1.1
        args.append((min(base, 4.0) if tau > 128 else base, tau, int(rng.integers(1, 6)), int(rng.choice([256, 1024, 4096]))))
    rp, hp = [ref.params(*a) for a in args], [B.params(*a) for a in args]
    if implicit:
        rc_ref, blob_ref, so_ref = ref.compress_segmented(keys, vals, offs, rp)
        assert rc_ref == ref.OK
        rc, status, blob, so = G.hip_compress_segmented(None, vals, offs, hp)
        assert rc == B.OK and status == 0
        assert np.array_equal(so, so_ref) and np.array_equal(blob, blob_ref)
    else:
        check_segmented(keys, vals, offs, rp, hp)


def test_batch_of_the_largest_number_of_segments():
    # 65536 segments (the limit), most of them tiny, some empty, a few that span several key blocks
    torch, B, G = _gpu()
    rng = np.random.default_rng(65536)
    sizes = rng.integers(0, 40, 65536)
    sizes[rng.integers(0, 65536, 50)] = rng.integers(3000, 9000, 50)
    sizes[[0, 1, 65535]] = [0, 5000, 0]
    offs = np.concatenate([[0], np.cumsum(sizes)]).astype(np.uint64)
    n = int(offs[-1])
    keys = (np.arange(n, dtype=np.uint64) - np.repeat(offs[:-1], sizes)).astype(np.uint32)
    vals = (rng.standard_normal(n) * np.repeat(10.0 ** rng.uniform(-6, -2, 65536), sizes)).astype(np.float32)
    check_segmented(keys, vals, offs, ref.params(1.02, 128, 2, 256), B.params(1.02, 128, 2, 256))
    rc, status, blob, so = G.hip_compress_segmented(keys, vals, np.append(offs, offs[-1]), B.params(1.02, 128, 2, 256))
    assert rc == B.ERR_INVALID_ARG                         # 65537 segments
