"""GPU parity at the full sizes of the five workload configurations, in the launch configuration the
benchmark times.  The oracle finishes these in seconds, so whole streams are compared byte for byte."""
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


def full_check(w, base, keep):
    torch, B, G = _gpu()
    print(f"[fullsize] {w.name} n={w.values.size} keep={keep} base={base!r}", flush=True)
    rc_ref, st_ref = ref.compress(w.keys, w.values, ref.params(base))
    assert rc_ref == ref.OK
    rc, status, st, bufs = G.hip_compress(w.keys, w.values, B.params(base))
    assert rc == B.OK and status == 0
    assert st.size == st_ref.size and np.array_equal(st, st_ref), "stream differs from the oracle"
    d = int(st_ref[40:48].view("<u8")[0])
    assert abs(d - keep * w.values.size) <= 0.02 * keep * w.values.size + 2
    rc_ref, k_ref, v_ref = ref.decompress(st_ref)
    rc, status, k, v = G.hip_decompress(st_ref, capacity=d)
    assert rc == B.OK and status == 0 and rc_ref == ref.OK
    assert np.array_equal(k, k_ref)
    assert np.all(np.abs(v.astype(np.float64) - v_ref.astype(np.float64)) <= 1e-6 * np.abs(v_ref.astype(np.float64)))
    return st_ref.size


def test_config2_dense_25m():
    w = W.config2()
    full_check(w, W.solve_bases(w.values, [0.01])[0], 0.01)


def test_config3_sparse_zipf_10m():
    w = W.config3()
    size = full_check(w, W.solve_bases(w.values, [0.001])[0], 0.001)
    assert 8.0 * w.values.size / size > 1000          # three orders of magnitude, as planned


@pytest.mark.parametrize("keep", [0.10, 0.01, 0.001, 0.0001])
def test_config4_dense_124m(keep):
    w = W.config4()
    full_check(w, W.solve_bases(w.values, [keep])[0], keep)


def test_config5_segmented_60m():
    torch, B, G = _gpu()
    w = W.config5()
    offs = w.seg_offsets
    nseg = len(offs) - 1
    assert nseg == 160 and 57_000_000 <= w.values.size <= 63_000_000
    bases = [W.solve_bases(w.values[int(offs[i]):int(offs[i + 1])], [0.01])[0] for i in range(nseg)]
    rc_ref, blob_ref, so_ref = ref.compress_segmented(w.keys, w.values, offs, [ref.params(b) for b in bases])
    assert rc_ref == ref.OK
    rc, status, blob, so = G.hip_compress_segmented(w.keys, w.values, offs, [B.params(b) for b in bases])
    assert rc == B.OK and status == 0
    assert np.array_equal(so, so_ref) and np.array_equal(blob, blob_ref)
    cap = int(sum(int(blob_ref[int(o) + 40:int(o) + 48].view("<u8")[0]) for o in so_ref[:-1]))
    rc_ref, k_ref, v_ref, po_ref = ref.decompress_segmented(blob_ref, so_ref, cap)
    rc, status, k, v, po = G.hip_decompress_segmented(blob_ref, so_ref, cap)
    assert rc == B.OK and status == 0
    assert np.array_equal(po, po_ref) and np.array_equal(k, k_ref)
    assert np.array_equal(v.view(np.uint32), v_ref.view(np.uint32))


@pytest.mark.parametrize("n", [(1 << 31) + 12345, (1 << 32) - 1024])
def test_gradients_beyond_2_to_the_31_and_at_the_size_limit(n):
    """The largest gradient the library takes (2^32 - 1024 elements, 17 GB of values, no key array) and one
    just past 2^31.  The oracle cannot hold such an input in this test's time, so the result is checked by
    what holds at any size: the header's sum against a binary64 sum, the surviving keys against the
    threshold of the oracle's table applied to every element on the device, the stream against the
    oracle's decoder, values against the quantization bound of Eq. 3 (sum / b^c <= |v| < sum / b^(c-1))."""
    torch, B, G = _gpu()
    free, _ = torch.cuda.mem_get_info()
    ws_bytes = B.workspace_size(n, 1, 1024)
    if free < 4 * n + ws_bytes + (8 << 30):
        pytest.skip("not enough device memory for the largest gradient")
    print(f"[fullsize] n={n} workspace={ws_bytes}", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(n & 0xFFFF)
    v = torch.empty(n, dtype=torch.float32, device="cuda")
    step = 1 << 28
    total = 0.0
    for lo in range(0, n, step):
        part = v[lo:lo + step]
        part.normal_(0.0, 1e-4, generator=gen)
    planted = sorted({0, 1, 255, 256, n // 3, (1 << 31) - 1, 1 << 31, (1 << 31) + 1, n - 1025, n - 2, n - 1})
    for i, pos in enumerate(planted):
        v[pos] = (-1.0) ** i * (3.0 + i)
    for lo in range(0, n, step):
        total += float(v[lo:lo + step].abs().sum(dtype=torch.float64))
    base = (total / 5.5e-4) ** (1.0 / 128.0)              # threshold about 5.5 sigma: a few hundred survivors
    p = B.params(base)
    cap = 1 << 20
    out = torch.empty(cap // 8, dtype=torch.int64, device="cuda")
    ws = torch.empty(ws_bytes // 8 + 32, dtype=torch.int64, device="cuda")
    nbytes = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    rc = B.compress(None, v, p, out, nbytes, status, ws, n=n, out_capacity=cap)
    torch.cuda.synchronize()
    assert rc == B.OK and int(status[0]) == 0
    st = out.view(torch.uint8)[:int(nbytes[0])].cpu().numpy().copy()
    s_hdr = float(st[24:32].view("<f8")[0])
    assert int(st[32:40].view("<u8")[0]) == n
    assert abs(s_hdr - total) <= 1e-9 * total
    Btab, Vtab = ref.tables(s_hdr, base, 128)
    thr_bits = int(Btab[128])
    keys = []
    for lo in range(0, n, step):
        bits = v[lo:lo + step].view(torch.int32).bitwise_and(0x7FFFFFFF)
        keys.append(torch.nonzero(bits >= thr_bits).flatten().cpu().numpy() + lo)
    keys = np.concatenate(keys).astype(np.uint64)
    assert set(planted) <= set(int(k) for k in keys) and 20 < keys.size < 100_000
    rc_ref, k_ref, v_ref = ref.decompress(st)
    assert rc_ref == ref.OK
    assert np.array_equal(k_ref.astype(np.uint64), keys)
    orig = v[torch.from_numpy(keys.astype(np.int64)).cuda()].cpu().numpy().astype(np.float64)
    dec = v_ref.astype(np.float64)
    assert np.array_equal(np.signbit(dec), np.signbit(orig))
    assert np.all(np.abs(dec) <= np.abs(orig) * (1 + 1e-6)) and np.all(np.abs(dec) * base * (1 + 1e-6) > np.abs(orig))
    del v, ws
    rc, status, k, vals = G.hip_decompress(st, capacity=keys.size)
    assert rc == B.OK and status == 0
    assert np.array_equal(k, k_ref) and np.array_equal(vals.view(np.uint32), v_ref.view(np.uint32))


def test_largest_gradient_with_a_hundred_million_survivors():
    """2^32 - 1024 elements again, now with about 3 % of them kept: 4 million key blocks, ranks up to 2^27,
    a stream of about 200 MB.  Keys: the decoder's output against the threshold applied on the device.
    Stream: the oracle's decoder must read it and agree with the GPU decoder on every pair."""
    torch, B, G = _gpu()
    n = (1 << 32) - 1024
    free, _ = torch.cuda.mem_get_info()
    ws_bytes = B.workspace_size(n, 1, 1024)
    if free < 4 * n + ws_bytes + (16 << 30):
        pytest.skip("not enough device memory for the largest gradient")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    v = torch.empty(n, dtype=torch.float32, device="cuda")
    step = 1 << 28
    total = 0.0
    for lo in range(0, n, step):
        v[lo:lo + step].normal_(0.0, 1e-4, generator=gen)
        total += float(v[lo:lo + step].abs().sum(dtype=torch.float64))
    base = (total / 2.17e-4) ** (1.0 / 128.0)             # threshold about 2.17 sigma: 3 % survive
    p = B.params(base)
    cap = 1 << 30
    out = torch.empty(cap // 8, dtype=torch.int64, device="cuda")
    ws = torch.empty(ws_bytes // 8 + 32, dtype=torch.int64, device="cuda")
    nbytes = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    print(f"[fullsize] n={n} dense case: compress", flush=True)
    rc = B.compress(None, v, p, out, nbytes, status, ws, n=n, out_capacity=cap)
    torch.cuda.synchronize()
    assert rc == B.OK and int(status[0]) == 0
    del ws
    sb = int(nbytes[0])
    hdr = out.view(torch.uint8)[:64].cpu().numpy()
    s_hdr, d = float(hdr[24:32].view("<f8")[0]), int(hdr[40:48].view("<u8")[0])
    assert abs(s_hdr - total) <= 1e-9 * total and 0.025 * n < d < 0.035 * n
    thr_bits = int(ref.tables(s_hdr, base, 128)[0][128])
    print(f"[fullsize] d={d} stream={sb}: decompress", flush=True)
    k_out = torch.empty(d, dtype=torch.int32, device="cuda")
    v_out = torch.empty(d, dtype=torch.float32, device="cuda")
    cnt = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    dws = B.decoder_workspace(1)
    rc = B.decompress(out, sb, k_out, v_out, cnt, status, dws, capacity=d)
    torch.cuda.synchronize()
    assert rc == B.OK and int(status[0]) == 0 and int(cnt[0]) == d
    got = k_out.to(torch.int64) & 0xFFFFFFFF
    pos = 0
    for lo in range(0, n, step):                          # the surviving indices, slice by slice
        bits = v[lo:lo + step].view(torch.int32).bitwise_and(0x7FFFFFFF)
        want = torch.nonzero(bits >= thr_bits).flatten() + lo
        assert torch.equal(got[pos:pos + want.numel()], want)
        pos += want.numel()
    assert pos == d
    orig = v[got]
    assert torch.equal(torch.signbit(orig), torch.signbit(v_out))
    assert bool((v_out.abs() <= orig.abs()).all()) and bool((v_out.abs().double() * base * (1 + 1e-6) > orig.abs().double()).all())
    del v, orig
    print("[fullsize] oracle decode of the stream", flush=True)
    st = out.view(torch.uint8)[:sb].cpu().numpy()
    rc_ref, k_ref, v_ref = ref.decompress(st)
    assert rc_ref == ref.OK and k_ref.size == d
    assert np.array_equal(k_ref, k_out.cpu().numpy().view(np.uint32))
    assert np.array_equal(v_ref.view(np.uint32), v_out.cpu().numpy().view(np.uint32))


def test_batch_of_three_largest_gradients_takes_more_than_4096_chunks():
    """Three gradients of 2^32 - 1024 elements in one call (52 GB of values, no key array): a chunk of the
    value pass may not be longer than 8184 rows, so this call is cut into 6150 chunks instead of the usual
    4096 or fewer.  Every stream of the batch must be, byte for byte, what a call on that gradient alone
    gives (2050 chunks of 8184 rows there against 4096 of 4096 rows here: the stream does not depend on the
    cut), and that call is checked against the oracle's decoder and the threshold in the test above."""
    torch, B, G = _gpu()
    n, nseg = (1 << 32) - 1024, 3
    ws_bytes = B.workspace_size(nseg * n, nseg, 256)
    free, _ = torch.cuda.mem_get_info()
    if free < 4 * nseg * n + ws_bytes + (8 << 30):
        pytest.skip("not enough device memory for three of the largest gradients")
    print(f"[fullsize] batch of {nseg} x {n} workspace={ws_bytes}", flush=True)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4096)
    v = torch.empty(nseg * n, dtype=torch.float32, device="cuda")
    step = 1 << 28
    plist = []
    for s in range(nseg):
        seg = v[s * n:(s + 1) * n]
        for lo in range(0, n, step):
            seg[lo:lo + step].normal_(0.0, 1e-4 * (s + 1), generator=gen)
        for i, pos in enumerate((0, 1, 255, n // 2 + s, n - 1025, n - 1)):
            seg[pos] = (-1.0) ** i * (3.0 + i + s)
        total = 0.0
        for lo in range(0, n, step):
            total += float(seg[lo:lo + step].abs().sum(dtype=torch.float64))
        plist.append(B.params((total / (5.5e-4 * (s + 1))) ** (1.0 / 128.0), 128, 1 + s, 256 << s))
    cap = 8 << 20
    out = torch.empty(cap // 8, dtype=torch.int64, device="cuda")
    ws = torch.empty(ws_bytes // 8 + 32, dtype=torch.int64, device="cuda")
    so = torch.full((nseg + 1,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    rc = B.compress_segmented(None, v, [s * n for s in range(nseg + 1)], plist, out, so, status, ws)
    torch.cuda.synchronize()
    assert rc == B.OK and int(status[0]) == 0
    offs = [int(x) for x in so.cpu()]
    blob = out.view(torch.uint8)[:offs[-1]].cpu().numpy().copy()
    one = torch.empty(cap // 8, dtype=torch.int64, device="cuda")
    nb = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    for s in range(nseg):
        print(f"[fullsize] gradient {s} alone", flush=True)
        rc = B.compress(None, v[s * n:(s + 1) * n], plist[s], one, nb, status, ws, n=n, out_capacity=cap)
        torch.cuda.synchronize()
        assert rc == B.OK and int(status[0]) == 0
        alone = one.view(torch.uint8)[:int(nb[0])].cpu().numpy()
        part = blob[offs[s]:offs[s + 1]]
        d = int(part[40:48].view("<u8")[0])
        assert 20 < d < 200_000 and int(part[32:40].view("<u8")[0]) == n
        assert part.size == alone.size and np.array_equal(part, alone), f"gradient {s}: batch and single call differ"
        rc_ref, k_ref, v_ref = ref.decompress(part)
        assert rc_ref == ref.OK and k_ref.size == d and int(k_ref[0]) == 0 and int(k_ref[-1]) == n - 1


def test_config4_aggregation_of_four_workers_in_one_pass():
    """Decode-and-aggregate at the benchmark's size: four workers' streams of the 124M-element gradient (rotated by
    a different amount per worker) at 10 % kept, added into a 124M vector -- the one-pass form with runs of twenty
    tiles per workgroup -- compared bit for bit with the oracle's sums."""
    torch, B, G = _gpu()
    from tests.test_gpu_aggregate import hip_accumulate
    w = W.config4()
    n = w.values.size
    base = W.solve_bases(w.values, [0.10])[0]
    blobs, offs = [], [0]
    for wkr in range(4):
        vals = np.roll(w.values, wkr * 15485863)
        rc, st = ref.compress(w.keys, vals, ref.params(base))
        assert rc == ref.OK
        blobs.append(st)
        offs.append(offs[-1] + st.size)
        print(f"[fullsize] worker {wkr}: {st.size} bytes", flush=True)
    blob, offs = np.concatenate(blobs), np.array(offs, np.uint64)
    assert 10 * blob.size >= n
    rng = np.random.default_rng(77)
    dense0 = rng.standard_normal(n, dtype=np.float32) * np.float32(1e-3)
    want = dense0.copy()
    rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
    assert rc_ref == ref.OK
    print("[fullsize] oracle sums done", flush=True)
    rc, status, cnt, got = hip_accumulate(blob, offs, dense0)
    assert rc == B.OK and status == 0 and cnt == cnt_ref
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))
