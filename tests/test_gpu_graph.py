"""The library enqueues kernels only (no copies, no memsets, no host synchronisation, no allocation), so a
compress + decompress pair can be captured into a HIP graph and replayed on new data.  Every replay is checked
against the oracle, with eager work and synchronisations between the replays."""
import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_compress_and_decompress_replayed_from_a_graph():
    import torch
    from paper_2112_04291_amd import binding as B
    from tests import gpu_util as G
    n = 300_000
    w = W.small_mixture(11, n)
    base = W.solve_base(w.values, 0.05)
    p = B.params(base)
    bufs = B.Buffers(n, p)
    keys = G.to_dev_u32(w.keys)
    vals = G.to_dev_f32(w.values)
    count = torch.zeros(2, dtype=torch.int64, device="cuda")
    dstatus = torch.zeros(2, dtype=torch.int32, device="cuda")

    def run():
        # the decoder reads the length from the header; it is handed the whole output buffer
        assert B.compress(keys, vals, p, bufs.out, bufs.out_offsets, bufs.status, bufs.workspace, n=n,
                          out_capacity=bufs.out_capacity) == B.OK
        assert B.decompress(bufs.out, bufs.out_capacity, bufs.keys_out, bufs.values_out, count, dstatus,
                            bufs.dec_workspace, capacity=n) == B.OK

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()                                              # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    rng = np.random.default_rng(3)
    for it in range(4):
        v_host = (w.values * np.float32(1.0 + 0.25 * it) + rng.standard_normal(n).astype(np.float32) * np.float32(1e-7 * it))
        vals.copy_(torch.from_numpy(v_host).cuda())        # eager work between the replays
        bufs.out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        rc_ref, st_ref = ref.compress(w.keys, v_host, ref.params(base))
        assert rc_ref == ref.OK
        nbytes = int(bufs.out_offsets[0])
        assert int(bufs.status[0]) == 0 and nbytes == st_ref.size, (it, nbytes, st_ref.size)
        assert np.array_equal(bufs.out_bytes_view()[:nbytes].cpu().numpy(), st_ref), it
        rc_ref, k_ref, v_ref = ref.decompress(st_ref)
        d = int(count[0])
        assert int(dstatus[0]) == 0 and d == k_ref.size
        assert np.array_equal(bufs.keys_out[:d].cpu().numpy().view(np.uint32), k_ref)
        assert np.array_equal(bufs.values_out[:d].cpu().numpy().view(np.uint32), v_ref.view(np.uint32))


def test_aggregation_in_one_pass_replayed_from_a_graph():
    """Four workers' streams (dense enough for the one-pass form) added into a dense vector by a captured graph,
    replayed on new streams and a new vector each time."""
    import torch
    from paper_2112_04291_amd import binding as B
    dim, nnz, n_workers = 150_000, 90_000, 4

    def streams(seed):
        rng = np.random.default_rng(seed)
        blobs, offs = [], [0]
        for wkr in range(n_workers):
            keys = np.sort(rng.choice(dim, nnz, replace=False)).astype(np.uint32)
            vals = rng.laplace(0.0, 1e-3 * (wkr + 1), nnz).astype(np.float32)
            rc, st = ref.compress(keys, vals, ref.params(W.solve_base(vals, 0.7)))
            assert rc == ref.OK
            blobs.append(st)
            offs.append(offs[-1] + st.size)
        return np.concatenate(blobs), np.array(offs, np.uint64)

    blob0, offs0 = streams(100)
    cap = 2 * blob0.size                                  # room for the streams of every replay
    assert 10 * blob0.size >= dim
    dev = torch.zeros(cap, dtype=torch.uint8, device="cuda")
    so = torch.zeros(n_workers + 1, dtype=torch.int64, device="cuda")
    dense = torch.zeros(dim, dtype=torch.float32, device="cuda")
    count = torch.zeros(2, dtype=torch.int64, device="cuda")
    status = torch.zeros(2, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(n_workers)

    def put(blob, offs):
        dev.zero_()
        dev[:blob.size].copy_(torch.from_numpy(blob).cuda())
        so.copy_(torch.from_numpy(offs.view(np.int64)).cuda())

    def run():
        # the total length travels in the offsets (on the device); the host passes the buffer's size
        assert B.decompress_accumulate(dev, cap, so, n_workers, dense, count, status, ws) == B.OK

    put(blob0, offs0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    rng = np.random.default_rng(4)
    for it in range(4):
        blob, offs = streams(200 + it)
        assert blob.size <= cap
        d0 = rng.standard_normal(dim).astype(np.float32)
        put(blob, offs)
        dense.copy_(torch.from_numpy(d0).cuda())
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        want = d0.copy()
        rc_ref, cnt_ref = ref.decompress_accumulate(blob, offs, want)
        assert rc_ref == ref.OK and int(status[0]) == 0 and int(count[0]) == cnt_ref, it
        assert np.array_equal(dense.cpu().numpy().view(np.uint32), want.view(np.uint32)), it
