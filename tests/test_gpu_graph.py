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
