"""Calls on different HIP streams run concurrently when each has a workspace of its own (the library keeps
no state between calls): three gradients compressed and decompressed on three streams at once, several
rounds without synchronising in between, each stream's last result against the oracle."""
import numpy as np
import pytest

from oracle import ref
from paper_2112_04291_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_concurrent_calls_on_three_streams_with_their_own_workspaces():
    import torch
    from paper_2112_04291_amd import binding as B
    from tests import gpu_util as G
    cases = [(2_000_003, 0.05, 128, 2, 1024), (700_001, 0.5, 200, 3, 256), (3_000_000, 0.002, 16, 1, 4096)]
    jobs = []
    for i, (n, keep, tau, l, kb) in enumerate(cases):
        w = W.small_mixture(40 + i, n)
        base = W.solve_base(w.values, keep, tau)
        p = B.params(min(base, 4.0) if tau > 128 else base, tau, l, kb)
        jobs.append(dict(w=w, p=p, args=(p.base, tau, l, kb), bufs=B.Buffers(n, p), keys=G.to_dev_u32(w.keys),
                         vals=G.to_dev_f32(w.values), stream=torch.cuda.Stream(),
                         count=torch.zeros(2, dtype=torch.int64, device="cuda"),
                         dstatus=torch.zeros(2, dtype=torch.int32, device="cuda")))
    torch.cuda.synchronize()
    for rnd in range(5):
        for j in jobs:                                     # interleaved launches, nothing waits for anything
            with torch.cuda.stream(j["stream"]):
                b = j["bufs"]
                n = j["w"].values.size
                assert B.compress(j["keys"], j["vals"], j["p"], b.out, b.out_offsets, b.status, b.workspace, n=n,
                                  out_capacity=b.out_capacity) == B.OK
                assert B.decompress(b.out, b.out_capacity, b.keys_out, b.values_out, j["count"], j["dstatus"],
                                    b.dec_workspace, capacity=n) == B.OK
    torch.cuda.synchronize()
    for j in jobs:
        b, w = j["bufs"], j["w"]
        rc_ref, st_ref = ref.compress(w.keys, w.values, ref.params(*j["args"]))
        assert rc_ref == ref.OK
        nbytes = int(b.out_offsets[0])
        assert int(b.status[0]) == 0 and nbytes == st_ref.size
        assert np.array_equal(b.out_bytes_view()[:nbytes].cpu().numpy(), st_ref)
        rc_ref, k_ref, v_ref = ref.decompress(st_ref)
        d = int(j["count"][0])
        assert int(j["dstatus"][0]) == 0 and d == k_ref.size
        assert np.array_equal(b.keys_out[:d].cpu().numpy().view(np.uint32), k_ref)
        assert np.array_equal(b.values_out[:d].cpu().numpy().view(np.uint32), v_ref.view(np.uint32))
