"""fastsgd_compress_static (the entry point for callers that cannot allocate: its workspace is a fixed array
inside the library) against fastsgd_compress, through the C ABI: byte-identical streams, two calls in a row,
the second on a smaller input, then the size limit."""
import numpy as np
import pytest

from paper_2112_04291_amd import workloads as W

pytestmark = pytest.mark.gpu


def test_static_workspace_variant_equals_fastsgd_compress():
    import torch
    from paper_2112_04291_amd import binding as B
    from tests import gpu_util as G
    assert torch.cuda.is_available()
    cases = [(B.STATIC_MAX_ELEMS, 0.1, 128, 2, 1024, True), (300_001, 0.02, 100, 3, 256, True),
             (70_001, 0.5, 200, 1, 512, False), (1, 1.0, 128, 2, 1024, True), (0, 1.0, 128, 2, 1024, True)]
    for n, keep, tau, l, kb, with_keys in cases:       # every call after the first is smaller than the one before
        w = W.small_mixture(4242 + n % 1000, n)
        base = W.solve_base(w.values, keep, tau) if n else 1.1
        p = B.params(base, tau, l, kb)
        keys = w.keys if with_keys else None
        print(f"[no-alloc] n={n} keep={keep} tau={tau} l={l} kb={kb} keys={'yes' if with_keys else 'none'}", flush=True)
        rc, status, want, bufs = G.hip_compress(keys, w.values, p)
        assert rc == B.OK and status == B.OK
        k = None if keys is None else G.to_dev_u32(keys)
        v = G.to_dev_f32(w.values)
        out = torch.full_like(bufs.out, -1)
        nbytes = torch.full((2,), -1, dtype=torch.int64, device="cuda")
        st = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        rc = B.compress_static(k, v, p, out, nbytes, st, n=n, out_capacity=bufs.out_capacity)
        torch.cuda.synchronize()
        assert rc == B.OK and int(st[0]) == B.OK
        assert int(nbytes[0]) == want.size
        got = out.view(torch.uint8)[:want.size].cpu().numpy()
        assert np.array_equal(got, want), "stream differs from fastsgd_compress"
    # beyond the fixed workspace: refused on the host, nothing enqueued
    n = B.STATIC_MAX_ELEMS + 1
    v = torch.zeros(n, dtype=torch.float32, device="cuda")
    out = torch.zeros(1024, dtype=torch.int64, device="cuda")
    nbytes = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    st = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    assert B.compress_static(None, v, B.params(), out, nbytes, st, n=n) == B.ERR_BUFFER_TOO_SMALL
    torch.cuda.synchronize()
    assert int(nbytes[0]) == -1 and int(st[0]) == -1
    # a device-detected condition comes back through the status word as in fastsgd_compress
    v = torch.full((5000,), float("nan"), dtype=torch.float32, device="cuda")
    assert B.compress_static(None, v, B.params(), out, nbytes, st) == B.OK
    torch.cuda.synchronize()
    assert int(st[0]) == B.ERR_NONFINITE and int(nbytes[0]) == 0
