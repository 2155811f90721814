"""GPU parity of decode-and-update (Adam step of Section 4.1 at the decoded keys) against the oracle.

The oracle evaluates the three equations in binary64 on the stored binary32 state and rounds each result
once; the kernel evaluates them in binary32 (4 roundings for m and v, 4 more for the step).  Bounds, with
u = 2^-24: |dm| <= 4u (|b1 m| + |(1-b1) g|), |dv| <= 4u v', and for theta one rounding of theta on each side
(2u max(|theta|, |theta'|)) plus 1e-6 of the step (relative errors of v' and four operations) plus the
absolute error of m' carried through the step, eta |dm| / sqrt(v' + eps) (m' can cancel)."""
import numpy as np
import pytest

from oracle import ref
from tests.test_oracle_adam import one_stream

pytestmark = pytest.mark.gpu
U = 2.0 ** -24


def hip_adam(st, theta, m, v, eta, b1=0.9, b2=0.999, eps=1e-8):
    import torch
    from paper_2112_04291_amd import binding as B
    s = np.ascontiguousarray(st, dtype=np.uint8)
    dev = torch.from_numpy(np.concatenate([s, np.zeros((-s.size) % 8 + 8, np.uint8)])).cuda()
    t, mm, vv = (torch.from_numpy(a.copy()).cuda() for a in (theta, m, v))
    count = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(1)
    rc = B.decompress_adam(dev, s.size, t, mm, vv, eta, b1, b2, eps, count, status, ws)
    torch.cuda.synchronize()
    return rc, int(status[0]), int(count[0]), t.cpu().numpy(), mm.cpu().numpy(), vv.cpu().numpy()


@pytest.mark.parametrize("dim,nnz,keep,seed,tau", [(50_000, 8_000, 0.5, 1, 128), (3_000_000, 600_000, 0.3, 2, 128),
                                                   (4_000, 4_000, 1.0, 3, 128), (300_000, 70_000, 0.6, 4, 200)])
def test_adam_matches_oracle(dim, nnz, keep, seed, tau):
    from paper_2112_04291_amd import binding as B
    st, k, g = one_stream(dim, nnz, keep, seed, tau)
    rng = np.random.default_rng(seed)
    theta0 = rng.standard_normal(dim).astype(np.float32)
    m0 = (rng.standard_normal(dim) * 1e-3).astype(np.float32)
    v0 = (rng.random(dim) * 1e-6).astype(np.float32)
    for steps in range(2):                       # second round starts from the first one's state
        t_ref, m_ref, v_ref = theta0.copy(), m0.copy(), v0.copy()
        rc, cnt_ref = ref.decompress_adam(st, t_ref, m_ref, v_ref, 0.01)
        assert rc == ref.OK
        rc, status, cnt, t, m, v = hip_adam(st, theta0, m0, v0, 0.01)
        assert rc == B.OK and status == 0 and cnt == cnt_ref == k.size
        untouched = np.ones(dim, bool)
        untouched[k] = False
        for got, old in ((t, theta0), (m, m0), (v, v0)):
            assert np.array_equal(got[untouched].view(np.uint32), old[untouched].view(np.uint32))
        g64 = g.astype(np.float64)
        dm = 4 * U * (np.abs(0.9 * m0[k]) + np.abs(0.1 * g64)) + 1e-45
        assert np.all(np.abs(m[k].astype(np.float64) - m_ref[k]) <= dm)
        assert np.all(np.abs(v[k].astype(np.float64) - v_ref[k]) <= 4 * U * v_ref[k] + 1e-45)
        step = np.abs(t_ref[k].astype(np.float64) - theta0[k])
        assert np.all(np.abs(t[k].astype(np.float64) - t_ref[k])
                      <= 2 * U * np.maximum(np.abs(t_ref[k]), np.abs(theta0[k])) + 1e-6 * step
                      + 0.01 * dm / np.sqrt(v_ref[k].astype(np.float64) + 1e-8))
        theta0, m0, v0 = t_ref, m_ref, v_ref


def test_adam_errors_match_oracle():
    from paper_2112_04291_amd import binding as B
    st, k, g = one_stream(10_000, 2_000, 0.5, 5)
    top = int(k.max())
    z = [np.zeros(top, np.float32) for _ in range(3)]
    assert ref.decompress_adam(st, *[a.copy() for a in z], 0.1)[0] == ref.ERR_BUFFER_TOO_SMALL
    rc, status, cnt, *_ = hip_adam(st, *z, 0.1)
    assert rc == B.OK and status == B.ERR_BUFFER_TOO_SMALL and cnt == 0
    bad = st.copy()
    bad[4] ^= 0x7
    z = [np.zeros(top + 1, np.float32) for _ in range(3)]
    rc, status, cnt, t, m, v = hip_adam(bad, *z, 0.1)
    assert rc == B.OK and status == B.ERR_CORRUPT_STREAM and cnt == 0
    assert not t.any() and not m.any() and not v.any()
    rc, *_ = hip_adam(st, *z, 0.1, b1=1.5)
    assert rc == B.ERR_INVALID_ARG
    # a stream in which a key repeats its predecessor would make the update depend on the order of the lanes
    from tests.streamparse import with_zero_delta
    for rank in (1, 500, k.size - 1):
        bad = with_zero_delta(st, rank)
        assert ref.decompress_adam(bad, *[a.copy() for a in z], 0.1)[0] == ref.ERR_CORRUPT_STREAM
        rc, status, cnt, *_ = hip_adam(bad, *z, 0.1)
        assert rc == B.OK and status == B.ERR_CORRUPT_STREAM and cnt == 0, rank
