"""Helpers for the GPU parity tests: run the HIP path through the C ABI binding on numpy inputs."""
import numpy as np
import torch

from paper_2112_04291_amd import binding as B


def to_dev_u32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint32).view(np.int32)).cuda()


def to_dev_f32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def hip_compress(keys, values, p, out_capacity=None, bufs=None):
    """Returns (host rc, device status, stream bytes as uint8 numpy array, bufs)."""
    n = int(np.asarray(values).size)
    bufs = bufs or B.Buffers(n, p, out_capacity=out_capacity)
    k, v = (None if keys is None else to_dev_u32(keys)), to_dev_f32(values)
    bufs.status.fill_(-1)
    bufs.out_offsets.fill_(-1)
    rc = B.compress(k, v, p, bufs.out, bufs.out_offsets, bufs.status, bufs.workspace, n=n,
                    out_capacity=bufs.out_capacity)
    torch.cuda.synchronize()
    if rc != B.OK:
        return rc, None, None, bufs
    status = int(bufs.status[0].item())
    nbytes = int(bufs.out_offsets[0].item())
    stream = bufs.out_bytes_view()[:nbytes].cpu().numpy().copy()
    return rc, status, stream, bufs


def hip_decompress(stream, capacity, bufs=None, p=None):
    """stream: uint8 numpy array.  Returns (host rc, device status, keys uint32, values float32)."""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    pad = (-s.size) % 8
    dev = torch.from_numpy(np.concatenate([s, np.zeros(pad + 8, np.uint8)])).cuda()
    keys_out = torch.empty(max(capacity, 1), dtype=torch.int32, device="cuda")
    vals_out = torch.empty(max(capacity, 1), dtype=torch.float32, device="cuda")
    count = torch.full((2,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(1)
    rc = B.decompress(dev, s.size, keys_out, vals_out, count, status, ws, capacity=capacity)
    torch.cuda.synchronize()
    if rc != B.OK:
        return rc, None, None, None
    c = int(count[0].item())
    return rc, int(status[0].item()), keys_out[:c].cpu().numpy().view(np.uint32).copy(), vals_out[:c].cpu().numpy().copy()


def hip_compress_segmented(keys, values, seg_offsets, plist):
    """Returns (host rc, device status, blob uint8, stream offsets uint64)."""
    n = int(np.asarray(values).size)
    nseg = len(seg_offsets) - 1
    min_kb = plist.block_keys if isinstance(plist, B.Params) else min(p.block_keys for p in plist)
    pmax = plist if isinstance(plist, B.Params) else B.params(1.1, 128, 5, min_kb)
    cap = B.compressed_size(max(n, 1), pmax) + (64 + 4096) * nseg
    out = torch.empty(cap // 8 + 8, dtype=torch.int64, device="cuda")
    ws = torch.empty(B.workspace_size(n, nseg, min_kb) // 8 + 32, dtype=torch.int64, device="cuda")
    offs = torch.full((nseg + 1,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    k, v = (None if keys is None else to_dev_u32(keys)), to_dev_f32(values)
    rc = B.compress_segmented(k, v, [int(x) for x in seg_offsets], plist, out, offs, status, ws)
    torch.cuda.synchronize()
    if rc != B.OK:
        return rc, None, None, None
    so = offs.cpu().numpy().astype(np.uint64)
    blob = out.view(torch.uint8)[:int(so[-1])].cpu().numpy().copy()
    return rc, int(status[0].item()), blob, so


def hip_decompress_segmented(blob, stream_offsets, capacity):
    """Returns (host rc, device status, keys, values, pair offsets)."""
    s = np.ascontiguousarray(blob, dtype=np.uint8)
    nseg = len(stream_offsets) - 1
    dev = torch.from_numpy(np.concatenate([s, np.zeros((-s.size) % 8 + 8, np.uint8)])).cuda()
    so = torch.from_numpy(np.ascontiguousarray(stream_offsets, dtype=np.uint64).view(np.int64)).cuda()
    keys_out = torch.empty(max(capacity, 1), dtype=torch.int32, device="cuda")
    vals_out = torch.empty(max(capacity, 1), dtype=torch.float32, device="cuda")
    po = torch.full((nseg + 1,), -1, dtype=torch.int64, device="cuda")
    status = torch.full((2,), -1, dtype=torch.int32, device="cuda")
    ws = B.decoder_workspace(nseg)
    rc = B.lib().fastsgd_decompress_segmented(B._p(dev), s.size, B._p(so), nseg, B._p(keys_out), B._p(vals_out),
                                              int(capacity), B._p(po), B._p(status), B._p(ws),
                                              ws.numel() * 8, B._stream())
    torch.cuda.synchronize()
    if rc != B.OK:
        return rc, None, None, None, None
    pon = po.cpu().numpy().astype(np.uint64)
    c = int(pon[-1])
    return rc, int(status[0].item()), keys_out[:c].cpu().numpy().view(np.uint32).copy(), vals_out[:c].cpu().numpy().copy(), pon
