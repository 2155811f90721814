"""Thin ctypes binding over libfastsgd.so (declared in include/fastsgd.h and include/fastsgd_profile.h).

Argument marshalling only: every step of the codec runs in the library's HIP kernels.  PyTorch is
used for device memory and for the current stream handle.  There is no CPU fallback: if the library
is missing or no GPU is present the calls raise.
"""
import ctypes as C
import os

import torch  # imported first so the HIP runtime torch ships is the one the library binds to

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libfastsgd.so")

OK, ERR_INVALID_ARG, ERR_BUFFER_TOO_SMALL, ERR_NONFINITE, ERR_UNSORTED_KEYS, ERR_CORRUPT_STREAM, ERR_DEVICE = range(7)
STATUS_NAMES = ["OK", "INVALID_ARG", "BUFFER_TOO_SMALL", "NONFINITE", "UNSORTED_KEYS", "CORRUPT_STREAM", "DEVICE"]

EXPORTS = ["fastsgd_compressed_size", "fastsgd_workspace_size", "fastsgd_workspace_size_tau", "fastsgd_decompress_workspace_size",
           "fastsgd_compress", "fastsgd_compress_static", "fastsgd_decompress", "fastsgd_compress_segmented", "fastsgd_decompress_segmented",
           "fastsgd_decompress_accumulate", "fastsgd_decompress_adam",
           "fastsgd_profile_compress", "fastsgd_profile_decompress", "fastsgd_probe_read"]
COMPRESS_KERNELS = ["abs_sum", "tables", "encode_values", "measure_keys", "pack_keys"]
DECOMPRESS_KERNELS = ["decode"]


class Params(C.Structure):
    """fastsgd_params"""
    _fields_ = [("base", C.c_double), ("tau", C.c_uint32), ("flag_bits", C.c_uint32),
                ("block_keys", C.c_uint32), ("reserved", C.c_uint32)]


class Adam(C.Structure):
    """fastsgd_adam"""
    _fields_ = [("eta", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double)]


def params(base=1.1, tau=128, flag_bits=2, block_keys=1024):
    return Params(float(base), int(tau), int(flag_bits), int(block_keys), 0)


_lib = None


def lib():
    """Load the library (building it first only if it has never been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            from . import build as _build
            _build.build(force=True)
        L = C.CDLL(LIB_PATH)
        u64, u32, vp, sz = C.c_uint64, C.c_uint32, C.c_void_p, C.c_size_t
        PP = C.POINTER(Params)
        L.fastsgd_compressed_size.argtypes = [u64, PP]
        L.fastsgd_compressed_size.restype = sz
        L.fastsgd_workspace_size.argtypes = [u64, u32, u32]
        L.fastsgd_workspace_size.restype = sz
        L.fastsgd_workspace_size_tau.argtypes = [u64, u32, u32, u32]
        L.fastsgd_workspace_size_tau.restype = sz
        L.fastsgd_decompress_workspace_size.argtypes = [u32]
        L.fastsgd_decompress_workspace_size.restype = sz
        L.fastsgd_compress.argtypes = [vp, vp, u64, PP, vp, sz, vp, vp, vp, sz, vp]
        L.fastsgd_compress.restype = C.c_int
        L.fastsgd_compress_static.argtypes = [vp, vp, u64, PP, vp, sz, vp, vp, vp]
        L.fastsgd_compress_static.restype = C.c_int
        L.fastsgd_decompress.argtypes = [vp, sz, vp, vp, u64, vp, vp, vp, sz, vp]
        L.fastsgd_decompress.restype = C.c_int
        L.fastsgd_compress_segmented.argtypes = [vp, vp, C.POINTER(u64), u32, PP, u32, vp, sz, vp, vp, vp, sz, vp]
        L.fastsgd_compress_segmented.restype = C.c_int
        L.fastsgd_decompress_segmented.argtypes = [vp, sz, vp, u32, vp, vp, u64, vp, vp, vp, sz, vp]
        L.fastsgd_decompress_segmented.restype = C.c_int
        L.fastsgd_decompress_accumulate.argtypes = [vp, sz, vp, u32, vp, u64, vp, vp, vp, sz, vp]
        L.fastsgd_decompress_accumulate.restype = C.c_int
        L.fastsgd_decompress_adam.argtypes = [vp, sz, vp, vp, vp, u64, C.POINTER(Adam), vp, vp, vp, sz, vp]
        L.fastsgd_decompress_adam.restype = C.c_int
        fp = C.POINTER(C.c_float)
        L.fastsgd_profile_compress.argtypes = [vp, vp, u64, PP, vp, sz, vp, vp, vp, sz, vp, u32, fp]
        L.fastsgd_profile_compress.restype = C.c_int
        L.fastsgd_profile_decompress.argtypes = [vp, sz, vp, vp, u64, vp, vp, vp, sz, vp, u32, fp]
        L.fastsgd_profile_decompress.restype = C.c_int
        L.fastsgd_probe_read.argtypes = [vp, sz, vp, vp]
        L.fastsgd_probe_read.restype = C.c_int
        _lib = L
    return _lib


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return C.c_void_p(t.data_ptr() if t is not None else 0)


def compressed_size(n, p):
    return int(lib().fastsgd_compressed_size(int(n), C.byref(p)))


def workspace_size(total_n, n_segments=1, min_block_keys=1024, max_tau=None):
    """Bytes of encoder workspace; with max_tau (the largest threshold the caller will pass) the smaller amount
    that thresholds up to 128 get by with."""
    if max_tau is None:
        return int(lib().fastsgd_workspace_size(int(total_n), int(n_segments), int(min_block_keys)))
    return int(lib().fastsgd_workspace_size_tau(int(total_n), int(n_segments), int(min_block_keys), int(max_tau)))


def decompress_workspace_size(n_segments=1):
    return int(lib().fastsgd_decompress_workspace_size(int(n_segments)))


def compress(keys, values, p, out, out_bytes, status, workspace, n=None, out_capacity=None):
    """fastsgd_compress on device tensors; returns the host-side status.  Asynchronous."""
    n = values.numel() if n is None else int(n)
    cap = out.numel() * out.element_size() if out_capacity is None else int(out_capacity)
    return lib().fastsgd_compress(_p(keys), _p(values), n, C.byref(p), _p(out), cap, _p(out_bytes), _p(status),
                                  _p(workspace), workspace.numel() * workspace.element_size(), _stream())


STATIC_MAX_ELEMS = 1 << 20


def compress_static(keys, values, p, out, out_bytes, status, n=None, out_capacity=None):
    """fastsgd_compress_static: fastsgd_compress on the library's own fixed workspace (n <= STATIC_MAX_ELEMS)."""
    n = values.numel() if n is None else int(n)
    cap = out.numel() * out.element_size() if out_capacity is None else int(out_capacity)
    return lib().fastsgd_compress_static(_p(keys), _p(values), n, C.byref(p), _p(out), cap, _p(out_bytes), _p(status),
                                         _stream())


def decompress(stream, stream_bytes, keys_out, values_out, count, status, workspace, capacity=None):
    """fastsgd_decompress on device tensors; returns the host-side status.  Asynchronous."""
    capacity = keys_out.numel() if capacity is None else int(capacity)
    return lib().fastsgd_decompress(_p(stream), int(stream_bytes), _p(keys_out), _p(values_out), capacity, _p(count),
                                    _p(status), _p(workspace), workspace.numel() * workspace.element_size(), _stream())


def profile_compress(keys, values, p, out, out_bytes, status, workspace, iterations, n=None, out_capacity=None):
    """fastsgd_profile_compress: (host status, {kernel name: average ms}).  Waits for the stream."""
    n = values.numel() if n is None else int(n)
    cap = out.numel() * out.element_size() if out_capacity is None else int(out_capacity)
    ms = (C.c_float * len(COMPRESS_KERNELS))()
    rc = lib().fastsgd_profile_compress(_p(keys), _p(values), n, C.byref(p), _p(out), cap, _p(out_bytes), _p(status),
                                        _p(workspace), workspace.numel() * workspace.element_size(), _stream(),
                                        int(iterations), ms)
    return rc, dict(zip(COMPRESS_KERNELS, [float(x) for x in ms]))


def profile_decompress(stream, stream_bytes, keys_out, values_out, count, status, workspace, iterations, capacity=None):
    """fastsgd_profile_decompress: (host status, {kernel name: average ms}).  Waits for the stream."""
    capacity = keys_out.numel() if capacity is None else int(capacity)
    ms = (C.c_float * len(DECOMPRESS_KERNELS))()
    rc = lib().fastsgd_profile_decompress(_p(stream), int(stream_bytes), _p(keys_out), _p(values_out), capacity,
                                          _p(count), _p(status), _p(workspace),
                                          workspace.numel() * workspace.element_size(), _stream(), int(iterations), ms)
    return rc, dict(zip(DECOMPRESS_KERNELS, [float(x) for x in ms]))


def probe_read(src, sink):
    """fastsgd_probe_read over the whole device tensor `src`: a plain streaming read, to be timed by the caller."""
    return lib().fastsgd_probe_read(_p(src), src.numel() * src.element_size(), _p(sink), _stream())


def _params_array(plist, n_segments):
    if isinstance(plist, Params):
        return (Params * 1)(plist), 0
    assert len(plist) == n_segments
    return (Params * n_segments)(*plist), 1


def compress_segmented(keys, values, seg_offsets, plist, out, out_seg_offsets, status, workspace):
    """fastsgd_compress_segmented; seg_offsets is a host sequence of n_segments+1 element offsets."""
    nseg = len(seg_offsets) - 1
    offs = (C.c_uint64 * (nseg + 1))(*[int(x) for x in seg_offsets])
    arr, stride = _params_array(plist, nseg)
    return lib().fastsgd_compress_segmented(_p(keys), _p(values), offs, nseg, arr, stride, _p(out),
                                            out.numel() * out.element_size(), _p(out_seg_offsets), _p(status),
                                            _p(workspace), workspace.numel() * workspace.element_size(), _stream())


def decompress_segmented(streams, total_bytes, stream_offsets, n_segments, keys_out, values_out, pair_offsets, status,
                         workspace):
    """fastsgd_decompress_segmented; stream_offsets and pair_offsets are device uint64 tensors."""
    return lib().fastsgd_decompress_segmented(_p(streams), int(total_bytes), _p(stream_offsets), int(n_segments),
                                              _p(keys_out), _p(values_out), keys_out.numel(), _p(pair_offsets),
                                              _p(status), _p(workspace),
                                              workspace.numel() * workspace.element_size(), _stream())


def decompress_adam(stream, stream_bytes, theta, m, v, eta, beta1, beta2, eps, count, status, workspace):
    """fastsgd_decompress_adam; theta, m, v are device float32 tensors of one length."""
    h = Adam(float(eta), float(beta1), float(beta2), float(eps))
    return lib().fastsgd_decompress_adam(_p(stream), int(stream_bytes), _p(theta), _p(m), _p(v), theta.numel(),
                                         C.byref(h), _p(count), _p(status), _p(workspace),
                                         workspace.numel() * workspace.element_size(), _stream())


def decompress_accumulate(streams, total_bytes, stream_offsets, n_streams, dense, count, status, workspace):
    """fastsgd_decompress_accumulate; stream_offsets is a device uint64 tensor, dense a device float32 tensor."""
    return lib().fastsgd_decompress_accumulate(_p(streams), int(total_bytes), _p(stream_offsets), int(n_streams),
                                               _p(dense), dense.numel(), _p(count), _p(status), _p(workspace),
                                               workspace.numel() * workspace.element_size(), _stream())


def decoder_workspace(n_segments=1, device="cuda"):
    """A decoder workspace for n_segments streams, its control words cleared (the library asks for that
    once, before the first use, and leaves them clear after every call)."""
    return torch.zeros(decompress_workspace_size(n_segments) // 8 + 32, dtype=torch.int64, device=device)


# ----------------------------------------------------------------------------------------------------
# Buffer plumbing for callers that do not manage their own device memory (tests, benchmark, smoke).
class Buffers:
    """Device buffers sized for gradients of up to n elements in n_segments segments."""

    def __init__(self, n, p, n_segments=1, device="cuda", out_capacity=None, min_block_keys=None):
        kb = p.block_keys if min_block_keys is None else min_block_keys
        self.device = torch.device(device)
        self.n = int(n)
        self.n_segments = int(n_segments)
        cap = out_capacity if out_capacity is not None else compressed_size(n, p) + 80 * n_segments + 4096 * n_segments
        self.out = torch.empty((cap + 7) // 8, dtype=torch.int64, device=self.device)
        self.out_capacity = cap
        self.workspace = torch.empty(workspace_size(n, n_segments, kb) // 8 + 32, dtype=torch.int64, device=self.device)
        self.dec_workspace = decoder_workspace(n_segments, self.device)
        self.out_offsets = torch.zeros(n_segments + 1, dtype=torch.int64, device=self.device)
        self.pair_offsets = torch.zeros(n_segments + 1, dtype=torch.int64, device=self.device)
        self.status = torch.zeros(2, dtype=torch.int32, device=self.device)
        self.keys_out = torch.empty(max(n, 1), dtype=torch.int32, device=self.device)
        self.values_out = torch.empty(max(n, 1), dtype=torch.float32, device=self.device)

    def out_bytes_view(self):
        return self.out.view(torch.uint8)
