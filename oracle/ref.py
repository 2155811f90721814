"""ctypes view of the CPU oracle (oracle/fastsgd_ref.c) on numpy arrays.

Test infrastructure only: imported by tests, by the smoke check and by the benchmark's
CPU-baseline leg.  It neither imports nor is imported by the HIP path.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

OK, ERR_INVALID_ARG, ERR_BUFFER_TOO_SMALL, ERR_NONFINITE, ERR_UNSORTED_KEYS, ERR_CORRUPT_STREAM = range(6)


class Params(C.Structure):
    _fields_ = [("base", C.c_double), ("tau", C.c_uint32), ("flag_bits", C.c_uint32),
                ("block_keys", C.c_uint32), ("reserved", C.c_uint32)]


def params(base=1.1, tau=128, flag_bits=2, block_keys=1024):
    return Params(float(base), int(tau), int(flag_bits), int(block_keys), 0)


_lib = None


def load(path):
    """The oracle library at `path` with its prototypes declared (the tests of the pins load deliberately
    broken builds of the oracle through this)."""
    if True:        # (one block: the prototypes below)
        L = C.CDLL(path)
        u64, u32, vp = C.c_uint64, C.c_uint32, C.c_void_p
        L.fastsgd_ref_abs_sum.argtypes = [vp, u64, C.POINTER(C.c_double)]
        L.fastsgd_ref_abs_sum.restype = C.c_int
        L.fastsgd_ref_tables.argtypes = [C.c_double, C.c_double, u32, vp, vp]
        L.fastsgd_ref_tables.restype = None
        L.fastsgd_ref_compressed_size.argtypes = [u64, C.POINTER(Params)]
        L.fastsgd_ref_compressed_size.restype = u64
        L.fastsgd_ref_compress.argtypes = [vp, vp, u64, C.POINTER(Params), vp, u64, C.POINTER(u64)]
        L.fastsgd_ref_compress.restype = C.c_int
        L.fastsgd_ref_decompress.argtypes = [vp, u64, vp, vp, u64, C.POINTER(u64)]
        L.fastsgd_ref_decompress.restype = C.c_int
        L.fastsgd_ref_compress_segmented.argtypes = [vp, vp, vp, u32, C.POINTER(Params), u32, vp, u64, vp]
        L.fastsgd_ref_compress_segmented.restype = C.c_int
        L.fastsgd_ref_decompress_segmented.argtypes = [vp, vp, u32, vp, vp, u64, vp]
        L.fastsgd_ref_decompress_segmented.restype = C.c_int
        L.fastsgd_ref_decompress_accumulate.argtypes = [vp, vp, u32, vp, u64, C.POINTER(u64)]
        L.fastsgd_ref_decompress_accumulate.restype = C.c_int
        L.fastsgd_ref_decompress_adam.argtypes = [vp, u64, vp, vp, vp, u64, C.c_double, C.c_double, C.c_double,
                                                  C.c_double, C.POINTER(u64)]
        L.fastsgd_ref_decompress_adam.restype = C.c_int
        L.fastsgd_ref_key_tokens_text.argtypes = [vp, u32, u32, C.c_char_p, u64]
        L.fastsgd_ref_key_tokens_text.restype = u32
    return L


def lib():
    global _lib
    if _lib is None:
        _lib = load(_build.build(force=False))
    return _lib


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _u32(a):
    return np.ascontiguousarray(a, dtype=np.uint32)


def abs_sum(values):
    """(nonfinite, sum): the exact sum of |values| rounded once to float64."""
    v = _f32(values)
    s = C.c_double(0.0)
    bad = lib().fastsgd_ref_abs_sum(_ptr(v), v.size, C.byref(s))
    return bool(bad), s.value


def tables(s, base, tau):
    """Boundary bit patterns B[0..128] and decoded-magnitude bit patterns V[0..128] (index = code)."""
    B = np.zeros(257, np.uint32)
    V = np.zeros(257, np.uint32)
    lib().fastsgd_ref_tables(float(s), float(base), int(tau), _ptr(B), _ptr(V))
    return B, V


def compressed_size(n, p):
    return int(lib().fastsgd_ref_compressed_size(int(n), C.byref(p)))


def compress(keys, values, p, capacity=None):
    """(status, stream bytes as uint8 array)."""
    k, v = _u32(keys), _f32(values)
    assert k.size == v.size
    cap = compressed_size(v.size, p) if capacity is None else int(capacity)
    out = np.zeros(max(cap, 1), np.uint8)
    nbytes = C.c_uint64(0)
    rc = lib().fastsgd_ref_compress(_ptr(k), _ptr(v), v.size, C.byref(p), _ptr(out), cap, C.byref(nbytes))
    return rc, out[:nbytes.value].copy()


def decompress(stream, capacity=None):
    """(status, keys, values)."""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    if capacity is None:
        capacity = int(s[40:48].view("<u8")[0]) if s.size >= 64 else 0
        capacity = min(capacity, 1 << 32)
    keys = np.zeros(max(capacity, 1), np.uint32)
    vals = np.zeros(max(capacity, 1), np.float32)
    cnt = C.c_uint64(0)
    rc = lib().fastsgd_ref_decompress(_ptr(s), s.size, _ptr(keys), _ptr(vals), int(capacity), C.byref(cnt))
    return rc, keys[:cnt.value].copy(), vals[:cnt.value].copy()


def compress_segmented(keys, values, seg_offsets, plist):
    """plist: one Params (shared) or a list with one per segment.  (status, bytes, stream offsets)."""
    k, v = _u32(keys), _f32(values)
    so = np.ascontiguousarray(seg_offsets, dtype=np.uint64)
    nseg = so.size - 1
    if isinstance(plist, Params):
        arr, stride = (Params * 1)(plist), 0
        cap = sum(compressed_size(int(so[i + 1] - so[i]), plist) for i in range(nseg))
    else:
        arr, stride = (Params * nseg)(*plist), 1
        cap = sum(compressed_size(int(so[i + 1] - so[i]), plist[i]) for i in range(nseg))
    out = np.zeros(max(cap, 1), np.uint8)
    offs = np.zeros(nseg + 1, np.uint64)
    rc = lib().fastsgd_ref_compress_segmented(_ptr(k), _ptr(v), _ptr(so), nseg, arr, stride,
                                              _ptr(out), cap, _ptr(offs))
    return rc, out[:int(offs[-1])].copy(), offs


def decompress_segmented(streams, stream_offsets, capacity):
    s = np.ascontiguousarray(streams, dtype=np.uint8)
    so = np.ascontiguousarray(stream_offsets, dtype=np.uint64)
    nseg = so.size - 1
    keys = np.zeros(max(capacity, 1), np.uint32)
    vals = np.zeros(max(capacity, 1), np.float32)
    po = np.zeros(nseg + 1, np.uint64)
    rc = lib().fastsgd_ref_decompress_segmented(_ptr(s), _ptr(so), nseg, _ptr(keys), _ptr(vals),
                                                int(capacity), _ptr(po))
    return rc, keys[:int(po[-1])].copy(), vals[:int(po[-1])].copy(), po


def decompress_accumulate(streams, stream_offsets, dense):
    """dense[k] += v for every pair of every stream, in stream order; dense (float32) is updated in
    place.  Returns (status, pairs added)."""
    s = np.ascontiguousarray(streams, dtype=np.uint8)
    so = np.ascontiguousarray(stream_offsets, dtype=np.uint64)
    assert dense.dtype == np.float32 and dense.flags.c_contiguous
    cnt = C.c_uint64(0)
    rc = lib().fastsgd_ref_decompress_accumulate(_ptr(s), _ptr(so), so.size - 1, _ptr(dense), dense.size, C.byref(cnt))
    return rc, cnt.value


def decompress_adam(stream, theta, m, v, eta, beta1=0.9, beta2=0.999, eps=1e-8):
    """Adam step of Section 4.1 at the decoded keys of one stream; theta, m, v (float32) are updated in
    place.  Returns (status, pairs applied)."""
    s = np.ascontiguousarray(stream, dtype=np.uint8)
    for a in (theta, m, v):
        assert a.dtype == np.float32 and a.flags.c_contiguous and a.size == theta.size
    cnt = C.c_uint64(0)
    rc = lib().fastsgd_ref_decompress_adam(_ptr(s), s.size, _ptr(theta), _ptr(m), _ptr(v), theta.size, float(eta),
                                           float(beta1), float(beta2), float(eps), C.byref(cnt))
    return rc, cnt.value


def key_tokens_text(keys, flag_bits):
    """Algorithm 2 with one global M, tokens rendered as the paper prints them.  (M, text)."""
    k = _u32(keys)
    buf = C.create_string_buffer(40 * max(k.size, 1) + 8)
    M = lib().fastsgd_ref_key_tokens_text(_ptr(k), k.size, int(flag_bits), buf, len(buf))
    return int(M), buf.value.decode()
