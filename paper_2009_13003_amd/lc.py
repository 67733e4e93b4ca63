"""Thin ctypes binding of liblc.so: argument marshalling only, same names as include/lc.h.

Device buffers are torch CUDA tensors (torch is used for device memory and streams,
nothing else).  There is no CPU fallback: if the library is missing, importing fails.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_PATH = os.path.join(_HERE, "liblc.so")
if not os.path.exists(_PATH):
    raise ImportError("liblc.so is not built: run `python -m paper_2009_13003_amd.build` "
                      "(or __graft_entry__.build()) first")
_lib = ctypes.CDLL(_PATH)

OK, ERR_BADARG, ERR_NONFINITE, ERR_OUT_TOO_SMALL, ERR_BAD_BLOB, ERR_HIP, ERR_WORKSPACE = range(7)
MAX_N = 1 << 32
MAX_TICKETS = 32
MAX_MANY = 64
CHUNK = 16384

_u64, _i64, _int, _vp, _sz = ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t
_lib.lc_encode_bound.restype = _sz
_lib.lc_encode_bound.argtypes = [_u64, _int]
_lib.lc_workspace_bytes.restype = _sz
_lib.lc_workspace_bytes.argtypes = [_u64, _int]
_lib.lc_set_workspace.restype = _int
_lib.lc_set_workspace.argtypes = [_vp, _sz]
_lib.lc_encode.restype = _i64
_lib.lc_encode.argtypes = [_vp, _vp, _u64, _int, _vp, _vp]
_lib.lc_set_option.restype = _int
_lib.lc_set_option.argtypes = [_int, _int]
_lib.lc_encode_sized.restype = _i64
_lib.lc_encode_sized.argtypes = [_vp, _vp, _u64, _int, _vp, _sz, _int, _vp]
_lib.lc_decode_sized.restype = _i64
_lib.lc_decode_sized.argtypes = [_vp, _sz, _vp, _u64, _int, _vp]
_lib.lc_verify.restype = _i64
_lib.lc_verify.argtypes = [_vp, _sz, _u64, _int, _vp]
_lib.lc_encode_static.restype = _int
_lib.lc_encode_static.argtypes = [_vp, _vp, _u64, _int, _vp, _vp]
_lib.lc_encode_t.restype = _i64
_lib.lc_encode_t.argtypes = [_vp, _vp, _u64, _int, _vp, _int, _vp]
_lib.lc_decode_t.restype = _i64
_lib.lc_decode_t.argtypes = [_vp, _vp, _u64, _int, _vp]
_lib.lc_batch_workspace_bytes.restype = _sz
_lib.lc_batch_workspace_bytes.argtypes = [ctypes.POINTER(_u64), _int, _int]
_lib.lc_encode_batch.restype = _i64
_lib.lc_encode_batch.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_u64), _int, _int,
                                 ctypes.POINTER(_vp), ctypes.POINTER(_i64), _vp]
_lib.lc_encode_batch_t.restype = _i64
_lib.lc_encode_batch_t.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_u64), _int, _int,
                                   ctypes.POINTER(_vp), ctypes.POINTER(_i64), _int, _vp]
_lib.lc_decode_batch_t.restype = _i64
_lib.lc_decode_batch_t.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_u64), _int, ctypes.POINTER(_i64), _int, _vp]
_lib.lc_decode_batch.restype = _i64
_lib.lc_decode_batch.argtypes = [ctypes.POINTER(_vp), ctypes.POINTER(_vp), ctypes.POINTER(_u64), _int, ctypes.POINTER(_i64), _vp]
_lib.lc_encode_cached.restype = _i64
_lib.lc_encode_cached.argtypes = [_vp, _vp, _u64, _int, _vp, _vp, ctypes.POINTER(_int), _vp]
_lib.lc_encode_cached_t.restype = _i64
_lib.lc_encode_cached_t.argtypes = [_vp, _vp, _u64, _int, _vp, _int, _vp, ctypes.POINTER(_int), _vp]
_lib.lc_encode_async_t.restype = _int
_lib.lc_encode_async_t.argtypes = [_vp, _vp, _u64, _int, _vp, _int, _vp, _vp]
_lib.lc_encode_async.restype = _int
_lib.lc_encode_async.argtypes = [_vp, _vp, _u64, _int, _vp, _vp, _vp]
_lib.lc_encode_release_inputs.restype = _int
_lib.lc_encode_release_inputs.argtypes = [_int, _vp]
_lib.lc_encode_wait.restype = _i64
_lib.lc_encode_wait.argtypes = [_int, ctypes.POINTER(_int)]
_lib.lc_decode.restype = _i64
_lib.lc_decode.argtypes = [_vp, _vp, _u64, _vp]
_lib.lc_decode_many.restype = _i64
_lib.lc_decode_many_t.restype = _i64
_lib.lc_decode_many_t.argtypes = [ctypes.POINTER(_vp), _int, _vp, _u64, _int, _vp]
_lib.lc_decode_many.argtypes = [ctypes.POINTER(_vp), _int, _vp, _u64, _vp]
_lib.lc_blob_info.restype = _int
_lib.lc_blob_info.argtypes = [_vp, ctypes.POINTER(_u64), ctypes.POINTER(_int), ctypes.POINTER(_u64), ctypes.POINTER(_int)]
_lib.lc_blob_sizes.restype = _int
_lib.lc_blob_sizes.argtypes = [_vp, ctypes.POINTER(_u64)]
_lib.lc_shutdown.restype = None
_lib.lc_shutdown.argtypes = []
_lib.lc_strerror.restype = ctypes.c_char_p
_lib.lc_strerror.argtypes = [_int]
_lib.lc_profile.restype = _int
_lib.lc_profile.argtypes = [_int]
_lib.lc_profile_read.restype = _int
_lib.lc_profile_read.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(_u64), _int]
_lib.lc_profile_name.restype = ctypes.c_char_p
_lib.lc_profile_name.argtypes = [_int]


class LcError(RuntimeError):
    def __init__(self, status):
        super().__init__("lc status %d: %s" % (status, lc_strerror(status)))
        self.status = status


def lc_strerror(status):
    return _lib.lc_strerror(int(status)).decode()


def lc_encode_bound(n, nbits):
    return int(_lib.lc_encode_bound(n, nbits))


def lc_workspace_bytes(n, nbits):
    return int(_lib.lc_workspace_bytes(n, nbits))


try:                                    # torch's current stream as a raw handle, without building a Stream object
    _raw_current_stream = torch._C._cuda_getCurrentRawStream
    _current_device = torch._C._cuda_getDevice
except AttributeError:                  # (other torch builds: the public, slower way)
    _raw_current_stream = None


def _stream(stream):
    if stream is None:
        if _raw_current_stream is not None:
            return ctypes.c_void_p(_raw_current_stream(_current_device()))
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _dev_f32(t):
    assert t.is_cuda and t.dtype == torch.float32 and t.is_contiguous(), "need a contiguous CUDA float32 tensor"
    return ctypes.c_void_p(t.data_ptr())


def lc_set_workspace(ws):
    """ws: a CUDA uint8 tensor (kept alive by the caller) or None."""
    if ws is None:
        return int(_lib.lc_set_workspace(None, 0))
    assert ws.is_cuda and ws.dtype == torch.uint8 and ws.is_contiguous()
    return int(_lib.lc_set_workspace(ctypes.c_void_p(ws.data_ptr()), ws.numel()))


def lc_encode(w, w_ref, nbits, out, stream=None, n=None):
    """Returns the blob size in bytes (blob is out[:size]); raises LcError on a negative status."""
    n = w.numel() if n is None else n
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    r = int(_lib.lc_encode(_dev_f32(w), _dev_f32(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


STATIC_MAX_N = 1 << 23


def lc_encode_static(w, w_ref, nbits, out, stream=None, n=None):
    """lc_encode without any allocation and without waiting: enqueues only; the blob's size and status are in its
    header once the stream has run the call.  Raises LcError on a status other than LC_OK."""
    n = w.numel() if n is None else n
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    st = int(_lib.lc_encode_static(_dev_f32(w), _dev_f32(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), _stream(stream)))
    if st != OK:
        raise LcError(st)


DTYPES = {torch.float32: 0, torch.bfloat16: 1, torch.float16: 2, torch.float64: 3}


def _dev_any(t):
    assert t.is_cuda and t.dtype in DTYPES and t.is_contiguous(), "need a contiguous CUDA float32 / bfloat16 / float16 / float64 tensor"
    return ctypes.c_void_p(t.data_ptr())


def lc_encode_t(w, w_ref, nbits, out, stream=None, n=None):
    """lc_encode for float32, bfloat16, float16 or float64 parameters (w and w_ref of the same dtype)."""
    n = w.numel() if n is None else n
    assert w.dtype == w_ref.dtype
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    r = int(_lib.lc_encode_t(_dev_any(w), _dev_any(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), DTYPES[w.dtype], _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_decode_t(blob, w_ref, stream=None, n=None):
    """lc_decode for float32, bfloat16, float16 or float64 parameters."""
    n = w_ref.numel() if n is None else n
    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    r = int(_lib.lc_decode_t(ctypes.c_void_p(blob.data_ptr()), _dev_any(w_ref), n, DTYPES[w_ref.dtype], _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


OPT_KEY_STAGING, STAGING_AUTO, STAGING_ALWAYS, STAGING_NEVER = 1, 0, 1, 2
OPT_VERIFY_FIRST = 2


def lc_set_option(option, value):
    st = int(_lib.lc_set_option(option, value))
    if st != OK:
        raise LcError(st)


def lc_encode_sized(w, w_ref, nbits, out, stream=None, n=None):
    """lc_encode_t with the size of `out` stated: ERR_OUT_TOO_SMALL if it is below lc_encode_bound."""
    n = w.numel() if n is None else n
    assert w.dtype == w_ref.dtype and out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    r = int(_lib.lc_encode_sized(_dev_any(w), _dev_any(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), out.numel(),
                                 DTYPES[w.dtype], _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_decode_sized(blob, w_ref, stream=None, n=None):
    """lc_decode_t with the size of `blob` stated: a header that claims more bytes is refused."""
    n = w_ref.numel() if n is None else n
    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    r = int(_lib.lc_decode_sized(ctypes.c_void_p(blob.data_ptr()), blob.numel(), _dev_any(w_ref), n, DTYPES[w_ref.dtype],
                                 _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


class EncodeBatch:
    """The marshalled arguments of one lc_encode_batch call, kept for the next call on the same tensors: a
    training loop checkpoints the same parameter tensors every time, and checking and converting a few hundred
    tensors costs more host time than the call.  The tensors must stay alive and in place."""

    def __init__(self, ws, w_refs, nbits, outs):
        count = len(ws)
        assert count == len(w_refs) == len(outs) and count >= 1
        self.dtype = ws[0].dtype                             # float32, bfloat16 or float16, the same for every tensor
        for w, r, o in zip(ws, w_refs, outs):
            assert w.is_cuda and w.dtype == self.dtype and w.is_contiguous() and r.is_cuda and r.dtype == self.dtype
            assert r.is_contiguous() and r.numel() == w.numel() and o.is_cuda and o.dtype == torch.uint8 and o.is_contiguous()
            assert o.numel() >= lc_encode_bound(w.numel(), nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
        self.keep = (list(ws), list(w_refs), list(outs))
        self.count, self.nbits = count, nbits
        self.wp = (_vp * count)(*[t.data_ptr() if t.numel() else None for t in ws])
        self.rp = (_vp * count)(*[t.data_ptr() if t.numel() else None for t in w_refs])
        self.op = (_vp * count)(*[t.data_ptr() for t in outs])
        self.ns = (_u64 * count)(*[t.numel() for t in ws])
        self.sizes = (_i64 * count)()

    def run(self, stream=None):
        if self.dtype == torch.float32:
            r = int(_lib.lc_encode_batch(self.wp, self.rp, self.ns, self.count, self.nbits, self.op, self.sizes, _stream(stream)))
        else:
            r = int(_lib.lc_encode_batch_t(self.wp, self.rp, self.ns, self.count, self.nbits, self.op, self.sizes,
                                           DTYPES[self.dtype], _stream(stream)))
        sizes = list(self.sizes)
        if r < 0 and all(s >= 0 for s in sizes):
            raise LcError(-r)
        return sizes


def lc_encode_batch(ws, w_refs, nbits, outs, stream=None):
    """One table per tensor, all tensors in one call. Returns the list of blob sizes (negative: -(status) of that
    tensor); raises LcError only for errors that concern the whole call."""
    return EncodeBatch(ws, w_refs, nbits, outs).run(stream)


lc_encode_batch_t = lc_encode_batch      # (EncodeBatch picks the entry point by the tensors' dtype)


def lc_blob_sizes(header_bytes):
    """Checkpoint size in bits after each stage (Section 4.3): dict(E, EP, EPH), from the first 64+ bytes of a blob."""
    buf = ctypes.create_string_buffer(bytes(header_bytes[:512]), 512)
    bits = (_u64 * 3)()
    st = int(_lib.lc_blob_sizes(buf, bits))
    if st != 0:
        raise LcError(st)
    return dict(E=int(bits[0]), EP=int(bits[1]), EPH=int(bits[2]))


class DecodeBatch:
    """The marshalled arguments of one lc_decode_batch call, kept for the next call on the same tensors (see EncodeBatch)."""

    def __init__(self, blobs, w_refs):
        count = len(blobs)
        assert count == len(w_refs) and count >= 1
        self.dtype = w_refs[0].dtype
        for b, r in zip(blobs, w_refs):
            assert b.is_cuda and b.dtype == torch.uint8 and b.is_contiguous()
            assert r.is_cuda and r.dtype == self.dtype and r.is_contiguous()
        self.keep = (list(blobs), list(w_refs))
        self.count = count
        self.bp = (_vp * count)(*[t.data_ptr() for t in blobs])
        self.rp = (_vp * count)(*[t.data_ptr() if t.numel() else None for t in w_refs])
        self.ns = (_u64 * count)(*[t.numel() for t in w_refs])
        self.sizes = (_i64 * count)()

    def run(self, stream=None):
        if self.dtype == torch.float32:
            r = int(_lib.lc_decode_batch(self.bp, self.rp, self.ns, self.count, self.sizes, _stream(stream)))
        else:
            r = int(_lib.lc_decode_batch_t(self.bp, self.rp, self.ns, self.count, self.sizes, DTYPES[self.dtype], _stream(stream)))
        sizes = list(self.sizes)
        if r < 0 and all(s >= 0 for s in sizes):
            raise LcError(-r)
        return sizes


def lc_decode_batch(blobs, w_refs, stream=None):
    """Restores every tensor from its blob in one call. Returns the list of bytes consumed (negative: -(status))."""
    return DecodeBatch(blobs, w_refs).run(stream)


lc_decode_batch_t = lc_decode_batch      # (DecodeBatch picks the entry point by the tensors' dtype)


CACHE_BYTES = 256


def new_cache(device="cuda"):
    """An empty code table cache for lc_encode_cached."""
    return torch.zeros(CACHE_BYTES, dtype=torch.uint8, device=device)


def lc_encode_cached(w, w_ref, nbits, out, cache, stream=None, n=None):
    """lc_encode with a code table cache (a tensor from new_cache). Returns (blob size, used_cache)."""
    n = w.numel() if n is None else n
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    assert cache.is_cuda and cache.dtype == torch.uint8 and cache.is_contiguous() and cache.numel() >= CACHE_BYTES
    used = _int(0)
    r = int(_lib.lc_encode_cached(_dev_f32(w), _dev_f32(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()),
                                  ctypes.c_void_p(cache.data_ptr()), ctypes.byref(used), _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r, bool(used.value)


def lc_encode_cached_t(w, w_ref, nbits, out, cache, stream=None, n=None):
    """lc_encode_cached for float32, bfloat16 or float16 parameters (w and w_ref of the same dtype)."""
    n = w.numel() if n is None else n
    assert w.dtype == w_ref.dtype
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    assert cache.is_cuda and cache.dtype == torch.uint8 and cache.is_contiguous() and cache.numel() >= CACHE_BYTES
    used = _int(0)
    r = int(_lib.lc_encode_cached_t(_dev_any(w), _dev_any(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), DTYPES[w.dtype],
                                    ctypes.c_void_p(cache.data_ptr()), ctypes.byref(used), _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r, bool(used.value)


def lc_encode_async_t(w, w_ref, nbits, out, cache=None, stream=None, n=None):
    """lc_encode_async for float32, bfloat16 or float16 parameters."""
    n = w.numel() if n is None else n
    assert w.dtype == w_ref.dtype
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    c = None
    if cache is not None:
        assert cache.is_cuda and cache.dtype == torch.uint8 and cache.is_contiguous() and cache.numel() >= CACHE_BYTES
        c = ctypes.c_void_p(cache.data_ptr())
    r = int(_lib.lc_encode_async_t(_dev_any(w), _dev_any(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), DTYPES[w.dtype], c,
                                   _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_encode_async(w, w_ref, nbits, out, cache=None, stream=None, n=None):
    """Enqueues lc_encode (or lc_encode_cached if `cache` is given) and returns a ticket at once."""
    n = w.numel() if n is None else n
    assert out.is_cuda and out.dtype == torch.uint8 and out.is_contiguous()
    assert out.numel() >= lc_encode_bound(n, nbits) > 0 or not (1 <= nbits <= 4), "out is smaller than lc_encode_bound"
    c = None
    if cache is not None:
        assert cache.is_cuda and cache.dtype == torch.uint8 and cache.is_contiguous() and cache.numel() >= CACHE_BYTES
        c = ctypes.c_void_p(cache.data_ptr())
    r = int(_lib.lc_encode_async(_dev_f32(w), _dev_f32(w_ref), n, nbits, ctypes.c_void_p(out.data_ptr()), c, _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_encode_release_inputs(ticket, stream=None):
    """Work enqueued on `stream` after this waits until the call has read w and w_ref for the last time."""
    r = int(_lib.lc_encode_release_inputs(ticket, _stream(stream)))
    if r != 0:
        raise LcError(r)


def lc_encode_wait(ticket):
    """Blocks until the call has finished. Returns (blob size, used_cache)."""
    used = _int(0)
    r = int(_lib.lc_encode_wait(ticket, ctypes.byref(used)))
    if r < 0:
        raise LcError(-r)
    return r, bool(used.value)


def lc_verify(blob, n, dtype=torch.float32, stream=None, blob_bytes=None):
    """Checks a blob from end to end (header, tables, offsets, every lane string) without touching any parameters;
    returns the blob's size in bytes; raises LcError on a negative status."""
    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    size = blob.numel() if blob_bytes is None else blob_bytes
    r = int(_lib.lc_verify(ctypes.c_void_p(blob.data_ptr()), size, n, DTYPES[dtype], _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_decode(blob, w_ref, stream=None, n=None):
    """Updates w_ref in place; returns the bytes consumed; raises LcError on a negative status."""
    n = w_ref.numel() if n is None else n
    assert blob.is_cuda and blob.dtype == torch.uint8 and blob.is_contiguous()
    r = int(_lib.lc_decode(ctypes.c_void_p(blob.data_ptr()), _dev_f32(w_ref), n, _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_decode_many(blobs, w_ref, stream=None, n=None):
    """Applies the blobs (a list of CUDA uint8 tensors) to w_ref in order; returns the bytes consumed."""
    n = w_ref.numel() if n is None else n
    for b in blobs:
        assert b.is_cuda and b.dtype == torch.uint8 and b.is_contiguous()
    ptrs = (_vp * len(blobs))(*[b.data_ptr() for b in blobs])
    r = int(_lib.lc_decode_many(ptrs, len(blobs), _dev_f32(w_ref), n, _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_decode_many_t(blobs, w_ref, stream=None, n=None):
    """lc_decode_many for float32, bfloat16 or float16 parameters."""
    n = w_ref.numel() if n is None else n
    for b in blobs:
        assert b.is_cuda and b.dtype == torch.uint8 and b.is_contiguous()
    ptrs = (_vp * len(blobs))(*[b.data_ptr() for b in blobs])
    r = int(_lib.lc_decode_many_t(ptrs, len(blobs), _dev_any(w_ref), n, DTYPES[w_ref.dtype], _stream(stream)))
    if r < 0:
        raise LcError(-r)
    return r


def lc_blob_info(host_header):
    """host_header: bytes-like, at least 64 bytes, in host memory."""
    buf = (ctypes.c_uint8 * 64).from_buffer_copy(bytes(host_header[:64]))
    n, nbits, total, status = _u64(), _int(), _u64(), _int()
    st = int(_lib.lc_blob_info(buf, ctypes.byref(n), ctypes.byref(nbits), ctypes.byref(total), ctypes.byref(status)))
    if st != OK:
        raise LcError(st)
    return dict(n=n.value, nbits=nbits.value, total_bytes=total.value, status=status.value)


def lc_shutdown():
    _lib.lc_shutdown()


def lc_profile(enable):
    st = int(_lib.lc_profile(1 if enable else 0))
    if st != OK:
        raise LcError(st)


def lc_profile_read():
    """{kernel name: (total ms, launches)} since lc_profile(True)."""
    k = int(_lib.lc_profile_read(None, None, 0))
    ms = (ctypes.c_double * k)()
    cnt = (_u64 * k)()
    _lib.lc_profile_read(ms, cnt, k)
    return {_lib.lc_profile_name(i).decode(): (ms[i], int(cnt[i])) for i in range(k)}


def alloc_out(n, nbits, device="cuda"):
    """A device buffer large enough for any blob of (n, nbits)."""
    return torch.empty(lc_encode_bound(n, nbits), dtype=torch.uint8, device=device)
