"""ctypes front end of the CPU oracle (oracle/lc_oracle.c).

TEST INFRASTRUCTURE: only tests, the smoke check and the benchmark's
cpu_baseline leg may import this module.  It never touches the HIP library.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lc_oracle.c")
_LIB = os.path.join(_HERE, "liblc_oracle.so")

OK, BADARG, NONFINITE, OUT_TOO_SMALL, BAD_BLOB = 0, 1, 2, 3, 4


def build(force=False):
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-Wall", "-Wextra", "-ffp-contract=off", "-fno-fast-math",
             "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        u64, i64, i32, u32, vp = ctypes.c_uint64, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, ctypes.c_void_p
        L.lco_bucket_stats.restype = i32
        L.lco_bucket_stats.argtypes = [vp, vp, u64, vp, vp, vp]
        L.lco_promote.restype = i32
        L.lco_promote.argtypes = [vp, i32, vp, vp]
        L.lco_representative.restype = u32
        L.lco_representative.argtypes = [u32, u32, u32]
        L.lco_huffman_lengths.restype = None
        L.lco_huffman_lengths.argtypes = [vp, i32, vp]
        L.lco_canonical_codes.restype = None
        L.lco_canonical_codes.argtypes = [vp, i32, vp]
        L.lco_quantize.restype = i32
        L.lco_quantize.argtypes = [vp, vp, u64, i32, vp, vp, vp]
        L.lco_encode_bound.restype = u64
        L.lco_encode_bound.argtypes = [u64, i32]
        L.lco_encode.restype = i64
        L.lco_encode.argtypes = [vp, vp, u64, i32, vp, u64]
        L.lco_encode_cached.restype = i64
        L.lco_encode_cached.argtypes = [vp, vp, u64, i32, vp, u64, vp, vp]
        L.lco_decode.restype = i64
        L.lco_decode.argtypes = [vp, u64, vp, u64]
        L.lco_accounting.restype = i32
        L.lco_accounting.argtypes = [vp, vp]
        L.lco_size_exponent_only.restype = u64
        L.lco_size_exponent_only.argtypes = [u64, u32, u32]
        L.lco_bucket_stats64.restype = i32
        L.lco_bucket_stats64.argtypes = [vp, vp, u64, vp, vp, vp]
        L.lco_promote64.restype = i32
        L.lco_promote64.argtypes = [vp, i32, vp, vp]
        L.lco_representative64.restype = u64
        L.lco_representative64.argtypes = [u32, u64, u64]
        L.lco_quantize64.restype = i32
        L.lco_quantize64.argtypes = [vp, vp, u64, i32, vp, vp, vp]
        L.lco_encode64.restype = i64
        L.lco_encode64.argtypes = [vp, vp, u64, i32, vp, u64]
        L.lco_encode_cached64.restype = i64
        L.lco_encode_cached64.argtypes = [vp, vp, u64, i32, vp, u64, vp, vp]
        L.lco_decode64.restype = i64
        L.lco_decode64.argtypes = [vp, u64, vp, u64]
        _lib = L
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


class OracleError(RuntimeError):
    def __init__(self, status):
        super().__init__("oracle status %d" % status)
        self.status = status


def bucket_stats(w, w_ref):
    w, w_ref = _f32(w), _f32(w_ref)
    count = np.zeros(512, np.uint64); mmin = np.zeros(512, np.uint32); mmax = np.zeros(512, np.uint32)
    st = lib().lco_bucket_stats(_p(w), _p(w_ref), w.size, _p(count), _p(mmin), _p(mmax))
    return st, count, mmin, mmax


def promote(count, nbits):
    count = np.ascontiguousarray(count, dtype=np.uint64)
    kept = np.zeros(16, np.uint16); sym = np.zeros(512, np.uint8)
    K = lib().lco_promote(_p(count), nbits, _p(kept), _p(sym))
    return K, kept[:K].copy(), sym


def representative(bucket, mmin, mmax):
    return int(lib().lco_representative(int(bucket), int(mmin), int(mmax)))


def huffman_lengths(cnt):
    cnt = np.ascontiguousarray(cnt, dtype=np.uint64)
    assert cnt.size <= 16
    out = np.zeros(cnt.size, np.uint8)
    lib().lco_huffman_lengths(_p(cnt), cnt.size, _p(out))
    return out


def canonical_codes(lens):
    lens = np.ascontiguousarray(lens, dtype=np.uint8)
    out = np.zeros(lens.size, np.uint16)
    lib().lco_canonical_codes(_p(lens), lens.size, _p(out))
    return out


def quantize(w, w_ref, nbits):
    """Symbols and dequantized deltas in memory order: (sym u8[n], dq f32[n], K, k_E)."""
    w, w_ref = _f32(w), _f32(w_ref)
    sym = np.zeros(w.size, np.uint8); dq = np.zeros(w.size, np.float32); info = np.zeros(2, np.uint32)
    st = lib().lco_quantize(_p(w), _p(w_ref), w.size, nbits, _p(sym), _p(dq), _p(info))
    if st != OK:
        raise OracleError(st)
    return sym, dq, int(info[0]), int(info[1])


def encode_bound(n, nbits):
    return int(lib().lco_encode_bound(n, nbits))


def encode(w, w_ref, nbits, cap=None):
    """Returns the blob as a uint8 array (exact size).  Raises OracleError."""
    w, w_ref = _f32(w), _f32(w_ref)
    assert w.size == w_ref.size
    if cap is None:
        cap = encode_bound(w.size, min(max(nbits, 1), 4))
    out = np.zeros(max(cap, 1), np.uint8)
    r = lib().lco_encode(_p(w), _p(w_ref), w.size, nbits, _p(out), cap)
    if r < 0:
        err = OracleError(-r)
        err.header = out[:512].copy()
        raise err
    return out[:r].copy()


CACHE_WORDS = 36    # valid, nbits, K, pad, kept[16], len[16]: uint32 each


def new_cache():
    """An empty table cache for encode_cached."""
    return np.zeros(CACHE_WORDS, np.uint32)


def encode_cached(w, w_ref, nbits, cache):
    """Section 3.2 table caching: returns (blob, used_cache); `cache` (from new_cache) is updated in place."""
    w, w_ref = _f32(w), _f32(w_ref)
    assert w.size == w_ref.size and cache.dtype == np.uint32 and cache.size == CACHE_WORDS
    cap = encode_bound(w.size, min(max(nbits, 1), 4))
    out = np.zeros(max(cap, 1), np.uint8)
    used = ctypes.c_int(0)
    r = lib().lco_encode_cached(_p(w), _p(w_ref), w.size, nbits, _p(out), cap, _p(cache), ctypes.byref(used))
    if r < 0:
        err = OracleError(-r)
        err.header = out[:512].copy()
        raise err
    return out[:r].copy(), bool(used.value)


def decode(blob, w_ref):
    """Updates w_ref (float32 contiguous numpy array) in place; returns bytes consumed."""
    assert w_ref.dtype == np.float32 and w_ref.flags.c_contiguous
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    r = lib().lco_decode(_p(blob), blob.size, _p(w_ref), w_ref.size)
    if r < 0:
        raise OracleError(-r)
    return int(r)


# ---- binary64 parameters (Section 3.1.1, footnote on the bucket count: sign and 11 exponent bits, at most 2^12 buckets)
def _f64(a):
    return np.ascontiguousarray(a, dtype=np.float64)


def bucket_stats64(w, w_ref):
    w, w_ref = _f64(w), _f64(w_ref)
    count = np.zeros(4096, np.uint64); mmin = np.zeros(4096, np.uint64); mmax = np.zeros(4096, np.uint64)
    st = lib().lco_bucket_stats64(_p(w), _p(w_ref), w.size, _p(count), _p(mmin), _p(mmax))
    return st, count, mmin, mmax


def promote64(count, nbits):
    count = np.ascontiguousarray(count, dtype=np.uint64)
    kept = np.zeros(16, np.uint16); sym = np.zeros(4096, np.uint8)
    K = lib().lco_promote64(_p(count), nbits, _p(kept), _p(sym))
    return K, kept[:K].copy(), sym


def representative64(bucket, mmin, mmax):
    return int(lib().lco_representative64(int(bucket), int(mmin), int(mmax)))


def quantize64(w, w_ref, nbits):
    w, w_ref = _f64(w), _f64(w_ref)
    sym = np.zeros(w.size, np.uint8); dq = np.zeros(w.size, np.float64); info = np.zeros(2, np.uint32)
    st = lib().lco_quantize64(_p(w), _p(w_ref), w.size, nbits, _p(sym), _p(dq), _p(info))
    if st != OK:
        raise OracleError(st)
    return sym, dq, int(info[0]), int(info[1])


def encode64(w, w_ref, nbits):
    w, w_ref = _f64(w), _f64(w_ref)
    assert w.size == w_ref.size
    cap = encode_bound(w.size, min(max(nbits, 1), 4))
    out = np.zeros(max(cap, 1), np.uint8)
    r = lib().lco_encode64(_p(w), _p(w_ref), w.size, nbits, _p(out), cap)
    if r < 0:
        err = OracleError(-r)
        err.header = out[:512].copy()
        raise err
    return out[:r].copy()


def encode_cached64(w, w_ref, nbits, cache):
    """Section 3.2 table caching for binary64 parameters: returns (blob, used_cache); `cache` is updated in place."""
    w, w_ref = _f64(w), _f64(w_ref)
    assert w.size == w_ref.size and cache.dtype == np.uint32 and cache.size == CACHE_WORDS
    cap = encode_bound(w.size, min(max(nbits, 1), 4))
    out = np.zeros(max(cap, 1), np.uint8)
    used = ctypes.c_int(0)
    r = lib().lco_encode_cached64(_p(w), _p(w_ref), w.size, nbits, _p(out), cap, _p(cache), ctypes.byref(used))
    if r < 0:
        err = OracleError(-r)
        err.header = out[:512].copy()
        raise err
    return out[:r].copy(), bool(used.value)


def decode64(blob, w_ref):
    """Updates w_ref (float64 contiguous numpy array) in place; returns bytes consumed."""
    assert w_ref.dtype == np.float64 and w_ref.flags.c_contiguous
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    r = lib().lco_decode64(_p(blob), blob.size, _p(w_ref), w_ref.size)
    if r < 0:
        raise OracleError(-r)
    return int(r)


# ---- 16-bit parameters.  The method works on the fp32 delta (Algorithm 1 line 4), so parameters stored as bf16 or
# fp16 are widened exactly to fp32, coded as fp32, and the restored value fl32(w_ref + rep) is rounded once, to nearest
# even, back to the storage type.  The blob says which type it restores (header offset 60: 0 fp32, 1 bf16, 2 fp16).
DT_F32, DT_BF16, DT_F16, DT_F64 = 0, 1, 2, 3


def widen(a, dtype):
    """Exact conversion to float32. bf16 arrays are uint16 bit patterns, fp16 arrays are numpy float16."""
    if dtype == DT_F32:
        return _f32(a)
    if dtype == DT_F16:
        assert a.dtype == np.float16
        return np.ascontiguousarray(a).astype(np.float32)
    assert dtype == DT_BF16 and a.dtype == np.uint16
    return (np.ascontiguousarray(a).astype(np.uint32) << 16).view(np.float32)


def narrow(x, dtype):
    """Round finite float32 values to the storage type, to nearest, ties to even."""
    x = _f32(x)
    if dtype == DT_F32:
        return x
    if dtype == DT_F16:
        return x.astype(np.float16)
    bits = x.view(np.uint32).astype(np.uint64)
    return ((bits + 0x7FFF + ((bits >> 16) & 1)) >> 16).astype(np.uint16)


def encode_t(w, w_ref, nbits, dtype):
    if dtype == DT_F64:
        return encode64(w, w_ref, nbits)
    blob = encode(widen(w, dtype), widen(w_ref, dtype), nbits)
    blob[60:64] = np.frombuffer(np.uint32(dtype).tobytes(), np.uint8)
    return blob


def encode_cached_t(w, w_ref, nbits, dtype, cache):
    """encode_cached on the exactly widened vectors (16-bit storage types code the fp32 delta, as in encode_t);
    the blob names the storage type.  Returns (blob, used_cache)."""
    if dtype == DT_F64:
        return encode_cached64(w, w_ref, nbits, cache)
    assert dtype in (DT_F32, DT_BF16, DT_F16)
    blob, used = encode_cached(widen(w, dtype), widen(w_ref, dtype), nbits, cache)
    blob[60:64] = np.frombuffer(np.uint32(dtype).tobytes(), np.uint8)
    return blob, used


def decode_t(blob, w_ref, dtype):
    """Updates w_ref (storage type array) in place; returns bytes consumed."""
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    if dtype == DT_F64:
        return decode64(blob, w_ref)
    if blob.size >= 64 and int(np.frombuffer(blob[60:64].tobytes(), np.uint32)[0]) != dtype:
        raise OracleError(1)
    as_f32 = blob.copy()
    if as_f32.size >= 64:
        as_f32[60:64] = 0
    tmp = widen(w_ref, dtype).copy()
    r = decode(as_f32, tmp)
    w_ref[...] = narrow(tmp, dtype)
    return r


def accounting(blob):
    blob = np.ascontiguousarray(blob, dtype=np.uint8)
    acct = np.zeros(5, np.float64)
    st = lib().lco_accounting(_p(blob), _p(acct))
    if st != OK:
        raise OracleError(st)
    return dict(bits_E=acct[0], bits_EP=acct[1], bits_EPH=acct[2], entropy=acct[3], mean_len=acct[4])


def size_exponent_only(n, k, b=32):
    return int(lib().lco_size_exponent_only(n, k, b))
