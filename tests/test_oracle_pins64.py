"""Pins for the binary64 part of the CPU oracle (Section 3.1.1, footnote on the bucket count: sign and 11 exponent
bits, at most 2^12 buckets): exact rational arithmetic for the representative, an independent numpy quantizer, the
independent blob reader, closed forms and the relation to the binary32 path.  CPU only."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import lc_oracle as orc
from tests import lcb1_reader


def bits64(a):
    return np.ascontiguousarray(a, dtype=np.float64).view(np.uint64)


def rand_case64(n, seed, scale=1e-3, zero_frac=0.0):
    rng = np.random.default_rng(seed)
    w_ref = 0.05 * rng.standard_normal(n)
    d = rng.laplace(0.0, scale, n)
    if zero_frac:
        d[rng.random(n) < zero_frac] = 0.0
    return w_ref + d, w_ref


def np_quantize64(w, w_ref, nbits):
    """Section 3.1.1 on values: buckets by the top 12 bits, keep the 2^x-1 non-empty normal buckets of largest
    exponent (+ before -), midrange of the members' max and min rounded once (exact rationals), everything else 0."""
    d = w - w_ref
    b = (d.view(np.uint64) >> np.uint64(52)).astype(np.int64)
    normal = (b & 2047) != 0
    cand = sorted(set(int(x) for x in b[normal]), key=lambda x: (-(x & 2047), x >> 11))
    kept = cand[:2 ** nbits - 1]
    K = len(kept)
    sym = np.full(d.size, K, np.uint8)
    dq = np.zeros(d.size, np.float64)
    for j, bk in enumerate(kept):
        m = b == bk
        vals = d[m]
        dq[m] = float((Fraction(float(vals.max())) + Fraction(float(vals.min()))) / 2)    # correctly rounded, ties to even
        sym[m] = j
    return d, sym, dq, kept


def test_representative64_is_the_exactly_rounded_midrange():
    rng = np.random.default_rng(5)
    top = (1 << 52) - 1
    for _ in range(3000):
        bucket = int(rng.integers(0, 2)) << 11 | int(rng.integers(1, 2047))
        m = sorted(int(x) for x in rng.integers(0, 1 << 52, size=2, dtype=np.uint64))
        if rng.random() < 0.4:
            m[1] = min(m[0] + int(rng.integers(0, 4)), top)
        lo = np.uint64((bucket << 52) | m[0]).view(np.float64)
        hi = np.uint64((bucket << 52) | m[1]).view(np.float64)
        want = float((Fraction(float(lo)) + Fraction(float(hi))) / 2)
        got = np.uint64(orc.representative64(bucket, m[0], m[1])).view(np.float64)
        assert got == want and (int(got.view(np.uint64)) >> 52) == bucket
        t = m[0] + m[1]; mm = t >> 1                       # integer form: halve the mantissa sum, ties to even
        if (t & 1) and (mm & 1):
            mm += 1
        assert int(got.view(np.uint64)) == (bucket << 52) | mm


def test_representative64_special_cases():
    top = (1 << 52) - 1
    assert orc.representative64(1030, 12345, 12345) == (1030 << 52) | 12345
    assert orc.representative64(1030, 0, 2) == (1030 << 52) | 1
    assert orc.representative64(1030, 0, 1) == (1030 << 52) | 0                 # tie -> even
    assert orc.representative64(1030, 1, 2) == (1030 << 52) | 2                 # tie 1.5 -> even
    assert orc.representative64(2046, top, top) == (2046 << 52) | top           # no overflow at the top
    assert orc.representative64(2048 + 1, 0, top - 1) == ((2048 + 1) << 52) | (top >> 1)
    assert orc.representative64(1030, top - 1, top) == (1030 << 52) | (top - 1)  # a sum of 54 significant bits, tie -> even


def test_promotion64_order_and_zero_class():
    count = np.zeros(4096, np.uint64)
    for b in (1023, 2048 + 1023, 1022, 2048 + 1020, 1, 2048 + 2046, 0, 2048):   # zero class entries must be ignored
        count[b] = 5
    K, kept, sym = orc.promote64(count, 2)
    assert K == 3 and list(kept) == [2048 + 2046, 1023, 2048 + 1023]              # largest exponent first, + before -
    assert sym[2048 + 2046] == 0 and sym[1023] == 1 and sym[2048 + 1023] == 2
    assert sym[1022] == 3 and sym[0] == 3 and sym[2048] == 3 and sym[1] == 3
    K, kept, _ = orc.promote64(count, 4)
    assert K == 6 and list(kept) == [2048 + 2046, 1023, 2048 + 1023, 1022, 2048 + 1020, 1]


@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
@pytest.mark.parametrize("n", [1, 7, 1000, 40000])
def test_quantize64_matches_numpy_definition(n, nbits):
    w, w_ref = rand_case64(n, seed=n + nbits, zero_frac=0.1)
    d, sym_np, dq_np, kept = np_quantize64(w, w_ref, nbits)
    sym, dq, K, k_E = orc.quantize64(w, w_ref, nbits)
    assert K == len(kept)
    assert np.array_equal(sym, sym_np)
    assert np.array_equal(bits64(dq), bits64(dq_np))
    b = (bits64(d) >> np.uint64(52)).astype(np.int64)
    assert k_E == len(set(b[(b & 2047) != 0])) + (1 if np.any((b & 2047) == 0) else 0)
    # kept elements: the representative lies in the element's own binade, within half its width
    keptm = sym < K
    e = (b & 2047) - 1023
    assert np.all(np.abs(d[keptm] - dq[keptm]) <= 2.0 ** (e[keptm] - 1.0))


SIZES = [0, 1, 5, 257, 16383, 16384, 16385, 2 * 16384 + 77]


@pytest.mark.parametrize("n", SIZES)
def test_blob64_structure_and_round_trip(n):
    nbits = 1 + n % 4
    w, w_ref = rand_case64(n, seed=n, zero_frac=0.05)
    blob = orc.encode64(w, w_ref, nbits)
    assert blob.size <= orc.encode_bound(n, nbits)
    h, sym_r, lane_bits, off = lcb1_reader.read(blob)
    sym, dq, K, k_E = orc.quantize64(w, w_ref, nbits)
    assert h["magic"] == b"LCB1" and h["dtype"] == 3 and set(h["reserved"]) <= {0}
    assert (h["n"], h["nbits"], h["K"], h["W"], h["V"], h["R"]) == (n, nbits, K, 64, 4, 64)
    assert h["status"] == 0 and h["k_E"] == k_E
    assert np.array_equal(sym_r, sym)
    for j in range(16):
        s = h["slots"][j]
        if j <= K:
            assert s["cnt"] == int(np.sum(sym == j)) and (s["len"] > 0) == (s["cnt"] > 0) and s["pad"] == 0
            if j < K:
                assert s["rep_bits"] == int(bits64(dq[sym == j])[0]) and s["bucket"] == s["rep_bits"] >> 52
            else:
                assert s["rep_bits"] == 0 and s["bucket"] == 0xFFFF
        else:
            assert s == dict(bucket=0, len=0, pad=0, rep_bits=0, cnt=0)
    lens = [s["len"] for s in h["slots"]]
    assert list(orc.huffman_lengths([s["cnt"] for s in h["slots"][:K + 1]])) == lens[:K + 1]
    assert sum(int(lb.sum()) for lb in lane_bits) == sum(s["cnt"] * s["len"] for s in h["slots"])
    rec = w_ref.copy()
    assert orc.decode64(blob, rec) == blob.size
    assert np.array_equal(bits64(rec), bits64(w_ref + dq))              # one binary64 add; zero symbols add +0
    assert np.array_equal(blob, orc.encode64(w, w_ref, nbits))
    assert np.array_equal(blob, orc.encode_t(w, w_ref, nbits, orc.DT_F64))


def test_binary64_path_agrees_with_binary32_on_values_both_hold_exactly():
    """Deltas that are small powers of two on integer weights are exact in both formats: same symbols, same code
    lengths, same payload; only the header (type, bucket ids, representatives) differs."""
    rng = np.random.default_rng(9)
    n = 20000
    w_ref = rng.integers(-1000, 1000, n).astype(np.float64)
    d = rng.choice([-1, 1], n) * 2.0 ** rng.integers(-3, 0, n)               # six buckets, all kept at 3 bits
    d[rng.random(n) < 0.2] = 0
    w = w_ref + d
    b64 = orc.encode64(w, w_ref, 3)
    b32 = orc.encode(w.astype(np.float32), w_ref.astype(np.float32), 3)
    assert b64.size == b32.size and np.array_equal(b64[512:], b32[512:])
    h64, h32 = lcb1_reader.parse_header(b64), lcb1_reader.parse_header(b32)
    for s64, s32 in zip(h64["slots"], h32["slots"]):
        assert (s64["len"], s64["cnt"]) == (s32["len"], s32["cnt"])
        if s64["len"] and s64["bucket"] != 0xFFFF:
            v64 = np.uint64(s64["rep_bits"]).view(np.float64); v32 = np.uint32(s32["rep_bits"]).view(np.float32)
            assert float(v64) == float(v32)
            assert (s64["bucket"] >> 11, (s64["bucket"] & 2047) - 1023) == (s32["bucket"] >> 8, (s32["bucket"] & 255) - 127)
    rec = w_ref.copy()
    orc.decode64(b64, rec)
    assert np.array_equal(bits64(rec), bits64(w))                        # one value per bucket: lossless


def test_binary64_sees_exponents_binary32_cannot():
    n = 1000
    w_ref = np.zeros(n)
    i = np.arange(n)
    zero, sub = i % 7 == 0, i == 5
    huge = (i % 3 == 0) & ~zero & ~sub
    tiny = ~huge & ~zero & ~sub
    w = np.where(huge, -1e200, np.where(tiny, 1e-200, 0.0)); w[5] = 5e-324       # huge, tiny, zero, subnormal
    sym, dq, K, k_E = orc.quantize64(w, w_ref, 2)
    assert K == 2 and k_E == 3
    assert np.all(sym[huge] == 0) and np.all(dq[huge] == -1e200)
    assert np.all(sym[tiny] == 1) and np.all(dq[tiny] == 1e-200)
    assert np.all(sym[zero | sub] == 2) and np.all(dq[zero | sub] == 0)


def test_nonfinite_and_bad_arguments64():
    w_ref = np.zeros(10); w = np.ones(10); w[3] = np.inf
    with pytest.raises(orc.OracleError) as e:
        orc.encode64(w, w_ref, 3)
    assert e.value.status == orc.NONFINITE
    hdr = lcb1_reader.parse_header(e.value.header)
    assert hdr["status"] == orc.NONFINITE and hdr["dtype"] == 3 and hdr["total_bytes"] == 512
    w[3] = 1.7e308; w_ref[3] = -1.7e308                                  # the difference overflows
    with pytest.raises(orc.OracleError):
        orc.encode64(w, w_ref, 3)
    good = orc.encode64(np.ones(10), np.zeros(10), 3)
    with pytest.raises(orc.OracleError) as e:                             # a binary64 blob is not restored into fp32 weights
        orc.decode(good, np.zeros(10, np.float32))
    assert e.value.status == orc.BADARG
    with pytest.raises(orc.OracleError) as e:
        orc.decode64(orc.encode(np.ones(10, np.float32), np.zeros(10, np.float32), 3), np.zeros(10))
    assert e.value.status == orc.BADARG
    with pytest.raises(orc.OracleError) as e:
        orc.decode64(good, np.zeros(11))
    assert e.value.status == orc.BADARG


def test_decode64_rejects_damage_in_the_high_half_of_a_representative():
    w, w_ref = rand_case64(5000, seed=3)
    blob = orc.encode64(w, w_ref, 3)
    bad = blob.copy(); bad[320 + 3] ^= 0x10                             # exponent bits of slot 0's representative
    rec = w_ref.copy()
    with pytest.raises(orc.OracleError) as e:
        orc.decode64(bad, rec)
    assert e.value.status == orc.BAD_BLOB and np.array_equal(rec, w_ref)


def test_accounting64_uses_64_bit_bucket_values():
    n = 10; w_ref = np.zeros(n)
    w = np.array([1.0, 1.5, 2.0, 3.0, 4.0, 5.0, -1.0, -2.0, 0.0, 0.0])
    blob = orc.encode64(w, w_ref, 2)
    a = orc.accounting(blob)
    h = lcb1_reader.parse_header(blob)
    k = h["k_E"]
    assert k == 6 and a["bits_E"] == n * 3 + 64 * k == orc.size_exponent_only(n, k, 64)
    assert a["bits_EP"] == n * 2 + 64 * 4


# ---------------------------------------------------------------- code table caching (Section 3.2), binary64
def test_cached_encode64_follows_the_binary32_rule():
    """lco_encode_cached64 against what pins lco_encode_cached: the first call is the plain blob and fills the cache
    with its 12-bit bucket ids and lengths; a second checkpoint with the same buckets carries the cached lengths (the
    plain blob's symbols, counts and representatives; payload = sum of count x cached length); a new largest
    exponent, another nbits, a payload above n * nbits bits and a cache made by a binary32 encode are misses."""
    from tests import lcb1_reader
    rng = np.random.RandomState(64)
    n, nbits = 3 * lcb1_reader.C + 77, 3
    w0 = 0.05 * rng.randn(n)
    d1 = 1e-3 * rng.laplace(size=n); d2 = 0.8e-3 * rng.laplace(size=n)
    for d in (d1, d2):
        d[:4] = [0.02, -0.02, 0.011, -0.011]
    cache = orc.new_cache()
    w1 = w0 + d1
    b1, u1 = orc.encode_cached64(w1, w0, nbits, cache)
    assert not u1 and np.array_equal(b1, orc.encode64(w1, w0, nbits))
    h1 = lcb1_reader.parse_header(b1)
    assert cache[0] == 1 and cache[1] == nbits and cache[2] == h1["K"]
    assert [int(x) for x in cache[4:4 + h1["K"]]] == [s["bucket"] for s in h1["slots"][:h1["K"]]]
    assert all(int(x) >= 512 or (int(x) >> 11) == 0 for x in cache[4:4 + h1["K"]])       # 12-bit ids: sign << 11 | exponent
    ref = w0.copy(); orc.decode64(b1, ref)
    w2 = w1 + d2
    stale = cache.copy()
    c2, u2 = orc.encode_cached64(w2, ref, nbits, cache)
    p2 = orc.encode64(w2, ref, nbits)
    assert u2 and c2.size >= p2.size
    hp, hc = lcb1_reader.parse_header(p2), lcb1_reader.parse_header(c2)
    K = hp["K"]
    for j in range(K + 1):
        assert hc["slots"][j]["bucket"] == hp["slots"][j]["bucket"] and hc["slots"][j]["cnt"] == hp["slots"][j]["cnt"]
        assert hc["slots"][j]["rep_bits"] == hp["slots"][j]["rep_bits"]
        assert hc["slots"][j]["len"] == int(stale[20 + j])
    assert c2[320:384].tobytes() == p2[320:384].tobytes()                                 # high halves of the representatives
    bits_expected = sum(hc["slots"][j]["cnt"] * int(stale[20 + j]) for j in range(K + 1))
    area = 512 + (4 * (hc["num_chunks"] + 1) + 15) // 16 * 16
    lane_bits = 0
    off = np.frombuffer(c2[512:512 + 4 * (hc["num_chunks"] + 1)].tobytes(), "<u4")
    for c in range(hc["num_chunks"]):
        lane_bits += int(np.frombuffer(c2[area + 4 * int(off[c]):area + 4 * int(off[c]) + 128].tobytes(), "<u2").sum())
    assert lane_bits == bits_expected
    a, b = ref.copy(), ref.copy()
    orc.decode64(p2, a); orc.decode64(c2, b)
    assert np.array_equal(a.view(np.uint64), b.view(np.uint64))
    # misses
    d3 = d2.copy(); d3[9] = 0.3
    c = stale.copy()
    blob, used = orc.encode_cached64(w1 + d3, ref, nbits, c)
    assert not used and np.array_equal(blob, orc.encode64(w1 + d3, ref, nbits))
    c = stale.copy()
    blob, used = orc.encode_cached64(w2, ref, 2, c)
    assert not used and np.array_equal(blob, orc.encode64(w2, ref, 2))
    c32 = orc.new_cache()
    orc.encode_cached(w2.astype(np.float32), ref.astype(np.float32), nbits, c32)
    blob, used = orc.encode_cached64(w2, ref, nbits, c32)
    assert not used and np.array_equal(blob, p2)
    # a stale table that would outgrow the bound: reversed populations
    m = 65536
    mags = [2.0 ** -e for e in range(1, 8)]
    skew = [m >> (j + 1) for j in range(7)]; skew.append(m - sum(skew))
    def by_symbol(counts, seed):
        d = np.concatenate([np.full(c_, v) for c_, v in zip(counts[:-1], mags)] + [np.zeros(counts[-1])])
        np.random.RandomState(seed).shuffle(d)
        return d
    zero = np.zeros(m)
    c = orc.new_cache()
    orc.encode_cached64(by_symbol(skew, 0), zero, 3, c)
    assert [int(x) for x in c[20:28]] == [1, 2, 3, 4, 5, 6, 7, 7]
    d_rev = by_symbol(skew[::-1], 1)
    blob, used = orc.encode_cached64(d_rev, zero, 3, c)
    assert not used and np.array_equal(blob, orc.encode64(d_rev, zero, 3)) and blob.size <= orc.encode_bound(m, 3)
