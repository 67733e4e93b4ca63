"""Pins for the CPU oracle: the paper's printed example, closed forms, brute force on
tiny inputs, an independent numpy quantizer, and an independent bit-level reader of
the blob.  CPU only; nothing here touches the HIP library."""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

from oracle import lc_oracle as orc
from tests import lcb1_reader

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def golden(name):
    out = {}
    for line in open(os.path.join(GOLDEN, name)):
        if line.startswith("#") or not line.strip():
            continue
        k, v = line.split()
        out[k] = float(v) if "." in v else int(v)
    return out


def bits(a):
    return np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)


def rand_case(n, seed, scale=1e-3, zero_frac=0.0):
    rng = np.random.default_rng(seed)
    w_ref = (0.05 * rng.standard_normal(n)).astype(np.float32)
    d = rng.laplace(0.0, scale, n).astype(np.float32)
    if zero_frac:
        d[rng.random(n) < zero_frac] = 0.0
    w = (w_ref + d).astype(np.float32)
    return w, w_ref


# ------------------------------------------------------------------ independent numpy quantizer
def np_quantize(w, w_ref, nbits):
    """Section 3.1.1 restated with numpy on values (not mantissas): buckets by top 9 bits,
    keep the 2^x-1 non-empty normal buckets of largest exponent (+ before -), midrange of
    the members' max and min, everything else 0."""
    d = (w.astype(np.float32) - w_ref.astype(np.float32)).astype(np.float32)
    b = d.view(np.uint32) >> 23
    normal = (b & 255) != 0
    cand = sorted(set(int(x) for x in b[normal]), key=lambda x: (-(x & 255), x >> 8))
    kept = cand[:2 ** nbits - 1]
    K = len(kept)
    sym = np.full(d.size, K, np.uint8)
    dq = np.zeros(d.size, np.float32)
    for j, bk in enumerate(kept):
        m = b == bk
        vals = d[m].astype(np.float64)
        dq[m] = np.float32((vals.max() + vals.min()) / 2.0)
        sym[m] = j
    return d, sym, dq, kept


# ------------------------------------------------------------------ the paper's printed example
def test_worked_example_size_and_rate():
    g = golden("worked_example.txt")
    assert orc.size_exponent_only(g["n"], g["k"], g["b"]) == g["bits_exponent_quantized"] == 190
    assert round(g["bits_uncompressed"] / orc.size_exponent_only(g["n"], g["k"], g["b"]), 2) == g["rate"]


def five_bucket_delta():
    # ten deltas in five (sign, exponent) buckets
    d = np.array([0.75, 0.6, -0.3, -0.26, 0.1, 0.11, 0.09, 0.05, 0.04, -0.013], np.float32)
    assert len(set(bits(d) >> 23)) == 5
    w_ref = np.zeros(10, np.float32)
    return (w_ref + d).astype(np.float32), w_ref


def test_worked_example_through_the_encoder():
    g = golden("worked_example.txt")
    w, w_ref = five_bucket_delta()
    blob = orc.encode(w, w_ref, 3)               # 7 >= 5: nothing merged
    acct = orc.accounting(blob)
    assert acct["bits_E"] == g["bits_exponent_quantized"]
    assert lcb1_reader.parse_header(blob)["k_E"] == g["k"]


def test_two_bit_promotion_example():
    g = golden("worked_example.txt")
    w, w_ref = five_bucket_delta()
    sym, dq, K, k_E = orc.quantize(w, w_ref, g["promotion_bits"])
    assert k_E == g["k"] and K == g["kept_buckets"] and K + 1 == g["buckets_after_promotion"]
    d = w - w_ref
    order = np.argsort(-np.abs(d))
    # the two smallest-exponent buckets (0.05, 0.04 and -0.013) are merged into value 0, stored last
    merged = sym == g["zero_symbol_index"]
    assert set(np.nonzero(merged)[0]) == {7, 8, 9} and np.all(dq[merged] == 0)
    assert len(set(bits(d[merged]) >> 23)) == g["merged_buckets"]
    assert sym[order[0]] == 0                    # largest exponent first


# ------------------------------------------------------------------ promotion
@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
def test_promotion_keeps_exactly_the_highest_priority_buckets(nbits):
    rng = np.random.default_rng(nbits)
    for trial in range(200):
        count = np.zeros(512, np.uint64)
        k = rng.integers(0, 40)
        idx = rng.choice(512, size=k, replace=False)
        count[idx] = rng.integers(1, 1000, size=k)
        count[255] = count[511] = 0              # Inf/NaN deltas are rejected before promotion
        K, kept, sym = orc.promote(count, nbits)
        cand = [b for b in range(512) if count[b] > 0 and (b & 255) != 0]
        cand.sort(key=lambda b: (-(b & 255), b >> 8))
        assert K == min(2 ** nbits - 1, len(cand))
        assert list(kept) == cand[:K]
        for b in range(512):
            assert sym[b] == (cand.index(b) if b in cand[:K] else K)
        # population plays no part: scaling counts changes nothing
        K2, kept2, _ = orc.promote(count * np.uint64(7), nbits)
        assert K2 == K and list(kept2) == list(kept)


def test_promotion_ignores_zero_class_and_prefers_positive():
    count = np.zeros(512, np.uint64)
    count[0] = 10**9; count[256] = 5          # +0/subnormal and -0/subnormal
    count[100] = 1; count[256 + 100] = 1; count[99] = 1
    K, kept, sym = orc.promote(count, 1)
    assert K == 1 and kept[0] == 100 and sym[0] == 1 and sym[256] == 1 and sym[356] == 1
    K, kept, sym = orc.promote(count, 2)
    assert list(kept) == [100, 356, 99]


# ------------------------------------------------------------------ representative
def nearest_f32_even(x):
    """Exact rational -> nearest binary32, ties to even, by search over the two neighbours."""
    f = np.float32(float(x))
    cands = {f, np.nextafter(f, np.float32(np.inf)), np.nextafter(f, np.float32(-np.inf))}
    best = None
    for c in cands:
        err = abs(Fraction(float(c)) - x)
        key = (err, int(np.float32(c).view(np.uint32)) & 1)
        if best is None or key < best[0]:
            best = (key, c)
    return np.float32(best[1])


def test_representative_is_the_exactly_rounded_midrange():
    rng = np.random.default_rng(5)
    for _ in range(3000):
        bucket = int(rng.integers(0, 2)) << 8 | int(rng.integers(1, 255))
        m = np.sort(rng.integers(0, 1 << 23, size=2))
        if rng.random() < 0.3:
            m[1] = min(m[0] + rng.integers(0, 4), (1 << 23) - 1)
        lo = np.uint32((bucket << 23) | int(m[0])).view(np.float32)
        hi = np.uint32((bucket << 23) | int(m[1])).view(np.float32)
        exact = (Fraction(float(lo)) + Fraction(float(hi))) / 2
        want = nearest_f32_even(exact)
        got = np.uint32(orc.representative(bucket, m[0], m[1])).view(np.float32)
        assert got == want and (got.view(np.uint32) >> 23) == bucket
        # integer form of the same rounding: halve the mantissa sum, ties to even
        t = int(m[0]) + int(m[1]); mm = t >> 1
        if (t & 1) and (mm & 1):
            mm += 1
        assert int(got.view(np.uint32)) == (bucket << 23) | mm


def test_representative_special_cases():
    assert orc.representative(130, 12345, 12345) == (130 << 23) | 12345        # min == max
    assert orc.representative(130, 0, 2) == (130 << 23) | 1                    # exact
    assert orc.representative(130, 0, 1) == (130 << 23) | 0                    # tie -> even (0)
    assert orc.representative(130, 1, 2) == (130 << 23) | 2                    # tie 1.5 -> even (2)
    assert orc.representative(254, 0x7FFFFF, 0x7FFFFF) == (254 << 23) | 0x7FFFFF  # no overflow at the top
    assert orc.representative(256 + 1, 0, 0x7FFFFE) == ((256 + 1) << 23) | 0x3FFFFF


# ------------------------------------------------------------------ Huffman
_FEASIBLE = {}


def brute_force_cost(cnt):
    """Optimal prefix-code cost by enumerating every length vector that satisfies Kraft."""
    m = len(cnt)
    if m == 1:
        return cnt[0]
    if m not in _FEASIBLE:
        _FEASIBLE[m] = [lens for lens in itertools.product(range(1, m), repeat=m)
                        if sum(Fraction(1, 2 ** l) for l in lens) <= 1]
    return min(sum(a * l for a, l in zip(cnt, lens)) for lens in _FEASIBLE[m])


@pytest.mark.parametrize("m", [1, 2, 3, 4, 5, 6])
def test_huffman_cost_is_the_brute_force_optimum(m):
    rng = np.random.default_rng(m)
    cases = [list(c) for c in itertools.product([1, 2, 3, 5], repeat=m)][:300]
    cases += [list(rng.integers(1, 50, size=m)) for _ in range(60)]
    cases += [list(rng.integers(1, 4, size=m) * rng.integers(1, 10**9)) for _ in range(20)]
    for cnt in cases:
        lens = orc.huffman_lengths(cnt)
        assert sum(int(a) * int(l) for a, l in zip(cnt, lens)) == brute_force_cost([int(a) for a in cnt]), cnt
        if m >= 2:
            assert sum(Fraction(1, 2 ** int(l)) for l in lens) == 1


def test_huffman_larger_alphabets_against_heap_construction():
    import heapq
    rng = np.random.default_rng(11)
    for _ in range(300):
        m = int(rng.integers(2, 17))
        cnt = rng.integers(1, 10**6, size=m) if rng.random() < 0.5 else (2.0 ** rng.integers(0, 30, size=m)).astype(np.int64)
        heap = [int(c) for c in cnt]
        heapq.heapify(heap)
        cost = 0
        while len(heap) > 1:
            a, b = heapq.heappop(heap), heapq.heappop(heap)
            cost += a + b
            heapq.heappush(heap, a + b)
        lens = orc.huffman_lengths(cnt)
        assert sum(int(a) * int(l) for a, l in zip(cnt, lens)) == cost       # sum of merges = optimal cost
        assert sum(Fraction(1, 2 ** int(l)) for l in lens) == 1
        n = int(cnt.sum())
        H = -sum(int(c) / n * math.log2(int(c) / n) for c in cnt)
        L = sum(int(c) * int(l) for c, l in zip(cnt, lens)) / n
        assert H - 1e-9 <= L < H + 1
        assert lens.max() <= m - 1


def test_huffman_closed_forms_and_tie_break():
    # textbook six-letter example (weights 45,13,12,16,9,5 -> cost 224, lengths 1,3,3,3,4,4)
    assert list(orc.huffman_lengths([45, 13, 12, 16, 9, 5])) == [1, 3, 3, 3, 4, 4]
    # Fibonacci weights give the maximally skewed tree
    assert sorted(orc.huffman_lengths([1, 1, 2, 3, 5, 8, 13, 21])) == [1, 2, 3, 4, 5, 6, 7, 7]
    # equal weights over 2^k symbols give a fixed-length code
    assert list(orc.huffman_lengths([7] * 8)) == [3] * 8
    assert list(orc.huffman_lengths([7] * 16)) == [4] * 16
    # zero-count symbols get no code; one active symbol gets one bit; none -> nothing
    assert list(orc.huffman_lengths([0, 9, 0, 0])) == [0, 1, 0, 0]
    assert list(orc.huffman_lengths([0, 0, 0])) == [0, 0, 0]
    assert list(orc.huffman_lengths([3, 0, 5])) == [1, 0, 1]
    # tie-break: leaves before joined nodes, lower index first.  Weights 1,1,2,2:
    # join(1,1)=2'; next smallest are the leaves 2,2 (leaf before joined) -> 4'; join(2',4').
    assert list(orc.huffman_lengths([1, 1, 2, 2])) == [2, 2, 2, 2]
    # weights 1,1,1,1,1: join(s0,s1)=2a, join(s2,s3)=2b, then leaf s4 (1) with 2a, then 2b with 3.
    assert list(orc.huffman_lengths([1, 1, 1, 1, 1])) == [3, 3, 2, 2, 2]
    # all 2^64-safe: counts up to 2^32 each over 16 symbols
    assert orc.huffman_lengths([2 ** 32] * 16).tolist() == [4] * 16


def test_canonical_codes():
    assert list(orc.canonical_codes([1, 2, 3, 3])) == [0b0, 0b10, 0b110, 0b111]
    assert list(orc.canonical_codes([3, 3, 2, 1])) == [0b110, 0b111, 0b10, 0b0]
    assert list(orc.canonical_codes([2, 0, 2, 2, 2])) == [0, 0, 1, 2, 3]
    assert list(orc.canonical_codes([0, 1])) == [0, 0]
    rng = np.random.default_rng(3)
    for _ in range(200):
        m = int(rng.integers(2, 17))
        lens = orc.huffman_lengths(rng.integers(1, 1000, size=m))
        codes = orc.canonical_codes(lens)
        strs = [format(int(c), "0%db" % int(l)) for c, l in zip(codes, lens)]
        for i in range(m):
            for j in range(m):
                if i != j:
                    assert not strs[j].startswith(strs[i])            # prefix free
        assert strs == [lcb1_reader.canonical(list(lens))[s] for s in range(m)]
        # canonical: sorted by (len, index) the code values, left aligned, strictly increase
        order = sorted(range(m), key=lambda s: (lens[s], s))
        left = [int(codes[s]) << (16 - int(lens[s])) for s in order]
        assert left == sorted(left) and len(set(left)) == m


# ------------------------------------------------------------------ quantizer against numpy
@pytest.mark.parametrize("nbits", [1, 2, 3, 4])
@pytest.mark.parametrize("n", [1, 7, 1000, 40000])
def test_quantize_matches_numpy_definition(n, nbits):
    w, w_ref = rand_case(n, seed=n + nbits, zero_frac=0.1)
    d, sym_np, dq_np, kept = np_quantize(w, w_ref, nbits)
    sym, dq, K, k_E = orc.quantize(w, w_ref, nbits)
    assert K == len(kept)
    assert np.array_equal(sym, sym_np)
    assert np.array_equal(bits(dq), bits(dq_np))
    b = bits(d) >> 23
    assert k_E == len(set(b[(b & 255) != 0])) + (1 if np.any((b & 255) == 0) else 0)


def test_error_bounds():
    for nbits in (2, 3, 4):
        w, w_ref = rand_case(50000, seed=nbits)
        d, _, _, kept = np_quantize(w, w_ref, nbits)
        sym, dq, K, _ = orc.quantize(w, w_ref, nbits)
        e = ((bits(d) >> 23) & 255).astype(np.int64) - 127
        keptm = sym < K
        # kept: within half the bucket width 2^e, and the representative stays inside the bucket
        assert np.all(np.abs(d[keptm].astype(np.float64) - dq[keptm]) <= 2.0 ** (e[keptm] - 1))
        assert np.array_equal(bits(dq[keptm]) >> 23, bits(d[keptm]) >> 23)
        # merged: strictly below the top of the lowest kept binade
        e_cut = min((b & 255) - 127 for b in kept)
        assert np.all(np.abs(d[~keptm]) < 2.0 ** (e_cut + 1)) and np.all(dq[~keptm] == 0)
        # every merged element has lower priority than every kept bucket
        key = lambda b: ((b & 255), 1 - (b >> 8))
        lowest_kept = min(key(b) for b in kept)
        assert all(key(int(x)) < lowest_kept for x in set(bits(d[~keptm]) >> 23) if (int(x) & 255) != 0)


def test_lossless_when_buckets_hold_one_value_each():
    rng = np.random.default_rng(9)
    n = 5000
    w_ref = rng.integers(-1000, 1000, n).astype(np.float32)        # integers: sums with small powers of two are exact
    d = (rng.choice([-1, 1], n) * 2.0 ** rng.integers(-3, 0, n)).astype(np.float32)   # 6 buckets, one value each
    d[rng.random(n) < 0.2] = 0
    w = (w_ref + d).astype(np.float32)
    blob = orc.encode(w, w_ref, 3)
    rec = w_ref.copy()
    orc.decode(blob, rec)
    assert np.array_equal(bits(rec), bits(w))


def test_zero_class_zero_subnormal_and_negative_zero():
    n = 3000
    w, w_ref = rand_case(n, seed=21)
    w_ref[::7] = 0.0
    w0 = w.copy(); w0[::7] = 0.0                                   # delta exactly +0
    w1 = w0.copy(); w1[::14] = np.float32(1e-41)                   # subnormal delta
    w2 = w0.copy(); w2[::21] = np.float32(-0.0)                    # -0 delta
    b0, b1, b2 = orc.encode(w0, w_ref, 3), orc.encode(w1, w_ref, 3), orc.encode(w2, w_ref, 3)
    h0 = lcb1_reader.parse_header(b0)
    assert np.array_equal(b0[60:], b1[60:]) and np.array_equal(b0[60:], b2[60:])
    # stored -0.0 in w_ref survives a zero symbol (no write, not "+ 0.0")
    ref = w_ref.copy(); ref[::7] = np.float32(-0.0)
    wn = w0.copy(); wn[::7] = np.float32(-0.0)
    rec = ref.copy()
    orc.decode(orc.encode(wn, ref, 3), rec)
    assert np.all(bits(rec[::7]) == 0x80000000)
    assert h0["status"] == 0


def test_nonfinite_is_rejected():
    w, w_ref = rand_case(100, seed=2)
    for bad in (np.inf, -np.inf, np.nan):
        wb = w.copy(); wb[37] = bad
        with pytest.raises(orc.OracleError) as e:
            orc.encode(wb, w_ref, 3)
        assert e.value.status == orc.NONFINITE
        assert lcb1_reader.parse_header(e.value.header)["status"] == orc.NONFINITE
    wb = w.copy(); wb[5] = np.float32(3e38); rb = w_ref.copy(); rb[5] = np.float32(-3e38)   # overflow in the subtraction
    with pytest.raises(orc.OracleError):
        orc.encode(wb, rb, 3)


# ------------------------------------------------------------------ blob, read by the second reader
SIZES = [0, 1, 3, 4, 5, 255, 256, 257, 1000, 16383, 16384, 16385, 2 * 16384 + 77]


@pytest.mark.parametrize("n", SIZES)
def test_blob_structure_and_round_trip(n):
    nbits = 1 + n % 4
    w, w_ref = rand_case(n, seed=n, zero_frac=0.05)
    blob = orc.encode(w, w_ref, nbits)
    assert blob.size <= orc.encode_bound(n, nbits)
    h, sym_r, lane_bits, off = lcb1_reader.read(blob)
    sym, dq, K, k_E = orc.quantize(w, w_ref, nbits)
    assert h["magic"] == b"LCB1" and h["version"] == 1 and h["header_bytes"] == 512
    assert (h["n"], h["nbits"], h["K"], h["W"], h["V"], h["R"]) == (n, nbits, K, 64, 4, 64)
    assert h["status"] == 0 and h["k_E"] == k_E and set(h["reserved"]) <= {0} and h["dtype"] == 0
    assert np.array_equal(sym_r, sym)
    # symbol table: counts, representatives, bucket ids, unused slots zero, zero symbol last
    for j in range(16):
        s = h["slots"][j]
        if j <= K:
            assert s["cnt"] == int(np.sum(sym == j)) and (s["len"] > 0) == (s["cnt"] > 0) and s["pad"] == 0
            if j < K:
                assert s["rep_bits"] == int(bits(dq[sym == j])[0]) and s["bucket"] == s["rep_bits"] >> 23
            else:
                assert s["rep_bits"] == 0 and s["bucket"] == 0xFFFF
        else:
            assert s == dict(bucket=0, len=0, pad=0, rep_bits=0, cnt=0)
    lens = [s["len"] for s in h["slots"]]
    assert list(orc.huffman_lengths([s["cnt"] for s in h["slots"][:K + 1]])) == lens[:K + 1]
    assert h["max_len"] == max(lens)
    # payload bits = sum cnt*len exactly
    assert sum(int(lb.sum()) for lb in lane_bits) == sum(s["cnt"] * s["len"] for s in h["slots"])
    # restore: w_ref + dq in one binary32 add; zero symbols untouched
    rec = w_ref.copy()
    assert orc.decode(blob, rec) == blob.size
    assert np.array_equal(bits(rec), bits((w_ref + dq).astype(np.float32)))
    # determinism
    assert np.array_equal(blob, orc.encode(w, w_ref, nbits))


def test_lane_ownership_order():
    # one chunk and a bit; element i gets a symbol that depends on i only through a known pattern
    n = 16384 + 300
    w_ref = np.zeros(n, np.float32)
    d = np.where(np.arange(n) % 3 == 0, 1.0, np.where(np.arange(n) % 3 == 1, 0.25, 0.0)).astype(np.float32)
    blob = orc.encode(d, w_ref, 2)
    h, sym, lane_bits, _ = lcb1_reader.read(blob)
    assert np.array_equal(sym, np.arange(n) % 3)
    lens = [s["len"] for s in h["slots"]]
    # lane l of chunk 0 owns elements r*256 + 4l + v
    for lane in (0, 1, 63):
        idx = np.array([r * 256 + 4 * lane + v for r in range(64) for v in range(4)])
        assert lane_bits[0][lane] == sum(lens[s] for s in idx % 3)
    # tail chunk: 300 elements -> lanes 0..10 own 8 (two rows), lane 11 owns 4 (one row) ... none after lane 63's row 0
    tail = np.arange(300)
    for lane in (0, 10, 11, 12, 63):
        own = tail[(tail % 256) // 4 == lane]
        assert lane_bits[1][lane] == sum(lens[s] for s in (16384 + own) % 3)


def test_decode_rejects_damaged_blobs_before_touching_wref():
    n = 40000
    w, w_ref = rand_case(n, seed=77)
    blob = orc.encode(w, w_ref, 3)

    def expect_bad(b, n_arg=n):
        rec = w_ref.copy()
        with pytest.raises(orc.OracleError):
            orc.decode(b, rec[:n_arg] if n_arg <= n else np.zeros(n_arg, np.float32))
        assert np.array_equal(bits(rec), bits(w_ref))
    expect_bad(blob[:100])                                   # shorter than a header
    expect_bad(blob[:-4])                                    # truncated
    for off, val in ((0, ord("X")), (4, 2), (16, 9), (20, 15), (24, 32), (36, 1), (48, 2), (66, 9)):
        b = blob.copy(); b[off] = val
        expect_bad(b)
    b = blob.copy(); b[512 + 4] ^= 1                          # chunk offset table
    expect_bad(b)
    area = 512 + 16
    b = blob.copy(); b[area] ^= 64                            # a lane length, enough to change the word count
    expect_bad(b)
    b = blob.copy(); b[area] ^= 1                             # off by one bit: same word count, found during the sweep
    with pytest.raises(orc.OracleError):
        orc.decode(b, w_ref.copy())
    b = blob.copy(); b[area + 128 + 40] ^= 0x10               # payload damage: some lane no longer ends on its length
    with pytest.raises(orc.OracleError):
        orc.decode(b, w_ref.copy())
    expect_bad(blob, n_arg=n - 1)                             # n mismatch


def test_checkpoint_chain_restores_the_tracked_state():
    """Algorithm 1: encode against the recovered state, track it; restoring from u_0 and the blobs
    gives the tracked state bit for bit, and the tracked state follows the live one."""
    rng = np.random.default_rng(4)
    n = 20000
    u = (0.05 * rng.standard_normal(n)).astype(np.float32)
    u0 = u.copy(); tracked = u.copy(); drift = np.zeros(n, np.float32); blobs = []
    for t in range(6):
        drift = (0.9 * drift + rng.laplace(0, 5e-5, n)).astype(np.float32)
        u = (u + drift).astype(np.float32)
        blob = orc.encode(u, tracked, 3)
        orc.decode(blob, tracked)
        blobs.append(blob)
        sym, dq, K, _ = orc.quantize(u, tracked, 3)   # residual after the update
    restored = u0.copy()
    for b in blobs:
        orc.decode(b, restored)
    assert np.array_equal(bits(restored), bits(tracked))
    assert np.abs(u - tracked).max() < np.abs(u - u0).max() / 4


def test_encode_bound_holds_for_flat_symbol_distribution():
    # 15 equally likely kept buckets: the least compressible input for nbits = 4
    rng = np.random.default_rng(8)
    n = 100000
    d = (rng.choice([-1.0, 1.0], n) * 2.0 ** rng.integers(-8, 0, n) * (1 + rng.random(n))).astype(np.float32)
    blob = orc.encode(d, np.zeros(n, np.float32), 4)
    assert blob.size <= orc.encode_bound(n, 4)
    assert orc.accounting(blob)["mean_len"] <= 4.0
    with pytest.raises(orc.OracleError) as e:
        orc.encode(d, np.zeros(n, np.float32), 4, cap=orc.encode_bound(n, 4) - 1)
    assert e.value.status == orc.OUT_TOO_SMALL


def test_bad_arguments():
    w, w_ref = rand_case(10, seed=1)
    for nb in (0, 5, -1):
        with pytest.raises(orc.OracleError) as e:
            orc.encode(w, w_ref, nb)
        assert e.value.status == orc.BADARG


# ---------------------------------------------------------------- table caching (Section 3.2)
def _drift_pair(n, seed, scale2=1.0, extra=None):
    """Two successive deltas with the same spread of magnitudes (so the same kept set), and the states."""
    rng = np.random.RandomState(seed)
    w0 = (0.05 * rng.randn(n)).astype(np.float32)
    d1 = (1e-3 * rng.laplace(size=n)).astype(np.float32)
    d2 = (1e-3 * scale2 * rng.laplace(size=n)).astype(np.float32)
    # pin the top of the range so both deltas have the same largest exponents, whatever the draw
    for d in (d1, d2):
        d[:4] = np.float32([0.02, -0.02, 0.011, -0.011])
    if extra is not None:
        d2[7] = extra
    return w0, d1, d2


def _chain_two(w0, d1, d2, nbits):
    """Regular blobs and cached blobs of two successive checkpoints (each against the recovered state)."""
    cache = orc.new_cache()
    ref = w0.copy()
    w1 = (ref + d1).astype(np.float32)
    b1 = orc.encode(w1, ref, nbits)
    c1, used1 = orc.encode_cached(w1, ref, nbits, cache)
    cache_after_1 = cache.copy()
    orc.decode(b1, ref)
    w2 = (w1 + d2).astype(np.float32)
    b2 = orc.encode(w2, ref, nbits)
    c2, used2 = orc.encode_cached(w2, ref, nbits, cache)
    return dict(b1=b1, c1=c1, used1=used1, cache1=cache_after_1, b2=b2, c2=c2, used2=used2, cache2=cache.copy(),
                ref1=ref, w2=w2)


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_cached_encode_first_call_is_plain_encode_and_fills_the_cache(nbits):
    w0, d1, d2 = _drift_pair(3 * lcb1_reader.C + 77, seed=nbits)
    r = _chain_two(w0, d1, d2, nbits)
    assert not r["used1"] and np.array_equal(r["b1"], r["c1"])
    h = lcb1_reader.parse_header(r["b1"])
    c = r["cache1"]
    assert c[0] == 1 and c[1] == nbits and c[2] == h["K"]
    assert [int(x) for x in c[4:4 + h["K"]]] == [s["bucket"] for s in h["slots"][:h["K"]]]
    assert [int(x) for x in c[20:20 + h["K"] + 1]] == [s["len"] for s in h["slots"][:h["K"] + 1]]


@pytest.mark.parametrize("nbits", [2, 3, 4])
def test_cached_encode_hit_same_values_cached_lengths(nbits):
    """Same kept set, same occurring symbols: the blob carries the cached lengths, and an independent reader
    finds in it the very symbols, counts and representatives of the plain blob; its payload is
    sum(count * cached length) bits; restoring from it gives the same weights bit for bit."""
    w0, d1, d2 = _drift_pair(3 * lcb1_reader.C + 77, seed=10 + nbits, scale2=0.8)
    r = _chain_two(w0, d1, d2, nbits)
    assert r["used2"]
    hp, sym_plain, _, _ = lcb1_reader.read(r["b2"])
    hc, sym_cached, lane_bits_cached, _ = lcb1_reader.read(r["c2"])
    K = hp["K"]
    assert hc["K"] == K and hc["n"] == hp["n"] and hc["k_E"] == hp["k_E"]
    for j in range(K + 1):
        assert hc["slots"][j]["bucket"] == hp["slots"][j]["bucket"]
        assert hc["slots"][j]["rep_bits"] == hp["slots"][j]["rep_bits"]
        assert hc["slots"][j]["cnt"] == hp["slots"][j]["cnt"]
        assert hc["slots"][j]["len"] == int(r["cache1"][20 + j])           # the lengths of checkpoint 1
    assert np.array_equal(sym_plain, sym_cached)
    bits_expected = sum(hc["slots"][j]["cnt"] * int(r["cache1"][20 + j]) for j in range(K + 1))
    assert int(sum(lb.sum() for lb in lane_bits_cached)) == bits_expected
    assert r["c2"].size >= r["b2"].size                                     # Huffman lengths are optimal for these counts
    if nbits >= 3:      # here this delta's own Huffman lengths differ from the cached ones, so the test can tell them apart
        assert [s["len"] for s in hc["slots"]] != [s["len"] for s in hp["slots"]] and r["c2"].size > r["b2"].size
    a, b = r["ref1"].copy(), r["ref1"].copy()
    orc.decode(r["b2"], a); orc.decode(r["c2"], b)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(r["cache2"], r["cache1"])                          # same table stays cached


def test_cached_encode_misses():
    n, nbits = 2 * lcb1_reader.C + 5, 3
    # a new, larger exponent appears: the kept set moves, the cache must not be used
    w0, d1, d2 = _drift_pair(n, seed=3, extra=np.float32(0.3))
    r = _chain_two(w0, d1, d2, nbits)
    assert not r["used2"] and np.array_equal(r["b2"], r["c2"])
    h = lcb1_reader.parse_header(r["c2"])
    assert [int(x) for x in r["cache2"][4:4 + h["K"]]] == [s["bucket"] for s in h["slots"][:h["K"]]]   # refreshed
    # the merged bucket stops occurring (every delta lands in a kept bucket): the cached code for it has no user
    rng = np.random.RandomState(5)
    w0 = (0.05 * rng.randn(n)).astype(np.float32)
    mags = np.float32([0.02, 0.011, 0.006, 0.003])
    d1 = (rng.choice(mags, n) * rng.choice(np.float32([1, -1]), n)).astype(np.float32)
    d1[::3] = 0
    d2 = (rng.choice(mags, n) * rng.choice(np.float32([1, -1]), n)).astype(np.float32)
    # make the deltas exact in fp32 against the recovered state: work on a zero state
    w0[:] = 0
    cache = orc.new_cache()
    b1, u1 = orc.encode_cached(d1, w0, 4, cache)
    ref = w0.copy(); orc.decode(b1, ref)
    w2 = (ref + d2).astype(np.float32)
    b2, u2 = orc.encode_cached(w2, ref, 4, cache)
    assert not u1 and not u2 and np.array_equal(b2, orc.encode(w2, ref, 4))
    # another nbits: miss
    w0, d1, d2 = _drift_pair(n, seed=4)
    cache = orc.new_cache()
    orc.encode_cached((w0 + d1).astype(np.float32), w0, 3, cache)
    b, u = orc.encode_cached((w0 + d1).astype(np.float32), w0, 2, cache)
    assert not u and np.array_equal(b, orc.encode((w0 + d1).astype(np.float32), w0, 2))
    # the same checkpoint again with the right nbits: hit, and identical to the plain blob (same lengths)
    b, u = orc.encode_cached((w0 + d1).astype(np.float32), w0, 2, cache)
    assert u and np.array_equal(b, orc.encode((w0 + d1).astype(np.float32), w0, 2))


def _by_symbol(counts, mags, seed=0):
    """A delta on a zero state whose symbol j (priority order: larger magnitude first) occurs counts[j] times;
    the last count is the number of zeros (the merged bucket)."""
    parts = [np.full(c, m, np.float32) for c, m in zip(counts[:-1], mags)] + [np.zeros(counts[-1], np.float32)]
    d = np.concatenate(parts)
    np.random.RandomState(seed).shuffle(d)
    return d


def test_cached_encode_never_outgrows_the_bound():
    """A table cached on skewed populations, then the populations reversed: the cached lengths would need about
    7 bits per element where lc_encode_bound promises nbits = 3, so the cache must not be used and the blob is the
    plain one (Section 3.2 re-sorts the buckets by population before a table is reused; this reading does not, so
    it must at least refuse a reuse that outgrows the buffer)."""
    n, nbits = 65536, 3
    mags = np.float32([2.0 ** -e for e in range(1, 8)])                  # 7 kept buckets, all positive
    skew = [n >> (j + 1) for j in range(7)]                               # 32768, 16384, ... 512
    skew.append(n - sum(skew))                                            # merged bucket: 512
    zero = np.zeros(n, np.float32)
    cache = orc.new_cache()
    d1 = _by_symbol(skew, mags)
    b1, u1 = orc.encode_cached(d1, zero, nbits, cache)
    assert not u1 and [int(x) for x in cache[20:28]] == [1, 2, 3, 4, 5, 6, 7, 7]
    d2 = _by_symbol(skew[::-1], mags, seed=1)                             # same buckets, populations reversed
    stale = cache.copy()
    b2, u2 = orc.encode_cached(d2, zero, nbits, cache)
    plain = orc.encode(d2, zero, nbits)
    assert not u2 and np.array_equal(b2, plain) and b2.size <= orc.encode_bound(n, nbits)
    assert not np.array_equal(cache, stale)                               # the cache now describes this blob
    assert [int(x) for x in cache[20:28]] == [s["len"] for s in lcb1_reader.parse_header(plain)["slots"][:8]]
    # the same populations as the cached ones again: a hit
    cache = stale.copy()
    b3, u3 = orc.encode_cached(_by_symbol(skew, mags, seed=2), zero, nbits, cache)
    assert u3


def test_cached_encode_reuse_limit_is_n_times_nbits_bits():
    """The limit itself: a reuse whose payload is exactly n * nbits bits is taken, one bit more is not."""
    nbits, n = 2, 1000
    mags = np.float32([0.5, 0.25, 0.125])
    zero = np.zeros(n, np.float32)
    hand = orc.new_cache()
    hand[0], hand[1], hand[2] = 1, nbits, 3
    hand[4:7] = [126, 125, 124]                                           # buckets of 0.5, 0.25, 0.125
    hand[20:24] = [1, 2, 3, 3]
    at = [300, 400, 200, 100]                                             # 300 + 800 + 600 + 300 = 2000 = n * nbits
    c = hand.copy()
    blob, used = orc.encode_cached(_by_symbol(at, mags), zero, nbits, c)
    assert used and [s["len"] for s in lcb1_reader.parse_header(blob)["slots"][:4]] == [1, 2, 3, 3]
    _, _, lane_bits, _ = lcb1_reader.read(blob)
    assert int(sum(lb.sum() for lb in lane_bits)) == n * nbits
    over = [299, 400, 201, 100]                                           # 2002 bits
    c = hand.copy()
    d = _by_symbol(over, mags)
    blob, used = orc.encode_cached(d, zero, nbits, c)
    assert not used and np.array_equal(blob, orc.encode(d, zero, nbits))


def test_cached_encode_rejects_a_damaged_cache():
    """A cache whose lengths are not a complete prefix code is not used, whatever else matches."""
    n, nbits = lcb1_reader.C + 9, 3
    w0, d1, d2 = _drift_pair(n, seed=6)
    w1 = (w0 + d1).astype(np.float32)
    cache = orc.new_cache()
    plain, _ = orc.encode_cached(w1, w0, nbits, cache)
    good = cache.copy()
    for damage in ("len", "valid", "kept"):
        c = good.copy()
        if damage == "len":
            j = int(np.argmax(c[20:36])); c[20 + j] += 1          # Kraft sum drops below 1
        elif damage == "valid":
            c[0] = 2
        else:
            c[4] ^= 1
        b, u = orc.encode_cached(w1, w0, nbits, c)
        assert not u and np.array_equal(b, plain), damage
        assert np.array_equal(c, good), damage                      # and it is repaired
    # non-finite delta: error, cache untouched
    bad = w1.copy(); bad[3] = np.inf
    c = good.copy()
    with pytest.raises(orc.OracleError) as e:
        orc.encode_cached(bad, w0, nbits, c)
    assert e.value.status == 2 and np.array_equal(c, good)


# ---------------------------------------------------------------- 16-bit parameters
def test_narrow_to_bf16_is_round_to_nearest_even():
    """Against torch's float32 -> bfloat16 conversion (a library routine), ties included."""
    torch = pytest.importorskip("torch")
    rng = np.random.RandomState(1)
    x = np.concatenate([rng.randn(20000).astype(np.float32) * np.float32(10.0) ** rng.randint(-8, 8, 20000).astype(np.float32),
                        np.float32([0.0, -0.0, 1.0, 1.00390625, 1.01171875, -1.00390625, 3.3895314e38, 1e-40])])
    # exact ties: low 16 bits = 0x8000, with the kept mantissa bit even and odd
    ties = (rng.randint(0, 1 << 15, 2000).astype(np.uint32) << 16 | 0x8000).view(np.float32)
    x = np.concatenate([x, ties[np.isfinite(ties)]])
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.narrow(x, orc.DT_BF16), want)
    assert np.array_equal(orc.widen(want, orc.DT_BF16).view(np.uint32), want.astype(np.uint32) << 16)


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_16_bit_parameters_round_trip_against_torch(dtype):
    """Restore of bf16 / fp16 parameters = storage_type(float(w_ref) + dequantized delta), checked with torch's casts."""
    torch = pytest.importorskip("torch")
    tdt, code = (torch.bfloat16, orc.DT_BF16) if dtype == "bf16" else (torch.float16, orc.DT_F16)
    g = torch.Generator().manual_seed(3)
    n, nbits = 2 * lcb1_reader.C + 333, 3
    ref_t = (0.05 * torch.randn(n, generator=g)).to(tdt)
    w_t = (ref_t.float() + 1e-3 * torch.randn(n, generator=g)).to(tdt)
    raw = (lambda t: t.view(torch.int16).numpy().view(np.uint16)) if dtype == "bf16" else (lambda t: t.numpy())
    w, ref = raw(w_t).copy(), raw(ref_t).copy()
    blob = orc.encode_t(w, ref, nbits, code)
    assert int(np.frombuffer(blob[60:64].tobytes(), np.uint32)[0]) == code
    sym, dq, K, _ = orc.quantize(w_t.float().numpy(), ref_t.float().numpy(), nbits)
    want_t = (ref_t.float() + torch.from_numpy(dq)).to(tdt)
    zero = torch.from_numpy(sym == K)
    want_t[zero] = ref_t[zero]                                    # the merged symbol leaves the stored value alone
    got = ref.copy()
    assert orc.decode_t(blob, got, code) == blob.size
    assert np.array_equal(got.view(np.uint16), raw(want_t).view(np.uint16))
    # the blob names its element type: restoring another type is refused
    with pytest.raises(orc.OracleError) as e:
        orc.decode(blob, ref_t.float().numpy().copy())
    assert e.value.status == 1
    with pytest.raises(orc.OracleError) as e:
        orc.decode_t(orc.encode(w_t.float().numpy(), ref_t.float().numpy(), nbits), got, code)
    assert e.value.status == 1


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_cached_encode_of_16_bit_parameters_is_the_fp32_method_on_the_widened_vectors(dtype):
    """encode_cached_t: with an empty cache the blob is encode_t's; a hit keeps kept buckets, counts and
    representatives (bytes 64.. of every slot but the length), names the storage type, and restores the same
    values as encode_t's blob (torch's casts give the 16-bit inputs)."""
    torch = pytest.importorskip("torch")
    tdt, code = (torch.bfloat16, orc.DT_BF16) if dtype == "bf16" else (torch.float16, orc.DT_F16)
    g = torch.Generator().manual_seed(11)
    n, nbits = lcb1_reader.C + 77, 3
    ref_t = (0.05 * torch.randn(n, generator=g)).to(tdt)
    raw = (lambda t: t.view(torch.int16).numpy().view(np.uint16).copy()) if dtype == "bf16" else (lambda t: t.numpy().copy())
    cache = orc.new_cache()
    blobs = []
    for step in range(2):
        w_t = (ref_t.float() + 2e-3 * torch.randn(n, generator=g)).to(tdt)
        # the seven largest buckets occupied at every step, so that the kept set repeats
        w_t[:7] = (ref_t[:7].float() + torch.tensor([0.02, -0.02, 0.011, -0.011, 0.005, -0.005, 0.0025])).to(tdt)
        plain = orc.encode_t(raw(w_t), raw(ref_t), nbits, code)
        blob, used = orc.encode_cached_t(raw(w_t), raw(ref_t), nbits, code, cache)
        assert used == (step == 1)
        assert int(np.frombuffer(blob[60:64].tobytes(), np.uint32)[0]) == code
        if step == 0:
            assert np.array_equal(blob, plain)
        hp, hc = lcb1_reader.parse_header(plain), lcb1_reader.parse_header(blob)
        for a, b in zip(hp["slots"], hc["slots"]):
            assert (a["bucket"], a["rep_bits"], a["cnt"]) == (b["bucket"], b["rep_bits"], b["cnt"])
        r1, r2 = raw(ref_t), raw(ref_t)
        orc.decode_t(plain, r1, code); orc.decode_t(blob, r2, code)
        assert np.array_equal(r1.view(np.uint16), r2.view(np.uint16))
        blobs.append(blob)
