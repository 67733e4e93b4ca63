"""A second, independent reading of the LCB1 blob format, in plain Python.

Written from the format text (include/lc.h), not from the oracle or the HIP
code: it parses a blob bit by bit and returns the header fields and the symbol of
every element.  Pure-Python loops, so only for small n.
"""
import struct

import numpy as np

W, V, R = 64, 4, 64
C = W * V * R
HEADER = 512


def parse_header(blob):
    b = bytes(blob[:HEADER])
    magic, version, hbytes = b[0:4], *struct.unpack_from("<HH", b, 4)
    n, nbits, K, w, v, r, nchunks, total, status, k_e, maxlen = struct.unpack_from("<QIIIIIIQIII", b, 8)
    slots = []
    for j in range(16):
        bucket, ln, pad, rep, cnt = struct.unpack_from("<HBBIQ", b, 64 + 16 * j)
        slots.append(dict(bucket=bucket, len=ln, pad=pad, rep_bits=rep, cnt=cnt))
    dtype, = struct.unpack_from("<I", b, 60)
    rep_hi = list(struct.unpack_from("<16I", b, 320))
    if dtype == 3:                      # binary64 parameters: 64-bit representatives, high halves at 320 + 4 j
        for j in range(16):
            slots[j]["rep_bits"] |= rep_hi[j] << 32
        reserved = b[384:512]
    else:
        reserved = b[320:512]
    return dict(magic=magic, version=version, header_bytes=hbytes, n=n, nbits=nbits, K=K, W=w, V=v, R=r,
                num_chunks=nchunks, total_bytes=total, status=status, k_E=k_e, max_len=maxlen, slots=slots,
                dtype=dtype, reserved=reserved)


def canonical(lens):
    """Canonical codes as bit strings, from lengths: order (len, index), count up, pad with zeros on growth."""
    order = sorted((l, s) for s, l in enumerate(lens) if l > 0)
    codes, val, prev = {}, 0, None
    for l, s in order:
        if prev is not None:
            val = (val + 1) << (l - prev)
        prev = l
        codes[s] = format(val, "0%db" % l)
    return codes


def read(blob):
    """Returns (header, sym[n] uint8, lane_bits[num_chunks][64], chunk_word_off)."""
    blob = np.asarray(blob, dtype=np.uint8)
    h = parse_header(blob)
    n, nchunks = h["n"], h["num_chunks"]
    assert nchunks == (n + C - 1) // C
    table_bytes = 4 * (nchunks + 1)
    area = HEADER + (table_bytes + 15) // 16 * 16
    off = np.frombuffer(bytes(blob[HEADER:HEADER + table_bytes]), dtype="<u4")
    assert bytes(blob[HEADER + table_bytes:area]) == b"\0" * (area - HEADER - table_bytes)
    codes = canonical([s["len"] for s in h["slots"]])
    decode_map = {bits: s for s, bits in codes.items()}
    sym = np.full(n, 255, np.uint8)
    lane_bits_all = []
    for c in range(nchunks):
        rec = area + 4 * int(off[c])
        lane_bits = np.frombuffer(bytes(blob[rec:rec + 2 * W]), dtype="<u2").astype(np.int64)
        lane_bits_all.append(lane_bits)
        nwords = (int(lane_bits.sum()) + 31) // 32
        assert int(off[c + 1]) - int(off[c]) == 2 * W // 4 + nwords, "chunk %d size" % c
        words = np.frombuffer(bytes(blob[rec + 2 * W:rec + 2 * W + 4 * nwords]), dtype="<u4")
        bits = "".join(format(int(x), "032b") for x in words)
        p = 0
        for lane in range(W):
            end = p + int(lane_bits[lane])
            for r in range(R):
                for v in range(V):
                    i = c * C + r * W * V + lane * V + v
                    if i >= n:
                        continue
                    cur = ""
                    while cur not in decode_map:
                        assert p < end, "lane stream overrun"
                        cur += bits[p]
                        p += 1
                    sym[i] = decode_map[cur]
            assert p == end, "lane stream length"
        assert set(bits[p:]) <= {"0"}, "padding must be zero"
    assert area + 4 * int(off[nchunks]) == h["total_bytes"] == blob.size
    return h, sym, lane_bits_all, off
