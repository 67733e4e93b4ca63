/*
 * lc_oracle.c -- CPU oracle for the LC-Checkpoint compress / restore path.
 *
 * THIS IS TEST INFRASTRUCTURE.  It is the slow, plain, single-threaded statement
 * of what the method computes, written from the paper (arXiv 2009.13003,
 * "On Efficient Constructions of Checkpoints") and from the LCB1 blob format.
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
 * It shares no code, header, table or constant generator with the HIP library.
 *
 * What follows the paper, and where:
 *   delta                 Algorithm 1 line 4; Section 3, component C1
 *   (sign, exponent) buckets, <= 2^9 of them for fp32, <= 2^12 for fp64 (second part of the file)
 *                         Section 3.1.1 "Exponent-based Quantization" + footnote
 *   bucket representative = average of the bucket's max and min
 *                         Section 3.1.1 "Exponent-based Quantization"
 *   size formula n*log2(k) + k*b, worked example 190 bits
 *                         Section 3.1.1 (rate formula and the n=10,k=5 example)
 *   x-bit priority promotion: keep 2^x - 1 buckets of larger exponent, merge the
 *   rest into one bucket of value 0 stored last
 *                         Section 3.1.1 "Priority Promotion"; Section 4.4 (last bucket stores 0)
 *   exponent -127 <=> value 0
 *                         Figure 2 caption
 *   Huffman coding of the bucket indices
 *                         Section 3.1.2
 *   restore u~_t = u~_{t-1} + delta~_t
 *                         Algorithm 1 line 7; Section 3, component C1
 *
 * What the paper leaves open and this file fixes by convention (parity unpinned
 * by the paper, pinned only by the format text and the tests' second decoder):
 *   - +bucket before -bucket when two candidates share an exponent,
 *   - Huffman tie-break (see lco_huffman_lengths),
 *   - canonical code assignment,
 *   - Inf/NaN deltas are rejected,
 *   - the blob layout "LCB1".
 *
 * Everything is little-endian; the host is assumed little-endian.
 * Build: gcc -O2 -std=c11 -ffp-contract=off -fno-fast-math -shared -fPIC
 */
#include <stdint.h>
#include <stddef.h>
#include <string.h>
#include <math.h>

/* ---- LCB1 geometry (format text: lane-striped chunks) ---- */
#define LCO_W 64u            /* lanes per chunk                               */
#define LCO_V 4u             /* consecutive floats a lane owns per row        */
#define LCO_R 64u            /* rows per chunk                                */
#define LCO_C (LCO_W * LCO_V * LCO_R)   /* 16384 elements per chunk           */
#define LCO_HEADER 512u
#define LCO_SLOTS 16
#define LCO_MAX_N (1ull << 32)

enum { LCO_OK = 0, LCO_BADARG = 1, LCO_NONFINITE = 2, LCO_OUT_TOO_SMALL = 3, LCO_BAD_BLOB = 4 };

static uint32_t f2u(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float u2f(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* Algorithm 1 line 4: one IEEE binary32 subtraction, round to nearest even. */
static float delta_of(float w, float wref) {
    volatile float d = w - wref;   /* volatile: no excess precision, no contraction */
    return d;
}

/*
 * Section 3.1.1, exponent-based quantization.  Bucket id = sign bit and the 8
 * exponent bits = top 9 bits of the fp32 pattern.  For every bucket: how many
 * elements, and the smallest and largest 23-bit mantissa among them (inside one
 * (sign, exponent) bucket the mantissa orders the magnitudes).  Biased exponent
 * 0 (zeros and subnormals) is the zero class (Figure 2 caption): it is counted
 * but has no min/max.  Biased exponent 255 (Inf/NaN) is an error.
 */
int lco_bucket_stats(const float* w, const float* wref, uint64_t n,
                     uint64_t count[512], uint32_t mmin[512], uint32_t mmax[512]) {
    for (int b = 0; b < 512; ++b) { count[b] = 0; mmin[b] = 0x7FFFFFu; mmax[b] = 0; }
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t u = f2u(delta_of(w[i], wref[i]));
        uint32_t b = u >> 23, E = b & 255u, m = u & 0x7FFFFFu;
        if (E == 255u) bad = 1;
        count[b] += 1;
        if (E != 0u) {
            if (m < mmin[b]) mmin[b] = m;
            if (m > mmax[b]) mmax[b] = m;
        }
    }
    return bad ? LCO_NONFINITE : LCO_OK;
}

/*
 * Section 3.1.1, priority promotion.  Candidates are the non-empty buckets with
 * a normal exponent.  They are ranked by exponent, larger first; of two buckets
 * with the same exponent the positive one ranks first.  The first
 * min(2^x - 1, #candidates) are kept and numbered 0..K-1 in rank order; every
 * other bucket (and the zero class) maps to symbol K, whose value is 0 and which
 * is stored last (Section 4.4).  Returns K.
 */
int lco_promote(const uint64_t count[512], int nbits, uint16_t kept[LCO_SLOTS],
                uint8_t sym_of_bucket[512]) {
    int kmax = (1 << nbits) - 1, K = 0;
    for (int i = 0; i < LCO_SLOTS; ++i) kept[i] = 0xFFFFu;
    for (int E = 254; E >= 1 && K < kmax; --E) {
        for (int s = 0; s <= 1 && K < kmax; ++s) {
            int b = (s << 8) | E;
            if (count[b] > 0) kept[K++] = (uint16_t)b;
        }
    }
    for (int b = 0; b < 512; ++b) sym_of_bucket[b] = (uint8_t)K;
    for (int j = 0; j < K; ++j) sym_of_bucket[kept[j]] = (uint8_t)j;
    return K;
}

/*
 * Section 3.1.1: a bucket is represented by the average of its maximum and its
 * minimum.  Both lie in one binade, so their sum is exact in binary64, halving
 * is exact, and the single rounding happens in the conversion to binary32
 * (round to nearest even).
 */
uint32_t lco_representative(uint32_t bucket, uint32_t mmin, uint32_t mmax) {
    double lo = (double)u2f((bucket << 23) | mmin);
    double hi = (double)u2f((bucket << 23) | mmax);
    float rep = (float)((lo + hi) * 0.5);
    return f2u(rep);
}

/*
 * Section 3.1.2: Huffman code lengths for m symbols with counts cnt[].  Symbols
 * with count 0 get length 0 (no code).  The construction is the textbook one:
 * repeatedly join the two smallest nodes.  "Smallest" uses the total order
 * (weight, leaf before joined node, symbol index for leaves / creation order for
 * joined nodes), which makes the lengths unique.  The first node taken becomes
 * child 0.  One active symbol gets length 1.
 */
void lco_huffman_lengths(const uint64_t* cnt, int m, uint8_t* len) {
    enum { MAXN = 2 * LCO_SLOTS };
    uint64_t weight[MAXN]; int parent[MAXN], alive[MAXN], is_joined[MAXN], order[MAXN];
    int nodes = 0, leaf_of[LCO_SLOTS], active = 0;
    for (int s = 0; s < m; ++s) {
        len[s] = 0; leaf_of[s] = -1;
        if (cnt[s] > 0) {
            weight[nodes] = cnt[s]; parent[nodes] = -1; alive[nodes] = 1;
            is_joined[nodes] = 0; order[nodes] = s; leaf_of[s] = nodes; ++nodes; ++active;
        }
    }
    if (active == 0) return;
    if (active == 1) { for (int s = 0; s < m; ++s) if (cnt[s] > 0) len[s] = 1; return; }
    int created = 0;
    for (int remaining = active; remaining > 1; --remaining) {
        int pick[2];
        for (int k = 0; k < 2; ++k) {
            int best = -1;
            for (int i = 0; i < nodes; ++i) {
                if (!alive[i]) continue;
                if (best < 0) { best = i; continue; }
                int less;
                if (weight[i] != weight[best]) less = weight[i] < weight[best];
                else if (is_joined[i] != is_joined[best]) less = is_joined[i] < is_joined[best];
                else less = order[i] < order[best];
                if (less) best = i;
            }
            pick[k] = best; alive[best] = 0;
        }
        weight[nodes] = weight[pick[0]] + weight[pick[1]];
        parent[nodes] = -1; alive[nodes] = 1; is_joined[nodes] = 1; order[nodes] = created++;
        parent[pick[0]] = nodes; parent[pick[1]] = nodes; ++nodes;
    }
    for (int s = 0; s < m; ++s) {
        if (leaf_of[s] < 0) continue;
        int d = 0;
        for (int i = leaf_of[s]; parent[i] >= 0; i = parent[i]) ++d;
        len[s] = (uint8_t)d;
    }
}

/*
 * Canonical prefix code from lengths: symbols ordered by (length, index); the
 * first gets code 0; each next code is the previous plus one, shifted left by
 * the growth in length.  Codes are read most significant bit first.
 */
void lco_canonical_codes(const uint8_t* len, int m, uint16_t* code) {
    uint32_t next = 0; int prev_len = 0, first = 1;
    for (int s = 0; s < m; ++s) code[s] = 0;
    for (int L = 1; L <= 15; ++L) {
        for (int s = 0; s < m; ++s) {
            if (len[s] != L) continue;
            if (first) { next = 0; first = 0; }
            else next = (next + 1) << (L - prev_len);
            prev_len = L;
            code[s] = (uint16_t)next;
        }
    }
}

/* ---- the quantizer as a whole (Algorithm 1 lines 4-5), no bitstream ---- */
typedef struct {
    int K;                       /* kept buckets; zero symbol = K                 */
    uint16_t kept[LCO_SLOTS];    /* bucket id of symbol j < K                     */
    uint32_t rep_bits[LCO_SLOTS + 1];
    uint64_t cnt[LCO_SLOTS + 1]; /* elements per symbol                           */
    uint8_t  len[LCO_SLOTS + 1];
    uint16_t code[LCO_SLOTS + 1];
    uint8_t  sym_of_bucket[512];
    uint32_t k_E;                /* non-empty buckets before promotion            */
} lco_model;

static int build_model(const float* w, const float* wref, uint64_t n, int nbits, lco_model* M) {
    uint64_t count[512]; uint32_t mmin[512], mmax[512];
    memset(M, 0, sizeof *M);
    int st = lco_bucket_stats(w, wref, n, count, mmin, mmax);
    if (st != LCO_OK) return st;
    M->K = lco_promote(count, nbits, M->kept, M->sym_of_bucket);
    uint64_t kept_total = 0;
    for (int j = 0; j < M->K; ++j) {
        M->cnt[j] = count[M->kept[j]];
        kept_total += M->cnt[j];
        M->rep_bits[j] = lco_representative(M->kept[j], mmin[M->kept[j]], mmax[M->kept[j]]);
    }
    M->cnt[M->K] = n - kept_total;
    M->rep_bits[M->K] = 0;                      /* the merged bucket's value is +0 */
    lco_huffman_lengths(M->cnt, M->K + 1, M->len);
    lco_canonical_codes(M->len, M->K + 1, M->code);
    /* k for the E-only size: every non-empty normal bucket, plus the zero class once */
    uint32_t k = 0; uint64_t zero_class = 0;
    for (int b = 0; b < 512; ++b) {
        if ((b & 255) == 0) zero_class += count[b];
        else if (count[b] > 0) ++k;
    }
    M->k_E = k + (zero_class > 0 ? 1u : 0u);
    return LCO_OK;
}

/*
 * Symbols and dequantized deltas, element by element, in memory order.
 * sym[i] in [0, K]; dq[i] = representative of the element's bucket, or +0.
 * info[0] = K, info[1] = k_E.
 */
int lco_quantize(const float* w, const float* wref, uint64_t n, int nbits,
                 uint8_t* sym, float* dq, uint32_t info[2]) {
    if (nbits < 1 || nbits > 4) return LCO_BADARG;
    lco_model M; int st = build_model(w, wref, n, nbits, &M);
    if (st != LCO_OK) return st;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t b = f2u(delta_of(w[i], wref[i])) >> 23;
        uint8_t s = M.sym_of_bucket[b];
        sym[i] = s; dq[i] = u2f(M.rep_bits[s]);
    }
    info[0] = (uint32_t)M.K; info[1] = M.k_E;
    return LCO_OK;
}

/* ---- LCB1 blob ---- */
static void put16(uint8_t* p, uint32_t v) { p[0] = (uint8_t)v; p[1] = (uint8_t)(v >> 8); }
static void put32(uint8_t* p, uint32_t v) { put16(p, v & 0xFFFFu); put16(p + 2, v >> 16); }
static void put64(uint8_t* p, uint64_t v) { put32(p, (uint32_t)v); put32(p + 4, (uint32_t)(v >> 32)); }
static uint32_t get16(const uint8_t* p) { return (uint32_t)p[0] | ((uint32_t)p[1] << 8); }
static uint32_t get32(const uint8_t* p) { return get16(p) | (get16(p + 2) << 16); }
static uint64_t get64(const uint8_t* p) { return (uint64_t)get32(p) | ((uint64_t)get32(p + 4) << 32); }

static uint64_t num_chunks_of(uint64_t n) { return (n + LCO_C - 1) / LCO_C; }
static uint64_t chunk_area_of(uint64_t nchunks) {
    uint64_t table = 4 * (nchunks + 1);
    return LCO_HEADER + ((table + 15) / 16) * 16;
}

/* Worst-case blob size: an optimal prefix code never needs more than nbits per symbol on average. */
uint64_t lco_encode_bound(uint64_t n, int nbits) {
    uint64_t nc = num_chunks_of(n);
    return chunk_area_of(nc) + nc * (2 * LCO_W + 4) + (n * (uint64_t)nbits + 7) / 8;
}

/* Bit p of a chunk payload lives in 32-bit word p/32 at bit position 31 - p%32. */
static void put_bit(uint8_t* payload, uint64_t p, uint32_t bit) {
    uint8_t* wp = payload + 4 * (p >> 5);
    uint32_t word = get32(wp);
    word |= (bit & 1u) << (31 - (uint32_t)(p & 31));
    put32(wp, word);
}
static uint32_t get_bit(const uint8_t* payload, uint64_t p) {
    return (get32(payload + 4 * (p >> 5)) >> (31 - (uint32_t)(p & 31))) & 1u;
}

static void write_header(uint8_t* out, uint64_t n, int nbits, const lco_model* M,
                         uint64_t nchunks, uint64_t total, uint32_t status) {
    memset(out, 0, LCO_HEADER);
    out[0] = 'L'; out[1] = 'C'; out[2] = 'B'; out[3] = '1';
    put16(out + 4, 1); put16(out + 6, LCO_HEADER);
    put64(out + 8, n); put32(out + 16, (uint32_t)nbits);
    put32(out + 24, LCO_W); put32(out + 28, LCO_V); put32(out + 32, LCO_R);
    put64(out + 40, total); put32(out + 48, status);
    if (!M) return;
    put32(out + 20, (uint32_t)M->K); put32(out + 36, (uint32_t)nchunks);
    put32(out + 52, M->k_E);
    uint32_t maxlen = 0;
    for (int j = 0; j <= M->K; ++j) {
        uint8_t* s = out + 64 + 16 * j;
        put16(s, j < M->K ? M->kept[j] : 0xFFFFu);
        s[2] = M->len[j]; s[3] = 0;
        put32(s + 4, M->rep_bits[j]); put64(s + 8, M->cnt[j]);
        if (M->len[j] > maxlen) maxlen = M->len[j];
    }
    put32(out + 56, maxlen);
}

/*
 * The blob of one checkpoint for a finished model M (kept set, representatives,
 * counts, code lengths and codes).  Returns the blob size in bytes.
 *
 * Element order inside chunk c: lane l = 0..63 owns, in this order, elements
 * c*C + r*256 + l*4 + v for r = 0..63, v = 0..3 that are < n.  A lane's codes
 * are concatenated; the 64 lane streams are concatenated in lane order without
 * gaps; the payload is zero-padded to a whole 32-bit word.  A chunk record is
 * the 64 lane bit-lengths (u16 each) followed by the payload.
 */
static int64_t write_blob(const float* w, const float* wref, uint64_t n, int nbits, const lco_model* M,
                          uint8_t* out, uint64_t cap) {
    uint64_t nchunks = num_chunks_of(n), area = chunk_area_of(nchunks);
    /* bits are OR-ed in below, so everything past the header starts at zero */
    memset(out + LCO_HEADER, 0, lco_encode_bound(n, nbits) - LCO_HEADER);
    uint64_t word_off = 0;
    for (uint64_t c = 0; c < nchunks; ++c) {
        put32(out + LCO_HEADER + 4 * c, (uint32_t)word_off);
        uint8_t* rec = out + area + 4 * word_off;
        uint8_t* payload = rec + 2 * LCO_W;
        uint64_t p = 0;                               /* bit position in the payload */
        for (uint32_t l = 0; l < LCO_W; ++l) {
            uint64_t start = p;
            for (uint32_t r = 0; r < LCO_R; ++r) for (uint32_t v = 0; v < LCO_V; ++v) {
                uint64_t i = c * LCO_C + (uint64_t)r * (LCO_W * LCO_V) + l * LCO_V + v;
                if (i >= n) continue;
                uint32_t b = f2u(delta_of(w[i], wref[i])) >> 23;
                uint32_t s = M->sym_of_bucket[b];
                if ((uint64_t)(payload - out) + 4 * ((p + M->len[s] + 31) / 32) > cap) return -LCO_OUT_TOO_SMALL;
                for (int k = M->len[s] - 1; k >= 0; --k) put_bit(payload, p++, (M->code[s] >> k) & 1u);
            }
            put16(rec + 2 * l, (uint32_t)(p - start));
        }
        word_off += (2 * LCO_W) / 4 + (p + 31) / 32;
    }
    put32(out + LCO_HEADER + 4 * nchunks, (uint32_t)word_off);
    uint64_t total = area + 4 * word_off;
    write_header(out, n, nbits, M, nchunks, total, LCO_OK);
    return (int64_t)total;
}

/*
 * Algorithm 1 lines 4-6 for one checkpoint.  Returns the blob size in bytes, or
 * -(status).  On NONFINITE the first 512 bytes of out hold a header whose status
 * field says so (if cap allows).
 */
int64_t lco_encode(const float* w, const float* wref, uint64_t n, int nbits,
                   uint8_t* out, uint64_t cap) {
    if (nbits < 1 || nbits > 4 || n > LCO_MAX_N || !out || (n && (!w || !wref))) return -LCO_BADARG;
    if (cap < lco_encode_bound(n, nbits)) return -LCO_OUT_TOO_SMALL;
    lco_model M; int st = build_model(w, wref, n, nbits, &M);
    if (st == LCO_NONFINITE) { write_header(out, n, nbits, NULL, 0, LCO_HEADER, LCO_NONFINITE); return -LCO_NONFINITE; }
    return write_blob(w, wref, n, nbits, &M, out, cap);
}

/*
 * Section 3.2, "Huffman Code Table Caching": the code table of an earlier checkpoint
 * is reused when the buckets stay the same.  Reading taken here (the paper re-sorts the
 * buckets by population first, which needs this checkpoint's populations before any code
 * is written; here the cached assignment of lengths to symbols is reused unchanged, so
 * that codes can be written while the populations are still being counted):
 *
 *   The cache holds the kept set and the code lengths of the last blob encoded with it.
 *   It is used for this checkpoint iff it is valid, was made with the same nbits, its
 *   lengths are a complete prefix code (Kraft sum 1, or a single symbol of length 1),
 *   this checkpoint's kept set (priority promotion on this delta's populations) is
 *   the cached one, exactly the symbols with a cached code occur, and the coding fits the
 *   size every blob of (n, nbits) is promised to fit: sum of count x cached length at most
 *   n * nbits bits (a stale table on shifted populations can need more than that; this
 *   checkpoint's own Huffman code never does).  Then the blob is that of lco_encode with
 *   the cached lengths in place of this delta's Huffman lengths: same quantized values,
 *   same counts and representatives, a valid but possibly longer coding.  Otherwise the
 *   blob is exactly lco_encode's.  Either way the cache afterwards holds this blob's kept
 *   set and lengths; on an error it is left alone.
 *   *used (may be NULL) = 1 if the cached table was used.
 */
typedef struct { uint32_t valid, nbits, K, pad; uint32_t kept[LCO_SLOTS]; uint32_t len[LCO_SLOTS]; } lco_cache;

int64_t lco_encode_cached(const float* w, const float* wref, uint64_t n, int nbits,
                          uint8_t* out, uint64_t cap, lco_cache* cache, int* used) {
    if (nbits < 1 || nbits > 4 || n > LCO_MAX_N || !out || !cache || (n && (!w || !wref))) return -LCO_BADARG;
    if (cap < lco_encode_bound(n, nbits)) return -LCO_OUT_TOO_SMALL;
    if (used) *used = 0;
    lco_model M; int st = build_model(w, wref, n, nbits, &M);
    if (st == LCO_NONFINITE) { write_header(out, n, nbits, NULL, 0, LCO_HEADER, LCO_NONFINITE); return -LCO_NONFINITE; }
    int ok = cache->valid == 1 && cache->nbits == (uint32_t)nbits && cache->K == (uint32_t)M.K;
    if (ok) {
        uint32_t kraft = 0; int active = 0;
        for (int j = 0; j <= M.K; ++j) {
            uint32_t l = cache->len[j];
            if (l > 15) { ok = 0; break; }
            if (l) { kraft += 1u << (15 - l); ++active; }
            if (j < M.K && cache->kept[j] != M.kept[j]) ok = 0;
            if ((l > 0) != (M.cnt[j] > 0)) ok = 0;
        }
        if (active >= 2 && kraft != (1u << 15)) ok = 0;
        if (active == 1 && kraft != (1u << 14)) ok = 0;
    }
    if (ok) {
        /* the payload under the cached lengths, against what lco_encode_bound allows for it */
        uint64_t payload_bits = 0;
        for (int j = 0; j <= M.K; ++j) payload_bits += M.cnt[j] * (uint64_t)cache->len[j];
        if (payload_bits > n * (uint64_t)nbits) ok = 0;
    }
    if (ok) {
        for (int j = 0; j <= M.K; ++j) M.len[j] = (uint8_t)cache->len[j];
        lco_canonical_codes(M.len, M.K + 1, M.code);
        if (used) *used = 1;
    }
    int64_t r = write_blob(w, wref, n, nbits, &M, out, cap);
    if (r < 0) return r;
    memset(cache, 0, sizeof *cache);
    cache->valid = 1; cache->nbits = (uint32_t)nbits; cache->K = (uint32_t)M.K;
    for (int j = 0; j < M.K; ++j) cache->kept[j] = M.kept[j];
    for (int j = 0; j <= M.K; ++j) cache->len[j] = M.len[j];
    return r;
}

/*
 * Algorithm 1 line 7 / Section 3 (restore): walk the blob, decode each lane
 * stream bit by bit against the canonical code, and add the symbol's
 * representative to the recovered weight.  An element whose symbol is the zero
 * symbol is not written at all.  Returns bytes consumed or -(status); the blob is
 * checked before wref is touched, except that a lane stream which does not
 * decode to exactly its stated length is found on the way (wref is then partly
 * updated).
 */
int64_t lco_decode(const uint8_t* blob, uint64_t blob_bytes, float* wref, uint64_t n) {
    if (!blob || blob_bytes < LCO_HEADER) return -LCO_BAD_BLOB;
    if (memcmp(blob, "LCB1", 4) != 0 || get16(blob + 4) != 1 || get16(blob + 6) != LCO_HEADER) return -LCO_BAD_BLOB;
    if (get32(blob + 48) != LCO_OK) return -LCO_BAD_BLOB;
    uint64_t hn = get64(blob + 8); uint32_t nbits = get32(blob + 16), K = get32(blob + 20);
    if (hn != n) return -LCO_BADARG;
    if (get32(blob + 60) != 0) return -LCO_BADARG;      /* element type of the parameters: this routine restores fp32 */
    if (nbits < 1 || nbits > 4 || K > (1u << nbits) - 1) return -LCO_BAD_BLOB;
    if (get32(blob + 24) != LCO_W || get32(blob + 28) != LCO_V || get32(blob + 32) != LCO_R) return -LCO_BAD_BLOB;
    uint64_t nchunks = num_chunks_of(n), area = chunk_area_of(nchunks);
    if (get32(blob + 36) != nchunks) return -LCO_BAD_BLOB;
    uint64_t total = get64(blob + 40);
    if (total > blob_bytes || total < area) return -LCO_BAD_BLOB;
    uint8_t len[LCO_SLOTS + 1]; uint16_t code[LCO_SLOTS + 1]; uint32_t rep[LCO_SLOTS + 1];
    uint64_t cnt_sum = 0; uint32_t kraft = 0; int active = 0;
    memset(len, 0, sizeof len);
    for (uint32_t j = 0; j <= K; ++j) {
        const uint8_t* s = blob + 64 + 16 * j;
        len[j] = s[2]; rep[j] = get32(s + 4);
        uint64_t c = get64(s + 8); cnt_sum += c;
        if ((c > 0) != (len[j] > 0) || len[j] > 15) return -LCO_BAD_BLOB;
        if (j < K && (get16(s) >= 512u || (get16(s) & 255u) == 0 || (get16(s) & 255u) == 255u)) return -LCO_BAD_BLOB;
        if (j < K && (rep[j] >> 23) != get16(s)) return -LCO_BAD_BLOB;
        if (len[j]) { kraft += 1u << (15 - len[j]); ++active; }
    }
    if (rep[K] != 0 || cnt_sum != n) return -LCO_BAD_BLOB;
    if (active >= 2 && kraft != (1u << 15)) return -LCO_BAD_BLOB;
    if (active == 1 && kraft != (1u << 14)) return -LCO_BAD_BLOB;
    lco_canonical_codes(len, (int)K + 1, code);
    /* structure first: offsets and lane lengths */
    uint64_t expect = 0;
    for (uint64_t c = 0; c < nchunks; ++c) {
        if (get32(blob + LCO_HEADER + 4 * c) != expect) return -LCO_BAD_BLOB;
        if (area + 4 * expect + 2 * LCO_W > total) return -LCO_BAD_BLOB;
        const uint8_t* rec = blob + area + 4 * expect;
        uint64_t bits = 0;
        for (uint32_t l = 0; l < LCO_W; ++l) bits += get16(rec + 2 * l);
        expect += (2 * LCO_W) / 4 + (bits + 31) / 32;
        if (area + 4 * expect > total) return -LCO_BAD_BLOB;
    }
    if (get32(blob + LCO_HEADER + 4 * nchunks) != expect || area + 4 * expect != total) return -LCO_BAD_BLOB;
    /* then the sweep */
    for (uint64_t c = 0; c < nchunks; ++c) {
        const uint8_t* rec = blob + area + 4 * (uint64_t)get32(blob + LCO_HEADER + 4 * c);
        const uint8_t* payload = rec + 2 * LCO_W;
        uint64_t p = 0;
        for (uint32_t l = 0; l < LCO_W; ++l) {
            uint64_t end = p + get16(rec + 2 * l);
            for (uint32_t r = 0; r < LCO_R; ++r) for (uint32_t v = 0; v < LCO_V; ++v) {
                uint64_t i = c * LCO_C + (uint64_t)r * (LCO_W * LCO_V) + l * LCO_V + v;
                if (i >= n) continue;
                uint32_t acc = 0; int L = 0, s = -1;
                while (s < 0) {
                    if (p >= end || L >= 15) return -LCO_BAD_BLOB;
                    acc = (acc << 1) | get_bit(payload, p++); ++L;
                    for (uint32_t j = 0; j <= K; ++j) if (len[j] == L && code[j] == acc) { s = (int)j; break; }
                }
                if ((uint32_t)s < K) {
                    volatile float sum = wref[i] + u2f(rep[s]);   /* one binary32 add */
                    wref[i] = sum;
                }
            }
            if (p != end) return -LCO_BAD_BLOB;
        }
    }
    return (int64_t)total;
}

/*
 * Size accounting of Section 3.1.1 / Section 4.3, in bits:
 *   acct[0] = n*ceil(log2 k) + b*k         exponent quantization alone (E), k = k_E, b = 32 (64 for binary64 blobs)
 *   acct[1] = n*x + b*2^x                  after x-bit promotion (E+P)
 *   acct[2] = 8 * blob bytes               after Huffman, all overheads included (E+P+H)
 *   acct[3] = Shannon entropy of the symbol counts, bits per element
 *   acct[4] = mean code length, bits per element (sum cnt*len / n)
 */
int lco_accounting(const uint8_t* blob, double acct[5]) {
    if (memcmp(blob, "LCB1", 4) != 0) return LCO_BAD_BLOB;
    uint64_t n = get64(blob + 8); uint32_t x = get32(blob + 16), K = get32(blob + 20), k = get32(blob + 52);
    uint32_t lg = 0; while ((1u << lg) < k) ++lg;
    double b = get32(blob + 60) == 3 ? 64.0 : 32.0;     /* bits of a stored bucket value (Section 3.1.1, rate formula) */
    acct[0] = (double)n * lg + b * k;
    acct[1] = (double)n * x + b * (double)(1u << x);
    acct[2] = 8.0 * (double)get64(blob + 40);
    double H = 0, L = 0;
    for (uint32_t j = 0; j <= K; ++j) {
        uint64_t c = get64(blob + 64 + 16 * j + 8);
        if (c == 0 || n == 0) continue;
        double pr = (double)c / (double)n;
        H -= pr * log2(pr); L += pr * blob[64 + 16 * j + 2];
    }
    acct[3] = H; acct[4] = L;
    return LCO_OK;
}

/* The E-only size of Section 3.1.1 for given n, k, b: n*ceil(log2 k) + k*b bits. */
uint64_t lco_size_exponent_only(uint64_t n, uint32_t k, uint32_t b) {
    uint32_t lg = 0; while ((1u << lg) < k) ++lg;
    return n * lg + (uint64_t)k * b;
}

/* =====================================================================================
 * Double-precision parameters.  Section 3.1.1 (footnote on the bucket count): the same
 * method with the sign and the 11 exponent bits of binary64, at most 2^12 buckets.
 * Everything is as above with 64-bit patterns: delta = fl64(w - wref), bucket = top 12
 * bits, biased exponent 0 is the zero class, 2047 is an error, mantissas have 52 bits,
 * the restore is one binary64 addition.  The blob says so at header offset 60 (3); a
 * slot holds the low 32 bits of its representative, the high 32 bits are at 320 + 4 j.
 * ===================================================================================== */
#define LCO_NB64 4096

static uint64_t d2u(double d) { uint64_t u; memcpy(&u, &d, 8); return u; }
static double u2d(uint64_t u) { double d; memcpy(&d, &u, 8); return d; }

static double delta_of64(double w, double wref) {
    volatile double d = w - wref;
    return d;
}

int lco_bucket_stats64(const double* w, const double* wref, uint64_t n,
                       uint64_t count[LCO_NB64], uint64_t mmin[LCO_NB64], uint64_t mmax[LCO_NB64]) {
    for (int b = 0; b < LCO_NB64; ++b) { count[b] = 0; mmin[b] = 0xFFFFFFFFFFFFFull; mmax[b] = 0; }
    int bad = 0;
    for (uint64_t i = 0; i < n; ++i) {
        uint64_t u = d2u(delta_of64(w[i], wref[i]));
        uint32_t b = (uint32_t)(u >> 52), E = b & 2047u;
        uint64_t m = u & 0xFFFFFFFFFFFFFull;
        if (E == 2047u) bad = 1;
        count[b] += 1;
        if (E != 0u) {
            if (m < mmin[b]) mmin[b] = m;
            if (m > mmax[b]) mmax[b] = m;
        }
    }
    return bad ? LCO_NONFINITE : LCO_OK;
}

/* Priority promotion over the 2 x 2046 normal buckets, as lco_promote. */
int lco_promote64(const uint64_t count[LCO_NB64], int nbits, uint16_t kept[LCO_SLOTS],
                  uint8_t sym_of_bucket[LCO_NB64]) {
    int kmax = (1 << nbits) - 1, K = 0;
    for (int i = 0; i < LCO_SLOTS; ++i) kept[i] = 0xFFFFu;
    for (int E = 2046; E >= 1 && K < kmax; --E) {
        for (int s = 0; s <= 1 && K < kmax; ++s) {
            int b = (s << 11) | E;
            if (count[b] > 0) kept[K++] = (uint16_t)b;
        }
    }
    for (int b = 0; b < LCO_NB64; ++b) sym_of_bucket[b] = (uint8_t)K;
    for (int j = 0; j < K; ++j) sym_of_bucket[kept[j]] = (uint8_t)j;
    return K;
}

/*
 * Average of the bucket's maximum and minimum.  Two binary64 values of one binade add
 * up to at most 54 significant bits: exact in the x87 extended format (64 bits), as is
 * the halving; the one rounding is the conversion back to binary64 (nearest even).
 */
uint64_t lco_representative64(uint32_t bucket, uint64_t mmin, uint64_t mmax) {
    _Static_assert(sizeof(long double) >= 10 && __LDBL_MANT_DIG__ >= 64, "needs a 64-bit significand");
    long double lo = (long double)u2d(((uint64_t)bucket << 52) | mmin);
    long double hi = (long double)u2d(((uint64_t)bucket << 52) | mmax);
    volatile double rep = (double)((lo + hi) * 0.5L);
    return d2u(rep);
}

typedef struct {
    int K;
    uint16_t kept[LCO_SLOTS];
    uint64_t rep_bits[LCO_SLOTS + 1];
    uint64_t cnt[LCO_SLOTS + 1];
    uint8_t  len[LCO_SLOTS + 1];
    uint16_t code[LCO_SLOTS + 1];
    uint8_t  sym_of_bucket[LCO_NB64];
    uint32_t k_E;
} lco_model64;

static uint64_t s_count64[LCO_NB64], s_mmin64[LCO_NB64], s_mmax64[LCO_NB64];   /* (single-threaded by design) */

static int build_model64(const double* w, const double* wref, uint64_t n, int nbits, lco_model64* M) {
    memset(M, 0, sizeof *M);
    int st = lco_bucket_stats64(w, wref, n, s_count64, s_mmin64, s_mmax64);
    if (st != LCO_OK) return st;
    M->K = lco_promote64(s_count64, nbits, M->kept, M->sym_of_bucket);
    uint64_t kept_total = 0;
    for (int j = 0; j < M->K; ++j) {
        M->cnt[j] = s_count64[M->kept[j]];
        kept_total += M->cnt[j];
        M->rep_bits[j] = lco_representative64(M->kept[j], s_mmin64[M->kept[j]], s_mmax64[M->kept[j]]);
    }
    M->cnt[M->K] = n - kept_total;
    M->rep_bits[M->K] = 0;
    lco_huffman_lengths(M->cnt, M->K + 1, M->len);
    lco_canonical_codes(M->len, M->K + 1, M->code);
    uint32_t k = 0; uint64_t zero_class = 0;
    for (int b = 0; b < LCO_NB64; ++b) {
        if ((b & 2047) == 0) zero_class += s_count64[b];
        else if (s_count64[b] > 0) ++k;
    }
    M->k_E = k + (zero_class > 0 ? 1u : 0u);
    return LCO_OK;
}

/* Symbols and dequantized deltas, element by element (as lco_quantize). */
int lco_quantize64(const double* w, const double* wref, uint64_t n, int nbits,
                   uint8_t* sym, double* dq, uint32_t info[2]) {
    if (nbits < 1 || nbits > 4) return LCO_BADARG;
    lco_model64 M; int st = build_model64(w, wref, n, nbits, &M);
    if (st != LCO_OK) return st;
    for (uint64_t i = 0; i < n; ++i) {
        uint32_t b = (uint32_t)(d2u(delta_of64(w[i], wref[i])) >> 52);
        uint8_t s = M.sym_of_bucket[b];
        sym[i] = s; dq[i] = u2d(M.rep_bits[s]);
    }
    info[0] = (uint32_t)M.K; info[1] = M.k_E;
    return LCO_OK;
}

static void write_header64(uint8_t* out, uint64_t n, int nbits, const lco_model64* M,
                           uint64_t nchunks, uint64_t total, uint32_t status) {
    memset(out, 0, LCO_HEADER);
    out[0] = 'L'; out[1] = 'C'; out[2] = 'B'; out[3] = '1';
    put16(out + 4, 1); put16(out + 6, LCO_HEADER);
    put64(out + 8, n); put32(out + 16, (uint32_t)nbits);
    put32(out + 24, LCO_W); put32(out + 28, LCO_V); put32(out + 32, LCO_R);
    put64(out + 40, total); put32(out + 48, status);
    put32(out + 60, 3);                                  /* element type: binary64 */
    if (!M) return;
    put32(out + 20, (uint32_t)M->K); put32(out + 36, (uint32_t)nchunks);
    put32(out + 52, M->k_E);
    uint32_t maxlen = 0;
    for (int j = 0; j <= M->K; ++j) {
        uint8_t* s = out + 64 + 16 * j;
        put16(s, j < M->K ? M->kept[j] : 0xFFFFu);
        s[2] = M->len[j]; s[3] = 0;
        put32(s + 4, (uint32_t)M->rep_bits[j]); put64(s + 8, M->cnt[j]);
        put32(out + 320 + 4 * j, (uint32_t)(M->rep_bits[j] >> 32));
        if (M->len[j] > maxlen) maxlen = M->len[j];
    }
    put32(out + 56, maxlen);
}

/* The blob of one binary64 checkpoint for a finished model; element order and records as in write_blob. */
static int64_t write_blob64(const double* w, const double* wref, uint64_t n, int nbits, const lco_model64* M,
                            uint8_t* out, uint64_t cap) {
    uint64_t nchunks = num_chunks_of(n), area = chunk_area_of(nchunks);
    memset(out + LCO_HEADER, 0, lco_encode_bound(n, nbits) - LCO_HEADER);
    uint64_t word_off = 0;
    for (uint64_t c = 0; c < nchunks; ++c) {
        put32(out + LCO_HEADER + 4 * c, (uint32_t)word_off);
        uint8_t* rec = out + area + 4 * word_off;
        uint8_t* payload = rec + 2 * LCO_W;
        uint64_t p = 0;
        for (uint32_t l = 0; l < LCO_W; ++l) {
            uint64_t start = p;
            for (uint32_t r = 0; r < LCO_R; ++r) for (uint32_t v = 0; v < LCO_V; ++v) {
                uint64_t i = c * LCO_C + (uint64_t)r * (LCO_W * LCO_V) + l * LCO_V + v;
                if (i >= n) continue;
                uint32_t b = (uint32_t)(d2u(delta_of64(w[i], wref[i])) >> 52);
                uint32_t s = M->sym_of_bucket[b];
                if ((uint64_t)(payload - out) + 4 * ((p + M->len[s] + 31) / 32) > cap) return -LCO_OUT_TOO_SMALL;
                for (int k = M->len[s] - 1; k >= 0; --k) put_bit(payload, p++, (M->code[s] >> k) & 1u);
            }
            put16(rec + 2 * l, (uint32_t)(p - start));
        }
        word_off += (2 * LCO_W) / 4 + (p + 31) / 32;
    }
    put32(out + LCO_HEADER + 4 * nchunks, (uint32_t)word_off);
    uint64_t total = area + 4 * word_off;
    write_header64(out, n, nbits, M, nchunks, total, LCO_OK);
    return (int64_t)total;
}

/* Algorithm 1 lines 4-6 for binary64 parameters. */
int64_t lco_encode64(const double* w, const double* wref, uint64_t n, int nbits,
                     uint8_t* out, uint64_t cap) {
    if (nbits < 1 || nbits > 4 || n > LCO_MAX_N || !out || (n && (!w || !wref))) return -LCO_BADARG;
    if (cap < lco_encode_bound(n, nbits)) return -LCO_OUT_TOO_SMALL;
    lco_model64 M; int st = build_model64(w, wref, n, nbits, &M);
    if (st == LCO_NONFINITE) { write_header64(out, n, nbits, NULL, 0, LCO_HEADER, LCO_NONFINITE); return -LCO_NONFINITE; }
    return write_blob64(w, wref, n, nbits, &M, out, cap);
}

/*
 * Section 3.2 table caching for binary64 parameters: the rule of lco_encode_cached word for word, on the 12-bit
 * bucket ids (a cache made by a binary32 encode names other buckets and simply does not match).
 */
int64_t lco_encode_cached64(const double* w, const double* wref, uint64_t n, int nbits,
                            uint8_t* out, uint64_t cap, lco_cache* cache, int* used) {
    if (nbits < 1 || nbits > 4 || n > LCO_MAX_N || !out || !cache || (n && (!w || !wref))) return -LCO_BADARG;
    if (cap < lco_encode_bound(n, nbits)) return -LCO_OUT_TOO_SMALL;
    if (used) *used = 0;
    lco_model64 M; int st = build_model64(w, wref, n, nbits, &M);
    if (st == LCO_NONFINITE) { write_header64(out, n, nbits, NULL, 0, LCO_HEADER, LCO_NONFINITE); return -LCO_NONFINITE; }
    int ok = cache->valid == 1 && cache->nbits == (uint32_t)nbits && cache->K == (uint32_t)M.K;
    if (ok) {
        uint32_t kraft = 0; int active = 0;
        uint64_t payload_bits = 0;
        for (int j = 0; j <= M.K; ++j) {
            uint32_t l = cache->len[j];
            if (l > 15) { ok = 0; break; }
            if (l) { kraft += 1u << (15 - l); ++active; }
            if (j < M.K && cache->kept[j] != M.kept[j]) ok = 0;
            if ((l > 0) != (M.cnt[j] > 0)) ok = 0;
            payload_bits += M.cnt[j] * (uint64_t)l;
        }
        if (active >= 2 && kraft != (1u << 15)) ok = 0;
        if (active == 1 && kraft != (1u << 14)) ok = 0;
        if (payload_bits > n * (uint64_t)nbits) ok = 0;
    }
    if (ok) {
        for (int j = 0; j <= M.K; ++j) M.len[j] = (uint8_t)cache->len[j];
        lco_canonical_codes(M.len, M.K + 1, M.code);
        if (used) *used = 1;
    }
    int64_t r = write_blob64(w, wref, n, nbits, &M, out, cap);
    if (r < 0) return r;
    memset(cache, 0, sizeof *cache);
    cache->valid = 1; cache->nbits = (uint32_t)nbits; cache->K = (uint32_t)M.K;
    for (int j = 0; j < M.K; ++j) cache->kept[j] = M.kept[j];
    for (int j = 0; j <= M.K; ++j) cache->len[j] = M.len[j];
    return r;
}

/* Algorithm 1 line 7 for binary64 parameters; checks as in lco_decode. */
int64_t lco_decode64(const uint8_t* blob, uint64_t blob_bytes, double* wref, uint64_t n) {
    if (!blob || blob_bytes < LCO_HEADER) return -LCO_BAD_BLOB;
    if (memcmp(blob, "LCB1", 4) != 0 || get16(blob + 4) != 1 || get16(blob + 6) != LCO_HEADER) return -LCO_BAD_BLOB;
    if (get32(blob + 48) != LCO_OK) return -LCO_BAD_BLOB;
    uint64_t hn = get64(blob + 8); uint32_t nbits = get32(blob + 16), K = get32(blob + 20);
    if (hn != n) return -LCO_BADARG;
    if (get32(blob + 60) != 3) return -LCO_BADARG;
    if (nbits < 1 || nbits > 4 || K > (1u << nbits) - 1) return -LCO_BAD_BLOB;
    if (get32(blob + 24) != LCO_W || get32(blob + 28) != LCO_V || get32(blob + 32) != LCO_R) return -LCO_BAD_BLOB;
    uint64_t nchunks = num_chunks_of(n), area = chunk_area_of(nchunks);
    if (get32(blob + 36) != nchunks) return -LCO_BAD_BLOB;
    uint64_t total = get64(blob + 40);
    if (total > blob_bytes || total < area) return -LCO_BAD_BLOB;
    uint8_t len[LCO_SLOTS + 1]; uint16_t code[LCO_SLOTS + 1]; uint64_t rep[LCO_SLOTS + 1];
    uint64_t cnt_sum = 0; uint32_t kraft = 0; int active = 0;
    memset(len, 0, sizeof len);
    for (uint32_t j = 0; j <= K; ++j) {
        const uint8_t* s = blob + 64 + 16 * j;
        len[j] = s[2]; rep[j] = (uint64_t)get32(s + 4) | ((uint64_t)get32(blob + 320 + 4 * j) << 32);
        uint64_t c = get64(s + 8); cnt_sum += c;
        if ((c > 0) != (len[j] > 0) || len[j] > 15) return -LCO_BAD_BLOB;
        if (j < K && (get16(s) >= 4096u || (get16(s) & 2047u) == 0 || (get16(s) & 2047u) == 2047u)) return -LCO_BAD_BLOB;
        if (j < K && (rep[j] >> 52) != get16(s)) return -LCO_BAD_BLOB;
        if (len[j]) { kraft += 1u << (15 - len[j]); ++active; }
    }
    if (rep[K] != 0 || cnt_sum != n) return -LCO_BAD_BLOB;
    if (active >= 2 && kraft != (1u << 15)) return -LCO_BAD_BLOB;
    if (active == 1 && kraft != (1u << 14)) return -LCO_BAD_BLOB;
    lco_canonical_codes(len, (int)K + 1, code);
    uint64_t expect = 0;
    for (uint64_t c = 0; c < nchunks; ++c) {
        if (get32(blob + LCO_HEADER + 4 * c) != expect) return -LCO_BAD_BLOB;
        if (area + 4 * expect + 2 * LCO_W > total) return -LCO_BAD_BLOB;
        const uint8_t* rec = blob + area + 4 * expect;
        uint64_t bits = 0;
        for (uint32_t l = 0; l < LCO_W; ++l) bits += get16(rec + 2 * l);
        expect += (2 * LCO_W) / 4 + (bits + 31) / 32;
        if (area + 4 * expect > total) return -LCO_BAD_BLOB;
    }
    if (get32(blob + LCO_HEADER + 4 * nchunks) != expect || area + 4 * expect != total) return -LCO_BAD_BLOB;
    for (uint64_t c = 0; c < nchunks; ++c) {
        const uint8_t* rec = blob + area + 4 * (uint64_t)get32(blob + LCO_HEADER + 4 * c);
        const uint8_t* payload = rec + 2 * LCO_W;
        uint64_t p = 0;
        for (uint32_t l = 0; l < LCO_W; ++l) {
            uint64_t end = p + get16(rec + 2 * l);
            for (uint32_t r = 0; r < LCO_R; ++r) for (uint32_t v = 0; v < LCO_V; ++v) {
                uint64_t i = c * LCO_C + (uint64_t)r * (LCO_W * LCO_V) + l * LCO_V + v;
                if (i >= n) continue;
                uint32_t acc = 0; int L = 0, s = -1;
                while (s < 0) {
                    if (p >= end || L >= 15) return -LCO_BAD_BLOB;
                    acc = (acc << 1) | get_bit(payload, p++); ++L;
                    for (uint32_t j = 0; j <= K; ++j) if (len[j] == L && code[j] == acc) { s = (int)j; break; }
                }
                if ((uint32_t)s < K) {
                    volatile double sum = wref[i] + u2d(rep[s]);   /* one binary64 add */
                    wref[i] = sum;
                }
            }
            if (p != end) return -LCO_BAD_BLOB;
        }
    }
    return (int64_t)total;
}
