// Decode kernels of the LC-Checkpoint compress / restore path for gfx950 (wave64): restore by
// accumulation (Algorithm 1 line 7; Section 3, C1).
//
// lc_decode:        k_dec_check -> k_decode (gated on the check's verdict, no host round trip between)
// lc_decode_many:   k_dec_check (all blobs) -> k_decode_fused<T> per sweep
// lc_decode_batch:  kb_dec_setup -> kb_dec_tables -> kb_dec_chunks -> kb_decode -> kb_dec_report
#include "lc_device.h"
#include <type_traits>

namespace lc {

// ----------------------------------------------------------------------------- k_dec_check
// Everything lc_decode verifies before w_ref is touched, in one launch.  Every workgroup
// re-reads the header and does the cheap sanity checks that keep its own reads in bounds;
// workgroup 0 additionally validates the symbol table, rebuilds the canonical codes and the
// look-up table; each wavefront checks one chunk: the offset table must be the running sum
// of the record sizes that the lane lengths imply, from 0 to the blob's stated size.
// Errors are raised with atomicMax on a word tagged with the call's epoch, so the word
// never needs clearing.
// Thread 0 of a workgroup: validates the header's symbol table, builds the canonical codes and fills
// D.info; s_len / s_code (LDS, kMaxSym entries) are left for dec_build_luts.  Returns whether the blob passes.
__device__ __forceinline__ bool dec_symbol_table(const u32* hdr, u64 n, u32 nchunks, u64 area, u64 tw, DecSet& D,
                                                 u32* s_len, u32* s_code) {
    const u32 nbits = hdr[4], K = hdr[5];
    // binary64 blobs (element type 3): 12-bit bucket ids, 64-bit representatives with the high halves at offset 320
    const bool wide = hdr[15] == (u32)kF64;
    const u32 emask = wide ? 2047u : 255u, nbuckets = 2 * (emask + 1);
    bool ok = nbits >= 1 && nbits <= 4 && K <= (1u << nbits) - 1 && hdr[6] == kW && hdr[7] == kV && hdr[8] == kR;
    if (nchunks == 0 && tw != 0) ok = false;
    u64 cnt_sum = 0; u32 kraft = 0, active = 0, max_len = 0;
    u32 per_len[17];
    for (int L = 0; L <= 16; ++L) per_len[L] = 0;
    for (u32 j = 0; j < kMaxSym; ++j) { s_len[j] = 0; s_code[j] = 0; D.info.rep_bits[j] = 0; D.info.rep_hi[j] = 0; }
    if (ok) {
        for (u32 j = 0; j <= K; ++j) {
            const u32 w0 = hdr[16 + 4 * j], rep = hdr[17 + 4 * j];
            const u64 cn = hdr[18 + 4 * j] | ((u64)hdr[19 + 4 * j] << 32);
            const u32 bucket = w0 & 0xFFFFu, len = (w0 >> 16) & 0xFFu;
            cnt_sum += cn;
            if ((cn > 0) != (len > 0) || len > 15 || (w0 >> 24) != 0) { ok = false; continue; }
            const u32 rep_hi = wide ? hdr[80 + j] : 0u;
            if (j < K && (bucket >= nbuckets || (bucket & emask) == 0 || (bucket & emask) == emask)) ok = false;
            if (j < K && (wide ? (rep_hi >> 20) : (rep >> 23)) != bucket) ok = false;
            if (j == K && (rep | rep_hi) != 0) ok = false;
            s_len[j] = len; D.info.rep_bits[j] = rep; D.info.rep_hi[j] = rep_hi;
            if (len) { kraft += 1u << (15 - len); ++active; per_len[len]++; if (len > max_len) max_len = len; }
        }
        if (cnt_sum != n) ok = false;
        if (active >= 2 && kraft != (1u << 15)) ok = false;
        if (active == 1 && kraft != (1u << 14)) ok = false;
    }
    if (ok) {
        u32 next_code[17], code = 0;
        for (int L = 1; L <= 16; ++L) { code = (code + per_len[L - 1]) << 1; next_code[L] = code; }
        for (u32 j = 0; j < kMaxSym; ++j) {
            s_code[j] = s_len[j] ? next_code[s_len[j]]++ : 0;
            D.info.len[j] = s_len[j]; D.info.code[j] = s_code[j];
        }
    }
    D.info.K = K; D.info.max_len = max_len;
    D.info.area = area; D.info.total_words = tw;
    return ok;
}

// Two tables over the next P bits of a lane's string, entry = symbol | len << 4.  A prefix that
// starts no code: symbol K with length 0 (the lane then falls short of its stated length); a
// prefix of a code longer than P bits: 0xFF.  The first table (P = min(max_len, 7): 128 bytes,
// one 32-bit word per LDS bank) resolves the frequent short codes without bank conflicts.
__device__ __forceinline__ void dec_build_luts(DecSet& D, const u32* s_len, const u32* s_code, u32 t, u32 nthr) {
    const u32 M = D.info.max_len, K = D.info.K;
    const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits, P2 = M < kDecLut2Bits ? M : kDecLut2Bits;
    for (u32 pass = 0; pass < 2; ++pass) {
        const u32 P = pass ? P2 : P1;
        uint8_t* lut = pass ? D.lut2 : D.lut1;
        if (pass && M <= kDecLut1Bits) break;
        // every thread of the workgroup takes part: first "starts no code" everywhere, then each code's own range
        // of prefixes (the ranges of a prefix code do not overlap), all threads sharing the entries of a range
        for (u32 i = t; i < (1u << P); i += nthr) lut[i] = (uint8_t)K;
        __syncthreads();
        for (u32 j = 0; j <= K; ++j) {
            const u32 L = s_len[j];
            if (L == 0) continue;
            if (L <= P) {
                const u32 first = s_code[j] << (P - L), count = 1u << (P - L);
                for (u32 i = t; i < count; i += nthr) lut[first + i] = (uint8_t)(j | (L << 4));
            } else if (t == 0) {
                lut[s_code[j] >> (L - P)] = 0xFF;
            }
        }
        __syncthreads();
    }
}

// One chunk's place in the offset table against the lane lengths of its record, by one wavefront.
__device__ __forceinline__ bool dec_chunk_ok(const uint8_t* blob, u64 area, u64 tw, u32 nchunks, u32 c) {
    const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
    const u64 o0 = off_tab[c], o1 = off_tab[c + 1];
    bool ok = o0 <= o1 && o1 <= tw && o1 - o0 >= kLaneBitsWords && (c > 0 || o0 == 0) && (c + 1 < nchunks || o1 == tw);
    if (ok) {
        const u32 lb = reinterpret_cast<const uint16_t*>(blob + area + 4 * o0)[lane_id()];
        const u32 sum = wave_sum32(lb);
        ok = (o1 - o0 == kLaneBitsWords + ((sum + 31) >> 5)) && sum > 0 && !__any(lb > kR * kV * 15);
    }
    return ok;
}

// The same for chunks c0 .. c0 + 3 at once (their loads in flight together); false if any of those below nchunks fails.
__device__ __forceinline__ bool dec_chunks_ok4(const uint8_t* blob, u64 area, u64 tw, u32 nchunks, u32 c0) {
    const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
    const u32 lane = lane_id();
    u64 o[5];
#pragma unroll
    for (u32 k = 0; k < 5; ++k) o[k] = c0 + k <= nchunks ? off_tab[c0 + k] : 0;
    bool ok[4];
    u32 lb[4];
#pragma unroll
    for (u32 k = 0; k < 4; ++k) {
        const u32 c = c0 + k;
        ok[k] = c < nchunks && o[k] <= o[k + 1] && o[k + 1] <= tw && o[k + 1] - o[k] >= kLaneBitsWords && (c > 0 || o[k] == 0) &&
                (c + 1 < nchunks || o[k + 1] == tw);
        lb[k] = ok[k] ? reinterpret_cast<const uint16_t*>(blob + area + 4 * o[k])[lane] : 0u;
    }
    bool all = true;
#pragma unroll
    for (u32 k = 0; k < 4; ++k) {
        if (c0 + k >= nchunks) continue;
        const u32 sum = wave_sum32(lb[k]);
        all = all && ok[k] && (o[k + 1] - o[k] == kLaneBitsWords + ((sum + 31) >> 5)) && sum > 0 && !__any(lb[k] > kR * kV * 15);
    }
    return all;
}

__device__ __forceinline__ void raise_status(Workspace* ws, HostResult* host, u64 epoch, u32 status) {
    const u64 word = (epoch << 8) | status;
    atomicMax(&ws->dec_status, word);     // gates the decode sweep on the device
    host->dec_status = word;              // what the host reads after waiting for the stream (any finding will do)
}

// PER: chunks per wavefront, 1 or 4 (4 when one chunk each would take many rounds of workgroups: several blobs, or a long one)
template <int PER>
__global__ __launch_bounds__(256) void k_dec_check(BlobList blobs, u32 first, u64 n, u64 max_total, Workspace* ws,
                                                   u32 nchunks, u64 epoch, HostResult* host, u32 dtype) {
    const u32 set = first + blockIdx.y, host_slot = set;     // one grid row per blob
    const uint8_t* blob = blobs.p[set];
    __shared__ u32 hdr[kHeaderBytes / 4];
    __shared__ u32 s_ok;
    __shared__ u32 s_len[kMaxSym], s_code[kMaxSym];
    const u32 t = threadIdx.x, lane = lane_id();
    if (t < kHeaderBytes / 4) hdr[t] = reinterpret_cast<const u32*>(blob)[t];
    __syncthreads();
    const u64 hn = hdr[2] | ((u64)hdr[3] << 32), total = hdr[10] | ((u64)hdr[11] << 32);
    const u64 area = chunk_area_of(nchunks);
    const bool head_ok = hdr[0] == 0x3142434Cu && hdr[1] == (1u | (kHeaderBytes << 16)) && hdr[12] == 0 &&
                         hn == n && hdr[15] == dtype && hdr[9] == nchunks && total >= area && total <= max_total &&
                         ((total - area) & 3) == 0;
    if (!head_ok) {
        if (blockIdx.x == 0 && t == 0) {
            const bool n_mismatch = hdr[0] == 0x3142434Cu && hdr[1] == (1u | (kHeaderBytes << 16)) && hdr[12] == 0 &&
                                    (hn != n || hdr[15] != dtype);       // a sound blob for another vector or element type
            raise_status(ws, host, epoch, n_mismatch ? 1u : 4u);
            host->bytes[host_slot] = 0; host->max_len[host_slot] = 0;
        }
        return;
    }
    const u64 tw = (total - area) / 4;
    // ---- one chunk, or four, per wavefront
    const u32 c0 = (blockIdx.x * 4 + (t >> 6)) * PER;
    if (c0 < nchunks) {
        const bool ok = PER == 4 ? dec_chunks_ok4(blob, area, tw, nchunks, c0) : dec_chunk_ok(blob, area, tw, nchunks, c0);
        if (!ok && lane == 0) raise_status(ws, host, epoch, 4u);
    }
    if (blockIdx.x != 0) return;
    // ---- workgroup 0: symbol table, codes, look-up table
    DecSet& D = ws->dec_set[set];
    if (t == 0) {
        const bool ok = dec_symbol_table(hdr, n, nchunks, area, tw, D, s_len, s_code);
        if (!ok) raise_status(ws, host, epoch, 4u);
        host->bytes[host_slot] = total; host->max_len[host_slot] = D.info.max_len;
        s_ok = ok;
    }
    __syncthreads();
    if (!s_ok) return;
    dec_build_luts(D, s_len, s_code, t, 256);
}

// ----------------------------------------------------------------------------- k_decode
// Algorithm 1 line 7: one wavefront per chunk, lane l decoding its own string with a 64-bit
// MSB-first window.  The chunk's payload is first copied to LDS with coalesced 16-byte loads, so
// the lanes' word-by-word refills never go to memory.  Symbols come from the two look-up tables
// (codes longer than 12 bits take a short search); the merged symbol adds -0.0, which leaves
// every fp32 pattern unchanged, and a row in which no lane decoded a kept symbol is not written
// back at all.
constexpr u32 kPayWords = 2048;      // LDS room for one chunk's payload (4 bits per element on average) when the
                                     // compute unit is shared by as many workgroups as fit; more when fewer are needed
constexpr u32 kSparseSlack = 512;    // bits above an all-merged chunk up to which a chunk is decoded symbols first
constexpr u32 kPayWordsMax = 3808;   // what keeps a workgroup's LDS within 64 KB (7.4 bits per element on average)

struct DecLds {
    uint8_t lut1[1u << kDecLut1Bits];
    uint8_t lut2[1u << kDecLut2Bits];
    float rep[kMaxSym];
    u32 len[kMaxSym], code[kMaxSym];
    double rep64[kMaxSym];            // binary64 blobs: the representatives (rep is not used then)
    template <int DT> __device__ __forceinline__ typename Val<DT>::type rep_of(u32 sy) const {
        if constexpr (DT == kF64) return rep64[sy];
        else return rep[sy];
    }
};

template <typename LDS>
__device__ __noinline__ u32 decode_long(const LDS& L, u64 win, u32 K) {
    const u32 peek = (u32)(win >> (64 - 15));
    for (u32 j = 0; j <= K; ++j) {
        const u32 l = L.len[j];
        if (l > kDecLut2Bits && (peek >> (15 - l)) == L.code[j]) return j | (l << 4);
    }
    return K;
}

// MSB-first bit window over payload words that live in LDS (STAGED) or in global memory.
template <bool STAGED>
struct BitReader {
    const u32* pw;                   // payload words (index 0 = first word of the chunk's payload)
    u32 last;                        // index of the last payload word (reads are clamped to it)
    u64 win;                         // next bits, left aligned
    u32 avail, wi, next;             // valid bits in win; index of `next`; the word after the window
    __device__ __forceinline__ u32 word(u32 i) const { return pw[min(i, last)]; }
    __device__ __forceinline__ void start(const u32* words, u32 nwords, u32 first_bit) {
        pw = words; last = nwords - 1;
        wi = first_bit >> 5;
        const u32 sh = first_bit & 31;
        win = (((u64)word(wi) << 32) | word(wi + 1)) << sh;
        avail = 64 - sh;
        wi += 2;
        next = word(wi);
    }
    __device__ __forceinline__ void refill() {           // call when avail <= 32
        win |= (u64)next << (32 - avail);
        avail += 32; ++wi;
        next = word(wi);
    }
};

// `raise(code)` reports a lane string that does not decode to its stated length.
// DEEP: the launch has so few wavefronts that nothing hides a wavefront's waits on memory: rows are then fetched 8 at
// a time (2-byte elements: 16), two such batches in flight, instead of 4.
// VERIFY: the lane strings are only decoded and measured against their stated lengths; w_ref is not touched (nor read).
template <bool FAST, bool LV2, bool STAGED, int DT, bool DEEP, bool VERIFY, typename LDS, typename Raise>
__device__ __forceinline__ void decode_rows(const u32* words, u32 nwords, u32 first_bit, u32 lane_bits,
                                            void* __restrict__ w_ref, u64 n, u32 c,
                                            const LDS& L, u32 P1, u32 P2, u32 K, u32 row_zero_bits, bool sparse, Raise& raise) {
    const u32 lane = lane_id();
    BitReader<STAGED> br;
    br.start(words, nwords, first_bit);
    const u32 wi0 = br.wi, avail0 = br.avail;
    const u32 shr1 = 64 - P1, shr2 = 64 - P2;
    const u64 base = (u64)c * kChunk;
    if constexpr (VERIFY) {
        auto symbols_of_row = [&](u64 idx) {
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (FAST || idx + v < n) {
                    u32 e = L.lut1[(u32)(br.win >> shr1)];
                    if (LV2 && e == 0xFF) {
                        e = L.lut2[(u32)(br.win >> shr2)];
                        if (e == 0xFF) e = decode_long(L, br.win, K);
                    }
                    const u32 len = e >> 4;
                    br.win <<= len; br.avail -= len;
                }
                if ((v & 1) && br.avail <= 32) br.refill();
            }
        };
        if (sparse && row_zero_bits != 0) {
            // a chunk with few kept symbols: a whole row of merged symbols whose code is zeros is passed over as in
            // the restoring sweep (in a loop of its own: elsewhere the test costs more than it saves)
            for (u32 r = 0; r < kR && (FAST || base + (u64)r * kRowElems < n); ++r) {
                if ((FAST || base + (u64)(r + 1) * kRowElems <= n) && !__any((u32)(br.win >> (64 - row_zero_bits)) != 0)) {
                    br.win <<= row_zero_bits; br.avail -= row_zero_bits;
                    if (br.avail <= 32) br.refill();
                    continue;
                }
                symbols_of_row(base + (u64)r * kRowElems + lane * kV);
            }
        } else {
            for (u32 r = 0; r < kR && (FAST || base + (u64)r * kRowElems < n); ++r) symbols_of_row(base + (u64)r * kRowElems + lane * kV);
        }
        const u32 used = avail0 + 32 * (br.wi - wi0) - br.avail;
        if (__any(used != lane_bits) && lane == 0) raise(4u);
        return;
    }
    // one row of the chunk; WHOLE: all 4 elements of every lane exist and the row can be stored as vectors
    typedef typename Val<DT>::type val_t;
    auto row = [&](auto whole, u64 idx, val_t (&x)[4]) {
        constexpr bool WHOLE = decltype(whole)::value;
        // row_zero_bits = 4 x the merged symbol's code length when that code is all zero bits (at most 32): so many
        // zero bits at the head of every lane's window are 4 merged symbols each, and the row stays as it is
        if (WHOLE && row_zero_bits != 0 && !__any((u32)(br.win >> (64 - row_zero_bits)) != 0)) {
            br.win <<= row_zero_bits; br.avail -= row_zero_bits;
            if (br.avail <= 32) br.refill();
            return;
        }
        u32 smin = K;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (WHOLE || idx + v < n) {
                u32 e = L.lut1[(u32)(br.win >> shr1)];
                if (LV2 && e == 0xFF) {
                    e = L.lut2[(u32)(br.win >> shr2)];
                    if (e == 0xFF) e = decode_long(L, br.win, K);
                }
                const u32 len = e >> 4, sy = e & 15;
                br.win <<= len; br.avail -= len;
                smin = min(smin, sy);
                x[v] = add_rn(x[v], L.template rep_of<DT>(sy));
            }
            if ((v & 1) && br.avail <= 32) br.refill();
        }
        if (WHOLE) {
            if (__any(smin < K)) store4_v<DT>(w_ref, idx, x);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) if (idx + v < n) store_one_v<DT>(w_ref, idx + v, x[v]);
        }
    };
    typedef std::integral_constant<bool, true> yes;
    typedef std::integral_constant<bool, false> no;
    const bool vec = FAST || (reinterpret_cast<uintptr_t>(w_ref) & (DT == kF64 ? 15 : 4 * elem_bytes<DT>() - 1)) == 0;
    if (sparse && vec) {
        // A chunk that holds few kept symbols (its caller has seen that from its size): a row of merged symbols
        // needs no look at w_ref at all, so the symbols come first, a group of rows at a time, and only the rows
        // in which some lane decoded a kept symbol are then fetched (together), added to and stored.  The one
        // wavefront that owns such a chunk no longer waits for 64 rows of memory, only for the few it changes.
        constexpr u32 G = DT == kF64 ? 4 : 8;
        // the symbols of one whole row: 4 representatives per lane; true if any lane holds a kept symbol
        auto row_reps = [&](val_t (&rp)[4]) -> bool {
            if (row_zero_bits != 0 && !__any((u32)(br.win >> (64 - row_zero_bits)) != 0)) {
                br.win <<= row_zero_bits; br.avail -= row_zero_bits;
                if (br.avail <= 32) br.refill();
                return false;
            }
            u32 smin = K;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                u32 e = L.lut1[(u32)(br.win >> shr1)];
                if (LV2 && e == 0xFF) {
                    e = L.lut2[(u32)(br.win >> shr2)];
                    if (e == 0xFF) e = decode_long(L, br.win, K);
                }
                const u32 len = e >> 4, sy = e & 15;
                br.win <<= len; br.avail -= len;
                smin = min(smin, sy);
                rp[v] = L.template rep_of<DT>(sy);
                if ((v & 1) && br.avail <= 32) br.refill();
            }
            return __any(smin < K);
        };
        const u64 left = n - base;
        const u32 whole_rows = FAST ? kR : (u32)(left / kRowElems < kR ? left / kRowElems : kR);
        u32 r = 0;
        for (; r + G <= whole_rows; r += G) {
            val_t rp[G][4], x[G][4];
            bool kept[G];
#pragma unroll
            for (u32 k = 0; k < G; ++k) kept[k] = row_reps(rp[k]);
#pragma unroll
            for (u32 k = 0; k < G; ++k)
                if (kept[k]) load_row_v<true, DT>(w_ref, base + (u64)(r + k) * kRowElems + lane * kV, n, x[k]);
#pragma unroll
            for (u32 k = 0; k < G; ++k) {
                if (kept[k]) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) x[k][v] = add_rn(x[k][v], rp[k][v]);
                    store4_v<DT>(w_ref, base + (u64)(r + k) * kRowElems + lane * kV, x[k]);
                }
            }
        }
        for (; r < whole_rows; ++r) {
            val_t rp[4], x[4];
            if (row_reps(rp)) {
                const u64 idx = base + (u64)r * kRowElems + lane * kV;
                load_row_v<true, DT>(w_ref, idx, n, x);
#pragma unroll
                for (int v = 0; v < 4; ++v) x[v] = add_rn(x[v], rp[v]);
                store4_v<DT>(w_ref, idx, x);
            }
        }
        for (; r < kR && base + (u64)r * kRowElems < n; ++r) {
            const u64 idx = base + (u64)r * kRowElems + lane * kV;
            val_t x[4];
            load_row_v<false, DT>(w_ref, idx, n, x);
            row(no(), idx, x);
        }
    } else if (FAST && DT == kF32 && !DEEP) {
#pragma unroll 4
        for (u32 r = 0; r < kR; ++r) {
            const u64 idx = base + (u64)r * kRowElems + lane * kV;
            val_t x[4];
            load_row_v<true, DT>(w_ref, idx, n, x);
            row(yes(), idx, x);
        }
    } else if (FAST) {
        // 2-byte and 8-byte elements: rows in batches of 4, the next batch fetched before this one is decoded and stored
        // (in program order: the compiler does not move a load above an earlier store of the same kind).  13 % faster
        // than the loop above for bf16, 1 % for fp64; 3 % slower for fp32, which keeps the loop.
        constexpr u32 PF = DEEP ? ((DT == kF64 || DT == kF32) ? 8 : 16) : 4;        // (two workgroups must still fit a compute unit)
        typedef typename Raw<DT>::type raw_t;
        auto fetch = [&](raw_t (&X)[PF], u32 r0) {
#pragma unroll
            for (u32 k = 0; k < PF; ++k) X[k] = load_raw<DT>(w_ref, base + (u64)(r0 + k) * kRowElems + lane * kV);
        };
        auto batch = [&](const raw_t (&X)[PF], u32 r0) {
#pragma unroll
            for (u32 k = 0; k < PF; ++k) {
                val_t x[4];
                if constexpr (DT == kF64) unpack64(X[k], x); else unpack<DT>(X[k], x);
                row(yes(), base + (u64)(r0 + k) * kRowElems + lane * kV, x);
            }
        };
        raw_t A[PF], B[PF];
        fetch(A, 0);
        for (u32 r0 = 0; r0 < kR; r0 += 2 * PF) {
            fetch(B, r0 + PF);
            batch(A, r0);
            if (r0 + 2 * PF < kR) fetch(A, r0 + 2 * PF);
            batch(B, r0 + PF);
        }
    } else {
        // A ragged or unaligned chunk (the vector's last chunk is one wavefront's work from start to end, so its
        // memory round trips count): whole rows of an aligned array as in a full chunk, four fetched before the
        // first is decoded; the rest with guarded element accesses.
        u32 r = 0;
        if (vec) {
            constexpr u32 RB = 4;
            for (; r + RB <= kR && base + (u64)(r + RB) * kRowElems <= n; r += RB) {
                val_t x[RB][4];
#pragma unroll
                for (u32 k = 0; k < RB; ++k) load_row_v<true, DT>(w_ref, base + (u64)(r + k) * kRowElems + lane * kV, n, x[k]);
#pragma unroll
                for (u32 k = 0; k < RB; ++k) row(yes(), base + (u64)(r + k) * kRowElems + lane * kV, x[k]);
            }
        }
        for (; r < kR && base + (u64)r * kRowElems < n; ++r) {
            const u64 idx = base + (u64)r * kRowElems + lane * kV;
            val_t x[4];
            load_row_v<false, DT>(w_ref, idx, n, x);
            row(no(), idx, x);
        }
    }
    const u32 used = avail0 + 32 * (br.wi - wi0) - br.avail;
    if (__any(used != lane_bits) && lane == 0) raise(4u);
}

// zero_bits: what every lane length of a full chunk is when all its elements are the merged symbol and that
// symbol's code is all zero bits (the canonical first code), else 0.  Such a chunk with an all-zero payload
// decodes to the merged symbol throughout, exactly: it changes nothing and is left without reading w_ref.
__device__ __forceinline__ u32 zero_chunk_bits(u32 len_merged, u32 code_merged) {
    return (len_merged != 0 && code_merged == 0) ? kR * kV * len_merged : 0u;
}

// pay: this wavefront's LDS area of pay_words + 4 words for the chunk's payload
template <bool FAST, bool LV2, int DT, bool DEEP = false, bool VERIFY = false, typename LDS, typename Raise>
__device__ __forceinline__ void decode_chunk(const uint8_t* __restrict__ blob, void* __restrict__ w_ref, u64 n,
                                             u32 c, u32 o0, u32 o1, LDS& L, uint4* pay, u32 pay_words, u32 P1, u32 P2, u32 K,
                                             u64 area, u32 zero_bits, Raise& raise) {
    // o0, o1: the chunk's entries c and c + 1 of the offset table (fetched by the caller, ahead of time)
    const u32 lane = lane_id();
    const uint8_t* rec = blob + area + 4 * (u64)o0;
    const u32 nwords = o1 - o0 - kLaneBitsWords;        // >= 1 (validated)
    const u32 lane_bits = reinterpret_cast<const uint16_t*>(rec)[lane];
    const u32 o = wave_incl_scan(lane_bits) - lane_bits;
    const u32* gw = reinterpret_cast<const u32*>(rec + 2 * kW);
    const u32 k0 = (u32)((reinterpret_cast<uintptr_t>(gw) >> 2) & 3);     // words between the 16-byte boundary and the payload
    // 4 merged symbols in a row are this many zero bits (when the merged code is zeros, and short enough to test)
    const u32 whole_zero = zero_chunk_bits(L.len[K], L.code[K]);
    const u32 row_zero_bits = whole_zero / (kR * kV) * kV <= 32 ? whole_zero / (kR * kV) * kV : 0u;
    // Few kept symbols?  When the merged symbol's code is shorter than every other, each kept symbol costs at least
    // one bit more, so a chunk of at most kSparseSlack bits above (elements x merged length) holds at most that many.
    u32 len_merged = L.len[K];
    for (u32 j = 0; j < K; ++j) if (L.len[j] != 0 && L.len[j] <= L.len[K]) len_merged = 0;
    const u64 left = n - (u64)c * kChunk;
    const u32 elems = left < kChunk ? (u32)left : kChunk;
    const u32 chunk_bits = read_lane(o + lane_bits, kW - 1);
    const bool sparse = len_merged != 0 && chunk_bits <= elems * len_merged + kSparseSlack;
    if (nwords + k0 <= pay_words) {
        // coalesced copy of [aligned start, payload end) to LDS; the bytes before the payload are the
        // record's own lane lengths, and the last vector is read word by word so no read passes the end
        const uint4* gv = reinterpret_cast<const uint4*>(gw - k0);
        const u32 nvec = (nwords + k0 + 3) >> 2;
        u32 nonzero = 0;
        for (u32 i = lane; i < nvec; i += kW) {
            uint4 q;
            if (4 * i + 4 <= nwords + k0) q = gv[i];
            else {
                const u32* t = reinterpret_cast<const u32*>(gv + i);
                const u32 left = nwords + k0 - 4 * i;
                q.x = t[0]; q.y = left > 1 ? t[1] : 0; q.z = left > 2 ? t[2] : 0; q.w = 0;
            }
            pay[i] = q;
            // payload words only: the first vector may start with up to 3 words of lane lengths
            nonzero |= (i == 0) ? ((k0 < 1 ? q.x : 0u) | (k0 < 2 ? q.y : 0u) | (k0 < 3 ? q.z : 0u) | q.w) : (q.x | q.y | q.z | q.w);
        }
        if (zero_bits != 0 && !__any(lane_bits != zero_bits || nonzero != 0)) return;
        decode_rows<FAST, LV2, true, DT, DEEP, VERIFY>(reinterpret_cast<const u32*>(pay) + k0, nwords, o, lane_bits,
                                         w_ref, n, c, L, P1, P2, K, row_zero_bits, sparse, raise);
    } else {
        decode_rows<FAST, LV2, false, DT, DEEP, VERIFY>(gw, nwords, o, lane_bits, w_ref, n, c, L, P1, P2, K, row_zero_bits, sparse, raise);
    }
}

// VERIFY: lc_verify's sweep (and the one lc_decode runs first when asked to): the same walk over the blob, decoding
// only; `w_ref` is not used.
template <int DT, bool DEEP, bool VERIFY = false>
__global__ __launch_bounds__(256) void k_decode(const uint8_t* __restrict__ blob, void* __restrict__ w_ref, u64 n,
                                                Workspace* ws, u32 nchunks, int aligned, u64 epoch, HostResult* host,
                                                u32 pay_words, u32 set) {
    __shared__ DecLds L;
    extern __shared__ uint4 dec_pay[];                   // 4 areas of pay_words + 4 payload words, one per wavefront
    // What the check kernel left (the verdict and the blob's tables) is fetched in one go: a failed check leaves
    // tables that mean nothing, but reading them is harmless.  If it found something, nothing else is touched.
    const u32 t = threadIdx.x;
    const DecSet& D = ws->dec_set[set];
    const u64 verdict = __hip_atomic_load(&ws->dec_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    u32 M = D.info.max_len, K = D.info.K;
    u64 area = D.info.area;
    u32 lut1_entry = t < (1u << kDecLut1Bits) ? D.lut1[t] : 0u;
    u32 sym_rep = 0, sym_rep_hi = 0, sym_len = 0, sym_code = 0;
    if (t < kMaxSym) { sym_rep = D.info.rep_bits[t]; sym_rep_hi = D.info.rep_hi[t]; sym_len = D.info.len[t]; sym_code = D.info.code[t]; }
    // (the empty statement keeps these loads ahead of the branch; the values every lane holds alike go back to scalars)
    asm volatile("" : "+v"(M), "+v"(K), "+v"(area), "+v"(lut1_entry), "+v"(sym_rep), "+v"(sym_rep_hi), "+v"(sym_len), "+v"(sym_code));
    M = __builtin_amdgcn_readfirstlane(M); K = __builtin_amdgcn_readfirstlane(K);
    area = ((u64)__builtin_amdgcn_readfirstlane((u32)(area >> 32)) << 32) | __builtin_amdgcn_readfirstlane((u32)area);
    if ((verdict >> 8) != epoch) {
        const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits, P2 = M < kDecLut2Bits ? M : kDecLut2Bits;
        const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
        const u32 wave = t >> 6, stride = gridDim.x * 4;
        u32 c = blockIdx.x * 4 + wave;
        u32 o0 = 0, o1 = 0;
        if (c < nchunks) { o0 = off_tab[c]; o1 = off_tab[c + 1]; }
        if (t < (1u << P1)) L.lut1[t] = (uint8_t)lut1_entry;
        if (M > kDecLut1Bits) {
            if ((1u << P2) >= 4096) {
                const uint4* src = reinterpret_cast<const uint4*>(D.lut2);
                uint4* dst = reinterpret_cast<uint4*>(L.lut2);
                for (u32 i = t; i < (1u << P2) / 16; i += 256) dst[i] = src[i];
            } else {
                for (u32 i = t; i < (1u << P2); i += 256) L.lut2[i] = D.lut2[i];
            }
        }
        if (t < kMaxSym) {
            L.rep[t] = __uint_as_float(t < K ? sym_rep : 0x80000000u);
            L.rep64[t] = t < K ? __hiloint2double((int)sym_rep_hi, (int)sym_rep) : -0.0;
            L.len[t] = sym_len; L.code[t] = sym_code;
        }
        __syncthreads();
        uint4* pay = dec_pay + wave * (pay_words / 4 + 1);
        const u32 zero_bits = zero_chunk_bits(L.len[K], L.code[K]);
        auto raise = [&](u32 code) { raise_status(ws, host, epoch, code); };
        while (c < nchunks) {
            // the next chunk's place in the offset table is on its way while this one is decoded
            const u32 cn = c + stride;
            u32 n0 = 0, n1 = 0;
            if (cn < nchunks) { n0 = off_tab[cn]; n1 = off_tab[cn + 1]; }
            const bool full = (u64)(c + 1) * kChunk <= n;
            if (full && aligned) {
                if (M > kDecLut1Bits) decode_chunk<true, true, DT, DEEP, VERIFY>(blob, w_ref, n, c, o0, o1, L, pay, pay_words, P1, P2, K, area, zero_bits, raise);
                else decode_chunk<true, false, DT, DEEP, VERIFY>(blob, w_ref, n, c, o0, o1, L, pay, pay_words, P1, P2, K, area, zero_bits, raise);
            } else {
                decode_chunk<false, true, DT, false, VERIFY>(blob, w_ref, n, c, o0, o1, L, pay, pay_words, P1, P2, K, area, full ? zero_bits : 0u, raise);
            }
            c = cn; o0 = n0; o1 = n1;
        }
    }
}

// ----------------------------------------------------------------------------- batched decode
// lc_decode_batch: the blobs of many tensors restored in five launches.  Every blob is validated as
// lc_decode validates it (header and symbol table per tensor, then every chunk's place in its offset
// table) before the sweep; a tensor whose blob fails is left untouched and reported, the others are
// restored.  The sweep deals the chunks of all tensors round-robin to single-wavefront workgroups,
// which reload their look-up tables when they move on to another tensor's chunk.
__global__ __launch_bounds__(256) void kb_dec_setup(BatchDecArgs a) {
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x, nthr = gridDim.x * blockDim.x;
    for (u32 g = i; g < a.total_chunks; g += nthr) {
        u32 lo = 0, hi = a.count - 1;
        while (lo < hi) {
            const u32 mid = (lo + hi + 1) >> 1;
            if (a.segs[mid].chunk0 <= g) lo = mid; else hi = mid - 1;
        }
        while (lo > 0 && (a.segs[lo].nchunks == 0 || g >= a.segs[lo].chunk0 + a.segs[lo].nchunks)) --lo;
        a.seg_of_chunk[g] = lo;
    }
    for (u32 t = i; t < a.count; t += nthr) a.seg_status[t] = 0;
}

// One workgroup per tensor: header, symbol table, codes, look-up tables.
__global__ __launch_bounds__(256) void kb_dec_tables(BatchDecArgs a) {
    __shared__ u32 hdr[kHeaderBytes / 4];
    __shared__ u32 s_ok;
    __shared__ u32 s_len[kMaxSym], s_code[kMaxSym];
    const u32 t = threadIdx.x, sidx = blockIdx.x;
    const SegD& sg = a.segs[sidx];
    DecSet& D = a.sets[sidx];
    if (t < kHeaderBytes / 4) hdr[t] = reinterpret_cast<const u32*>(sg.blob)[t];
    __syncthreads();
    if (t == 0) {
        const u64 hn = hdr[2] | ((u64)hdr[3] << 32), total = hdr[10] | ((u64)hdr[11] << 32);
        const u64 area = chunk_area_of(sg.nchunks);
        // the largest blob lc_encode can produce for this n (nbits 4): header + offsets + 132 bytes per chunk + n/2
        const u64 max_total = area + (u64)sg.nchunks * (2 * kW + 4) + (sg.n * 4 + 7) / 8;
        const bool sound = hdr[0] == 0x3142434Cu && hdr[1] == (1u | (kHeaderBytes << 16)) && hdr[12] == 0;
        const bool head_ok = sound && hn == sg.n && hdr[15] == (u32)a.dtype && hdr[9] == sg.nchunks && total >= area &&
                             total <= max_total && ((total - area) & 3) == 0;
        bool ok = head_ok;
        u32 status = 0;
        if (!head_ok) status = (sound && (hn != sg.n || hdr[15] != (u32)a.dtype)) ? 1u : 4u;
        else if (!dec_symbol_table(hdr, sg.n, sg.nchunks, area, (total - area) / 4, D, s_len, s_code)) { ok = false; status = 4u; }
        if (!ok) { atomicMax(&a.seg_status[sidx], status); D.info.area = 0; D.info.total_words = 0; D.info.max_len = 0; D.info.K = 0; }
        D.info.pad[0] = ok ? 1u : 0u;                        // the chunk checks and the sweep look here first
        D.info.pad[1] = 0;
        s_ok = ok;
    }
    __syncthreads();
    if (s_ok) dec_build_luts(D, s_len, s_code, t, 256);
}

// Also leaves, per chunk, what the sweep needs to find it: {tensor, chunk index there, the chunk's two offset-table
// entries}, so that the sweep's wavefronts get each chunk's place with one load that they can issue a chunk ahead.
__global__ __launch_bounds__(256) void kb_dec_chunks(BatchDecArgs a) {
    const u32 g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= a.total_chunks) return;
    const u32 sidx = a.seg_of_chunk[g];
    const SegD& sg = a.segs[sidx];
    const DecInfo& I = a.sets[sidx].info;
    const u32 c = g - sg.chunk0;
    uint4 info = make_uint4(sidx, c, 0u, 0u);
    if (I.pad[0]) {                                   // (a blob whose header failed: its tensor's status says so, the sweep skips it)
        const u32* off_tab = reinterpret_cast<const u32*>(sg.blob + kHeaderBytes);
        info.z = off_tab[c]; info.w = off_tab[c + 1];
        if (!dec_chunk_ok(sg.blob, I.area, I.total_words, sg.nchunks, c) && lane_id() == 0) atomicMax(&a.seg_status[sidx], 4u);
    }
    if (lane_id() == 0) reinterpret_cast<uint4*>(a.chunk_info)[g] = info;
}

template <int DT>
__global__ __launch_bounds__(64) void kb_decode(BatchDecArgs a) {
    __shared__ DecLds L;
    __shared__ uint4 pay[kPayWords / 4 + 1];
    const u32 lane = threadIdx.x;
    u32 active = 0xFFFFFFFFu, M = 0, K = 0, P1 = 0, P2 = 0;
    u64 area = 0;
    const uint4* chunk_info = reinterpret_cast<const uint4*>(a.chunk_info);
    auto info_of = [&](u32 g) {                      // (the same in every lane: back to scalar registers)
        uint4 q = g < a.total_chunks ? chunk_info[g] : make_uint4(0u, 0u, 0u, 0u);
        q.x = __builtin_amdgcn_readfirstlane(q.x); q.y = __builtin_amdgcn_readfirstlane(q.y);
        q.z = __builtin_amdgcn_readfirstlane(q.z); q.w = __builtin_amdgcn_readfirstlane(q.w);
        return q;
    };
    uint4 next = info_of(blockIdx.x);
    for (u32 g = blockIdx.x; g < a.total_chunks; g += gridDim.x) {
        const uint4 info = next;
        next = info_of(g + gridDim.x);               // on its way while this chunk is decoded
        const u32 sidx = info.x;
        // a tensor whose blob failed a check is not touched
        if (__hip_atomic_load(&a.seg_status[sidx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) continue;
        const SegD& sg = a.segs[sidx];
        if (sidx != active) {
            active = sidx;
            const DecSet& D = a.sets[sidx];
            M = D.info.max_len; K = D.info.K; area = D.info.area;
            P1 = M < kDecLut1Bits ? M : kDecLut1Bits; P2 = M < kDecLut2Bits ? M : kDecLut2Bits;
            __syncthreads();
            for (u32 i = lane; i < (1u << P1); i += kW) L.lut1[i] = D.lut1[i];
            if (M > kDecLut1Bits) {
                const u32* src = reinterpret_cast<const u32*>(D.lut2);
                u32* dst = reinterpret_cast<u32*>(L.lut2);
                for (u32 i = lane; i < ((1u << P2) + 3) / 4; i += kW) dst[i] = src[i];
            }
            if (lane < kMaxSym) {
                L.rep[lane] = __uint_as_float(lane < K ? D.info.rep_bits[lane] : 0x80000000u);
                L.len[lane] = D.info.len[lane]; L.code[lane] = D.info.code[lane];
            }
            __syncthreads();
        }
        auto raise = [&](u32 code) { atomicMax(&a.seg_status[sidx], code); };
        const u32 c = info.y, o0 = info.z, o1 = info.w;
        const bool full = (u64)(c + 1) * kChunk <= sg.n;
        const u32 zero_bits = full ? zero_chunk_bits(L.len[K], L.code[K]) : 0u;
        if (full && sg.aligned) {
            if (M > kDecLut1Bits) decode_chunk<true, true, DT>(sg.blob, sg.w_ref, sg.n, c, o0, o1, L, pay, kPayWords, P1, P2, K, area, zero_bits, raise);
            else decode_chunk<true, false, DT>(sg.blob, sg.w_ref, sg.n, c, o0, o1, L, pay, kPayWords, P1, P2, K, area, zero_bits, raise);
        } else {
            decode_chunk<false, true, DT>(sg.blob, sg.w_ref, sg.n, c, o0, o1, L, pay, kPayWords, P1, P2, K, area, zero_bits, raise);
        }
    }
}

__global__ __launch_bounds__(256) void kb_dec_report(BatchDecArgs a) {
    const u32 t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= a.count) return;
    const u32 st = a.seg_status[t];
    const DecInfo& I = a.sets[t].info;
    a.results[t].status = st;
    a.results[t].bytes = st ? 0 : I.area + 4 * I.total_words;
    a.results[t].used_cache = 0;
}

// ----------------------------------------------------------------------------- k_decode_fused
// Restore from several checkpoints in one sweep (Section 3, C1: u_t = u_0 + sum of the decoded
// deltas; Section 3.2, checkpoint merging): up to kMaxMany blobs of the same n are decoded side
// by side and their values added to w_ref in blob order, one fp32 add per blob and element, so
// the result equals that of applying the blobs one call after the other, with one read and
// one write of w_ref instead of one per blob.
// T is a compile-time constant, so the T bit strings of a
// lane are T independent dependency chains that the scheduler interleaves.  One wavefront per
// workgroup; the payloads of a chunk (all T blobs) are staged in the workgroup's LDS area with
// coalesced loads (the host sizes the area to the blobs, which also sets how many wavefronts
// share a compute unit).  With codes of at most 7 bits (always the case for nbits <= 3) a row's 4 codes
// of one blob take at most 28 bits, so each blob's 32-bit window is re-read once per row from the bit
// position alone, without a branch; with longer codes (LONG) twice per row.  Both look-up
// tables are free of LDS bank conflicts: 128 one-byte entries over the next 7 bits (code length
// and symbol), then the symbol's representative.  A chunk whose payloads do not fit the LDS
// area reads them from memory instead.
template <int T>
struct FusedHead {
    uint16_t lut[T][1u << kDecLut1Bits];         // next 7 bits -> e = (len << 4 | symbol) << 2
    u32 rep[T][128];                             // byte offset e -> representative bits (-0.0: merged symbol); a symbol
                                                 // has one length, so distinct entries in use lie in distinct banks
    const uint8_t* rec_base[T];                  // start of the chunk records
    const u32* off_tab[T];
    // Codes longer than the 7 bits of lut (its entry is then kFusedEscape): the symbols in canonical order
    // (shorter codes first, then by index) have increasing left-justified codes, so the rank of the symbol a
    // window starts with is the number of codes not above the window; only the long ones need comparing.
    u32 lj[T][kMaxSym];                          // rank -> code, left-justified in 32 bits
    uint16_t e_rank[T][kMaxSym];                 // rank -> (len << 4 | symbol) << 2
    u32 rep_sym[T][kMaxSym];                     // symbol -> representative bits
    u32 first_long[(T + 3) / 4 * 4];             // rank of the first code longer than 7 bits
    u32 nranks[(T + 3) / 4 * 4];                 // symbols with a code
    u32 zero_bits[(T + 3) / 4 * 4];              // per blob: lane length of a chunk of merged symbols only (0: never skip)
    u32 pad[3];
    u32 before_pay;                              // the word in front of the payload area (read, never used)
};
constexpr u32 kFusedEscape = 0xFFu << 2;         // what lut holds for a prefix of a longer code (no short entry has length 15)
constexpr u32 kFusedSlack = 128;                 // words behind the payloads that a damaged lane string may run into:
                                                 // 256 codes of at most 15 bits past a start that validation bounds

// Bit positions are kept as p = 31 + bits from the start of the payload area (staged) or of the
// blob's payload (from memory): the window is then the low 32 bits of {word[(p >> 5) - 1],
// word[p >> 5]} >> (~p & 31), which is one v_alignbit.
// LONG: some blob of the sweep has codes longer than 7 bits.  Two codes then take up to 30 bits, so the window is
// re-read after the second code of a row, and a window that starts with a long code is ranked against the long
// codes (a handful of compares; rare, since long codes belong to rare symbols).
template <int T, bool FAST, bool STAGED, bool LONG, int DT>
__device__ __forceinline__ void fused_row(const FusedHead<T>& H, const u32* pay, u32 pay_words, const u32* const (&gw)[T],
                                          const u32 (&nw)[T], u32 (&pos)[T], void* __restrict__ w_ref, u64 n, u64 idx,
                                          float (&x)[4]) {
    // Written step by step across the blobs (all windows, then the first code of every blob, ...), so
    // that the T look-ups of a step are in flight together.
    u32 win[T], rep[4][T];
    auto windows = [&]() {
#pragma unroll
        for (int t = 0; t < T; ++t) {
            u32 hi, lo;                                   // the two payload words around the lane's position
            if (STAGED) {
                const u32 wi = pos[t] >> 5;              // stays inside the area and its slack
                hi = pay[(int)wi - 1]; lo = pay[wi];
            } else {
                const u32 wi = pos[t] >> 5, last = nw[t] - 1;
                hi = wi ? gw[t][min(wi - 1, last)] : 0u; lo = gw[t][min(wi, last)];
            }
            win[t] = __builtin_amdgcn_alignbit(hi, lo, ~pos[t]);
        }
    };
    windows();
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (LONG && v == 2) windows();
        if (FAST || idx + v < n) {
            u32 e[T];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                e[t] = H.lut[t][win[t] >> (32 - kDecLut1Bits)];
                asm("" : "+v"(e[t]));                 // keep e a 32-bit value (no 16-bit shift plus re-extension)
            }
            if (LONG) {
#pragma unroll
                for (int t = 0; t < T; ++t) {
                    if (__any(e[t] == kFusedEscape)) {
                        const u32 first = H.first_long[t], nr = H.nranks[t];
                        u32 r = first;
                        for (u32 j = first + 1; j < nr; ++j) r += win[t] >= H.lj[t][j] ? 1u : 0u;
                        if (e[t] == kFusedEscape) e[t] = H.e_rank[t][r];
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const u32 len = e[t] >> 6;
                if (LONG) rep[v][t] = H.rep_sym[t][(e[t] >> 2) & 15u];
                else rep[v][t] = *reinterpret_cast<const u32*>(reinterpret_cast<const uint8_t*>(H.rep[t]) + e[t]);
                win[t] <<= len; pos[t] += len;
            }
        } else {
#pragma unroll
            for (int t = 0; t < T; ++t) rep[v][t] = 0x80000000u;
        }
    }
    u32 kept = 1;                                     // a single blob often leaves whole rows unchanged: skip their write
    if (T == 1) kept = (rep[0][0] | rep[1][0] | rep[2][0] | rep[3][0]) & 0x7FFFFFFFu;
    if (FAST) {
        if (T > 1 || __any(kept != 0)) {
#pragma unroll
            for (int v = 0; v < 4; ++v)
#pragma unroll
                for (int t = 0; t < T; ++t) x[v] = stored<DT>(__fadd_rn(x[v], __uint_as_float(rep[v][t])));   // in blob order
            // (binary32 rows as a plain float4 store: with non-temporal stores, or with the same 16 bytes stored through
            // a compiler vector type, the first sweep over parameters that a device copy had just written took 830-880 us
            // instead of 600-650)
            if constexpr (DT == kF32) *reinterpret_cast<float4*>(static_cast<float*>(w_ref) + idx) = make_float4(x[0], x[1], x[2], x[3]);
            else store4<DT, false>(w_ref, idx, x);
        }
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (idx + v < n) {
#pragma unroll
                for (int t = 0; t < T; ++t) x[v] = stored<DT>(__fadd_rn(x[v], __uint_as_float(rep[v][t])));
                store_one<DT>(w_ref, idx + v, x[v]);
            }
        }
    }
}

// All rows of a full, aligned chunk with staged payloads: w_ref is read PF rows ahead in two
// alternating register batches, so the reads of the next rows are in flight while these decode.
template <int T, bool LONG, int DT>
__device__ __forceinline__ void fused_rows_fast(const FusedHead<T>& H, const u32* pay, u32 pay_words, const u32* const (&gw)[T],
                                                const u32 (&nw)[T], u32 (&pos)[T], void* __restrict__ w_ref, u64 n, u32 c) {
    constexpr int PF = 4;
    typedef typename Raw<DT>::type RowT;
    const u32 lane = lane_id();
    const u64 base = (u64)c * kChunk + lane * kV;
    RowT A[PF], B[PF];
#pragma unroll
    for (int k = 0; k < PF; ++k) A[k] = load_raw<DT>(w_ref, base + (u64)k * kRowElems);
    auto batch = [&](RowT (&X)[PF], u32 r0) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            float x[4];
            unpack<DT>(X[k], x);
            fused_row<T, true, true, LONG, DT>(H, pay, pay_words, gw, nw, pos, w_ref, n, base + (u64)(r0 + k) * kRowElems, x);
        }
    };
    for (u32 r0 = 0; r0 < kR; r0 += 2 * PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) B[k] = load_raw<DT>(w_ref, base + (u64)(r0 + PF + k) * kRowElems);
        batch(A, r0);
        if (r0 + 2 * PF < kR) {
#pragma unroll
            for (int k = 0; k < PF; ++k) A[k] = load_raw<DT>(w_ref, base + (u64)(r0 + 2 * PF + k) * kRowElems);
        }
        batch(B, r0 + PF);
    }
}

// Any chunk (ragged, unaligned, or payloads read from memory), row by row.
template <int T, bool FAST, bool LONG, int DT>
__device__ __forceinline__ void fused_rows_plain(const FusedHead<T>& H, const u32* const (&gw)[T], const u32 (&nw)[T], u32 (&pos)[T],
                                              void* __restrict__ w_ref, u64 n, u32 c) {
    const u32 lane = lane_id();
    const u64 base = (u64)c * kChunk;
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        if (!FAST && idx >= n) break;
        float x[4];
        load_row<FAST, DT>(w_ref, idx, n, x);
        fused_row<T, FAST, false, LONG, DT>(H, nullptr, 0, gw, nw, pos, w_ref, n, idx, x);
    }
}

template <typename P>
__device__ __forceinline__ P* uniform_ptr(P* p) {        // a pointer every lane holds alike, moved to scalar registers
    const u64 v = reinterpret_cast<u64>(p);
    const u32 lo = __builtin_amdgcn_readfirstlane((u32)v), hi = __builtin_amdgcn_readfirstlane((u32)(v >> 32));
    return reinterpret_cast<P*>(((u64)hi << 32) | lo);
}

template <int T, bool FAST, bool LONG, int DT>
__device__ __forceinline__ void fused_chunk(const FusedHead<T>& H, u32* pay, u32 pay_words, void* __restrict__ w_ref, u64 n,
                                            Workspace* ws, HostResult* host, u32 c, u32 nchunks, u64 epoch) {
    const u32 lane = lane_id();
    const u32* gw[T];
    u32 nw[T], k0[T], wbase[T], pos[T], start[T], lane_bits[T];
    u32 total = 0;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const u32* ot = uniform_ptr(H.off_tab[t]);
        const u32 o0 = ot[c], o1 = ot[c + 1];
        const uint8_t* rec = uniform_ptr(H.rec_base[t]) + 4 * (u64)o0;
        nw[t] = o1 - o0 - kLaneBitsWords;                 // >= 1 (validated)
        lane_bits[t] = reinterpret_cast<const uint16_t*>(rec)[lane];
        gw[t] = reinterpret_cast<const u32*>(rec + 2 * kW);
        k0[t] = (u32)((reinterpret_cast<uintptr_t>(gw[t]) >> 2) & 3);
        wbase[t] = total;
        total += (nw[t] + k0[t] + 3) & ~3u;
    }
    const bool staged = FAST && total <= pay_words;
    if (staged) {
        // Coalesced copies of [16-byte aligned start, payload end) into the LDS area; the words before a
        // payload are its record's lane lengths.  A last partial vector may read up to 12 bytes past the
        // payload: into the next record, except in the last chunk, which reads that vector word by word.
        constexpr int CV = T > 4 ? 2 : 4;                 // vectors per lane and blob in flight
        const bool guard = c + 1 == nchunks;
        u32 most = 0;
#pragma unroll
        for (int t = 0; t < T; ++t) most = max(most, (nw[t] + k0[t] + 3) >> 2);
        u32 nonzero = 0;                                  // OR of this lane's share of the payload words
        for (u32 i0 = 0; i0 < most; i0 += CV * kW) {
            uint4 q[T][CV];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const uint4* gv = reinterpret_cast<const uint4*>(gw[t] - k0[t]);
                const u32 have = nw[t] + k0[t], nvec = (have + 3) >> 2;
#pragma unroll
                for (int k = 0; k < CV; ++k) {
                    const u32 i = i0 + k * kW + lane;
                    if (i < nvec) {
                        if (!guard || 4 * i + 4 <= have) q[t][k] = gv[i];
                        else {
                            const u32* tw = reinterpret_cast<const u32*>(gv + i);
                            const u32 left = have - 4 * i;
                            q[t][k].x = tw[0]; q[t][k].y = left > 1 ? tw[1] : 0; q[t][k].z = left > 2 ? tw[2] : 0; q[t][k].w = 0;
                        }
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                uint4* dst = reinterpret_cast<uint4*>(pay + wbase[t]);
                const u32 have = nw[t] + k0[t], nvec = (have + 3) >> 2;
#pragma unroll
                for (int k = 0; k < CV; ++k) {
                    const u32 i = i0 + k * kW + lane;
                    if (i < nvec) {
                        dst[i] = q[t][k];
                        const u32 j = 4 * i;              // words [k0, have) of the copied range are payload
                        nonzero |= (j >= k0[t] && j < have ? q[t][k].x : 0u) | (j + 1 >= k0[t] && j + 1 < have ? q[t][k].y : 0u) |
                                   (j + 2 >= k0[t] && j + 2 < have ? q[t][k].z : 0u) | (j + 3 >= k0[t] && j + 3 < have ? q[t][k].w : 0u);
                    }
                }
            }
        }
        // every blob's chunk holds merged symbols only (see zero_chunk_bits): nothing changes, w_ref is not read
        bool all_merged = true;
#pragma unroll
        for (int t = 0; t < T; ++t) all_merged = all_merged && H.zero_bits[t] != 0 && lane_bits[t] == H.zero_bits[t];
        if (!__any(!all_merged || nonzero != 0)) return;
    }
#pragma unroll
    for (int t = 0; t < T; ++t) start[t] = 31 + wave_incl_scan(lane_bits[t]) - lane_bits[t];
    if (staged) {
#pragma unroll
        for (int t = 0; t < T; ++t) { start[t] += 32 * (wbase[t] + k0[t]); pos[t] = start[t]; }
        fused_rows_fast<T, LONG, DT>(H, pay, pay_words, gw, nw, pos, w_ref, n, c);
    } else {
#pragma unroll
        for (int t = 0; t < T; ++t) pos[t] = start[t];
        fused_rows_plain<T, FAST, LONG, DT>(H, gw, nw, pos, w_ref, n, c);
    }
    bool bad = false;
#pragma unroll
    for (int t = 0; t < T; ++t) bad = bad || (pos[t] - start[t] != lane_bits[t]);
    if (__any(bad) && lane == 0) raise_status(ws, host, epoch, 4u);
}

template <int T, bool LONG, int DT>
__global__ __launch_bounds__(64) void k_decode_fused(BlobList blobs, u32 first, void* __restrict__ w_ref, u64 n,
                                                     Workspace* ws, u32 nchunks, int aligned, u64 epoch,
                                                     HostResult* host, u32 pay_words) {
    __shared__ FusedHead<T> H;
    static_assert(sizeof(FusedHead<T>) % 16 == 0, "payload area must stay 16-byte aligned");
    extern __shared__ uint4 fused_pay[];                 // pay_words + kFusedSlack payload words, right behind H
    u32* pay = reinterpret_cast<u32*>(fused_pay);
    // if a check found something, touch nothing
    if ((__hip_atomic_load(&ws->dec_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 8) == epoch) return;
    const u32 tid = threadIdx.x;
#pragma unroll
    for (int t = 0; t < T; ++t) {
        const DecSet& D = ws->dec_set[first + t];
        const u32 M = D.info.max_len, K = D.info.K;       // entries of codes of at most 7 bits: e < 512
        const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits;
        for (u32 i = tid; i < (1u << kDecLut1Bits); i += kW) {
            const u32 e = D.lut1[i >> (kDecLut1Bits - P1)];
            H.lut[t][i] = (uint16_t)(e << 2);
            H.rep[t][i] = (i & 15) < K ? D.info.rep_bits[i & 15] : 0x80000000u;
        }
        if (LONG && tid < kMaxSym) {
            // this symbol's rank in canonical order (shorter codes first, then by index)
            const u32 j = tid, own = D.info.len[j];
            u32 rank = 0, coded = 0, short_codes = 0;
            for (u32 i = 0; i < kMaxSym; ++i) {
                const u32 li = D.info.len[i];
                if (li == 0) continue;
                ++coded;
                if (li <= kDecLut1Bits) ++short_codes;
                if (own && (li < own || (li == own && i < j))) ++rank;
            }
            H.rep_sym[t][j] = j < K ? D.info.rep_bits[j] : 0x80000000u;
            if (own) { H.lj[t][rank] = D.info.code[j] << (32 - own); H.e_rank[t][rank] = (uint16_t)(((own << 4) | j) << 2); }
            if (tid == 0) { H.first_long[t] = short_codes; H.nranks[t] = coded; }
        }
        if (tid == 0) {
            const uint8_t* blob = blobs.p[first + t];
            H.zero_bits[t] = zero_chunk_bits(D.info.len[K], D.info.code[K]);
            H.rec_base[t] = blob + D.info.area;
            H.off_tab[t] = reinterpret_cast<const u32*>(blob + kHeaderBytes);
        }
    }
    if (tid == 0) H.before_pay = 0;
    __syncthreads();
    for (u32 c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const bool full = (u64)(c + 1) * kChunk <= n;
        if (full && aligned) fused_chunk<T, true, LONG, DT>(H, pay, pay_words, w_ref, n, ws, host, c, nchunks, epoch);
        else fused_chunk<T, false, LONG, DT>(H, pay, pay_words, w_ref, n, ws, host, c, nchunks, epoch);
    }
}
// ----------------------------------------------------------------------------- launchers
void launch_batch_decode(const BatchDecArgs& a, const Tuning& tune, hipStream_t s) {
    const u32 cap = (u32)tune.num_cu * 8;
    u32 setup_blocks = (a.total_chunks + 255) / 256;
    if (setup_blocks > cap) setup_blocks = cap;
    if (setup_blocks < 1) setup_blocks = 1;
    hipLaunchKernelGGL(kb_dec_setup, dim3(setup_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(kb_dec_tables, dim3(a.count), dim3(256), 0, s, a);
    if (a.total_chunks) {
        hipLaunchKernelGGL(kb_dec_chunks, dim3((a.total_chunks + 3) / 4), dim3(256), 0, s, a);
        // single-wavefront workgroups, three times as many as the compute units hold at once (12 each, by their LDS)
        // as long as there are chunks for them: workgroups that draw cheap chunks (nothing but merged symbols) make
        // room for the next, which evens out the load better than a fixed deal of chunks to resident wavefronts
        // (VGG-16's 32 tensors: 60 us against 80)
        u32 waves = (u32)tune.num_cu * (u32)tune.decode_blocks_per_cu * 4u;
        if (waves > a.total_chunks) waves = a.total_chunks;
        if (a.dtype == kBF16) hipLaunchKernelGGL(kb_decode<kBF16>, dim3(waves), dim3(64), 0, s, a);
        else if (a.dtype == kF16) hipLaunchKernelGGL(kb_decode<kF16>, dim3(waves), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(kb_decode<kF32>, dim3(waves), dim3(64), 0, s, a);
    }
    hipLaunchKernelGGL(kb_dec_report, dim3((a.count + 255) / 256), dim3(256), 0, s, a);
}

void launch_dec_check(const BlobList& blobs, int first, int count, uint64_t n, int dtype, uint64_t max_total, Workspace* ws,
                      uint64_t epoch, HostResult* host, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    // one chunk per wavefront while that is at most a few rounds of workgroups on the chip, else four
    const bool four = (u64)count * ((nchunks + 3) / 4) > 8192;
    const u64 per_block = four ? 16 : 4;
    const u64 blocks = nchunks ? (nchunks + per_block - 1) / per_block : 1;
    if (four) hipLaunchKernelGGL(k_dec_check<4>, dim3((u32)blocks, (u32)count), dim3(256), 0, s, blobs, (u32)first, (u64)n, (u64)max_total,
                                 ws, (u32)nchunks, (u64)epoch, host, (u32)dtype);
    else hipLaunchKernelGGL(k_dec_check<1>, dim3((u32)blocks, (u32)count), dim3(256), 0, s, blobs, (u32)first, (u64)n, (u64)max_total,
                            ws, (u32)nchunks, (u64)epoch, host, (u32)dtype);
}



template <int T, int DT>
static void launch_fused_td(const BlobList& blobs, int first, void* w_ref, uint64_t n, Workspace* ws, uint64_t epoch,
                            HostResult* host, u32 blocks, u32 pay_words, bool long_codes, hipStream_t s) {
    const size_t lds = 4 * (size_t)(pay_words + kFusedSlack);
    const int al = aligned_rows(w_ref, DT);
    if (long_codes) hipLaunchKernelGGL((k_decode_fused<T, true, DT>), dim3(blocks), dim3(64), lds, s, blobs, (u32)first, w_ref,
                                       (u64)n, ws, (u32)num_chunks_of(n), al, (u64)epoch, host, pay_words);
    else hipLaunchKernelGGL((k_decode_fused<T, false, DT>), dim3(blocks), dim3(64), lds, s, blobs, (u32)first, w_ref,
                            (u64)n, ws, (u32)num_chunks_of(n), al, (u64)epoch, host, pay_words);
}

template <int T>
static void launch_fused_t(const BlobList& blobs, int first, void* w_ref, uint64_t n, int dtype, Workspace* ws, uint64_t epoch,
                           HostResult* host, u32 blocks, u32 pay_words, bool long_codes, hipStream_t s) {
    if (dtype == kBF16) launch_fused_td<T, kBF16>(blobs, first, w_ref, n, ws, epoch, host, blocks, pay_words, long_codes, s);
    else if (dtype == kF16) launch_fused_td<T, kF16>(blobs, first, w_ref, n, ws, epoch, host, blocks, pay_words, long_codes, s);
    else launch_fused_td<T, kF32>(blobs, first, w_ref, n, ws, epoch, host, blocks, pay_words, long_codes, s);
}

size_t fused_lds_bytes(int count, uint32_t pay_words) {
    static const size_t head[kMaxMany] = {sizeof(FusedHead<1>), sizeof(FusedHead<2>), sizeof(FusedHead<3>), sizeof(FusedHead<4>),
                                          sizeof(FusedHead<5>), sizeof(FusedHead<6>), sizeof(FusedHead<7>), sizeof(FusedHead<8>)};
    return head[count - 1] + 4 * (size_t)(pay_words + kFusedSlack);
}

void launch_decode_fused(const BlobList& blobs, int first, int count, void* w_ref, uint64_t n, int dtype, Workspace* ws,
                         uint64_t epoch, HostResult* host, uint32_t pay_words, bool long_codes, const Tuning& tune,
                         hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    // one wavefront per workgroup; as many workgroups per compute unit as their LDS areas allow
    u64 per_cu = kLdsPerCu / fused_lds_bytes(count, pay_words);
    if (per_cu > (u64)tune.fused_waves_per_cu) per_cu = tune.fused_waves_per_cu;
    if (per_cu < 1) per_cu = 1;
    u64 blocks = (u64)tune.num_cu * per_cu;
    if (blocks > nchunks) blocks = nchunks;
    const u32 b = (u32)blocks;
    switch (count) {
        case 1: launch_fused_t<1>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 2: launch_fused_t<2>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 3: launch_fused_t<3>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 4: launch_fused_t<4>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 5: launch_fused_t<5>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 6: launch_fused_t<6>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        case 7: launch_fused_t<7>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
        default: launch_fused_t<8>(blobs, first, w_ref, n, dtype, ws, epoch, host, b, pay_words, long_codes, s); break;
    }
}

// w_ref null: the verifying sweep (nothing but the blob is read)
void launch_decode(const uint8_t* blob, void* w_ref, uint64_t n, int dtype, Workspace* ws, int set, uint64_t epoch, HostResult* host,
                   const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    const bool verify = w_ref == nullptr;
    const u64 blocks = balanced_workers((nchunks + 3) / 4, (u64)tune.num_cu * tune.decode_blocks_per_cu);
    const dim3 grid((u32)blocks), wg(256);
    const int al = verify ? 1 : aligned_rows(w_ref, dtype);
    // LDS payload areas: the usual size when every compute unit gets as many workgroups as fit beside each other
    // (4); with fewer workgroups than that, what the unit's LDS leaves each, so that chunks with long payloads
    // (codes of 5 and more bits on average) need not read their lane strings from memory
    const u64 per_cu = (blocks + tune.num_cu - 1) / tune.num_cu;
    u32 pay_words = kPayWords;
    if (per_cu < 4) {
        static_assert(sizeof(DecLds) + 4 * (kPayWordsMax / 4 + 1) * sizeof(uint4) <= 64 * 1024, "one workgroup's LDS");
        const size_t room = kLdsPerCu / (size_t)per_cu - sizeof(DecLds) - 1024;
        const u64 fit = room / 16 / 4 * 4 - 4;                      // words per wavefront, a multiple of 4
        pay_words = (u32)(fit > kPayWordsMax ? kPayWordsMax : fit);
        if (pay_words < kPayWords) pay_words = kPayWords;
    }
    const size_t lds = 4 * (size_t)(pay_words / 4 + 1) * sizeof(uint4);
    // At most two workgroups per compute unit: a wavefront has its SIMD almost to itself and nothing hides its waits
    // on memory, so the kernel's form with rows fetched far ahead runs (it needs more registers than would let more
    // workgroups share a unit).
    const bool deep = per_cu <= 2;
    if (verify) {
        hipLaunchKernelGGL((k_decode<kF32, false, true>), grid, wg, lds, s, blob, (void*)nullptr, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host, pay_words, (u32)set);
        return;
    }
#define LC_DECODE(DT) \
    if (deep) hipLaunchKernelGGL((k_decode<DT, true>), grid, wg, lds, s, blob, w_ref, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host, pay_words, (u32)set); \
    else hipLaunchKernelGGL((k_decode<DT, false>), grid, wg, lds, s, blob, w_ref, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host, pay_words, (u32)set)
    if (dtype == kF64) { LC_DECODE(kF64); }
    else if (dtype == kBF16) { LC_DECODE(kBF16); }
    else if (dtype == kF16) { LC_DECODE(kF16); }
    else { LC_DECODE(kF32); }
#undef LC_DECODE
}

}  // namespace lc
