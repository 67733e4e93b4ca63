// HIP kernels of the LC-Checkpoint compress / restore path for gfx950 (wave64).
//
// encode:  k_reset -> k_hist -> k_table -> k_pack -> k_finalize
// decode:  k_dec_prepare -> k_dec_validate -> (host checks status) -> k_decode
//
// The paper (arXiv 2009.13003) defines what is computed: delta against the last
// recovered state (Algorithm 1 line 4), (sign, exponent) buckets represented by the
// mean of their extremes and x-bit priority promotion (Section 3.1.1), Huffman
// coding of the bucket indices (Section 3.1.2), restore by accumulation
// (Algorithm 1 line 7).  How it is laid out on the GPU is this library's own.
#include "lc_internal.h"

namespace lc {

typedef unsigned long long u64;
typedef uint32_t u32;

// ----------------------------------------------------------------------------- small helpers
__device__ __forceinline__ u32 lane_id() { return __lane_id(); }

__device__ __forceinline__ u32 wave_incl_scan(u32 v) {
    const u32 lane = lane_id();
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        u32 t = __shfl_up(v, d, 64);
        if (lane >= (u32)d) v += t;
    }
    return v;
}

__device__ __forceinline__ u64 wave_sum64(u64 v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

__device__ __forceinline__ u32 wave_sum32(u32 v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// delta of Algorithm 1 line 4: one IEEE binary32 subtraction (never fused or reassociated).
__device__ __forceinline__ u32 delta_bits(float w, float w_ref) { return __float_as_uint(__fsub_rn(w, w_ref)); }

template <bool FAST>
__device__ __forceinline__ void load_row(const float* __restrict__ p, u64 idx, u64 n, float (&x)[4]) {
    if (FAST) {
        const float4 t = *reinterpret_cast<const float4*>(p + idx);
        x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w;
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = (idx + v < n) ? p[idx + v] : 0.0f;
    }
}

// ----------------------------------------------------------------------------- k_reset
__global__ void k_reset(Workspace* ws, u64* state, u64 nchunks) {
    const u64 tid = (u64)blockIdx.x * blockDim.x + threadIdx.x;
    if (blockIdx.x == 0) {
        for (u32 i = threadIdx.x; i < 512; i += blockDim.x) ws->hist[i] = 0;
        if (threadIdx.x < kMaxSym) { ws->mmin[threadIdx.x] = 0x7FFFFFu; ws->mmax[threadIdx.x] = 0; }
        if (threadIdx.x == 0) { ws->ticket = 0; ws->total_words = 0; ws->table.status = 0; }
    }
    for (u64 i = tid; i < nchunks; i += (u64)gridDim.x * blockDim.x) state[i] = 0;
}

// ----------------------------------------------------------------------------- k_hist
// Sweep 1 (Section 3.1.1, exponent-based quantization): population of each of the 2^9
// (sign, exponent) buckets.  LDS histogram replicated 8 times (copy = lane & 7, copies
// of one bin in different banks) so that lanes hitting the same popular bucket rarely
// collide; merged into 64-bit global counters once per workgroup.
constexpr int kHistCopies = 8;

template <bool ALIGNED>
__global__ __launch_bounds__(256) void k_hist(const float* __restrict__ w, const float* __restrict__ w_ref,
                                              u64 n, Workspace* ws) {
    __shared__ u32 h[512 * kHistCopies];
    const u32 tid = threadIdx.x;
    for (u32 i = tid; i < 512 * kHistCopies; i += 256) h[i] = 0;
    __syncthreads();
    const u32 copy = tid & (kHistCopies - 1);
    const u64 n4 = n / 4;
    const u64 stride = (u64)gridDim.x * 256;
    u64 u = (u64)blockIdx.x * 256 + tid;
    for (; u + 3 * stride < n4; u += 4 * stride) {
        float a[4][4], b[4][4];
#pragma unroll
        for (int k = 0; k < 4; ++k) { load_row<ALIGNED>(w, 4 * (u + k * stride), n, a[k]); load_row<ALIGNED>(w_ref, 4 * (u + k * stride), n, b[k]); }
#pragma unroll
        for (int k = 0; k < 4; ++k)
#pragma unroll
            for (int v = 0; v < 4; ++v) atomicAdd(&h[(delta_bits(a[k][v], b[k][v]) >> 23) * kHistCopies + copy], 1u);
    }
    for (; u < n4; u += stride) {
        float a[4], b[4];
        load_row<ALIGNED>(w, 4 * u, n, a); load_row<ALIGNED>(w_ref, 4 * u, n, b);
#pragma unroll
        for (int v = 0; v < 4; ++v) atomicAdd(&h[(delta_bits(a[v], b[v]) >> 23) * kHistCopies + copy], 1u);
    }
    if (blockIdx.x == 0 && tid < (u32)(n - 4 * n4)) {
        const u64 i = 4 * n4 + tid;
        atomicAdd(&h[(delta_bits(w[i], w_ref[i]) >> 23) * kHistCopies + copy], 1u);
    }
    __syncthreads();
    for (u32 b = tid; b < 512; b += 256) {
        u32 s = 0;
#pragma unroll
        for (int k = 0; k < kHistCopies; ++k) s += h[b * kHistCopies + k];
        if (s) atomicAdd(&ws->hist[b], (u64)s);
    }
}

// ----------------------------------------------------------------------------- k_table
// Priority promotion (Section 3.1.1) and the Huffman table (Section 3.1.2), one
// workgroup of 512 threads, thread t looking at the bucket of priority rank t
// (exponent descending, + before -).
__global__ __launch_bounds__(512) void k_table(Workspace* ws, u64 n, int nbits) {
    __shared__ u32 wave_tot[8];
    __shared__ u32 flag_nonfinite, flag_zero;
    __shared__ uint8_t s_sym[512];
    __shared__ u64 s_cnt[kMaxSym];
    __shared__ u32 s_kept[kMaxSym], s_len[kMaxSym + 1], s_code[kMaxSym];
    // Huffman scratch (thread 0 only)
    __shared__ u32 leaf[kMaxSym], left[kMaxSym], right[kMaxSym], depth[kMaxSym];
    __shared__ u64 node_w[kMaxSym];

    const u32 t = threadIdx.x, lane = t & 63, wv = t >> 6;
    const u32 E = 255 - (t >> 1), sgn = t & 1, b = (sgn << 8) | E;
    const u64 c = ws->hist[b];
    const bool cand = c > 0 && E >= 1 && E <= 254;
    const u64 m = __ballot(cand);
    const u32 within = __popcll(m & ((1ull << lane) - 1));
    if (lane == 0) wave_tot[wv] = __popcll(m);
    if (t == 0) { flag_nonfinite = 0; flag_zero = 0; }
    if (t < kMaxSym) { s_cnt[t] = 0; s_kept[t] = 0; s_len[t] = 0; s_code[t] = 0; }
    __syncthreads();
    if (E == 255 && c > 0) flag_nonfinite = 1;
    if (E == 0 && c > 0) flag_zero = 1;
    u32 before = 0, total = 0;
    for (u32 i = 0; i < 8; ++i) { if (i < wv) before += wave_tot[i]; total += wave_tot[i]; }
    const u32 rank = before + within;
    const u32 kmax = (1u << nbits) - 1;
    const u32 K = total < kmax ? total : kmax;
    const bool is_kept = cand && rank < K;
    if (is_kept) { s_kept[rank] = b; s_cnt[rank] = c; }
    s_sym[b] = (uint8_t)(is_kept ? rank : K);
    __syncthreads();

    if (t == 0) {
        Table& T = ws->table;
        u64 kept_total = 0;
        for (u32 j = 0; j < K; ++j) kept_total += s_cnt[j];
        s_cnt[K] = n - kept_total;
        const u32 msym = K + 1;
        // leaves in ascending (count, symbol) order
        u32 nl = 0;
        for (u32 s = 0; s < msym; ++s) {
            if (s_cnt[s] == 0) continue;
            u32 p = nl++;
            while (p > 0 && s_cnt[leaf[p - 1]] > s_cnt[s]) { leaf[p] = leaf[p - 1]; --p; }
            leaf[p] = s;
        }
        u32 max_len = 0;
        if (nl == 1) { s_len[leaf[0]] = 1; max_len = 1; }
        else if (nl >= 2) {
            // two queues: sorted leaves and joined nodes in creation order (their weights never
            // decrease); on equal weight the leaf is taken first.  Ids >= 16 are joined nodes.
            u32 li = 0, qi = 0, ni = 0;
            for (u32 k = 0; k + 1 < nl; ++k) {
                u32 pick[2]; u64 wsum = 0;
                for (int q = 0; q < 2; ++q) {
                    const bool take_leaf = li < nl && (qi >= ni || s_cnt[leaf[li]] <= node_w[qi]);
                    if (take_leaf) { pick[q] = leaf[li]; wsum += s_cnt[leaf[li]]; ++li; }
                    else { pick[q] = 16 + qi; wsum += node_w[qi]; ++qi; }
                }
                node_w[ni] = wsum; left[ni] = pick[0]; right[ni] = pick[1]; ++ni;
            }
            depth[ni - 1] = 0;
            for (int i = (int)ni - 1; i >= 0; --i) {
                const u32 d = depth[i] + 1, ch[2] = {left[i], right[i]};
                for (int q = 0; q < 2; ++q) {
                    if (ch[q] >= 16) depth[ch[q] - 16] = d;
                    else { s_len[ch[q]] = d; if (d > max_len) max_len = d; }
                }
            }
        }
        // canonical codes by counting codes per length
        u32 per_len[17], next_code[17];
        for (int L = 0; L <= 16; ++L) per_len[L] = 0;
        for (u32 s = 0; s < msym; ++s) per_len[s_len[s]]++;
        per_len[0] = 0;
        u32 code = 0;
        for (int L = 1; L <= 16; ++L) { code = (code + per_len[L - 1]) << 1; next_code[L] = code; }
        for (u32 s = 0; s < msym; ++s) if (s_len[s]) s_code[s] = next_code[s_len[s]]++;
        for (u32 s = 0; s < kMaxSym; ++s) {
            T.codelen[s] = s < msym ? ((s_code[s] << 5) | s_len[s]) : 0;
            T.kept[s] = s < K ? s_kept[s] : 0;
            T.cnt[s] = s < msym ? s_cnt[s] : 0;
        }
        T.K = K; T.max_len = max_len; T.k_E = total + flag_zero;
        T.status = flag_nonfinite ? 2u : 0u;
    }
    __syncthreads();
    const u32 s = s_sym[b];
    ws->table.symlen_of_bucket[b] = (uint8_t)(s | (s_len[s] << 4));
}

// ----------------------------------------------------------------------------- k_pack
// Sweep 2: one wavefront per chunk.  Pass A re-derives each element's symbol, keeps it
// (4 bits) in LDS, sums the lane's code lengths and tracks the mantissa extremes of the
// kept buckets.  The chunk's size is then known; a decoupled look-back over a per-chunk
// state word gives its word offset (chunks are handed out by an atomic ticket, so every
// predecessor is already running).  Pass B emits the codes straight to their final place:
// every payload word is stored exactly once by the lane whose stream holds its first bit;
// partial words at lane boundaries travel through LDS.
constexpr int kMmCopies = 8;
constexpr u64 kFlagAgg = 1ull << 62, kFlagIncl = 2ull << 62, kValMask = (1ull << 62) - 1;

__device__ __forceinline__ u64 lookback(u64* state, u32 c, u32 size_words) {
    const u32 lane = lane_id();
    if (c == 0) {
        if (lane == 0) __hip_atomic_store(&state[0], kFlagIncl | size_words, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        return 0;
    }
    if (lane == 0) __hip_atomic_store(&state[c], kFlagAgg | size_words, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    u64 excl = 0;
    long long base = (long long)c - 1;
    while (true) {
        const long long idx = base - (long long)lane;
        u64 v = kFlagIncl;                       // before chunk 0: an inclusive prefix of 0
        if (idx >= 0) {
            do {
                v = __hip_atomic_load(&state[idx], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                if ((v >> 62) == 0) __builtin_amdgcn_s_sleep(2);
            } while ((v >> 62) == 0);
        }
        const u64 incl = __ballot((v >> 62) == 2);
        if (incl) {
            const u32 p = __ffsll((long long)incl) - 1;      // nearest predecessor holding an inclusive prefix
            excl += wave_sum64(lane <= p ? (v & kValMask) : 0);
            break;
        }
        excl += wave_sum64(v & kValMask);
        base -= 64;
    }
    if (lane == 0) __hip_atomic_store(&state[c], kFlagIncl | (excl + size_words), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return excl;
}

struct PackLds {
    uint8_t symlen[512];
    u32 codelen[kMaxSym];
    u32 mn[kMaxSym * kMmCopies], mx[kMaxSym * kMmCopies];
    u32 off[kW + 1];
    u32 hw[kW];
    uint16_t sym[kR * kW];       // 4 symbols (one row) per lane per entry
};

template <bool FAST>
__device__ __forceinline__ void pack_chunk(const float* __restrict__ w, const float* __restrict__ w_ref, u64 n,
                                           uint8_t* out, u64 area, Workspace* ws, u64* state,
                                           u32 c, u32 nchunks, u32 K, PackLds& L) {
    const u32 lane = lane_id();
    const u64 base = (u64)c * kChunk;
    // ---- pass A
    u32 bits = 0;
#pragma unroll 8
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        float a[4], b[4];
        load_row<FAST>(w, idx, n, a); load_row<FAST>(w_ref, idx, n, b);
        u32 packed = 0;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (!FAST && idx + v >= n) continue;
            const u32 u = delta_bits(a[v], b[v]);
            const u32 sl = L.symlen[u >> 23], s = sl & 15;
            bits += sl >> 4;
            packed |= s << (4 * v);
            if (s < K) {
                atomicMin(&L.mn[s * kMmCopies + (lane & (kMmCopies - 1))], u & 0x7FFFFFu);
                atomicMax(&L.mx[s * kMmCopies + (lane & (kMmCopies - 1))], u & 0x7FFFFFu);
            }
        }
        L.sym[r * kW + lane] = (uint16_t)packed;
    }
    // ---- size, offsets
    const u32 incl = wave_incl_scan(bits);
    const u32 o = incl - bits;                                  // first bit of this lane's stream
    const u32 total_bits = __shfl(incl, 63, 64);
    const u32 nwords = (total_bits + 31) >> 5;
    const u32 size_words = kLaneBitsWords + nwords;
    const u64 word_off = lookback(state, c, size_words);
    u32* off_tab = reinterpret_cast<u32*>(out + kHeaderBytes);
    if (lane == 0) {
        off_tab[c] = (u32)word_off;
        if (c + 1 == nchunks) ws->total_words = word_off + size_words;
    }
    uint8_t* rec = out + area + 4 * word_off;
    reinterpret_cast<uint16_t*>(rec)[lane] = (uint16_t)bits;
    u32* payload = reinterpret_cast<u32*>(rec + 2 * kW);
    L.off[lane] = o; L.hw[lane] = 0;
    if (lane == 0) L.off[kW] = total_bits;
    // ---- pass B
    u64 acc = 0;
    u32 nb = o & 31, widx = o >> 5;
    auto flush = [&]() {
        if (nb >= 32) {
            const u32 word = (u32)(acc >> (nb - 32));
            nb -= 32;
            if (widx * 32 >= o) payload[widx] = word; else L.hw[lane] = word;
            ++widx;
        }
    };
    if (bits > 0) {
#pragma unroll 4
        for (u32 r = 0; r < kR; ++r) {
            const u64 idx = base + (u64)r * kRowElems + lane * kV;
            const u32 p = L.sym[r * kW + lane];
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (FAST || idx + v < n) {
                    const u32 cl = L.codelen[(p >> (4 * v)) & 15];
                    acc = (acc << (cl & 31)) | (cl >> 5);
                    nb += cl & 31;
                }
                if (v & 1) flush();
            }
        }
    }
    u32 tail = 0; bool own_tail = false;
    if (bits > 0 && nb > 0) {
        tail = (u32)(acc << (32 - nb));
        if (widx * 32 >= o) own_tail = true; else L.hw[lane] = tail;   // stream inside one foreign word
    }
    __syncthreads();
    if (own_tail) {
        for (u32 q = lane + 1; q < kW && (L.off[q] >> 5) == widx; ++q) tail |= L.hw[q];
        payload[widx] = tail;
    }
    __syncthreads();
}

__global__ __launch_bounds__(64) void k_pack(const float* __restrict__ w, const float* __restrict__ w_ref, u64 n,
                                             uint8_t* out, Workspace* ws, u64* state, u32 nchunks, int aligned) {
    __shared__ PackLds L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    if (T.status != 0) return;
    for (u32 i = lane; i < 512; i += 64) L.symlen[i] = T.symlen_of_bucket[i];
    if (lane < kMaxSym) L.codelen[lane] = T.codelen[lane];
    for (u32 i = lane; i < kMaxSym * kMmCopies; i += 64) { L.mn[i] = 0x7FFFFFu; L.mx[i] = 0; }
    const u32 K = T.K;
    const u64 area = chunk_area_of(nchunks);
    __syncthreads();
    while (true) {
        u32 c = 0;
        if (lane == 0) c = atomicAdd(&ws->ticket, 1u);
        c = __builtin_amdgcn_readfirstlane(c);
        if (c >= nchunks) break;
        const bool full = (u64)(c + 1) * kChunk <= n;
        if (full && aligned) pack_chunk<true>(w, w_ref, n, out, area, ws, state, c, nchunks, K, L);
        else pack_chunk<false>(w, w_ref, n, out, area, ws, state, c, nchunks, K, L);
    }
    __syncthreads();
    if (lane < K) {
        u32 mn = 0x7FFFFFu, mx = 0;
#pragma unroll
        for (int k = 0; k < kMmCopies; ++k) { mn = min(mn, L.mn[lane * kMmCopies + k]); mx = max(mx, L.mx[lane * kMmCopies + k]); }
        if (mn <= mx) { atomicMin(&ws->mmin[lane], mn); atomicMax(&ws->mmax[lane], mx); }
    }
}

// ----------------------------------------------------------------------------- k_finalize
// Representatives (Section 3.1.1: mean of the bucket's largest and smallest member,
// rounded once to fp32, ties to even, done on the mantissas since both share a binade)
// and the header.
__global__ __launch_bounds__(128) void k_finalize(uint8_t* out, Workspace* ws, u64 n, int nbits, u32 nchunks) {
    __shared__ u32 hdr[kHeaderBytes / 4];
    const u32 t = threadIdx.x;
    const Table& T = ws->table;
    hdr[t] = 0;
    __syncthreads();
    const bool ok = T.status == 0;
    const u64 area = chunk_area_of(nchunks);
    const u64 total = ok ? area + 4 * ws->total_words : kHeaderBytes;
    if (t == 0) {
        hdr[0] = 0x3142434Cu;                     // "LCB1"
        hdr[1] = 1u | (kHeaderBytes << 16);
        hdr[2] = (u32)n; hdr[3] = (u32)(n >> 32);
        hdr[4] = (u32)nbits;
        hdr[6] = kW; hdr[7] = kV; hdr[8] = kR;
        hdr[10] = (u32)total; hdr[11] = (u32)(total >> 32);
        hdr[12] = T.status;
        if (ok) { hdr[5] = T.K; hdr[9] = nchunks; hdr[13] = T.k_E; hdr[14] = T.max_len; }
        ws->result.bytes = total; ws->result.status = T.status; ws->result.pad = 0;
    }
    if (ok && t <= T.K) {
        const u32 len = T.codelen[t] & 31;
        u32 bucket = 0xFFFFu, rep = 0;
        if (t < T.K) {
            bucket = T.kept[t];
            const u32 sum = ws->mmin[t] + ws->mmax[t];
            u32 mm = sum >> 1;
            if ((sum & 1) && (mm & 1)) ++mm;
            rep = (bucket << 23) | mm;
        }
        hdr[16 + 4 * t + 0] = bucket | (len << 16);
        hdr[16 + 4 * t + 1] = rep;
        hdr[16 + 4 * t + 2] = (u32)T.cnt[t];
        hdr[16 + 4 * t + 3] = (u32)(T.cnt[t] >> 32);
    }
    __syncthreads();
    reinterpret_cast<u32*>(out)[t] = hdr[t];
    if (ok) {
        // last offset entry and the zero padding of the offset table
        u32* off_tab = reinterpret_cast<u32*>(out + kHeaderBytes);
        const u32 entries = (u32)((area - kHeaderBytes) / 4);
        if (t == 0) off_tab[nchunks] = (u32)ws->total_words;
        if (t >= 1 && nchunks + t < entries) off_tab[nchunks + t] = 0;
    }
}

// ----------------------------------------------------------------------------- k_dec_prepare
__global__ __launch_bounds__(256) void k_dec_prepare(const uint8_t* blob, u64 n, u64 max_total, Workspace* ws) {
    __shared__ u32 hdr[kHeaderBytes / 4];
    __shared__ u32 s_ok, s_K, s_max_len;
    __shared__ u32 s_len[kMaxSym], s_code[kMaxSym];
    const u32 t = threadIdx.x;
    if (t < kHeaderBytes / 4) hdr[t] = reinterpret_cast<const u32*>(blob)[t];
    __syncthreads();
    if (t == 0) {
        const u64 hn = hdr[2] | ((u64)hdr[3] << 32), total = hdr[10] | ((u64)hdr[11] << 32);
        const u32 nbits = hdr[4], K = hdr[5];
        const u64 nchunks = (n + kChunk - 1) / kChunk, area = chunk_area_of(nchunks);
        u32 status = 0;
        bool ok = hdr[0] == 0x3142434Cu && hdr[1] == (1u | (kHeaderBytes << 16)) && hdr[12] == 0;
        if (ok && hn != n) { ok = false; status = 1; }
        ok = ok && nbits >= 1 && nbits <= 4 && K <= (1u << nbits) - 1;
        ok = ok && hdr[6] == kW && hdr[7] == kV && hdr[8] == kR && hdr[9] == nchunks;
        ok = ok && total >= area && total <= max_total && ((total - area) & 3) == 0;
        u64 cnt_sum = 0; u32 kraft = 0, active = 0, max_len = 0;
        u32 per_len[17];
        for (int L = 0; L <= 16; ++L) per_len[L] = 0;
        if (ok) {
            for (u32 j = 0; j <= K; ++j) {
                const u32 w0 = hdr[16 + 4 * j], rep = hdr[17 + 4 * j];
                const u64 c = hdr[18 + 4 * j] | ((u64)hdr[19 + 4 * j] << 32);
                const u32 bucket = w0 & 0xFFFFu, len = (w0 >> 16) & 0xFFu;
                cnt_sum += c;
                if ((c > 0) != (len > 0) || len > 15 || (w0 >> 24) != 0) ok = false;
                if (j < K && (bucket >= 512 || (bucket & 255) == 0 || (bucket & 255) == 255 || (rep >> 23) != bucket)) ok = false;
                if (j == K && rep != 0) ok = false;
                s_len[j] = len; ws->dec.rep_bits[j] = rep;
                if (len && len <= 15) { kraft += 1u << (15 - len); ++active; per_len[len]++; if (len > max_len) max_len = len; }
            }
            for (u32 j = K + 1; j < kMaxSym; ++j) { s_len[j] = 0; ws->dec.rep_bits[j] = 0; }
            if (cnt_sum != n) ok = false;
            if (active >= 2 && kraft != (1u << 15)) ok = false;
            if (active == 1 && kraft != (1u << 14)) ok = false;
        }
        if (ok) {
            u32 next_code[17], code = 0;
            for (int L = 1; L <= 16; ++L) { code = (code + per_len[L - 1]) << 1; next_code[L] = code; }
            for (u32 j = 0; j < kMaxSym; ++j) s_code[j] = s_len[j] ? next_code[s_len[j]]++ : 0;
        }
        if (!ok && status == 0) status = 4;
        ws->dec.K = K; ws->dec.max_len = max_len; ws->dec.num_chunks = (u32)nchunks; ws->dec.status = status;
        ws->dec.area = area; ws->dec.total_words = ok ? (total - area) / 4 : 0;
        ws->dec_status = status;
        ws->result.bytes = total; ws->result.status = status; ws->result.pad = max_len;
        s_ok = ok; s_K = K; s_max_len = max_len;
    }
    __syncthreads();
    if (!s_ok) return;
    const u32 M = s_max_len, K = s_K;
    for (u32 i = t; i < (1u << M); i += 256) {
        u32 entry = K;                             // length 0: "no code starts like this"
        for (u32 j = 0; j <= K; ++j)
            if (s_len[j] && (i >> (M - s_len[j])) == s_code[j]) entry = j | (s_len[j] << 4);
        ws->dec_lut[i] = (uint8_t)entry;
    }
}

// ----------------------------------------------------------------------------- k_dec_validate
// One wavefront per chunk: the offset table must be the running sum of the record sizes
// that the lane lengths imply, starting at 0 and ending at the blob's stated size.
__global__ __launch_bounds__(256) void k_dec_validate(const uint8_t* blob, Workspace* ws, u32 nchunks) {
    if (ws->dec.status != 0) return;
    const u32 c = blockIdx.x * 4 + (threadIdx.x >> 6), lane = lane_id();
    if (c >= nchunks) return;
    const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
    const u64 o0 = off_tab[c], o1 = off_tab[c + 1], tw = ws->dec.total_words;
    bool ok = o0 <= o1 && o1 <= tw && o1 - o0 >= kLaneBitsWords && (c > 0 || o0 == 0) && (c + 1 < nchunks || o1 == tw);
    if (ok) {
        const u32 lb = reinterpret_cast<const uint16_t*>(blob + ws->dec.area + 4 * o0)[lane];
        const u32 sum = wave_sum32(lb);
        ok = (o1 - o0 == kLaneBitsWords + ((sum + 31) >> 5)) && sum > 0 && !__any(lb > kR * kV * 15);
    }
    if (!ok && lane == 0) atomicOr(&ws->dec_status, 4u);
}

// ----------------------------------------------------------------------------- k_decode
// Algorithm 1 line 7: one wavefront per chunk, lane l decoding its own stream with a
// 64-bit MSB-first window and a 2^max_len-entry look-up table in LDS, adding the
// representative into w_ref with 16-byte read-modify-writes.
template <bool FAST>
__device__ __forceinline__ void decode_chunk(const uint8_t* __restrict__ blob, float* __restrict__ w_ref, u64 n,
                                             Workspace* ws, u32 c, const uint8_t* lut, const float* s_rep,
                                             u32 M, u32 K, u64 area) {
    const u32 lane = lane_id();
    const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
    const u32 o0 = off_tab[c], o1 = off_tab[c + 1];
    const uint8_t* rec = blob + area + 4 * (u64)o0;
    const u32 nwords = o1 - o0 - kLaneBitsWords;        // >= 1 (validated)
    const u32 lane_bits = reinterpret_cast<const uint16_t*>(rec)[lane];
    const u32* __restrict__ pw = reinterpret_cast<const u32*>(rec + 2 * kW);
    const u32 o = wave_incl_scan(lane_bits) - lane_bits;
    const u32 last = nwords - 1;
    u32 wi = o >> 5;
    const u32 sh = o & 31;
    const u32 w0 = pw[min(wi, last)], w1 = pw[min(wi + 1, last)];
    u64 win = (((u64)w0 << 32) | w1) << sh;
    u32 avail = 64 - sh, used = 0;
    wi += 2;
    u32 next = pw[min(wi, last)];
    const u64 base = (u64)c * kChunk;
    const u32 shr = 64 - M;
#pragma unroll 4
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        if (!FAST && idx >= n) break;
        float x[4];
        load_row<FAST>(w_ref, idx, n, x);
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (FAST || idx + v < n) {
                const u32 e = lut[(u32)(win >> shr)];
                const u32 len = e >> 4, s = e & 15;
                win <<= len; avail -= len; used += len;
                const float rep = s_rep[s];
                x[v] = (s < K) ? __fadd_rn(x[v], rep) : x[v];
            }
            if ((v & 1) && avail <= 32) {
                win |= (u64)next << (32 - avail);
                avail += 32; ++wi;
                next = pw[min(wi, last)];
            }
        }
        if (FAST) {
            *reinterpret_cast<float4*>(w_ref + idx) = make_float4(x[0], x[1], x[2], x[3]);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) if (idx + v < n) w_ref[idx + v] = x[v];
        }
    }
    if (__any(used != lane_bits) && lane == 0) atomicOr(&ws->dec_status, 4u);
}

__global__ __launch_bounds__(256) void k_decode(const uint8_t* __restrict__ blob, float* __restrict__ w_ref, u64 n,
                                                Workspace* ws, u32 nchunks, int aligned) {
    extern __shared__ __align__(16) uint8_t lut[];
    __shared__ float s_rep[kMaxSym];
    const u32 t = threadIdx.x;
    const u32 M = ws->dec.max_len, K = ws->dec.K;
    const u64 area = ws->dec.area;
    {
        const u32 nlut = 1u << M;
        if (nlut >= 1024) {
            const uint4* src = reinterpret_cast<const uint4*>(ws->dec_lut);
            uint4* dst = reinterpret_cast<uint4*>(lut);
            for (u32 i = t; i < nlut / 16; i += 256) dst[i] = src[i];
        } else {
            for (u32 i = t; i < nlut; i += 256) lut[i] = ws->dec_lut[i];
        }
    }
    if (t < kMaxSym) s_rep[t] = __uint_as_float(ws->dec.rep_bits[t]);
    __syncthreads();
    const u32 wave = t >> 6;
    for (u32 c = blockIdx.x * 4 + wave; c < nchunks; c += gridDim.x * 4) {
        const bool full = (u64)(c + 1) * kChunk <= n;
        if (full && aligned) decode_chunk<true>(blob, w_ref, n, ws, c, lut, s_rep, M, K, area);
        else decode_chunk<false>(blob, w_ref, n, ws, c, lut, s_rep, M, K, area);
    }
}

// ----------------------------------------------------------------------------- launchers
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

void launch_reset(Workspace* ws, u64* state, uint64_t nchunks, hipStream_t s) {
    const u32 blocks = (u32)((nchunks + 255) / 256);
    hipLaunchKernelGGL(k_reset, dim3(blocks < 1 ? 1 : (blocks > 1024 ? 1024 : blocks)), dim3(256), 0, s, ws, state, (u64)nchunks);
}

void launch_hist(const float* w, const float* w_ref, uint64_t n, Workspace* ws, int num_cu, hipStream_t s) {
    if (n == 0) return;
    u64 blocks = (n / 4 + 1023) / 1024;
    const u64 cap = (u64)num_cu * 8;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    if (aligned16(w) && aligned16(w_ref)) hipLaunchKernelGGL(k_hist<true>, dim3((u32)blocks), dim3(256), 0, s, w, w_ref, (u64)n, ws);
    else hipLaunchKernelGGL(k_hist<false>, dim3((u32)blocks), dim3(256), 0, s, w, w_ref, (u64)n, ws);
}

void launch_table(Workspace* ws, uint64_t n, int nbits, hipStream_t s) {
    hipLaunchKernelGGL(k_table, dim3(1), dim3(512), 0, s, ws, (u64)n, nbits);
}

void launch_pack(const float* w, const float* w_ref, uint64_t n, uint8_t* out, Workspace* ws,
                 u64* state, int num_cu, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (u64)num_cu * 12;
    if (blocks > nchunks) blocks = nchunks;
    const int al = aligned16(w) && aligned16(w_ref);
    hipLaunchKernelGGL(k_pack, dim3((u32)blocks), dim3(64), 0, s, w, w_ref, (u64)n, out, ws, state, (u32)nchunks, al);
}

void launch_finalize(uint8_t* out, Workspace* ws, uint64_t n, int nbits, hipStream_t s) {
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(128), 0, s, out, ws, (u64)n, nbits, (u32)num_chunks_of(n));
}

void launch_dec_prepare(const uint8_t* blob, uint64_t n, uint64_t max_total, Workspace* ws, hipStream_t s) {
    hipLaunchKernelGGL(k_dec_prepare, dim3(1), dim3(256), 0, s, blob, (u64)n, (u64)max_total, ws);
}

void launch_dec_validate(const uint8_t* blob, uint64_t n, Workspace* ws, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    hipLaunchKernelGGL(k_dec_validate, dim3((u32)((nchunks + 3) / 4)), dim3(256), 0, s, blob, ws, (u32)nchunks);
}

void launch_decode(const uint8_t* blob, float* w_ref, uint64_t n, Workspace* ws, uint32_t max_len,
                   int num_cu, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (nchunks + 3) / 4;
    const u64 cap = (u64)num_cu * 4;
    if (blocks > cap) blocks = cap;
    const size_t lds = (size_t)1 << (max_len < 4 ? 4 : max_len);
    hipLaunchKernelGGL(k_decode, dim3((u32)blocks), dim3(256), lds, s, blob, w_ref, (u64)n, ws, (u32)nchunks,
                       (int)aligned16(w_ref));
}

}  // namespace lc
