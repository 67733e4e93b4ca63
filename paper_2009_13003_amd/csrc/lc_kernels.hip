// HIP kernels of the LC-Checkpoint compress / restore path for gfx950 (wave64).
//
// encode:  k_hist -> k_table -> k_pack -> k_place -> k_finalize (which also clears the scratch state
//          for the next call); k_reset only for a fresh scratch area
// decode:  k_dec_check -> k_decode (gated on the check's verdict, no host round trip between)
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

// 16-byte load of data that is read once: marked non-temporal so that the stream does not push
// other lines out of the caches (measured: +10 % read bandwidth on the sweeps).
typedef float f32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ float4 load_stream(const float4* p) {
    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(v.x, v.y, v.z, v.w);
}

// ---- element types of the parameter arrays.  The method works on the fp32 delta (Algorithm 1 line 4):
// bf16 / fp16 parameters are widened exactly on load, and the restored value fl32(w_ref + rep) is rounded
// once, to nearest even, on store.  Raw<DT> is what one lane holds of one row: 4 consecutive elements.
template <int DT> struct Raw { typedef uint2 type; };
template <> struct Raw<kF32> { typedef float4 type; };
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

template <int DT> __device__ __forceinline__ constexpr u32 elem_bytes() { return DT == kF32 ? 4u : 2u; }

// 4 consecutive elements starting at element index i (a multiple of 4, base aligned to 4 elements), non-temporal
template <int DT>
__device__ __forceinline__ typename Raw<DT>::type load_raw(const void* base, u64 i) {
    if constexpr (DT == kF32) {
        return load_stream(reinterpret_cast<const float4*>(static_cast<const float*>(base) + i));
    } else {
        const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(static_cast<const uint16_t*>(base) + i));
        return make_uint2(v.x, v.y);
    }
}

__device__ __forceinline__ float widen16(u32 h, bool bf16) {
    return bf16 ? __uint_as_float(h << 16) : (float)__builtin_bit_cast(_Float16, (unsigned short)h);
}
__device__ __forceinline__ u32 narrow16(float x, bool bf16) {      // finite x, round to nearest even
    if (bf16) { const u32 u = __float_as_uint(x); return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16; }
    return (u32)__builtin_bit_cast(unsigned short, (_Float16)x);      // v_cvt_f16_f32, round to nearest even
}

template <int DT>
__device__ __forceinline__ void unpack(const typename Raw<DT>::type& r, float (&x)[4]) {
    if constexpr (DT == kF32) { x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w; }
    else {
        x[0] = widen16(r.x & 0xFFFFu, DT == kBF16); x[1] = widen16(r.x >> 16, DT == kBF16);
        x[2] = widen16(r.y & 0xFFFFu, DT == kBF16); x[3] = widen16(r.y >> 16, DT == kBF16);
    }
}

template <int DT>
__device__ __forceinline__ float load_one(const void* base, u64 i) {
    if constexpr (DT == kF32) return static_cast<const float*>(base)[i];
    else return widen16(static_cast<const uint16_t*>(base)[i], DT == kBF16);
}

template <int DT>
__device__ __forceinline__ void store_one(void* base, u64 i, float x) {
    if constexpr (DT == kF32) static_cast<float*>(base)[i] = x;
    else static_cast<uint16_t*>(base)[i] = (uint16_t)narrow16(x, DT == kBF16);
}

template <int DT>
__device__ __forceinline__ void store4(void* base, u64 i, const float (&x)[4]) {
    if constexpr (DT == kF32) {
        *reinterpret_cast<float4*>(static_cast<float*>(base) + i) = make_float4(x[0], x[1], x[2], x[3]);
    } else {
        *reinterpret_cast<uint2*>(static_cast<uint16_t*>(base) + i) =
            make_uint2(narrow16(x[0], DT == kBF16) | (narrow16(x[1], DT == kBF16) << 16),
                       narrow16(x[2], DT == kBF16) | (narrow16(x[3], DT == kBF16) << 16));
    }
}

template <bool FAST, int DT = kF32>
__device__ __forceinline__ void load_row(const void* __restrict__ p, u64 idx, u64 n, float (&x)[4]) {
    if (FAST) {
        unpack<DT>(load_raw<DT>(p, idx), x);
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = (idx + v < n) ? load_one<DT>(p, idx + v) : 0.0f;
    }
}

// ----------------------------------------------------------------------------- k_reset
// Brings the scratch state to what every encode call expects to find (and leaves behind):
// zero bucket counts, empty extremes, zero group sums and arrival counters.  Only launched
// for a fresh scratch area or after a call that did not run to its end.
__device__ __forceinline__ void clear_encode_state(EncState* ws, u32* group_words, u32 ngroups, u32 tid, u32 nthr) {
    for (u32 i = tid; i < ngroups; i += nthr) group_words[i] = 0;
    for (u32 i = tid; i < 512; i += nthr) ws->hist[i] = 0;
    if (tid < kMaxSym) { ws->mmin[tid] = 0x7FFFFFu; ws->mmax[tid] = 0; }
    if (tid == 0) { ws->total_words = 0; ws->spec = 0; ws->spec_ok = 0; }
}

__global__ void k_reset(EncState* ws, u32* group_words, u32 ngroups) {
    clear_encode_state(ws, group_words, ngroups, threadIdx.x, blockDim.x);
}

// ----------------------------------------------------------------------------- k_hist
// Sweep 1 (Section 3.1.1, exponent-based quantization): population of each of the 2^9
// (sign, exponent) buckets.  LDS histogram replicated 8 times (copy = lane & 7, copies
// of one bin in different banks) so that lanes hitting the same popular bucket rarely
// collide; merged into 64-bit global counters once per workgroup.
constexpr int kHistCopies = 8;

// One 16-byte unit = EPU consecutive elements (4 fp32, 8 bf16 / fp16): counting does not care which lane
// sees which element, so every type is read in 16-byte accesses and kept as loaded until it is counted.
template <int DT, int EPU>
__device__ __forceinline__ void unpack_unit(const float4& t, float (&x)[EPU]) {
    if constexpr (DT == kF32) { x[0] = t.x; x[1] = t.y; x[2] = t.z; x[3] = t.w; }
    else {
        const u32 q[4] = {__float_as_uint(t.x), __float_as_uint(t.y), __float_as_uint(t.z), __float_as_uint(t.w)};
#pragma unroll
        for (int k = 0; k < 4; ++k) { x[2 * k] = widen16(q[k] & 0xFFFFu, DT == kBF16); x[2 * k + 1] = widen16(q[k] >> 16, DT == kBF16); }
    }
}

template <bool ALIGNED, int DT, int EPU>
__device__ __forceinline__ float4 load_unit(const void* __restrict__ p, u64 unit) {
    if (ALIGNED) return load_stream(reinterpret_cast<const float4*>(p) + unit);
    // whole units only, so every element is in range; assemble the same 16 bytes from element loads
    if constexpr (DT == kF32) {
        const float* q = static_cast<const float*>(p) + unit * 4;
        return make_float4(q[0], q[1], q[2], q[3]);
    } else {
        const uint16_t* q = static_cast<const uint16_t*>(p) + unit * 8;
        return make_float4(__uint_as_float(q[0] | ((u32)q[1] << 16)), __uint_as_float(q[2] | ((u32)q[3] << 16)),
                           __uint_as_float(q[4] | ((u32)q[5] << 16)), __uint_as_float(q[6] | ((u32)q[7] << 16)));
    }
}

template <bool ALIGNED, int DT>
__global__ __launch_bounds__(1024) void k_hist(const void* __restrict__ w, const void* __restrict__ w_ref,
                                               u64 n, EncState* ws) {
    __shared__ u32 h[512 * kHistCopies];
    constexpr int EPU = 16 / (int)elem_bytes<DT>();
    const u32 tid = threadIdx.x, nthr = blockDim.x;
    for (u32 i = tid; i < 512 * kHistCopies; i += nthr) h[i] = 0;
    __syncthreads();
    const u32 copy = tid & (kHistCopies - 1);
    const u64 nu = n / EPU;
    const u64 stride = (u64)gridDim.x * nthr;
    u64 u = (u64)blockIdx.x * nthr + tid;
    // Batches of PF 16-byte units per thread, one batch in flight while the previous one is counted.
    constexpr int PF = 4;
    float4 a0[PF], b0[PF], a1[PF], b1[PF];
    auto fetch = [&](float4 (&a)[PF], float4 (&b)[PF], u64 at) {
#pragma unroll
        for (int k = 0; k < PF; ++k) { a[k] = load_unit<ALIGNED, DT, EPU>(w, at + k * stride); b[k] = load_unit<ALIGNED, DT, EPU>(w_ref, at + k * stride); }
    };
    auto count_unit = [&](const float4& a, const float4& b) {
        float x[EPU], y[EPU];
        unpack_unit<DT, EPU>(a, x); unpack_unit<DT, EPU>(b, y);
#pragma unroll
        for (int v = 0; v < EPU; ++v) atomicAdd(&h[(delta_bits(x[v], y[v]) >> 23) * kHistCopies + copy], 1u);
    };
    auto count = [&](float4 (&a)[PF], float4 (&b)[PF]) {
#pragma unroll
        for (int k = 0; k < PF; ++k) count_unit(a[k], b[k]);
    };
    const u64 step = PF * stride;
    if (u + (PF - 1) * stride < nu) {
        fetch(a0, b0, u);
        while (true) {
            const bool more1 = u + step + (PF - 1) * stride < nu;
            if (more1) fetch(a1, b1, u + step);
            count(a0, b0);
            u += step;
            if (!more1) break;
            const bool more0 = u + step + (PF - 1) * stride < nu;
            if (more0) fetch(a0, b0, u + step);
            count(a1, b1);
            u += step;
            if (!more0) break;
        }
    }
    for (; u < nu; u += stride) count_unit(load_unit<ALIGNED, DT, EPU>(w, u), load_unit<ALIGNED, DT, EPU>(w_ref, u));
    if (blockIdx.x == 0 && tid < (u32)(n - EPU * nu)) {
        const u64 i = EPU * nu + tid;
        atomicAdd(&h[(delta_bits(load_one<DT>(w, i), load_one<DT>(w_ref, i)) >> 23) * kHistCopies + copy], 1u);
    }
    __syncthreads();
    for (u32 b = tid; b < 512; b += nthr) {
        u32 s = 0;
#pragma unroll
        for (int k = 0; k < kHistCopies; ++k) s += h[b * kHistCopies + k];
        if (s) atomicAdd(&ws->hist[b], (u64)s);
    }
}

// ----------------------------------------------------------------------------- k_table
// Priority promotion (Section 3.1.1) and the Huffman table (Section 3.1.2), one wavefront.  Lane l looks at one exponent level (both signs) per step, from
// the largest exponent down; a ballot/popcount scan ranks the non-empty buckets (+ before - at
// equal exponent).  Lane 0 then builds the code lengths with two queues and the canonical codes
// with per-length counters.
struct TableLds {
    uint8_t sym[512];
    u64 cnt[kMaxSym + 1];
    u32 kept[kMaxSym], len[kMaxSym + 1], code[kMaxSym + 1];
    u32 leaf[kMaxSym], left[kMaxSym], right[kMaxSym], depth[kMaxSym];
    u64 node_w[kMaxSym];
};

// When the sweep before it coded speculatively with a cached table (ws->spec), the kernel also decides
// whether that stands: this checkpoint's kept set must be the cached one and exactly the symbols with a
// cached code must occur.  If so the cached lengths are kept and the sweep's output is final (spec_ok);
// if not, the traces of the speculative coding are cleared and the table is this checkpoint's own.
__device__ __forceinline__ void table_build(EncState* ws, u64 n, int nbits, u32* group_words, u32 ngroups) {
    __shared__ TableLds S;
    __shared__ u32 s_reuse;
    const u32 lane = lane_id();
    const bool active = threadIdx.x < kW;
    const u32 kmax = (1u << nbits) - 1;
    if (active) for (u32 i = lane; i <= kMaxSym; i += kW) { S.cnt[i] = 0; S.len[i] = 0; S.code[i] = 0; if (i < kMaxSym) S.kept[i] = 0; }
    u32 total = 0;
    bool nonfinite = false, zero_class = false;
    for (u32 step = 0; active && step < 4; ++step) {
        const u32 E = 255 - (step * kW + lane);
        const u64 c0 = ws->hist[E], c1 = ws->hist[256 + E];
        const bool normal = E >= 1 && E <= 254;
        const bool cand0 = normal && c0 > 0, cand1 = normal && c1 > 0;
        const u64 m0 = __ballot(cand0), m1 = __ballot(cand1), lt = (1ull << lane) - 1;
        const u32 r0 = total + __popcll(m0 & lt) + __popcll(m1 & lt), r1 = r0 + (cand0 ? 1u : 0u);
        S.sym[E] = 0xFF; S.sym[256 + E] = 0xFF;
        if (cand0 && r0 < kmax) { S.kept[r0] = E; S.cnt[r0] = c0; S.sym[E] = (uint8_t)r0; }
        if (cand1 && r1 < kmax) { S.kept[r1] = 256 + E; S.cnt[r1] = c1; S.sym[256 + E] = (uint8_t)r1; }
        total += __popcll(m0) + __popcll(m1);
        nonfinite = nonfinite || __any(E == 255 && (c0 | c1) != 0);
        zero_class = zero_class || __any(E == 0 && (c0 | c1) != 0);
    }
    const u32 K = total < kmax ? total : kmax;
    __syncthreads();
    if (threadIdx.x == 0) {
        Table& T = ws->table;
        u64 kept_total = 0;
        for (u32 j = 0; j < K; ++j) kept_total += S.cnt[j];
        S.cnt[K] = n - kept_total;
        const u32 msym = K + 1;
        u32 max_len = 0;
        bool reuse = false;
        if (ws->spec) {
            reuse = !nonfinite && T.K == K;
            for (u32 j = 0; j < K && reuse; ++j) reuse = T.kept[j] == S.kept[j];
            for (u32 j = 0; j < msym && reuse; ++j) reuse = ((T.codelen[j] & 31) != 0) == (S.cnt[j] != 0);
            if (reuse) for (u32 j = 0; j < msym; ++j) { S.len[j] = T.codelen[j] & 31; if (S.len[j] > max_len) max_len = S.len[j]; }
        }
        s_reuse = reuse;
        ws->spec_ok = reuse;
        // leaves in ascending (count, symbol) order
        u32 nl = 0;
        if (!reuse) {
            for (u32 sy = 0; sy < msym; ++sy) {
                if (S.cnt[sy] == 0) continue;
                u32 p = nl++;
                while (p > 0 && S.cnt[S.leaf[p - 1]] > S.cnt[sy]) { S.leaf[p] = S.leaf[p - 1]; --p; }
                S.leaf[p] = sy;
            }
            if (nl == 1) { S.len[S.leaf[0]] = 1; max_len = 1; }
            else if (nl >= 2) {
                // two queues: sorted leaves and joined nodes in creation order (their weights never
                // decrease); on equal weight the leaf is taken first.  Ids >= 16 are joined nodes.
                u32 li = 0, qi = 0, ni = 0;
                for (u32 k = 0; k + 1 < nl; ++k) {
                    u32 pick[2]; u64 wsum = 0;
                    for (int q = 0; q < 2; ++q) {
                        const bool take_leaf = li < nl && (qi >= ni || S.cnt[S.leaf[li]] <= S.node_w[qi]);
                        if (take_leaf) { pick[q] = S.leaf[li]; wsum += S.cnt[S.leaf[li]]; ++li; }
                        else { pick[q] = 16 + qi; wsum += S.node_w[qi]; ++qi; }
                    }
                    S.node_w[ni] = wsum; S.left[ni] = pick[0]; S.right[ni] = pick[1]; ++ni;
                }
                S.depth[ni - 1] = 0;
                for (int i = (int)ni - 1; i >= 0; --i) {
                    const u32 d = S.depth[i] + 1, ch[2] = {S.left[i], S.right[i]};
                    for (int q = 0; q < 2; ++q) {
                        if (ch[q] >= 16) S.depth[ch[q] - 16] = d;
                        else { S.len[ch[q]] = d; if (d > max_len) max_len = d; }
                    }
                }
            }
        }
        // canonical codes by counting codes per length
        u32 per_len[17], next_code[17];
        for (int L = 0; L <= 16; ++L) per_len[L] = 0;
        for (u32 sy = 0; sy < msym; ++sy) per_len[S.len[sy]]++;
        per_len[0] = 0;
        u32 code = 0;
        for (int L = 1; L <= 16; ++L) { code = (code + per_len[L - 1]) << 1; next_code[L] = code; }
        for (u32 sy = 0; sy < msym; ++sy) if (S.len[sy]) S.code[sy] = next_code[S.len[sy]]++;
        for (u32 sy = 0; sy < kMaxSym; ++sy) {
            T.codelen[sy] = sy < msym ? ((S.code[sy] << 5) | S.len[sy]) : 0;
            T.kept[sy] = sy < K ? S.kept[sy] : 0;
            T.cnt[sy] = sy < msym ? S.cnt[sy] : 0;
        }
        T.K = K; T.max_len = max_len; T.k_E = total + (zero_class ? 1u : 0u);
        T.status = nonfinite ? 2u : 0u;
    }
    __syncthreads();
    if (active) for (u32 b = lane; b < 512; b += kW) {
        const u32 sy = S.sym[b] == 0xFF ? K : S.sym[b];
        ws->table.symlen_of_bucket[b] = (uint8_t)(sy | (S.len[sy] << 4));
    }
    if (active && ws->spec && !s_reuse) {          // the speculative coding is void: forget its extremes and sizes
        for (u32 i = lane; i < ngroups; i += kW) group_words[i] = 0;
        if (lane < kMaxSym) { ws->mmin[lane] = 0x7FFFFFu; ws->mmax[lane] = 0; }
    }
}

__global__ __launch_bounds__(64) void k_table(EncState* ws, u64 n, int nbits, u32* group_words, u32 ngroups) {
    table_build(ws, n, nbits, group_words, ngroups);
}

// ----------------------------------------------------------------------------- k_spec_table
// lc_encode_cached, before the sweep: turns a usable cache (valid, same nbits, kept buckets in strict
// priority order, lengths forming a complete prefix code) into the table the sweep codes with.
__global__ __launch_bounds__(64) void k_spec_table(EncState* ws, const TableCache* cache, int nbits) {
    __shared__ u32 s_ok, s_len[kMaxSym + 1], s_sym[512];
    const u32 lane = threadIdx.x;
    Table& T = ws->table;
    for (u32 b = lane; b < 512; b += kW) s_sym[b] = 0xFF;
    __syncthreads();
    if (lane == 0) {
        const u32 kmax = (1u << nbits) - 1, K = cache->K;
        bool ok = cache->valid == 1 && cache->nbits == (u32)nbits && K <= kmax;
        u32 kraft = 0, nact = 0, max_len = 0, per_len[17];
        for (int L = 0; L <= 16; ++L) per_len[L] = 0;
        for (u32 j = 0; j <= kMaxSym; ++j) s_len[j] = 0;
        if (ok) {
            u32 prev_key = 0xFFFFFFFFu;
            for (u32 j = 0; j < K; ++j) {
                const u32 b = cache->kept[j], e = b & 255;
                const u32 key = (e << 1) | (1u - ((b >> 8) & 1u));     // larger exponent first, + before -
                if (b >= 512 || e == 0 || e == 255 || key >= prev_key) { ok = false; break; }
                prev_key = key;
            }
            for (u32 j = 0; j <= K && ok; ++j) {
                const u32 l = cache->len[j];
                if (l > 15) { ok = false; break; }
                s_len[j] = l;
                if (l) { kraft += 1u << (15 - l); ++nact; per_len[l]++; if (l > max_len) max_len = l; }
            }
            if (nact >= 2 && kraft != (1u << 15)) ok = false;
            if (nact == 1 && kraft != (1u << 14)) ok = false;
        }
        if (ok) {
            u32 next_code[17], code = 0;
            for (int L = 1; L <= 16; ++L) { code = (code + per_len[L - 1]) << 1; next_code[L] = code; }
            for (u32 j = 0; j < kMaxSym; ++j) {
                const u32 c = (j <= K && s_len[j]) ? next_code[s_len[j]]++ : 0;
                T.codelen[j] = j <= K ? ((c << 5) | s_len[j]) : 0;
                T.kept[j] = j < K ? cache->kept[j] : 0;
                T.cnt[j] = 0;
                if (j < K) s_sym[cache->kept[j]] = j;
            }
            T.K = K; T.max_len = max_len; T.k_E = 0; T.status = 0;
        }
        s_ok = ok;
        ws->spec = ok; ws->spec_ok = 0;
    }
    __syncthreads();
    if (s_ok) {
        const u32 K = cache->K;
        for (u32 b = lane; b < 512; b += kW) {
            const u32 sy = s_sym[b] == 0xFF ? K : s_sym[b];
            T.symlen_of_bucket[b] = (uint8_t)(sy | (s_len[sy] << 4));
        }
    }
}

// ----------------------------------------------------------------------------- k_pack
// Sweep 2: one wavefront per chunk, no communication between wavefronts.  Each lane codes its
// 256 elements into a bit string of its own, written word by word to the chunk's slot in the
// scratch area (lane-private, word k of lane l at slot[32 + 64 k + l]); the 64 bit lengths go
// to the head of the slot, their sum to chunk_bits[c].  Where the strings end up in the blob is
// decided afterwards by k_place, which knows all sizes.  A full, 16-byte aligned chunk takes
// the fast path: rows are fetched eight at a time, one batch ahead (and the next chunk's first
// batch before the current one ends), the table look-ups of 16 elements are issued together and
// two symbols are coded per look-up.  Ragged or unaligned chunks take a plain path.  The
// mantissa extremes of the kept buckets (Section 3.1.1: the representative is the mean of the
// bucket's largest and smallest member) are tracked on the way.
constexpr int kMmCopies = 32;       // LDS copies of the per-symbol extremes, one per lane of a half wave

constexpr u32 kStageRows = 32;      // code words per lane that a chunk gathers in LDS before they go to its slot

constexpr int kSpecCopies = 4;      // LDS copies of the bucket histogram in the speculative sweep

template <bool HIST>
struct PackLds {
    uint8_t sym8[512];               // bucket -> symbol << 3
    u32 codelen[kMaxSym];            // (code << 5) | len
    uint2 pair[256];                 // (symbol a, symbol b) -> {code of a followed by b, its length}
    u32 mn[kMaxSym * kMmCopies], mx[kMaxSym * kMmCopies];   // extremes of the delta bit patterns per symbol
    alignas(16) u32 stage[kStageRows * kW];                 // word k of lane l at [64 k + l], as in the slot
    u32 hist[HIST ? 512 * kSpecCopies : 1];                 // bucket populations (speculative sweep only)
};

// chunk_bits[c] = payload bits of chunk c; group_words[g] = record words of chunks 64g .. 64g+63
// (integer atomics: the sums do not depend on the order of arrival).
// One chunk's work as the coding loop sees it: the vector it belongs to, its index there, and where its
// code words, its bit count and its group's word sum go.
struct ChunkRef {
    const void* w; const void* w_ref;
    u64 n;
    u32 c;
    u32* slot; u32* bits_at; u32* group_at;
    u32 seg;                     // batched calls: which tensor
    bool valid, fast;            // fast: a full chunk of aligned arrays
};

__device__ __forceinline__ void finish_lane_sizes(const ChunkRef& ch, u32 nb, u32 nw) {
    const u32 lane = lane_id();
    const u32 bits = 32 * nw + nb;
    reinterpret_cast<uint16_t*>(ch.slot)[lane] = (uint16_t)bits;
    const u32 total = wave_sum32(bits);
    if (lane == 0) {
        *ch.bits_at = total;
        atomicAdd(ch.group_at, kLaneBitsWords + ((total + 31) >> 5));
    }
}

// Any size, any alignment: guarded scalar loads, one symbol per look-up.
template <bool HIST, bool PACK, int DT>
__device__ __noinline__ void pack_chunk_plain(const ChunkRef ch, PackLds<HIST>& L) {
    const u32 lane = lane_id();
    const void* __restrict__ w = ch.w; const void* __restrict__ w_ref = ch.w_ref;
    const u64 n = ch.n, base = (u64)ch.c * kChunk;
    u32* slot = ch.slot;
    const u32 mm = lane & (kMmCopies - 1);
    u64 acc = 0;
    u32 nb = 0, nw = 0;
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (idx + v < n) {
                const u32 u = delta_bits(load_one<DT>(w, idx + v), load_one<DT>(w_ref, idx + v));
                if (HIST) atomicAdd(&L.hist[(u >> 23) * kSpecCopies + (lane & (kSpecCopies - 1))], 1u);
                if (!PACK) continue;
                const u32 sy = L.sym8[u >> 23] >> 3;
                const u32 cl = L.codelen[sy];
                atomicMin(&L.mn[sy * kMmCopies + mm], u);
                atomicMax(&L.mx[sy * kMmCopies + mm], u);
                acc = (acc << (cl & 31)) | (cl >> 5);
                nb += cl & 31;
            }
            if (PACK && (v & 1) && nb >= 32) {
                slot[kLaneBitsWords + nw * kW + lane] = (u32)(acc >> (nb - 32));
                ++nw; nb -= 32;
            }
        }
    }
    if (!PACK) return;
    if (nb > 0) slot[kLaneBitsWords + nw * kW + lane] = (u32)(acc << (32 - nb));
    finish_lane_sizes(ch, nb, nw);
}

constexpr int kPackPF = 8;          // rows per prefetch batch of the coding loop

// element index of this lane's 4 elements in row r of chunk c
__device__ __forceinline__ u64 row_at(u32 c, u32 r) { return (u64)c * kChunk + (u64)(r * kW + lane_id()) * kV; }

template <int DT>
__device__ __forceinline__ void fetch_first_batch(const ChunkRef& ch, typename Raw<DT>::type (&A)[kPackPF],
                                                  typename Raw<DT>::type (&B)[kPackPF]) {
#pragma unroll
    for (int k = 0; k < kPackPF; ++k) { A[k] = load_raw<DT>(ch.w, row_at(ch.c, k)); B[k] = load_raw<DT>(ch.w_ref, row_at(ch.c, k)); }
}

// A full, aligned chunk whose first batch of rows is already in A0/B0; leaves the first batch of `next`
// there if that chunk takes this path too.
template <bool ROWCHK, bool HIST, bool PACK, int DT>
__device__ __forceinline__ void pack_chunk_fast(const ChunkRef& cur, const ChunkRef& next,
                                                typename Raw<DT>::type (&A0)[kPackPF], typename Raw<DT>::type (&B0)[kPackPF],
                                                u32 K8, PackLds<HIST>& L) {
    constexpr int PF = kPackPF;
    typedef typename Raw<DT>::type raw_t;
    const u32 lane = lane_id();
    const u32 mm = lane & (kMmCopies - 1);
    const void* __restrict__ w = cur.w; const void* __restrict__ w_ref = cur.w_ref;
    const u32 c = cur.c;
    raw_t A1[PF], B1[PF];
    const bool next_fast = next.valid && next.fast;
    u32* lane_words = cur.slot + kLaneBitsWords + lane;
    u64 acc = 0;
    u32 nb = 0, nw = 0;                       // bits waiting in acc, words written
    // Lanes fill their words at different times; gathering them in LDS and storing whole rows at
    // the end of the chunk turns many partial-line stores into a few full ones.
    auto flush = [&]() {
        if (nb >= 32) {
            const u32 word = (u32)(acc >> (nb - 32));
            if (nw < kStageRows) L.stage[nw * kW + lane] = word;
            else lane_words[nw * kW] = word;
            ++nw; nb -= 32;
        }
    };
    // Four rows at a time: all table look-ups of the 16 elements are issued together, so the
    // LDS latency is paid twice per group instead of three times per row; only the shift/or
    // chain that grows the lane's bit string is serial.
    auto group = [&](const raw_t* a, const raw_t* b) {
        u32 u[16], t[16];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            float xa[4], xb[4];
            unpack<DT>(a[k], xa); unpack<DT>(b[k], xb);
#pragma unroll
            for (int v = 0; v < 4; ++v) u[4 * k + v] = delta_bits(xa[v], xb[v]);
        }
        if (HIST) {
#pragma unroll
            for (int i = 0; i < 16; ++i) atomicAdd(&L.hist[(u[i] >> 23) * kSpecCopies + (lane & (kSpecCopies - 1))], 1u);
        }
        if (!PACK) return;
#pragma unroll
        for (int i = 0; i < 16; ++i) t[i] = L.sym8[u[i] >> 23];
        uint2 p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            p[i] = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint8_t*>(L.pair) + ((t[2 * i] << 4) | t[2 * i + 1]));
        u32 tmin = t[0];
#pragma unroll
        for (int i = 1; i < 16; ++i) tmin = min(tmin, t[i]);
        if (__any(tmin < K8)) {
            // some lane holds a kept element: everyone updates the extremes of its symbols
            // (the merged symbol has a slot of its own that nobody reads)
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                atomicMin(&L.mn[t[i] * (kMmCopies / 8) + mm], u[i]);
                atomicMax(&L.mx[t[i] * (kMmCopies / 8) + mm], u[i]);
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            acc = (acc << p[i].y) | p[i].x; nb += p[i].y;
            if (!ROWCHK || (i & 1)) flush();
        }
    };
    for (u32 r0 = 0; r0 < kR; r0 += 2 * PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) { A1[k] = load_raw<DT>(w, row_at(c, r0 + PF + k)); B1[k] = load_raw<DT>(w_ref, row_at(c, r0 + PF + k)); }
        group(A0, B0); group(A0 + 4, B0 + 4);
        if (r0 + 2 * PF < kR) {
#pragma unroll
            for (int k = 0; k < PF; ++k) { A0[k] = load_raw<DT>(w, row_at(c, r0 + 2 * PF + k)); B0[k] = load_raw<DT>(w_ref, row_at(c, r0 + 2 * PF + k)); }
        } else if (next_fast) {
            fetch_first_batch<DT>(next, A0, B0);
        }
        group(A1, B1); group(A1 + 4, B1 + 4);
    }
    if (!PACK) return;
    // the last, partly filled word, then rows 0 .. (most words of any lane) - 1, four rows per store
    if (nb > 0) {
        const u32 word = (u32)(acc << (32 - nb));
        if (nw < kStageRows) L.stage[nw * kW + lane] = word;
        else lane_words[nw * kW] = word;
    }
    u32 rows = min(nw + (nb > 0 ? 1u : 0u), kStageRows);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) rows = max(rows, (u32)__shfl_xor(rows, d, 64));
    {
        const uint4* src = reinterpret_cast<const uint4*>(L.stage);
        uint4* dst = reinterpret_cast<uint4*>(cur.slot + kLaneBitsWords);
        for (u32 i = lane; i < rows * (kW / 4); i += kW) dst[i] = src[i];
    }
    finish_lane_sizes(cur, nb, nw);
}

// The coding loop of one wavefront over the chunks its source hands out.  Src::get(k) is the wavefront's
// k-th chunk, Src::enter(chunk, L) runs before each (a batched call switches tables there), Src::K8() and
// Src::rowchk() describe the table in force: symbol K << 3, and whether a lane's 64-bit accumulator can
// take a whole row (31 waiting bits + 4 codes of <= 8 bits) between flushes.
// ROWSEL: 1 / 0 = rowchk() is known to be true / false for every chunk (one vector, one table);
// -1 = ask per chunk (a batched call, where tables change).
template <bool HIST, bool PACK, int DT, int ROWSEL, typename Src>
__device__ __forceinline__ void pack_loop(Src& src, PackLds<HIST>& L) {
    typedef typename Raw<DT>::type raw_t;
    raw_t A0[kPackPF], B0[kPackPF];
    ChunkRef cur = src.get(0);
    if (cur.valid && cur.fast) fetch_first_batch<DT>(cur, A0, B0);
    for (u32 k = 0; cur.valid; ++k) {
        const ChunkRef next = src.get(k + 1);
        src.enter(cur, L);
        if (!cur.fast) {
            pack_chunk_plain<HIST, PACK, DT>(cur, L);
            if (next.valid && next.fast) fetch_first_batch<DT>(next, A0, B0);
        } else if (ROWSEL == 1 || (ROWSEL < 0 && src.rowchk())) {
            pack_chunk_fast<true, HIST, PACK, DT>(cur, next, A0, B0, src.K8(), L);
        } else {
            pack_chunk_fast<false, HIST, PACK, DT>(cur, next, A0, B0, src.K8(), L);
        }
        cur = next;
    }
}

// The chunks of one vector, dealt round-robin to the wavefronts of the grid.
struct VectorChunks {
    const void* w; const void* w_ref;
    u64 n;
    u32* prov; u32 slot_words; u32* chunk_bits; u32* group_words;
    u32 nchunks; bool aligned;
    u32 k8; bool row;
    __device__ __forceinline__ ChunkRef get(u32 k) const {
        ChunkRef ch;
        ch.c = blockIdx.x + k * gridDim.x;
        ch.valid = ch.c < nchunks;
        ch.w = w; ch.w_ref = w_ref; ch.n = n;
        ch.fast = aligned && (u64)(ch.c + 1) * kChunk <= n;
        ch.slot = prov + (u64)ch.c * slot_words;
        ch.bits_at = chunk_bits + ch.c;
        ch.group_at = group_words + (ch.c >> 6);
        ch.seg = 0;
        return ch;
    }
    template <bool HIST> __device__ __forceinline__ void enter(const ChunkRef&, PackLds<HIST>&) const {}
    __device__ __forceinline__ u32 K8() const { return k8; }
    __device__ __forceinline__ bool rowchk() const { return row; }
};

template <bool HIST>
__device__ __forceinline__ void pack_setup(PackLds<HIST>& L, const Table& T, u32 lane) {
    for (u32 i = lane; i < 512; i += 64) L.sym8[i] = (uint8_t)((T.symlen_of_bucket[i] & 15) << 3);
    if (lane < kMaxSym) L.codelen[lane] = T.codelen[lane];
    for (u32 i = lane; i < 256; i += 64) {
        const u32 ca = T.codelen[i >> 4], cb = T.codelen[i & 15];
        L.pair[i] = make_uint2(((ca >> 5) << (cb & 31)) | (cb >> 5), (ca & 31) + (cb & 31));
    }
    for (u32 i = lane; i < kMaxSym * kMmCopies; i += 64) { L.mn[i] = 0xFFFFFFFFu; L.mx[i] = 0; }
}

template <bool HIST>
__device__ __forceinline__ void pack_merge_extremes(PackLds<HIST>& L, EncState* ws, u32 K, u32 lane) {
    if (lane < K) {
        u32 mn = 0xFFFFFFFFu, mx = 0;
#pragma unroll
        for (int k = 0; k < kMmCopies; ++k) { mn = min(mn, L.mn[lane * kMmCopies + k]); mx = max(mx, L.mx[lane * kMmCopies + k]); }
        if (mn <= mx) { atomicMin(&ws->mmin[lane], mn & 0x7FFFFFu); atomicMax(&ws->mmax[lane], mx & 0x7FFFFFu); }
    }
}

template <int DT>
__global__ __launch_bounds__(64) void k_pack(const void* __restrict__ w, const void* __restrict__ w_ref, u64 n,
                                             EncState* ws, u32* chunk_bits, u32* group_words, u32* prov,
                                             u32 slot_words, u32 nchunks, int aligned) {
    __shared__ PackLds<false> L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    if (T.status != 0 || ws->spec_ok != 0) return;     // nothing to code, or the speculative sweep already did
    pack_setup(L, T, lane);
    const u32 K = T.K;
    __syncthreads();
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, aligned != 0, K << 3, T.max_len <= 8};
    if (src.row) pack_loop<false, true, DT, 1>(src, L);
    else pack_loop<false, true, DT, 0>(src, L);
    __syncthreads();
    pack_merge_extremes(L, ws, K, lane);
}

// ----------------------------------------------------------------------------- k_spec_sweep
// lc_encode_cached: the single sweep.  Counts the bucket populations like k_hist and, when a cached
// table is in place (ws->spec), codes every chunk with it like k_pack in the same pass over w and
// w_ref.  k_table then either confirms the coding or voids it.
template <int DT>
__global__ __launch_bounds__(64) void k_spec_sweep(const void* __restrict__ w, const void* __restrict__ w_ref, u64 n,
                                                   EncState* ws, u32* chunk_bits, u32* group_words, u32* prov,
                                                   u32 slot_words, u32 nchunks, int aligned) {
    __shared__ PackLds<true> L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    const bool spec = ws->spec != 0;
    for (u32 i = lane; i < 512 * kSpecCopies; i += 64) L.hist[i] = 0;
    if (spec) pack_setup(L, T, lane);
    const u32 K = spec ? T.K : 0;
    __syncthreads();
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, aligned != 0, K << 3, !spec || T.max_len <= 8};
    if (!spec) pack_loop<true, false, DT, 1>(src, L);
    else if (src.row) pack_loop<true, true, DT, 1>(src, L);
    else pack_loop<true, true, DT, 0>(src, L);
    __syncthreads();
    for (u32 b = lane; b < 512; b += 64) {
        u32 sum = 0;
#pragma unroll
        for (int k = 0; k < kSpecCopies; ++k) sum += L.hist[b * kSpecCopies + k];
        if (sum) atomicAdd(&ws->hist[b], (u64)sum);
    }
    if (spec) pack_merge_extremes(L, ws, K, lane);
}

// ----------------------------------------------------------------------------- k_place
// Builds the chunk area of the blob from the per-chunk slots, one wavefront per chunk.  The
// chunk's word offset is the sum of the record sizes before it (whole groups of 64 chunks from
// group_words, the rest from chunk_bits).  The 64 lane strings are joined without gaps: payload
// word W0 + j of a lane takes the low bits of its word j-1 and the high bits of its word j.
// A payload of up to kPlaceWords words is assembled in LDS (every lane ORs its shifted words
// into a cleared buffer, so words shared by neighbouring lanes need no special care) and
// written out with coalesced stores.  A larger payload is written directly: every word exactly
// once, by the lane whose string holds its first bit, boundary words merged through LDS.
constexpr u32 kPlaceWords = 2048;

// Representatives (Section 3.1.1: mean of the bucket's largest and smallest member, rounded once
// to fp32, ties to even, done on the mantissas since both share a binade), the header, the last
// offset entry, the result for the host; then the scratch state is cleared for the next call.
__device__ __forceinline__ void finalize_blob(uint8_t* out, EncState* ws, Result* host_result, TableCache* cache,
                                              u64 n, int nbits, u32 nchunks, u32 dtype) {
    __shared__ u32 hdr[kHeaderBytes / 4];
    const u32 t = threadIdx.x;
    const Table& T = ws->table;
    if (t < kHeaderBytes / 4) hdr[t] = 0;
    __syncthreads();
    const u32 status = T.status;
    const bool ok = status == 0;
    const u64 area = chunk_area_of(nchunks);
    const u64 total_words = ws->total_words;
    const u64 total = ok ? area + 4 * total_words : kHeaderBytes;
    if (t == 0) {
        hdr[0] = 0x3142434Cu;                     // "LCB1"
        hdr[1] = 1u | (kHeaderBytes << 16);
        hdr[2] = (u32)n; hdr[3] = (u32)(n >> 32);
        hdr[4] = (u32)nbits;
        hdr[6] = kW; hdr[7] = kV; hdr[8] = kR;
        hdr[10] = (u32)total; hdr[11] = (u32)(total >> 32);
        hdr[12] = status;
        hdr[15] = dtype;
        if (ok) { hdr[5] = T.K; hdr[9] = nchunks; hdr[13] = T.k_E; hdr[14] = T.max_len; }
        host_result->bytes = total; host_result->status = status; host_result->used_cache = ws->spec_ok;
        if (cache && ok) { cache->valid = 1; cache->nbits = (u32)nbits; cache->K = T.K; cache->pad = 0; }
    }
    if (cache && ok && t < kMaxSym) {              // what this blob was coded with, for the next call
        cache->kept[t] = t < T.K ? T.kept[t] : 0;
        cache->len[t] = t <= T.K ? (T.codelen[t] & 31) : 0;
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
    if (t < kHeaderBytes / 4) reinterpret_cast<u32*>(out)[t] = hdr[t];
    if (ok) {
        // last offset entry and the zero padding of the offset table
        u32* off_tab = reinterpret_cast<u32*>(out + kHeaderBytes);
        const u32 entries = (u32)((area - kHeaderBytes) / 4);
        if (t == 0) off_tab[nchunks] = (u32)total_words;
        if (t >= 1 && t < 4 && nchunks + t < entries) off_tab[nchunks + t] = 0;
    }
    __syncthreads();
}

__global__ __launch_bounds__(256) void k_finalize(uint8_t* out, EncState* ws, Result* host_result, u32* group_words,
                                                  TableCache* cache, u64 n, int nbits, u32 nchunks, u32 dtype) {
    finalize_blob(out, ws, host_result, cache, n, nbits, nchunks, dtype);
    clear_encode_state(ws, group_words, (nchunks + 63) / 64, threadIdx.x, blockDim.x);
    __threadfence_system();
}

// Chunk c of one vector, by one wavefront of a workgroup of four; `valid` false: an idle wavefront that only
// keeps the workgroup's barrier company.
__device__ __forceinline__ void place_chunk(uint8_t* out, EncState* ws, const u32* __restrict__ chunk_bits,
                                            const u32* __restrict__ group_words, const u32* __restrict__ prov,
                                            u32 slot_words, u32 nchunks, u32 c, bool valid) {
    __shared__ u32 s_off_all[4][kW + 1], s_hw_all[4][kW];
    __shared__ u32 s_buf_all[4][kPlaceWords];
    const u32 lane = lane_id(), wv = threadIdx.x >> 6;
    u32* s_off = s_off_all[wv];
    u32* s_hw = s_hw_all[wv];
    u32* s_buf = s_buf_all[wv];
    const u32* slot = prov + (u64)(valid ? c : 0) * slot_words;
    const u32 bits = valid ? reinterpret_cast<const uint16_t*>(slot)[lane] : 0;
    const u32 g = c >> 6;
    u64 part = (valid && 64 * g + lane < c) ? kLaneBitsWords + ((chunk_bits[64 * g + lane] + 31) >> 5) : 0;
    if (valid) {
#pragma unroll 4
        for (u32 j = lane; j < g; j += kW) part += group_words[j];
    }
    const u64 word_off = wave_sum64(part);
    const u32 incl = wave_incl_scan(bits);
    const u32 o = incl - bits;                               // first bit of this lane's string
    const u32 total_bits = __shfl(incl, 63, 64);
    const u32 nwords = (total_bits + 31) >> 5;
    uint8_t* rec = out + chunk_area_of(nchunks) + 4 * word_off;
    u32* payload = reinterpret_cast<u32*>(rec + 2 * kW);
    if (valid) {
        reinterpret_cast<uint16_t*>(rec)[lane] = (uint16_t)bits;
        if (lane == 0) {
            reinterpret_cast<u32*>(out + kHeaderBytes)[c] = (u32)word_off;
            if (c + 1 == nchunks) ws->total_words = word_off + kLaneBitsWords + nwords;
        }
    }
    const u32 sh = o & 31, W0 = o >> 5, nloc = (bits + 31) >> 5;
    const u32 nt = bits ? ((o + bits - 1) >> 5) - W0 + 1 : 0;   // payload words this lane touches
    u32 nt_max = nt;
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) nt_max = max(nt_max, (u32)__shfl_xor(nt_max, d, 64));
    const u32* lane_words = slot + kLaneBitsWords + lane;
    const bool staged = nwords <= kPlaceWords;               // wave-uniform
    if (staged) {
        for (u32 i = lane; i < nwords; i += kW) s_buf[i] = 0;
    } else {
        s_off[lane] = o; s_hw[lane] = 0;
        if (lane == 0) s_off[kW] = total_bits;
    }
    u32 prev = 0, tail = 0;
    bool own_tail = false;
    for (u32 j0 = 0; j0 < nt_max; j0 += 8) {
        u32 buf[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) buf[k] = (j0 + k < nloc) ? lane_words[(j0 + k) * kW] : 0;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const u32 j = j0 + k;
            if (j < nt) {
                const u32 val = __builtin_amdgcn_alignbit(prev, buf[k], sh);
                prev = buf[k];
                if (staged) {
                    atomicOr(&s_buf[W0 + j], val);
                } else {
                    const bool owned = j > 0 || sh == 0;         // the word's first bit is this lane's
                    if (!owned) s_hw[lane] = val;
                    else if (j + 1 == nt) { tail = val; own_tail = true; }
                    else payload[W0 + j] = val;
                }
            }
        }
    }
    __syncthreads();
    if (staged) {
        for (u32 i = lane; i < nwords; i += kW) payload[i] = s_buf[i];
    } else if (own_tail) {                                       // following lanes may start inside this word
        const u32 W = W0 + nt - 1;
        for (u32 q = lane + 1; q < kW && (s_off[q] >> 5) == W; ++q) tail |= s_hw[q];
        payload[W] = tail;
    }
}

__global__ __launch_bounds__(256) void k_place(uint8_t* out, EncState* ws, const u32* __restrict__ chunk_bits,
                                               const u32* __restrict__ group_words, const u32* __restrict__ prov,
                                               u32 slot_words, u32 nchunks) {
    const u32 c = blockIdx.x * 4 + (threadIdx.x >> 6);
    // the last workgroup may hold idle wavefronts
    place_chunk(out, ws, chunk_bits, group_words, prov, slot_words, nchunks, c, c < nchunks && ws->table.status == 0);
}

// ----------------------------------------------------------------------------- batched encode
// lc_encode_batch: many vectors, one table each, in six launches.  The chunks of all tensors are numbered
// through; the sweeps deal those dense chunks round-robin to their wavefronts exactly as for one vector,
// and a wavefront that moves on to a chunk of another tensor first hands in what it gathered for the last
// one (bucket counts, extremes) and loads the new tensor's table.
__global__ __launch_bounds__(256) void kb_setup(BatchArgs a) {
    const u32 i = blockIdx.x * blockDim.x + threadIdx.x, nthr = gridDim.x * blockDim.x;
    for (u32 g = i; g < a.total_chunks; g += nthr) {          // tensor of dense chunk g: last one starting at or before it
        u32 lo = 0, hi = a.count - 1;
        while (lo < hi) {
            const u32 mid = (lo + hi + 1) >> 1;
            if (a.segs[mid].chunk0 <= g) lo = mid; else hi = mid - 1;
        }
        // tensors without chunks share their successor's chunk0: step to the one that owns g
        while (lo > 0 && (a.segs[lo].nchunks == 0 || g >= a.segs[lo].chunk0 + a.segs[lo].nchunks)) --lo;
        a.seg_of_chunk[g] = lo;
    }
    for (u32 g = i; g < a.total_groups; g += nthr) a.group_words[g] = 0;
    constexpr u32 per = 512 + 2 * kMaxSym + 4;                // words of state to set per tensor
    for (u64 k = i; k < (u64)a.count * per; k += nthr) {
        EncState& st = a.states[k / per];
        const u32 j = (u32)(k % per);
        if (j < 512) st.hist[j] = 0;
        else if (j < 512 + kMaxSym) st.mmin[j - 512] = 0x7FFFFFu;
        else if (j < 512 + 2 * kMaxSym) st.mmax[j - 512 - kMaxSym] = 0;
        else if (j == 512 + 2 * kMaxSym) st.spec = 0;
        else if (j == 512 + 2 * kMaxSym + 1) st.spec_ok = 0;
        else if (j == 512 + 2 * kMaxSym + 2) st.total_words = 0;
        else st.table.status = 0;
    }
}

// The dense chunks of a batched call as a chunk source for the coding loop.
template <bool HIST, bool PACK>
struct BatchChunks {
    BatchArgs a;
    u32 active;                  // tensor whose counts / extremes / table the LDS holds (0xFFFFFFFF: none yet)
    u32 k8; bool row;
    __device__ __forceinline__ ChunkRef get(u32 k) const {
        ChunkRef ch;
        const u32 g = blockIdx.x + k * gridDim.x;
        ch.valid = g < a.total_chunks;
        ch.seg = 0; ch.c = 0; ch.w = nullptr; ch.w_ref = nullptr; ch.n = 0; ch.fast = false;
        ch.slot = nullptr; ch.bits_at = nullptr; ch.group_at = nullptr;
        if (ch.valid) {
            ch.seg = __builtin_amdgcn_readfirstlane(a.seg_of_chunk[g]);
            const Seg& sg = a.segs[ch.seg];
            ch.c = g - sg.chunk0;
            ch.w = sg.w; ch.w_ref = sg.w_ref; ch.n = sg.n;
            ch.fast = sg.aligned && (u64)(ch.c + 1) * kChunk <= sg.n;
            ch.slot = a.prov + (u64)g * a.slot_words;
            ch.bits_at = a.chunk_bits + g;
            ch.group_at = a.group_words + sg.group0 + (ch.c >> 6);
            // a tensor whose delta is not finite gets a header-only blob: nothing to code
            if (PACK && a.states[ch.seg].table.status != 0) { ch.n = 0; ch.fast = false; }
        }
        return ch;
    }
    __device__ __forceinline__ void hand_in(PackLds<HIST>& L) {
        if (active == 0xFFFFFFFFu) return;
        const u32 lane = lane_id();
        EncState* st = &a.states[active];
        if (HIST) {
            for (u32 b = lane; b < 512; b += kW) {
                u32 sum = 0;
#pragma unroll
                for (int k = 0; k < kSpecCopies; ++k) { sum += L.hist[b * kSpecCopies + k]; L.hist[b * kSpecCopies + k] = 0; }
                if (sum) atomicAdd(&st->hist[b], (u64)sum);
            }
        }
        if (PACK) pack_merge_extremes(L, st, st->table.K, lane);
    }
    __device__ __forceinline__ void enter(const ChunkRef& ch, PackLds<HIST>& L) {
        if (ch.seg == active) return;
        hand_in(L);
        active = ch.seg;
        if (PACK) {
            const Table& T = a.states[active].table;
            __syncthreads();                  // one wavefront per workgroup: orders the LDS traffic around the switch
            pack_setup(L, T, lane_id());
            k8 = T.K << 3; row = T.max_len <= 8;
            __syncthreads();
        }
    }
    __device__ __forceinline__ u32 K8() const { return k8; }
    __device__ __forceinline__ bool rowchk() const { return row; }
};

__global__ __launch_bounds__(64) void kb_hist(BatchArgs a) {
    __shared__ PackLds<true> L;
    for (u32 i = threadIdx.x; i < 512 * kSpecCopies; i += 64) L.hist[i] = 0;
    __syncthreads();
    BatchChunks<true, false> src = {a, 0xFFFFFFFFu, 0, true};
    pack_loop<true, false, kF32, 1>(src, L);
    src.hand_in(L);
}

__global__ __launch_bounds__(64) void kb_table(BatchArgs a) {
    table_build(&a.states[blockIdx.x], a.segs[blockIdx.x].n, a.nbits, nullptr, 0);
}

__global__ __launch_bounds__(64) void kb_pack(BatchArgs a) {
    __shared__ PackLds<false> L;
    BatchChunks<false, true> src = {a, 0xFFFFFFFFu, 0, true};
    pack_loop<false, true, kF32, 0>(src, L);      // flush per pair of codes: right for every table of the batch
    src.hand_in(L);
}

__global__ __launch_bounds__(256) void kb_place(BatchArgs a) {
    const u32 g = blockIdx.x * 4 + (threadIdx.x >> 6);
    const bool in_range = g < a.total_chunks;
    const u32 sidx = in_range ? a.seg_of_chunk[g] : 0;
    const Seg& sg = a.segs[sidx];
    EncState* st = &a.states[sidx];
    place_chunk(sg.out, st, a.chunk_bits + sg.chunk0, a.group_words + sg.group0, a.prov + (u64)sg.chunk0 * a.slot_words,
                a.slot_words, sg.nchunks, in_range ? g - sg.chunk0 : 0, in_range && st->table.status == 0);
}

__global__ __launch_bounds__(256) void kb_finalize(BatchArgs a) {
    const Seg& sg = a.segs[blockIdx.x];
    finalize_blob(sg.out, &a.states[blockIdx.x], &a.results[blockIdx.x], nullptr, sg.n, a.nbits, sg.nchunks, (u32)kF32);
    if (blockIdx.x == gridDim.x - 1) __threadfence_system();
}

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
    bool ok = nbits >= 1 && nbits <= 4 && K <= (1u << nbits) - 1 && hdr[6] == kW && hdr[7] == kV && hdr[8] == kR;
    if (nchunks == 0 && tw != 0) ok = false;
    u64 cnt_sum = 0; u32 kraft = 0, active = 0, max_len = 0;
    u32 per_len[17];
    for (int L = 0; L <= 16; ++L) per_len[L] = 0;
    for (u32 j = 0; j < kMaxSym; ++j) { s_len[j] = 0; s_code[j] = 0; D.info.rep_bits[j] = 0; }
    if (ok) {
        for (u32 j = 0; j <= K; ++j) {
            const u32 w0 = hdr[16 + 4 * j], rep = hdr[17 + 4 * j];
            const u64 cn = hdr[18 + 4 * j] | ((u64)hdr[19 + 4 * j] << 32);
            const u32 bucket = w0 & 0xFFFFu, len = (w0 >> 16) & 0xFFu;
            cnt_sum += cn;
            if ((cn > 0) != (len > 0) || len > 15 || (w0 >> 24) != 0) { ok = false; continue; }
            if (j < K && (bucket >= 512 || (bucket & 255) == 0 || (bucket & 255) == 255 || (rep >> 23) != bucket)) ok = false;
            if (j == K && rep != 0) ok = false;
            s_len[j] = len; D.info.rep_bits[j] = rep;
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
        for (u32 i = t; i < (1u << P); i += nthr) {
            u32 entry = K;
            for (u32 j = 0; j <= K; ++j) {
                const u32 L = s_len[j];
                if (L == 0) continue;
                if (L <= P) { if ((i >> (P - L)) == s_code[j]) entry = j | (L << 4); }
                else if ((s_code[j] >> (L - P)) == i) entry = 0xFF;
            }
            lut[i] = (uint8_t)entry;
        }
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

__device__ __forceinline__ void raise_status(Workspace* ws, HostResult* host, u64 epoch, u32 status) {
    const u64 word = (epoch << 8) | status;
    atomicMax(&ws->dec_status, word);     // gates the decode sweep on the device
    host->dec_status = word;              // what the host reads after waiting for the stream (any finding will do)
}

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
    // ---- one chunk per wavefront
    const u32 c = blockIdx.x * 4 + (t >> 6);
    if (c < nchunks && !dec_chunk_ok(blob, area, tw, nchunks, c) && lane == 0) raise_status(ws, host, epoch, 4u);
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
constexpr u32 kPayWords = 2048;      // LDS room for one chunk's payload (4 bits per element on average)

template <int WAVES>
struct DecLdsT {
    uint8_t lut1[1u << kDecLut1Bits];
    uint8_t lut2[1u << kDecLut2Bits];
    float rep[kMaxSym];
    u32 len[kMaxSym], code[kMaxSym];
    uint4 payload[WAVES][kPayWords / 4 + 1];
};
typedef DecLdsT<4> DecLds;

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
template <bool FAST, bool LV2, bool STAGED, int DT, typename LDS, typename Raise>
__device__ __forceinline__ void decode_rows(const u32* words, u32 nwords, u32 first_bit, u32 lane_bits,
                                            void* __restrict__ w_ref, u64 n, u32 c,
                                            const LDS& L, u32 P1, u32 P2, u32 K, Raise& raise) {
    const u32 lane = lane_id();
    BitReader<STAGED> br;
    br.start(words, nwords, first_bit);
    const u32 wi0 = br.wi, avail0 = br.avail;
    const u32 shr1 = 64 - P1, shr2 = 64 - P2;
    const u64 base = (u64)c * kChunk;
#pragma unroll 4
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        if (!FAST && idx >= n) break;
        float x[4];
        load_row<FAST, DT>(w_ref, idx, n, x);
        u32 smin = K;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (FAST || idx + v < n) {
                u32 e = L.lut1[(u32)(br.win >> shr1)];
                if (LV2 && e == 0xFF) {
                    e = L.lut2[(u32)(br.win >> shr2)];
                    if (e == 0xFF) e = decode_long(L, br.win, K);
                }
                const u32 len = e >> 4, sy = e & 15;
                br.win <<= len; br.avail -= len;
                smin = min(smin, sy);
                x[v] = __fadd_rn(x[v], L.rep[sy]);
            }
            if ((v & 1) && br.avail <= 32) br.refill();
        }
        if (FAST) {
            if (__any(smin < K)) store4<DT>(w_ref, idx, x);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) if (idx + v < n) store_one<DT>(w_ref, idx + v, x[v]);
        }
    }
    const u32 used = avail0 + 32 * (br.wi - wi0) - br.avail;
    if (__any(used != lane_bits) && lane == 0) raise(4u);
}

template <bool FAST, bool LV2, int DT, typename LDS, typename Raise>
__device__ __forceinline__ void decode_chunk(const uint8_t* __restrict__ blob, void* __restrict__ w_ref, u64 n,
                                             u32 c, LDS& L, u32 P1, u32 P2, u32 K, u64 area, Raise& raise) {
    const u32 lane = lane_id(), wv = threadIdx.x >> 6;
    const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
    const u32 o0 = off_tab[c], o1 = off_tab[c + 1];
    const uint8_t* rec = blob + area + 4 * (u64)o0;
    const u32 nwords = o1 - o0 - kLaneBitsWords;        // >= 1 (validated)
    const u32 lane_bits = reinterpret_cast<const uint16_t*>(rec)[lane];
    const u32 o = wave_incl_scan(lane_bits) - lane_bits;
    const u32* gw = reinterpret_cast<const u32*>(rec + 2 * kW);
    const u32 k0 = (u32)((reinterpret_cast<uintptr_t>(gw) >> 2) & 3);     // words between the 16-byte boundary and the payload
    if (nwords + k0 <= kPayWords) {
        // coalesced copy of [aligned start, payload end) to LDS; the bytes before the payload are the
        // record's own lane lengths, and the last vector is read word by word so no read passes the end
        const uint4* gv = reinterpret_cast<const uint4*>(gw - k0);
        const u32 nvec = (nwords + k0 + 3) >> 2;
        for (u32 i = lane; i < nvec; i += kW) {
            uint4 q;
            if (4 * i + 4 <= nwords + k0) q = gv[i];
            else {
                const u32* t = reinterpret_cast<const u32*>(gv + i);
                const u32 left = nwords + k0 - 4 * i;
                q.x = t[0]; q.y = left > 1 ? t[1] : 0; q.z = left > 2 ? t[2] : 0; q.w = 0;
            }
            L.payload[wv][i] = q;
        }
        decode_rows<FAST, LV2, true, DT>(reinterpret_cast<const u32*>(L.payload[wv]) + k0, nwords, o, lane_bits,
                                         w_ref, n, c, L, P1, P2, K, raise);
    } else {
        decode_rows<FAST, LV2, false, DT>(gw, nwords, o, lane_bits, w_ref, n, c, L, P1, P2, K, raise);
    }
}

template <int DT>
__global__ __launch_bounds__(256) void k_decode(const uint8_t* __restrict__ blob, void* __restrict__ w_ref, u64 n,
                                                Workspace* ws, u32 nchunks, int aligned, u64 epoch, HostResult* host) {
    __shared__ DecLds L;
    // if the check kernel found something, touch nothing
    if ((__hip_atomic_load(&ws->dec_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 8) != epoch) {
        const u32 t = threadIdx.x;
        const DecSet& D = ws->dec_set[0];
        const u32 M = D.info.max_len, K = D.info.K;
        const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits, P2 = M < kDecLut2Bits ? M : kDecLut2Bits;
        const u64 area = D.info.area;
        if (t < (1u << P1)) L.lut1[t] = D.lut1[t];
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
            L.rep[t] = __uint_as_float(t < K ? D.info.rep_bits[t] : 0x80000000u);
            L.len[t] = D.info.len[t]; L.code[t] = D.info.code[t];
        }
        __syncthreads();
        const u32 wave = t >> 6;
        auto raise = [&](u32 code) { raise_status(ws, host, epoch, code); };
        for (u32 c = blockIdx.x * 4 + wave; c < nchunks; c += gridDim.x * 4) {
            const bool full = (u64)(c + 1) * kChunk <= n;
            if (full && aligned) {
                if (M > kDecLut1Bits) decode_chunk<true, true, DT>(blob, w_ref, n, c, L, P1, P2, K, area, raise);
                else decode_chunk<true, false, DT>(blob, w_ref, n, c, L, P1, P2, K, area, raise);
            } else {
                decode_chunk<false, true, DT>(blob, w_ref, n, c, L, P1, P2, K, area, raise);
            }
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
        const bool head_ok = sound && hn == sg.n && hdr[15] == (u32)kF32 && hdr[9] == sg.nchunks && total >= area &&
                             total <= max_total && ((total - area) & 3) == 0;
        bool ok = head_ok;
        u32 status = 0;
        if (!head_ok) status = (sound && (hn != sg.n || hdr[15] != (u32)kF32)) ? 1u : 4u;
        else if (!dec_symbol_table(hdr, sg.n, sg.nchunks, area, (total - area) / 4, D, s_len, s_code)) { ok = false; status = 4u; }
        if (!ok) { atomicMax(&a.seg_status[sidx], status); D.info.area = 0; D.info.total_words = 0; D.info.max_len = 0; D.info.K = 0; }
        D.info.pad[0] = ok ? 1u : 0u;                        // the chunk checks and the sweep look here first
        D.info.pad[1] = 0;
        s_ok = ok;
    }
    __syncthreads();
    if (s_ok) dec_build_luts(D, s_len, s_code, t, 256);
}

__global__ __launch_bounds__(256) void kb_dec_chunks(BatchDecArgs a) {
    const u32 g = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (g >= a.total_chunks) return;
    const u32 sidx = a.seg_of_chunk[g];
    const SegD& sg = a.segs[sidx];
    const DecInfo& I = a.sets[sidx].info;
    if (!I.pad[0]) return;
    if (!dec_chunk_ok(sg.blob, I.area, I.total_words, sg.nchunks, g - sg.chunk0) && lane_id() == 0) atomicMax(&a.seg_status[sidx], 4u);
}

__global__ __launch_bounds__(64) void kb_decode(BatchDecArgs a) {
    __shared__ DecLdsT<1> L;
    const u32 lane = threadIdx.x;
    u32 active = 0xFFFFFFFFu, M = 0, K = 0, P1 = 0, P2 = 0;
    u64 area = 0;
    for (u32 g = blockIdx.x; g < a.total_chunks; g += gridDim.x) {
        const u32 sidx = __builtin_amdgcn_readfirstlane(a.seg_of_chunk[g]);
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
        const u32 c = g - sg.chunk0;
        const bool full = (u64)(c + 1) * kChunk <= sg.n;
        if (full && sg.aligned) {
            if (M > kDecLut1Bits) decode_chunk<true, true, kF32>(sg.blob, sg.w_ref, sg.n, c, L, P1, P2, K, area, raise);
            else decode_chunk<true, false, kF32>(sg.blob, sg.w_ref, sg.n, c, L, P1, P2, K, area, raise);
        } else {
            decode_chunk<false, true, kF32>(sg.blob, sg.w_ref, sg.n, c, L, P1, P2, K, area, raise);
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

// ----------------------------------------------------------------------------- k_decode_many
// Restore from several checkpoints in one sweep (Section 3, C1: u_t = u_0 + sum of the decoded
// deltas; Section 3.2, checkpoint merging): up to kMaxMany blobs of the same n are decoded side
// by side and their values added to w_ref in blob order, one fp32 add per blob and element, so
// the result equals that of applying the blobs one call after the other, with one read and
// one write of w_ref instead of one per blob.  Lane strings are read straight from memory.
struct ManyLds {
    uint8_t lut1[kMaxMany][1u << kDecLut1Bits];
    uint8_t lut2[kMaxMany][1u << kDecLut2Bits];
    float rep[kMaxMany][kMaxSym];
    u32 len[kMaxMany][kMaxSym], code[kMaxMany][kMaxSym];
    u32 K[kMaxMany], P1[kMaxMany], P2[kMaxMany];
    u64 area[kMaxMany];
};

__device__ __noinline__ u32 decode_long_many(const ManyLds& L, u32 t, u64 win) {
    const u32 peek = (u32)(win >> (64 - 15)), K = L.K[t];
    for (u32 j = 0; j <= K; ++j) {
        const u32 l = L.len[t][j];
        if (l > kDecLut2Bits && (peek >> (15 - l)) == L.code[t][j]) return j | (l << 4);
    }
    return K;
}

template <bool FAST>
__device__ __forceinline__ void decode_many_chunk(const BlobList& blobs, u32 first, u32 T, float* __restrict__ w_ref, u64 n,
                                                  Workspace* ws, HostResult* host, u32 c, const ManyLds& L, u64 epoch) {
    const u32 lane = lane_id();
    BitReader<false> br[kMaxMany];
    u32 wi0[kMaxMany], avail0[kMaxMany], lane_bits[kMaxMany];
#pragma unroll
    for (int t = 0; t < kMaxMany; ++t) {
        if ((u32)t < T) {
            const uint8_t* blob = blobs.p[first + t];
            const u32* off_tab = reinterpret_cast<const u32*>(blob + kHeaderBytes);
            const u32 o0 = off_tab[c], o1 = off_tab[c + 1];
            const uint8_t* rec = blob + L.area[t] + 4 * (u64)o0;
            lane_bits[t] = reinterpret_cast<const uint16_t*>(rec)[lane];
            const u32 o = wave_incl_scan(lane_bits[t]) - lane_bits[t];
            br[t].start(reinterpret_cast<const u32*>(rec + 2 * kW), o1 - o0 - kLaneBitsWords, o);
            wi0[t] = br[t].wi; avail0[t] = br[t].avail;
        }
    }
    const u64 base = (u64)c * kChunk;
#pragma unroll 2
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        if (!FAST && idx >= n) break;
        float x[4];
        load_row<FAST>(w_ref, idx, n, x);
        u32 kept = 0;
#pragma unroll
        for (int t = 0; t < kMaxMany; ++t) {
            if ((u32)t < T) {
                const u32 shr1 = 64 - L.P1[t], shr2 = 64 - L.P2[t], K = L.K[t];
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    if (FAST || idx + v < n) {
                        u32 e = L.lut1[t][(u32)(br[t].win >> shr1)];
                        if (e == 0xFF) {
                            e = L.lut2[t][(u32)(br[t].win >> shr2)];
                            if (e == 0xFF) e = decode_long_many(L, t, br[t].win);
                        }
                        const u32 len = e >> 4, sy = e & 15;
                        br[t].win <<= len; br[t].avail -= len;
                        kept |= K - sy;
                        x[v] = __fadd_rn(x[v], L.rep[t][sy]);
                    }
                    if ((v & 1) && br[t].avail <= 32) br[t].refill();
                }
            }
        }
        if (FAST) {
            if (__any(kept != 0)) *reinterpret_cast<float4*>(w_ref + idx) = make_float4(x[0], x[1], x[2], x[3]);
        } else {
#pragma unroll
            for (int v = 0; v < 4; ++v) if (idx + v < n) w_ref[idx + v] = x[v];
        }
    }
    bool bad = false;
#pragma unroll
    for (int t = 0; t < kMaxMany; ++t)
        if ((u32)t < T) bad = bad || (avail0[t] + 32 * (br[t].wi - wi0[t]) - br[t].avail != lane_bits[t]);
    if (__any(bad) && lane == 0) raise_status(ws, host, epoch, 4u);
}

__global__ __launch_bounds__(256) void k_decode_many(BlobList blobs, u32 first, u32 T, float* __restrict__ w_ref, u64 n,
                                                     Workspace* ws, u32 nchunks, int aligned, u64 epoch, HostResult* host) {
    __shared__ ManyLds L;
    // if a check found something, touch nothing
    if ((__hip_atomic_load(&ws->dec_status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) >> 8) != epoch) {
        const u32 tid = threadIdx.x;
        for (u32 t = 0; t < T; ++t) {
            const DecSet& D = ws->dec_set[first + t];
            const u32 M = D.info.max_len, K = D.info.K;
            const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits, P2 = M < kDecLut2Bits ? M : kDecLut2Bits;
            if (tid < (1u << P1)) L.lut1[t][tid] = D.lut1[tid];
            if (M > kDecLut1Bits) for (u32 i = tid; i < (1u << P2); i += 256) L.lut2[t][i] = D.lut2[i];
            if (tid < kMaxSym) {
                L.rep[t][tid] = __uint_as_float(tid < K ? D.info.rep_bits[tid] : 0x80000000u);
                L.len[t][tid] = D.info.len[tid]; L.code[t][tid] = D.info.code[tid];
            }
            if (tid == 0) { L.K[t] = K; L.P1[t] = P1; L.P2[t] = P2; L.area[t] = D.info.area; }
        }
        __syncthreads();
        const u32 wave = tid >> 6;
        for (u32 c = blockIdx.x * 4 + wave; c < nchunks; c += gridDim.x * 4) {
            const bool full = (u64)(c + 1) * kChunk <= n;
            if (full && aligned) decode_many_chunk<true>(blobs, first, T, w_ref, n, ws, host, c, L, epoch);
            else decode_many_chunk<false>(blobs, first, T, w_ref, n, ws, host, c, L, epoch);
        }
    }
}

// ----------------------------------------------------------------------------- k_decode_fused
// The same restore for blobs whose codes are all at most 7 bits long (always the case for
// nbits <= 3), built for throughput.  T is a compile-time constant, so the T bit strings of a
// lane are T independent dependency chains that the scheduler interleaves.  One wavefront per
// workgroup; the payloads of a chunk (all T blobs) are staged in the workgroup's LDS area with
// coalesced loads (the host sizes the area to the blobs, which also sets how many wavefronts
// share a compute unit).  A row's 4 codes of one blob take at most 28 bits, so each blob's 32-bit
// window is re-read once per row from the bit position alone, without a branch.  Both look-up
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
    u32 pad[3];
    u32 before_pay;                              // the word in front of the payload area (read, never used)
};
constexpr u32 kFusedSlack = 64;                  // words behind the payloads that a damaged lane string may run into:
                                                 // 256 codes of at most 7 bits past a start that validation bounds

// Bit positions are kept as p = 31 + bits from the start of the payload area (staged) or of the
// blob's payload (from memory): the window is then the low 32 bits of {word[(p >> 5) - 1],
// word[p >> 5]} >> (~p & 31), which is one v_alignbit.
template <int T, bool FAST, bool STAGED>
__device__ __forceinline__ void fused_row(const FusedHead<T>& H, const u32* pay, u32 pay_words, const u32* const (&gw)[T],
                                          const u32 (&nw)[T], u32 (&pos)[T], float* __restrict__ w_ref, u64 n, u64 idx,
                                          float (&x)[4]) {
    // Written step by step across the blobs (all windows, then the first code of every blob, ...), so
    // that the T look-ups of a step are in flight together.
    u32 win[T], rep[4][T];
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
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        if (FAST || idx + v < n) {
            u32 e[T];
#pragma unroll
            for (int t = 0; t < T; ++t) {
                e[t] = H.lut[t][win[t] >> (32 - kDecLut1Bits)];
                asm("" : "+v"(e[t]));                 // keep e a 32-bit value (no 16-bit shift plus re-extension)
            }
#pragma unroll
            for (int t = 0; t < T; ++t) {
                const u32 len = e[t] >> 6;
                rep[v][t] = *reinterpret_cast<const u32*>(reinterpret_cast<const uint8_t*>(H.rep[t]) + e[t]);
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
                for (int t = 0; t < T; ++t) x[v] = __fadd_rn(x[v], __uint_as_float(rep[v][t]));   // in blob order
            *reinterpret_cast<float4*>(w_ref + idx) = make_float4(x[0], x[1], x[2], x[3]);
        }
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (idx + v < n) {
#pragma unroll
                for (int t = 0; t < T; ++t) x[v] = __fadd_rn(x[v], __uint_as_float(rep[v][t]));
                w_ref[idx + v] = x[v];
            }
        }
    }
}

// All rows of a full, aligned chunk with staged payloads: w_ref is read PF rows ahead in two
// alternating register batches, so the reads of the next rows are in flight while these decode.
template <int T>
__device__ __forceinline__ void fused_rows_fast(const FusedHead<T>& H, const u32* pay, u32 pay_words, const u32* const (&gw)[T],
                                                const u32 (&nw)[T], u32 (&pos)[T], float* __restrict__ w_ref, u64 n, u32 c) {
    constexpr int PF = 4;
    const u32 lane = lane_id();
    float4* rows = reinterpret_cast<float4*>(w_ref + (u64)c * kChunk) + lane;
    const u64 base = (u64)c * kChunk + lane * kV;
    float4 A[PF], B[PF];
#pragma unroll
    for (int k = 0; k < PF; ++k) A[k] = load_stream(rows + k * kW);
    auto batch = [&](float4 (&X)[PF], u32 r0) {
#pragma unroll
        for (int k = 0; k < PF; ++k) {
            float x[4] = {X[k].x, X[k].y, X[k].z, X[k].w};
            fused_row<T, true, true>(H, pay, pay_words, gw, nw, pos, w_ref, n, base + (u64)(r0 + k) * kRowElems, x);
        }
    };
    for (u32 r0 = 0; r0 < kR; r0 += 2 * PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) B[k] = load_stream(rows + (r0 + PF + k) * kW);
        batch(A, r0);
        if (r0 + 2 * PF < kR) {
#pragma unroll
            for (int k = 0; k < PF; ++k) A[k] = load_stream(rows + (r0 + 2 * PF + k) * kW);
        }
        batch(B, r0 + PF);
    }
}

// Any chunk (ragged, unaligned, or payloads read from memory), row by row.
template <int T, bool FAST>
__device__ __forceinline__ void fused_rows_plain(const FusedHead<T>& H, const u32* const (&gw)[T], const u32 (&nw)[T], u32 (&pos)[T],
                                              float* __restrict__ w_ref, u64 n, u32 c) {
    const u32 lane = lane_id();
    const u64 base = (u64)c * kChunk;
    for (u32 r = 0; r < kR; ++r) {
        const u64 idx = base + (u64)r * kRowElems + lane * kV;
        if (!FAST && idx >= n) break;
        float x[4];
        load_row<FAST>(w_ref, idx, n, x);
        fused_row<T, FAST, false>(H, nullptr, 0, gw, nw, pos, w_ref, n, idx, x);
    }
}

template <typename P>
__device__ __forceinline__ P* uniform_ptr(P* p) {        // a pointer every lane holds alike, moved to scalar registers
    const u64 v = reinterpret_cast<u64>(p);
    const u32 lo = __builtin_amdgcn_readfirstlane((u32)v), hi = __builtin_amdgcn_readfirstlane((u32)(v >> 32));
    return reinterpret_cast<P*>(((u64)hi << 32) | lo);
}

template <int T, bool FAST>
__device__ __forceinline__ void fused_chunk(const FusedHead<T>& H, u32* pay, u32 pay_words, float* __restrict__ w_ref, u64 n,
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
                const u32 nvec = (nw[t] + k0[t] + 3) >> 2;
#pragma unroll
                for (int k = 0; k < CV; ++k) {
                    const u32 i = i0 + k * kW + lane;
                    if (i < nvec) dst[i] = q[t][k];
                }
            }
        }
    }
#pragma unroll
    for (int t = 0; t < T; ++t) start[t] = 31 + wave_incl_scan(lane_bits[t]) - lane_bits[t];
    if (staged) {
#pragma unroll
        for (int t = 0; t < T; ++t) { start[t] += 32 * (wbase[t] + k0[t]); pos[t] = start[t]; }
        fused_rows_fast<T>(H, pay, pay_words, gw, nw, pos, w_ref, n, c);
    } else {
#pragma unroll
        for (int t = 0; t < T; ++t) pos[t] = start[t];
        fused_rows_plain<T, FAST>(H, gw, nw, pos, w_ref, n, c);
    }
    bool bad = false;
#pragma unroll
    for (int t = 0; t < T; ++t) bad = bad || (pos[t] - start[t] != lane_bits[t]);
    if (__any(bad) && lane == 0) raise_status(ws, host, epoch, 4u);
}

template <int T>
__global__ __launch_bounds__(64) void k_decode_fused(BlobList blobs, u32 first, float* __restrict__ w_ref, u64 n,
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
        const u32 M = D.info.max_len, K = D.info.K;       // M <= 7: e < 128
        const u32 P1 = M < kDecLut1Bits ? M : kDecLut1Bits;
        for (u32 i = tid; i < (1u << kDecLut1Bits); i += kW) {
            const u32 e = D.lut1[i >> (kDecLut1Bits - P1)];
            H.lut[t][i] = (uint16_t)(e << 2);
            H.rep[t][i] = (i & 15) < K ? D.info.rep_bits[i & 15] : 0x80000000u;
        }
        if (tid == 0) {
            const uint8_t* blob = blobs.p[first + t];
            H.rec_base[t] = blob + D.info.area;
            H.off_tab[t] = reinterpret_cast<const u32*>(blob + kHeaderBytes);
        }
    }
    if (tid == 0) H.before_pay = 0;
    __syncthreads();
    for (u32 c = blockIdx.x; c < nchunks; c += gridDim.x) {
        const bool full = (u64)(c + 1) * kChunk <= n;
        if (full && aligned) fused_chunk<T, true>(H, pay, pay_words, w_ref, n, ws, host, c, nchunks, epoch);
        else fused_chunk<T, false>(H, pay, pay_words, w_ref, n, ws, host, c, nchunks, epoch);
    }
}

// ----------------------------------------------------------------------------- launchers
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

void launch_reset(Workspace* ws, uint32_t* group_words, hipStream_t s) {
    hipLaunchKernelGGL(k_reset, dim3(1), dim3(256), 0, s, ws, group_words, (u32)kMaxGroups);
}

static inline bool aligned_rows(const void* p, int dtype) {     // 4 consecutive elements per access
    return (reinterpret_cast<uintptr_t>(p) & (dtype == kF32 ? 15 : 7)) == 0;
}

template <int DT>
static void launch_hist_t(const void* w, const void* w_ref, uint64_t n, Workspace* ws, u32 blocks, u32 threads, hipStream_t s) {
    if (aligned16(w) && aligned16(w_ref)) hipLaunchKernelGGL((k_hist<true, DT>), dim3(blocks), dim3(threads), 0, s, w, w_ref, (u64)n, ws);
    else hipLaunchKernelGGL((k_hist<false, DT>), dim3(blocks), dim3(threads), 0, s, w, w_ref, (u64)n, ws);
}

void launch_hist(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, const Tuning& tune, hipStream_t s) {
    if (n == 0) return;
    const u32 threads = tune.hist_threads;
    const u64 units = n / (dtype == kF32 ? 4 : 8);                 // 16-byte units
    u64 blocks = (units + 4 * threads - 1) / (4 * threads);
    const u64 cap = (u64)tune.num_cu * tune.hist_blocks_per_cu;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    if (dtype == kBF16) launch_hist_t<kBF16>(w, w_ref, n, ws, (u32)blocks, threads, s);
    else if (dtype == kF16) launch_hist_t<kF16>(w, w_ref, n, ws, (u32)blocks, threads, s);
    else launch_hist_t<kF32>(w, w_ref, n, ws, (u32)blocks, threads, s);
}

void launch_table(Workspace* ws, uint64_t n, int nbits, uint32_t* group_words, hipStream_t s) {
    hipLaunchKernelGGL(k_table, dim3(1), dim3(64), 0, s, ws, (u64)n, nbits, group_words, (u32)((num_chunks_of(n) + 63) / 64));
}

void launch_spec_table(Workspace* ws, const TableCache* cache, int nbits, hipStream_t s) {
    hipLaunchKernelGGL(k_spec_table, dim3(1), dim3(64), 0, s, ws, cache, nbits);
}

void launch_spec_sweep(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                       uint32_t* group_words, uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (u64)tune.num_cu * tune.pack_waves_per_cu;
    if (blocks > nchunks) blocks = nchunks;
    const int al = aligned_rows(w, dtype) && aligned_rows(w_ref, dtype);
    const dim3 grid((u32)blocks), wg(64);
    if (dtype == kBF16) hipLaunchKernelGGL(k_spec_sweep<kBF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else if (dtype == kF16) hipLaunchKernelGGL(k_spec_sweep<kF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else hipLaunchKernelGGL(k_spec_sweep<kF32>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
}

void launch_pack(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                 uint32_t* group_words, uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (u64)tune.num_cu * tune.pack_waves_per_cu;
    if (blocks > nchunks) blocks = nchunks;
    const int al = aligned_rows(w, dtype) && aligned_rows(w_ref, dtype);
    const dim3 grid((u32)blocks), wg(64);
    if (dtype == kBF16) hipLaunchKernelGGL(k_pack<kBF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else if (dtype == kF16) hipLaunchKernelGGL(k_pack<kF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else hipLaunchKernelGGL(k_pack<kF32>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
}

void launch_place(uint8_t* out, Workspace* ws, const uint32_t* chunk_bits, const uint32_t* group_words,
                  const uint32_t* prov, uint32_t slot_words, uint64_t n, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    hipLaunchKernelGGL(k_place, dim3((u32)((nchunks + 3) / 4)), dim3(256), 0, s, out, ws, chunk_bits, group_words, prov,
                       slot_words, (u32)nchunks);
}

void launch_finalize(uint8_t* out, Workspace* ws, Result* host_result, uint32_t* group_words, TableCache* cache,
                     uint64_t n, int nbits, int dtype, hipStream_t s) {
    hipLaunchKernelGGL(k_finalize, dim3(1), dim3(256), 0, s, out, ws, host_result, group_words, cache, (u64)n, nbits,
                       (u32)num_chunks_of(n), (u32)dtype);
}

void launch_batch_encode(const BatchArgs& a, const Tuning& tune, hipStream_t s) {
    const u32 cap = (u32)tune.num_cu * 8;
    u32 setup_blocks = (a.total_chunks + 255) / 256;
    if (setup_blocks < a.count * 3) setup_blocks = a.count * 3;
    if (setup_blocks > cap) setup_blocks = cap;
    if (setup_blocks < 1) setup_blocks = 1;
    hipLaunchKernelGGL(kb_setup, dim3(setup_blocks), dim3(256), 0, s, a);
    if (a.total_chunks) {
        u32 waves = (u32)tune.num_cu * (u32)tune.pack_waves_per_cu;
        if (waves > a.total_chunks) waves = a.total_chunks;
        hipLaunchKernelGGL(kb_hist, dim3(waves), dim3(64), 0, s, a);
    }
    hipLaunchKernelGGL(kb_table, dim3(a.count), dim3(64), 0, s, a);
    if (a.total_chunks) {
        u32 waves = (u32)tune.num_cu * (u32)tune.pack_waves_per_cu;
        if (waves > a.total_chunks) waves = a.total_chunks;
        hipLaunchKernelGGL(kb_pack, dim3(waves), dim3(64), 0, s, a);
        hipLaunchKernelGGL(kb_place, dim3((a.total_chunks + 3) / 4), dim3(256), 0, s, a);
    }
    hipLaunchKernelGGL(kb_finalize, dim3(a.count), dim3(256), 0, s, a);
}

void launch_batch_decode(const BatchDecArgs& a, const Tuning& tune, hipStream_t s) {
    const u32 cap = (u32)tune.num_cu * 8;
    u32 setup_blocks = (a.total_chunks + 255) / 256;
    if (setup_blocks > cap) setup_blocks = cap;
    if (setup_blocks < 1) setup_blocks = 1;
    hipLaunchKernelGGL(kb_dec_setup, dim3(setup_blocks), dim3(256), 0, s, a);
    hipLaunchKernelGGL(kb_dec_tables, dim3(a.count), dim3(256), 0, s, a);
    if (a.total_chunks) {
        hipLaunchKernelGGL(kb_dec_chunks, dim3((a.total_chunks + 3) / 4), dim3(256), 0, s, a);
        u32 waves = (u32)tune.num_cu * (u32)tune.decode_blocks_per_cu * 4u;
        if (waves > a.total_chunks) waves = a.total_chunks;
        hipLaunchKernelGGL(kb_decode, dim3(waves), dim3(64), 0, s, a);
    }
    hipLaunchKernelGGL(kb_dec_report, dim3((a.count + 255) / 256), dim3(256), 0, s, a);
}

void launch_dec_check(const BlobList& blobs, int first, int count, uint64_t n, int dtype, uint64_t max_total, Workspace* ws,
                      uint64_t epoch, HostResult* host, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    const u64 blocks = nchunks ? (nchunks + 3) / 4 : 1;
    hipLaunchKernelGGL(k_dec_check, dim3((u32)blocks, (u32)count), dim3(256), 0, s, blobs, (u32)first, (u64)n, (u64)max_total,
                       ws, (u32)nchunks, (u64)epoch, host, (u32)dtype);
}

void launch_decode_many(const BlobList& blobs, int first, int count, float* w_ref, uint64_t n, Workspace* ws,
                        uint64_t epoch, HostResult* host, const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (nchunks + 3) / 4;
    const u64 cap = (u64)tune.num_cu * tune.many_blocks_per_cu;
    if (blocks > cap) blocks = cap;
    hipLaunchKernelGGL(k_decode_many, dim3((u32)blocks), dim3(256), 0, s, blobs, (u32)first, (u32)count, w_ref, (u64)n, ws,
                       (u32)nchunks, (int)aligned16(w_ref), (u64)epoch, host);
}


template <int T>
static void launch_fused_t(const BlobList& blobs, int first, float* w_ref, uint64_t n, Workspace* ws, uint64_t epoch,
                           HostResult* host, u32 blocks, u32 pay_words, hipStream_t s) {
    hipLaunchKernelGGL(k_decode_fused<T>, dim3(blocks), dim3(64), 4 * (size_t)(pay_words + kFusedSlack), s, blobs, (u32)first, w_ref,
                       (u64)n, ws, (u32)num_chunks_of(n), (int)aligned16(w_ref), (u64)epoch, host, pay_words);
}

size_t fused_lds_bytes(int count, uint32_t pay_words) {
    static const size_t head[kMaxMany] = {sizeof(FusedHead<1>), sizeof(FusedHead<2>), sizeof(FusedHead<3>), sizeof(FusedHead<4>),
                                          sizeof(FusedHead<5>), sizeof(FusedHead<6>), sizeof(FusedHead<7>), sizeof(FusedHead<8>)};
    return head[count - 1] + 4 * (size_t)(pay_words + kFusedSlack);
}

void launch_decode_fused(const BlobList& blobs, int first, int count, float* w_ref, uint64_t n, Workspace* ws,
                         uint64_t epoch, HostResult* host, uint32_t pay_words, const Tuning& tune, hipStream_t s) {
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
        case 1: launch_fused_t<1>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 2: launch_fused_t<2>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 3: launch_fused_t<3>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 4: launch_fused_t<4>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 5: launch_fused_t<5>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 6: launch_fused_t<6>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        case 7: launch_fused_t<7>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
        default: launch_fused_t<8>(blobs, first, w_ref, n, ws, epoch, host, b, pay_words, s); break;
    }
}

void launch_decode(const uint8_t* blob, void* w_ref, uint64_t n, int dtype, Workspace* ws, uint64_t epoch, HostResult* host,
                   const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    u64 blocks = (nchunks + 3) / 4;
    const u64 cap = (u64)tune.num_cu * tune.decode_blocks_per_cu;
    if (blocks > cap) blocks = cap;
    const dim3 grid((u32)blocks), wg(256);
    const int al = aligned_rows(w_ref, dtype);
    if (dtype == kBF16) hipLaunchKernelGGL(k_decode<kBF16>, grid, wg, 0, s, blob, w_ref, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host);
    else if (dtype == kF16) hipLaunchKernelGGL(k_decode<kF16>, grid, wg, 0, s, blob, w_ref, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host);
    else hipLaunchKernelGGL(k_decode<kF32>, grid, wg, 0, s, blob, w_ref, (u64)n, ws, (u32)nchunks, al, (u64)epoch, host);
}

}  // namespace lc
