// Encode kernels of the LC-Checkpoint compress / restore path for gfx950 (wave64).
//
// lc_encode:         k_hist -> k_table -> k_pack -> k_place (whose first workgroup writes the header) (which also clears the scratch
//                    state for the next call, k_place the per-chunk maxima); k_reset only for a fresh scratch area
//                    (fp64 parameters: k_hist64 -> k_table<11> -> k_pack64 -> k_place)
// lc_encode_cached:  k_spec_table -> k_spec_sweep -> k_table -> k_pack (nothing to do on a hit) -> k_place
// lc_encode_batch:   kb_setup -> kb_hist -> kb_table -> kb_list -> kb_pack -> kb_place (whose first workgroups write the headers)
//
// The paper (arXiv 2009.13003) defines what is computed: delta against the last
// recovered state (Algorithm 1 line 4), (sign, exponent) buckets represented by the
// mean of their extremes and x-bit priority promotion (Section 3.1.1), Huffman
// coding of the bucket indices (Section 3.1.2).  How it is laid out on the GPU is this library's own.
#include "lc_device.h"
#include <type_traits>

namespace lc {

// ----------------------------------------------------------------------------- k_reset
// Brings the scratch state to what every encode call expects to find (and leaves behind):
// zero bucket counts, empty extremes, zero group sums and per-chunk exponent maxima.  Only launched
// for a fresh scratch area or after a call that did not run to its end.
__device__ __forceinline__ void clear_extremes(EncState* ws, u32 tid, u32 nthr) {
    u32* mn = &ws->mmin[0][0]; u32* mx = &ws->mmax[0][0];            // all copies
    for (u32 i = tid; i < kExtCopies * kMaxSym; i += nthr) { mn[i] = 0x7FFFFFu; mx[i] = 0; }
}

__device__ __forceinline__ void clear_encode_state(EncState* ws, u32* group_words, u32 ngroups, u32 tid, u32 nthr) {
    for (u32 i = tid; i < ngroups; i += nthr) group_words[i] = 0;
    for (u32 i = tid; i < 512; i += nthr) ws->hist[i] = 0;
    clear_extremes(ws, tid, nthr);
    if (tid == 0) { ws->spec = 0; ws->spec_ok = 0; ws->list_count = 0; }
}

__device__ __forceinline__ void clear_ext64(Ext64* ext, u32 tid, u32 nthr) {
    for (u32 i = tid; i < kBuckets64; i += nthr) ext->hist[i] = 0;
    if (tid < kMaxSym) { ext->mmin[tid] = 0xFFFFFFFFFFFFFull; ext->mmax[tid] = 0; }
}

__device__ __forceinline__ void clear_bucket_extremes(Workspace* ws, u32 tid, u32 nthr) {
    for (u32 i = tid; i < 512; i += nthr) { ws->bucket_min[i] = 0xFFFFFFFFu; ws->bucket_max[i] = 0; }
}

__global__ void k_reset(Workspace* ws, u32* group_words, u32 ngroups, u32* chunk_maxexp, u32 nchunks) {
    clear_encode_state(ws, group_words, ngroups, threadIdx.x, blockDim.x);
    clear_ext64(&ws->ext64, threadIdx.x, blockDim.x);
    clear_bucket_extremes(ws, threadIdx.x, blockDim.x);
    for (u32 i = threadIdx.x; i < nchunks; i += blockDim.x) chunk_maxexp[i] = 0;
}

// The same for a scratch area that only ever serves calls of at most `nchunks` chunks (their entries of the
// transposed maxima, their groups of 64 chunks): what such an area needs cleared before every call of its own.
__global__ void k_reset_chunks(EncState* ws, u32* group_words, u32 ngroups, u32* chunk_maxexp, u32 nchunks) {
    clear_encode_state(ws, group_words, ngroups, threadIdx.x, blockDim.x);
    for (u32 c = threadIdx.x; c < nchunks; c += blockDim.x) chunk_maxexp[maxexp_slot(c)] = 0;
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

// Largest magnitude among the EPU deltas of one unit and m (its exponent field is the largest biased exponent).
// A NaN may drop out of a floating-point maximum: a vector with such a delta is not coded at all
// (the table's status says so), and nobody looks at the chunk maxima then.
template <int EPU>
__device__ __forceinline__ float max_magnitude(const u32 (&u)[EPU], float m) {
#pragma unroll
    for (int v = 0; v < EPU; ++v) m = fmaxf(m, fabsf(__uint_as_float(u[v])));
    return m;
}

// Every wavefront takes batches of PF consecutive rows of 64 units (PF KiB of each array), so a batch lies in
// one chunk of the coding sweep and its largest exponent goes to chunk_maxexp with one atomic per batch.
// batch_max (or null) receives every whole batch's largest exponent as a byte of its own: the coding sweep then
// knows which parts of a chunk it has to read.
// A wavefront keeps the maxima of its last 64 batches in LDS and writes them out 64 at a time, one per lane: a
// global write after every batch, however small, holds back the loads issued behind it (both are counted, in
// order, by the one vector-memory counter) and cost the sweep 4 % of its rate.
// KEYS (binary32, aligned arrays): the sweep also stages a 9-bit key per element of every whole batch -- the 16
// exponent bytes and the 16 sign bits of the 16 elements a lane holds of a batch, which are the lane's own elements of
// 4 rows of the coding sweep's chunk -- and, being then the only sweep that sees the mantissas, tracks the smallest and
// largest delta bit pattern of every bucket (Section 3.1.1: the representative is the mean of these two).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
template <bool ALIGNED, int DT, bool KEYS = false>
__global__ __launch_bounds__(1024) void k_hist(const void* __restrict__ w, const void* __restrict__ w_ref,
                                               u64 n, Workspace* ws, u32* chunk_maxexp, uint8_t* batch_max, KeyPlanes keys) {
    __shared__ u32 h[512 * kHistCopies];
    __shared__ u32 mn[KEYS ? 512 * kHistCopies : 1], mx[KEYS ? 512 * kHistCopies : 1];
    __shared__ uint16_t pend[1024 / kW][kW];         // per wavefront: the maxima of its batches not yet written out
    static_assert(!KEYS || (ALIGNED && DT == kF32), "keys are staged for aligned binary32 arrays only");
    constexpr int EPU = 16 / (int)elem_bytes<DT>();
    const u32 tid = threadIdx.x, nthr = blockDim.x;
    for (u32 i = tid; i < 512 * kHistCopies; i += nthr) { h[i] = 0; if (KEYS) { mn[i] = 0xFFFFFFFFu; mx[i] = 0; } }
    __syncthreads();
    const u32 copy = tid & (kHistCopies - 1);
    const u64 nu = n / EPU;
    // Batches of PF rows per wavefront, one batch in flight while the previous one is counted.
    constexpr int PF = 4;
    constexpr u32 kBatchUnits = PF * kW;
    static_assert(kChunk % (kBatchUnits * EPU) == 0, "a batch must not straddle two chunks");
    const u64 nbatch = nu / kBatchUnits;
    const u64 stride = (u64)gridDim.x * (nthr / kW);                    // wavefronts in the grid
    u64 b = (u64)blockIdx.x * (nthr / kW) + tid / kW;
    float4 a0[PF], b0[PF], a1[PF], b1[PF];
    auto fetch = [&](float4 (&a)[PF], float4 (&bb)[PF], u64 batch) {
        const u64 at = batch * kBatchUnits + (tid & (kW - 1));
#pragma unroll
        for (int k = 0; k < PF; ++k) { a[k] = load_unit<ALIGNED, DT, EPU>(w, at + k * kW); bb[k] = load_unit<ALIGNED, DT, EPU>(w_ref, at + k * kW); }
    };
    u32 pending = 0;                                 // maxima waiting in pend, those of batches pend_first, + stride, ...
    u64 pend_first = b;
    auto write_maxima = [&]() {
        __builtin_amdgcn_wave_barrier();
        const u32 lane = tid & (kW - 1);
        if (lane < pending) {
            const u64 batch = pend_first + (u64)lane * stride;
            const u32 m = pend[tid / kW][lane];
            atomicMax(&chunk_maxexp[maxexp_slot((u32)((batch * kBatchUnits * EPU) / kChunk))], m);
            if (batch_max) batch_max[batch] = (uint8_t)m;
        }
        __builtin_amdgcn_wave_barrier();
    };
    u32 key_word = 0, key_signs = 0;                 // KEYS: exponent bytes of the unit just counted; sign bits of the batch so far
    auto count_one = [&](u32 u) {
        const u32 at = (u >> 23) * kHistCopies + copy;
        atomicAdd(&h[at], 1u);
        if (KEYS) { atomicMin(&mn[at], u); atomicMax(&mx[at], u); }
    };
    auto count_unit = [&](const float4& a, const float4& bb, float m) {
        float x[EPU], y[EPU];
        u32 u[EPU];
        unpack_unit<DT, EPU>(a, x); unpack_unit<DT, EPU>(bb, y);
        key_word = 0;
#pragma unroll
        for (int v = 0; v < EPU; ++v) {
            u[v] = delta_bits(x[v], y[v]);
            count_one(u[v]);
            if (KEYS) { key_word |= ((u[v] >> 23) & 255u) << (8 * v); key_signs = (key_signs >> 1) | ((u[v] >> 31) << 15); }
        }
        return max_magnitude<EPU>(u, m);
    };
    auto count = [&](float4 (&a)[PF], float4 (&bb)[PF], u64 batch) {
        float mf = 0.f;
        u32 kw[PF];
#pragma unroll
        for (int k = 0; k < PF; ++k) { mf = count_unit(a[k], bb[k], mf); kw[k] = key_word; }
        if constexpr (KEYS) {
            // (after 16 elements the sign bit of element 4 k + v has arrived at bit 4 k + v)
            static_assert(PF == 4 && EPU == 4, "a batch is 4 rows of 4 elements per lane");
            const u32x4 kv = {kw[0], kw[1], kw[2], kw[3]};
            const u64 at = batch * kW + (tid & (kW - 1));
            __builtin_nontemporal_store(kv, reinterpret_cast<u32x4*>(keys.exp) + at);
            __builtin_nontemporal_store((uint16_t)key_signs, keys.sign + at);
        }
        const u32 m = wave_max_u32(__float_as_uint(mf));     // whole wavefronts only: b < nbatch is the same for all lanes
        if ((tid & (kW - 1)) == 0) pend[tid / kW][pending] = (uint16_t)(m >> 23);
        if (++pending == kW) { write_maxima(); pending = 0; pend_first = batch + stride; }
    };
    if (b < nbatch) {
        // The loads of the batch after next are issued without a branch around them (at the end the current
        // batch is simply read again): only then does the compiler wait for the older batch alone.
        fetch(a0, b0, b);
        while (true) {
            const bool more1 = b + stride < nbatch;
            fetch(a1, b1, more1 ? b + stride : b);
            count(a0, b0, b);
            if (!more1) break;
            b += stride;
            const bool more0 = b + stride < nbatch;
            fetch(a0, b0, more0 ? b + stride : b);
            count(a1, b1, b);
            if (!more0) break;
            b += stride;
        }
        write_maxima();
    }
    // what is left of the vector: fewer than one batch of units, then fewer than one unit of elements
    if (blockIdx.x == 0) {
        for (u64 u = nbatch * kBatchUnits + tid; u < nu; u += nthr) {
            const float mf = count_unit(load_unit<ALIGNED, DT, EPU>(w, u), load_unit<ALIGNED, DT, EPU>(w_ref, u), 0.f);
            atomicMax(&chunk_maxexp[maxexp_slot((u32)((u * EPU) / kChunk))], __float_as_uint(mf) >> 23);
        }
        if (tid < (u32)(n - EPU * nu)) {
            const u64 i = EPU * nu + tid;
            const u32 u = delta_bits(load_one<DT>(w, i), load_one<DT>(w_ref, i));
            count_one(u);
            atomicMax(&chunk_maxexp[maxexp_slot((u32)(i / kChunk))], (u >> 23) & 255u);
        }
    }
    __syncthreads();
    for (u32 bk = tid; bk < 512; bk += nthr) {
        u32 sum = 0, lo = 0xFFFFFFFFu, hi = 0;
#pragma unroll
        for (int k = 0; k < kHistCopies; ++k) {
            sum += h[bk * kHistCopies + k];
            if (KEYS) { lo = min(lo, mn[bk * kHistCopies + k]); hi = max(hi, mx[bk * kHistCopies + k]); }
        }
        if (sum) {
            atomicAdd(&ws->hist[bk], (u64)sum);
            if (KEYS) { atomicMin(&ws->bucket_min[bk], lo); atomicMax(&ws->bucket_max[bk], hi); }
        }
    }
}

// ----------------------------------------------------------------------------- k_hist64
// Sweep 1 for binary64 parameters: the same walk over the arrays (a 16-byte unit holds 2 elements, a batch of 4 rows
// 512), 2^12 buckets (sign and 11 exponent bits; Section 3.1.1, footnote on the bucket count) in 2 LDS copies,
// counts and chunk maxima of the binary64 delta.
constexpr int kHistCopies64 = 2;

template <bool ALIGNED>
__device__ __forceinline__ float4 load_unit64(const void* __restrict__ p, u64 unit) {
    if (ALIGNED) return load_stream(reinterpret_cast<const float4*>(p) + unit);
    const double* q = static_cast<const double*>(p) + unit * 2;
    const double a = q[0], b = q[1];
    return make_float4(__int_as_float(__double2loint(a)), __int_as_float(__double2hiint(a)),
                       __int_as_float(__double2loint(b)), __int_as_float(__double2hiint(b)));
}

template <bool ALIGNED>
__global__ __launch_bounds__(1024) void k_hist64(const void* __restrict__ w, const void* __restrict__ w_ref,
                                                 u64 n, Ext64* ext, u32* chunk_maxexp, uint16_t* part_max) {
    __shared__ u32 h[kBuckets64 * kHistCopies64];
    __shared__ uint16_t pend[1024 / kW][kW];         // as in k_hist: maxima written out 64 batches at a time
    constexpr int EPU = 2;
    const u32 tid = threadIdx.x, nthr = blockDim.x;
    for (u32 i = tid; i < kBuckets64 * kHistCopies64; i += nthr) h[i] = 0;
    __syncthreads();
    const u32 copy = tid & (kHistCopies64 - 1);
    const u64 nu = n / EPU;
    constexpr int PF = 4;
    constexpr u32 kBatchUnits = PF * kW;
    static_assert(kChunk % (kBatchUnits * EPU) == 0, "a batch must not straddle two chunks");
    const u64 nbatch = nu / kBatchUnits;
    const u64 stride = (u64)gridDim.x * (nthr / kW);
    u64 b = (u64)blockIdx.x * (nthr / kW) + tid / kW;
    float4 a0[PF], b0[PF], a1[PF], b1[PF];
    auto fetch = [&](float4 (&a)[PF], float4 (&bb)[PF], u64 batch) {
        const u64 at = batch * kBatchUnits + (tid & (kW - 1));
#pragma unroll
        for (int k = 0; k < PF; ++k) { a[k] = load_unit64<ALIGNED>(w, at + k * kW); bb[k] = load_unit64<ALIGNED>(w_ref, at + k * kW); }
    };
    u32 pending = 0;
    u64 pend_first = b;
    // (a batch is 4 KiB of each array: the largest exponent of every such part lets sweep 2 read a mostly merged
    // chunk part by part, as for the other element types; 11 exponent bits: two bytes each)
    auto write_maxima = [&]() {
        __builtin_amdgcn_wave_barrier();
        const u32 lane = tid & (kW - 1);
        if (lane < pending) {
            const u64 batch = pend_first + (u64)lane * stride;
            const u32 m = pend[tid / kW][lane];
            atomicMax(&chunk_maxexp[maxexp_slot((u32)((batch * kBatchUnits * EPU) / kChunk))], m);
            if (part_max) part_max[batch] = (uint16_t)m;
        }
        __builtin_amdgcn_wave_barrier();
    };
    auto as_double = [](float lo, float hi) { return __hiloint2double(__float_as_int(hi), __float_as_int(lo)); };
    auto count_one = [&](double x, double y, u32 m) {       // returns the larger of m and the delta's biased exponent
        const u64 u = delta_bits(x, y);
        atomicAdd(&h[bucket_of(u) * kHistCopies64 + copy], 1u);
        return max(m, bucket_of(u) & 2047u);
    };
    auto count_unit = [&](const float4& a, const float4& bb, u32 m) {
        m = count_one(as_double(a.x, a.y), as_double(bb.x, bb.y), m);
        return count_one(as_double(a.z, a.w), as_double(bb.z, bb.w), m);
    };
    auto count = [&](float4 (&a)[PF], float4 (&bb)[PF], u64 batch) {
        u32 m = 0;
#pragma unroll
        for (int k = 0; k < PF; ++k) m = count_unit(a[k], bb[k], m);
        m = wave_max_u32(m);
        if ((tid & (kW - 1)) == 0) pend[tid / kW][pending] = (uint16_t)m;
        if (++pending == kW) { write_maxima(); pending = 0; pend_first = batch + stride; }
    };
    if (b < nbatch) {
        fetch(a0, b0, b);
        while (true) {
            const bool more1 = b + stride < nbatch;
            fetch(a1, b1, more1 ? b + stride : b);
            count(a0, b0, b);
            if (!more1) break;
            b += stride;
            const bool more0 = b + stride < nbatch;
            fetch(a0, b0, more0 ? b + stride : b);
            count(a1, b1, b);
            if (!more0) break;
            b += stride;
        }
        write_maxima();
    }
    if (blockIdx.x == 0) {
        for (u64 u = nbatch * kBatchUnits + tid; u < nu; u += nthr) {
            const u32 m = count_unit(load_unit64<ALIGNED>(w, u), load_unit64<ALIGNED>(w_ref, u), 0);
            atomicMax(&chunk_maxexp[maxexp_slot((u32)((u * EPU) / kChunk))], m);
        }
        if (tid < (u32)(n - EPU * nu)) {
            const u64 i = EPU * nu + tid;
            const u32 m = count_one(static_cast<const double*>(w)[i], static_cast<const double*>(w_ref)[i], 0);
            atomicMax(&chunk_maxexp[maxexp_slot((u32)(i / kChunk))], m);
        }
    }
    __syncthreads();
    for (u32 bk = tid; bk < kBuckets64; bk += nthr) {
        const u32 sum = h[bk * kHistCopies64] + h[bk * kHistCopies64 + 1];
        if (sum) atomicAdd(&ext->hist[bk], (u64)sum);
    }
}

// ----------------------------------------------------------------------------- k_table
// Priority promotion (Section 3.1.1) and the Huffman table (Section 3.1.2), one wavefront.  Lane l looks at one exponent level (both signs) per step, from
// the largest exponent down; a ballot/popcount scan ranks the non-empty buckets (+ before - at
// equal exponent).  Lane 0 then builds the code lengths with two queues and the canonical codes
// with per-length counters.
template <int EB>                         // EB: exponent bits of the parameters' delta (8, or 11 for binary64)
struct TableLds {
    uint8_t sym[2u << EB];
    u64 cnt[kMaxSym + 1];
    u32 kept[kMaxSym], len[kMaxSym + 1];
};

// When the sweep before it coded speculatively with a cached table (ws->spec), the kernel also decides
// whether that stands: this checkpoint's kept set must be the cached one and exactly the symbols with a
// cached code must occur, in a coding of at most n * nbits payload bits.  If so the cached lengths are kept and the sweep's output is final (spec_ok);
// if not, the traces of the speculative coding are cleared and the table is this checkpoint's own.
// With chunk_list (and a workgroup of more than one wavefront) the other wavefronts meanwhile list the chunks
// that sweep 2 has to read: all but the full chunks whose largest exponent lies below every kept bucket.
template <int EB>
__device__ __forceinline__ void table_build(EncState* ws, Ext64* ext, u64 n, int nbits, u32* group_words, u32 ngroups,
                                            const u32* chunk_maxexp, u32* chunk_list) {
    __shared__ TableLds<EB> S;
    constexpr u32 kEmax = (1u << EB) - 1, kSteps = (1u << EB) / kW, kNeg = 1u << EB;
    const unsigned long long* hist = EB == 8 ? ws->hist : ext->hist;
    __shared__ u32 s_reuse, s_min_kept_exp, s_listed;
    const u32 lane = lane_id();
    const bool active = threadIdx.x < kW;
    const u32 kmax = (1u << nbits) - 1;
    // The groups' record sizes start from zero in every call: the last call's placement read them to its end, so they
    // are cleared here, ahead of the coding sweep that adds to them (a cached table's speculative coding has already
    // added to them: then k_spec_table has cleared them).
    if (group_words && !ws->spec) for (u32 i = threadIdx.x; i < ngroups; i += blockDim.x) group_words[i] = 0;
    if (active) for (u32 i = lane; i <= kMaxSym; i += kW) { S.cnt[i] = 0; S.len[i] = 0; if (i < kMaxSym) S.kept[i] = 0; }
    u32 total = 0;
    bool nonfinite = false, zero_class = false;
    // all counts of this lane first (8, or 64 for binary64), the ranking steps below then run without waiting on memory
    // (binary64, 32 steps with the loads inside the loop: 28 us for the kernel instead of 24)
    u64 cnt0[kSteps], cnt1[kSteps];
#pragma unroll
    for (u32 step = 0; step < kSteps; ++step) {
        cnt0[step] = active ? hist[kEmax - (step * kW + lane)] : 0;
        cnt1[step] = active ? hist[kNeg + kEmax - (step * kW + lane)] : 0;
    }
#pragma unroll
    for (u32 step = 0; step < kSteps; ++step) {
        if (!active) break;
        const u32 E = kEmax - (step * kW + lane);
        const u64 c0 = cnt0[step], c1 = cnt1[step];
        const bool normal = E >= 1 && E <= kEmax - 1;
        const bool cand0 = normal && c0 > 0, cand1 = normal && c1 > 0;
        const u64 m0 = __ballot(cand0), m1 = __ballot(cand1), lt = (1ull << lane) - 1;
        const u32 r0 = total + __popcll(m0 & lt) + __popcll(m1 & lt), r1 = r0 + (cand0 ? 1u : 0u);
        S.sym[E] = 0xFF; S.sym[kNeg + E] = 0xFF;
        if (cand0 && r0 < kmax) { S.kept[r0] = E; S.cnt[r0] = c0; S.sym[E] = (uint8_t)r0; }
        if (cand1 && r1 < kmax) { S.kept[r1] = kNeg + E; S.cnt[r1] = c1; S.sym[kNeg + E] = (uint8_t)r1; }
        total += __popcll(m0) + __popcll(m1);
        nonfinite = nonfinite || __any(E == kEmax && (c0 | c1) != 0);
        zero_class = zero_class || __any(E == 0 && (c0 | c1) != 0);
    }
    // The other wavefronts list chunks; the maxima of their first batch are already on their way while the
    // first wavefront ranks the buckets (a chunk with a ragged end is always read).  Work item t stands for
    // slot (hi << 9) | lo of the transposed maxima, hi = t / per_row, so that a wavefront's loads fall on a few
    // cache lines; its chunk is (lo << 9) | hi.  One batch covers the 16384 chunks of a 2^28-element call.
    constexpr u32 kListBatch = 18;
    const bool lister = chunk_list && threadIdx.x >= kW;
    const u32 workers = blockDim.x - kW, list_first = (threadIdx.x - kW) & ~(kW - 1);
    const u32 nchunks = (u32)num_chunks_of(n), nfull = (u32)(n / kChunk);
    const u32 per_row = nchunks > 512 ? (nchunks + 511) >> 9 : 1, items = 512 * per_row;
    const float inv_per_row = 1.0f / (float)per_row;
    u32 maxima[kListBatch], chunk_of[kListBatch];
    auto fetch_maxima = [&](u32 t0) {
#pragma unroll
        for (u32 u = 0; u < kListBatch; ++u) {
            const u32 t = t0 + u * workers + lane;
            u32 hi = (u32)((float)t * inv_per_row);                    // t < 2^18: off by one at most
            if (hi * per_row > t) --hi; else if ((hi + 1) * per_row <= t) ++hi;
            const u32 lo = t - hi * per_row, c = (lo << 9) | hi;
            chunk_of[u] = t < items ? c : 0xFFFFFFFFu;
            maxima[u] = (t < items && c < nfull) ? chunk_maxexp[(hi << 9) | lo] : 0xFFFFFFFFu;
        }
    };
    if (lister) fetch_maxima(list_first);
    const u32 K = total < kmax ? total : kmax;              // (meaningful in the first wavefront only)
    __syncthreads();
    if (threadIdx.x == 0) { s_min_kept_exp = K ? (S.kept[K - 1] & kEmax) : kEmax + 1; s_listed = 0; }   // kept buckets are in descending exponent order
    __syncthreads();
    if (lister) {
        const u32 min_kept_exp = s_min_kept_exp;
        for (u32 t0 = list_first; t0 < items; t0 += kListBatch * workers) {
            if (t0 != list_first) fetch_maxima(t0);
            u64 m[kListBatch];
            u32 found = 0;
#pragma unroll
            for (u32 u = 0; u < kListBatch; ++u) {
                m[u] = __ballot(chunk_of[u] < nchunks && maxima[u] >= min_kept_exp);
                found += (u32)__popcll(m[u]);
            }
            if (found == 0) continue;
            u32 base = 0;                                  // one claim on the list per batch
            if (lane == 0) base = atomicAdd(&s_listed, found);
            base = __builtin_amdgcn_readfirstlane(base);
#pragma unroll
            for (u32 u = 0; u < kListBatch; ++u) {
                if ((m[u] >> lane) & 1) chunk_list[base + __popcll(m[u] & ((1ull << lane) - 1))] = chunk_of[u];
                base += (u32)__popcll(m[u]);
            }
        }
    }
    if (active) {
        // The first wavefront builds the code.  Lane j holds what belongs to symbol j (count, length, code),
        // to the j-th lightest leaf and to the j-th joined node; single values travel between lanes by
        // readlane, so that no step waits on memory.
        Table& T = ws->table;
        u64 c = lane < K ? S.cnt[lane] : 0;
        u64 kept_total = 0;
        for (u32 j = 0; j < K; ++j) kept_total += read_lane64(c, j);
        if (lane == K) c = n - kept_total;
        const u32 msym = K + 1;
        const bool have = lane < msym && c != 0;
        const u32 nl = (u32)__popcll(__ballot(have));
        u32 len = 0;
        bool reuse = false;
        if (ws->spec) {
            bool differs = false;
            u32 cached_len = 0;
            if (lane < K) differs = T.kept[lane] != S.kept[lane];
            if (lane < msym) { cached_len = T.codelen[lane] & 31; differs = differs || ((cached_len != 0) != (c != 0)); }
            // ... and the cached lengths must not need more than the n * nbits payload bits every blob is promised to
            // fit (a stale table on shifted populations can; this checkpoint's own Huffman code never does)
            const u64 payload_bits = wave_sum64(lane < msym ? c * cached_len : 0ull);
            reuse = !nonfinite && T.K == K && !__any(differs) && payload_bits <= n * (u64)nbits;
            if (reuse) len = cached_len;
        }
        if (!reuse && nl == 1) len = have ? 1u : 0u;
        if (!reuse && nl >= 2) {
            // place of every occurring symbol in ascending (count, symbol) order, then the leaves in that order
            u32 place = 0;
            for (u32 i = 0; i < msym; ++i) {
                const u64 ci = read_lane64(c, i);
                place += (ci != 0 && (ci < c || (ci == c && i < lane))) ? 1u : 0u;
            }
            u64 leaf_w = 0; u32 leaf_sym = 0;
            for (u32 i = 0; i < msym; ++i) {
                const u64 ci = read_lane64(c, i);
                const u32 pi = read_lane(place, i);
                if (ci != 0 && pi == lane) { leaf_w = ci; leaf_sym = i; }
            }
            // two queues: sorted leaves and joined nodes in creation order (their weights never decrease);
            // on equal weight the leaf is taken first.  Ids >= 16 are joined nodes.
            u64 node_w = 0; u32 left = 0, right = 0;
            u32 li = 0, qi = 0, ni = 0;
            for (u32 k = 0; k + 1 < nl; ++k) {
                u32 pick[2]; u64 wsum = 0;
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const u64 lw = read_lane64(leaf_w, li < nl ? li : 0), nw = read_lane64(node_w, qi < ni ? qi : 0);
                    const bool take_leaf = li < nl && (qi >= ni || lw <= nw);
                    if (take_leaf) { pick[q] = read_lane(leaf_sym, li); wsum += lw; ++li; }
                    else { pick[q] = 16 + qi; wsum += nw; ++qi; }
                }
                if (lane == ni) { node_w = wsum; left = pick[0]; right = pick[1]; }
                ++ni;
            }
            u32 depth = 0;                                   // of node `lane`; the root (the last node) has depth 0
            for (int i = (int)ni - 1; i >= 0; --i) {
                const u32 d = read_lane(depth, (u32)i) + 1, ch[2] = {read_lane(left, (u32)i), read_lane(right, (u32)i)};
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    if (ch[q] >= 16) { if (lane == ch[q] - 16) depth = d; }
                    else if (lane == ch[q]) len = d;
                }
            }
        }
        // canonical codes: within a length in symbol order, the first code of a length from the counts below it
        u32 code = 0, first = 0, shorter = 0;
        for (u32 L = 1; L < kMaxSym; ++L) {
            const u64 m = __ballot(len == L);
            first = (first + shorter) << 1;
            shorter = (u32)__popcll(m);
            if (len == L) code = first + (u32)__popcll(m & ((1ull << lane) - 1));
        }
        const u32 max_len = wave_max_u32(len);
        if (lane < kMaxSym) {
            T.codelen[lane] = lane < msym ? ((code << 5) | len) : 0;
            T.kept[lane] = lane < K ? S.kept[lane] : 0;
            T.cnt[lane] = lane < msym ? c : 0;
        }
        if (lane <= kMaxSym) S.len[lane] = len;
        if (lane == 0) {
            s_reuse = reuse;
            ws->spec_ok = reuse;
            T.K = K; T.max_len = max_len; T.k_E = total + (zero_class ? 1u : 0u);
            T.min_kept_exp = s_min_kept_exp;
            T.status = nonfinite ? 2u : 0u;
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) ws->list_count = s_listed;
    uint8_t* symlen_of_bucket = EB == 8 ? ws->table.symlen_of_bucket : ext->symlen_of_bucket;
    if (active) for (u32 b = lane; b < (2u << EB); b += kW) {
        const u32 sy = S.sym[b] == 0xFF ? K : S.sym[b];
        symlen_of_bucket[b] = (uint8_t)(sy | (S.len[sy] << 4));
    }
    if (active && ws->spec && !s_reuse) {          // the speculative coding is void: forget its extremes and sizes
        for (u32 i = lane; i < ngroups; i += kW) group_words[i] = 0;
        clear_extremes(ws, lane, kW);
    }
}

template <int EB>
__global__ __launch_bounds__(1024) void k_table(EncState* ws, Ext64* ext, u64 n, int nbits, u32* group_words, u32 ngroups,
                                                 const u32* chunk_maxexp, u32* chunk_list) {
    table_build<EB>(ws, ext, n, nbits, group_words, ngroups, chunk_maxexp, chunk_list);
}

// ----------------------------------------------------------------------------- k_spec_table
// lc_encode_cached, before the sweep: turns a usable cache (valid, same nbits, kept buckets in strict
// priority order, lengths forming a complete prefix code) into the table the sweep codes with.
template <int EB>                         // EB: exponent bits of the parameters' delta (8, or 11 for binary64)
__global__ __launch_bounds__(64) void k_spec_table(EncState* ws, Ext64* ext, const TableCache* cache, int nbits,
                                                   u32* group_words, u32 ngroups) {
    constexpr u32 kBuckets = 2u << EB, kEmax = (1u << EB) - 1;
    __shared__ u32 s_ok, s_len[kMaxSym + 1];
    __shared__ uint8_t s_sym[kBuckets];
    const u32 lane = threadIdx.x;
    Table& T = ws->table;
    for (u32 i = lane; i < ngroups; i += kW) group_words[i] = 0;      // (the sweep that follows may add to them: see k_table)
    for (u32 b = lane; b < kBuckets; b += kW) s_sym[b] = 0xFF;
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
                const u32 b = cache->kept[j], e = b & kEmax;
                const u32 key = (e << 1) | (1u - ((b >> EB) & 1u));    // larger exponent first, + before -
                if (b >= kBuckets || e == 0 || e == kEmax || key >= prev_key) { ok = false; break; }
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
            T.min_kept_exp = K ? (cache->kept[K - 1] & kEmax) : kEmax + 1;
        }
        s_ok = ok;
        ws->spec = ok; ws->spec_ok = 0;
    }
    __syncthreads();
    if (s_ok) {
        const u32 K = cache->K;
        uint8_t* symlen_of_bucket = EB == 8 ? T.symlen_of_bucket : ext->symlen_of_bucket;
        for (u32 b = lane; b < kBuckets; b += kW) {
            const u32 sy = s_sym[b] == 0xFF ? K : s_sym[b];
            symlen_of_bucket[b] = (uint8_t)(sy | (s_len[sy] << 4));
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

constexpr int kSpecCopies = 2;      // LDS copies of the bucket histogram in the speculative sweep (4 copies leave room for 6
                                    // wavefronts per compute unit instead of 8: 0.443 against 0.428 ms per 2^28 elements)

// Where copy `copy` of bucket b's count lies in PackLds::hist.  The two signs of an exponent would otherwise share an LDS
// bank (512 words apart), and a delta's sign is a coin toss: bit 4 of the index is flipped for the negative half.
__device__ __forceinline__ u32 hist_slot(u32 b, u32 copy) { return (b * kSpecCopies + copy) ^ ((b >> 8) << 4); }

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
    bool vec;                    // the arrays are aligned for 4-element accesses (whole rows of a ragged chunk too)
    bool by_parts;               // a chunk of aligned arrays that is mostly merged: coded part by part, and
    u32 parts;                   // which of its whole parts have to be read
};

// Where the counting sweep of a batched call notes a chunk's largest exponent and those of its 4 KiB parts (one byte
// each); both null where nobody wants them.  (Not part of ChunkRef: the coding kernels carry that in registers.)
struct MaximaAt {
    u32* chunk;
    uint8_t* parts;
};

// The counting sweep of a batched call also notes the largest |delta| exponent of every chunk and of each of its 4 KiB
// parts (one wavefront owns the chunk: plain stores).  From these the chunks that hold merged elements only are told
// before the coding sweep, and of a mostly merged chunk the parts that have to be read.
template <int DT>
struct ChunkMaxima {
    static constexpr u32 kRowsPerPart = 4096 / (kRowElems * elem_bytes<DT>());      // 4 (4-byte elements) or 8 (2-byte)
    static constexpr u32 kParts = kR / kRowsPerPart;
    u32 umax = 0, part_max = 0;               // the chunk's largest |delta| pattern (per lane); lane p: exponent of part p
    // `gm`: this lane's largest pattern among the 4 rows that start at row r0
    __device__ __forceinline__ void group(u32 gm, u32 r0) {
        umax = max(umax, gm);
        const u32 pm = wave_max_u32(gm) >> 23;
        if (lane_id() == r0 / kRowsPerPart) part_max = max(part_max, pm);
    }
    __device__ __forceinline__ void note(const MaximaAt& at) {
        const u32 m = wave_max_u32(umax);
        if (lane_id() == 0) *at.chunk = m >> 23;
        if (lane_id() < kParts) at.parts[lane_id()] = (uint8_t)part_max;
    }
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

// Any size, any alignment, one symbol per look-up.  The vector's ragged last chunk is one wavefront's work from
// start to end, so its memory round trips count: the rows that lie wholly inside an aligned vector are fetched as
// in a full chunk, four at a time and one batch ahead; what is left takes guarded element loads.
constexpr int kPlainRows = 4;

template <bool HIST, bool PACK, int DT>
__device__ __noinline__ void pack_chunk_plain(const ChunkRef ch, PackLds<HIST>& L, const MaximaAt at = MaximaAt{nullptr, nullptr}) {
    const u32 lane = lane_id();
    const void* __restrict__ w = ch.w; const void* __restrict__ w_ref = ch.w_ref;
    const u64 n = ch.n, base = (u64)ch.c * kChunk;
    u32* slot = ch.slot;
    const u32 mm = lane & (kMmCopies - 1);
    u64 acc = 0;
    u32 nb = 0, nw = 0;
    ChunkMaxima<DT> cm;                       // counting only
    u32 gmax = 0;                             // ... this lane's largest |delta| pattern since it was last handed to cm
    auto code_row = [&](auto whole, u64 idx, const float (&xa)[4], const float (&xb)[4]) {
        constexpr bool WHOLE = decltype(whole)::value;
#pragma unroll
        for (int v = 0; v < 4; ++v) {
            if (WHOLE || idx + v < n) {
                const u32 u = delta_bits(xa[v], xb[v]);
                if (HIST) atomicAdd(&L.hist[hist_slot(u >> 23, lane & (kSpecCopies - 1))], 1u);
                if (HIST && !PACK) gmax = max(gmax, u & 0x7FFFFFFFu);
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
    };
    typedef std::integral_constant<bool, true> yes;
    typedef std::integral_constant<bool, false> no;
    auto row_at_ = [&](u32 r) { return base + (u64)r * kRowElems + lane * kV; };
    // whole rows of an aligned vector, in batches of kPlainRows
    u32 r = 0;
    const u64 inside = n > base ? n - base : 0;
    const u32 whole_rows = ch.vec ? (u32)min((u64)kR, inside / kRowElems) / kPlainRows * kPlainRows : 0u;
    if (whole_rows) {
        float xa[kPlainRows][4], xb[kPlainRows][4], ya[kPlainRows][4], yb[kPlainRows][4];
        auto fetch = [&](float (&a)[kPlainRows][4], float (&b)[kPlainRows][4], u32 r0) {
#pragma unroll
            for (int k = 0; k < kPlainRows; ++k) { load_row<true, DT>(w, row_at_(r0 + k), n, a[k]); load_row<true, DT>(w_ref, row_at_(r0 + k), n, b[k]); }
        };
        auto code = [&](const float (&a)[kPlainRows][4], const float (&b)[kPlainRows][4], u32 r0) {
#pragma unroll
            for (int k = 0; k < kPlainRows; ++k) code_row(yes(), row_at_(r0 + k), a[k], b[k]);
            if (HIST && !PACK && at.chunk) { cm.group(gmax, r0); gmax = 0; }
        };
        fetch(xa, xb, 0);
        for (; r < whole_rows; r += 2 * kPlainRows) {
            // the batch after this one, or (none left) this one again: loads on every path, see k_hist
            fetch(ya, yb, r + kPlainRows < whole_rows ? r + kPlainRows : r);
            code(xa, xb, r);
            if (r + kPlainRows >= whole_rows) { r += kPlainRows; break; }
            fetch(xa, xb, r + 2 * kPlainRows < whole_rows ? r + 2 * kPlainRows : r);
            code(ya, yb, r + kPlainRows);
        }
    }
    for (; r < kR && base + (u64)r * kRowElems < n; r += kPlainRows) {
        float xa[kPlainRows][4], xb[kPlainRows][4];
#pragma unroll
        for (int k = 0; k < kPlainRows; ++k) { load_row<false, DT>(w, row_at_(r + k), n, xa[k]); load_row<false, DT>(w_ref, row_at_(r + k), n, xb[k]); }
#pragma unroll
        for (int k = 0; k < kPlainRows; ++k) code_row(no(), row_at_(r + k), xa[k], xb[k]);
    }
    if (HIST && !PACK && at.chunk) { cm.umax = max(cm.umax, gmax); cm.note(at); }     // (rows behind the last whole part: the chunk's maximum only)
    if (!PACK) return;
    if (nb > 0) slot[kLaneBitsWords + nw * kW + lane] = (u32)(acc << (32 - nb));
    finish_lane_sizes(ch, nb, nw);
}

// element index of this lane's 4 elements in row r of chunk c
__device__ __forceinline__ u64 row_at(u32 c, u32 r) { return (u64)c * kChunk + (u64)(r * kW + lane_id()) * kV; }

// A chunk of aligned arrays of which sweep 1 has seen that only a few parts hold anything but merged elements
// (a part = one batch of that sweep: 4 KiB of each array; bit p of `parts` set = part p has to be read).  The lone
// wavefront that codes such a chunk would otherwise wait for all 64 rows of both arrays; here it fetches the
// marked parts only and writes the merged code for every element of the others; the rows of a ragged chunk
// behind its last whole part are read as they are.  Same lane strings as any path.
template <int DT>
__device__ __noinline__ void pack_chunk_parts(const ChunkRef ch, u32 cl_merged, PackLds<false>& L) {
    constexpr u32 kRowsPerPart = 4096 / (kRowElems * elem_bytes<DT>());      // 4 (4-byte elements) or 8 (2-byte)
    constexpr u32 kParts = kR / kRowsPerPart;
    const u32 lane = lane_id();
    u32* slot = ch.slot;
    const u32 mm = lane & (kMmCopies - 1);
    u64 acc = 0;
    u32 nb = 0, nw = 0;
    auto flush = [&]() {
        if (nb >= 32) { slot[kLaneBitsWords + nw * kW + lane] = (u32)(acc >> (nb - 32)); ++nw; nb -= 32; }
    };
    // (a chunk with an unmarked part holds merged elements, so their symbol has a code; without one nothing is skipped)
    const u32 len_merged = cl_merged & 31, per_step = len_merged ? 32 / len_merged : 1;
    u32 run = 0;                                                             // per_step copies of the merged code
    for (u32 i = 0; i < per_step; ++i) run = (run << len_merged) | (cl_merged >> 5);
    auto code_element = [&](float a, float b) {
        const u32 u = delta_bits(a, b);
        const u32 sy = L.sym8[u >> 23] >> 3;
        const u32 cl = L.codelen[sy];
        atomicMin(&L.mn[sy * kMmCopies + mm], u);
        atomicMax(&L.mx[sy * kMmCopies + mm], u);
        acc = (acc << (cl & 31)) | (cl >> 5);
        nb += cl & 31;
    };
    const u64 n = ch.n, inside = n - (u64)ch.c * kChunk;
    const u32 whole = inside >= kChunk ? kParts : (u32)(inside / (kRowsPerPart * kRowElems));
    for (u32 p = 0; p < whole; ++p) {
        if ((ch.parts >> p) & 1u) {
            float xa[kRowsPerPart][4], xb[kRowsPerPart][4];
#pragma unroll
            for (u32 k = 0; k < kRowsPerPart; ++k) {
                load_row<true, DT>(ch.w, row_at(ch.c, p * kRowsPerPart + k), ch.n, xa[k]);
                load_row<true, DT>(ch.w_ref, row_at(ch.c, p * kRowsPerPart + k), ch.n, xb[k]);
            }
#pragma unroll
            for (u32 k = 0; k < kRowsPerPart; ++k) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    code_element(xa[k][v], xb[k][v]);
                    if (v & 1) flush();
                }
            }
        } else {
            // the merged code kRowsPerPart * 4 times, as many copies per step as fit 32 bits
            for (u32 left = kRowsPerPart * kV; left != 0;) {
                const u32 k = left < per_step ? left : per_step;
                acc = (acc << (k * len_merged)) | (u64)(run >> ((per_step - k) * len_merged));
                nb += k * len_merged;
                flush();
                left -= k;
            }
        }
    }
    if (whole < kParts) {
        // a ragged chunk's last rows (fewer than one part), fetched together, elements past the end left out
        float xa[kRowsPerPart][4], xb[kRowsPerPart][4];
#pragma unroll
        for (u32 k = 0; k < kRowsPerPart; ++k) {
            const u64 idx = row_at(ch.c, whole * kRowsPerPart + k);
            load_row<false, DT>(ch.w, idx, n, xa[k]);
            load_row<false, DT>(ch.w_ref, idx, n, xb[k]);
        }
#pragma unroll
        for (u32 k = 0; k < kRowsPerPart; ++k) {
            const u64 idx = row_at(ch.c, whole * kRowsPerPart + k);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (idx + v < n) code_element(xa[k][v], xb[k][v]);
                if (v & 1) flush();
            }
        }
    }
    if (nb > 0) slot[kLaneBitsWords + nw * kW + lane] = (u32)(acc << (32 - nb));
    finish_lane_sizes(ch, nb, nw);
}

// A full chunk whose largest exponent (sweep 1 recorded it) lies below every kept bucket: all 16384 symbols
// are the merged one (Section 3.1.1, priority promotion) and each lane's string is 256 copies of its code.
// Such a chunk gets no slot: sweep 2 only notes its size, with kMergedChunk set in chunk_bits, and k_place
// writes the repeated code straight into the blob.
constexpr u32 kMergedChunk = 0x80000000u;

constexpr int kPackPF = 8;          // rows per prefetch batch of the coding loop


// `rot`: the row a wavefront starts a chunk with (a multiple of kPackPF; rows wrap around).  Coding has to take the
// rows in order (0); counting does not, and wavefronts that start their chunks together on the same row keep asking the
// same few memory channels at a time: chunk starts are 64 KiB apart, and a bare read of two arrays in this pattern runs
// at 5.9 TB/s, with every wavefront starting one batch of rows later than its neighbour at 6.8.
template <int DT>
__device__ __forceinline__ void fetch_first_batch(const ChunkRef& ch, typename Raw<DT>::type (&A)[kPackPF],
                                                  typename Raw<DT>::type (&B)[kPackPF], u32 rot = 0) {
#pragma unroll
    for (int k = 0; k < kPackPF; ++k) { A[k] = load_raw<DT>(ch.w, row_at(ch.c, rot + k)); B[k] = load_raw<DT>(ch.w_ref, row_at(ch.c, rot + k)); }
}

// A full, aligned chunk whose first batch of rows is already in A0/B0; leaves the first batch of `next`
// there if that chunk takes this path too.
template <bool ROWCHK, bool HIST, bool PACK, int DT>
__device__ __forceinline__ void pack_chunk_fast(const ChunkRef& cur, const ChunkRef& next,
                                                typename Raw<DT>::type (&A0)[kPackPF], typename Raw<DT>::type (&B0)[kPackPF],
                                                u32 K8, PackLds<HIST>& L, const MaximaAt at = MaximaAt{nullptr, nullptr},
                                                u32 rot = 0) {
    constexpr int PF = kPackPF;
    static_assert((kR & (kR - 1)) == 0 && kR % (2 * kPackPF) == 0, "rows wrap with a mask");
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
    ChunkMaxima<DT> cm;                       // counting only
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
    auto group = [&](const raw_t* a, const raw_t* b, u32 r0) {
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
            for (int i = 0; i < 16; ++i) atomicAdd(&L.hist[hist_slot(u[i] >> 23, lane & (kSpecCopies - 1))], 1u);
        }
        if (HIST && !PACK && at.chunk) {
            u32 gm = 0;
#pragma unroll
            for (int i = 0; i < 16; ++i) gm = max(gm, u[i] & 0x7FFFFFFFu);
            cm.group(gm, r0);
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
    // (row: the chunk's row that step r0 starts with; rot is 0 unless this is the counting sweep)
    auto row = [&](u32 r) { return (HIST && !PACK) ? ((r + rot) & (kR - 1)) : r; };
    for (u32 r0 = 0; r0 < kR; r0 += 2 * PF) {
#pragma unroll
        for (int k = 0; k < PF; ++k) { A1[k] = load_raw<DT>(w, row_at(c, row(r0 + PF) + k)); B1[k] = load_raw<DT>(w_ref, row_at(c, row(r0 + PF) + k)); }
        group(A0, B0, row(r0)); group(A0 + 4, B0 + 4, row(r0) + 4);
        if (r0 + 2 * PF < kR) {
#pragma unroll
            for (int k = 0; k < PF; ++k) { A0[k] = load_raw<DT>(w, row_at(c, row(r0 + 2 * PF) + k)); B0[k] = load_raw<DT>(w_ref, row_at(c, row(r0 + 2 * PF) + k)); }
        } else if (next_fast) {
            fetch_first_batch<DT>(next, A0, B0, (HIST && !PACK) ? rot : 0u);
        }
        group(A1, B1, row(r0 + PF)); group(A1 + 4, B1 + 4, row(r0 + PF) + 4);
    }
    if (HIST && !PACK && at.chunk) cm.note(at);
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
// Src::take() is the wavefront's next chunk.
template <bool HIST, bool PACK, int DT, int ROWSEL, typename Src>
__device__ __forceinline__ void pack_loop(Src& src, PackLds<HIST>& L) {
    typedef typename Raw<DT>::type raw_t;
    raw_t A0[kPackPF], B0[kPackPF];
    // the counting sweep: every wavefront starts its chunks one batch of rows after its neighbour (see fetch_first_batch)
    const u32 rot = (HIST && !PACK) ? (blockIdx.x % (kR / kPackPF)) * kPackPF : 0u;
    ChunkRef cur = src.take();
    if (cur.valid && cur.fast) fetch_first_batch<DT>(cur, A0, B0, rot);
    while (cur.valid) {
        const ChunkRef next = src.take();
        src.enter(cur, L);
        if constexpr (HIST && !PACK) {
            // counting only
            const MaximaAt at = src.maxima_at(cur);
            if (!cur.fast) {
                pack_chunk_plain<HIST, PACK, DT>(cur, L, at);
                if (next.valid && next.fast) fetch_first_batch<DT>(next, A0, B0, rot);
            } else {
                pack_chunk_fast<true, HIST, PACK, DT>(cur, next, A0, B0, src.K8(), L, at, rot);
            }
        } else if (!cur.fast) {
            if constexpr (!HIST && PACK) {
                if (cur.by_parts) pack_chunk_parts<DT>(cur, src.merged_codelen(), L);
                else pack_chunk_plain<HIST, PACK, DT>(cur, L);
            } else {
                pack_chunk_plain<HIST, PACK, DT>(cur, L);
            }
            if (next.valid && next.fast) fetch_first_batch<DT>(next, A0, B0);
        } else if (ROWSEL == 1 || (ROWSEL < 0 && src.rowchk())) {
            pack_chunk_fast<true, HIST, PACK, DT>(cur, next, A0, B0, src.K8(), L);
        } else {
            pack_chunk_fast<false, HIST, PACK, DT>(cur, next, A0, B0, src.K8(), L);
        }
        cur = next;
    }
}

// Which of the first `whole` parts of a chunk hold an exponent of a kept bucket (`maxima`: the largest exponent of each
// of its parts_per_chunk parts, one byte each, 4-byte aligned); false if those are more than a quarter of a chunk's
// parts (the chunk then takes the usual paths).
__device__ __forceinline__ bool parts_to_read(const uint8_t* maxima, u32 parts_per_chunk, u32 min_kept_exp, u32 whole, u32* parts) {
    const u32* p = reinterpret_cast<const u32*>(maxima);
    u32 mask = 0;
    for (u32 i = 0; i < parts_per_chunk / 4; ++i) {
        const u32 word = load_uniform(p + i);
#pragma unroll
        for (u32 b = 0; b < 4; ++b) mask |= (((word >> (8 * b)) & 255u) >= min_kept_exp ? 1u : 0u) << (4 * i + b);
    }
    mask &= (1u << whole) - 1u;                   // (a ragged chunk: the bytes of its missing parts mean nothing)
    *parts = mask;
    return (u32)__popc(mask) <= parts_per_chunk / 4;
}

// The same for binary64 parameters: 32 parts of 512 elements per chunk, two bytes per maximum (11 exponent bits).
__device__ __forceinline__ bool parts_to_read64(const uint16_t* maxima, u32 min_kept_exp, u32 whole, u32* parts) {
    const u32* p = reinterpret_cast<const u32*>(maxima);
    u32 mask = 0;
    for (u32 i = 0; i < 16; ++i) {
        const u32 word = load_uniform(p + i);
        mask |= ((word & 0xFFFFu) >= min_kept_exp ? 1u : 0u) << (2 * i);
        mask |= ((word >> 16) >= min_kept_exp ? 1u : 0u) << (2 * i + 1);
    }
    if (whole < 32) mask &= (1u << whole) - 1u;
    *parts = mask;
    return (u32)__popc(mask) <= 8u;
}

// The chunks of one vector that have to be read, dealt round-robin to the wavefronts of the grid: all of
// them, or with chunk_list the `listed` ones named there.
struct VectorChunks {
    const void* w; const void* w_ref;
    u64 n;
    u32* prov; u32 slot_words; u32* chunk_bits; u32* group_words;
    u32 nchunks; bool aligned;
    u32 k8; bool row;
    const u32* chunk_list; u32 listed;
    u32 pos;
    const uint8_t* batch_max; u32 parts_per_chunk, min_kept_exp, cl_merged;     // what sweep 1 recorded per 4 KiB batch, or null
    bool wide;                   // binary64: two bytes per recorded maximum
    __device__ __forceinline__ u32 merged_codelen() const { return cl_merged; }
    __device__ __forceinline__ ChunkRef ref(u32 c, bool valid) const {
        ChunkRef ch;
        ch.c = c;
        ch.valid = valid;
        ch.w = w; ch.w_ref = w_ref; ch.n = n;
        ch.fast = aligned && (u64)(c + 1) * kChunk <= n;
        ch.vec = aligned;
        ch.slot = prov + (u64)c * slot_words;
        ch.bits_at = chunk_bits + c;
        ch.group_at = group_words + (c >> 6);
        ch.seg = 0;
        ch.parts = 0; ch.by_parts = false;
        if (valid && aligned && batch_max) {
            const u64 inside = n - (u64)c * kChunk, part_elems = kChunk / parts_per_chunk;
            const u32 whole = inside >= kChunk ? parts_per_chunk : (u32)(inside / part_elems);
            // (less than one whole part: the guarded path)
            ch.by_parts = whole != 0 && (wide ? parts_to_read64(reinterpret_cast<const uint16_t*>(batch_max) + (u64)c * parts_per_chunk, min_kept_exp, whole, &ch.parts)
                                              : parts_to_read(batch_max + (u64)c * parts_per_chunk, parts_per_chunk, min_kept_exp, whole, &ch.parts));
            if (ch.by_parts) ch.fast = false;        // off the pipelined path: see pack_chunk_parts
        }
        return ch;
    }
    __device__ __forceinline__ ChunkRef take() {
        const u32 i = blockIdx.x + (pos++) * gridDim.x;
        if (!chunk_list) return ref(i, i < nchunks);
        return i < listed ? ref(load_uniform(chunk_list + i), true) : ref(nchunks, false);
    }
    template <bool HIST> __device__ __forceinline__ void enter(const ChunkRef&, PackLds<HIST>&) const {}
    __device__ __forceinline__ MaximaAt maxima_at(const ChunkRef&) const { return MaximaAt{nullptr, nullptr}; }
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
        // Wavefronts that code chunks of one vector finish at about the same time, and atomics on one cache line are
        // served one after the other (a 1000-chunk tensor's queued up for 30 us): each workgroup hands its extremes to
        // one of kExtCopies copies, which the workgroup that writes the header joins.
        const u32 copy = blockIdx.x % kExtCopies;
        if (mn <= mx) { atomicMin(&ws->mmin[copy][lane], mn & 0x7FFFFFu); atomicMax(&ws->mmax[copy][lane], mx & 0x7FFFFFu); }
    }
}

// The chunks k_table left off the list (full ones that hold merged elements only): their sizes, a group of 64 per step.
__device__ __forceinline__ void note_merged_chunks(const Table& T, u64 n, u32* chunk_bits, u32* group_words,
                                                   const u32* chunk_maxexp) {
    const u32 lane = lane_id();
    const u32 nfull = (u32)(n / kChunk), min_kept_exp = T.min_kept_exp, len_merged = T.codelen[T.K] & 31;
    for (u32 c0 = blockIdx.x * kW; c0 < nfull; c0 += gridDim.x * kW) {
        const u32 c = c0 + lane;
        const bool merged = c < nfull && chunk_maxexp[maxexp_slot(c)] < min_kept_exp;
        if (merged) chunk_bits[c] = kMergedChunk | (kChunk * len_merged);
        const u32 count = (u32)__popcll(__ballot(merged));
        if (lane == 0 && count) atomicAdd(&group_words[c0 >> 6], count * (kLaneBitsWords + kChunk / 32 * len_merged));
    }
}

template <int DT>
__global__ __launch_bounds__(64) void k_pack(const void* __restrict__ w, const void* __restrict__ w_ref, u64 n,
                                             EncState* ws, u32* chunk_bits, u32* group_words,
                                             const u32* chunk_maxexp, const u32* chunk_list, const uint8_t* batch_max,
                                             u32* prov, u32 slot_words, u32 nchunks, int aligned) {
    __shared__ PackLds<false> L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    if (T.status != 0 || ws->spec_ok != 0) return;     // nothing to code, or the speculative sweep already did
    pack_setup(L, T, lane);
    const u32 K = T.K;
    __syncthreads();
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, aligned != 0, K << 3, T.max_len <= 8,
                        chunk_list, chunk_list ? ws->list_count : 0, 0,
                        chunk_list ? batch_max : nullptr, 4096u / (kRowElems * elem_bytes<DT>()) == 4 ? 16u : 8u, T.min_kept_exp,
                        T.codelen[K]};
    if (chunk_list) note_merged_chunks(T, n, chunk_bits, group_words, chunk_maxexp);
    if (src.row) pack_loop<false, true, DT, 1>(src, L);
    else pack_loop<false, true, DT, 0>(src, L);
    __syncthreads();
    pack_merge_extremes(L, ws, K, lane);
}

// ----------------------------------------------------------------------------- k_pack_keys
// Sweep 2 of an encode with staged keys: the same chunks, slots and lane strings as k_pack, coded from the 9-bit keys
// sweep 1 left (16 exponent bytes + 16 sign bits per lane and batch of 4 rows) instead of from w and w_ref: 1.125
// bytes per element read instead of 8.  The extremes of the kept buckets are sweep 1's business then.  A full chunk
// takes 16 key loads per lane, all in flight together, and the next chunk's are issued before this one is coded; the
// vector's ragged last chunk (whose tail has no keys) is coded from w and w_ref like any ragged chunk.
constexpr u32 kKeyBatches = kR / 4;             // batches of 4 rows per chunk
constexpr u32 kHalfBatches = kKeyBatches / 2;

// The keys of half a chunk as one lane holds them: 8 batches of 16 exponent bytes and 16 sign bits.
struct HalfKeys { u32x4 exp[kHalfBatches]; u32 sign[kHalfBatches]; };

__device__ __forceinline__ void fetch_half(const KeyPlanes& keys, u32 c, u32 half, HalfKeys& k) {
    const u64 at = ((u64)c * kKeyBatches + half * kHalfBatches) * kW + lane_id();
#pragma unroll
    for (u32 b = 0; b < kHalfBatches; ++b) {
        k.exp[b] = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(keys.exp) + at + b * kW);
        k.sign[b] = __builtin_nontemporal_load(keys.sign + at + b * kW);
    }
}

// A lane's growing code string of one chunk.
struct LaneString {
    u64 acc; u32 nb, nw;                // bits waiting in acc (nb of them), words written
    u32* lane_words;
    __device__ __forceinline__ void start(const ChunkRef& ch) { acc = 0; nb = 0; nw = 0; lane_words = ch.slot + kLaneBitsWords + lane_id(); }
    __device__ __forceinline__ void put(u32 word, PackLds<false>& L) {
        if (nw < kStageRows) L.stage[nw * kW + lane_id()] = word;
        else lane_words[nw * kW] = word;
    }
    __device__ __forceinline__ void flush(PackLds<false>& L) {
        if (nb >= 32) { put((u32)(acc >> (nb - 32)), L); ++nw; nb -= 32; }
    }
};

template <bool ROWCHK>
__device__ __forceinline__ void code_half(const HalfKeys& k, LaneString& S, PackLds<false>& L) {
#pragma unroll
    for (u32 b = 0; b < kHalfBatches; ++b) {
        const u32 wv[4] = {k.exp[b].x, k.exp[b].y, k.exp[b].z, k.exp[b].w};
        u32 t[16];
#pragma unroll
        for (int i = 0; i < 16; ++i)        // bucket id = sign << 8 | exponent, as the top 9 bits of the delta
            t[i] = L.sym8[((wv[i >> 2] >> (8 * (i & 3))) & 255u) | (((k.sign[b] >> i) & 1u) << 8)];
        uint2 p[8];
#pragma unroll
        for (int i = 0; i < 8; ++i)
            p[i] = *reinterpret_cast<const uint2*>(reinterpret_cast<const uint8_t*>(L.pair) + ((t[2 * i] << 4) | t[2 * i + 1]));
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            S.acc = (S.acc << p[i].y) | p[i].x; S.nb += p[i].y;
            if (!ROWCHK || (i & 1)) S.flush(L);
        }
    }
}

// the last, partly filled word, then the staged rows to the slot (as pack_chunk_fast), then the sizes
__device__ __forceinline__ void finish_chunk_keys(const ChunkRef& cur, LaneString& S, PackLds<false>& L) {
    const u32 lane = lane_id();
    if (S.nb > 0) S.put((u32)(S.acc << (32 - S.nb)), L);
    u32 rows = min(S.nw + (S.nb > 0 ? 1u : 0u), kStageRows);
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) rows = max(rows, (u32)__shfl_xor(rows, d, 64));
    const uint4* src = reinterpret_cast<const uint4*>(L.stage);
    uint4* dst = reinterpret_cast<uint4*>(cur.slot + kLaneBitsWords);
    for (u32 i = lane; i < rows * (kW / 4); i += kW) dst[i] = src[i];
    finish_lane_sizes(cur, S.nb, S.nw);
}

// Half a chunk's keys are always on their way while the half before is coded, across chunk borders too.
template <bool ROWCHK>
__device__ __forceinline__ void pack_keys_loop(VectorChunks& src, const KeyPlanes& keys, PackLds<false>& L) {
    HalfKeys A, B;
    ChunkRef cur = src.take();
    if (cur.valid && cur.fast) fetch_half(keys, cur.c, 0, A);
    while (cur.valid) {
        const ChunkRef next = src.take();
        if (cur.fast) {
            LaneString S;
            S.start(cur);
            fetch_half(keys, cur.c, 1, B);
            code_half<ROWCHK>(A, S, L);
            if (next.valid && next.fast) fetch_half(keys, next.c, 0, A);
            code_half<ROWCHK>(B, S, L);
            finish_chunk_keys(cur, S, L);
        } else {
            pack_chunk_plain<false, true, kF32>(cur, L);
            if (next.valid && next.fast) fetch_half(keys, next.c, 0, A);
        }
        cur = next;
    }
}

__global__ __launch_bounds__(64) void k_pack_keys(const void* __restrict__ w, const void* __restrict__ w_ref, u64 n,
                                                  EncState* ws, u32* chunk_bits, u32* group_words, const u32* chunk_maxexp,
                                                  const u32* chunk_list, KeyPlanes keys, u32* prov, u32 slot_words, u32 nchunks) {
    __shared__ PackLds<false> L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    if (T.status != 0) return;
    pack_setup(L, T, lane);
    const u32 K = T.K;
    __syncthreads();
    // (aligned arrays by construction; no part-by-part coding: a listed chunk's keys are 18 KB, read whole)
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, true, K << 3, T.max_len <= 8,
                        chunk_list, ws->list_count, 0, nullptr, 16u, T.min_kept_exp, T.codelen[K]};
    note_merged_chunks(T, n, chunk_bits, group_words, chunk_maxexp);
    if (src.row) pack_keys_loop<true>(src, keys, L);
    else pack_keys_loop<false>(src, keys, L);
}

// ----------------------------------------------------------------------------- k_pack64
// Sweep 2 for binary64 parameters: the same chunks, slots and lane strings; the symbol of an element comes from the
// top 12 bits of its binary64 delta, the extremes are 64-bit patterns.  One symbol per look-up, rows fetched four
// at a time (a row is 32 bytes per lane), code words stored as they fill.
constexpr int kMmCopies64 = 16;

struct PackLds64 {
    uint8_t sym[kBuckets64];
    u32 codelen[kMaxSym];
    unsigned long long mn[kMaxSym * kMmCopies64], mx[kMaxSym * kMmCopies64];
};

template <bool WHOLE>            // WHOLE: a full chunk of 16-byte aligned arrays
__device__ __forceinline__ void pack_chunk64(const ChunkRef& ch, PackLds64& L, u32 K) {
    constexpr int RB = 4;
    const u32 lane = lane_id();
    const u64 n = ch.n, base = (u64)ch.c * kChunk;
    u32* lane_words = ch.slot + kLaneBitsWords + lane;
    const u32 mm = lane & (kMmCopies64 - 1);
    u64 acc = 0;
    u32 nb = 0, nw = 0;
    for (u32 r0 = 0; r0 < kR && (WHOLE || base + (u64)r0 * kRowElems < n); r0 += RB) {
        double xa[RB][4], xb[RB][4];
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const u64 idx = base + (u64)(r0 + k) * kRowElems + lane * kV;
            load_row64<WHOLE>(ch.w, idx, n, xa[k]); load_row64<WHOLE>(ch.w_ref, idx, n, xb[k]);
        }
#pragma unroll
        for (int k = 0; k < RB; ++k) {
            const u64 idx = base + (u64)(r0 + k) * kRowElems + lane * kV;
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (WHOLE || idx + v < n) {
                    const u64 u = delta_bits(xa[k][v], xb[k][v]);
                    const u32 sy = L.sym[bucket_of(u)];
                    const u32 cl = L.codelen[sy];
                    if (sy < K) { atomicMin(&L.mn[sy * kMmCopies64 + mm], u); atomicMax(&L.mx[sy * kMmCopies64 + mm], u); }
                    acc = (acc << (cl & 31)) | (cl >> 5);
                    nb += cl & 31;
                }
                if ((v & 1) && nb >= 32) {
                    lane_words[nw * kW] = (u32)(acc >> (nb - 32));
                    ++nw; nb -= 32;
                }
            }
        }
    }
    if (nb > 0) lane_words[nw * kW] = (u32)(acc << (32 - nb));
    finish_lane_sizes(ch, nb, nw);
}

// A chunk of which at most a quarter of the 4 KiB parts (2 rows of doubles each) hold anything but merged elements:
// see pack_chunk_parts.
__device__ __noinline__ void pack_chunk64_parts(const ChunkRef ch, u32 cl_merged, PackLds64& L, u32 K) {
    constexpr u32 kRowsPerPart = 2, kParts = kR / kRowsPerPart;
    const u32 lane = lane_id();
    u32* lane_words = ch.slot + kLaneBitsWords + lane;
    const u32 mm = lane & (kMmCopies64 - 1);
    u64 acc = 0;
    u32 nb = 0, nw = 0;
    auto flush = [&]() {
        if (nb >= 32) { lane_words[nw * kW] = (u32)(acc >> (nb - 32)); ++nw; nb -= 32; }
    };
    const u32 len_merged = cl_merged & 31, per_step = len_merged ? 32 / len_merged : 1;
    u32 run = 0;                                                             // per_step copies of the merged code
    for (u32 i = 0; i < per_step; ++i) run = (run << len_merged) | (cl_merged >> 5);
    auto code_element = [&](double a, double b) {
        const u64 u = delta_bits(a, b);
        const u32 sy = L.sym[bucket_of(u)];
        const u32 cl = L.codelen[sy];
        if (sy < K) { atomicMin(&L.mn[sy * kMmCopies64 + mm], u); atomicMax(&L.mx[sy * kMmCopies64 + mm], u); }
        acc = (acc << (cl & 31)) | (cl >> 5);
        nb += cl & 31;
    };
    const u64 n = ch.n, base = (u64)ch.c * kChunk, inside = n - base;
    const u32 whole = inside >= kChunk ? kParts : (u32)(inside / (kRowsPerPart * kRowElems));
    auto row_idx = [&](u32 r) { return base + (u64)r * kRowElems + lane * kV; };
    for (u32 p = 0; p < whole; ++p) {
        if ((ch.parts >> p) & 1u) {
            double xa[kRowsPerPart][4], xb[kRowsPerPart][4];
#pragma unroll
            for (u32 k = 0; k < kRowsPerPart; ++k) {
                load_row64<true>(ch.w, row_idx(p * kRowsPerPart + k), n, xa[k]);
                load_row64<true>(ch.w_ref, row_idx(p * kRowsPerPart + k), n, xb[k]);
            }
#pragma unroll
            for (u32 k = 0; k < kRowsPerPart; ++k) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    code_element(xa[k][v], xb[k][v]);
                    if (v & 1) flush();
                }
            }
        } else {
            for (u32 left = kRowsPerPart * kV; left != 0;) {
                const u32 k = left < per_step ? left : per_step;
                acc = (acc << (k * len_merged)) | (u64)(run >> ((per_step - k) * len_merged));
                nb += k * len_merged;
                flush();
                left -= k;
            }
        }
    }
    if (whole < kParts) {
        // a ragged chunk's last rows (fewer than one part), elements past the end left out
        double xa[kRowsPerPart][4], xb[kRowsPerPart][4];
#pragma unroll
        for (u32 k = 0; k < kRowsPerPart; ++k) {
            load_row64<false>(ch.w, row_idx(whole * kRowsPerPart + k), n, xa[k]);
            load_row64<false>(ch.w_ref, row_idx(whole * kRowsPerPart + k), n, xb[k]);
        }
#pragma unroll
        for (u32 k = 0; k < kRowsPerPart; ++k) {
            const u64 idx = row_idx(whole * kRowsPerPart + k);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                if (idx + v < n) code_element(xa[k][v], xb[k][v]);
                if (v & 1) flush();
            }
        }
    }
    if (nb > 0) lane_words[nw * kW] = (u32)(acc << (32 - nb));
    finish_lane_sizes(ch, nb, nw);
}

__global__ __launch_bounds__(64) void k_pack64(const void* __restrict__ w, const void* __restrict__ w_ref, u64 n,
                                               EncState* ws, Ext64* ext, u32* chunk_bits, u32* group_words,
                                               const u32* chunk_maxexp, const u32* chunk_list, const uint8_t* part_max, u32* prov,
                                               u32 slot_words, u32 nchunks, int aligned) {
    __shared__ PackLds64 L;
    const u32 lane = threadIdx.x;
    const Table& T = ws->table;
    if (T.status != 0) return;
    const u32 K = T.K;
    for (u32 i = lane; i < kBuckets64; i += kW) L.sym[i] = ext->symlen_of_bucket[i] & 15;
    if (lane < kMaxSym) L.codelen[lane] = T.codelen[lane];
    for (u32 i = lane; i < kMaxSym * kMmCopies64; i += kW) { L.mn[i] = ~0ull; L.mx[i] = 0; }
    __syncthreads();
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, aligned != 0, K << 3, true,
                        chunk_list, chunk_list ? ws->list_count : 0, 0, chunk_list ? part_max : nullptr, 32u, T.min_kept_exp,
                        T.codelen[K], true};
    if (chunk_list) note_merged_chunks(T, n, chunk_bits, group_words, chunk_maxexp);
    for (ChunkRef ch = src.take(); ch.valid; ch = src.take()) {
        if (ch.by_parts) pack_chunk64_parts(ch, src.merged_codelen(), L, K);
        else if (ch.fast) pack_chunk64<true>(ch, L, K);
        else pack_chunk64<false>(ch, L, K);
    }
    __syncthreads();
    if (lane < K) {
        u64 mn = ~0ull, mx = 0;
#pragma unroll
        for (int k = 0; k < kMmCopies64; ++k) { mn = min(mn, (u64)L.mn[lane * kMmCopies64 + k]); mx = max(mx, (u64)L.mx[lane * kMmCopies64 + k]); }
        if (mn <= mx) { atomicMin(&ext->mmin[lane], mn & 0xFFFFFFFFFFFFFull); atomicMax(&ext->mmax[lane], mx & 0xFFFFFFFFFFFFFull); }
    }
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
    VectorChunks src = {w, w_ref, n, prov, slot_words, chunk_bits, group_words, nchunks, aligned != 0, K << 3,
                        !spec || T.max_len <= 8, nullptr, 0, 0, nullptr, 16u, 0u, 0u};
    if (!spec) pack_loop<true, false, DT, 1>(src, L);
    else if (src.row) pack_loop<true, true, DT, 1>(src, L);
    else pack_loop<true, true, DT, 0>(src, L);
    __syncthreads();
    for (u32 b = lane; b < 512; b += 64) {
        u32 sum = 0;
#pragma unroll
        for (int k = 0; k < kSpecCopies; ++k) sum += L.hist[hist_slot(b, k)];
        if (sum) atomicAdd(&ws->hist[b], (u64)sum);
    }
    if (spec) pack_merge_extremes(L, ws, K, lane);
}

// ----------------------------------------------------------------------------- k_place
// Builds the chunk area of the blob from the per-chunk slots, one wavefront per chunk.  The
// chunk's word offset is the sum of the record sizes before it (whole groups of 64 chunks from
// group_words, the rest from chunk_bits).  The 64 lane strings are joined without gaps: payload
// word W0 + j of a lane takes the low bits of its word j-1 and the high bits of its word j.
// The payload is assembled in LDS, kPlaceWords words at a time: every lane ORs the words of its shifted string
// that fall into the window into a cleared buffer (so words shared by neighbouring lanes need no special care),
// then the window is written out with coalesced stores.  Most chunks fit one window.  PW words per window: 1024
// lets twice as many workgroups share a compute unit as 2048, which a call with few chunks (all of its workgroups
// resident anyway, one chunk's latency what counts) takes instead.
constexpr u32 kPlaceWords = 1024, kPlaceWordsFew = 2048;

// Representatives (Section 3.1.1: mean of the bucket's largest and smallest member, rounded once
// to fp32, ties to even, done on the mantissas since both share a binade), the header, the last
// offset entry, the result for the host; then the scratch state is cleared for the next call.
// The header of one vector's blob and the call's outcome for the host, by a workgroup of 256 threads.  group_words: the
// record sizes of the vector's groups of 64 chunks; their sum is the size of the chunk area.  Everything a thread needs
// from memory is asked for before the first use of any of it (the workgroup runs beside a whole placement sweep: every
// dependent round trip costs microseconds there).
__device__ __forceinline__ void finalize_blob(uint8_t* out, EncState* ws, Result* host_result, TableCache* cache,
                                              u64 n, int nbits, u32 nchunks, u32 dtype, const u32* group_words,
                                              const Ext64* ext = nullptr, const u32* bucket_min = nullptr,
                                              const u32* bucket_max = nullptr) {
    __shared__ u32 hdr[kHeaderBytes / 4];
    __shared__ unsigned long long s_total;
    const u32 t = threadIdx.x;
    const Table& T = ws->table;
    u64 part = 0;
    for (u32 g = t; g < (nchunks + 63) / 64; g += blockDim.x) part += group_words[g];
    if (t == 0) s_total = 0;
    // this thread's symbol (threads 0 .. 15): code, bucket, population, extremes
    const u32 sym = t < kMaxSym ? t : 0;
    const u32 my_codelen = T.codelen[sym], my_kept = T.kept[sym];
    const u64 my_cnt = T.cnt[sym];
    u32 mn = 0x7FFFFFu, mx = 0;
    u64 mn64 = 0, mx64 = 0;
    if (dtype != kF64) {
#pragma unroll
        for (u32 k = 0; k < kExtCopies; ++k) { mn = min(mn, ws->mmin[k][sym]); mx = max(mx, ws->mmax[k][sym]); }
        // (an encode with staged keys: the extremes of every bucket were gathered by sweep 1)
        if (bucket_min) { mn = bucket_min[my_kept & 511u] & 0x7FFFFFu; mx = bucket_max[my_kept & 511u] & 0x7FFFFFu; }
    } else {
        mn64 = ext->mmin[sym]; mx64 = ext->mmax[sym];
    }
    const u32 status = T.status, K = T.K, k_E = T.k_E, max_len = T.max_len;
    const u32 spec_ok = ws->spec_ok, listed = ws->list_count;
    if (t < kHeaderBytes / 4) hdr[t] = 0;
    __syncthreads();
    part = wave_sum64(part);
    if (lane_id() == 0 && part) atomicAdd(&s_total, (unsigned long long)part);
    __syncthreads();
    const u64 total_words = s_total;
    const bool ok = status == 0;
    const u64 area = chunk_area_of(nchunks);
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
        if (ok) { hdr[5] = K; hdr[9] = nchunks; hdr[13] = k_E; hdr[14] = max_len; }
        host_result->bytes = total; host_result->status = status; host_result->used_cache = spec_ok;
        host_result->listed = listed; host_result->pad_r = 0;
        if (cache && ok) { cache->valid = 1; cache->nbits = (u32)nbits; cache->K = K; cache->pad = 0; }
    }
    if (cache && ok && t < kMaxSym) {              // what this blob was coded with, for the next call
        cache->kept[t] = t < K ? my_kept : 0;
        cache->len[t] = t <= K ? (my_codelen & 31) : 0;
    }
    if (ok && t <= K) {
        const u32 len = my_codelen & 31;
        // representative = midrange of the bucket's extremes, rounded once to nearest even (Section 3.1.1):
        // halve the mantissa sum; an odd sum lies halfway between two mantissas and goes to the even one
        u32 bucket = 0xFFFFu, rep = 0;
        if (t < K && dtype != kF64) {
            bucket = my_kept;
            const u32 sum = mn + mx;
            u32 mm = sum >> 1;
            if ((sum & 1) && (mm & 1)) ++mm;
            rep = (bucket << 23) | mm;
        } else if (t < K) {                            // binary64: 52-bit mantissas, high half at header offset 320 + 4 t
            bucket = my_kept;
            const u64 sum = mn64 + mx64;
            u64 mm = sum >> 1;
            if ((sum & 1) && (mm & 1)) ++mm;
            const u64 rep64 = ((u64)bucket << 52) | mm;
            rep = (u32)rep64;
            hdr[80 + t] = (u32)(rep64 >> 32);
        }
        hdr[16 + 4 * t + 0] = bucket | (len << 16);
        hdr[16 + 4 * t + 1] = rep;
        hdr[16 + 4 * t + 2] = (u32)my_cnt;
        hdr[16 + 4 * t + 3] = (u32)(my_cnt >> 32);
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

// The header of a single vector's blob, the call's outcome for the host, and the scratch state left as the next call
// expects it; by one workgroup of 256 threads.  It runs as the first workgroup of k_place, beside the workgroups that
// place the chunks: everything it needs is final before that kernel starts (table, extremes, and the size of the blob,
// which is the sum of the groups' record sizes), and what it clears none of them reads.  The groups' sums, which they
// do read, are cleared by the next call's first kernel that precedes their use (k_table, or k_spec_table).
__device__ __forceinline__ void finalize_vector(uint8_t* out, Workspace* ws, Result* host_result, const u32* group_words,
                                                TableCache* cache, u64 n, int nbits, u32 nchunks, u32 dtype, int staged) {
    finalize_blob(out, ws, host_result, cache, n, nbits, nchunks, dtype, group_words, &ws->ext64, staged ? ws->bucket_min : nullptr,
                  staged ? ws->bucket_max : nullptr);
    clear_encode_state(ws, nullptr, 0, threadIdx.x, blockDim.x);
    if (dtype == kF64) clear_ext64(&ws->ext64, threadIdx.x, blockDim.x);
    if (staged) clear_bucket_extremes(ws, threadIdx.x, blockDim.x);
    // (no fence: the host reads its result after waiting for the stream, and the end of the kernel makes every store
    // visible; a system-scope fence here would have to write back what the other workgroups have just placed)
}

// Chunk c of one vector, by one wavefront of a workgroup of four; `valid` false: an idle wavefront.
template <u32 PW>
__device__ __forceinline__ void place_chunk(uint8_t* out, EncState* ws, const u32* __restrict__ chunk_bits,
                                            const u32* __restrict__ group_words, const u32* __restrict__ prov,
                                            u32 slot_words, u32 nchunks, u32 c, bool valid) {
    __shared__ u32 s_buf_all[4][PW];
    const u32 lane = lane_id(), wv = threadIdx.x >> 6;
    u32* s_buf = s_buf_all[wv];
    const u32* slot = prov + (u64)(valid ? c : 0) * slot_words;
    const u32 own = valid ? __builtin_amdgcn_readfirstlane(chunk_bits[c]) : 0;
    const bool merged = (own & kMergedChunk) != 0;               // wave-uniform: no slot, 256 copies of one code per lane
    const u32 bits = !valid ? 0 : merged ? (own & ~kMergedChunk) / kW : reinterpret_cast<const uint16_t*>(slot)[lane];
    const u32 g = c >> 6;
    u64 part = (valid && 64 * g + lane < c) ? kLaneBitsWords + (((chunk_bits[64 * g + lane] & ~kMergedChunk) + 31) >> 5) : 0;
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
        }
    }
    if (merged) {
        // every lane's string is a whole number of codes and of words, so the payload is the code repeated
        // 16384 times: word i holds the 32 bits from bit 32 i of that endless repetition on
        const u32 codelen = __builtin_amdgcn_readfirstlane(ws->table.codelen[ws->table.K]);
        const u32 len = max(codelen & 31, 1u);                  // (a merged symbol that occurs has a code)
        u64 rep = (u64)(codelen >> 5) << (64 - len);            // the code repeated from bit 63 downwards
        for (u32 filled = len; filled < 64; filled <<= 1) rep |= rep >> filled;
        u32 phase = (32 * lane) % len;                          // bit of the code that word i starts with
        const u32 step = (32 * kW) % len;
        for (u32 i = lane; i < nwords; i += kW) {
            payload[i] = (u32)((rep << phase) >> 32);
            phase += step;
            if (phase >= len) phase -= len;
        }
    }
    const u32 sh = o & 31, W0 = o >> 5, nloc = (bits + 31) >> 5;
    const u32 nt = (bits && !merged) ? ((o + bits - 1) >> 5) - W0 + 1 : 0;   // payload words this lane touches
    const u32* lane_words = slot + kLaneBitsWords + lane;
    if (merged) return;
    // Only this wavefront touches its buffer, and a wavefront's LDS operations take effect in program order: no
    // barrier between clearing, ORing and reading a window.
    for (u32 win = 0; win < nwords; win += PW) {
        const u32 wlen = min(PW, nwords - win);
        for (u32 i = lane; i < wlen; i += kW) s_buf[i] = 0;
        // the touched words j of this lane (payload word W0 + j) that lie inside the window
        const u32 jlo = win > W0 ? win - W0 : 0;
        const u32 jend = win + wlen > W0 ? win + wlen - W0 : 0;
        const u32 jhi = jend < nt ? jend : nt;
        const u32 cnt = jhi > jlo ? jhi - jlo : 0;
        const u32 cnt_max = wave_max_u32(cnt);
        u32 prev = (cnt != 0 && jlo != 0) ? lane_words[(jlo - 1) * kW] : 0;   // (jlo - 1 < nloc whenever jlo < nt)
        for (u32 i0 = 0; i0 < cnt_max; i0 += 8) {
            u32 buf[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const u32 j = jlo + i0 + k;
                buf[k] = (i0 + k < cnt && j < nloc) ? lane_words[j * kW] : 0;
            }
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                if (i0 + k < cnt) {
                    const u32 val = __builtin_amdgcn_alignbit(prev, buf[k], sh);
                    prev = buf[k];
                    atomicOr(&s_buf[W0 + jlo + i0 + k - win], val);
                }
            }
        }
        for (u32 i = lane; i < wlen; i += kW) payload[win + i] = s_buf[i];
    }
}

// Workgroup 0 writes the header and reports the outcome (finalize_vector); the others place four chunks each.
struct FinalizeArgs { Result* host_result; TableCache* cache; u64 n; int nbits; u32 dtype; int staged; };

template <u32 PW>
__global__ __launch_bounds__(256) void k_place(uint8_t* out, Workspace* ws, const u32* __restrict__ chunk_bits,
                                               const u32* __restrict__ group_words, const u32* __restrict__ prov,
                                               u32 slot_words, u32 nchunks, u32* chunk_maxexp, FinalizeArgs fin) {
    if (blockIdx.x == 0) {
        finalize_vector(out, ws, fin.host_result, group_words, fin.cache, fin.n, fin.nbits, nchunks, fin.dtype, fin.staged);
        return;
    }
    const u32 c = (blockIdx.x - 1) * 4 + (threadIdx.x >> 6);
    // sweep 2 was the last to look at the chunk maxima: leave them cleared for the next call, whatever this one's outcome
    if (c < nchunks && lane_id() == 0) chunk_maxexp[maxexp_slot(c)] = 0;
    // the last workgroup may hold idle wavefronts
    place_chunk<PW>(out, ws, chunk_bits, group_words, prov, slot_words, nchunks, c, c < nchunks && ws->table.status == 0);
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
    if (i == 0) *a.list_count = 0;
    constexpr u32 kExt = kExtCopies * kMaxSym;
    constexpr u32 per = 512 + 2 * kExt + 3;                   // words of state to set per tensor
    for (u64 k = i; k < (u64)a.count * per; k += nthr) {
        EncState& st = a.states[k / per];
        const u32 j = (u32)(k % per);
        if (j < 512) st.hist[j] = 0;
        else if (j < 512 + kExt) (&st.mmin[0][0])[j - 512] = 0x7FFFFFu;
        else if (j < 512 + 2 * kExt) (&st.mmax[0][0])[j - 512 - kExt] = 0;
        else if (j == 512 + 2 * kExt) st.spec = 0;
        else if (j == 512 + 2 * kExt + 1) st.spec_ok = 0;
        else st.table.status = 0;
    }
}

// The dense chunks of a batched call as a chunk source for the coding loop.
template <bool HIST, bool PACK>
struct BatchChunks {
    BatchArgs a;
    u32 active;                  // tensor whose counts / extremes / table the LDS holds (0xFFFFFFFF: none yet)
    u32 k8; bool row;
    u32 pos;
    u32 listed;                  // coding sweep: entries of a.chunk_list (the counting sweep takes every chunk)
    u32 cl_merged;               // (code << 5) | length of the active tensor's merged symbol
    u32 stride;                  // wavefronts that share the chunks
    __device__ __forceinline__ ChunkRef take() {
        ChunkRef ch;
        const u32 i = blockIdx.x + (pos++) * stride;
        ch.valid = i < (PACK ? listed : a.total_chunks);
        const u32 g = (PACK && ch.valid) ? load_uniform(a.chunk_list + i) : i;
        ch.seg = 0; ch.c = 0; ch.w = nullptr; ch.w_ref = nullptr; ch.n = 0; ch.fast = false; ch.vec = false; ch.by_parts = false; ch.parts = 0;
        ch.slot = nullptr; ch.bits_at = nullptr; ch.group_at = nullptr;
        if (ch.valid) {
            ch.seg = __builtin_amdgcn_readfirstlane(a.seg_of_chunk[g]);
            const Seg& sg = a.segs[ch.seg];
            ch.c = g - sg.chunk0;
            ch.w = sg.w; ch.w_ref = sg.w_ref; ch.n = sg.n;
            ch.fast = sg.aligned && (u64)(ch.c + 1) * kChunk <= sg.n;
            ch.vec = sg.aligned != 0;
            ch.slot = a.prov + (u64)g * a.slot_words;
            ch.bits_at = a.chunk_bits + g;
            ch.group_at = a.group_words + sg.group0 + (ch.c >> 6);
            // a tensor whose delta is not finite gets a header-only blob: nothing to code
            if (PACK && a.states[ch.seg].table.status != 0) { ch.n = 0; ch.fast = false; }
            else if (PACK && sg.aligned) {
                // a mostly merged chunk: only its parts with a kept element are read (see pack_chunk_parts)
                const u32 ppc = a.dtype == kF32 ? 16u : 8u;
                const u64 inside = sg.n - (u64)ch.c * kChunk, part_elems = kChunk / ppc;
                const u32 whole = inside >= kChunk ? ppc : (u32)(inside / part_elems);
                ch.by_parts = whole != 0 && parts_to_read(a.part_max + (u64)g * kPartBytes, ppc,
                                                         load_uniform(&a.states[ch.seg].table.min_kept_exp), whole, &ch.parts);
                if (ch.by_parts) ch.fast = false;
            }
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
                for (int k = 0; k < kSpecCopies; ++k) { sum += L.hist[hist_slot(b, k)]; L.hist[hist_slot(b, k)] = 0; }
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
            k8 = T.K << 3; row = T.max_len <= 8; cl_merged = T.codelen[T.K];
            __syncthreads();
        }
    }
    __device__ __forceinline__ MaximaAt maxima_at(const ChunkRef& ch) const {
        const u32 g = load_uniform(&a.segs[ch.seg].chunk0) + ch.c;
        return MaximaAt{a.chunk_maxexp + g, a.part_max + (u64)g * kPartBytes};
    }
    __device__ __forceinline__ u32 K8() const { return k8; }
    __device__ __forceinline__ bool rowchk() const { return row; }
    __device__ __forceinline__ u32 merged_codelen() const { return cl_merged; }
};

template <int DT>
__global__ __launch_bounds__(64) void kb_hist(BatchArgs a) {
    __shared__ PackLds<true> L;
    for (u32 i = threadIdx.x; i < 512 * kSpecCopies; i += 64) L.hist[i] = 0;
    __syncthreads();
    BatchChunks<true, false> src = {a, 0xFFFFFFFFu, 0, true, 0, 0, 0, gridDim.x};
    pack_loop<true, false, DT, 1>(src, L);
    src.hand_in(L);
}

__global__ __launch_bounds__(64) void kb_table(BatchArgs a) {
    table_build<8>(&a.states[blockIdx.x], nullptr, a.segs[blockIdx.x].n, a.nbits, nullptr, 0, nullptr, nullptr);
}

// Between the tables and the coding sweep: which chunks that sweep has to read.  A full chunk whose largest exponent
// lies below every kept bucket of its tensor holds the merged symbol 16384 times (Section 3.1.1): it gets its size and
// the flag that lets kb_place write the repeated code, and stays off the list; all others are listed, in no particular
// order (one claim on the list per wavefront).
__global__ __launch_bounds__(256) void kb_list(BatchArgs a) {
    const u32 g = blockIdx.x * blockDim.x + threadIdx.x, lane = lane_id();
    bool listed = false;
    u32 group = 0xFFFFFFFFu, words = 0;
    if (g < a.total_chunks) {
        const u32 sidx = a.seg_of_chunk[g];
        const Seg& sg = a.segs[sidx];
        const Table& T = a.states[sidx].table;
        const u32 c = g - sg.chunk0;
        const bool merged = T.status == 0 && (u64)(c + 1) * kChunk <= sg.n && a.chunk_maxexp[g] < T.min_kept_exp;
        listed = !merged;
        if (merged) {
            const u32 len_merged = T.codelen[T.K] & 31;
            a.chunk_bits[g] = kMergedChunk | (kChunk * len_merged);
            group = sg.group0 + (c >> 6);
            words = kLaneBitsWords + kChunk / 32 * len_merged;
        }
    }
    // the merged chunks' records go into their groups' sums, one addition per group that the wavefront's chunks touch
    // (a group belongs to one tensor, so its merged chunks have records of one size)
    for (u64 pending = __ballot(group != 0xFFFFFFFFu); pending != 0;) {
        const u32 first = (u32)__ffsll((unsigned long long)pending) - 1;
        const u32 key = read_lane(group, first);
        const u64 same = __ballot(group == key);
        if (lane == first) atomicAdd(&a.group_words[key], (u32)__popcll(same) * words);
        pending &= ~same;
    }
    const u64 m = __ballot(listed);
    if (m == 0) return;
    u32 base = 0;
    if (lane == 0) base = atomicAdd(a.list_count, (u32)__popcll(m));
    base = __builtin_amdgcn_readfirstlane(base);
    if (listed) a.chunk_list[base + (u32)__popcll(m & ((1ull << lane) - 1))] = g;
}

template <int DT>
__global__ __launch_bounds__(64) void kb_pack(BatchArgs a) {
    __shared__ PackLds<false> L;
    // The grid was sized before anyone knew how many chunks would be listed: up to gridDim.x of them get a wavefront
    // each (the others leave at once); more are dealt to as many wavefronts as suit a long sweep, evenly.
    const u32 listed = load_uniform(a.list_count);
    u32 waves = listed;
    if (listed > gridDim.x) {
        const u32 turns = (listed + a.waves_long - 1) / a.waves_long;
        waves = (listed + turns - 1) / turns;
    }
    if (blockIdx.x >= waves) return;
    BatchChunks<false, true> src = {a, 0xFFFFFFFFu, 0, true, 0, listed, 0, waves};
    pack_loop<false, true, DT, 0>(src, L);      // flush per pair of codes: right for every table of the batch
    src.hand_in(L);
}

// The first `count` workgroups write the tensors' headers and report their outcomes (everything that takes is final
// before the placement starts, as for a single vector: see finalize_vector); the others place four chunks each.
__global__ __launch_bounds__(256) void kb_place(BatchArgs a) {
    if (blockIdx.x < a.count) {
        const Seg& sg = a.segs[blockIdx.x];
        finalize_blob(sg.out, &a.states[blockIdx.x], &a.results[blockIdx.x], nullptr, sg.n, a.nbits, sg.nchunks, (u32)a.dtype,
                      a.group_words + sg.group0);
        return;
    }
    const u32 g = (blockIdx.x - a.count) * 4 + (threadIdx.x >> 6);
    const bool in_range = g < a.total_chunks;
    const u32 sidx = in_range ? a.seg_of_chunk[g] : 0;
    const Seg& sg = a.segs[sidx];
    EncState* st = &a.states[sidx];
    place_chunk<kPlaceWords>(sg.out, st, a.chunk_bits + sg.chunk0, a.group_words + sg.group0, a.prov + (u64)sg.chunk0 * a.slot_words,
                a.slot_words, sg.nchunks, in_range ? g - sg.chunk0 : 0, in_range && st->table.status == 0);
}

// ----------------------------------------------------------------------------- launchers
void launch_reset(Workspace* ws, uint32_t* group_words, uint32_t* chunk_maxexp, hipStream_t s) {
    hipLaunchKernelGGL(k_reset, dim3(1), dim3(1024), 0, s, ws, group_words, (u32)kMaxGroups, chunk_maxexp, (u32)kMaxChunks);
}

void launch_reset_chunks(Workspace* ws, uint32_t* group_words, uint32_t* chunk_maxexp, uint32_t nchunks, hipStream_t s) {
    hipLaunchKernelGGL(k_reset_chunks, dim3(1), dim3(1024), 0, s, ws, group_words, (nchunks + 63) / 64, chunk_maxexp, nchunks);
}

template <int DT>
static void launch_hist_t(const void* w, const void* w_ref, uint64_t n, Workspace* ws, u32* chunk_maxexp, uint8_t* batch_max,
                          u32 blocks, u32 threads, hipStream_t s) {
    const KeyPlanes none = {nullptr, nullptr};
    if (aligned16(w) && aligned16(w_ref)) hipLaunchKernelGGL((k_hist<true, DT>), dim3(blocks), dim3(threads), 0, s, w, w_ref, (u64)n, ws, chunk_maxexp, batch_max, none);
    else hipLaunchKernelGGL((k_hist<false, DT>), dim3(blocks), dim3(threads), 0, s, w, w_ref, (u64)n, ws, chunk_maxexp, batch_max, none);
}

// keys.exp != null: stage keys (binary32, both arrays 16-byte aligned: the caller has checked)
void launch_hist(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_maxexp, uint8_t* batch_max,
                 KeyPlanes keys, const Tuning& tune, hipStream_t s) {
    if (n == 0) return;
    const u32 threads = tune.hist_threads;
    const u64 units = n / (dtype == kF32 ? 4 : dtype == kF64 ? 2 : 8);   // 16-byte units
    u64 blocks = (units + 4 * threads - 1) / (4 * threads);
    const u64 cap = (u64)tune.num_cu * tune.hist_blocks_per_cu;
    if (blocks > cap) blocks = cap;
    if (blocks < 1) blocks = 1;
    if (dtype == kF64) {
        uint16_t* part_max = reinterpret_cast<uint16_t*>(batch_max);
        if (aligned16(w) && aligned16(w_ref)) hipLaunchKernelGGL(k_hist64<true>, dim3((u32)blocks), dim3(threads), 0, s, w, w_ref, (u64)n, &ws->ext64, chunk_maxexp, part_max);
        else hipLaunchKernelGGL(k_hist64<false>, dim3((u32)blocks), dim3(threads), 0, s, w, w_ref, (u64)n, &ws->ext64, chunk_maxexp, part_max);
        return;
    }
    if (dtype == kBF16) launch_hist_t<kBF16>(w, w_ref, n, ws, chunk_maxexp, batch_max, (u32)blocks, threads, s);
    else if (dtype == kF16) launch_hist_t<kF16>(w, w_ref, n, ws, chunk_maxexp, batch_max, (u32)blocks, threads, s);
    else if (keys.exp) hipLaunchKernelGGL((k_hist<true, kF32, true>), dim3((u32)blocks), dim3(threads), 0, s, w, w_ref, (u64)n, ws, chunk_maxexp, batch_max, keys);
    else launch_hist_t<kF32>(w, w_ref, n, ws, chunk_maxexp, batch_max, (u32)blocks, threads, s);
}

static u32 even_waves(u64 nchunks, u64 cap);

void launch_pack_keys(const void* w, const void* w_ref, uint64_t n, Workspace* ws, uint32_t* chunk_bits, uint32_t* group_words,
                      const uint32_t* chunk_maxexp, const uint32_t* chunk_list, KeyPlanes keys, uint32_t* prov, uint32_t slot_words,
                      const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    const u32 blocks = even_waves(nchunks, (u64)tune.num_cu * tune.keys_waves_per_cu);
    hipLaunchKernelGGL(k_pack_keys, dim3(blocks), dim3(64), 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list,
                       keys, prov, slot_words, (u32)nchunks);
}

// chunk_list: where to list the chunks sweep 2 has to read (chunk_maxexp then holds what k_hist recorded), or null
void launch_table(Workspace* ws, uint64_t n, int nbits, int dtype, uint32_t* group_words, const uint32_t* chunk_maxexp,
                  uint32_t* chunk_list, hipStream_t s) {
    const dim3 wg(chunk_list ? 1024 : 64);
    const u32 ngroups = (u32)((num_chunks_of(n) + 63) / 64);
    if (dtype == kF64) hipLaunchKernelGGL(k_table<11>, dim3(1), wg, 0, s, ws, &ws->ext64, (u64)n, nbits, group_words, ngroups, chunk_maxexp, chunk_list);
    else hipLaunchKernelGGL(k_table<8>, dim3(1), wg, 0, s, ws, (Ext64*)nullptr, (u64)n, nbits, group_words, ngroups, chunk_maxexp, chunk_list);
}

// Single-wave workgroups for a sweep over `nchunks` chunks dealt round-robin, at most `cap`: the largest count that
// gives every wavefront the same number of chunks (to within one), so that none is left with a turn of its own.
static u32 even_waves(u64 nchunks, u64 cap) {
    if (nchunks <= cap) return (u32)nchunks;
    const u64 turns = (nchunks + cap - 1) / cap;
    return (u32)((nchunks + turns - 1) / turns);
}

void launch_spec_table(Workspace* ws, const TableCache* cache, uint64_t n, int nbits, int dtype, uint32_t* group_words, hipStream_t s) {
    const u32 ngroups = (u32)((num_chunks_of(n) + 63) / 64);
    if (dtype == kF64) hipLaunchKernelGGL(k_spec_table<11>, dim3(1), dim3(64), 0, s, ws, &ws->ext64, cache, nbits, group_words, ngroups);
    else hipLaunchKernelGGL(k_spec_table<8>, dim3(1), dim3(64), 0, s, ws, (Ext64*)nullptr, cache, nbits, group_words, ngroups);
}

void launch_spec_sweep(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                       uint32_t* group_words, uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    const u32 blocks = even_waves(nchunks, (u64)tune.num_cu * tune.spec_waves_per_cu);
    const int al = aligned_rows(w, dtype) && aligned_rows(w_ref, dtype);
    const dim3 grid(blocks), wg(64);
    if (dtype == kBF16) hipLaunchKernelGGL(k_spec_sweep<kBF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else if (dtype == kF16) hipLaunchKernelGGL(k_spec_sweep<kF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
    else hipLaunchKernelGGL(k_spec_sweep<kF32>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, prov, slot_words, (u32)nchunks, al);
}

// chunk_maxexp, chunk_list: what k_hist recorded and k_table listed for this vector, or both null
void launch_pack(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                 uint32_t* group_words, const uint32_t* chunk_maxexp, const uint32_t* chunk_list, const uint8_t* batch_max,
                 uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    if (nchunks == 0) return;
    const u32 blocks = even_waves(nchunks, (u64)tune.num_cu * tune.pack_waves_per_cu);
    const int al = aligned_rows(w, dtype) && aligned_rows(w_ref, dtype);
    const dim3 grid(blocks), wg(64);
    if (dtype == kF64) hipLaunchKernelGGL(k_pack64, grid, wg, 0, s, w, w_ref, (u64)n, ws, &ws->ext64, chunk_bits, group_words, chunk_maxexp, chunk_list, batch_max, prov, slot_words, (u32)nchunks, al);
    else if (dtype == kBF16) hipLaunchKernelGGL(k_pack<kBF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list, batch_max, prov, slot_words, (u32)nchunks, al);
    else if (dtype == kF16) hipLaunchKernelGGL(k_pack<kF16>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list, batch_max, prov, slot_words, (u32)nchunks, al);
    else hipLaunchKernelGGL(k_pack<kF32>, grid, wg, 0, s, w, w_ref, (u64)n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list, batch_max, prov, slot_words, (u32)nchunks, al);
}

// The placement of all chunks and, in the same launch, the header and the call's outcome (result: mapped host memory;
// cache: lc_encode_cached's, or null; staged: the extremes come from sweep 1's per-bucket record).
void launch_place(uint8_t* out, Workspace* ws, const uint32_t* chunk_bits, const uint32_t* group_words,
                  const uint32_t* prov, uint32_t slot_words, uint64_t n, uint32_t* chunk_maxexp, Result* host_result,
                  TableCache* cache, int nbits, int dtype, bool staged, hipStream_t s) {
    const u64 nchunks = num_chunks_of(n);
    const u32 blocks = (u32)((nchunks + 3) / 4) + 1;             // + the workgroup that writes the header
    const FinalizeArgs fin = {host_result, cache, (u64)n, nbits, (u32)dtype, staged ? 1 : 0};
    // (up to 1024 workgroups are resident together on this chip even with the larger windows)
    if (blocks <= 1024u) hipLaunchKernelGGL(k_place<kPlaceWordsFew>, dim3(blocks), dim3(256), 0, s, out, ws, chunk_bits, group_words, prov,
                                                slot_words, (u32)nchunks, chunk_maxexp, fin);
    else hipLaunchKernelGGL(k_place<kPlaceWords>, dim3(blocks), dim3(256), 0, s, out, ws, chunk_bits, group_words, prov,
                            slot_words, (u32)nchunks, chunk_maxexp, fin);
}

void launch_batch_encode(const BatchArgs& args, const Tuning& tune, hipStream_t s) {
    BatchArgs a = args;
    a.waves_long = (u32)tune.num_cu * tune.batch_waves_per_cu;
    const u32 cap = (u32)tune.num_cu * 8;
    u32 setup_blocks = (a.total_chunks + 255) / 256;
    if (setup_blocks < a.count * 3) setup_blocks = a.count * 3;
    if (setup_blocks > cap) setup_blocks = cap;
    if (setup_blocks < 1) setup_blocks = 1;
    hipLaunchKernelGGL(kb_setup, dim3(setup_blocks), dim3(256), 0, s, a);
    if (a.total_chunks) {
        // (a counting workgroup needs 19 KB of LDS: 8 fit a compute unit, and a grid of more leaves the last ones a
        // round of their own: 0.20 ms instead of 0.18 on VGG-16's 32 tensors)
        const int per_cu = tune.batch_waves_per_cu < 8 ? tune.batch_waves_per_cu : 8;
        const u32 waves = even_waves(a.total_chunks, (u64)tune.num_cu * per_cu);
        if (a.dtype == kBF16) hipLaunchKernelGGL(kb_hist<kBF16>, dim3(waves), dim3(64), 0, s, a);
        else if (a.dtype == kF16) hipLaunchKernelGGL(kb_hist<kF16>, dim3(waves), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(kb_hist<kF32>, dim3(waves), dim3(64), 0, s, a);
    }
    hipLaunchKernelGGL(kb_table, dim3(a.count), dim3(64), 0, s, a);
    if (a.total_chunks) {
        hipLaunchKernelGGL(kb_list, dim3((a.total_chunks + 255) / 256), dim3(256), 0, s, a);
        const u32 most = (u32)tune.num_cu * 16;
        const u32 waves = a.total_chunks < most ? a.total_chunks : most;
        if (a.dtype == kBF16) hipLaunchKernelGGL(kb_pack<kBF16>, dim3(waves), dim3(64), 0, s, a);
        else if (a.dtype == kF16) hipLaunchKernelGGL(kb_pack<kF16>, dim3(waves), dim3(64), 0, s, a);
        else hipLaunchKernelGGL(kb_pack<kF32>, dim3(waves), dim3(64), 0, s, a);
    }
    hipLaunchKernelGGL(kb_place, dim3(a.count + (a.total_chunks + 3) / 4), dim3(256), 0, s, a);
}

}  // namespace lc
