// Device-side helpers shared by the encode and the decode kernels (gfx950, wave64): wavefront
// reductions and scans, the fp32 delta, streaming loads, and the element types of the parameter arrays.
#pragma once
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

// A word of memory that no kernel now running writes (tables and lists a previous kernel left), at an address that
// is the same in all lanes: read as constant memory it goes through the scalar cache, and waiting for it does not
// mean waiting for every vector load and store the wavefront has in flight.
__device__ __forceinline__ u32 load_uniform(const u32* p) {
    typedef const __attribute__((address_space(4))) u32* const_ptr;
    return *(const_ptr)(p);
}

// Where chunk c's entry lies in chunk_maxexp[kMaxChunks]: sweep 1 works on a window of consecutive chunks at any
// moment, and their atomics would all land in one or two cache lines (one memory channel); transposing the
// 512 x 512 index puts neighbouring chunks 2 KiB apart.
__device__ __forceinline__ u32 maxexp_slot(u32 c) {
    static_assert(kMaxChunks == 512u * 512u, "the transposition assumes 2^18 entries");
    return ((c & 511u) << 9) | (c >> 9);
}

// Largest value over the wavefront (all 64 lanes active), in every lane: row-wise running maxima with DPP
// shifts, then the row results carried across rows (row_bcast), no LDS traffic.
__device__ __forceinline__ u32 wave_max_u32(u32 v) {
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x111, 0xf, 0xf, false));     // row_shr:1
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x112, 0xf, 0xf, false));     // row_shr:2
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x114, 0xf, 0xf, false));     // row_shr:4
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x118, 0xf, 0xf, false));     // row_shr:8
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x142, 0xa, 0xf, false));     // row_bcast:15 into rows 1, 3
    v = max(v, (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x143, 0xc, 0xf, false));     // row_bcast:31 into rows 2, 3
    return (u32)__builtin_amdgcn_readlane((int)v, 63);
}

// Value of one lane (the same index in every lane), in every lane.
__device__ __forceinline__ u32 read_lane(u32 v, u32 l) { return (u32)__builtin_amdgcn_readlane((int)v, (int)l); }
__device__ __forceinline__ u64 read_lane64(u64 v, u32 l) { return ((u64)read_lane((u32)(v >> 32), l) << 32) | read_lane((u32)v, l); }

__device__ __forceinline__ u32 wave_sum32(u32 v) {
#pragma unroll
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    return v;
}

// delta of Algorithm 1 line 4: one IEEE binary32 subtraction (never fused or reassociated).
__device__ __forceinline__ u32 delta_bits(float w, float w_ref) { return __float_as_uint(__fsub_rn(w, w_ref)); }
// ... and for binary64 parameters one binary64 subtraction
__device__ __forceinline__ u64 delta_bits(double w, double w_ref) { return (u64)__double_as_longlong(__dsub_rn(w, w_ref)); }

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
// binary64 parameters are coded on the binary64 delta, with 2^12 buckets (Section 3.1.1, footnote on the bucket
// count); Val<DT> is the type the arithmetic runs in, Bits<DT> its bit pattern.
struct Row64 { double x[4]; };
template <int DT> struct Raw { typedef uint2 type; };
template <> struct Raw<kF32> { typedef float4 type; };
template <> struct Raw<kF64> { typedef Row64 type; };
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));
template <int DT> struct Val { typedef float type; typedef u32 bits; };
template <> struct Val<kF64> { typedef double type; typedef u64 bits; };

template <int DT> __device__ __forceinline__ constexpr u32 elem_bytes() { return DT == kF32 ? 4u : DT == kF64 ? 8u : 2u; }
template <int DT> __device__ __forceinline__ constexpr u32 exp_bits() { return DT == kF64 ? 11u : 8u; }
template <int DT> __device__ __forceinline__ constexpr u32 num_buckets() { return 2u << exp_bits<DT>(); }
// bucket id (sign and exponent bits) and biased exponent of a delta's bit pattern
__device__ __forceinline__ u32 bucket_of(u32 u) { return u >> 23; }
__device__ __forceinline__ u32 bucket_of(u64 u) { return (u32)(u >> 52); }

// 4 consecutive elements starting at element index i (a multiple of 4, base aligned to 4 elements), non-temporal
template <int DT>
__device__ __forceinline__ typename Raw<DT>::type load_raw(const void* base, u64 i) {
    if constexpr (DT == kF32) {
        return load_stream(reinterpret_cast<const float4*>(static_cast<const float*>(base) + i));
    } else if constexpr (DT == kF64) {
        const float4* p = reinterpret_cast<const float4*>(static_cast<const double*>(base) + i);
        const float4 a = load_stream(p), b = load_stream(p + 1);
        Row64 r;
        r.x[0] = __hiloint2double(__float_as_int(a.y), __float_as_int(a.x)); r.x[1] = __hiloint2double(__float_as_int(a.w), __float_as_int(a.z));
        r.x[2] = __hiloint2double(__float_as_int(b.y), __float_as_int(b.x)); r.x[3] = __hiloint2double(__float_as_int(b.w), __float_as_int(b.z));
        return r;
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

// Two values at once, a in the low half.  bf16: v_cvt_pk_bf16_f32, which rounds every finite binary32 value as the
// integer formula above does (compared over all 2^32 patterns); infinities stay infinities.
typedef __bf16 lc_bf16x2 __attribute__((ext_vector_type(2)));
typedef float lc_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32 narrow16_pair(float a, float b, bool bf16) {
    if (bf16) { const lc_f32x2 f = {a, b}; return __builtin_bit_cast(u32, __builtin_convertvector(f, lc_bf16x2)); }
    return narrow16(a, false) | (narrow16(b, false) << 16);
}

__device__ __forceinline__ void unpack64(const Row64& r, double (&x)[4]) {
#pragma unroll
    for (int v = 0; v < 4; ++v) x[v] = r.x[v];
}

template <int DT>
__device__ __forceinline__ void unpack(const typename Raw<DT>::type& r, float (&x)[4]) {
    if constexpr (DT == kF32) { x[0] = r.x; x[1] = r.y; x[2] = r.z; x[3] = r.w; }
    else {
        x[0] = widen16(r.x & 0xFFFFu, DT == kBF16); x[1] = widen16(r.x >> 16, DT == kBF16);
        x[2] = widen16(r.y & 0xFFFFu, DT == kBF16); x[3] = widen16(r.y >> 16, DT == kBF16);
    }
}

// x as it reads back after a store in the storage type (rounded to nearest even; binary32: x itself)
template <int DT>
__device__ __forceinline__ float stored(float x) {
    if constexpr (DT == kF32) return x;
    else return widen16(narrow16(x, DT == kBF16), DT == kBF16);
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

// Restored rows are written once and not read again by the sweep: non-temporal stores, like the loads (a bare
// read-modify-write sweep in this access pattern runs 4-5 % faster with both marked than with the loads alone).
// (STREAM false: plain stores, which the sweep over several blobs keeps.)
template <int DT, bool STREAM = true>
__device__ __forceinline__ void store4(void* base, u64 i, const float (&x)[4]) {
    if constexpr (DT == kF32) {
        const f32x4 v = {x[0], x[1], x[2], x[3]};
        if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<f32x4*>(static_cast<float*>(base) + i));
        else *reinterpret_cast<f32x4*>(static_cast<float*>(base) + i) = v;
    } else {
        const u32x2 v = {narrow16_pair(x[0], x[1], DT == kBF16), narrow16_pair(x[2], x[3], DT == kBF16)};
        if constexpr (STREAM) __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(static_cast<uint16_t*>(base) + i));
        else *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(base) + i) = v;
    }
}

// the same for binary64 parameters
template <bool FAST>
__device__ __forceinline__ void load_row64(const void* __restrict__ p, u64 idx, u64 n, double (&x)[4]) {
    if (FAST) {
        unpack64(load_raw<kF64>(p, idx), x);
    } else {
#pragma unroll
        for (int v = 0; v < 4; ++v) x[v] = (idx + v < n) ? static_cast<const double*>(p)[idx + v] : 0.0;
    }
}
// (plain stores: marked non-temporal, the two 16-byte halves of a lane's 32 bytes made this sweep 15 % slower)
__device__ __forceinline__ void store4_64(void* base, u64 i, const double (&x)[4]) {
    double2* q = reinterpret_cast<double2*>(static_cast<double*>(base) + i);
    q[0] = make_double2(x[0], x[1]); q[1] = make_double2(x[2], x[3]);
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

// ---- the same three accesses and the restoring addition for any element type, on the type the arithmetic runs in
template <bool FAST, int DT>
__device__ __forceinline__ void load_row_v(const void* __restrict__ p, u64 idx, u64 n, typename Val<DT>::type (&x)[4]) {
    if constexpr (DT == kF64) load_row64<FAST>(p, idx, n, x);
    else load_row<FAST, DT>(p, idx, n, x);
}
template <int DT>
__device__ __forceinline__ void store4_v(void* base, u64 i, const typename Val<DT>::type (&x)[4]) {
    if constexpr (DT == kF64) store4_64(base, i, x);
    else store4<DT>(base, i, x);
}
template <int DT>
__device__ __forceinline__ void store_one_v(void* base, u64 i, typename Val<DT>::type x) {
    if constexpr (DT == kF64) static_cast<double*>(base)[i] = x;
    else store_one<DT>(base, i, x);
}
// Algorithm 1 line 7: one IEEE addition in the parameters' arithmetic type (never fused or reassociated)
__device__ __forceinline__ float add_rn(float a, float b) { return __fadd_rn(a, b); }
__device__ __forceinline__ double add_rn(double a, double b) { return __dadd_rn(a, b); }

// ---- host-side helpers of the launchers
// Work items dealt round-robin to at most `cap` workers: the smallest worker count that keeps the number of
// rounds, so that every worker has the same load (+-1) and nobody idles through a last, half-empty round.
static inline uint64_t balanced_workers(uint64_t items, uint64_t cap) {
    if (items <= cap || cap == 0) return items;
    const uint64_t rounds = (items + cap - 1) / cap;
    return (items + rounds - 1) / rounds;
}
static inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }
static inline bool aligned_rows(const void* p, int dtype) {     // 4 consecutive elements per access
    return (reinterpret_cast<uintptr_t>(p) & (dtype == kF32 || dtype == kF64 ? 15 : 7)) == 0;
}

}  // namespace lc
