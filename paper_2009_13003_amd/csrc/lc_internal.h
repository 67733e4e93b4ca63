// Shared between the kernels (lc_encode.hip, lc_decode.hip) and the host API (lc_api.hip):
// the device scratch layout and the launch entry points.  gfx950 only.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lc {

constexpr uint32_t kW = 64;                 // lanes per chunk = one wavefront
constexpr uint32_t kV = 4;                  // floats per lane per row (one 16-byte access)
constexpr uint32_t kR = 64;                 // rows per chunk
constexpr uint32_t kRowElems = kW * kV;     // 256
constexpr uint32_t kChunk = kRowElems * kR; // 16384 elements
constexpr uint32_t kHeaderBytes = 512;
constexpr uint32_t kLaneBitsWords = (2 * kW) / 4;   // 32 words of u16 lane lengths per chunk record
constexpr uint32_t kMaxSym = 16;
constexpr uint32_t kExtCopies = 16;
enum ElemType { kF32 = 0, kBF16 = 1, kF16 = 2, kF64 = 3 };   // element type of the parameter arrays (= LC_F32 ...)
constexpr uint32_t kDecLut1Bits = 7;        // first decode table: conflict-free in LDS
constexpr uint32_t kDecLut2Bits = 12;       // second decode table, for codes of 8..12 bits

// Written by the table kernel, read by pack / finalize.
struct Table {
    uint32_t K;              // kept buckets; zero symbol = K
    uint32_t max_len;
    uint32_t status;         // lc_status of the encode so far
    uint32_t k_E;            // non-empty buckets before promotion
    uint32_t codelen[kMaxSym];   // (code << 5) | len, per symbol
    uint32_t kept[kMaxSym];      // bucket id of symbol j < K
    uint64_t cnt[kMaxSym];
    uint8_t  symlen_of_bucket[512];   // low nibble symbol, high nibble code length
    uint32_t min_kept_exp;            // smallest biased exponent among the kept buckets (256: none kept)
    uint32_t pad_t;
};

// Written by the decode-prepare kernel.
struct DecInfo {
    uint32_t K, max_len, pad[2];
    uint64_t area;           // byte offset of the chunk area
    uint64_t total_words;    // chunk area size in 32-bit words
    uint32_t rep_bits[kMaxSym];
    uint32_t len[kMaxSym], code[kMaxSym];
    uint32_t rep_hi[kMaxSym];    // binary64 blobs: high halves of the representatives (rep_bits holds the low halves)
};

constexpr int kMaxMany = 8;  // blobs one fused restore sweep can apply
constexpr int kMaxSets = 64; // blobs one lc_decode_many call accepts (= LC_MAX_MANY), each with a set of its own

// Everything the decode sweep needs to know about one blob, written by k_dec_check.
struct DecSet {
    DecInfo info;
    alignas(16) uint8_t lut1[1u << kDecLut1Bits];   // symbol | len << 4 over the next 7 bits
    alignas(16) uint8_t lut2[1u << kDecLut2Bits];   // ... over the next 12 bits
};

struct Result {
    uint64_t bytes;
    uint32_t status;
    uint32_t used_cache;     // lc_encode_cached: 1 if the blob carries the cached code table
    uint32_t listed;         // chunks sweep 2 had to read (the others hold the merged symbol only)
    uint32_t pad_r;
};

// Caller-owned device memory of lc_encode_cached (LC_CACHE_BYTES, all-zero = empty): the kept set and
// the code lengths of the last blob encoded with it.
struct TableCache {
    uint32_t valid, nbits, K, pad;
    uint32_t kept[kMaxSym];
    uint32_t len[kMaxSym];
};

// Lives in mapped, pinned host memory, one per call in progress: kernels write the outcome of the call here with
// plain stores, and the host reads it after waiting for the stream.
struct HostResult {
    Result enc;                                  // encode calls: blob bytes, lc_status, ...
    unsigned long long dec_status;               // lc_decode*: (epoch << 8) | lc_status of the worst finding
    unsigned long long bytes[kMaxSets];          // lc_decode*: total_bytes of each blob
    uint32_t max_len[kMaxSets];                  // lc_decode*: longest code of each blob
};

// What the encode kernels of one vector share: bucket populations, extremes of the kept buckets, the
// code table.  One per call; a batched call (one table per tensor) has one per tensor.
struct EncState {
    unsigned long long hist[512];
    uint32_t mmin[kExtCopies][kMaxSym];      // smallest / largest mantissa seen of every kept bucket: a workgroup of the coding
    uint32_t mmax[kExtCopies][kMaxSym];      // sweep updates copy (its index mod kExtCopies), the workgroup that writes the header joins them
    uint32_t spec;                   // lc_encode_cached: the table in `table` comes from the cache and the sweep coded with it
    uint32_t spec_ok;                // ... and this checkpoint's statistics confirmed it: the blob is already in the slots
    uint32_t list_count;             // entries of chunk_list (the chunks sweep 2 has to read), written by k_table
    uint32_t pad_e;
    Table table;
};

// Fixed part of the per-device scratch.  It is followed by group_words[kMaxGroups] and
// chunk_maxexp[kMaxChunks] (u32, at fixed places so that they can be left cleared from one call to the
// next), chunk_list[kMaxChunks] (u32), chunk_bits[num_chunks] (u32, padded to 256 bytes), one slot of
// slot_words_of(nbits) 32-bit words per chunk and, 256-byte aligned behind the slots, kPartMaxBytes per chunk for the
// largest exponent of every 4 KiB batch of sweep 1.
// What an encode of binary64 parameters keeps instead of EncState's counts, extremes and bucket map: 2^12
// (sign, exponent) buckets, 52-bit mantissas (Section 3.1.1, footnote on the bucket count).  Left cleared like them.
constexpr uint32_t kBuckets64 = 4096;
struct Ext64 {
    unsigned long long hist[kBuckets64];
    unsigned long long mmin[kMaxSym], mmax[kMaxSym];
    uint8_t symlen_of_bucket[kBuckets64];
};

struct Workspace : EncState {
    unsigned long long dec_status;   // (epoch << 8) | lc_status, raised with atomicMax
    DecSet dec_set[kMaxSets];        // one per blob of the call
    Ext64 ext64;
    // An encode with staged keys: smallest / largest delta bit pattern of every (sign, exponent) bucket, gathered by
    // sweep 1 (which is then the only sweep that sees the mantissas).  Left cleared (all ones / zero) like the rest.
    uint32_t bucket_min[512], bucket_max[512];
};

constexpr size_t kWorkspaceFixed = (sizeof(Workspace) + 255) / 256 * 256;
constexpr uint32_t kMaxGroups = 4096;       // 2^32 elements / 16384 per chunk / 64 chunks per group
constexpr uint32_t kMaxChunks = 1u << 18;   // 2^32 elements / 16384 per chunk
// fixed part + group_words[kMaxGroups] + chunk_maxexp[kMaxChunks] (largest biased exponent of |delta| per chunk,
// written by sweep 1, kept cleared between calls like group_words) + chunk_list[kMaxChunks] (the chunks that
// sweep 2 has to read, in no particular order)
constexpr size_t kWorkspaceHead = kWorkspaceFixed + 4 * kMaxGroups + 8 * (size_t)kMaxChunks;

__host__ __device__ inline uint64_t num_chunks_of(uint64_t n) { return (n + kChunk - 1) / kChunk; }
// Slot of one chunk in the scratch area: 64 lane lengths (u16), then up to 8 * max_len words
// per lane (256 codes of at most max_len = 2^nbits - 1 bits), word k of lane l at [32 + 64 k + l].
__host__ __device__ inline uint32_t slot_words_of(int nbits) { return kLaneBitsWords + kW * 8u * ((1u << nbits) - 1u); }
__host__ __device__ inline uint64_t chunk_area_of(uint64_t nchunks) { return kHeaderBytes + (4 * (nchunks + 1) + 15) / 16 * 16; }

enum Slot { kSlotReset = 0, kSlotHist, kSlotTable, kSlotPack, kSlotPlace, kSlotSpecTable, kSlotSpecSweep,
            kSlotDecCheck, kSlotDecode, kSlotDecodeFused, kSlotHistKeys, kSlotPackKeys, kSlotVerify, kNumSlots };

// Launch shapes; defaults chosen by measurement, overridable through LC_TUNE_* environment
// variables (read once) for sweeps.
struct Tuning {
    int num_cu = 256;
    int hist_blocks_per_cu = 1;
    int hist_threads = 256;
    int pack_waves_per_cu = 8;         // single-wave workgroups of k_pack per compute unit
    int keys_waves_per_cu = 10;        // ... of the sweep that codes from staged keys (3 fit a SIMD; 10 measured best)
    int key_staging = 0;               // 0: by the vector's last call, 1: whenever it applies, 2: never
    int spec_waves_per_cu = 8;         // of the single sweep of the cached encode (what its LDS and registers allow)
    int batch_waves_per_cu = 8;        // of the batch kernels
    int decode_blocks_per_cu = 9;     // (LDS lets 4 run at once; more, smaller shares even out chunks that decode to nothing)
    int fused_waves_per_cu = 16;       // most wavefronts per compute unit
    int fused_min_waves_per_cu = 8;    // a sweep takes as many blobs as still leave LDS for this many
};

// Launchers (lc_encode.hip, lc_decode.hip).
void launch_reset(Workspace* ws, uint32_t* group_words, uint32_t* chunk_maxexp, hipStream_t s);
void launch_reset_chunks(Workspace* ws, uint32_t* group_words, uint32_t* chunk_maxexp, uint32_t nchunks, hipStream_t s);
// The keys of an encode with staged keys (fp32, 16-byte aligned arrays): sweep 1 leaves, for every whole batch of 4 rows
// (1024 elements) and lane, the 16 exponent bytes of the lane's elements (row-major: byte 4 k + v = row k, element v) and
// their 16 sign bits, and sweep 2 codes from those 9 bits per element instead of reading w and w_ref again.
struct KeyPlanes {
    uint8_t* exp;            // 16 bytes per lane and batch: [batch][lane][16]   (null: no staging)
    uint16_t* sign;          // 16 bits per lane and batch:  [batch][lane]
};
constexpr uint32_t kKeyBatch = 4 * kRowElems;          // elements per batch
__host__ __device__ inline uint64_t key_exp_bytes(uint64_t n) { return (n / kKeyBatch) * kKeyBatch; }
__host__ __device__ inline uint64_t key_sign_bytes(uint64_t n) { return (n / kKeyBatch) * (kKeyBatch / 8); }
void launch_hist(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_maxexp, uint8_t* batch_max,
                 KeyPlanes keys, const Tuning& tune, hipStream_t s);
void launch_pack_keys(const void* w, const void* w_ref, uint64_t n, Workspace* ws, uint32_t* chunk_bits, uint32_t* group_words,
                      const uint32_t* chunk_maxexp, const uint32_t* chunk_list, KeyPlanes keys, uint32_t* prov, uint32_t slot_words,
                      const Tuning& tune, hipStream_t s);
void launch_table(Workspace* ws, uint64_t n, int nbits, int dtype, uint32_t* group_words, const uint32_t* chunk_maxexp,
                  uint32_t* chunk_list, hipStream_t s);
void launch_spec_table(Workspace* ws, const TableCache* cache, uint64_t n, int nbits, int dtype, uint32_t* group_words, hipStream_t s);
void launch_spec_sweep(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                       uint32_t* group_words, uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s);
void launch_pack(const void* w, const void* w_ref, uint64_t n, int dtype, Workspace* ws, uint32_t* chunk_bits,
                 uint32_t* group_words, const uint32_t* chunk_maxexp, const uint32_t* chunk_list, const uint8_t* batch_max,
                 uint32_t* prov, uint32_t slot_words, const Tuning& tune, hipStream_t s);
void launch_place(uint8_t* out, Workspace* ws, const uint32_t* chunk_bits, const uint32_t* group_words,
                  const uint32_t* prov, uint32_t slot_words, uint64_t n, uint32_t* chunk_maxexp, Result* host_result,
                  TableCache* cache, int nbits, int dtype, bool staged, hipStream_t s);
// One tensor of a batched call (lc_encode_batch): every tensor has its own EncState, blob and run of
// chunks; chunks, groups of 64 chunks and slots of all tensors are numbered through ("dense" indices).
struct Seg {
    const void* w; const void* w_ref; uint8_t* out;
    uint64_t n;
    uint32_t nchunks, chunk0, group0, aligned;
};
constexpr int kMaxBatch = 1024;
constexpr uint32_t kPartBytes = 16;
// ... of a single-vector call: one byte per 4 KiB part (16 parts of 4-byte elements, 8 of 2-byte), two bytes each for the
// 32 parts of 8-byte elements
constexpr uint32_t kPartMaxBytes = 64;
struct BatchArgs {
    Seg* segs; EncState* states; Result* results;     // device (results: mapped host memory)
    uint32_t* seg_of_chunk; uint32_t* group_words; uint32_t* chunk_bits; uint32_t* prov;
    uint32_t* chunk_maxexp;      // largest |delta| exponent of every chunk (chunks of all tensors numbered through), from the counting sweep
    uint8_t* part_max;           // ... and of each of its 4 KiB parts: kPartBytes per chunk (16 parts of 4-byte elements, 8 of 2-byte)
    uint32_t* chunk_list;        // the chunks the coding sweep has to read, and
    uint32_t* list_count;        // how many those are
    uint32_t count, total_chunks, total_groups, slot_words;
    int nbits, dtype;                                  // dtype: element type of every tensor of the call
    uint32_t waves_long, pad_b;                        // wavefronts of the coding sweep when more chunks are listed than its grid has
};
void launch_batch_encode(const BatchArgs& a, const Tuning& tune, hipStream_t s);

// lc_decode_batch: one blob and one vector per tensor.
struct SegD {
    const uint8_t* blob; void* w_ref;
    uint64_t n;
    uint32_t nchunks, chunk0, aligned, pad;
};
struct BatchDecArgs {
    SegD* segs; DecSet* sets; Result* results;         // device (results: mapped host memory)
    uint32_t* seg_of_chunk; uint32_t* seg_status;      // seg_status: lc_status per tensor, raised with atomicMax
    uint32_t* chunk_info;                              // per chunk {tensor, chunk index there, its two offset-table entries}, 16 bytes
    uint32_t count, total_chunks;
    int dtype, pad;
};
void launch_batch_decode(const BatchDecArgs& a, const Tuning& tune, hipStream_t s);

struct BlobList { const uint8_t* p[kMaxSets]; };
// Checks blobs.p[first .. first+count) into dec_set[first ..] and host->bytes / max_len[first ..].
void launch_dec_check(const BlobList& blobs, int first, int count, uint64_t n, int dtype, uint64_t max_total, Workspace* ws,
                      uint64_t epoch, HostResult* host, hipStream_t s);
// (set: which of the workspace's decode sets the check kernel filled for this blob; w_ref null: only verify the lane strings)
void launch_decode(const uint8_t* blob, void* w_ref, uint64_t n, int dtype, Workspace* ws, int set, uint64_t epoch, HostResult* host,
                   const Tuning& tune, hipStream_t s);
// Both apply blobs.p[first .. first+count), count <= kMaxMany, using dec_set[first ..]; the fused
// kernel requires every code of these blobs to be at most kDecLut1Bits long.
// pay_words: LDS words each wavefront gets for the payloads of one chunk of all `count` blobs.
void launch_decode_fused(const BlobList& blobs, int first, int count, void* w_ref, uint64_t n, int dtype, Workspace* ws,
                         uint64_t epoch, HostResult* host, uint32_t pay_words, bool long_codes, const Tuning& tune,
                         hipStream_t s);

constexpr uint32_t kLdsPerCu = 160 * 1024;        // gfx950
constexpr uint32_t kFusedMinWords = 1024;
// LDS bytes one wavefront (= workgroup) of the fused kernel takes for `count` blobs and pay_words payload words.
size_t fused_lds_bytes(int count, uint32_t pay_words);

}  // namespace lc
