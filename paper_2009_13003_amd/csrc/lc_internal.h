// Shared between the kernels (lc_kernels.hip) and the host API (lc_api.hip):
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
constexpr uint32_t kMaxLutBits = 15;

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
};

// Written by the decode-prepare kernel.
struct DecInfo {
    uint32_t K, max_len, num_chunks, status;
    uint64_t area;           // byte offset of the chunk area
    uint64_t total_words;    // chunk area size in 32-bit words
    uint32_t rep_bits[kMaxSym];
};

struct Result {              // copied to pinned host memory at the end of a call
    uint64_t bytes;
    uint32_t status;
    uint32_t pad;
};

// Fixed part of the per-device scratch; the per-chunk scan state follows it.
struct Workspace {
    unsigned long long hist[512];
    uint32_t mmin[kMaxSym];
    uint32_t mmax[kMaxSym];
    uint32_t ticket;
    uint32_t dec_status;
    unsigned long long total_words;
    Table table;
    DecInfo dec;
    Result result;
    alignas(16) uint8_t dec_lut[1u << kMaxLutBits];
};

constexpr size_t kWorkspaceFixed = (sizeof(Workspace) + 255) / 256 * 256;

__host__ __device__ inline uint64_t num_chunks_of(uint64_t n) { return (n + kChunk - 1) / kChunk; }
__host__ __device__ inline uint64_t chunk_area_of(uint64_t nchunks) { return kHeaderBytes + (4 * (nchunks + 1) + 15) / 16 * 16; }

enum Slot { kSlotReset = 0, kSlotHist, kSlotTable, kSlotPack, kSlotFinalize,
            kSlotDecPrep, kSlotDecValidate, kSlotDecode, kNumSlots };

// Launchers (lc_kernels.hip).  `state` is the per-chunk scan state (num_chunks u64).
void launch_reset(Workspace* ws, unsigned long long* state, uint64_t nchunks, hipStream_t s);
void launch_hist(const float* w, const float* w_ref, uint64_t n, Workspace* ws, int num_cu, hipStream_t s);
void launch_table(Workspace* ws, uint64_t n, int nbits, hipStream_t s);
void launch_pack(const float* w, const float* w_ref, uint64_t n, uint8_t* out, Workspace* ws,
                 unsigned long long* state, int num_cu, hipStream_t s);
void launch_finalize(uint8_t* out, Workspace* ws, uint64_t n, int nbits, hipStream_t s);
void launch_dec_prepare(const uint8_t* blob, uint64_t n, uint64_t max_total, Workspace* ws, hipStream_t s);
void launch_dec_validate(const uint8_t* blob, uint64_t n, Workspace* ws, hipStream_t s);
void launch_decode(const uint8_t* blob, float* w_ref, uint64_t n, Workspace* ws, uint32_t max_len,
                   int num_cu, hipStream_t s);

}  // namespace lc
