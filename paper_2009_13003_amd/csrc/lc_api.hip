// Host side of the C ABI declared in include/lc.h: argument checks, per-device scratch,
// launch order, the small size/status read-back, optional per-kernel event timing.
// No step of the method runs here.
#include "../../include/lc.h"
#include "../../include/lc_bench.h"
#include "lc_internal.h"

#include <mutex>
#include <stdlib.h>
#include <string.h>

namespace {

using namespace lc;

constexpr int kMaxDevices = 16;

constexpr int kHintBits = 10, kHints = 1 << kHintBits;
struct DeviceState {
    void* owned = nullptr;       // library-owned scratch
    size_t owned_bytes = 0;
    void* user = nullptr;        // caller-supplied scratch (lc_set_workspace)
    size_t user_bytes = 0;
    Tuning tune;
    bool tuned = false;
    const void* clean = nullptr;  // scratch area whose encode state is known to be cleared
    hipEvent_t last = nullptr;    // end of the latest asynchronous call on this device
    bool pending = false;         // ... which later calls must order themselves after (they share the scratch)
    // What the last encode of a vector (told apart by address and length) found: the share of its chunks that sweep 2
    // had to read.  Decides whether the next encode of that vector stages keys (see stage_keys()).
    struct Hint { const void* w = nullptr; uint64_t n = 0; float listed = 0; };
    Hint hint[kHints];
};

// lc_encode_async: a call in flight.
constexpr int kMaxTickets = 16;
struct Ticket {
    bool busy = false;
    int dev = 0; const void* w = nullptr; uint64_t n = 0;   // whose hint its outcome updates
    hipEvent_t inputs = nullptr;  // after the last kernel that reads w / w_ref
    hipEvent_t done = nullptr;    // after the last kernel
};
Ticket g_ticket[kMaxTickets];

// lc_encode_batch: pinned host memory for the tensor list on its way to the device and for the
// per-tensor outcomes the kernels write (mapped).
struct BatchHost {
    union { Seg segs[kMaxBatch]; SegD dsegs[kMaxBatch]; };
    Result results[kMaxBatch];
};
BatchHost* g_batch = nullptr;
BatchHost* g_batch_dev = nullptr;
static_assert(sizeof(((HostResult*)0)->enc_async) / sizeof(Result) == kMaxTickets, "one result per ticket");

std::mutex g_mu;
DeviceState g_dev[kMaxDevices];
static_assert(sizeof(TableCache) <= LC_CACHE_BYTES, "LC_CACHE_BYTES too small");
static_assert(sizeof(((HostResult*)0)->bytes) / sizeof(unsigned long long) >= LC_MAX_MANY, "HostResult too small");
HostResult* g_pinned = nullptr;  // mapped pinned host memory the kernels write their outcome to
HostResult* g_pinned_dev = nullptr;   // the same memory as the device sees it
uint64_t g_epoch = 0;            // tags the decode status word of each call

int g_key_staging = -1;          // LC_OPT_KEY_STAGING (-1: not yet read from the environment)
bool g_prof = false;
double g_prof_ms[kNumSlots];
uint64_t g_prof_n[kNumSlots];
hipEvent_t g_ev[kNumSlots][2];
bool g_ev_made = false;
const char* const kSlotNames[kNumSlots] = {"k_reset", "k_hist", "k_table", "k_pack", "k_place", "k_finalize", "k_spec_table", "k_spec_sweep",
                                           "k_dec_check", "k_decode", "k_decode_fused", "k_hist_keys", "k_pack_keys"};

int env_int(const char* name, int dflt, int lo, int hi) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    const long x = strtol(v, nullptr, 10);
    return x < lo ? lo : (x > hi ? hi : (int)x);
}

#define LC_HIP(call) do { if ((call) != hipSuccess) { (void)hipGetLastError(); return -(lc_ssize)LC_ERR_HIP; } } while (0)

struct Timed {                   // records a pair of events around a launch when profiling is on
    int slot; hipStream_t s; bool on;
    Timed(int slot_, hipStream_t s_) : slot(slot_), s(s_), on(g_prof) { if (on) (void)hipEventRecord(g_ev[slot][0], s); }
    ~Timed() { if (on) (void)hipEventRecord(g_ev[slot][1], s); }
};

void collect(const int* slots, int count) {   // after the stream has been waited for
    if (!g_prof) return;
    for (int i = 0; i < count; ++i) {
        float ms = 0;
        if (hipEventElapsedTime(&ms, g_ev[slots[i]][0], g_ev[slots[i]][1]) == hipSuccess) {
            g_prof_ms[slots[i]] += ms; g_prof_n[slots[i]] += 1;
        } else (void)hipGetLastError();
    }
}

// Launch shapes of a device: the compute unit count and the LC_TUNE_* overrides, read once.  Allocates nothing.
void read_tuning(DeviceState& ds, int dev) {
    if (ds.tuned) return;
    int cu = 0;
    if (hipDeviceGetAttribute(&cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cu <= 0) { (void)hipGetLastError(); cu = 256; }
    ds.tune.num_cu = cu;
    ds.tune.hist_blocks_per_cu = env_int("LC_TUNE_HIST_BLOCKS_PER_CU", ds.tune.hist_blocks_per_cu, 1, 64);
    ds.tune.hist_threads = env_int("LC_TUNE_HIST_THREADS", ds.tune.hist_threads, 64, 1024) / 64 * 64;
    ds.tune.pack_waves_per_cu = env_int("LC_TUNE_PACK_WAVES_PER_CU", ds.tune.pack_waves_per_cu, 1, 64);
    ds.tune.spec_waves_per_cu = env_int("LC_TUNE_SPEC_WAVES_PER_CU", ds.tune.spec_waves_per_cu, 1, 64);
    ds.tune.keys_waves_per_cu = env_int("LC_TUNE_KEYS_WAVES_PER_CU", ds.tune.keys_waves_per_cu, 1, 64);
    if (g_key_staging < 0) g_key_staging = env_int("LC_TUNE_KEY_STAGING", 0, 0, 2);
    ds.tune.batch_waves_per_cu = env_int("LC_TUNE_BATCH_WAVES_PER_CU", ds.tune.batch_waves_per_cu, 1, 64);
    ds.tune.decode_blocks_per_cu = env_int("LC_TUNE_DECODE_BLOCKS_PER_CU", ds.tune.decode_blocks_per_cu, 1, 64);
    ds.tune.fused_waves_per_cu = env_int("LC_TUNE_FUSED_WAVES_PER_CU", ds.tune.fused_waves_per_cu, 1, 32);
    ds.tune.fused_min_waves_per_cu = env_int("LC_TUNE_FUSED_MIN_WAVES_PER_CU", ds.tune.fused_min_waves_per_cu, 1, 32);
    ds.tuned = true;
}

// Scratch for the current device, at least `need` bytes.  Returns nullptr with *err set.
Workspace* get_workspace(size_t need, int* err, DeviceState** ds_out) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); *err = LC_ERR_HIP; return nullptr; }
    DeviceState& ds = g_dev[dev];
    read_tuning(ds, dev);
    if (!g_pinned) {
        if (hipHostMalloc(reinterpret_cast<void**>(&g_pinned), sizeof(HostResult), hipHostMallocMapped | hipHostMallocPortable) != hipSuccess ||
            hipHostGetDevicePointer(reinterpret_cast<void**>(&g_pinned_dev), g_pinned, 0) != hipSuccess) {
            (void)hipGetLastError();
            if (g_pinned) (void)hipHostFree(g_pinned);
            g_pinned = nullptr; *err = LC_ERR_HIP; return nullptr;
        }
        memset(g_pinned, 0, sizeof(HostResult));
    }
    *ds_out = &ds;
    if (ds.user) {
        if (ds.user_bytes < need) { *err = LC_ERR_WORKSPACE; return nullptr; }
        return static_cast<Workspace*>(ds.user);
    }
    if (ds.owned_bytes < need) {
        if (ds.owned) { (void)hipDeviceSynchronize(); (void)hipFree(ds.owned); ds.owned = nullptr; ds.owned_bytes = 0; }
        size_t want = need < (4u << 20) ? (4u << 20) : need;     // never smaller than the head that is cleared below
        static_assert(kWorkspaceHead <= (4u << 20), "the smallest scratch area must hold the fixed head");
        if (hipMalloc(&ds.owned, want) != hipSuccess) { (void)hipGetLastError(); ds.owned = nullptr; *err = LC_ERR_HIP; return nullptr; }
        if (hipMemset(ds.owned, 0, kWorkspaceHead) != hipSuccess) { (void)hipGetLastError(); (void)hipFree(ds.owned); ds.owned = nullptr; *err = LC_ERR_HIP; return nullptr; }
        ds.owned_bytes = want;
        ds.clean = nullptr;      // new memory (possibly at the old address): its encode state is not set up yet
    }
    return static_cast<Workspace*>(ds.owned);
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Bytes of scratch an encode of nc chunks at nbits takes (what lc_workspace_bytes reports), and where its parts lie.
constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }
constexpr size_t encode_scratch_bytes(uint64_t nc, int nbits) {
    return kWorkspaceHead + up256(4 * nc) + (size_t)(nc * (kLaneBitsWords + kW * 8u * ((1u << nbits) - 1u)) * 4) +
           256 + up256(16 * nc);                                  // + the per-batch maxima of sweep 1
}
// ... and with staged keys behind that: a byte and a bit per element of every whole batch
size_t staged_scratch_bytes(uint64_t n, int nbits) {
    return encode_scratch_bytes(num_chunks_of(n), nbits) + up256(key_exp_bytes(n)) + up256(key_sign_bytes(n));
}
struct Scratch {
    Workspace* ws;
    uint32_t *group_words, *chunk_maxexp, *chunk_list, *chunk_bits, *prov;
    uint8_t* batch_max;                                           // one byte per 4 KiB batch of sweep 1 (16 per chunk at most), behind the slots
    uint32_t slot_words;
    Scratch(void* base, uint64_t nc, int nbits) {
        ws = static_cast<Workspace*>(base);
        group_words = reinterpret_cast<uint32_t*>(static_cast<uint8_t*>(base) + kWorkspaceFixed);
        chunk_maxexp = group_words + kMaxGroups;
        chunk_list = chunk_maxexp + kMaxChunks;
        chunk_bits = chunk_list + kMaxChunks;
        prov = chunk_bits + (nc + 63) / 64 * 64;
        slot_words = slot_words_of(nbits);
        batch_max = reinterpret_cast<uint8_t*>((reinterpret_cast<uintptr_t>(prov + nc * slot_words) + 255) & ~(uintptr_t)255);
    }
    KeyPlanes keys(uint64_t n) const {                            // (only an area of staged_scratch_bytes has them)
        const uint64_t nc = num_chunks_of(n);
        uint8_t* e = batch_max + up256(16 * nc);
        return KeyPlanes{e, reinterpret_cast<uint16_t*>(e + up256(key_exp_bytes(n)))};
    }
};

// Every call uses the device's one scratch area: work enqueued on `s` must not start before the
// latest asynchronous call has finished with it.
bool order_after_async(DeviceState* ds, hipStream_t s) {
    if (!ds->pending) return true;
    if (hipStreamWaitEvent(s, ds->last, 0) != hipSuccess) { (void)hipGetLastError(); return false; }
    return true;
}

}  // namespace

extern "C" {

size_t lc_encode_bound(uint64_t n, int nbits) {
    if (nbits < 1 || nbits > 4 || n > LC_MAX_N) return 0;
    const uint64_t nc = num_chunks_of(n);
    return (size_t)(chunk_area_of(nc) + nc * (2 * kW + 4) + (n * (uint64_t)nbits + 7) / 8);
}

size_t lc_workspace_bytes(uint64_t n, int nbits) {
    if (nbits < 1 || nbits > 4 || n > LC_MAX_N) return 0;
    return encode_scratch_bytes(num_chunks_of(n), nbits);
}

int lc_set_workspace(void* dev_ws, size_t bytes) {
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return LC_ERR_HIP; }
    if (dev_ws && (misaligned(dev_ws, 256) || bytes < kWorkspaceHead)) return LC_ERR_WORKSPACE;
    if (dev_ws && hipMemset(dev_ws, 0, kWorkspaceHead) != hipSuccess) { (void)hipGetLastError(); return LC_ERR_HIP; }
    g_dev[dev].user = dev_ws;
    g_dev[dev].user_bytes = dev_ws ? bytes : 0;
    g_dev[dev].clean = nullptr;
    return LC_OK;
}

}  // extern "C"

namespace {
// Whether this encode stages keys: sweep 1 then also writes 9 bits per element and sweep 2 reads those instead of w
// and w_ref again (10.25 + c/8 bytes per element moved instead of 16 + c/8).  That pays when sweep 2 has to read most
// of the vector; when it passes over most chunks (sparse updates) the plain second sweep is cheaper, since the keys
// of chunks nobody reads are written for nothing.  How much sweep 2 reads is known only after sweep 1, so the choice
// follows what the last encode of the same vector found (a training loop checkpoints the same tensors again and
// again); a vector seen for the first time takes the plain path.  The blob is the same either way.
DeviceState::Hint* hint_of(DeviceState* ds, const void* w, uint64_t n) {
    const uint64_t key = ((uint64_t)reinterpret_cast<uintptr_t>(w) + n) * 0x9E3779B97F4A7C15ull;   // (slices lie 2^30 bytes apart)
    return &ds->hint[key >> (64 - kHintBits)];
}
// Measured on 2^28-element calls: staging costs sweep 1 0.06 to 0.11 ms (the key writes) and saves sweep 2 0.27 ms
// times the share of chunks it has to read; below some 2^26 elements the sweeps are too short for either to show.
constexpr float kStageAbove = 0.30f;
constexpr uint64_t kStageFromN = 1ull << 26;
bool stage_keys(DeviceState* ds, const void* w, const void* w_ref, uint64_t n, int dtype, bool cached) {
    if (dtype != LC_F32 || cached || n < kChunk || misaligned(w, 16) || misaligned(w_ref, 16)) return false;
    if (g_key_staging == 1) return true;
    if (g_key_staging == 2 || n < kStageFromN) return false;
    const DeviceState::Hint* h = hint_of(ds, w, n);
    return h->w == w && h->n == n && h->listed > kStageAbove;
}
void note_outcome(DeviceState* ds, const void* w, uint64_t n, const Result& r) {
    if (r.status != LC_OK || n < kChunk) return;
    DeviceState::Hint* h = hint_of(ds, w, n);
    h->w = w; h->n = n; h->listed = (float)r.listed / (float)num_chunks_of(n);
}

// lc_encode (cache == nullptr: two sweeps) and lc_encode_cached (one sweep that counts and, when the
// cache holds a usable table, codes with it; k_table confirms or voids that, and only then does the
// second sweep have anything to do).
lc_ssize encode_impl(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, TableCache* cache,
                     int* used, void* stream, bool async) {
    if (nbits < 1 || nbits > 4 || n > LC_MAX_N || !out || misaligned(out, 16)) return -LC_ERR_BADARG;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    if (dtype == LC_F64 && (cache || async)) return -LC_ERR_BADARG;          // those forms code the fp32 delta only
    const uintptr_t esize = dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2;
    if (n && (!w || !w_ref || misaligned(w, esize) || misaligned(w_ref, esize))) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0; DeviceState* ds = nullptr;
    Workspace* ws = get_workspace(lc_workspace_bytes(n, nbits), &err, &ds);
    if (!ws) return -(lc_ssize)err;
    bool staged = stage_keys(ds, w, w_ref, n, dtype, cache != nullptr);
    if (staged) {
        // the key planes lie behind the usual scratch; a caller's area that has no room for them keeps the plain path
        Workspace* bigger = get_workspace(staged_scratch_bytes(n, nbits), &err, &ds);
        if (bigger) ws = bigger; else staged = false;
    }
    hipStream_t s = static_cast<hipStream_t>(stream);
    const Scratch sc(ws, num_chunks_of(n), nbits);
    const KeyPlanes keys = staged ? sc.keys(n) : KeyPlanes{nullptr, nullptr};
    uint32_t *group_words = sc.group_words, *chunk_maxexp = sc.chunk_maxexp, *chunk_list = sc.chunk_list, *chunk_bits = sc.chunk_bits,
             *prov = sc.prov;
    const uint32_t slot_words = sc.slot_words;
    uint8_t* batch_max = sc.batch_max;
    uint8_t* o = static_cast<uint8_t*>(out);
    int ticket = -1;
    if (async) {
        for (int i = 0; i < kMaxTickets && ticket < 0; ++i) if (!g_ticket[i].busy) ticket = i;
        if (ticket < 0) return -LC_ERR_BADARG;                       // too many calls in flight
        Ticket& tk = g_ticket[ticket];
        if (!tk.done) {
            if (hipEventCreateWithFlags(&tk.inputs, hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&tk.done, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); tk.inputs = tk.done = nullptr; return -LC_ERR_HIP; }
        }
        if (!ds->last && hipEventCreateWithFlags(&ds->last, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); ds->last = nullptr; return -LC_ERR_HIP; }
    }
    if (!order_after_async(ds, s)) return -LC_ERR_HIP;
    Result* result = async ? &g_pinned_dev->enc_async[ticket] : &g_pinned_dev->enc;
    // Every call leaves the encode state cleared behind it; a fresh scratch area, or one whose last
    // call did not run to its end, is cleared first.
    if (ds->clean != ws) { Timed t(kSlotReset, s); launch_reset(ws, group_words, chunk_maxexp, s); }
    ds->clean = nullptr;
    if (cache) {
        { Timed t(kSlotSpecTable, s); launch_spec_table(ws, cache, nbits, s); }
        { Timed t(kSlotSpecSweep, s); launch_spec_sweep(w, w_ref, n, dtype, ws, chunk_bits, group_words, prov, slot_words, ds->tune, s); }
    } else {
        Timed t(staged ? kSlotHistKeys : kSlotHist, s); launch_hist(w, w_ref, n, dtype, ws, chunk_maxexp, batch_max, keys, ds->tune, s);
    }
    { Timed t(kSlotTable, s);    launch_table(ws, n, nbits, dtype, group_words, chunk_maxexp, cache ? nullptr : chunk_list, s); }
    if (staged) { Timed t(kSlotPackKeys, s); launch_pack_keys(w, w_ref, n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list, keys, prov, slot_words, ds->tune, s); }
    else { Timed t(kSlotPack, s); launch_pack(w, w_ref, n, dtype, ws, chunk_bits, group_words, chunk_maxexp, cache ? nullptr : chunk_list, batch_max, prov, slot_words, ds->tune, s); }
    if (async) LC_HIP(hipEventRecord(g_ticket[ticket].inputs, s));   // w and w_ref are not read past this point
    { Timed t(kSlotPlace, s);    launch_place(o, ws, chunk_bits, group_words, prov, slot_words, n, chunk_maxexp, s); }
    { Timed t(kSlotFinalize, s); launch_finalize(o, ws, result, group_words, cache, n, nbits, dtype, staged, s); }
    LC_HIP(hipGetLastError());
    if (async) {
        LC_HIP(hipEventRecord(g_ticket[ticket].done, s));
        LC_HIP(hipEventRecord(ds->last, s));
        ds->pending = true;
        ds->clean = ws;              // later calls are ordered after this one
        Ticket& tk = g_ticket[ticket];
        tk.busy = true;
        tk.dev = (int)(ds - g_dev); tk.w = cache ? nullptr : w; tk.n = n;
        return ticket;
    }
    LC_HIP(hipStreamSynchronize(s));
    ds->pending = false;             // this call was ordered after every asynchronous one
    ds->clean = ws;
    const int slots[] = {cache ? kSlotSpecTable : staged ? kSlotHistKeys : kSlotHist, kSlotTable, staged ? kSlotPackKeys : kSlotPack,
                         kSlotPlace, kSlotFinalize, kSlotSpecSweep};
    collect(slots, cache ? 6 : 5);
    if (!cache && dtype == LC_F32) note_outcome(ds, w, n, g_pinned->enc);
    if (used) *used = (int)g_pinned->enc.used_cache;
    if (g_pinned->enc.status != LC_OK) return -(lc_ssize)g_pinned->enc.status;
    return (lc_ssize)g_pinned->enc.bytes;
}
}  // namespace

extern "C" {

lc_ssize lc_encode(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* stream) {
    return encode_impl(w, w_ref, n, nbits, out, LC_F32, nullptr, nullptr, stream, false);
}

}  // extern "C"

// ---- lc_encode_static: the scratch area lives in the library's own device image
namespace {
constexpr uint64_t kStaticChunks = LC_STATIC_MAX_N / kChunk;
static_assert(LC_STATIC_MAX_N % kChunk == 0, "whole chunks");
// the scratch of the largest call it accepts (nbits 4), then the call's outcome as the kernels report it
constexpr size_t kStaticResultAt = up256(encode_scratch_bytes(kStaticChunks, 4));
constexpr size_t kStaticBytes = kStaticResultAt + 256;
}  // namespace
static __device__ __align__(256) unsigned char scratch[kStaticBytes];
namespace {
void* g_static[kMaxDevices];      // each device's copy of `scratch`, as hipGetSymbolAddress reports it there
}  // namespace

extern "C" {

int lc_encode_static(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* stream) {
    if (nbits < 1 || nbits > 4 || !out || misaligned(out, 16)) return LC_ERR_BADARG;
    if (n > LC_STATIC_MAX_N) return LC_ERR_WORKSPACE;                 // more than the built-in scratch area holds
    if (n && (!w || !w_ref || misaligned(w, 4) || misaligned(w_ref, 4))) return LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return LC_ERR_HIP; }
    if (!g_static[dev]) {
        // `scratch` itself is no device address on the host side; every device holds its own copy at its own address
        void* ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) { (void)hipGetLastError(); return LC_ERR_HIP; }
        g_static[dev] = ptr;
    }
    DeviceState& ds = g_dev[dev];
    read_tuning(ds, dev);
    hipStream_t s = static_cast<hipStream_t>(stream);
    uint8_t* base = static_cast<uint8_t*>(g_static[dev]);
    const Scratch sc(base, num_chunks_of(n), nbits);
    Result* result = reinterpret_cast<Result*>(base + kStaticResultAt);
    uint8_t* o = static_cast<uint8_t*>(out);
    // The area keeps what the last call on this device left (a call that ran to its end leaves the state cleared,
    // one that was captured and never replayed to its end does not): cleared by a kernel before every call.
    launch_reset_chunks(sc.ws, sc.group_words, sc.chunk_maxexp, (uint32_t)kStaticChunks, s);
    launch_hist(w, w_ref, n, LC_F32, sc.ws, sc.chunk_maxexp, sc.batch_max, KeyPlanes{nullptr, nullptr}, ds.tune, s);
    launch_table(sc.ws, n, nbits, LC_F32, sc.group_words, sc.chunk_maxexp, sc.chunk_list, s);
    launch_pack(w, w_ref, n, LC_F32, sc.ws, sc.chunk_bits, sc.group_words, sc.chunk_maxexp, sc.chunk_list, sc.batch_max, sc.prov,
                sc.slot_words, ds.tune, s);
    launch_place(o, sc.ws, sc.chunk_bits, sc.group_words, sc.prov, sc.slot_words, n, sc.chunk_maxexp, s);
    launch_finalize(o, sc.ws, result, sc.group_words, nullptr, n, nbits, LC_F32, false, s);
    if (hipGetLastError() != hipSuccess) return LC_ERR_HIP;
    return LC_OK;
}

lc_ssize lc_encode_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, void* stream) {
    return encode_impl(w, w_ref, n, nbits, out, dtype, nullptr, nullptr, stream, false);
}

int lc_encode_async_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, void* cache,
                      void* stream) {
    if (cache && misaligned(cache, 16)) return -LC_ERR_BADARG;
    return (int)encode_impl(w, w_ref, n, nbits, out, dtype, static_cast<TableCache*>(cache), nullptr, stream, true);
}

int lc_encode_async(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* cache, void* stream) {
    return lc_encode_async_t(w, w_ref, n, nbits, out, LC_F32, cache, stream);
}

int lc_encode_release_inputs(int ticket, void* other_stream) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (ticket < 0 || ticket >= kMaxTickets || !g_ticket[ticket].busy) return LC_ERR_BADARG;
    if (hipStreamWaitEvent(static_cast<hipStream_t>(other_stream), g_ticket[ticket].inputs, 0) != hipSuccess) { (void)hipGetLastError(); return LC_ERR_HIP; }
    return LC_OK;
}

lc_ssize lc_encode_wait(int ticket, int* used) {
    hipEvent_t done;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (ticket < 0 || ticket >= kMaxTickets || !g_ticket[ticket].busy) return -LC_ERR_BADARG;
        done = g_ticket[ticket].done;
    }
    const hipError_t e = hipEventSynchronize(done);          // not under the lock: other threads may keep calling
    std::lock_guard<std::mutex> lock(g_mu);
    g_ticket[ticket].busy = false;
    if (e != hipSuccess) { (void)hipGetLastError(); return -LC_ERR_HIP; }
    const Result r = g_pinned->enc_async[ticket];
    if (g_ticket[ticket].w) note_outcome(&g_dev[g_ticket[ticket].dev], g_ticket[ticket].w, g_ticket[ticket].n, r);
    if (used) *used = (int)r.used_cache;
    if (r.status != LC_OK) return -(lc_ssize)r.status;
    return (lc_ssize)r.bytes;
}

lc_ssize lc_encode_cached_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, void* cache,
                            int* used, void* stream) {
    if (used) *used = 0;
    if (!cache || misaligned(cache, 16)) return -LC_ERR_BADARG;
    return encode_impl(w, w_ref, n, nbits, out, dtype, static_cast<TableCache*>(cache), used, stream, false);
}

lc_ssize lc_encode_cached(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* cache, int* used,
                          void* stream) {
    return lc_encode_cached_t(w, w_ref, n, nbits, out, LC_F32, cache, used, stream);
}

}  // extern "C"

namespace {
// blob_bytes: what the caller says its buffer holds (SIZE_MAX: not stated); the header's total may not pass it
lc_ssize decode_impl(const void* blob, size_t blob_bytes, void* w_ref, uint64_t n, int dtype, void* stream) {
    if (!blob || misaligned(blob, 16) || n > LC_MAX_N) return -LC_ERR_BADARG;
    if (blob_bytes < kHeaderBytes) return -LC_ERR_BAD_BLOB;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    if (n && (!w_ref || misaligned(w_ref, dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2))) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0; DeviceState* ds = nullptr;
    Workspace* ws = get_workspace(kWorkspaceFixed, &err, &ds);
    if (!ws) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    const uint64_t epoch = ++g_epoch;
    if (!order_after_async(ds, s)) return -LC_ERR_HIP;
    BlobList list;
    for (int t = 0; t < kMaxSets; ++t) list.p[t] = b;
    const uint64_t bound = lc_encode_bound(n, 4), max_total = blob_bytes < bound ? blob_bytes : bound;
    { Timed t(kSlotDecCheck, s); launch_dec_check(list, 0, 1, n, dtype, max_total, ws, epoch, g_pinned_dev, s); }
    { Timed t(kSlotDecode, s);   launch_decode(b, w_ref, n, dtype, ws, epoch, g_pinned_dev, ds->tune, s); }
    LC_HIP(hipGetLastError());
    LC_HIP(hipStreamSynchronize(s));
    ds->pending = false;
    const int slots[] = {kSlotDecCheck, kSlotDecode};
    collect(slots, 2);
    if ((g_pinned->dec_status >> 8) == epoch) return -(lc_ssize)(g_pinned->dec_status & 0xFF);
    return (lc_ssize)g_pinned->bytes[0];
}
}  // namespace

extern "C" {

lc_ssize lc_decode_t(const void* blob, void* w_ref, uint64_t n, int dtype, void* stream) {
    return decode_impl(blob, SIZE_MAX, w_ref, n, dtype, stream);
}

lc_ssize lc_decode_sized(const void* blob, size_t blob_bytes, void* w_ref, uint64_t n, int dtype, void* stream) {
    return decode_impl(blob, blob_bytes, w_ref, n, dtype, stream);
}

lc_ssize lc_encode_sized(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, size_t out_bytes, int dtype,
                         void* stream) {
    const size_t bound = lc_encode_bound(n, nbits);
    if (bound == 0) return -LC_ERR_BADARG;
    if (out_bytes < bound) return -LC_ERR_OUT_TOO_SMALL;
    return encode_impl(w, w_ref, n, nbits, out, dtype, nullptr, nullptr, stream, false);
}

lc_ssize lc_decode(const void* blob, float* w_ref, uint64_t n, void* stream) {
    return lc_decode_t(blob, w_ref, n, LC_F32, stream);
}

lc_ssize lc_decode_many(const void* const* blobs, int count, float* w_ref, uint64_t n, void* stream) {
    return lc_decode_many_t(blobs, count, w_ref, n, LC_F32, stream);
}

lc_ssize lc_decode_many_t(const void* const* blobs, int count, void* w_ref, uint64_t n, int dtype, void* stream) {
    if (!blobs || count < 1 || count > LC_MAX_MANY || n > LC_MAX_N) return -LC_ERR_BADARG;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16) return -LC_ERR_BADARG;
    if (n && (!w_ref || misaligned(w_ref, dtype == LC_F32 ? 4 : 2))) return -LC_ERR_BADARG;
    for (int i = 0; i < count; ++i) if (!blobs[i] || misaligned(blobs[i], 16)) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0; DeviceState* ds = nullptr;
    Workspace* ws = get_workspace(kWorkspaceFixed, &err, &ds);
    if (!ws) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const uint64_t epoch = ++g_epoch, bound = lc_encode_bound(n, 4);
    if (!order_after_async(ds, s)) return -LC_ERR_HIP;
    BlobList list;
    for (int t = 0; t < kMaxSets; ++t) list.p[t] = static_cast<const uint8_t*>(blobs[t < count ? t : 0]);
    // every blob is validated (one launch, one grid row per blob) before w_ref is touched
    { Timed tm(kSlotDecCheck, s); launch_dec_check(list, 0, count, n, dtype, bound, ws, epoch, g_pinned_dev, s); }
    LC_HIP(hipGetLastError());
    LC_HIP(hipStreamSynchronize(s));
    ds->pending = false;
    if ((g_pinned->dec_status >> 8) == epoch) return -(lc_ssize)(g_pinned->dec_status & 0xFF);
    uint64_t total = 0;
    for (int i = 0; i < count; ++i) total += g_pinned->bytes[i];
    // Sweeps of up to kMaxMany blobs through the fused kernel.  Its LDS payload area is sized to 1.1 x the blobs'
    // average chunk payloads (a chunk above that still decodes, from memory), and a sweep takes only as many
    // blobs as leave room for fused_min_waves_per_cu wavefronts per compute unit.  Blobs with codes longer than
    // the first decode table (7 bits) are grouped apart from those without: they take the kernel's LONG form.
    const uint64_t nchunks = num_chunks_of(n), area = chunk_area_of(nchunks);
    const size_t lds_budget = kLdsPerCu / (size_t)ds->tune.fused_min_waves_per_cu;
    auto pay_words_of = [](double words) {
        uint32_t w = ((uint32_t)(words * 1.1) + 63u) & ~63u;
        return w < kFusedMinWords ? kFusedMinWords : w;
    };
    for (int g0 = 0; g0 < count;) {
        const bool short_codes = g_pinned->max_len[g0] <= kDecLut1Bits;
        int T = 0;
        double words = 0;
        while (g0 + T < count && T < kMaxMany && (g_pinned->max_len[g0 + T] <= kDecLut1Bits) == short_codes) {
            if (nchunks) {
                const double avg = (double)(g_pinned->bytes[g0 + T] - area) / 4.0 / (double)nchunks - kLaneBitsWords + 6.0;
                if (T > 0 && fused_lds_bytes(T + 1, pay_words_of(words + avg)) > lds_budget) break;
                words += avg;
            }
            ++T;
        }
        {
            const uint32_t pay_words = pay_words_of(words);
            Timed tm(kSlotDecodeFused, s);
            launch_decode_fused(list, g0, T, w_ref, n, dtype, ws, epoch, g_pinned_dev, pay_words, !short_codes, ds->tune, s);
        }
        LC_HIP(hipGetLastError());
        g0 += T;
    }
    LC_HIP(hipStreamSynchronize(s));
    int slots[2] = {kSlotDecCheck, kSlotDecodeFused};
    collect(slots, 2);
    if ((g_pinned->dec_status >> 8) == epoch) return -(lc_ssize)(g_pinned->dec_status & 0xFF);
    return (lc_ssize)total;
}

}  // extern "C"

namespace {
bool batch_host() {
    if (g_batch) return true;
    if (hipHostMalloc(reinterpret_cast<void**>(&g_batch), sizeof(BatchHost), hipHostMallocMapped | hipHostMallocPortable) != hipSuccess ||
        hipHostGetDevicePointer(reinterpret_cast<void**>(&g_batch_dev), g_batch, 0) != hipSuccess) {
        (void)hipGetLastError();
        if (g_batch) (void)hipHostFree(g_batch);
        g_batch = nullptr;
        return false;
    }
    return true;
}

size_t batch_decode_bytes(const uint64_t* n, int count, uint64_t* chunks_out) {
    uint64_t chunks = 0;
    for (int t = 0; t < count; ++t) chunks += num_chunks_of(n[t]);
    if (chunks_out) *chunks_out = chunks;
    auto up = [](uint64_t x) { return (x + 255) / 256 * 256; };
    return (size_t)(kWorkspaceHead + up((uint64_t)count * sizeof(DecSet)) + up((uint64_t)count * sizeof(SegD)) + up(4 * chunks) + up(4ull * count));
}
}  // namespace

extern "C" {

lc_ssize lc_decode_batch(const void* const* blobs, float* const* w_ref, const uint64_t* n, int count, int64_t* sizes,
                         void* stream) {
    return lc_decode_batch_t(blobs, reinterpret_cast<void* const*>(w_ref), n, count, sizes, LC_F32, stream);
}

lc_ssize lc_decode_batch_t(const void* const* blobs, void* const* w_ref, const uint64_t* n, int count, int64_t* sizes,
                           int dtype, void* stream) {
    if (!blobs || !w_ref || !n || count < 1 || count > kMaxBatch) return -LC_ERR_BADARG;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16) return -LC_ERR_BADARG;
    const uintptr_t esize = dtype == LC_F32 ? 4 : 2;
    for (int t = 0; t < count; ++t) {
        if (n[t] > LC_MAX_N || !blobs[t] || misaligned(blobs[t], 16)) return -LC_ERR_BADARG;
        if (n[t] && (!w_ref[t] || misaligned(w_ref[t], esize))) return -LC_ERR_BADARG;
    }
    uint64_t chunks64 = 0;
    const size_t need = batch_decode_bytes(n, count, &chunks64);
    if (chunks64 > 0xFFFFFFFFull) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0; DeviceState* ds = nullptr;
    Workspace* ws = get_workspace(need, &err, &ds);
    if (!ws) return -(lc_ssize)err;
    if (!batch_host()) return -LC_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!order_after_async(ds, s)) return -LC_ERR_HIP;
    auto up = [](uint64_t x) { return (x + 255) / 256 * 256; };
    uint8_t* base = reinterpret_cast<uint8_t*>(ws) + kWorkspaceHead;
    BatchDecArgs a;
    uint32_t chunks = 0;
    for (int t = 0; t < count; ++t) {
        SegD& sg = g_batch->dsegs[t];
        sg.blob = static_cast<const uint8_t*>(blobs[t]); sg.w_ref = w_ref[t]; sg.n = n[t];
        sg.nchunks = (uint32_t)num_chunks_of(n[t]); sg.chunk0 = chunks; sg.aligned = !misaligned(w_ref[t], 4 * esize); sg.pad = 0;
        chunks += sg.nchunks;
        g_batch->results[t].bytes = 0; g_batch->results[t].status = LC_ERR_HIP; g_batch->results[t].used_cache = 0;
    }
    a.sets = reinterpret_cast<DecSet*>(base);                base += up((uint64_t)count * sizeof(DecSet));
    a.segs = reinterpret_cast<SegD*>(base);                  base += up((uint64_t)count * sizeof(SegD));
    a.seg_of_chunk = reinterpret_cast<uint32_t*>(base);      base += up(4ull * chunks);
    a.seg_status = reinterpret_cast<uint32_t*>(base);
    a.results = g_batch_dev->results;
    a.count = (uint32_t)count; a.total_chunks = chunks; a.dtype = dtype; a.pad = 0;
    LC_HIP(hipMemcpyAsync(a.segs, g_batch->dsegs, (size_t)count * sizeof(SegD), hipMemcpyHostToDevice, s));
    launch_batch_decode(a, ds->tune, s);
    LC_HIP(hipGetLastError());
    LC_HIP(hipStreamSynchronize(s));
    ds->pending = false;
    lc_ssize total = 0; int first_err = 0;
    for (int t = 0; t < count; ++t) {
        const Result& r = g_batch->results[t];
        if (r.status != LC_OK) { if (!first_err) first_err = (int)r.status; if (sizes) sizes[t] = -(int64_t)r.status; }
        else { total += (lc_ssize)r.bytes; if (sizes) sizes[t] = (int64_t)r.bytes; }
    }
    return first_err ? -(lc_ssize)first_err : total;
}

size_t lc_batch_workspace_bytes(const uint64_t* n, int count, int nbits) {
    if (!n || count < 1 || count > kMaxBatch || nbits < 1 || nbits > 4) return 0;
    uint64_t chunks = 0, groups = 0;
    for (int t = 0; t < count; ++t) {
        if (n[t] > LC_MAX_N) return 0;
        const uint64_t nc = num_chunks_of(n[t]);
        chunks += nc; groups += (nc + 63) / 64;
    }
    if (chunks > 0xFFFFFFFFull) return 0;
    auto up = [](uint64_t x) { return (x + 255) / 256 * 256; };
    const size_t enc = (size_t)(kWorkspaceHead + up((uint64_t)count * sizeof(EncState)) + up((uint64_t)count * sizeof(Seg)) +
                                up(4 * chunks) + up(4 * groups) + up(4 * chunks) + chunks * slot_words_of(nbits) * 4);
    const size_t dec = batch_decode_bytes(n, count, nullptr);
    return enc > dec ? enc : dec;
}

lc_ssize lc_encode_batch(const float* const* w, const float* const* w_ref, const uint64_t* n, int count, int nbits,
                         void* const* out, int64_t* sizes, void* stream) {
    return lc_encode_batch_t(reinterpret_cast<const void* const*>(w), reinterpret_cast<const void* const*>(w_ref), n, count,
                             nbits, out, sizes, LC_F32, stream);
}

lc_ssize lc_encode_batch_t(const void* const* w, const void* const* w_ref, const uint64_t* n, int count, int nbits,
                           void* const* out, int64_t* sizes, int dtype, void* stream) {
    if (!w || !w_ref || !n || !out || count < 1 || count > kMaxBatch || nbits < 1 || nbits > 4) return -LC_ERR_BADARG;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16) return -LC_ERR_BADARG;
    const uintptr_t esize = dtype == LC_F32 ? 4 : 2;
    for (int t = 0; t < count; ++t) {
        if (n[t] > LC_MAX_N || !out[t] || misaligned(out[t], 16)) return -LC_ERR_BADARG;
        if (n[t] && (!w[t] || !w_ref[t] || misaligned(w[t], esize) || misaligned(w_ref[t], esize))) return -LC_ERR_BADARG;
    }
    const size_t need = lc_batch_workspace_bytes(n, count, nbits);
    if (!need) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0; DeviceState* ds = nullptr;
    Workspace* ws = get_workspace(need, &err, &ds);
    if (!ws) return -(lc_ssize)err;
    if (!batch_host()) return -LC_ERR_HIP;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (!order_after_async(ds, s)) return -LC_ERR_HIP;
    // carve the scratch behind the single-vector head (which this call leaves alone)
    auto up = [](uint64_t x) { return (x + 255) / 256 * 256; };
    uint8_t* base = reinterpret_cast<uint8_t*>(ws) + kWorkspaceHead;
    BatchArgs a;
    uint32_t chunks = 0, groups = 0;
    for (int t = 0; t < count; ++t) {
        Seg& sg = g_batch->segs[t];
        sg.w = w[t]; sg.w_ref = w_ref[t]; sg.out = static_cast<uint8_t*>(out[t]); sg.n = n[t];
        sg.nchunks = (uint32_t)num_chunks_of(n[t]); sg.chunk0 = chunks; sg.group0 = groups;
        sg.aligned = !misaligned(w[t], 4 * esize) && !misaligned(w_ref[t], 4 * esize);
        chunks += sg.nchunks; groups += (sg.nchunks + 63) / 64;
        g_batch->results[t].bytes = 0; g_batch->results[t].status = LC_ERR_HIP; g_batch->results[t].used_cache = 0;
    }
    a.states = reinterpret_cast<EncState*>(base);            base += up((uint64_t)count * sizeof(EncState));
    a.segs = reinterpret_cast<Seg*>(base);                   base += up((uint64_t)count * sizeof(Seg));
    a.seg_of_chunk = reinterpret_cast<uint32_t*>(base);      base += up(4ull * chunks);
    a.group_words = reinterpret_cast<uint32_t*>(base);       base += up(4ull * groups);
    a.chunk_bits = reinterpret_cast<uint32_t*>(base);        base += up(4ull * chunks);
    a.prov = reinterpret_cast<uint32_t*>(base);
    a.results = g_batch_dev->results;
    a.count = (uint32_t)count; a.total_chunks = chunks; a.total_groups = groups;
    a.slot_words = slot_words_of(nbits); a.nbits = nbits; a.dtype = dtype;
    LC_HIP(hipMemcpyAsync(a.segs, g_batch->segs, (size_t)count * sizeof(Seg), hipMemcpyHostToDevice, s));
    launch_batch_encode(a, ds->tune, s);
    LC_HIP(hipGetLastError());
    LC_HIP(hipStreamSynchronize(s));
    ds->pending = false;
    lc_ssize total = 0; int first_err = 0;
    for (int t = 0; t < count; ++t) {
        const Result& r = g_batch->results[t];
        if (r.status != LC_OK) { if (!first_err) first_err = (int)r.status; if (sizes) sizes[t] = -(int64_t)r.status; }
        else { total += (lc_ssize)r.bytes; if (sizes) sizes[t] = (int64_t)r.bytes; }
    }
    return first_err ? -(lc_ssize)first_err : total;
}

int lc_blob_info(const void* host_header, uint64_t* n, int* nbits, uint64_t* total_bytes, int* status) {
    if (!host_header) return LC_ERR_BADARG;
    const uint8_t* h = static_cast<const uint8_t*>(host_header);
    uint16_t version; uint64_t hn, total; uint32_t hb, st;
    memcpy(&version, h + 4, 2); memcpy(&hn, h + 8, 8); memcpy(&hb, h + 16, 4); memcpy(&total, h + 40, 8); memcpy(&st, h + 48, 4);
    if (memcmp(h, "LCB1", 4) != 0 || version != 1) return LC_ERR_BAD_BLOB;
    if (n) *n = hn;
    if (nbits) *nbits = (int)hb;
    if (total_bytes) *total_bytes = total;
    if (status) *status = (int)st;
    return LC_OK;
}

int lc_blob_sizes(const void* host_header, uint64_t bits[3]) {
    if (!host_header || !bits) return LC_ERR_BADARG;
    const uint8_t* h = static_cast<const uint8_t*>(host_header);
    uint16_t version; uint64_t n, total; uint32_t x, k, dtype;
    memcpy(&version, h + 4, 2); memcpy(&n, h + 8, 8); memcpy(&x, h + 16, 4); memcpy(&total, h + 40, 8); memcpy(&k, h + 52, 4);
    memcpy(&dtype, h + 60, 4);
    const uint64_t b = dtype == LC_F64 ? 64 : 32;             // bits of one stored bucket value (the delta's type)
    if (memcmp(h, "LCB1", 4) != 0 || version != 1 || x < 1 || x > 4 || k > (dtype == LC_F64 ? 4096u : 512u)) return LC_ERR_BAD_BLOB;
    uint32_t lg = 0;
    while ((1u << lg) < k) ++lg;
    bits[0] = n * lg + b * k;                   // index of one of k buckets per element + k representatives
    bits[1] = n * x + b * (1u << x);            // x bits per element + 2^x representatives
    bits[2] = 8 * total;                        // the blob as stored
    return LC_OK;
}

int lc_set_option(int option, int value) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (option == LC_OPT_KEY_STAGING && value >= LC_STAGING_AUTO && value <= LC_STAGING_NEVER) { g_key_staging = value; return LC_OK; }
    return LC_ERR_BADARG;
}

void lc_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        if (g_dev[d].owned) {
            if (hipSetDevice(d) == hipSuccess) { (void)hipDeviceSynchronize(); (void)hipFree(g_dev[d].owned); }
            g_dev[d].owned = nullptr; g_dev[d].owned_bytes = 0;
        }
        g_dev[d].user = nullptr; g_dev[d].user_bytes = 0;
    }
    if (have_cur) (void)hipSetDevice(cur);
    for (int i = 0; i < kMaxTickets; ++i) {
        if (g_ticket[i].done) { (void)hipEventDestroy(g_ticket[i].inputs); (void)hipEventDestroy(g_ticket[i].done); }
        g_ticket[i] = Ticket();
    }
    for (int d = 0; d < kMaxDevices; ++d) {
        if (g_dev[d].last) { (void)hipEventDestroy(g_dev[d].last); g_dev[d].last = nullptr; }
        g_dev[d].pending = false;
    }
    if (g_pinned) { (void)hipHostFree(g_pinned); g_pinned = nullptr; g_pinned_dev = nullptr; }
    if (g_batch) { (void)hipHostFree(g_batch); g_batch = nullptr; g_batch_dev = nullptr; }
    for (int d = 0; d < kMaxDevices; ++d) g_dev[d].clean = nullptr;
    if (g_ev_made) {
        for (int i = 0; i < kNumSlots; ++i) { (void)hipEventDestroy(g_ev[i][0]); (void)hipEventDestroy(g_ev[i][1]); }
        g_ev_made = false; g_prof = false;
    }
    (void)hipGetLastError();
}

const char* lc_strerror(int status) {
    switch (status < 0 ? -status : status) {
        case LC_OK: return "ok";
        case LC_ERR_BADARG: return "bad argument";
        case LC_ERR_NONFINITE: return "non-finite delta (Inf or NaN)";
        case LC_ERR_OUT_TOO_SMALL: return "output buffer too small";
        case LC_ERR_BAD_BLOB: return "blob failed validation";
        case LC_ERR_HIP: return "HIP runtime error";
        case LC_ERR_WORKSPACE: return "workspace too small or misaligned";
        default: return "unknown status";
    }
}

int lc_profile(int enable) {
    std::lock_guard<std::mutex> lock(g_mu);
    if (enable && !g_ev_made) {
        for (int i = 0; i < kNumSlots; ++i)
            for (int k = 0; k < 2; ++k)
                if (hipEventCreate(&g_ev[i][k]) != hipSuccess) { (void)hipGetLastError(); return LC_ERR_HIP; }
        g_ev_made = true;
    }
    g_prof = enable != 0;
    for (int i = 0; i < kNumSlots; ++i) { g_prof_ms[i] = 0; g_prof_n[i] = 0; }
    return LC_OK;
}

int lc_profile_read(double* ms_total, uint64_t* launches, int cap) {
    std::lock_guard<std::mutex> lock(g_mu);
    for (int i = 0; i < kNumSlots && i < cap; ++i) {
        if (ms_total) ms_total[i] = g_prof_ms[i];
        if (launches) launches[i] = g_prof_n[i];
    }
    return kNumSlots;
}

const char* lc_profile_name(int slot) { return slot >= 0 && slot < kNumSlots ? kSlotNames[slot] : nullptr; }

}  // extern "C"
