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

// One scratch area (lc_workspace_bytes and more) of a device.  A call takes the area its stream used last (calls on one
// stream are ordered, so they share an area without waiting), else an idle one, else a new one (at most kMaxAreas per
// device), else the least recently used one, which its stream then waits for.  Calls on different streams thus
// get different areas and overlap on the device.
constexpr int kMaxAreas = 8;
struct Area {
    void* mem = nullptr;
    size_t bytes = 0;
    bool user = false;            // caller-supplied (lc_set_workspace): never freed, never grown
    hipStream_t stream = nullptr; // the stream of the last call that used it
    bool used = false;
    hipEvent_t idle = nullptr;    // recorded behind the last call that used it
    bool clean = false;           // its encode state is known to be cleared
    uint64_t stamp = 0;           // when it was last taken
};

struct DeviceState {
    Area area[kMaxAreas];
    void* user = nullptr;        // caller-supplied scratch (lc_set_workspace): then the only area
    size_t user_bytes = 0;
    uint64_t clock = 0;
    Tuning tune;
    bool tuned = false;
    // What the last encode of a vector (told apart by address and length) found: the share of its chunks that sweep 2
    // had to read.  Decides whether the next encode of that vector stages keys (see stage_keys()).
    struct Hint { const void* w = nullptr; uint64_t n = 0; float listed = 0; };
    Hint hint[kHints];
};

// A call in progress: where its kernels report (g_pinned[slot]) and, for lc_encode_async, its events.  Asynchronous
// calls hand their slot out as the ticket; at most LC_MAX_TICKETS of them are in flight, the other slots serve
// calls that wait themselves (several host threads may be inside such calls at once).
constexpr int kMaxTickets = LC_MAX_TICKETS, kCallSlots = 2 * LC_MAX_TICKETS;
struct CallSlot {
    bool busy = false, async = false;
    int dev = 0; const void* w = nullptr; uint64_t n = 0;   // whose hint its outcome updates
    hipEvent_t inputs = nullptr;  // after the last kernel that reads w / w_ref
    hipEvent_t done = nullptr;    // after the last kernel
};
CallSlot g_slot[kCallSlots];
int g_async_in_flight = 0;

// lc_encode_batch: pinned host memory for the tensor list on its way to the device and for the
// per-tensor outcomes the kernels write (mapped).
struct BatchHost {
    union { Seg segs[kMaxBatch]; SegD dsegs[kMaxBatch]; };
    Result results[kMaxBatch];
};
BatchHost* g_batch = nullptr;
BatchHost* g_batch_dev = nullptr;

std::mutex g_mu;
DeviceState g_dev[kMaxDevices];
static_assert(sizeof(TableCache) <= LC_CACHE_BYTES, "LC_CACHE_BYTES too small");
static_assert(sizeof(((HostResult*)0)->bytes) / sizeof(unsigned long long) >= LC_MAX_MANY, "HostResult too small");
HostResult* g_pinned = nullptr;  // mapped pinned host memory, kCallSlots records: the kernels write their outcome there
HostResult* g_pinned_dev = nullptr;   // the same memory as the device sees it
uint64_t g_epoch = 0;            // tags the decode status word of each call

int g_key_staging = -1;          // LC_OPT_KEY_STAGING (-1: not yet read from the environment)
bool g_verify_first = false;     // LC_OPT_VERIFY_FIRST
bool g_prof = false;
double g_prof_ms[kNumSlots];
uint64_t g_prof_n[kNumSlots];
hipEvent_t g_ev[kNumSlots][2];
bool g_ev_made = false;
const char* const kSlotNames[kNumSlots] = {"k_reset", "k_hist", "k_table", "k_pack", "k_place", "k_spec_table", "k_spec_sweep",
                                           "k_dec_check", "k_decode", "k_decode_fused", "k_hist_keys", "k_pack_keys", "k_verify"};

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

// The current device's state, with the pinned result records in place.  Returns nullptr with *err set.
DeviceState* device_state(int* err) {
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); *err = LC_ERR_HIP; return nullptr; }
    DeviceState& ds = g_dev[dev];
    read_tuning(ds, dev);
    if (!g_pinned) {
        if (hipHostMalloc(reinterpret_cast<void**>(&g_pinned), kCallSlots * sizeof(HostResult), hipHostMallocMapped | hipHostMallocPortable) != hipSuccess ||
            hipHostGetDevicePointer(reinterpret_cast<void**>(&g_pinned_dev), g_pinned, 0) != hipSuccess) {
            (void)hipGetLastError();
            if (g_pinned) (void)hipHostFree(g_pinned);
            g_pinned = nullptr; *err = LC_ERR_HIP; return nullptr;
        }
        memset(g_pinned, 0, kCallSlots * sizeof(HostResult));
    }
    return &ds;
}

// A scratch area of at least `need` bytes for a call on stream s (see Area).  Returns nullptr with *err set.
Area* acquire(DeviceState* ds, hipStream_t s, size_t need, int* err) {
    Area* a = nullptr;
    if (ds->user) {
        // the caller's area is the only one: calls on other streams are ordered behind its last user
        a = &ds->area[0];
        if (ds->user_bytes < need) { *err = LC_ERR_WORKSPACE; return nullptr; }
    } else {
        Area *same = nullptr, *idle = nullptr, *empty = nullptr, *lru = nullptr;
        for (int i = 0; i < kMaxAreas; ++i) {
            Area* c = &ds->area[i];
            if (!c->mem) { if (!empty) empty = c; continue; }
            if (c->used && c->stream == s) { if (!same || c->stamp > same->stamp) same = c; continue; }
            bool is_idle = !c->used;
            if (!is_idle) {
                const hipError_t q = hipEventQuery(c->idle);
                if (q == hipSuccess) is_idle = true; else (void)hipGetLastError();
            }
            if (is_idle && (!idle || (idle->bytes < need && c->bytes > idle->bytes))) idle = c;
            if (!lru || c->stamp < lru->stamp) lru = c;
        }
        a = same ? same : idle ? idle : empty ? empty : lru;
    }
    if (!a->idle && hipEventCreateWithFlags(&a->idle, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); a->idle = nullptr; *err = LC_ERR_HIP; return nullptr; }
    if (a->used && a->stream != s) {
        // another stream's work may still be using it (the caller's single area, or every area busy): wait for that on s
        if (hipStreamWaitEvent(s, a->idle, 0) != hipSuccess) { (void)hipGetLastError(); *err = LC_ERR_HIP; return nullptr; }
    }
    if (ds->user) {
        if (a->mem != ds->user) { a->mem = ds->user; a->bytes = ds->user_bytes; a->user = true; a->clean = false; a->used = false; }
    } else if (a->bytes < need) {
        if (a->mem) {
            if (a->used) (void)hipEventSynchronize(a->idle);         // its last call must be through with the old memory
            (void)hipFree(a->mem); a->mem = nullptr; a->bytes = 0;
        }
        size_t want = need < (4u << 20) ? (4u << 20) : need;     // never smaller than the head that is cleared below
        static_assert(kWorkspaceHead <= (4u << 20), "the smallest scratch area must hold the fixed head");
        if (hipMalloc(&a->mem, want) != hipSuccess) { (void)hipGetLastError(); a->mem = nullptr; *err = LC_ERR_HIP; return nullptr; }
        // (on the call's own stream: a fill on the null stream is not ordered with a non-blocking stream's kernels and
        // has been seen to land behind the reset kernel that follows, which left the smallest mantissas at zero)
        if (hipMemsetAsync(a->mem, 0, kWorkspaceHead, s) != hipSuccess) { (void)hipGetLastError(); (void)hipFree(a->mem); a->mem = nullptr; *err = LC_ERR_HIP; return nullptr; }
        a->bytes = want; a->user = false; a->used = false;
        a->clean = false;        // new memory (possibly at the old address): its encode state is not set up yet
    }
    a->stream = s; a->stamp = ++ds->clock;
    return a;
}

// Behind the last kernel of a call that used the area.
bool release(Area* a, hipStream_t s) {
    a->used = true;
    if (hipEventRecord(a->idle, s) != hipSuccess) { (void)hipGetLastError(); return false; }
    return true;
}

// A free call slot (asynchronous calls: at most kMaxTickets in flight), or -1.
int take_slot(bool async) {
    if (async && g_async_in_flight >= kMaxTickets) return -1;
    for (int i = 0; i < kCallSlots; ++i) {
        if (g_slot[i].busy) continue;
        CallSlot& c = g_slot[i];
        if (async && !c.done) {
            if (hipEventCreateWithFlags(&c.inputs, hipEventDisableTiming) != hipSuccess ||
                hipEventCreateWithFlags(&c.done, hipEventDisableTiming) != hipSuccess) { (void)hipGetLastError(); c.inputs = c.done = nullptr; return -1; }
        }
        c.busy = true; c.async = async; c.w = nullptr; c.n = 0;
        if (async) ++g_async_in_flight;
        return i;
    }
    return -1;
}
void free_slot(int i) {
    if (g_slot[i].async) --g_async_in_flight;
    g_slot[i].busy = false; g_slot[i].async = false;
}

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// Bytes of scratch an encode of nc chunks at nbits takes (what lc_workspace_bytes reports), and where its parts lie.
constexpr size_t up256(size_t x) { return (x + 255) / 256 * 256; }
constexpr size_t encode_scratch_bytes(uint64_t nc, int nbits) {
    return kWorkspaceHead + up256(4 * nc) + (size_t)(nc * (kLaneBitsWords + kW * 8u * ((1u << nbits) - 1u)) * 4) +
           256 + up256(kPartMaxBytes * nc);                       // + the per-batch maxima of sweep 1
}
// ... and with staged keys behind that: a byte and a bit per element of every whole batch
size_t staged_scratch_bytes(uint64_t n, int nbits) {
    return encode_scratch_bytes(num_chunks_of(n), nbits) + up256(key_exp_bytes(n)) + up256(key_sign_bytes(n));
}
struct Scratch {
    Workspace* ws;
    uint32_t *group_words, *chunk_maxexp, *chunk_list, *chunk_bits, *prov;
    uint8_t* batch_max;                                           // the largest exponent of every 4 KiB batch of sweep 1, kPartMaxBytes per chunk, behind the slots
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
        uint8_t* e = batch_max + up256(kPartMaxBytes * nc);
        return KeyPlanes{e, reinterpret_cast<uint16_t*>(e + up256(key_exp_bytes(n)))};
    }
};

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
    (void)hipDeviceSynchronize();                 // no call may still be using the areas that change hands here
    if (dev_ws && (hipMemset(dev_ws, 0, kWorkspaceHead) != hipSuccess || hipDeviceSynchronize() != hipSuccess)) { (void)hipGetLastError(); return LC_ERR_HIP; }
    DeviceState& ds = g_dev[dev];
    if (ds.user && ds.area[0].mem == ds.user) { ds.area[0].mem = nullptr; ds.area[0].bytes = 0; ds.area[0].user = false; ds.area[0].used = false; }
    if (dev_ws) {
        // the caller's area becomes the only one: the library's own go
        for (int i = 0; i < kMaxAreas; ++i) {
            Area& a = ds.area[i];
            if (a.mem && !a.user) (void)hipFree(a.mem);
            a.mem = nullptr; a.bytes = 0; a.user = false; a.used = false; a.clean = false;
        }
    }
    ds.user = dev_ws;
    ds.user_bytes = dev_ws ? bytes : 0;
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
    const uintptr_t esize = dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2;
    if (n && (!w || !w_ref || misaligned(w, esize) || misaligned(w_ref, esize))) return -LC_ERR_BADARG;
    std::unique_lock<std::mutex> lock(g_mu);
    int err = 0;
    DeviceState* ds = device_state(&err);
    if (!ds) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    bool staged = stage_keys(ds, w, w_ref, n, dtype, cache != nullptr);
    Area* area = nullptr;
    if (staged) {
        // the key planes lie behind the usual scratch; a caller's area that has no room for them keeps the plain path
        area = acquire(ds, s, staged_scratch_bytes(n, nbits), &err);
        if (!area) staged = false;
    }
    if (!area) area = acquire(ds, s, lc_workspace_bytes(n, nbits), &err);
    if (!area) return -(lc_ssize)err;
    Workspace* ws = static_cast<Workspace*>(area->mem);
    const Scratch sc(ws, num_chunks_of(n), nbits);
    const KeyPlanes keys = staged ? sc.keys(n) : KeyPlanes{nullptr, nullptr};
    uint32_t *group_words = sc.group_words, *chunk_maxexp = sc.chunk_maxexp, *chunk_list = sc.chunk_list, *chunk_bits = sc.chunk_bits,
             *prov = sc.prov;
    const uint32_t slot_words = sc.slot_words;
    uint8_t* batch_max = sc.batch_max;
    uint8_t* o = static_cast<uint8_t*>(out);
    const int slot = take_slot(async);
    if (slot < 0) return async ? -LC_ERR_BADARG : -LC_ERR_HIP;      // too many calls in flight
    CallSlot& call = g_slot[slot];
    struct Undo { int slot; bool armed; ~Undo() { if (armed) free_slot(slot); } } undo{slot, true};   // (the lock is still held on every early return)
    Result* result = &g_pinned_dev[slot].enc;
    // Every call leaves the encode state cleared behind it; a fresh scratch area, or one whose last
    // call did not run to its end, is cleared first.
    if (!area->clean) { Timed t(kSlotReset, s); launch_reset(ws, group_words, chunk_maxexp, s); }
    area->clean = false;
    // (binary64 with a cache: two sweeps, the second one coding with the cached lengths when k_table confirms them)
    const bool spec_sweep = cache && dtype != LC_F64;
    if (cache) { Timed t(kSlotSpecTable, s); launch_spec_table(ws, cache, n, nbits, dtype, group_words, s); }
    if (spec_sweep) {
        Timed t(kSlotSpecSweep, s); launch_spec_sweep(w, w_ref, n, dtype, ws, chunk_bits, group_words, prov, slot_words, ds->tune, s);
    } else {
        Timed t(staged ? kSlotHistKeys : kSlotHist, s); launch_hist(w, w_ref, n, dtype, ws, chunk_maxexp, batch_max, keys, ds->tune, s);
    }
    const bool listed = !spec_sweep;            // sweep 1 recorded the chunk maxima, so k_table can list the chunks to read
    { Timed t(kSlotTable, s);    launch_table(ws, n, nbits, dtype, group_words, chunk_maxexp, listed ? chunk_list : nullptr, s); }
    if (staged) { Timed t(kSlotPackKeys, s); launch_pack_keys(w, w_ref, n, ws, chunk_bits, group_words, chunk_maxexp, chunk_list, keys, prov, slot_words, ds->tune, s); }
    else { Timed t(kSlotPack, s); launch_pack(w, w_ref, n, dtype, ws, chunk_bits, group_words, chunk_maxexp, listed ? chunk_list : nullptr, batch_max, prov, slot_words, ds->tune, s); }
    if (async) LC_HIP(hipEventRecord(call.inputs, s));   // w and w_ref are not read past this point
    { Timed t(kSlotPlace, s);    launch_place(o, ws, chunk_bits, group_words, prov, slot_words, n, chunk_maxexp, result, cache, nbits, dtype, staged, s); }
    LC_HIP(hipGetLastError());
    if (!release(area, s)) return -LC_ERR_HIP;
    area->clean = true;              // whoever takes the area next is ordered behind this call
    call.dev = (int)(ds - g_dev); call.w = (!cache && dtype == LC_F32) ? w : nullptr; call.n = n;
    if (async) {
        LC_HIP(hipEventRecord(call.done, s));
        undo.armed = false;
        return slot;
    }
    // Waiting happens outside the lock, so that calls of other host threads on other streams go on meanwhile; with the
    // per-kernel timing switched on the calls stay one at a time (its events are shared).
    const bool serial = g_prof;
    if (!serial) lock.unlock();
    const hipError_t waited = hipStreamSynchronize(s);
    if (!serial) lock.lock();
    if (waited != hipSuccess) { (void)hipGetLastError(); area->clean = false; return -LC_ERR_HIP; }
    const int slots[] = {cache ? kSlotSpecTable : staged ? kSlotHistKeys : kSlotHist, kSlotTable, staged ? kSlotPackKeys : kSlotPack,
                         kSlotPlace, spec_sweep ? kSlotSpecSweep : kSlotHist};
    collect(slots, cache ? 5 : 4);
    const Result r = g_pinned[slot].enc;
    if (call.w) note_outcome(ds, call.w, call.n, r);
    if (used) *used = (int)r.used_cache;
    if (r.status != LC_OK) return -(lc_ssize)r.status;
    return (lc_ssize)r.bytes;
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
    launch_place(o, sc.ws, sc.chunk_bits, sc.group_words, sc.prov, sc.slot_words, n, sc.chunk_maxexp, result, nullptr, nbits, LC_F32, false, s);
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
    if (ticket < 0 || ticket >= kCallSlots || !g_slot[ticket].busy || !g_slot[ticket].async) return LC_ERR_BADARG;
    if (hipStreamWaitEvent(static_cast<hipStream_t>(other_stream), g_slot[ticket].inputs, 0) != hipSuccess) { (void)hipGetLastError(); return LC_ERR_HIP; }
    return LC_OK;
}

lc_ssize lc_encode_wait(int ticket, int* used) {
    hipEvent_t done;
    {
        std::lock_guard<std::mutex> lock(g_mu);
        if (ticket < 0 || ticket >= kCallSlots || !g_slot[ticket].busy || !g_slot[ticket].async) return -LC_ERR_BADARG;
        done = g_slot[ticket].done;
    }
    const hipError_t e = hipEventSynchronize(done);          // not under the lock: other threads may keep calling
    std::lock_guard<std::mutex> lock(g_mu);
    const CallSlot call = g_slot[ticket];
    free_slot(ticket);
    if (e != hipSuccess) { (void)hipGetLastError(); return -LC_ERR_HIP; }
    const Result r = g_pinned[ticket].enc;
    if (call.w) note_outcome(&g_dev[call.dev], call.w, call.n, r);
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
// verify_only: nothing but the blob is read (lc_verify); else the restore, after the same lane-string check if the
// option asks for it
lc_ssize decode_impl(const void* blob, size_t blob_bytes, void* w_ref, uint64_t n, int dtype, void* stream, bool verify_only = false) {
    if (!blob || misaligned(blob, 16) || n > LC_MAX_N) return -LC_ERR_BADARG;
    if (blob_bytes < kHeaderBytes) return -LC_ERR_BAD_BLOB;
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    if (!verify_only && n && (!w_ref || misaligned(w_ref, dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2))) return -LC_ERR_BADARG;
    std::unique_lock<std::mutex> lock(g_mu);
    int err = 0;
    DeviceState* ds = device_state(&err);
    if (!ds) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Area* area = acquire(ds, s, kWorkspaceFixed, &err);
    if (!area) return -(lc_ssize)err;
    Workspace* ws = static_cast<Workspace*>(area->mem);
    const int slot = take_slot(false);
    if (slot < 0) return -LC_ERR_HIP;
    struct Undo { int slot; ~Undo() { free_slot(slot); } } undo{slot};     // (the lock is held on every return)
    HostResult* host = &g_pinned_dev[slot];
    const uint8_t* b = static_cast<const uint8_t*>(blob);
    const uint64_t epoch = ++g_epoch;
    BlobList list;
    for (int t = 0; t < kMaxSets; ++t) list.p[t] = b;
    const uint64_t bound = lc_encode_bound(n, 4), max_total = blob_bytes < bound ? blob_bytes : bound;
    { Timed t(kSlotDecCheck, s); launch_dec_check(list, 0, 1, n, dtype, max_total, ws, epoch, host, s); }
    // (a finding of the verifying sweep gates the restoring one on the device, like a finding of the check)
    if (verify_only || g_verify_first) { Timed t(kSlotVerify, s); launch_decode(b, nullptr, n, dtype, ws, 0, epoch, host, ds->tune, s); }
    if (!verify_only) { Timed t(kSlotDecode, s); launch_decode(b, w_ref, n, dtype, ws, 0, epoch, host, ds->tune, s); }
    LC_HIP(hipGetLastError());
    if (!release(area, s)) return -LC_ERR_HIP;
    const bool serial = g_prof;              // (see encode_impl)
    if (!serial) lock.unlock();
    const hipError_t waited = hipStreamSynchronize(s);
    if (!serial) lock.lock();
    if (waited != hipSuccess) { (void)hipGetLastError(); return -LC_ERR_HIP; }
    int slots[3] = {kSlotDecCheck, 0, 0}, launched = 1;          // (only what this call launched has fresh events)
    if (verify_only || g_verify_first) slots[launched++] = kSlotVerify;
    if (!verify_only) slots[launched++] = kSlotDecode;
    collect(slots, launched);
    if ((g_pinned[slot].dec_status >> 8) == epoch) return -(lc_ssize)(g_pinned[slot].dec_status & 0xFF);
    return (lc_ssize)g_pinned[slot].bytes[0];
}
}  // namespace

extern "C" {

lc_ssize lc_decode_t(const void* blob, void* w_ref, uint64_t n, int dtype, void* stream) {
    return decode_impl(blob, SIZE_MAX, w_ref, n, dtype, stream);
}

lc_ssize lc_decode_sized(const void* blob, size_t blob_bytes, void* w_ref, uint64_t n, int dtype, void* stream) {
    return decode_impl(blob, blob_bytes, w_ref, n, dtype, stream);
}

lc_ssize lc_verify(const void* blob, size_t blob_bytes, uint64_t n, int dtype, void* stream) {
    return decode_impl(blob, blob_bytes, nullptr, n, dtype, stream, true);
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
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    if (n && (!w_ref || misaligned(w_ref, dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2))) return -LC_ERR_BADARG;
    for (int i = 0; i < count; ++i) if (!blobs[i] || misaligned(blobs[i], 16)) return -LC_ERR_BADARG;
    // (a call of several phases: it keeps the lock, so that no other call's check moves into its area between them)
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0;
    DeviceState* ds = device_state(&err);
    if (!ds) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Area* area = acquire(ds, s, kWorkspaceFixed, &err);
    if (!area) return -(lc_ssize)err;
    Workspace* ws = static_cast<Workspace*>(area->mem);
    const int slot = take_slot(false);
    if (slot < 0) return -LC_ERR_HIP;
    struct Undo { int slot; ~Undo() { free_slot(slot); } } undo{slot};
    HostResult* host = &g_pinned_dev[slot];
    const HostResult& got = g_pinned[slot];
    const uint64_t epoch = ++g_epoch, bound = lc_encode_bound(n, 4);
    BlobList list;
    for (int t = 0; t < kMaxSets; ++t) list.p[t] = static_cast<const uint8_t*>(blobs[t < count ? t : 0]);
    // every blob is validated (one launch, one grid row per blob) before w_ref is touched
    { Timed tm(kSlotDecCheck, s); launch_dec_check(list, 0, count, n, dtype, bound, ws, epoch, host, s); }
    if (g_verify_first) {
        for (int i = 0; i < count; ++i) { Timed tm(kSlotVerify, s); launch_decode(list.p[i], nullptr, n, dtype, ws, i, epoch, host, ds->tune, s); }
    }
    LC_HIP(hipGetLastError());
    if (!release(area, s)) return -LC_ERR_HIP;
    LC_HIP(hipStreamSynchronize(s));
    if ((got.dec_status >> 8) == epoch) return -(lc_ssize)(got.dec_status & 0xFF);
    uint64_t total = 0;
    for (int i = 0; i < count; ++i) total += got.bytes[i];
    if (dtype == LC_F64) {
        // binary64 parameters: the blobs one after the other (one read and one write of w_ref per blob), each sweep
        // with the tables the check left for its blob
        for (int i = 0; i < count; ++i) {
            Timed tm(kSlotDecode, s);
            launch_decode(list.p[i], w_ref, n, dtype, ws, i, epoch, host, ds->tune, s);
        }
        LC_HIP(hipGetLastError());
        if (!release(area, s)) return -LC_ERR_HIP;
        LC_HIP(hipStreamSynchronize(s));
        if ((got.dec_status >> 8) == epoch) return -(lc_ssize)(got.dec_status & 0xFF);
        return (lc_ssize)total;
    }
    // Sweeps of up to kMaxMany blobs through the fused kernel.  Its LDS payload area is sized to 1.1 x the blobs'
    // average chunk payloads (a chunk above that still decodes, from memory), and a sweep takes only as many
    // blobs as leave room for fused_min_waves_per_cu wavefronts per compute unit.  Blobs with codes longer than
    // the first decode table (7 bits) are grouped apart from those without: they take the kernel's LONG form.
    const uint64_t nchunks = num_chunks_of(n), area_at = chunk_area_of(nchunks);
    const size_t lds_budget = kLdsPerCu / (size_t)ds->tune.fused_min_waves_per_cu;
    auto pay_words_of = [](double words) {
        uint32_t w = ((uint32_t)(words * 1.1) + 63u) & ~63u;
        return w < kFusedMinWords ? kFusedMinWords : w;
    };
    for (int g0 = 0; g0 < count;) {
        const bool short_codes = got.max_len[g0] <= kDecLut1Bits;
        int T = 0;
        double words = 0;
        while (g0 + T < count && T < kMaxMany && (got.max_len[g0 + T] <= kDecLut1Bits) == short_codes) {
            if (nchunks) {
                const double avg = (double)(got.bytes[g0 + T] - area_at) / 4.0 / (double)nchunks - kLaneBitsWords + 6.0;
                if (T > 0 && fused_lds_bytes(T + 1, pay_words_of(words + avg)) > lds_budget) break;
                words += avg;
            }
            ++T;
        }
        {
            const uint32_t pay_words = pay_words_of(words);
            Timed tm(kSlotDecodeFused, s);
            launch_decode_fused(list, g0, T, w_ref, n, dtype, ws, epoch, host, pay_words, !short_codes, ds->tune, s);
        }
        LC_HIP(hipGetLastError());
        g0 += T;
    }
    if (!release(area, s)) return -LC_ERR_HIP;
    LC_HIP(hipStreamSynchronize(s));
    int slots[2] = {kSlotDecCheck, kSlotDecodeFused};
    collect(slots, 2);
    if ((got.dec_status >> 8) == epoch) return -(lc_ssize)(got.dec_status & 0xFF);
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
    return (size_t)(kWorkspaceHead + up((uint64_t)count * sizeof(DecSet)) + up((uint64_t)count * sizeof(SegD)) + up(4 * chunks) + up(4ull * count) + up(16 * chunks));
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
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    const uintptr_t esize = dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2;
    for (int t = 0; t < count; ++t) {
        if (n[t] > LC_MAX_N || !blobs[t] || misaligned(blobs[t], 16)) return -LC_ERR_BADARG;
        if (n[t] && (!w_ref[t] || misaligned(w_ref[t], esize))) return -LC_ERR_BADARG;
    }
    if (dtype == LC_F64) {
        // binary64 tensors: one lc_decode_t after the other (its kernels are not among the batched ones); a tensor
        // whose blob fails is left untouched and reported, the others are restored
        lc_ssize total = 0; int first_err = 0;
        for (int t = 0; t < count; ++t) {
            const lc_ssize r = decode_impl(blobs[t], SIZE_MAX, w_ref[t], n[t], dtype, stream);
            if (sizes) sizes[t] = r;
            if (r < 0) { if (!first_err) first_err = (int)-r; } else total += r;
        }
        return first_err ? -(lc_ssize)first_err : total;
    }
    uint64_t chunks64 = 0;
    const size_t need = batch_decode_bytes(n, count, &chunks64);
    if (chunks64 > 0xFFFFFFFFull) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0;
    DeviceState* ds = device_state(&err);
    if (!ds) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Area* area = acquire(ds, s, need, &err);
    if (!area) return -(lc_ssize)err;
    Workspace* ws = static_cast<Workspace*>(area->mem);
    if (!batch_host()) return -LC_ERR_HIP;
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
    a.seg_status = reinterpret_cast<uint32_t*>(base);        base += up(4ull * count);
    a.chunk_info = reinterpret_cast<uint32_t*>(base);
    a.results = g_batch_dev->results;
    a.count = (uint32_t)count; a.total_chunks = chunks; a.dtype = dtype; a.pad = 0;
    LC_HIP(hipMemcpyAsync(a.segs, g_batch->dsegs, (size_t)count * sizeof(SegD), hipMemcpyHostToDevice, s));
    launch_batch_decode(a, ds->tune, s);
    LC_HIP(hipGetLastError());
    if (!release(area, s)) return -LC_ERR_HIP;
    LC_HIP(hipStreamSynchronize(s));
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
                                up(4 * chunks) + up(4 * groups) + 3 * up(4 * chunks) + up(kPartBytes * chunks) + 256 +
                                chunks * slot_words_of(nbits) * 4);
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
    if (dtype != LC_F32 && dtype != LC_BF16 && dtype != LC_F16 && dtype != LC_F64) return -LC_ERR_BADARG;
    const uintptr_t esize = dtype == LC_F32 ? 4 : dtype == LC_F64 ? 8 : 2;
    for (int t = 0; t < count; ++t) {
        if (n[t] > LC_MAX_N || !out[t] || misaligned(out[t], 16)) return -LC_ERR_BADARG;
        if (n[t] && (!w[t] || !w_ref[t] || misaligned(w[t], esize) || misaligned(w_ref[t], esize))) return -LC_ERR_BADARG;
    }
    if (dtype == LC_F64) {
        // binary64 tensors: one lc_encode_t after the other (its kernels are not among the batched ones)
        lc_ssize total = 0; int first_err = 0;
        for (int t = 0; t < count; ++t) {
            const lc_ssize r = encode_impl(w[t], w_ref[t], n[t], nbits, out[t], dtype, nullptr, nullptr, stream, false);
            if (sizes) sizes[t] = r;
            if (r < 0) { if (!first_err) first_err = (int)-r; } else total += r;
        }
        return first_err ? -(lc_ssize)first_err : total;
    }
    const size_t need = lc_batch_workspace_bytes(n, count, nbits);
    if (!need) return -LC_ERR_BADARG;
    std::lock_guard<std::mutex> lock(g_mu);
    int err = 0;
    DeviceState* ds = device_state(&err);
    if (!ds) return -(lc_ssize)err;
    hipStream_t s = static_cast<hipStream_t>(stream);
    Area* area = acquire(ds, s, need, &err);
    if (!area) return -(lc_ssize)err;
    Workspace* ws = static_cast<Workspace*>(area->mem);
    if (!batch_host()) return -LC_ERR_HIP;
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
    a.chunk_maxexp = reinterpret_cast<uint32_t*>(base);      base += up(4ull * chunks);
    a.chunk_list = reinterpret_cast<uint32_t*>(base);        base += up(4ull * chunks);
    a.part_max = base;                                       base += up((uint64_t)kPartBytes * chunks);
    a.list_count = reinterpret_cast<uint32_t*>(base);        base += 256;
    a.prov = reinterpret_cast<uint32_t*>(base);
    a.results = g_batch_dev->results;
    a.count = (uint32_t)count; a.total_chunks = chunks; a.total_groups = groups;
    a.slot_words = slot_words_of(nbits); a.nbits = nbits; a.dtype = dtype;
    LC_HIP(hipMemcpyAsync(a.segs, g_batch->segs, (size_t)count * sizeof(Seg), hipMemcpyHostToDevice, s));
    launch_batch_encode(a, ds->tune, s);
    LC_HIP(hipGetLastError());
    if (!release(area, s)) return -LC_ERR_HIP;
    LC_HIP(hipStreamSynchronize(s));
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
    if (option == LC_OPT_VERIFY_FIRST && (value == 0 || value == 1)) { g_verify_first = value != 0; return LC_OK; }
    return LC_ERR_BADARG;
}

void lc_shutdown(void) {
    std::lock_guard<std::mutex> lock(g_mu);
    int cur = 0;
    const bool have_cur = hipGetDevice(&cur) == hipSuccess;
    for (int d = 0; d < kMaxDevices; ++d) {
        bool any = false;
        for (int i = 0; i < kMaxAreas; ++i) any = any || g_dev[d].area[i].mem || g_dev[d].area[i].idle;
        if (any && hipSetDevice(d) == hipSuccess) {
            (void)hipDeviceSynchronize();
            for (int i = 0; i < kMaxAreas; ++i) {
                Area& a = g_dev[d].area[i];
                if (a.mem && !a.user) (void)hipFree(a.mem);
                if (a.idle) (void)hipEventDestroy(a.idle);
            }
        }
        for (int i = 0; i < kMaxAreas; ++i) g_dev[d].area[i] = Area();
        g_dev[d].user = nullptr; g_dev[d].user_bytes = 0;
    }
    if (have_cur) (void)hipSetDevice(cur);
    for (int i = 0; i < kCallSlots; ++i) {
        if (g_slot[i].done) { (void)hipEventDestroy(g_slot[i].inputs); (void)hipEventDestroy(g_slot[i].done); }
        g_slot[i] = CallSlot();
    }
    g_async_in_flight = 0;
    if (g_pinned) { (void)hipHostFree(g_pinned); g_pinned = nullptr; g_pinned_dev = nullptr; }
    if (g_batch) { (void)hipHostFree(g_batch); g_batch = nullptr; g_batch_dev = nullptr; }
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
