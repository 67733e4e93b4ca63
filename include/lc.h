/*
 * lc.h -- C ABI of the MI355X (gfx950) compress / restore path of LC-Checkpoint
 * (arXiv 2009.13003, "On Efficient Constructions of Checkpoints").
 *
 * One checkpoint = one call:
 *   lc_encode  takes the live fp32 parameters u_t and the last *recovered* state
 *              u~_{t-1}, forms delta = u_t - u~_{t-1} (Algorithm 1 line 4), buckets
 *              every delta by (sign, exponent) and keeps the 2^nbits - 1 non-empty
 *              buckets of largest exponent, each represented by the mean of its
 *              largest and smallest member, everything else becoming 0 (Section 3.1.1:
 *              exponent-based quantization and x-bit priority promotion), then
 *              Huffman-codes the bucket indices (Section 3.1.2; Algorithm 1 lines 5-6)
 *              into an LCB1 blob in device memory.
 *   lc_decode  is Algorithm 1 line 7 / the restore of Section 3 (C1): Huffman decode,
 *              look up the representative, u~_t = u~_{t-1} + delta~_t in place.
 *
 * Every step runs in HIP kernels; nothing is computed on the host except argument
 * checks.  All pointers are DEVICE pointers unless a parameter says "host".
 * `stream` is a hipStream_t passed as void* (NULL = the null stream).  Calls may be
 * issued from several threads; the library keeps a scratch area per stream in use
 * (see lc_encode_async), so calls on different streams overlap on the device.
 *
 * ---------------------------------------------------------------------------
 * LCB1 blob layout (little-endian).  The paper says only "save to disk"; this
 * layout is this library's.
 *
 *   [0, 512)            header
 *   [512, A)            u32 chunk_word_off[num_chunks + 1], zero-padded to 16 bytes;
 *                       A = 512 + roundup16(4 * (num_chunks + 1))
 *   [A, total_bytes)    chunk records, record c starting at A + 4*chunk_word_off[c];
 *                       chunk_word_off[num_chunks] = size of the chunk area in words
 *
 *   Chunk c covers elements [c*C, min(n, (c+1)*C)), C = W*V*R = 64*4*64 = 16384.
 *   Lane l (0..63) owns, in this order, the elements c*C + r*256 + 4*l + v
 *   (r = 0..63, v = 0..3) that are < n.  A lane stream is the concatenation of the
 *   codes of the lane's elements, each code most significant bit first.
 *   Chunk record = u16 lane_bits[64] (bit length of each lane stream), then the
 *   payload: the 64 lane streams concatenated in lane order without gaps, zero
 *   padded to a whole 32-bit word.  Bit p of a payload is bit (31 - p%32) of
 *   u32 word p/32.
 *
 *   Header:
 *     0  char[4] "LCB1"        4  u16 version = 1       6  u16 header_bytes = 512
 *     8  u64 n                16  u32 nbits            20  u32 K (kept buckets; zero symbol = K)
 *    24  u32 W = 64           28  u32 V = 4            32  u32 R = 64
 *    36  u32 num_chunks       40  u64 total_bytes      48  u32 status (0, or 2 = non-finite delta)
 *    52  u32 k_E  non-empty buckets before promotion (the zero class counts once)
 *    56  u32 max_len  longest code length              60  u32 element type restored (0 fp32, 1 bf16, 2 fp16, 3 fp64)
 *    64  16 symbol slots of 16 bytes: { u16 bucket_id, u8 len, u8 0, u32 rep_bits, u64 count }
 *        slot j < K: bucket_id = (sign << 8) | biased exponent; rep_bits = the fp32
 *        representative; slot K: bucket_id 0xFFFF, rep_bits 0 (the merged bucket,
 *        "stored last", Section 4.4); slots > K are zero.  len = 0 iff count = 0.
 *   320  192 zero bytes; in an fp64 blob (element type 3) the first 64 are u32 rep_hi[16]: the method then runs
 *        on the binary64 delta (Section 3.1.1, footnote: sign and 11 exponent bits, at most 2^12 buckets),
 *        bucket_id = (sign << 11) | biased exponent, and slot j's representative is the binary64 pattern
 *        (rep_hi[j] << 32) | rep_bits
 *
 *   Symbols: j < K is the j-th kept bucket in priority order (larger exponent first,
 *   + before - at equal exponent).  Biased exponent 0 (zeros, subnormals: Figure 2
 *   caption) always belongs to the merged bucket.  Code lengths are Huffman lengths
 *   of the counts, built by repeatedly joining the two smallest nodes under the order
 *   (weight, leaf before joined node, symbol index / creation order); one active
 *   symbol gets length 1.  Codes are canonical: symbols sorted by (len, index), first
 *   code 0, each next = (previous + 1) << (growth in length).
 *   On a non-finite delta the blob is a header only (status 2, total_bytes 512).
 * ---------------------------------------------------------------------------
 */
#ifndef LC_H
#define LC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef int64_t lc_ssize;        /* >= 0: byte count;  < 0: -(enum lc_status) */

enum lc_status {
    LC_OK = 0,
    LC_ERR_BADARG = 1,           /* null/misaligned pointer, nbits outside [1,4], n too large, n mismatch */
    LC_ERR_NONFINITE = 2,        /* some delta is Inf or NaN */
    LC_ERR_OUT_TOO_SMALL = 3,    /* lc_encode_sized: out_bytes below lc_encode_bound (no blob ever exceeds that bound) */
    LC_ERR_BAD_BLOB = 4,         /* blob fails validation */
    LC_ERR_HIP = 5,              /* a HIP runtime call failed */
    LC_ERR_WORKSPACE = 6         /* caller-supplied workspace too small or misaligned */
};

#define LC_MAX_N (1ull << 32)    /* largest n per call; larger vectors are sliced by the caller */
#define LC_CHUNK 16384u
#define LC_MAX_MANY 64           /* most blobs one lc_decode_many call accepts */

/*
 * Worst-case blob size in bytes for (n, nbits); host only, no GPU needed.  An optimal
 * prefix code over at most 2^nbits symbols (Section 3.1.2) never averages more than
 * nbits bits per symbol, so the bound is header + offsets + 132 bytes per chunk +
 * ceil(n*nbits/8).  Returns 0 for invalid arguments.
 */
size_t lc_encode_bound(uint64_t n, int nbits);

/*
 * Device scratch lc_encode needs for (n, nbits): a fixed part of about 2.1 MB (tables,
 * and per-chunk notes sized for LC_MAX_N) plus, per chunk of 16384 elements, one slot that
 * can hold the chunk's code bits at their longest (2^nbits - 1 bits per element): about
 * 0.06 / 0.19 / 0.44 / 0.94 bytes per element for nbits = 1..4, and 16 bytes of notes per chunk.
 * lc_decode needs only the fixed part (lc_workspace_bytes(0, 1)).  Host only.
 */
size_t lc_workspace_bytes(uint64_t n, int nbits);

/*
 * Optional: hand the library a device scratch area for the current device instead of
 * letting it allocate (lazily, once, grown on demand, freed by lc_shutdown).
 * dev_ws must be 256-byte aligned and stay valid until replaced or lc_shutdown; the
 * library never frees it.  dev_ws = NULL returns to library-owned scratch.  Calls
 * whose lc_workspace_bytes exceeds `bytes` fail with LC_ERR_WORKSPACE.
 * Returns an lc_status.
 */
int lc_set_workspace(void* dev_ws, size_t bytes);

/*
 * Algorithm 1 lines 4-6 for one checkpoint (Sections 3, 3.1.1, 3.1.2).
 *   w      [n] fp32, device, read only: the live parameters u_t
 *   w_ref  [n] fp32, device, read only: the last recovered state u~_{t-1}
 *   n      0 <= n <= LC_MAX_N
 *   nbits  promotion bits x in [1, 4]: 2^x - 1 buckets are kept
 *   out    device, 16-byte aligned, at least lc_encode_bound(n, nbits) bytes, must not
 *          overlap w / w_ref; receives the LCB1 blob
 * w and w_ref need 4-byte alignment; 16-byte alignment of both takes the fast loads.
 * Enqueues on `stream`, then waits for that stream and returns the blob size in
 * bytes, or -(lc_status).  On LC_ERR_NONFINITE `out` holds a 512-byte header whose
 * status field says so.  Caller owns all buffers; nothing is retained.
 */
lc_ssize lc_encode(const float* w, const float* w_ref, uint64_t n, int nbits,
                   void* out, void* stream);

/*
 * How lc_encode (fp32, 16-byte aligned w and w_ref, no cache) feeds its second sweep.  With staged keys the first
 * sweep also writes the 9 bits of every element's bucket id (sign, exponent: Section 3.1.1) to scratch and gathers
 * the buckets' extremes, and the second sweep codes from those keys instead of reading w and w_ref again: 10.25 + c/8
 * bytes per element moved instead of 16 + c/8, but the keys of chunks that hold the merged bucket only are written for
 * nothing, so on sparse updates (where the plain second sweep passes over most chunks) it loses.
 *   LC_STAGING_AUTO    (default) stage keys for a vector of at least 2^26 elements (told by address and length) iff
 *                      its last encode on this device had to read more than 30 % of its chunks in the second sweep;
 *                      a vector's first encode: plain
 *   LC_STAGING_ALWAYS  whenever it applies;  LC_STAGING_NEVER  never
 * The blob is byte for byte the same either way.  Staging needs 1.125 bytes of scratch per element on top of
 * lc_workspace_bytes (a caller-supplied workspace without that room keeps the plain path).  Process-wide; the
 * environment variable LC_TUNE_KEY_STAGING=0|1|2 sets the initial value.  Returns LC_OK or LC_ERR_BADARG.
 */
enum lc_option { LC_OPT_KEY_STAGING = 1, LC_OPT_VERIFY_FIRST = 2 };
enum { LC_STAGING_AUTO = 0, LC_STAGING_ALWAYS = 1, LC_STAGING_NEVER = 2 };
int lc_set_option(int option, int value);

/*
 * The two calls with the sizes of the caller's buffers stated (any dtype of lc_encode_t / lc_decode_t):
 * lc_encode_sized returns -LC_ERR_OUT_TOO_SMALL without touching anything if out_bytes < lc_encode_bound(n, nbits),
 * and is lc_encode_t otherwise; lc_decode_sized is lc_decode_t that also refuses, before any read past the header
 * and with w_ref untouched, a blob whose header claims more than blob_bytes bytes (LC_ERR_BAD_BLOB; blob_bytes
 * below 512 likewise), so a forged size field cannot make the kernels read past a tightly allocated buffer.
 */
lc_ssize lc_encode_sized(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, size_t out_bytes, int dtype,
                         void* stream);
lc_ssize lc_decode_sized(const void* blob, size_t blob_bytes, void* w_ref, uint64_t n, int dtype, void* stream);

/*
 * lc_encode for callers that cannot allocate device or pinned memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc.  The same kernels as lc_encode, with their scratch (bucket counts, code
 * table, per-chunk notes, the slots that hold the code words before they are placed) in an array that is part of
 * the library's device image, LC_STATIC_MAX_N elements' worth: about 19 MB, which every GPU the library runs on
 * holds until the process ends.  The call allocates and frees nothing and does not wait: it enqueues on `stream`
 * and returns an lc_status (LC_OK, LC_ERR_BADARG as for lc_encode, LC_ERR_WORKSPACE if n > LC_STATIC_MAX_N,
 * LC_ERR_HIP).  Once the stream has reached the end of the call, `out` holds exactly what lc_encode would have
 * written: the blob, whose header carries its size (u64 at byte 40) and status (u32 at byte 48; 2 = non-finite
 * delta, header only).  w, w_ref: fp32, as for lc_encode.  All calls on one GPU share that GPU's array: calls that
 * overlap there (different streams, or replays of captured graphs in flight together) race; calls on one stream,
 * and calls of the other entry points, which have their own scratch, do not.
 */
#define LC_STATIC_MAX_N (1ull << 23)
int lc_encode_static(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* stream);

/*
 * Parameters stored as bf16 or fp16.  The method works on the fp32 delta (Algorithm 1 line 4), so the
 * 16-bit values are widened exactly to fp32, delta, buckets, representatives and codes are those of
 * lc_encode on the widened vectors, and the restore computes fl32(float(w_ref[i]) + representative) and
 * rounds it once, to nearest even, back to the storage type (elements of the merged bucket keep their
 * bits).  dtype: LC_F32 (then these are lc_encode / lc_decode), LC_BF16, LC_F16, LC_F64; w, w_ref: arrays of
 * that type, aligned to the element size (8-byte alignment of both takes the fast loads of 16-bit
 * types, 16-byte alignment those of fp64).  LC_F64: the whole method in binary64 (Section 3.1.1, footnote on
 * the bucket count): delta = fl64(w - w_ref), buckets by sign and the 11 exponent bits, representatives the
 * exactly rounded binary64 midranges, restore by one binary64 addition.  The blob records the element type at header offset 60 (0 for fp32 blobs) and restores only
 * into that type (else LC_ERR_BADARG); otherwise arguments, results and errors as lc_encode / lc_decode.
 */
enum lc_dtype { LC_F32 = 0, LC_BF16 = 1, LC_F16 = 2, LC_F64 = 3 };
lc_ssize lc_encode_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, void* stream);
lc_ssize lc_decode_t(const void* blob, void* w_ref, uint64_t n, int dtype, void* stream);

/*
 * lc_encode with a code table cache (Section 3.2, "Huffman Code Table Caching": the table of an
 * earlier checkpoint is reused while the buckets stay the same).  Here the reuse also saves the
 * first of lc_encode's two sweeps over w and w_ref: the cached table is applied while this
 * checkpoint's bucket populations are still being counted, and the coding is kept only if the
 * counts confirm it.
 *   cache  device memory, LC_CACHE_BYTES, 16-byte aligned, owned by the caller; all zero = empty.
 *          Holds the kept buckets and the code lengths of the last blob encoded with it.
 *   used   host pointer or NULL; receives 1 if the blob carries the cached table, else 0.
 * The cached table is used iff it is valid and was made with the same nbits, this checkpoint's
 * kept set (priority promotion on this delta's bucket populations) is the cached one, exactly
 * the symbols that have a cached code occur, and the payload under the cached lengths (the sum
 * of count x cached length) is at most n * nbits bits, so that the blob fits lc_encode_bound
 * like any other (a stale table on shifted populations could need more; this checkpoint's own
 * Huffman code never does).  The blob is then lc_encode's blob with the cached code lengths in
 * place of this delta's own Huffman lengths: the same kept buckets, counts and representatives,
 * hence the same restored weights, in a valid, possibly longer coding.  (Section 3.2 sorts the
 * buckets by population before a table is reused; that needs the populations before the first
 * code is written, i.e. the sweep this call saves, so the cached assignment is reused as it
 * is.)  Otherwise the blob is exactly lc_encode's.  Either way the cache afterwards describes
 * this blob; on an error it is left as it was.
 * Other arguments, return value and errors as lc_encode; cache NULL or misaligned: LC_ERR_BADARG.
 */
#define LC_CACHE_BYTES 256
lc_ssize lc_encode_cached(const float* w, const float* w_ref, uint64_t n, int nbits,
                          void* out, void* cache, int* used, void* stream);
/* The same for parameters of another type (dtype as for lc_encode_t).  A cache serves any of LC_F32, LC_BF16, LC_F16,
 * since all three code the fp32 delta.  LC_F64: the same rule on the binary64 delta's 12-bit bucket ids (a cache made
 * by the other types never matches), but coded in two sweeps like lc_encode_t: the reuse saves the Huffman build only. */
lc_ssize lc_encode_cached_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype,
                            void* cache, int* used, void* stream);

/*
 * Asynchronous form (Section 3.2, "Asynchronous Execution": only the first step depends on the model
 * state, the rest can run beside the next iteration).  lc_encode_async enqueues the kernels of
 * lc_encode (cache == NULL) or lc_encode_cached (cache != NULL) on `stream` and returns at once with
 * a ticket >= 0, or -(lc_status).  At most LC_MAX_TICKETS calls may be in flight (one more:
 * -LC_ERR_BADARG).  w and w_ref must stay unchanged until the call has read them for the last time:
 * lc_encode_release_inputs(ticket, other_stream) makes work enqueued on other_stream afterwards
 * (say the optimizer step that overwrites w) wait for exactly that point, without blocking the host;
 * it returns an lc_status.  out, and cache, belong to the call until lc_encode_wait(ticket, used)
 * returns: it blocks until the call has finished, returns what lc_encode / lc_encode_cached would
 * have returned (`used` may be NULL) and frees the ticket.
 * Calls on one stream run in order and share a scratch area; calls on different streams get different
 * areas (up to 8 per device, each of lc_workspace_bytes of the largest call it has served; with a
 * caller-supplied workspace there is one, and calls on other streams wait for each other) and run
 * side by side on the device.  So the slices of a large vector can be enqueued on one stream one
 * after the other and waited for once, and the tensors of a model can be spread over a few streams.
 */
#define LC_MAX_TICKETS 32
int lc_encode_async(const float* w, const float* w_ref, uint64_t n, int nbits, void* out, void* cache, void* stream);
/* lc_encode_async for parameters of type dtype (as for lc_encode_t / lc_encode_cached_t). */
int lc_encode_async_t(const void* w, const void* w_ref, uint64_t n, int nbits, void* out, int dtype, void* cache,
                      void* stream);
int lc_encode_release_inputs(int ticket, void* other_stream);
lc_ssize lc_encode_wait(int ticket, int* used);

/*
 * Algorithm 1 line 7 / Section 3 (C1): w_ref[i] += representative(symbol_i) in one
 * fp32 add; elements whose symbol is the merged (zero) bucket keep their exact bit
 * pattern.  `blob` is a device pointer to an LCB1 blob (16-byte aligned) whose header
 * n must equal `n`.  The header, the offset table and all lane lengths are validated
 * on the device before w_ref is touched (LC_ERR_BAD_BLOB leaves w_ref unchanged); a
 * lane stream that does not decode to exactly its stated length is only found
 * during the sweep and then also returns LC_ERR_BAD_BLOB, with w_ref partly updated.
 * Reads never leave [blob, blob + header.total_bytes) (lc_decode_sized also holds that size
 * against the caller's buffer).  A caller that must survive a damaged payload checks the blob with
 * lc_verify first (or sets LC_OPT_VERIFY_FIRST, below), or restores into a copy of w_ref.
 * Waits for `stream`; returns the bytes consumed or -(lc_status).
 */
lc_ssize lc_decode(const void* blob, float* w_ref, uint64_t n, void* stream);

/*
 * Everything lc_decode checks, from end to end, without any parameters: header, symbol table, offset table against
 * the lane lengths, and that every lane's string decodes (Algorithm 1 line 7's decoding, without the addition) to
 * exactly its stated length.  Reads [blob, blob + min(blob_bytes, header.total_bytes)) and nothing else; blob_bytes
 * as in lc_decode_sized (SIZE_MAX: trust the header).  n and dtype: what the blob is meant to restore.  Waits for
 * `stream`; returns the blob's size in bytes or -(lc_status).  A bit flipped inside a lane string that turns one code
 * into another of the same length is not damage any decoder can see.
 *
 * lc_set_option(LC_OPT_VERIFY_FIRST, 1) makes lc_decode, lc_decode_t, lc_decode_sized and lc_decode_many(_t) run
 * this lane-string check on every blob before the restoring sweep (gated on the device, no extra host round trip):
 * a blob with a damaged payload then leaves w_ref untouched like one with a damaged header, at the price of decoding
 * every blob twice (measured: a third more time for a dense restore of 2^28 elements, twice the 0.04 ms of a sparse
 * one of 138 M).  Off by default; process-wide; not applied by lc_decode_batch.
 */
lc_ssize lc_verify(const void* blob, size_t blob_bytes, uint64_t n, int dtype, void* stream);

/*
 * Restore from several checkpoints at once (Section 3, C1: u_t = u_0 + the sum of the decoded
 * deltas; Section 3.2, checkpoint merging): applies blobs[0], blobs[1], ... blobs[count-1] to
 * w_ref in this order.  The result is bit for bit what `count` successive lc_decode calls
 * give (one fp32 add per blob and element, in blob order), but w_ref is read and written
 * once per sweep of several blobs (up to 8; as many as the decoder's on-chip memory takes
 * at full occupancy, typically 4 to 6) instead of once per blob.
 *   blobs  HOST array of `count` DEVICE pointers to LCB1 blobs (16-byte aligned), each with
 *          header n equal to `n`; 1 <= count <= LC_MAX_MANY
 * Every blob is validated as in lc_decode before w_ref is touched.  Waits for `stream`;
 * returns the sum of the bytes consumed or -(lc_status).
 */
lc_ssize lc_decode_many(const void* const* blobs, int count, float* w_ref, uint64_t n, void* stream);
/* The same for parameters of type dtype, every blob of that type: bit for bit what `count` successive lc_decode_t
 * calls give, i.e. the running value is rounded to the storage type after every blob's addition.  LC_F64: every
 * blob is validated first as for the other types, then the blobs are applied one sweep each (one read and one write
 * of w_ref per blob). */
lc_ssize lc_decode_many_t(const void* const* blobs, int count, void* w_ref, uint64_t n, int dtype, void* stream);

/*
 * Many vectors in one call, each with a table of its own: tensor t is coded exactly as
 * lc_encode(w[t], w_ref[t], n[t], nbits, out[t]) would (the paper quantizes layer by layer: Figure 2,
 * Section 4.3; per-tensor tables keep small-scale tensors from being merged away by large-scale ones),
 * but the whole list takes six kernel launches instead of four per tensor.
 *   w, w_ref, out  HOST arrays of `count` DEVICE pointers (out[t]: 16-byte aligned, at least
 *                  lc_encode_bound(n[t], nbits) bytes); n: HOST array of lengths; 1 <= count <= LC_MAX_BATCH
 *   sizes          HOST array or NULL: blob size of each tensor, or -(lc_status) for a tensor whose delta
 *                  is not finite (its blob is then the 512-byte header with status 2; the others are fine)
 * Returns the sum of the blob sizes, or -(lc_status) of the first failing tensor.  Every blob is an
 * ordinary LCB1 blob for lc_decode.  lc_batch_workspace_bytes: scratch the call needs (host only).
 */
#define LC_MAX_BATCH 1024
size_t lc_batch_workspace_bytes(const uint64_t* n, int count, int nbits);
lc_ssize lc_encode_batch(const float* const* w, const float* const* w_ref, const uint64_t* n, int count, int nbits,
                         void* const* out, int64_t* sizes, void* stream);
/* The same for tensors that all hold parameters of type dtype: tensor t is coded as lc_encode_t(w[t], w_ref[t], n[t],
 * nbits, out[t], dtype) would.  LC_F64: by one such encode after the other inside the call. */
lc_ssize lc_encode_batch_t(const void* const* w, const void* const* w_ref, const uint64_t* n, int count, int nbits,
                           void* const* out, int64_t* sizes, int dtype, void* stream);

/*
 * The restore of such a list: tensor t as lc_decode(blobs[t], w_ref[t], n[t]) (Algorithm 1 line 7), all tensors
 * in five launches.  Every blob is validated like lc_decode's before the sweep; a tensor whose blob fails is
 * left untouched (its size comes back as -(lc_status)) while the others are restored.  Arrays as in
 * lc_encode_batch (blobs[t]: DEVICE pointer, 16-byte aligned; fp32 blobs only).  Returns the sum of the bytes
 * consumed, or -(lc_status) of the first failing tensor.
 */
lc_ssize lc_decode_batch(const void* const* blobs, float* const* w_ref, const uint64_t* n, int count, int64_t* sizes,
                         void* stream);
/* The same for tensors and blobs of element type dtype: tensor t as lc_decode_t(blobs[t], w_ref[t], n[t], dtype); a
 * blob of another element type fails with LC_ERR_BADARG.  LC_F64: by one such restore after the other inside the call. */
lc_ssize lc_decode_batch_t(const void* const* blobs, void* const* w_ref, const uint64_t* n, int count, int64_t* sizes,
                           int dtype, void* stream);

/*
 * Parse a header that the caller copied to HOST memory (at least 64 bytes).  Any
 * output pointer may be NULL.  Returns LC_OK, or LC_ERR_BAD_BLOB if magic/version
 * are wrong; `status` receives the header's status field.
 */
int lc_blob_info(const void* host_header, uint64_t* n, int* nbits, uint64_t* total_bytes, int* status);

/*
 * The size of a checkpoint after each stage of the method, in bits, from a header copied to HOST memory
 * (at least 64 bytes): bits[0] exponent-based quantization alone, n * ceil(log2 k) + 32 k with k the number
 * of non-empty buckets (Section 3.1.1); bits[1] after x-bit priority promotion, n * x + 32 * 2^x; bits[2]
 * after Huffman coding, the blob as stored with all its indices (the E, E+P, E+P+H of Section 4.3).
 * Returns LC_OK, LC_ERR_BADARG (NULL) or LC_ERR_BAD_BLOB (not an LCB1 header).
 */
int lc_blob_sizes(const void* host_header, uint64_t bits[3]);

/* Frees library-owned scratch on every device and the pinned result buffer. */
void lc_shutdown(void);

/* Static string for an lc_status (positive or negated). */
const char* lc_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* LC_H */
