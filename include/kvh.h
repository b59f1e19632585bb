/*
 * kvh.h — C ABI of the MI355X KV-cache level codec.
 *
 * The operations are the two compute steps of the AdaptCache executor (Design section: the
 * executor carries out the compression decisions; the estimator profiles what decompression
 * costs): compress a KV-cache entry with the quantisation method at a chosen rate, and
 * decompress a stored entry when it is loaded for reuse.  A KV-cache entry is a tensor of
 * l layers x N tokens x c channels for each of K and V (the paper's NumLayers, NumTokens,
 * NumChannels) stored at a quality level k (its Level); the only rate the paper names is
 * two bits per value (Preliminary Results).  The paper fixes no equations or formats for the codec; the
 * concrete definition implemented here is:
 *
 *   level 0/1/2 -> b = 8/4/2 bits per element, L = 2^b - 1
 *   K groups: 128 consecutive tokens of one channel; V groups: 128 consecutive channels of one
 *   token.  Per group: mn/mx = min/max (stored as raw 16-bit values, -0 as +0),
 *   r = f32(mx) - f32(mn); r < 2^-100 -> scale = inv = 0; else scale = r / L, inv = L / r;
 *   code q = clamp(rne((f32(x) - f32(mn)) * inv), 0, L); codes of a token row are packed in
 *   channel order, LSB-first; q == L decodes to mx, any other q to T16_rne(fma(q, scale, mn)).
 *
 * Blob (little-endian, position independent, movable with memcpy between storage tiers):
 *   64-byte header { u32 magic 'KVH1'; u16 version = 1; u8 dtype; u8 bits; u32 l; u32 n; u32 c;
 *                    u16 k_group = 128; u16 v_group = 128; u64 total_bytes;
 *                    u32 orig_tokens; u32 sink; u32 window (token dropping; 0 otherwise); zero padding }
 *   then for each layer:  kmeta[ceil(n/128)][c]{mn,mx}  kcodes[n][c*b/8]
 *                         vmeta[n][c/128]{mn,mx}        vcodes[n][c*b/8]
 *   each section padded with zero bytes to a multiple of 16.
 *   Level 3 (KVH_LEVEL_RAW) stores an entry in full quality — the paper's greedy step chooses per entry between
 *   evicting it, storing it in full quality and compressing it (Design section): bits = 16 in the header, no
 *   groups and no metadata sections, per layer the n K rows and then the n V rows exactly as given (every bit
 *   pattern is kept, non-finite values included).  Encode, decode, the token-dropping calls and the loader take
 *   it like any other level (token dropping at this level is dropping alone, without quantisation).
 *
 * Conventions
 *   - Pointers named *_dev are DEVICE pointers owned by the caller; everything else is host
 *     memory.  A blob pointer may also be pinned host memory that the device can address (the
 *     kernels then read or write it over the bus: encoding or transcoding straight into the host
 *     tier needs no staging copy).  The codec calls allocate nothing, keep no state, free nothing.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every call only
 *     ENQUEUES kernels and returns; results are valid once the caller has synchronised the
 *     stream.  Device buffers must stay alive until then.
 *   - Return value: KVH_OK or a negative kvh_status.  All argument errors are found on the host
 *     before anything is launched; on error nothing is enqueued.
 *   - Inputs must be finite.  Non-finite values give unspecified codes (never an out-of-bounds
 *     access).
 *   - Requirements: c a multiple of 128; blob bases 16-byte aligned; K/V bases 16-byte aligned
 *     and strides multiples of 8 elements (so every row segment is 16-byte aligned); channel
 *     stride 1.
 */
#ifndef KVH_H_
#define KVH_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { KVH_F16 = 0, KVH_BF16 = 1 } kvh_dtype;

typedef enum {
  KVH_OK = 0,
  KVH_E_ARG = -1,   /* null pointer, bad dtype, negative offset, bad block_tokens, too many items */
  KVH_E_LEVEL = -2, /* level outside 0..3, or the raw level passed to a call that only takes quantised levels */
  KVH_E_SHAPE = -3, /* l < 1, n < 1, c not a positive multiple of 128, chunk not a multiple of 128 */
  KVH_E_SIZE = -4,  /* blob capacity too small */
  KVH_E_ALIGN = -5, /* a base pointer or stride breaks the 16-byte rule */
  KVH_E_HIP = -6    /* the kernel launch itself failed */
} kvh_status;

/* Value written to *status_dev by a decode kernel whose blob header disagrees with the call. */
#define KVH_DEV_HEADER_MISMATCH 1

/* The level table (reading of the paper's Level k, its compression rate): 3 quantised levels, 0..2, and the
 * raw level below them in the numbering. */
int kvh_num_levels(void);
#define KVH_LEVEL_RAW 3
/* Bits per element of a level: 0,1,2 -> 8,4,2; KVH_LEVEL_RAW -> 16; anything else -> -1. */
int kvh_level_bits(int level);
/* Exact size in bytes of a blob holding n_tokens tokens; 0 on bad arguments.  This is the
 * size(i, M_i, R_i) term of the paper's utility for the quantisation method. */
size_t kvh_blob_size(int l, int n_tokens, int c, int level);

/* A K/V tensor pair in device memory.  Host struct; k and v are device pointers to 16-bit
 * elements.  Contiguous use: element (layer, token, ch) of K is k[layer*layer_stride +
 * token*token_stride + ch].  Paged use (decode only): the tensors are [l][P][block_tokens][c],
 * token_stride is the stride between slots of a block (normally c) and blocks are dense:
 * physical row = block * block_tokens + slot.  Strides are in elements.  A destination view needs
 * token_stride >= c (rows must not overlap); anything smaller is KVH_E_ARG. */
typedef struct {
  void* k;
  void* v;
  int64_t layer_stride;
  int64_t token_stride;
} kvh_kv_view;

/* Compress: encode tokens [0, N) of `kv` (all l layers, K and V) into ONE blob at `level`.
 * blob_cap must be >= kvh_blob_size(l, N, c, level).  The last K token-group may be partial. */
int kvh_encode(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int level, void* blob_dev, size_t blob_cap,
               void* stream);

/* Compress a long entry chunk by chunk (chunks are independently decodable): chunk i covers
 * tokens [i*chunk, min(N, (i+1)*chunk)), is encoded at levels[i] and written at
 * (char*)blobs_dev + blob_offsets[i].  `levels` and `blob_offsets` are HOST arrays of
 * ceil(N/chunk) entries; offsets must be multiples of 16 and every blob must end at or before
 * `cap`.  chunk must be a multiple of 128.  The descriptors travel in the kernel arguments, 32
 * chunks per launch (the library owns no device memory to put them in), all asynchronous on
 * `stream`. */
int kvh_encode_chunked(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int chunk, const int8_t* levels,
                       void* blobs_dev, const size_t* blob_offsets, size_t cap, void* stream);

/* One encode job of a batch.  The ARRAY of items lives in device memory. */
typedef struct {
  void* blob;         /* device pointer, 16-byte aligned, room for kvh_blob_size(l, n_tokens, c, level) */
  int64_t src_token0; /* first token of the source view covered by this blob */
  int32_t n_tokens;   /* 1 .. max_tokens_per_item */
  int32_t level;      /* 0 .. 2 */
} kvh_enc_item;

/* Compress many chunks of one source view in ONE launch.  The host cannot see the items, so
 * the caller guarantees their validity (levels in range, blobs large enough and disjoint,
 * source rows inside the view).  What the kernel can see it enforces: an item with n_tokens < 1,
 * a bad level, or n_tokens > max_tokens_per_item (more rows than the launch covers) is skipped as
 * a whole — nothing is written to its blob, not even the header, so a later decode of that buffer
 * reports KVH_DEV_HEADER_MISMATCH rather than returning half an entry.  n_items <= 65535. */
int kvh_encode_batch(const kvh_enc_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                     const kvh_kv_view* src, void* stream);

/* Decompress one blob of n_tokens tokens stored at `level` (the caller's index knows the
 * method and rate of every entry — the (M_i, R_i) of the paper's utility) into `dst`:
 *   page_table_dev == NULL: token t goes to row dst_token0 + t of the contiguous view;
 *   otherwise: logical position s = dst_token0 + t goes to physical block
 *              page_table_dev[s / block_tokens], slot s % block_tokens (one table for all layers
 *              and for K and V).
 * The kernel first compares the blob header with (dt, l, n_tokens, c, level); on disagreement it
 * writes KVH_DEV_HEADER_MISMATCH to *status_dev (if not NULL) and writes nothing else.  The
 * caller zeroes *status_dev beforehand; it is never written on success. */
int kvh_decode(const void* blob_dev, kvh_dtype dt, int l, int n_tokens, int c, int level, const kvh_kv_view* dst,
               int64_t dst_token0, const int32_t* page_table_dev, int block_tokens, int32_t* status_dev, void* stream);

/* Decompress a long entry chunk by chunk (the mirror of kvh_encode_chunked): chunk i holds tokens
 * [i*chunk, min(N, (i+1)*chunk)), was stored at levels[i], starts at (char*)blobs_dev + blob_offsets[i] and goes to
 * logical positions dst_token0 + i*chunk onward of `dst` (contiguous or paged, as kvh_decode).  `levels` and
 * `blob_offsets` are HOST arrays of ceil(N/chunk) entries; offsets must be multiples of 16.  status_dev, if not
 * NULL, has one zeroed int32 per chunk.  32 chunks per kernel launch (descriptors in the kernel arguments), all
 * asynchronous on `stream`, no synchronisation in between; a caller whose chunks arrive one at a time calls
 * kvh_decode per chunk instead. */
int kvh_decode_chunked(const void* blobs_dev, const size_t* blob_offsets, const int8_t* levels, kvh_dtype dt, int l, int N,
                       int c, int chunk, const kvh_kv_view* dst, int64_t dst_token0, const int32_t* page_table_dev,
                       int block_tokens, int32_t* status_dev, void* stream);

/* One decode job of a batch.  The ARRAY of items lives in device memory. */
typedef struct {
  const void* blob;          /* device pointer, 16-byte aligned */
  int32_t n_tokens;          /* 1 .. max_tokens_per_item */
  int32_t level;             /* level the blob was stored at */
  int64_t dst_token0;        /* logical position of the blob's first token in its request */
  const int32_t* page_table; /* device pointer to the request's table, or NULL for contiguous */
} kvh_item;

/* Decompress many blobs (mixed levels, mixed lengths) into one destination view in ONE launch.
 * status_dev, if not NULL, is an int32 array of n_items entries (zeroed by the caller); entry i
 * is set to KVH_DEV_HEADER_MISMATCH when item i's header disagrees, and that item writes
 * nothing.  The same happens to an item whose level is out of range, whose n_tokens exceeds
 * max_tokens_per_item (more rows than the launch covers), or whose rows would leave the 31-bit row
 * range (dst_token0 < 0 or dst_token0 + n_tokens > 2^31 - 1): refused as a whole, never decoded in
 * part.  Items with n_tokens < 1 are skipped silently.
 * Destinations of different items must not overlap.  n_items <= 65535. */
int kvh_decode_batch(const kvh_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                     const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream);

/* ---- Token dropping ------------------------------------------------------------------------------
 * The paper's second compression method: for contexts that matter mostly at their beginning and their
 * end, dropping the tokens in between suits (Introduction); the evaluation's fixed-rate
 * token-dropping baseline (Preliminary Results).  The paper defines nothing further; here an entry of N
 * tokens keeps its first `sink` and last `window` tokens (all of them if sink + window >= N) and the
 * kept tokens, in order, are stored as an ordinary blob of n = kvh_kept_tokens(N, sink, window) tokens
 * at a quantised level, so dropping composes with quantisation.  Header bytes 32..43 record
 * (N, sink, window); they are zero in ordinary blobs, and kvh_decode / kvh_decode_batch reject a blob
 * in which they are not. */

/* Number of tokens kept: min(N, sink + window); 0 on bad arguments (N < 1, negative, sink + window < 1). */
int kvh_kept_tokens(int N, int sink, int window);

/* Gather the kept tokens of `kv` (a view of N tokens) and encode them into one blob at `level`.
 * blob_cap must be >= kvh_blob_size(l, kvh_kept_tokens(N, sink, window), c, level). */
int kvh_encode_kept(const kvh_kv_view* kv, kvh_dtype dt, int l, int N, int c, int sink, int window, int level,
                    void* blob_dev, size_t blob_cap, void* stream);

/* Decode a token-dropped blob.  compact == 0: kept token i goes back to logical position dst_token0 +
 * (its original position), the rows of dropped tokens are not touched; compact != 0: to dst_token0 + i.
 * Contiguous or paged destination and status word as for kvh_decode; (N, sink, window) must equal the
 * values the blob was encoded with, else KVH_DEV_HEADER_MISMATCH and nothing is written. */
int kvh_decode_kept(const void* blob_dev, kvh_dtype dt, int l, int N, int c, int sink, int window, int level,
                    const kvh_kv_view* dst, int64_t dst_token0, int compact, const int32_t* page_table_dev,
                    int block_tokens, int32_t* status_dev, void* stream);

/* One token-dropping encode job of a batch.  The ARRAY of items lives in device memory. */
typedef struct {
  void* blob;          /* device pointer, 16-byte aligned, room for kvh_blob_size(l, kept tokens, c, level) */
  int64_t src_token0;  /* first token of the entry in the source view */
  int32_t orig_tokens; /* N: tokens of the entry */
  int32_t sink;        /* first tokens kept */
  int32_t window;      /* last tokens kept */
  int32_t level;       /* 0 .. 2 */
} kvh_kept_enc_item;

/* kvh_encode_kept for many entries of one source view in ONE launch.  max_kept_tokens_per_item bounds
 * kvh_kept_tokens(orig_tokens, sink, window) over the items.  The caller guarantees the items' validity
 * (as for kvh_encode_batch); items with a bad level, nothing kept, or more kept tokens than
 * max_kept_tokens_per_item are skipped as a whole (no header is written).  n_items <= 65535. */
int kvh_encode_kept_batch(const kvh_kept_enc_item* items_dev, int n_items, int max_kept_tokens_per_item, kvh_dtype dt,
                          int l, int c, const kvh_kv_view* src, void* stream);

/* One decode job of a batch that may hold token-dropped blobs.  The ARRAY lives in device memory.  For an
 * ordinary blob orig_tokens = sink = window = 0.  For a token-dropped blob they are the values it was encoded
 * with and n_tokens = kvh_kept_tokens(orig_tokens, sink, window); compact as for kvh_decode_kept. */
typedef struct {
  const void* blob;          /* device pointer, 16-byte aligned */
  int32_t n_tokens;          /* tokens stored in the blob, 1 .. max_tokens_per_item */
  int32_t level;             /* level the blob was stored at */
  int64_t dst_token0;        /* logical position of the entry's first token in its request */
  const int32_t* page_table; /* device pointer to the request's table, or NULL for contiguous */
  int32_t orig_tokens, sink, window;
  int32_t compact;
} kvh_kept_item;

/* kvh_decode_batch over items that may be token-dropped (mixed with ordinary ones).  An item whose header
 * disagrees, whose n_tokens is not what (orig_tokens, sink, window) keep, or which kvh_decode_batch would
 * refuse (n_tokens > max_tokens_per_item; rows outside the 31-bit range, counting orig_tokens rows for an
 * entry decoded back to its original positions) gets KVH_DEV_HEADER_MISMATCH and writes nothing. */
int kvh_decode_kept_batch(const kvh_kept_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l,
                          int c, const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream);

/* ---- Transcode ------------------------------------------------------------------------------------
 * The paper's policy lowers the quality of stored entries step by step (a further compression from
 * rate m to rate n; Design section, marginal utility drop).  kvh_transcode re-compresses a stored blob
 * from level_in to level_out in one kernel, without materialising 16-bit KV: the output is, byte for
 * byte, what kvh_encode would produce from the tensors kvh_decode writes for the source blob.
 * Precondition: the source blob was written by this library (encode, encode_kept or transcode), so that
 * every group holds its smallest and largest code; a hand-made blob without that property gets the
 * source's group statistics instead of recomputed ones.  Token-dropping header words are carried over.
 * Source and destination must not overlap.  Any pair of quantised levels is allowed (going up only re-packs
 * what the lower level kept).  The raw level is refused here (KVH_E_LEVEL; in a batch: KVH_DEV_HEADER_MISMATCH):
 * a raw blob holds rows, not codes, so compressing it further is kvh_encode on a view of its rows (K rows of
 * layer j start at byte 64 + j * 4 n c, the V rows 2 n c bytes later: k = blob + 64, v = blob + 64 + 2 n c,
 * layer_stride = 2 n c elements, token_stride = c), and expanding a quantised blob to it is kvh_decode. */

/* The kernel checks the source header against (dt, l, n_tokens, c, level_in) — n_tokens is the number
 * of tokens stored in the blob — and on disagreement writes KVH_DEV_HEADER_MISMATCH to *status_dev (if
 * not NULL; zeroed by the caller) and nothing else.  dst_cap must be >= kvh_blob_size(l, n_tokens, c,
 * level_out); the caller guarantees kvh_blob_size(l, n_tokens, c, level_in) readable bytes at src_dev. */
int kvh_transcode(const void* src_dev, kvh_dtype dt, int l, int n_tokens, int c, int level_in, int level_out,
                  void* dst_dev, size_t dst_cap, int32_t* status_dev, void* stream);

/* One transcode job of a batch.  The ARRAY of items lives in device memory. */
typedef struct {
  const void* src;   /* device pointer, 16-byte aligned: blob stored at level_in */
  void* dst;         /* device pointer, 16-byte aligned: room for kvh_blob_size(l, n_tokens, c, level_out) */
  int32_t n_tokens;  /* tokens stored in the blob, 1 .. max_tokens_per_item */
  int32_t level_in;  /* 0 .. 2 */
  int32_t level_out; /* 0 .. 2 */
  int32_t reserved;  /* 0 */
} kvh_tc_item;

/* Transcode many blobs (mixed lengths and level pairs) in ONE launch.  status_dev as for
 * kvh_decode_batch; items with n_tokens < 1 are skipped, items with a level out of range or with
 * n_tokens > max_tokens_per_item get KVH_DEV_HEADER_MISMATCH and write nothing (no destination
 * header either).  Buffers of different items must not overlap.  n_items <= 65535. */
int kvh_transcode_batch(const kvh_tc_item* items_dev, int n_items, int max_tokens_per_item, kvh_dtype dt, int l, int c,
                        int32_t* status_dev, void* stream);

/* ---- Load path ------------------------------------------------------------------------------------
 * A stored entry costs size / Bandwidth of loading delay before it can be reused, plus its decompression
 * (the paper's utility charges the first, its estimator profiles the second; Design section).  The loader
 * moves blobs that sit in PINNED host memory (the DRAM tier) through a ring of device staging slots and
 * decodes them.  Consecutive blobs are packed into groups that fill a slot; a group is moved by one launch
 * of a copy kernel that reads the host memory in place, then decoded by one batched decode launch, so the
 * copy of group g + 1 overlaps the decode of group g.  It is a host-side object: one copy stream (default
 * priority) and two events per slot; the staging buffer is the caller's device memory.  Not thread-safe; one
 * loader serves one device (the one current at creation). */
typedef struct kvh_loader kvh_loader;

/* One blob to load.  HOST array, host struct. */
typedef struct {
  const void* blob_host;     /* pinned (device-visible) host memory, 16-byte aligned, holding
                                kvh_blob_size(l, n_tokens, c, level) bytes; ordinary pageable memory is refused */
  int32_t n_tokens;          /* tokens in the blob */
  int32_t level;             /* level it was stored at */
  int64_t dst_token0;        /* logical position of its first token in the destination */
  const int32_t* page_table; /* DEVICE pointer to the request's table, or NULL for contiguous */
  int32_t orig_tokens, sink, window; /* all 0 for an ordinary blob; else what the blob was token-dropped with,
                                        and n_tokens = kvh_kept_tokens(orig_tokens, sink, window) */
  int32_t compact;           /* as for kvh_decode_kept */
} kvh_load_item;

/* Create a loader over `staging_dev` (device memory, 16-byte aligned, staging_bytes long), cut into n_slots
 * equal slots (1..64; 2 = double buffering).  The first 1.5 KiB of a slot holds descriptors; the rest
 * (kvh_loader_slot_bytes) must hold the largest blob that will be loaded and is best sized for several. */
int kvh_loader_create(kvh_loader** out, void* staging_dev, size_t staging_bytes, int n_slots);
/* Bytes a slot offers to blobs (0 for NULL). */
size_t kvh_loader_slot_bytes(const kvh_loader* loader);
/* Enqueue, group by group in item order: wait until the next slot is free, copy the group's blobs host ->
 * slot on the loader's copy stream, then decode them on `stream` into `dst` (contiguous or paged, as
 * kvh_decode_kept_batch: ordinary and token-dropped blobs may be mixed).  The copies start after the work already
 * enqueued on `stream` (so blobs that an earlier call on it writes into host memory are complete when they are
 * read).  Returns once everything is enqueued; results
 * are valid after `stream` has been synchronised; host blobs and the staging buffer must stay alive until
 * then.  status_dev, if not NULL, has one zeroed int32 per item (KVH_DEV_HEADER_MISMATCH as for
 * kvh_decode_batch).  All items are validated before anything is enqueued. */
int kvh_loader_run(kvh_loader* loader, const kvh_load_item* items, int n_items, kvh_dtype dt, int l, int c,
                   const kvh_kv_view* dst, int block_tokens, int32_t* status_dev, void* stream);
/* Wait for the loader's copies, then release its stream and events (not the staging buffer). */
int kvh_loader_destroy(kvh_loader* loader);

/* Allocation-free form of kvh_loader_run, for callers that cannot allocate or create anything: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same items, same checks, same result as
 * kvh_loader_run, but there is no loader object, no second stream and no event: the one staging slot is a
 * KVH_STATIC_SCRATCH_BYTES array inside the library's code object (every GPU the library runs on holds its own
 * copy until the process ends), and each group of blobs is copied into it and decoded from it on `stream`, one
 * after the other.  The call allocates and frees nothing (no hipMalloc/hipFree, no stream or event creation).
 * The first call on a device looks up the array's address there and should be made outside any capture.
 * A blob larger than KVH_STATIC_SCRATCH_BYTES - 1536 (the descriptor area) is refused with KVH_E_SIZE before
 * anything is enqueued.  All calls on one GPU share that GPU's array, which keeps the last call's bytes; nothing
 * in it has to start at zero.  Calls that overlap in time on one GPU (different streams, different threads)
 * race on it: keep them on one stream, or order them yourself. */
#define KVH_STATIC_SCRATCH_BYTES (40u << 20)
int kvh_load_static(const kvh_load_item* items, int n_items, kvh_dtype dt, int l, int c, const kvh_kv_view* dst,
                    int block_tokens, int32_t* status_dev, void* stream);

/* ---- Storage policy (host only; no device work) -------------------------------------------------------
 * The paper's policy optimizer (Design section): Utility(i) = Freq(i) * (alpha * Quality(i, M_i, R_i) -
 * size(i, M_i, R_i) / Bandwidth); the marginal utility drop of going from rate m to rate n is
 * (Utility(i, m) - Utility(i, n)) / (bytes the step frees); per storage tier the choice (evict, store in
 * full quality, compress) with the minimal marginal utility drop is taken greedily until the tier holds what
 * is left.  Readings: the utility's missing parenthesis closes after the fraction; eviction has size 0 and
 * utility 0; an entry starts at its best allowed choice; a step may go to any smaller choice (this walks the
 * upper convex hull and reaches the linear-relaxation optimum up to one fractional step); what a tier evicts
 * is offered to the next tier with that tier's bandwidth.  Quality values come from the caller (the paper's
 * estimator builds them from datasets; none are shipped here). */
typedef struct {
  double freq;        /* estimated future hit frequency, >= 0 */
  int32_t first;      /* index of the entry's first choice in `sizes` / `qualities` */
  int32_t n_choices;  /* >= 1; choices ordered by strictly decreasing size, choice 0 = full quality */
  int32_t min_choice; /* 0 for a new entry; for a stored entry the choice it is held at (it cannot regain quality) */
  int32_t reserved;   /* 0 */
} kvh_policy_entry;

typedef struct {
  double bandwidth; /* bytes per second from this tier to the GPU, > 0 */
  double capacity;  /* bytes, >= 0 (may be +inf) */
} kvh_policy_tier;

double kvh_policy_utility(double freq, double alpha, double quality, double size_bytes, double bandwidth);
double kvh_policy_marginal_utility_drop(double u_m, double u_n, double size_m, double size_n);

/* Plan all entries over the tiers (tier 0 first).  sizes[] are whole numbers of bytes (e.g. kvh_blob_size);
 * tier_out[i] = tier index or -1 (evicted everywhere), choice_out[i] = chosen choice or -1; *total_utility_out
 * (nullable) = sum of the utilities of the placed entries in index order.  Host arrays throughout.
 * Errors: KVH_E_ARG (null pointer, counts < 1, non-finite or negative values, sizes not whole or not strictly
 * decreasing), KVH_E_SHAPE (an entry's choice range or min_choice out of bounds), KVH_E_SIZE (the entries'
 * largest sizes add up to 2^53 bytes or more, where sums of doubles stop being exact). */
int kvh_policy_plan(const kvh_policy_entry* entries, int n_entries, const double* sizes, const double* qualities,
                    int n_choices_total, const kvh_policy_tier* tiers, int n_tiers, double alpha, int32_t* tier_out,
                    int32_t* choice_out, double* total_utility_out);

/* Plain device-to-device copy kernel of `bytes` bytes (a multiple of 16, both pointers 16-byte
 * aligned).  Not part of the codec: the benchmark uses it as the known-size reference that
 * scales the HBM byte counters and as the practical copy-bandwidth ceiling of the device. */
int kvh_copy_probe(void* dst_dev, const void* src_dev, size_t bytes, void* stream);

/* Traffic generator with a chosen mix of reads and writes and no arithmetic, also not part of the codec: a unit is
 * reads_per_unit x 16 bytes read per lane and writes_per_unit x 16 bytes written per lane (1 KiB per wave and
 * access, non-temporal stores); n_units units (a multiple of 256) are processed, so src_dev must hold n_units * reads_per_unit * 16
 * bytes and dst_dev n_units * writes_per_unit * 16 bytes (at least 16).  Supported (reads, writes): (1,0) pure
 * read, (0,1) pure fill, (1,1) copy, (1,2) (1,4) (1,8) the decoder's mixes at 8 / 4 / 2 bits, (2,1) (4,1) (8,1)
 * the encoder's; anything else is KVH_E_ARG.  The benchmark reports these next to the codec's kernels as the
 * ceilings the memory system sets for such streams. */
int kvh_stream_probe(void* dst_dev, const void* src_dev, size_t n_units, int reads_per_unit, int writes_per_unit,
                     void* stream);

/* Timing of one launch, for callers that profile (not part of the codec; Design section, Estimator: the decompression
 * overhead of an entry is something to be measured).  The two events (hipEvent_t, created by the caller with timing
 * enabled) are recorded by the NEXT encode, decode or transcode kernel that this host thread launches through the
 * library: `start_event` when that kernel starts executing, `stop_event` when it has finished, on the launch's
 * stream, so that hipEventElapsedTime(start, stop) is the kernel's own duration - what a kernel trace reports -
 * without the queue packets that events recorded around a launch put between neighbouring kernels.  The pair is
 * used once and forgotten; a call that launches several kernels times its first, and a call that is refused
 * before it launches anything leaves the pair waiting for the next launch.  Errors: KVH_E_ARG (null event). */
int kvh_time_next_launch(void* start_event, void* stop_event);

/* Self-test of the arithmetic shortcut behind the group parameters (Sec. 3.2's quantisation: scale = r / L and
 * inv = L / r are correctly rounded fp32 quotients).  The kernels form both with a reciprocal and two fused
 * corrections instead of the division sequence; that this returns the division's bits is a property of the
 * device's reciprocal instruction, which this call checks on the device it runs on: every finite fp32 range r from
 * 2^-100 (the smallest a non-degenerate group can have) upwards, about 1.9e9 values, at L = 255, 15, 3.  mismatches_dev: device array of 6 uint64 that the CALLER has zeroed (8-byte aligned); the kernel
 * adds the number of values whose r / L differs at 8 / 4 / 2 bits to [0..2] and whose L / r differs to [3..5].
 * All six are 0 on gfx950; anything else means the codec's parameters are not the specified ones on this device.
 * About one second of GPU time.  Errors: KVH_E_ARG (null or misaligned pointer), KVH_E_HIP. */
int kvh_selftest_division(uint64_t* mismatches_dev, void* stream);

/* Static description of a status code. */
const char* kvh_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* KVH_H_ */
