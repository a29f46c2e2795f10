/* rlkv.h - decode-time attention over a head-mixed KV cache on one MI355X (gfx950).
 *
 * The operation (paper Sec. 3.1, Sec. 3.3 last paragraph, Sec. 4.3, App. B "Local
 * Attention Implementation"): every (layer, KV head) is either
 *   - FULL        : keeps the K/V rows of every cached position, or
 *   - COMPRESSED  : keeps a constant-size store of the first `sink` positions plus the
 *                   most recent `recent` positions (a fixed-size circular buffer),
 * and one decode step computes, for every query head, ordinary scaled-dot-product
 * softmax attention over whatever its KV head retains.  Query heads are grouped
 * (GQA): query head i reads KV head i / (n_q_heads / n_kv_heads), and the
 * full/compressed choice is per KV head (Sec. 3.1).
 *
 * Conventions
 *   - plain C ABI; `void* stream` is a hipStream_t (NULL = the default stream).
 *   - "host" / "device" on every pointer says where the memory must live.
 *   - every call returns an rlkv_status_t; nothing throws or aborts.  All argument
 *     validation happens on the host before the first HIP call.
 *   - append / decode are asynchronous on `stream`; capacity and empty-cache errors come
 *     from a host-side mirror of the lengths, so no call waits for the GPU except the two
 *     rlkv_get_* introspection calls, rlkv_profile_collect and rlkv_cache_destroy, which wait
 *     for the stream the handle was last used on (never for the whole device).
 *   - a cache handle is not thread-safe and must be used from one stream at a time.
 *   - the library never owns q / k / v / out, and never frees a caller-provided arena.
 */
#ifndef RLKV_H
#define RLKV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rlkv_cache rlkv_cache_t; /* opaque, owned by the library */

typedef enum {
  RLKV_OK = 0,
  RLKV_ERR_INVALID_ARG = 1, /* null pointer, bad dimension, layer out of range, ...      */
  RLKV_ERR_OOM = 2,         /* arena too small / device allocation failed                */
  RLKV_ERR_CAPACITY = 3,    /* append would exceed max_len[seq], or the page pool is used up */
  RLKV_ERR_STATE = 4,       /* decode with an empty sequence; a call the cache was not created for */
  RLKV_ERR_HIP = 5,         /* a HIP runtime call failed (no usable GPU, launch error)   */
  RLKV_ERR_TOO_LARGE = 6    /* rlkv_decode_attention_noalloc: the static scratch buffer is too small for the call */
} rlkv_status_t;

typedef enum { RLKV_F32 = 0, RLKV_BF16 = 1 } rlkv_dtype_t;

/* Which decode kernel (and with it which in-HBM store layout) a cache uses.
 *   RLKV_KERNEL_VALU : row-major stores [slot][head_dim]; dot products on the vector
 *                      ALU with wavefront DPP reductions.  fp32 and bf16.  The fp32 path, and
 *                      for bf16 the comparison baseline: at a group size of 7 its bf16 form
 *                      is bound by the vector ALU, not by memory, and streams at less than
 *                      60 % of the rate of the MFMA kernel; the append of a fused step is a
 *                      launch of its own; no paging, no prefill.
 *   RLKV_KERNEL_MFMA : stores tiled so that a 128-bit load per lane lands directly in
 *                      MFMA operand registers; bf16 only.
 *   RLKV_KERNEL_AUTO : MFMA for bf16, VALU for fp32. */
typedef enum { RLKV_KERNEL_AUTO = 0, RLKV_KERNEL_VALU = 1, RLKV_KERNEL_MFMA = 2 } rlkv_kernel_t;

typedef struct {
  int32_t n_layers;
  int32_t n_q_heads;   /* multiple of n_kv_heads; group size n_q_heads/n_kv_heads <= 16 */
  int32_t n_kv_heads;
  int32_t head_dim;    /* must be 128                                                   */
  int32_t batch;       /* number of sequence slots; batch * n_kv_heads <= 65535         */
  int32_t sink;        /* S >= 0 : positions 0..S-1 are never evicted                   */
  int32_t recent;      /* R >= 1 : the newest R positions are retained (newest included) */
  int32_t dtype;       /* rlkv_dtype_t of K, V, Q and the output                        */
  int32_t kernel;      /* rlkv_kernel_t                                                 */
  int32_t device;      /* HIP device ordinal                                            */
  const uint8_t* full_mask; /* host [n_layers * n_kv_heads]; 1 = full, 0 = compressed; copied */
  const int32_t* max_len;   /* host [batch]; capacity of a full head, in tokens; copied      */
  void* arena;         /* device memory owned by the caller, or NULL: the library allocates */
  size_t arena_bytes;  /* size of `arena` (ignored when arena == NULL)                  */
  int32_t page_tokens; /* 0: every full head keeps one contiguous store of max_len[b] rows per
                          sequence.  > 0: full heads are paged (see below); a power of two in
                          [32, 65536]; needs the MFMA kernel                              */
  int32_t pool_pages;  /* paged only: pages in the pool of each full (layer, head)       */
  int32_t prefill_tokens; /* largest chunk (tokens per sequence) rlkv_prefill_attention will be given;
                          sizes its staging buffer (and adds 130 MiB of scratch to the arena, see
                          rlkv_prefill_attention).  0: that call is not available.  Needs the
                          MFMA kernel                                                    */
  /* Tuning, 0 = the library's default everywhere (what every measured figure uses): */
  int32_t decode_wgs_per_cu;       /* decode workgroups per compute unit, 1..8; default 1        */
  int32_t prefill_min_share_tiles; /* fewest 32-key tiles a share of a divided prefill workgroup may
                                      have (see rlkv_prefill_attention); default 80              */
  int32_t prefill_two_group_only;  /* 1: rlkv_prefill_attention never picks its single-group kernel form
                                      for a layer that does not blend (tests run small shapes through
                                      the form the large ones take); default 0                   */
} rlkv_config_t;

/* Paged full heads (Sec. 4.3: a standard paged cache for the full heads beside the fixed-size
 * buffers of the compressed ones).  With page_tokens > 0 each full (layer, KV head) owns a pool
 * of pool_pages pages of page_tokens rows; a sequence holds ceil(n / page_tokens) pages, named
 * by one block table per sequence that all layers and heads share (page i of a sequence has the
 * same index in every pool).  Pages are taken from a free list when an append first needs them
 * and returned by rlkv_cache_reset, so memory follows the tokens actually cached instead of
 * max_len, and max_len[b] only bounds the block table.  An append that finds the free list too
 * short returns RLKV_ERR_CAPACITY and writes nothing.  Results are identical to the contiguous
 * layout.  All calls on one handle must use one stream, as pages change owners in stream order. */

/* Bytes of device memory a cache with this configuration needs (stores, tables, split-K
 * scratch).  Reads only the host fields; returns 0 for an invalid configuration. */
size_t rlkv_cache_required_bytes(const rlkv_config_t* cfg /* host */);

/* Builds the cache (Sec. 4.3: one pool of full stores, one of fixed-size sink+ring
 * stores): lays the stores out in the arena, uploads the tables, sets all lengths to 0
 * and every ring slot to "empty".  `arena` must be 256-byte aligned and at least
 * rlkv_cache_required_bytes(cfg) long.  On success *out owns the handle.  A cache also holds a
 * block of pinned host memory (up to 64 MiB) in which the split-K work lists are written before
 * they are copied to the device; such blocks are recycled between caches and kept for the life
 * of the process. */
rlkv_status_t rlkv_cache_create(const rlkv_config_t* cfg /* host */, rlkv_cache_t** out /* host */);

/* Waits for the stream the handle was last used on (work of this cache may still be queued
 * there), then frees the handle and, if the library allocated it, the arena. */
rlkv_status_t rlkv_cache_destroy(rlkv_cache_t* cache);

/* Empties sequence `seq` in every layer (seq = -1: all sequences): length 0, ring slots
 * empty.  Asynchronous on `stream`. */
rlkv_status_t rlkv_cache_reset(rlkv_cache_t* cache, int32_t seq, void* stream);

/* Appends n_tokens new positions to every sequence of `layer`.
 *   k, v : device, [batch][n_kv_heads][n_tokens][head_dim] in cfg.dtype.
 * A full head stores position p at row p.  A compressed head stores p < S in slot p and
 * p >= S in slot S + ((p - S) mod R), overwriting (evicting) position p - R; with
 * n_tokens > R only the positions that survive are written, so the result equals
 * n_tokens single-token appends (App. B: only the first-S and recent-R tokens are kept).
 * RLKV_ERR_CAPACITY (nothing written) if any sequence would exceed its max_len. */
rlkv_status_t rlkv_append(rlkv_cache_t* cache, int32_t layer, const void* k /* device */,
                          const void* v /* device */, int32_t n_tokens, void* stream);

/* Same, with a per-sequence token count: sequence b appends the first n_tokens[b] rows
 * of its [stride_tokens] block (0 <= n_tokens[b] <= stride_tokens).
 *   k, v     : device, [batch][n_kv_heads][stride_tokens][head_dim]
 *   n_tokens : host, [batch]; copied before the call returns. */
rlkv_status_t rlkv_append_ragged(rlkv_cache_t* cache, int32_t layer, const void* k /* device */,
                                 const void* v /* device */, const int32_t* n_tokens /* host */,
                                 int32_t stride_tokens, void* stream);

/* One decode step of attention for `layer` (Sec. 3.1 Eq. 1 with every gate at 0 or 1,
 * as discretised at inference, Sec. 3.3): for each sequence b with n cached positions
 * and each query head i, out = softmax(softmax_scale * q . K^T) V over the positions its
 * KV head retains: all n for a full head; {j < S} U {j >= n - R} for a compressed head.
 *   q, out : device, [batch][n_q_heads][head_dim] in cfg.dtype.
 * Scores, softmax and accumulation are fp32; the output is rounded to cfg.dtype (RNE).
 * RLKV_ERR_STATE if any active sequence of the layer is empty (see rlkv_set_active). */
rlkv_status_t rlkv_decode_attention(rlkv_cache_t* cache, int32_t layer, const void* q /* device */,
                                    void* out /* device */, float softmax_scale, void* stream);

/* rlkv_decode_attention for callers that cannot allocate device memory or hand the library a
 * workspace at the time of the call: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, results (bit for bit) and errors as rlkv_decode_attention,
 * but the split-K partials of the call are kept in a buffer that is part of the library image
 * (a file-scope device array of 16384 rows x 130 floats = 8.1 MiB, held by every GPU the library
 * runs on until the process ends) instead of in the arena, and the call allocates nothing: no
 * hipMalloc / hipFree, no allocating library routine.  The caller still passes q and out.
 * A call needs (workgroups + batch * n_kv_heads) * group_size rows, workgroups = compute units *
 * cfg.decode_wgs_per_cu, twice that for a layer with a gate below 1; RLKV_ERR_TOO_LARGE (nothing
 * launched) beyond 16384 rows.  Every call on one GPU uses that GPU's one buffer, from any cache
 * and any stream: calls that overlap in time on one GPU race (calls on one stream do not overlap).
 * Nothing in the buffer has to start at zero: every row a call reads it has written before. */
rlkv_status_t rlkv_decode_attention_noalloc(rlkv_cache_t* cache, int32_t layer, const void* q /* device */,
                                            void* out /* device */, float softmax_scale, void* stream);

/* Continuous batching: which sequence slots take part in the calls that follow.  A serving
 * loop re-admits finished slots (Sec. 4.3: the memory compressed heads free admits more
 * concurrent requests): rlkv_cache_reset(seq) empties a slot, rlkv_append_ragged prefills
 * the newcomer, and this call switches slots on and off between steps.
 *   active : host [batch] of 0 / 1, copied; NULL = all slots active (the initial state).
 * An inactive slot is skipped by rlkv_append (uniform), rlkv_append_decode and
 * rlkv_decode_attention: nothing is appended to it, no attention is computed for it, and
 * its rows of `out` are left untouched.  rlkv_append_ragged states its counts explicitly and
 * is not gated.  Decoding with no active slot, or with an active slot that is empty, returns
 * RLKV_ERR_STATE.  Asynchronous on `stream`. */
rlkv_status_t rlkv_set_active(rlkv_cache_t* cache, const uint8_t* active /* host */, void* stream);

/* Mixed attention with gating adapters (Sec. 3.1, Eq. 1), the form used while the gates are
 * still continuous (rollouts of the head-identification phase, Sec. 3.2 / App. B): a FULL
 * head with gate g in [0, 1] returns, for each of its query heads,
 *     g * out_full_attn + (1 - g) * out_local_attn,
 * out_local_attn being attention over the first `sink` and the last `recent` positions of the
 * same store.  Applies to every later rlkv_decode_attention / rlkv_append_decode call.
 *   gates : host [n_layers * n_kv_heads], copied; NULL = all gates 1 (the initial state, plain
 *           full attention).  Entries of compressed heads are ignored: such a head holds
 *           only its local cache (the g = 0 case after discretisation, Sec. 3.3).
 * RLKV_ERR_INVALID_ARG if a gate lies outside [0, 1].  Asynchronous on `stream`. */
rlkv_status_t rlkv_set_gates(rlkv_cache_t* cache, const float* gates /* host */, void* stream);

/* One whole decode step of a layer in one call: rlkv_append of a single token per
 * sequence (k, v: device [batch][n_kv_heads][1][head_dim]) followed by
 * rlkv_decode_attention, with the same results and error codes as the two calls.  With
 * the MFMA kernel the append runs inside the attention kernel (the wavefront that reads
 * the tile holding a new slot also writes the row), which removes a launch per layer -
 * the counterpart of the dual-dispatch overhead the paper names in Sec. 4.3. */
rlkv_status_t rlkv_append_decode(rlkv_cache_t* cache, int32_t layer, const void* k /* device */,
                                 const void* v /* device */, const void* q /* device */,
                                 void* out /* device */, float softmax_scale, void* stream);

/* rlkv_append_decode in two halves, so that the device half can be recorded into a HIP graph and
 * replayed (Sec. 4.3 names the per-layer dispatch overhead of the two pools as what separates the
 * measured from the theoretical speedup; a recorded step removes the per-launch host work as well).
 *
 * rlkv_append_decode_prepare - the host half of one step of `layer`: capacity check (RLKV_ERR_CAPACITY,
 *   nothing changed), pages of a paged cache, a fresh work list when the current one has served its
 *   32 tokens (one small host-to-device copy on `stream`), and the host mirrors take the step.  Never
 *   recorded: RLKV_ERR_STATE if `stream` is capturing.
 * rlkv_append_decode_launch - the device half: the fused attention kernel and the merge kernel (with the
 *   vector-ALU kernel: the append kernel, the attention kernel and the merge kernel), nothing else; every
 *   argument is the same at every step (the kernels find the lengths on the device), so a recorded launch
 *   can be replayed.  On a stream that is not capturing it needs a prepared step
 *   (RLKV_ERR_STATE otherwise) and performs it.  On a capturing stream it only records.
 *
 * Replaying: call rlkv_append_decode_prepare for every recorded layer, on the stream the graph will be
 * launched on, before each launch of the graph; exactly one execution of the layer's launch - direct
 * or replayed - must follow each prepare before anything else is called for that layer.  A recorded
 * launch keeps the kernel variant of the moment it was recorded: record again after rlkv_set_gates
 * changes whether the layer blends.  k, v, q, out are read / written at the recorded addresses. */
rlkv_status_t rlkv_append_decode_prepare(rlkv_cache_t* cache, int32_t layer, void* stream);
rlkv_status_t rlkv_append_decode_launch(rlkv_cache_t* cache, int32_t layer, const void* k /* device */,
                                        const void* v /* device */, const void* q /* device */,
                                        void* out /* device */, float softmax_scale, void* stream);

/* Work lists planned and sent to the device since the cache was created (all layers).  A list serves
 * 32 tokens of growth of its layer; the layers' turns are spread over those 32 steps, so a decode
 * step of an L-layer cache plans about L / 32 lists.  -1 for a null handle. */
int64_t rlkv_worklists_built(const rlkv_cache_t* cache);

/* Prefill, or one chunk of a chunked prefill, of `layer` with mixed heads (Sec. 3.1: the causal
 * mask gives full KV cache access, the local mask - constant initial sink tokens plus recent
 * tokens - local access; App. B: prefilling applies the masks).  Sequence b brings n_tokens[b] new
 * positions; the query at chunk index c sits at position i = n + c (n = positions cached so far)
 * and attends over positions j <= i for a full head, and over j <= i with (j < sink or
 * i - j < recent) for a compressed head, the chunk's own keys included.  The chunk is then
 * appended exactly as by rlkv_append_ragged (so a compressed head keeps its sinks and the last
 * `recent` positions).
 *   q, out   : device, [batch][n_q_heads][stride_tokens][head_dim]; rows c >= n_tokens[b] are
 *              neither read nor written
 *   k, v     : device, [batch][n_kv_heads][stride_tokens][head_dim]
 *   n_tokens : host, [batch], 0 <= n_tokens[b] <= stride_tokens; copied before the call returns
 * stride_tokens <= cfg.prefill_tokens.  Scores, softmax and accumulation are fp32.  For most of
 * a full head's keys the softmax weights and V enter the weights x V product as fp16: V
 * magnitudes in [2^-14, 65536) are carried exactly, smaller ones with an absolute error of at
 * most 2^-24.  Once a larger one (or Inf / NaN) has been appended to a layer, by any call, the
 * prefill of that layer takes V as bf16 (slower), until rlkv_cache_reset empties the whole cache.
 * When the call has few long workgroups to hand out (one or two sequences, few full heads, a
 * long cached context), the keys before each workgroup's first query are divided among up to 8
 * workgroups whose shares, kept in scratch memory of the arena, a second kernel merges; how a
 * call is divided depends on its shapes and lengths only, so equal calls give equal bits.
 * (Tuning: cfg.prefill_min_share_tiles, cfg.prefill_two_group_only.)
 * A full head with a gate g < 1 (rlkv_set_gates; Eq. 1, the prompt of a rollout) returns
 * g * attention under the causal mask + (1 - g) * attention under the local mask.
 * RLKV_ERR_STATE if the cache was created with prefill_tokens = 0; RLKV_ERR_CAPACITY (nothing
 * computed, nothing written) as rlkv_append_ragged. */
rlkv_status_t rlkv_prefill_attention(rlkv_cache_t* cache, int32_t layer, const void* q /* device */,
                                     const void* k /* device */, const void* v /* device */,
                                     const int32_t* n_tokens /* host */, int32_t stride_tokens,
                                     void* out /* device */, float softmax_scale, void* stream);

/* Measurement aid.  After rlkv_profile_enable, every rlkv_decode_attention / rlkv_append_decode /
 * rlkv_prefill_attention call on this cache attaches a pair of HIP events to its attention kernel
 * (the kernel that streams the K/V stores); they receive that kernel's own begin and end
 * timestamps, for up to max_records calls.
 * rlkv_profile_collect waits for the handle's last stream, writes the kernel durations in milliseconds
 * (one per recorded call, in call order) to kernel_ms, sets *n_records, and disables
 * recording again.  Off by default. */
rlkv_status_t rlkv_profile_enable(rlkv_cache_t* cache, int32_t max_records);
rlkv_status_t rlkv_profile_collect(rlkv_cache_t* cache, float* kernel_ms /* host [max_records] */,
                                   int32_t* n_records /* host */);

/* Introspection for bit-exact tests.  Both wait for the stream the handle was last used on,
 * then copy to host memory. */
rlkv_status_t rlkv_get_lengths(rlkv_cache_t* cache, int32_t layer, int32_t* out /* host [batch] */);
/* Position held by every slot of a compressed head's store, -1 = empty.
 * RLKV_ERR_INVALID_ARG if (layer, kv_head) is a full head. */
rlkv_status_t rlkv_get_slot_positions(rlkv_cache_t* cache, int32_t layer, int32_t kv_head,
                                      int32_t seq, int32_t* out /* host [sink + recent] */);

/* Bytes of K/V stores resident for this cache (constant per compressed head: Sec. 4.3). */
size_t rlkv_resident_bytes(const rlkv_cache_t* cache);

/* Paged caches: pages still on the free list (each stands for one page in every full head's
 * pool); -1 for a contiguous cache.  A scheduler admits a request when this covers its prompt. */
int64_t rlkv_pool_pages_free(const rlkv_cache_t* cache);

/* Measurement aid for paged caches: permutes the free list with a seeded shuffle, so that the
 * pages handed out next are scattered over the pool the way they are after long service.
 * RLKV_ERR_STATE for a contiguous cache. */
rlkv_status_t rlkv_pool_shuffle(rlkv_cache_t* cache, uint64_t seed);

/* How rlkv_prefill_attention runs one chunk of a layer that does not blend (no gate below 1), exposed
 * for tests and tools (it touches no device).  The attention kernel has a form with two 16-column groups
 * of queries per wavefront and one with a single group (half the chunk positions per workgroup, less
 * efficient; the form that blends).  Long workgroups are those of full heads: 256 / group_size chunk
 * positions each.  When twice their number still fits n_compute_units, each one's unmasked tiles are
 * divided among as many workgroups (2..8) as fit one round over the compute units, provided the
 * shortest cached context leaves every share min_share_tiles 32-key tiles and the shares fit the
 * scratch slots; when none does and allow_narrow is set, the single-group form is used.
 *   n_tokens, cached : host [batch], chunk length and positions already cached per sequence
 *   narrow, n_split  : host, out: 1 = single-group form; shares per full-head workgroup (1 = undivided)
 * Returns 0, or -1 on an invalid argument. */
int32_t rlkv_plan_prefill_form(int32_t n_compute_units, int32_t n_q_heads, int32_t n_kv_heads, int32_t n_full_heads,
                               int32_t batch, const int32_t* n_tokens /* host */, const int32_t* cached /* host */,
                               int32_t min_share_tiles, int32_t allow_narrow, int32_t* narrow /* host */,
                               int32_t* n_split /* host */);

/* Which grid rows of a prefill chunk's attention launch are kept on one XCD each, exposed for tests and
 * tools (it touches no device).  A grid row is one (sequence, KV head); all its workgroups read the same
 * K/V tiles, and every XCD has an L2 of its own, so a row dealt whole to one XCD is fetched from memory once.
 * The rows of full heads of sequences that have a chunk come first ("heavy" rows, sequences ordered by
 * cached + chunk length, longest first), and of those the leading groups of 8 rows whose work differs by less
 * than 15 % within the group are dealt one row per XCD; the heavy rows after them are dealt workgroup by
 * workgroup, so that ragged chunks leave no XCD idle.  (Rows of compressed heads are light and always dealt
 * by rows.)  Work of a row: chunk tokens x (cached + chunk / 2 + 600).
 *   n_tokens, cached : host [batch], chunk length and positions already cached per sequence
 *   dealt_rows       : host, out: leading heavy rows dealt one row per XCD (a multiple of 8)
 *   heavy_rows       : host, out: rows of full heads of sequences with a chunk
 * Returns 0, or -1 on an invalid argument. */
int32_t rlkv_plan_prefill_rows(int32_t n_full_heads, int32_t batch, const int32_t* n_tokens /* host */,
                               const int32_t* cached /* host */, int32_t* dealt_rows /* host */,
                               int32_t* heavy_rows /* host */);

/* The (x, y) block of a prefill attention launch that the workgroup with linear index
 * blockIdx.x + grid_x * blockIdx.y works on, as the kernel computes it from the two counts of
 * rlkv_plan_prefill_rows; exposed for tests (it touches no device).  The hardware deals workgroups to the 8
 * XCDs in turn by that index; the map is a bijection of the grid under which every dealt row, and every whole
 * group of 8 light rows, is served by one XCD.  Returns 0, or -1 on an invalid argument. */
int32_t rlkv_plan_prefill_block(int32_t linear_index, int32_t grid_x, int32_t grid_y, int32_t dealt_rows,
                                int32_t heavy_rows, int32_t* block_x /* host */, int32_t* block_y /* host */);

/* The host-side plan of the split-K work list, exposed for tests and tools (it touches no device).
 * The scheduling units of all pairs are laid end to end - per pair one unit that marks its start,
 * then one unit per round of four 32-slot tiles - and cut into one contiguous share per workgroup;
 * a share costs 2 per round plus 3 per pair that starts in it, and the plan is the in-order
 * greedy deal at the smallest capacity that fits n_workgroups (Sec. 4.3: a compressed head costs
 * its sink + recent tokens, so both head types share one list and tiny heads idle nobody).
 *   rounds       : host [n_pairs], rounds of tiles per pair, 0 = the pair takes no part
 *   wg_begin     : host [n_workgroups + 1], out: share w = units [wg_begin[w], wg_begin[w + 1])
 *   seg_first,
 *   seg_count    : host [n_pairs], out: the consecutive workgroups that hold units of the pair
 * Returns the number of workgroups used, or -1 on an invalid argument. */
int32_t rlkv_plan_shares(const int32_t* rounds /* host */, int32_t n_pairs, int32_t n_workgroups,
                         int32_t* wg_begin /* host */, int32_t* seg_first /* host */,
                         int32_t* seg_count /* host */);

/* Measurement aid, independent of any cache: one plain streaming read of `bytes` (rounded down to
 * whole 16 KiB blocks) of `buf` with 128-bit non-temporal loads and no arithmetic, launched with
 * `workgroups` workgroups of 256 threads on `stream` of the current device.  Timed by the caller,
 * it gives the read bandwidth a kernel can reach on this machine - a measured ceiling beside the
 * nominal HBM peak.
 *   buf  : device, at least `bytes` long;  sink : device, 4 bytes the kernel may write. */
rlkv_status_t rlkv_probe_stream_read(const void* buf /* device */, size_t bytes, void* sink /* device */,
                                     int32_t workgroups, void* stream);

/* The kernel actually selected (resolves RLKV_KERNEL_AUTO). */
int32_t rlkv_cache_kernel(const rlkv_cache_t* cache);

const char* rlkv_status_string(rlkv_status_t status);

#ifdef __cplusplus
}
#endif
#endif /* RLKV_H */
