/*
 * mixattn.h - C ABI of the MixAttention KV-cache attention library for MI355X (gfx950).
 *
 * The library runs the inference-time attention of a layer stack that mixes
 * standard (full, causal) attention layers with sliding-window layers, where
 * groups of layers read one KV cache written by the first layer of the group
 * (arXiv 2409.15012, Section 3: "Sliding Window Attention Layers", "Standard
 * Attention Layers", "KV cache reuse"; Section 1 for why the KV cache is the
 * cost of long-context decoding).
 *
 * Conventions
 *  - Every function returns MIXATTN_OK (0) or a negative mixattn_status.  Nothing
 *    throws or aborts; on error no output buffer is written and no length changes.
 *  - "device" pointers are HIP device memory owned by the caller (for example a
 *    torch tensor's data_ptr()); "host" pointers are ordinary process memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Every
 *    call that takes a stream only enqueues work on it; calls on one layout must
 *    be issued on one stream (or be ordered by the caller), in layer order.
 *  - One layout is used by one host thread at a time, with the device that was current when it was created
 *    still current.
 *  - The layout owns its caches and scratch; they are allocated in
 *    mixattn_create_layout and freed in mixattn_destroy_layout.  The one exception is
 *    the staging area of prompt chunks (MFMA path), which mixattn_reserve_prefill sizes
 *    once (and mixattn_release_prefill gives back); a mixattn_prefill* call that finds it too small grows it (this synchronises
 *    the device and allocates) before it changes anything else.  No other hot call
 *    allocates or synchronises.
 *  - Sequence lengths live on the device, at addresses that never change, and are
 *    mirrored on the host without any device-to-host copy: every append advances every
 *    sequence by exactly one.  A decode step can therefore be captured into a HIP graph
 *    and replayed (mixattn_reserve_steps, mixattn_account_replays).
 *
 * Tensor layouts (row-major, contiguous, element type = config.kv_dtype unless noted)
 *  decode   q   [batch, n_q_heads, head_dim]
 *           out [batch, n_q_heads, head_dim]            (config.out_dtype)
 *  append   k,v [batch, n_kv_heads, head_dim]
 *  prefill  q   [batch, seq, n_q_heads, head_dim]
 *           k,v [batch, seq, n_kv_heads, head_dim]
 *           out [batch, seq, n_q_heads, head_dim]       (config.out_dtype)
 *  load_kv  k,v [sum(seq_lens), n_kv_heads, head_dim]   sequences back to back
 *
 * Query head j reads KV head j / (n_q_heads / n_kv_heads) (grouped-query attention,
 * Section 3, last paragraph).
 *
 * The physical arrangement of a cache in device memory is private to the library
 * (bf16 caches with head_dim 128 are stored in MFMA-operand tile order); the
 * contract for cache contents is mixattn_read_cache, which returns the row a
 * logical slot holds, and mixattn_slot_of / mixattn_slot_for for slot arithmetic.
 */
#ifndef MIXATTN_H
#define MIXATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct mixattn_layout mixattn_layout; /* opaque */

typedef enum { MIXATTN_FULL = 0, MIXATTN_SLIDING = 1 } mixattn_kind;
typedef enum { MIXATTN_F32 = 0, MIXATTN_BF16 = 1 } mixattn_dtype;

typedef enum {
  MIXATTN_OK = 0,
  MIXATTN_ERR_NULL = -1,       /* a required pointer is NULL */
  MIXATTN_ERR_LAYOUT = -2,     /* invalid descriptor: bad kind, window < 1, a reader that is neither like its
                                  writer nor a sliding reader of a full cache, heads not divisible, unsupported
                                  head_dim or dtype, batch < 1, batch or n_q_heads above 65535 */
  MIXATTN_ERR_LAYER = -3,      /* layer / cache / sequence / head / slot index out of range */
  MIXATTN_ERR_NOT_WRITER = -4, /* append, load or k/v commit on a layer that only reads a shared cache */
  MIXATTN_ERR_CAPACITY = -5,   /* a full cache would exceed capacity[b] */
  MIXATTN_ERR_ORDER = -6,      /* decode on an empty cache; load on a non-empty cache; reader prefill before its
                                  writer's, or of a ring past the first chunk without the staged copy; bad
                                  seq_len */
  MIXATTN_ERR_ALLOC = -7,      /* device or host allocation failed */
  MIXATTN_ERR_HIP = -8,        /* a HIP runtime call failed (see mixattn_last_hip_error) */
  MIXATTN_ERR_PARAM = -9,      /* unknown tuning parameter or value out of range */
  MIXATTN_ERR_SCRATCH = -10    /* mixattn_decode_noalloc: the call needs more split-K scratch than the static area holds */
} mixattn_status;

/* One layer (Section 3): its attention kind, its window (tokens, >= 1, SLIDING only; the query attends the
   last `window` keys including its own token), and the id of the KV cache it reads.  The lowest-index layer
   using a cache id is that cache's writer; later layers with the same id read it and store nothing.  Cache ids
   are arbitrary non-negative integers; sharers need not be consecutive layers (Section 5.1).  A reader must have
   its writer's kind and window, with one exception: a SLIDING layer may read a FULL layer's cache, in which case
   it attends the last `window` positions of that cache (nothing extra is stored). */
typedef struct {
  int32_t kind;     /* mixattn_kind */
  int32_t window;   /* SLIDING: window size in tokens; FULL: ignored */
  int32_t cache_id; /* >= 0 */
} mixattn_layer_desc;

typedef struct {
  int32_t n_layers;
  const mixattn_layer_desc* layers; /* host, [n_layers], borrowed for the call */
  int32_t batch;
  int32_t n_q_heads;
  int32_t n_kv_heads; /* divides n_q_heads */
  int32_t head_dim;   /* bf16: multiple of 8, <= 256 (128 takes the MFMA path when n_q_heads/n_kv_heads <= 8);
                         f32: 1..256 */
  const int32_t* capacity; /* host, [batch]: most tokens sequence b will ever hold in a FULL cache
                              (caches are packed, so capacities may differ).  May be NULL when no layer is
                              FULL.  Ring caches always hold `window` slots. */
  int32_t kv_dtype;  /* mixattn_dtype of q, k, v and the caches */
  int32_t out_dtype; /* mixattn_dtype of `out`; accumulation is fp32 either way */
  float softmax_scale; /* 0 => 1/sqrt(head_dim) */
} mixattn_config;

/* Pure host check of a descriptor (what mixattn_create_layout runs first).  Touches no device. */
int mixattn_validate_config(const mixattn_config* cfg);

/* Builds the layout: resolves cache ids to caches and writers, allocates zero-filled caches, length arrays and
   split-K scratch with hipMalloc on the current device.  *out receives the handle (untouched on error). */
int mixattn_create_layout(const mixattn_config* cfg, mixattn_layout** out);
/* The same layout with its FULL caches held in pages, as serving engines do (Section 4 measures through one): each
   FULL cache is a pool of pool_tokens / page_tokens pages of page_tokens tokens (all KV heads), shared by the
   sequences; a sequence takes a page from the pool whenever it grows into one (append, prefill, load) and gives all
   of them back on mixattn_reset / mixattn_release_sequence, so memory follows the tokens held, not the capacities.
   capacity[b] stays the most tokens sequence b may hold (it sizes the page table).  Ring caches are unaffected.
   page_tokens: a power of two, >= 32.  MFMA path only (bf16, head_dim 128, group size <= 8), LAYOUT otherwise.
   A call that needs more pages than the pool has left returns CAPACITY and changes nothing.  Results, cache
   contents (mixattn_read_cache) and every other call are the same as for a contiguous layout. */
int mixattn_create_layout_paged(const mixattn_config* cfg, int page_tokens, int64_t pool_tokens,
                                mixattn_layout** out);
int mixattn_destroy_layout(mixattn_layout* L);

/* Empties every cache (lengths to zero; cache bytes are left as they are and never read again before being
   overwritten).  Enqueued on `stream`. */
int mixattn_reset(mixattn_layout* L, void* stream);
/* Sequence b gives up its slot of the batch: every cache forgets it (a paged layout takes its pages back) and the
   slot is idle until a new request starts in it with a prompt chunk (mixattn_prefill, mixattn_prefill_varlen with
   seq_lens[b] > 0) or a bulk load.  While idle, mixattn_append_kv / mixattn_append_decode ignore its row of k, v
   and store nothing for it, every decode call writes zeros to its output rows, mixattn_seq_len reports 0, and the
   other sequences are unaffected.  (A sequence that has simply never been given a token is empty, not idle:
   appends start it, decode on it is ORDER.)  Enqueued on `stream`.  Errors: LAYER (b out of range). */
int mixattn_release_sequence(mixattn_layout* L, int b, void* stream);

/* Appends one token per sequence to the cache `layer` writes (Section 3: a sliding cache keeps the past
   `window` tokens).  k, v: device [batch, n_kv_heads, head_dim].  Token at absolute position p = n_b goes to
   slot p (FULL) or p mod window (SLIDING); n_b becomes n_b + 1.  Errors: NOT_WRITER, CAPACITY. */
int mixattn_append_kv(mixattn_layout* L, int layer, const void* k, const void* v, void* stream);

/* Decode-step attention of `layer` (Sections 1 and 3).  q: device [batch, n_q_heads, head_dim].  For sequence
   b holding n_b tokens the query sits at position n_b - 1 (its group's writer has already appended this step's
   token) and attends positions 0 .. n_b-1 (FULL) or max(0, n_b-window) .. n_b-1 (SLIDING):
   out = sum_p softmax_p(scale * q.k_p) v_p.  out: device [batch, n_q_heads, head_dim].  Errors: ORDER if any
   sequence is empty. */
int mixattn_decode(mixattn_layout* L, int layer, const void* q, void* out, void* stream);

/* mixattn_decode for callers that cannot allocate device memory or depend on memory a layout allocated for scratch:
   code under HIP graph capture that must not reference per-layout scratch, tight serving loops, harnesses that forbid
   hipMalloc.  Same arguments, same result (to rounding order) and same errors as mixattn_decode, MFMA path only
   (LAYOUT otherwise).  Split-K partial results go to a fixed 16 MiB area in the library's device image instead of the
   layout's scratch (each GPU holds its own copy until the process ends; its address is looked up when a layout is
   created on that GPU).  The call allocates nothing and frees nothing.  It is refused with SCRATCH, before anything
   is enqueued, when batch * n_q_heads * chunks * (head_dim + 2) * 4 bytes exceed the area (chunks = the split-K
   chunk count the call would use; calls that need no split use no scratch).  Every call on a GPU shares that GPU's
   area: calls that overlap on one GPU (several streams, several layouts) race; calls ordered on one stream do not.
   Nothing in the area has to be cleared between calls: a call writes every partial that it reads. */
int mixattn_decode_noalloc(mixattn_layout* L, int layer, const void* q, void* out, void* stream);

/* mixattn_append_kv followed by mixattn_decode on the same (writer) layer, as one call: same arguments, same
   result, same errors (NOT_WRITER, CAPACITY, NULL).  On the MFMA path (bf16, head_dim 128) it is a single launch:
   the decode kernel takes this step's token from k, v directly and stores it to the cache on the way. */
int mixattn_append_decode(mixattn_layout* L, int layer, const void* k, const void* v, const void* q, void* out,
                          void* stream);

/* Benchmark-side upper bound for a sharing group of sliding-window layers (Section 3, KV cache reuse): the decode
   step of `n_layers` layers that read one ring cache, served by ONE pass over the ring.  A model cannot call this
   (layer i + 1's query depends on layer i's output); it measures what sharing could save at most when the ring is
   read once per group instead of once per layer.
   layers: host array of n_layers distinct layer indices, all reading the same SLIDING cache; n_layers * group
   size (query heads per KV head) <= 16.  q, out: device [n_layers, batch, n_q_heads, head_dim], layer i of the
   array at index i; each layer's result is that of mixattn_decode for it.  k, v: both NULL (the step's token is
   already in the cache) or this step's token [batch, n_kv_heads, head_dim], appended by the same launch as in
   mixattn_append_decode; layers[0] must then be the cache's writer.  MFMA path only.
   Errors: NULL, LAYER (index out of range or repeated), LAYOUT (different caches, a full cache, too many layers,
   not the MFMA path), NOT_WRITER, ORDER (empty sequence and no token given). */
int mixattn_decode_group(mixattn_layout* L, const int32_t* layers, int n_layers, const void* k, const void* v,
                         const void* q, void* out, void* stream);

/* Prompt attention for seq_len new tokens per sequence (causal; SLIDING layers also mask keys more than window-1
   tokens back).  The tokens follow the n_b tokens the cache already holds, so a prompt may be fed in chunks: query
   row i of sequence b sits at position n_b + i and attends the cache contents and the chunk.
   Writer layer: k, v are the chunk's keys/values; they are attended over and committed to its cache (FULL: slots
   n_b .. n_b+seq_len-1; SLIDING: the ring keeps the last min(n, window) positions, each at slot p mod window) and
   every n_b grows by seq_len.  Reader layer: runs after its writer's call for the same chunk (its cache then holds
   n_b >= seq_len tokens, the last seq_len being the chunk); pass the writer's k, v again (attended over, not
   stored).  On the MFMA path (bf16, head_dim 128) a reader may instead pass k = v = NULL to reuse the tile-format
   copy of the chunk that its writer's prefill call staged (ORDER when there is none, or it was for other lengths).
   Every cache keeps that copy to itself until its next chunk, append, load or release, so its readers may come at
   any later point of the layer loop.  Passing NULL is the cheap way to run the readers of a sharing
   group, and the only way for readers of a SLIDING cache past the first chunk (the writer's commit has
   overwritten ring slots their first rows need; ORDER if k, v are passed there, and on the scalar path).  On the
   MFMA path V is staged as fp16 (values beyond +-65504 saturate).  Errors: ORDER, CAPACITY, NULL, ALLOC (only when
   the staging area has to grow, see mixattn_reserve_prefill; lengths and caches are then unchanged). */
int mixattn_prefill(mixattn_layout* L, int layer, const void* q, const void* k, const void* v, void* out,
                    int seq_len, void* stream);

/* mixattn_prefill with a chunk length of its own per sequence (a serving batch mixes prompts of many lengths;
   Section 4 measures 300 mixed requests).  seq_lens: host [batch], each >= 0, at least one > 0; a sequence with 0
   takes no part (its caches are left as they are).  q, out: device, packed by sequence
   [sum(seq_lens), n_q_heads, head_dim]; k, v: device [sum(seq_lens), n_kv_heads, head_dim] in the same order.
   Everything else as mixattn_prefill: row i of sequence b sits at position n_b + i, writers commit, readers follow
   their writer's call for the same chunk and may pass k = v = NULL (MFMA path) when the staged copy was made for
   the same cache and the same seq_lens.  Errors: ORDER (negative or all-zero seq_lens, ...), CAPACITY, NULL. */
int mixattn_prefill_varlen(mixattn_layout* L, int layer, const void* q, const void* k, const void* v, void* out,
                           const int32_t* seq_lens, void* stream);

/* Sizes the staging areas of prompt chunks for chunks of up to max_chunk_tokens tokens per sequence (MFMA path; a
   no-op otherwise): per standard cache an fp16 copy of V for capacity[b] tokens, per sliding cache K and V for
   window - 1 + max_chunk_tokens tokens.  Synchronises the device and allocates; call it once after creating the
   layout, and no later mixattn_prefill / mixattn_prefill_varlen call with chunks up to that length allocates or
   synchronises.  Errors: ORDER (max_chunk_tokens < 1), ALLOC (areas sized so far are kept). */
int mixattn_reserve_prefill(mixattn_layout* L, int max_chunk_tokens);

/* Frees every staging area (synchronises the device first).  For callers that have finished their prompts and want
   the memory back for the decode phase: the areas of standard caches are half the size of the cache itself.  A later
   prefill call sizes them again (and may then allocate); a reader's k = v = NULL call after this returns ORDER.
   mixattn_staging_bytes: device bytes the staging areas hold at present (not part of mixattn_kv_bytes_allocated). */
int mixattn_release_prefill(mixattn_layout* L);
int64_t mixattn_staging_bytes(const mixattn_layout* L);

/* Decode steps captured into a HIP graph (Section 4 measures a serving engine, which replays its decode step this
   way).  All kernel arguments of a decode step are fixed addresses and the kernels take the sequence lengths from
   device memory, so a stream capture around one step (every writer layer's mixattn_append_decode or mixattn_append_kv,
   every layer's decode) can be replayed, each replay appending one token per sequence and attending one position
   further.  The host side is told about the replays with these two calls:
   mixattn_reserve_steps: checks that every sequence can take `steps` more tokens (CAPACITY otherwise, nothing changed)
   and gives paged caches the pages for them now (their table entries are enqueued on `stream`), because a replay
   cannot reserve.  Call it before the capture with steps = 1 + the number of replays planned.
   mixattn_account_replays: the captured calls themselves count as one step on the host; after launching the graph
   r times call this with steps = r - 1 (or once per further launch with 1) so that the host lengths match the
   device again (CAPACITY if that exceeds a capacity: the replays were not reserved).  No device work.
   Launch plans (split-K chunking, balanced runs) are frozen at capture; the kernels adapt them to the lengths they
   find, so results stay correct while the sequences grow, and re-capturing every few thousand tokens restores the
   best plan.  A sequence at capacity takes no further token on the device either (its length stays). */
int mixattn_reserve_steps(mixattn_layout* L, int steps, void* stream);
int mixattn_account_replays(mixattn_layout* L, int steps);

/* Bulk fill of an empty cache without attention (sets up decode workloads and ragged batches).  Writer layers
   only.  k, v: device, packed [sum(seq_lens), n_kv_heads, head_dim]; seq_lens: host [batch], each >= 0.  n_b
   becomes seq_lens[b]; the cache ends in exactly the state seq_lens[b] appends would leave.  The host array is
   copied before the call returns. */
int mixattn_load_kv(mixattn_layout* L, int layer, const void* k, const void* v, const int32_t* seq_lens,
                    void* stream);

/* ---- introspection (host side, no device sync unless stated) ---- */
int mixattn_n_caches(const mixattn_layout* L);
/* cache index (0-based, in order of first use) and writer flag of a layer */
int mixattn_cache_of(const mixattn_layout* L, int layer, int* cache_index, int* is_writer);
/* tokens sequence b holds in a cache (host mirror) */
int mixattn_seq_len(const mixattn_layout* L, int cache_index, int b, int64_t* n);
/* slot that holds absolute position pos in this cache: pos (FULL) or pos mod window (SLIDING) */
int mixattn_slot_of(const mixattn_layout* L, int cache_index, int64_t pos, int64_t* slot);
/* the same arithmetic without a layout */
int mixattn_slot_for(int kind, int window, int64_t pos, int64_t* slot);
/* Debug read-back of one logical cache row.  Synchronises the device.  k_row, v_row: host buffers of head_dim
   elements of kv_dtype (either may be NULL).  slot must be < capacity[b] (FULL) or < window (SLIDING). */
int mixattn_read_cache(mixattn_layout* L, int cache_index, int b, int kv_head, int64_t slot, void* k_row,
                       void* v_row);
/* device lengths of one cache copied to host [batch]; synchronises (test helper) */
int mixattn_read_device_lens(mixattn_layout* L, int cache_index, int32_t* lens);
/* bytes of K+V storage resident for all caches (allocated) and bytes holding live tokens right now */
int64_t mixattn_kv_bytes_allocated(const mixattn_layout* L);
int64_t mixattn_kv_bytes_live(const mixattn_layout* L);
/* K+V bytes a decode of `layer` streams right now: sum_b min(n_b, window or inf) * 2*n_kv_heads*head_dim*elem
   (whole 32-key blocks are fetched, so a window that straddles a block boundary moves up to one block more) */
int64_t mixattn_step_read_bytes(const mixattn_layout* L, int layer);

/* ---- tuning knobs (defaults are chosen per call from the shapes) ---- */
typedef enum {
  MIXATTN_PARAM_CHUNK_KEYS = 0, /* split-K chunk length in keys for decode (multiple of 32; 0 = automatic) */
  /* 1 is not used */
  MIXATTN_PARAM_PREFILL_SIMPLE = 2, /* 1: force the scalar prefill kernel (testing) */
  MIXATTN_PARAM_PREFILL_WAVES = 3,  /* wavefronts per MFMA prefill workgroup: 4, 8, or 0 = by layer kind (8 full, 4 sliding) */
  MIXATTN_PARAM_PREFILL_HEADS = 4,  /* query heads of one KV head served by one MFMA prefill workgroup: 1, 2, 4, or
                                       0 = as many as divide the group size */
  MIXATTN_PARAM_BALANCED = 5,       /* decode over full caches: cut the blocks of all (sequence, kv head) streams,
                                       laid end to end, into equal runs, one per workgroup, instead of cutting
                                       every sequence by itself.  1 (default): when the longest sequence exceeds
                                       1.25 x the mean or the sequences have to be cut anyway; 0: never; 2: always.
                                       Ignored when CHUNK_KEYS is set and for batches above 1024. */
  MIXATTN_PARAM_TEST_FAIL_ALLOC = 6 /* testing aid, per calling thread (the layout argument is not used): n > 0 makes
                                       the n-th device allocation from now on fail with ALLOC; 0 switches it off */
} mixattn_param;
int mixattn_set_param(mixattn_layout* L, int param, int64_t value);
int mixattn_get_param(const mixattn_layout* L, int param, int64_t* value);

const char* mixattn_strerror(int status);
/* hipError_t of the most recent HIP failure seen by this thread's calls (0 if none) */
int mixattn_last_hip_error(void);
const char* mixattn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MIXATTN_H */
