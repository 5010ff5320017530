/*
 * ifx -- block-causal attention against a per-layer KV cache, and the cache
 * commit, for the semi-autoregressive (block-diffusion) decode loop of the
 * Inferix paper, as a C-ABI library for one MI355X (gfx950).
 *
 * The loop (paper, Introduction, framework paragraph): a block of video tokens
 * is denoised over several steps; at each step the block's attention reads a
 * global KV cache holding the blocks generated before it; when the block is
 * done, its K/V are added to the cache.  Inside the block attention is
 * bidirectional, across blocks it is causal (abstract: diffusion within each
 * block, conditioning on previous ones).  The cache is managed block-wise with
 * a sliding window (KV Management section): when full, committing a block
 * evicts the oldest whole block.
 *
 * Conventions for every call below
 *  - Pointers named q, k_blk, v_blk, out, k_out, v_out are DEVICE pointers,
 *    16-byte aligned, owned by the caller, contiguous [block_tokens, heads,
 *    head_dim] (token-major), element type = the cache's dtype (bf16 for IFX_FP8_E4M3).  The library
 *    keeps none of them after the call's work is enqueued.
 *  - `stream` is a hipStream_t passed as void*; NULL is the default stream.
 *    Work is enqueued, never waited for, unless a call says otherwise.  Host
 *    metadata (which slot holds which block) changes at call time, data moves
 *    in stream order: issue all calls on one cache on one stream, or order
 *    them yourself.  Two calls on one cache running at once on one GPU race.
 *  - Return value: IFX_OK or a negative IFX_ERR_* code; a failed call leaves
 *    the cache unchanged (one exception: with profiling on, a commit whose
 *    closing timing event cannot be recorded has taken place and still
 *    reports IFX_ERR_HIP).  ifx_last_error() gives a thread-local message.
 *    Nothing throws or aborts across this boundary.
 *  - The attention calls and ifx_attention_merge do nothing but enqueue
 *    kernels (profiling takes no sample on a capturing stream), so they may
 *    be recorded into a HIP graph and replayed while the cache's contents
 *    stay as they were at capture.
 *    The commits, reset and read depend on host metadata of the moment of the
 *    call and belong outside a graph.
 *  - There is no CPU fallback: without a usable HIP device every call that
 *    needs one fails with IFX_ERR_HIP.
 */
#ifndef IFX_H
#define IFX_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define IFX_F32 0  /* fp32 storage, fp32 arithmetic                                  */
#define IFX_BF16 1 /* bf16 storage, bf16 MFMA contractions, fp32 softmax + accumulate */
/*
 * A compressed cache (KV Management section: the KV store may be compressed;
 * Challenges section: KV-cache quantisation): the caller's tensors (q, k_blk,
 * v_blk, out, k_out, v_out) are bf16 as with IFX_BF16, but a committed block is
 * kept as OCP FP8 E4M3 codes (1 sign, 4 exponent, 3 mantissa bits, bias 7, no
 * infinities, largest magnitude 448), one byte per element, no scale factors:
 * half the memory of a bf16 cache.  ifx_kv_cache_commit rounds every element
 * to the nearest code (ties to the even code; magnitudes beyond 448 and
 * infinities become +-448; NaN stays NaN).  Attention reads the rounded
 * values exactly (every E4M3 value is a bf16 value) with the arithmetic of
 * IFX_BF16; the current block takes part unrounded.  ifx_kv_cache_read gives
 * the rounded values as bf16.  The paper names neither format nor rule; these
 * are this library's.
 */
#define IFX_FP8_E4M3 2

#define IFX_OK 0
#define IFX_ERR_INVALID_ARG (-1)
#define IFX_ERR_NOT_CONFIGURED (-2)
#define IFX_ERR_OOM (-3)
#define IFX_ERR_HIP (-4)
#define IFX_ERR_UNSUPPORTED (-5)

typedef struct ifx_kv_cache ifx_kv_cache; /* opaque, library-owned */
typedef void *ifx_stream_t;               /* a hipStream_t */

/* ---- the three calls of the hot path ------------------------------------ */

/*
 * A cache for `layers` attention layers of `heads` x `head_dim`, holding up to
 * `capacity_tokens` committed tokens per layer (the current block is extra).
 * Host-side only; device memory is taken by ifx_kv_cache_configure.
 * Returns NULL on invalid sizes or host allocation failure.
 * (KV Management section: unified interface over block-wise KV memory.)
 */
ifx_kv_cache *ifx_kv_cache_create(int layers, int heads, int head_dim, int64_t capacity_tokens);

/*
 * Attention of the current block against the layer's cache plus the block
 * itself (Introduction, framework paragraph; abstract):
 *
 *   out[i,h,:] = sum_j softmax_j( scale * <q[i,h,:], k[j,h,:]> ) * v[j,h,:]
 *
 * where j runs over every resident cached token of `layer` and every token of
 * (k_blk, v_blk).  No other mask exists on this path.  One kernel launch:
 * q, k_blk, v_blk and the resident blocks are read where they lie, out
 * [block_tokens, heads, head_dim] is written, nothing else is (so calls of
 * this function on one cache may run concurrently).
 * bf16: head_dim 128 only.  Non-finite values (NaN, +-inf) in q, k_blk, v_blk
 * or in committed blocks are not detected: the call still returns IFX_OK, never
 * faults and writes all of `out`, but the outputs of every (query, head) whose
 * key set or query holds such a value are unspecified (usually NaN); other
 * heads are unaffected.  Finite inputs give the defined result as long as the
 * scaled scores stay below about 2^30 in magnitude (they are fp32 numbers);
 * key norms may be of any size, even beyond fp32's range.
 */
int ifx_block_attention(ifx_kv_cache *cache, int layer, const void *q, const void *k_blk,
                        const void *v_blk, void *out, ifx_stream_t stream);

/*
 * Add the block's K/V to the layer's cache, bit for bit (Introduction,
 * framework paragraph: the finished block's KV updates the cache).  The block
 * goes to slot (blocks committed so far) mod (capacity in blocks); once the
 * cache is full this overwrites, i.e. evicts, the oldest block (KV Management
 * section: sliding-window access).
 */
int ifx_kv_cache_commit(ifx_kv_cache *cache, int layer, const void *k_blk, const void *v_blk,
                        ifx_stream_t stream);

/*
 * ifx_kv_cache_commit for layers first_layer .. first_layer + n_layers - 1 at
 * once (Introduction, framework paragraph: when a block is finished its KV
 * updates the cache - of every layer; KV Management section: block-wise KV
 * memory).  k_blks / v_blks are HOST arrays of n_layers DEVICE pointers, entry
 * i the block of layer first_layer + i, each as ifx_kv_cache_commit takes it.
 * Every layer's block goes to that layer's own next slot; the result is what
 * n_layers single commits give, bit for bit, in one kernel launch per 64
 * layers, which is what lets the copy run at the memory's rate (a single
 * layer's block is too small for that).  The arrays are read before the call
 * returns.  If a launch fails the layers enqueued before it stay committed and
 * the call reports the error.
 */
int ifx_kv_cache_commit_layers(ifx_kv_cache *cache, int first_layer, int n_layers, const void *const *k_blks,
                               const void *const *v_blks, ifx_stream_t stream);

/* ---- split attention: partial results over chosen blocks, and their merge -- */

/* Resident blocks [first_block, first_block + block_count) in logical order, 0 = the oldest. */
typedef struct ifx_block_range {
    int64_t first_block;
    int64_t block_count;
} ifx_block_range;

/*
 * ifx_block_attention over a chosen key set: the resident blocks named by
 * `ranges` (HOST pointer, n_ranges entries, ascending, not overlapping; e.g.
 * the first block plus the last w blocks) and, unless k_blk and v_blk are both
 * NULL, the current block.  (KV Management section: range-based chunked access
 * to the cache; Parallelism section: ring attention computes attention per
 * chunk of keys and combines the partial results.)
 * out [block_tokens, heads, head_dim] is the attention output normalised over
 * that key set.  lse (DEVICE, fp32 [block_tokens, heads], may be NULL)
 * receives ln sum_j exp(scale * <q_i, k_j>) over the same keys, which is what
 * ifx_attention_merge needs to combine two such results.
 * Same as ifx_block_attention_blocks with the ranges written out block by
 * block.
 * Errors: a range that is not resident, no key selected at all.
 */
int ifx_block_attention_ranges(ifx_kv_cache *cache, int layer, const void *q, const void *k_blk, const void *v_blk,
                               const ifx_block_range *ranges, int n_ranges, void *out, float *lse,
                               ifx_stream_t stream);

/*
 * The same over a list of resident blocks: `blocks` (HOST pointer, n_blocks
 * logical block numbers, 0 = the oldest resident one, in any order, each at
 * most once) and, unless k_blk and v_blk are both NULL, the current block.
 * (KV Management section: index-based selective fetch of cached blocks - the
 * caller's policy picks the blocks, this call attends to exactly those,
 * reading them where they lie.)  The order of the list does not change the
 * result beyond the rounding of a different summation order.
 * A selection of cached blocks that is not simply "every resident block in
 * slot order" goes through a block table.  Up to IFX_MAX_LISTED_BLOCKS entries
 * travel with the kernel launch; a longer list (any length: every resident
 * block may be listed) is first written to a list the cache keeps per layer in
 * device memory, by small launches on the same stream, and the kernel works
 * through it IFX_MAX_LISTED_BLOCKS entries at a time.  Two such calls on one
 * layer that run concurrently race for that list.
 * n_blocks = -1 (blocks ignored) stands for every resident block in slot
 * order: ifx_block_attention's key set and speed, with the lse output.
 * Errors: a block that is not resident or listed twice, no key selected at all.
 */
#define IFX_MAX_LISTED_BLOCKS 63
int ifx_block_attention_blocks(ifx_kv_cache *cache, int layer, const void *q, const void *k_blk, const void *v_blk,
                               const int64_t *blocks, int n_blocks, void *out, float *lse, ifx_stream_t stream);

/*
 * ifx_block_attention_blocks for callers that cannot allocate device memory
 * or must not touch memory that something else allocated for them: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * Same arguments, same result, bit for bit.  The block list does not go to
 * the cache's own per-layer list but, whenever the selection needs a list at
 * all (any selection that is not "every resident block in slot order"), to a
 * fixed array of IFX_NOALLOC_MAX_LISTED_BLOCKS entries (16 KiB) inside the
 * library's own image, one per GPU, held until the process ends.  The call
 * allocates and frees nothing on the device.  A longer list is
 * IFX_ERR_UNSUPPORTED.  The cache's device must be the current device.  Every
 * call of this function on one GPU shares that GPU's array (whatever the
 * cache, layer or stream) and overwrites the entries it uses: calls that
 * overlap in time on one GPU race, so keep them on one stream or order them.
 */
#define IFX_NOALLOC_MAX_LISTED_BLOCKS 4096
int ifx_block_attention_blocks_noalloc(ifx_kv_cache *cache, int layer, const void *q, const void *k_blk, const void *v_blk,
                                       const int64_t *blocks, int n_blocks, void *out, float *lse, ifx_stream_t stream);

/*
 * Combine two attention results over disjoint key sets (Parallelism section:
 * partial attention per key chunk, merged by the log-sum-exp weights):
 *   out = (e^lse_a out_a + e^lse_b out_b) / (e^lse_a + e^lse_b),  lse = ln(e^lse_a + e^lse_b).
 * All pointers are DEVICE pointers; out_* are [rows, head_dim] of `dtype`
 * (IFX_F32 / IFX_BF16, 16-byte aligned), lse_* fp32 [rows], rows = tokens *
 * heads.  lse may be NULL.  out may alias out_a or out_b; lse may alias lse_a
 * or lse_b when 64 % (head_dim / 8) == 0.  A side with lse = -inf (no keys)
 * gets weight 0.  Needs no cache.
 */
int ifx_attention_merge(const void *out_a, const float *lse_a, const void *out_b, const float *lse_b, void *out,
                        float *lse, int64_t rows, int head_dim, int dtype, ifx_stream_t stream);

/* ---- set-up and inspection (the three calls carry no size, dtype or scale) - */
/*
 * The calls of this section follow from the three above rather than from a
 * passage of the paper, except where one is named: something has to fix the
 * sizes the three calls do not carry, free the cache, and let a test see what
 * a commit did.
 */

/*
 * Fix the block size, dtype (IFX_F32 / IFX_BF16) and softmax scale (0 means
 * 1/sqrt(head_dim)), and allocate the device memory on the current device.
 * capacity_tokens must be a positive multiple of block_tokens; bf16 needs
 * block_tokens % 8 == 0.  May be called once per cache.  Synchronises.
 */
int ifx_kv_cache_configure(ifx_kv_cache *cache, int64_t block_tokens, int dtype, float softmax_scale);

/* Free device and host memory.  Synchronises the device.  NULL is allowed.
 * (No passage: forced by ifx_kv_cache_create.) */
void ifx_kv_cache_destroy(ifx_kv_cache *cache);

/*
 * Forget all committed blocks of `layer` (-1: every layer): the cache clear at
 * the start of a new video or a new prompt (Video Streaming section: when the
 * prompt changes during streaming, the cross-attention cache is cleared so the
 * old prompt stops acting; the same operation, here on this cache).  Host-only:
 * the slots are simply counted as empty, no device memory is touched.
 */
int ifx_kv_cache_reset(ifx_kv_cache *cache, int layer);

/*
 * Announce, between ifx_kv_cache_create and ifx_kv_cache_configure, that the
 * capacity may later grow up to max_capacity_tokens (a multiple of the block
 * size, at least capacity_tokens).  configure then lays the cache out for that
 * many tokens but takes address space only, and maps physical memory into it
 * for capacity_tokens; ifx_kv_cache_grow maps more.  The pages of the address
 * space are the cache's pages, the device's page table is its page table
 * (KV Management section: block-wise KV memory management; abstract:
 * variable-length generation).  The attention and commit kernels are the same
 * as without a reservation.  IFX_ERR_UNSUPPORTED (from configure) on a device
 * that cannot map memory into a reserved range.
 */
int ifx_kv_cache_reserve(ifx_kv_cache *cache, int64_t max_capacity_tokens);

/*
 * Raise the capacity to new_capacity_tokens (larger than now, a multiple of
 * block_tokens) without losing anything (abstract: block diffusion generates
 * sequences of variable length; KV Management section: block-wise memory).
 * Every layer keeps its resident blocks, their order and their numbers
 * (ifx_kv_cache_committed goes on counting), and the window now evicts only
 * once the larger capacity is full.
 *  - A cache with a reservation (ifx_kv_cache_reserve): memory is mapped behind
 *    every head's resident tokens; nothing is copied, no block changes its
 *    slot, the device is not synchronised and work already enqueued on the
 *    cache is not disturbed.  The new slots are used next; after that blocks
 *    are evicted oldest first as before.  Beyond the reservation:
 *    IFX_ERR_UNSUPPORTED.
 *  - A cache without one: the blocks move to new device memory, oldest block
 *    to slot 0, so ifx_kv_cache_block_ids reports new slots.  Synchronises the
 *    device before and after; needs old and new memory side by side while it
 *    runs.
 * On failure (IFX_ERR_OOM, ...) the cache is as it was.
 */
int ifx_kv_cache_grow(ifx_kv_cache *cache, int64_t new_capacity_tokens);

/* Resident committed tokens of `layer`, or a negative error code.
 * (No passage: lets the caller size ifx_kv_cache_read's buffers.) */
int64_t ifx_kv_cache_len(const ifx_kv_cache *cache, int layer);

/* Blocks ever committed to `layer` since create/reset, or a negative error code.
 * (No passage: the count the slot rule of ifx_kv_cache_commit is stated in.) */
int64_t ifx_kv_cache_committed(const ifx_kv_cache *cache, int layer);

/*
 * ids[s] = ordinal (0-based commit count at its commit) of the block held in
 * physical slot s, or -1 if the slot is empty, for s < min(max, capacity
 * blocks).  `ids` is a HOST pointer.  Returns the number of slots written or a
 * negative error code.  (No passage: makes the eviction order of the KV
 * Management section's sliding window checkable.)
 */
int ifx_kv_cache_block_ids(const ifx_kv_cache *cache, int layer, int64_t *ids, int max);

/*
 * Dump the resident tokens of `layer` to k_out / v_out (DEVICE pointers,
 * [ifx_kv_cache_len, heads, head_dim]); logical_order != 0: oldest block first,
 * else in physical slot order.  Enqueued on `stream`.  (No passage: makes
 * "the block's KV updates the cache" checkable bit for bit.)
 */
int ifx_kv_cache_read(const ifx_kv_cache *cache, int layer, void *k_out, void *v_out,
                      int logical_order, ifx_stream_t stream);

/*
 * Timing for benchmarks (no passage; beyond the hot path's calls): with
 * enable != 0 every later attention / commit call brackets everything it
 * enqueues with a pair of HIP events on the call's stream (not while the
 * stream is being captured).  ifx_kv_cache_profile_read waits for those
 * events, returns the summed milliseconds and call counts since the last read
 * (HOST pointers, any may be NULL) and clears them.  At most 2^20 samples are
 * kept per kind between reads; later calls run untimed.
 */
int ifx_kv_cache_profile(ifx_kv_cache *cache, int enable);
int ifx_kv_cache_profile_read(ifx_kv_cache *cache, double *attention_ms, int64_t *attention_launches,
                              double *commit_ms, int64_t *commit_launches);

/* Thread-local description of the last error on this thread ("" if none).
 * (No passage.) */
const char *ifx_last_error(void);

/* ---- the slot bookkeeping on its own (host only, no device needed) ------- */

/*
 * The ring of whole-block slots one layer uses (KV Management section:
 * block-wise management, sliding window).  Exposed so the bookkeeping can be
 * exercised without a GPU; the cache uses the same code.
 */
typedef struct ifx_ring ifx_ring;
ifx_ring *ifx_ring_create(int64_t capacity_blocks);       /* NULL if capacity_blocks <= 0 */
void ifx_ring_destroy(ifx_ring *ring);
int64_t ifx_ring_commit(ifx_ring *ring);                  /* slot the next block goes to; advances */
int64_t ifx_ring_next_slot(const ifx_ring *ring);         /* same, without advancing */
int64_t ifx_ring_resident(const ifx_ring *ring);          /* resident blocks */
int64_t ifx_ring_committed(const ifx_ring *ring);         /* blocks ever committed */
int64_t ifx_ring_slot_of_logical(const ifx_ring *ring, int64_t logical); /* logical 0 = oldest; -1 if out of range */
int ifx_ring_block_ids(const ifx_ring *ring, int64_t *ids, int max);
void ifx_ring_reset(ifx_ring *ring);
/* larger only; in_place == 0: the resident blocks have been moved to slots 0, 1, ... oldest first;
 * in_place != 0: they stay in their slots and the new slots are used next */
int ifx_ring_grow(ifx_ring *ring, int64_t new_capacity_blocks, int in_place);

/* ---- launch shape of the bf16 attention kernel, for CPU tests -------------------------------
 * No passage of the paper: which workgroup takes which head and which query rows is this
 * library's own arithmetic (host integers that the kernel decodes with the same function).
 * Pure host code, no device call.
 *
 * ifx_attention_launch_grid: workgroups of one attention launch over blocks of `block_tokens`
 * tokens and `heads` heads; IFX_ERR_INVALID_ARG (< 0) if either is < 1.
 * ifx_attention_launch_item: what workgroup `workgroup` of that launch does, written to item[0..4]:
 * head, query tile of the head, first query row, wavefronts that hold rows (32 rows each, 1..8;
 * 0: the workgroup exits at once, the other entries are then meaningless), XCD it runs on
 * (workgroup % 8).  IFX_ERR_INVALID_ARG for a workgroup outside the grid or item == NULL. */
int ifx_attention_launch_grid(int block_tokens, int heads);
int ifx_attention_launch_item(int block_tokens, int heads, int workgroup, int *item);

#ifdef __cplusplus
}
#endif
#endif /* IFX_H */
