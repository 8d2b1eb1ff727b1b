/*
 * liblamps -- the GPU work of one serving iteration under LAMPS
 * (arXiv 2410.18248), for one AMD MI355X (gfx950).
 *
 * The paper's scheduler (Algorithm 1) forms a running batch every iteration
 * and executes it; requests that reach an API call leave the batch and their
 * KV cache is handled by one of three strategies (Section 1, Section 4.2):
 *   Preserve -- the cache stays in GPU memory, the request is simply not run;
 *   Discard  -- the cache is dropped (blocks freed) and recomputed later;
 *   Swap     -- the cache is offloaded to CPU memory and reloaded on return.
 * This library is what sits under "Execute runningBatch": single-query
 * attention over a paged KV cache for the running requests (Section 2.2
 * equation; paging as in Section 7's description of paged attention), the
 * block copies that implement Swap, and the block free list.
 *
 * Conventions
 *   - Plain C ABI.  Every call returns a lamps_status (0 = ok, negative =
 *     error) unless stated otherwise.  On error nothing has been enqueued and
 *     no library state has changed; lamps_last_error() describes it.  The one
 *     exception is LAMPS_ERR_HIP (the HIP runtime refused a call): work
 *     enqueued before the refusal stays enqueued, and the call hands out no
 *     ticket.
 *   - The CALLER owns all data memory: both KV pools, the workspace, q / out /
 *     block tables / context lengths / masks (device memory) and the swap
 *     buffers (pinned host memory), and both HIP streams.  The library owns
 *     only the lamps_ctx (free list, ticket table, events, a small pinned
 *     ring for block-id lists).
 *   - "device" pointers are HIP device memory of the current device; "host"
 *     pointers are ordinary process memory unless marked pinned.
 *   - Arguments that live in device memory (block_table, ctx_lens,
 *     running_mask) are NOT validated: no call synchronises with the device.
 *     The kernels keep these mistakes harmless (no access outside the pools;
 *     the affected rows are meaningless): a context length beyond
 *     max_blocks_per_req * block_size is clamped to the row by the decode
 *     kernels, and ignored (nothing read, nothing written) by the append and
 *     many-token calls, as is a context shorter than its new tokens; a block
 *     table entry outside [0, num_blocks) is not followed.
 *     lamps_validate_args checks all of this on request (it synchronises).
 *   - A context is not thread-safe; calls on it must be serialised -- with one
 *     exception: the compute-stream calls (lamps_decode_attn, lamps_kv_append,
 *     lamps_kv_append_tokens, lamps_prefill_attn) read nothing of the context that
 *     ever changes, so ONE thread may make them while ONE other thread makes
 *     all the block-management and swap calls (alloc, free, swap, ticket, wait
 *     calls).  lamps_last_error then reports the most recent failure of either;
 *     read it from the thread whose call failed, before its next call.
 *   - lamps_decode_attn, lamps_kv_append, lamps_kv_append_tokens and
 *     lamps_prefill_attn enqueue kernels on the compute stream and nothing else
 *     (no memset, no copy, no allocation, no host wait): once each has run
 *     eagerly on the device, a caller may record them into a HIP graph by stream
 *     capture and replay a whole decode iteration.  The swap calls use events
 *     and copies on the side streams and are not meant for capture.
 *
 * KV pool layout (part of the ABI, so swap images can be checked byte by byte)
 *   Keys and values live in two pools of identical size
 *       pool[num_blocks][num_layers][num_kv_heads][tile]
 *   where a tile holds the block_size x head_dim elements of `dtype` of one
 *   (block, layer, kv head), C order.  Cached position t of a request is slot
 *   t % block_size of physical block block_table[request][t / block_size].
 *   A block id names that block in every layer, keys and values.
 *   Host image of one swapped block = its key-pool bytes (all layers)
 *   followed by its value-pool bytes; images follow each other in the order
 *   of the id list.
 *   Inside a tile, element (slot s, dim d) sits at element offset
 *     LAMPS_LAYOUT_PLAIN (fp32, and bf16 with H == H_kv), keys and values:
 *         s * head_dim + d
 *     LAMPS_LAYOUT_TILED (bf16 with H > H_kv): the tile is block_size/16
 *     sub-tiles of 16 slots; with u = s / 16, t = s % 16 and sub-tile base
 *     u * 16 * head_dim,
 *         keys:    base + ((d / 8) * 16 + t) * 8 + d % 8
 *         values:  base + ((((d / 32) * 4 + t / 4) * 16 + d % 16) * 2 + (d % 32) / 16) * 4 + t % 4
 *     (16-byte runs that a wavefront loads coalesced and feeds to the matrix
 *     cores unchanged: 8 dims of one key; 4 consecutive slots of two dims of a
 *     value).  lamps_kv_layout() tells which one a configuration uses.
 */
#ifndef LAMPS_H
#define LAMPS_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lamps_ctx lamps_ctx; /* opaque, library-owned */

typedef enum { LAMPS_F32 = 0, LAMPS_BF16 = 1 } lamps_dtype;
typedef enum { LAMPS_LAYOUT_PLAIN = 0, LAMPS_LAYOUT_TILED = 1 } lamps_layout;

typedef enum {
    LAMPS_OK = 0,
    LAMPS_ERR_INVALID = -1,     /* null pointer, bad size, unsupported geometry      */
    LAMPS_ERR_RANGE = -2,       /* block id / layer / batch / ticket out of range    */
    LAMPS_ERR_DUP = -3,         /* the same block id twice in one list               */
    LAMPS_ERR_DOUBLE_FREE = -4, /* id is not allocated (free, swap of a free block)  */
    LAMPS_ERR_BUSY = -5,        /* ticket not complete yet (lamps_ticket_query)      */
    LAMPS_ERR_NOMEM = -6,       /* not enough free blocks / host allocation failed   */
    LAMPS_ERR_HIP = -7          /* a HIP runtime call failed                         */
} lamps_status;

typedef struct {
    int32_t num_layers;         /* L >= 1                                            */
    int32_t num_q_heads;        /* H, a multiple of num_kv_heads                     */
    int32_t num_kv_heads;       /* H_kv; query head h reads kv head h / (H / H_kv)   */
    int32_t head_dim;           /* d_h: bf16 {64,128,256}, f32 {32,64,128}           */
    int32_t block_size;         /* tokens per block, a power of two >= 16            */
    int32_t num_blocks;         /* physical blocks in each pool                      */
    int32_t max_blocks_per_req; /* row length of the block table                     */
    int32_t max_batch;          /* largest `batch` passed to lamps_decode_attn       */
    int32_t dtype;              /* lamps_dtype of q, the pools and out               */
    float softmax_scale;        /* 0 => 1/sqrt(head_dim), the Section 2.2 equation   */
    int32_t part_tokens;        /* 0 => balanced shares (default: every wavefront gets
                                   an equal part of all cached tokens); > 0 => fixed
                                   partitions of this many tokens, multiple of
                                   block_size                                        */
    int64_t staging_bytes;      /* device staging per swap direction; 0 => default   */
    int64_t direct_copy_bytes;  /* a block whose share of ONE pool (all layers) is at
                                   least this large is swapped as two plain copies
                                   between the pools and the host buffer: no gather
                                   kernel, no staging, nothing runs on the compute
                                   units.  0 => the default, 4 MiB (a 40-layer model:
                                   such runs are long enough for the copy engines,
                                   and the decode step next to the swap slows by 2 %
                                   instead of 8 %); < 0 => never                     */
    int32_t zero_copy_workgroups; /* > 0: lamps_swap_out / lamps_swap_in move the blocks
                                   with ONE kernel of this many workgroups (at most
                                   1024) that reads or writes the pinned host buffer
                                   over the host link itself: no staging, no
                                   hipMemcpyAsync.  The host buffer must then be
                                   mapped into the device's address space
                                   (hipHostMalloc memory is) and 16-byte aligned.
                                   0 => off (the default); not together with
                                   direct_copy_bytes.  The layer-major calls always
                                   stage.                                            */
    int32_t max_swaps_in_flight;  /* > 0: a swap call first waits (on the host, polling)
                                   until fewer than this many swaps of its direction
                                   are unfinished.  With more than about two copies
                                   per direction queued ahead while both directions are
                                   busy, the runtime's copy path has been measured to
                                   drop to a quarter of the link rate for tens of
                                   milliseconds at a time; 2 keeps it at full rate.
                                   0 => no limit (the default: the calls never block;
                                   the caller paces them)                            */
} lamps_config;

/* ---- sizes (pure functions of the config; return 0 on an invalid config) ---- */

/* M of equations (1)-(3): bytes of KV cache per token over all layers,
 * 2 * L * H_kv * d_h * sizeof(dtype) (Section 2.2.1). */
size_t lamps_kv_bytes_per_token(const lamps_config *cfg);
/* lamps_layout of the tiles of both pools for this configuration (see the
 * layout section above), or LAMPS_ERR_INVALID. */
int lamps_kv_layout(const lamps_config *cfg);
/* Bytes of one block's host image: keys + values, all layers. */
size_t lamps_block_bytes(const lamps_config *cfg);
/* Bytes the caller must allocate for EACH of the two pools. */
size_t lamps_pool_bytes(const lamps_config *cfg);
/* Bytes of device workspace the caller must allocate (256-byte aligned):
 * split partition partials and the two swap staging areas. */
size_t lamps_workspace_bytes(const lamps_config *cfg);

/* ---- life cycle ---- */

/* Creates a context over caller-owned device memory and streams (hipStream_t
 * passed as void*; NULL = the default stream).  swap_out_stream and
 * swap_in_stream may be the same stream, and may equal compute_stream (then
 * nothing overlaps).  All blocks start free; a fresh pool hands out ids
 * 0, 1, 2, ...  Makes no HIP call. */
int lamps_create(const lamps_config *cfg, void *k_pool, void *v_pool, void *workspace,
                 void *compute_stream, void *swap_out_stream, void *swap_in_stream,
                 lamps_ctx **out);
/* Waits for the library's outstanding stream work, releases events and the
 * pinned id ring.  Caller memory is not touched. */
int lamps_destroy(lamps_ctx *ctx);

/* ---- decode attention: Section 2.2 equation over the paged cache ---- */

/* One layer of one iteration, enqueued on the compute stream; returns at once.
 * For every request r < batch with running_mask[r] != 0 and every query head h:
 *   out[r][h][:] = softmax(q[r][h] . K_r^T * scale) . V_r
 * over exactly the first ctx_lens[r] cached positions of r (kv head h / G).
 * Rows of requests with running_mask[r] == 0 (Preserve / Swap / Discard while
 * the API call lasts; not in Algorithm 1's running batch) are not written and
 * their blocks are not read.  ctx_lens[r] == 0 gives a zero row.  Table
 * entries at or beyond ceil(ctx_lens[r] / block_size) are never read, nor are
 * slots at or beyond ctx_lens[r].  Accumulation is fp32; bf16 output is
 * rounded to nearest even.  Results are bit-reproducible for fixed arguments
 * and do not depend on which physical blocks hold the data.
 *   q, out        device, [batch][H][d_h] dtype
 *   block_table   device, int32 [batch][max_blocks_per_req]
 *   ctx_lens      device, int32 [batch], each <= max_blocks_per_req*block_size
 *   running_mask  device, uint8 [batch]
 * Errors: INVALID (null), RANGE (layer, batch). */
int lamps_decode_attn(lamps_ctx *ctx, int32_t layer, int32_t batch, const void *q,
                      const int32_t *block_table, const int32_t *ctx_lens,
                      const uint8_t *running_mask, void *out);

/* A debug aid.  The calls above and below do not validate what lives in device
 * memory; this one does, at the price of a host synchronisation: it runs a small
 * kernel on the compute stream that reads block_table, ctx_lens and running_mask
 * (nothing else; the pools are not touched) and waits for it.  A request is bad if
 * its ctx_lens is negative or beyond max_blocks_per_req * block_size, or if it is
 * running and a block-table entry its context uses lies outside [0, num_blocks).
 * report (host, 4 ints, may be NULL): number of bad requests, the lowest bad
 * request (-1 if none), what is wrong with it (1 = length, 2 = table entry), the
 * offending value.
 * Returns LAMPS_OK if every request is good, LAMPS_ERR_RANGE if not (the text names
 * the first); errors: INVALID (null), RANGE (batch), HIP.
 * (The decode and prefill kernels do not follow a table entry outside the pool --
 * they read zeros, or the pool's last block, instead -- and clamp a length to the
 * row; the affected rows of out are then meaningless, which is what this call finds.) */
int lamps_validate_args(lamps_ctx *ctx, int32_t batch, const int32_t *block_table,
                        const int32_t *ctx_lens, const uint8_t *running_mask, int32_t *report);

/* ---- decode attention for callers that cannot allocate ---- */

/* Bytes of device memory the library's code object reserves on every GPU it is
 * loaded on for lamps_decode_attn_static (a file-scope device array; it lives
 * until the process ends). */
#define LAMPS_STATIC_SCRATCH_BYTES (33u << 20)

/* lamps_decode_attn without a context and without a workspace, for callers that
 * cannot allocate device memory: code running under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc.  Same kernels, same result,
 * bit for bit, as lamps_decode_attn on a context created from `cfg` with
 * part_tokens == 0; the split ranges' partial results and the per-share records
 * go to the library's own LAMPS_STATIC_SCRATCH_BYTES array on the current device
 * instead of a caller-provided workspace.  The call allocates nothing (no
 * hipMalloc / hipFree, no host heap) and enqueues the two kernels on
 * compute_stream (hipStream_t as void*, NULL = the default stream) of the
 * current device.
 *   cfg           host; validated as by lamps_create (staging / copy fields are ignored);
 *                 part_tokens must be 0
 *   k_pool,v_pool device, the two pools in the layout above, 16-byte aligned
 *   q, out, block_table, ctx_lens, running_mask: as for lamps_decode_attn
 * Limit: the partial slots of one launch -- two records of (heads per pass) x
 * (head_dim + 2) floats for each wavefront resident on the chip -- must fit
 * 32 MiB of the array (on an MI355X: 4.3 MB for 32 heads on 32 kv heads of 128,
 * 8.5 MB for 32 on 8, 34 MB -- too much -- for 64 on 4); a geometry beyond that
 * is refused with LAMPS_ERR_RANGE and nothing is enqueued.
 * All calls on one GPU share that GPU's array, which keeps the last call's
 * contents (nothing in it has to be cleared: every launch writes what it later
 * reads): calls that overlap on one GPU -- two streams, two threads -- race and
 * must be serialised by the caller.  The first call on a device looks the
 * array's address up and asks the occupancy of the kernel (both are kept per
 * device); make one eager call before capturing the call into a graph.
 * Errors: INVALID (null, bad cfg, part_tokens != 0, alignment), RANGE (layer,
 * batch > cfg->max_batch, geometry beyond the scratch array), HIP.  The text is
 * available from lamps_last_error(NULL) on the calling thread. */
int lamps_decode_attn_static(const lamps_config *cfg, void *compute_stream, int32_t layer,
                             int32_t batch, const void *q, const void *k_pool, const void *v_pool,
                             const int32_t *block_table, const int32_t *ctx_lens,
                             const uint8_t *running_mask, void *out);

/* ---- KV append: the cache grows by one position per iteration (Section 2.2.1) ---- */

/* One layer of one iteration, enqueued on the compute stream; returns at once.
 * For every request r < batch with running_mask[r] != 0, writes the key and
 * value vectors of the token being generated, k_new[r] and v_new[r], at cached
 * position ctx_lens[r] of layer `layer`: slot ctx_lens[r] % block_size of
 * physical block block_table[r][ctx_lens[r] / block_size], in the pools' tile
 * layout.  The caller has put an allocated block in that table entry (a new
 * one whenever ctx_lens[r] is a multiple of block_size; after
 * lamps_compute_wait_blocks if the block may still be the source of a
 * swap-out).  With advance != 0, ctx_lens[r] of the running requests is then
 * incremented on the device (pass it on the last layer of the iteration, and
 * follow with lamps_decode_attn over the grown cache, or append after
 * attention -- whether a token attends to itself is the caller's reading of
 * Section 2.2).  Requests with running_mask[r] == 0 append nothing and keep
 * their length.  A position outside the table row or a block id outside the
 * pool writes nothing (device arguments are not validated on the host).
 *   k_new, v_new  device, [batch][H_kv][d_h] dtype, 16-byte aligned
 *   block_table   device, int32 [batch][max_blocks_per_req]
 *   ctx_lens      device, int32 [batch], read and (with advance) written
 *   running_mask  device, uint8 [batch]
 * Errors: INVALID (null), RANGE (layer, batch). */
int lamps_kv_append(lamps_ctx *ctx, int32_t layer, int32_t batch, const void *k_new,
                    const void *v_new, const int32_t *block_table, int32_t *ctx_lens,
                    const uint8_t *running_mask, int32_t advance);

/* ---- several new tokens per request: Discard's recompute, prompts, API responses ---- */

/* The new tokens of request r < n_req are rows q_start[r] .. q_start[r+1]-1 of
 * the token-major arrays below and sit at the LAST positions of its context:
 * row q_start[r] + i is cached position ctx_lens[r] - n_r + i, n_r =
 * q_start[r+1] - q_start[r], with ctx_lens already counting the new tokens.
 * q_start[0] == 0 and q_start[n_req] == total_tokens (total_tokens is given on
 * the host because it sizes the launch; rows past q_start[n_req] are ignored).
 *   q_start      device, int32 [n_req + 1], non-decreasing
 *   block_table  device, int32 [n_req][max_blocks_per_req], covering ctx_lens
 *   ctx_lens     device, int32 [n_req]
 * Both calls enqueue on the compute stream and return at once.
 * Errors: INVALID (null), RANGE (layer, n_req > max_batch, negative sizes). */

/* Writes the keys and values of the new tokens into the paged cache of `layer`
 * (Section 4.2: a discarded context is recomputed into blocks the caller has
 * allocated again; after lamps_compute_wait_blocks if they may still be the
 * source of a swap-out).  k_new, v_new: device, [total_tokens][H_kv][d_h],
 * 16-byte aligned. */
int lamps_kv_append_tokens(lamps_ctx *ctx, int32_t layer, int32_t n_req, int32_t total_tokens,
                           const void *k_new, const void *v_new, const int32_t *q_start,
                           const int32_t *block_table, const int32_t *ctx_lens);
/* Attention of every new token over the cached positions up to and including
 * its own (the Section 2.2 equation per token; the new tokens' keys and values
 * must already be in the cache):
 *   out[n][h][:] = softmax(q[n][h] . K_r[0..p]^T * scale) . V_r[0..p],  p the position of row n.
 * q, out: device, [total_tokens][H][d_h] dtype, 16-byte aligned.  fp32 accumulation, bf16 output
 * rounded to nearest even, results independent of block placement.
 * max_new_tokens: an upper bound, known on the host, of the new tokens of any one
 * request (it sizes the launch; 0 = unknown, total_tokens is used; rows of a
 * request beyond a bound that is too small are left unwritten).  bf16 with at
 * most 32 query heads per kv head runs on the matrix cores (weights rounded to
 * bf16 before the second product); other geometries -- also pools whose blocks
 * lie 4 GiB or more apart -- and any geometry when max_new_tokens < 0, run one
 * wavefront per new token with fp32 weights. */
int lamps_prefill_attn(lamps_ctx *ctx, int32_t layer, int32_t n_req, int32_t total_tokens,
                       int32_t max_new_tokens, const void *q, const int32_t *q_start,
                       const int32_t *block_table, const int32_t *ctx_lens, void *out);

/* ---- Swap handling strategy (Section 1; Section 4.2) ---- */

/* Copies the n listed blocks (all layers, keys and values) into host_buf
 * (PINNED host memory, n * lamps_block_bytes bytes, alive until the ticket
 * completes) on the swap-out stream: blocks are gathered into contiguous
 * device staging, then moved by hipMemcpyAsync.  The copy is ordered after all
 * compute-stream work enqueued before this call and after earlier swap-ins
 * into the same blocks.  Large blocks (direct_copy_bytes) skip the gather: each
 * is two hipMemcpyAsync straight from the pools, same host image.  The pool is not modified and the blocks stay
 * allocated; the caller frees them afterwards with lamps_free_blocks.  The
 * library remembers the unfinished copy per block, so that a later swap-in
 * into a re-allocated block, or lamps_compute_wait_blocks, is ordered behind
 * it on the device (the delay before the memory is fully released,
 * Section 4.2).
 * block_ids is a HOST array, copied inside the call.  *ticket identifies the
 * copy.  n == 0 is allowed.
 * Errors: INVALID, RANGE, DUP, DOUBLE_FREE (a listed block is not allocated),
 * NOMEM, HIP. */
int lamps_swap_out(lamps_ctx *ctx, const int32_t *block_ids, int32_t n, void *host_buf,
                   uint64_t *ticket);
/* Mirror image: writes image i of host_buf into block block_ids[i] on the
 * swap-in stream (hipMemcpyAsync into staging, then scatter).  The listed
 * blocks must be allocated (typically just obtained from lamps_alloc_blocks;
 * they need not be the blocks the images came from).  No other block changes.
 * If host_buf overlaps the buffer of a swap-out that has not finished, the
 * copy is ordered after it on the device (and a swap-out into a buffer that
 * an unfinished swap-in still reads waits likewise), so a swap-in may be
 * enqueued right behind the swap-out that fills its buffer.  A request may run
 * again only in steps enqueued after lamps_compute_wait(ticket). */
int lamps_swap_in(lamps_ctx *ctx, const void *host_buf, const int32_t *block_ids, int32_t n,
                  uint64_t *ticket);

/* Layer-major variants of the two calls above (Section 4.2: the swap's time, the
 * term of equation (3), is what a returning request waits for; moved one layer
 * after the other, the first layers' attention can start while the rest is still
 * on its way).  The host image is laid out
 *   [layer][i][keys of block_ids[i], layer | values of block_ids[i], layer]
 * (same size as the block-major image of lamps_swap_out, NOT interchangeable
 * with it: an image written by lamps_swap_out_layered is read back only by
 * lamps_swap_in_layered, with the same n).  The copy proceeds in steps of one or
 * more whole layers (several when a layer of the list is small, so that no step
 * moves much less than 8 MiB); lamps_compute_wait_layer orders the compute stream
 * behind the step that holds a given layer.  Everything else -- ordering, guards,
 * errors, ticket calls -- is as for lamps_swap_out / lamps_swap_in. */
int lamps_swap_out_layered(lamps_ctx *ctx, const int32_t *block_ids, int32_t n, void *host_buf,
                           uint64_t *ticket);
int lamps_swap_in_layered(lamps_ctx *ctx, const void *host_buf, const int32_t *block_ids, int32_t n,
                          uint64_t *ticket);
/* Makes the compute stream wait (on the device) until layer `layer` of the
 * ticket's copy has landed.  For a ticket of the block-major calls this is
 * lamps_compute_wait.  Errors: INVALID, RANGE (unknown ticket, layer), HIP. */
int lamps_compute_wait_layer(lamps_ctx *ctx, uint64_t ticket, int32_t layer);

/* By default every swap call orders its copy behind ALL compute-stream work enqueued
 * before the call (it cannot know which of that work wrote, or still reads, the
 * listed blocks).  A serving loop that enqueues one iteration at a time pays
 * nothing for that; a caller that enqueues decode steps far ahead would make every
 * later swap wait for all of them, although the blocks of a request that sits in an
 * API call (Section 4.2: not in the running batch) are touched by none.  Such a
 * caller switches the automatic ordering off (enabled == 0) and states the ordering
 * itself, where it is needed, with lamps_swap_wait_compute: both swap streams then
 * wait for the compute-stream work enqueued so far.  Ordering between the two swap
 * directions (guards per block, host-buffer overlap) is not affected.
 * Errors: INVALID, HIP. */
int lamps_set_swap_fence(lamps_ctx *ctx, int32_t enabled);
int lamps_swap_wait_compute(lamps_ctx *ctx);

/* LAMPS_OK if the ticket's copy has finished, LAMPS_ERR_BUSY if not. */
int lamps_ticket_query(lamps_ctx *ctx, uint64_t ticket);
/* Blocks the calling host thread until the ticket's copy has finished. */
int lamps_ticket_wait(lamps_ctx *ctx, uint64_t ticket);
/* Makes the compute stream wait (on the device) for the ticket's copy. */
int lamps_compute_wait(lamps_ctx *ctx, uint64_t ticket);
/* Makes the compute stream wait (on the device) for every unfinished swap-out
 * or swap-in that touches one of the n listed (allocated) blocks: the release
 * of a swapped-out block is complete only when its copy is (Section 4.2), and
 * compute-stream work that overwrites such a block must come after it.
 * Errors: INVALID, RANGE, DUP, DOUBLE_FREE, HIP. */
int lamps_compute_wait_blocks(lamps_ctx *ctx, const int32_t *block_ids, int32_t n);

/* ---- block free list (Discard; and the release half of Swap) ---- */

/* Pops n ids (LIFO: the most recently freed id first; a fresh pool yields
 * 0, 1, 2, ...).  A popped block may still be the source of a swap-out that has
 * not finished: lamps_swap_in into it waits for that copy by itself; a caller
 * that will write it from the compute stream (recompute after Discard, KV
 * append) calls lamps_compute_wait_blocks first.  Makes no HIP call.
 * Errors: INVALID, NOMEM (fewer than n free; nothing is popped). */
int lamps_alloc_blocks(lamps_ctx *ctx, int32_t n, int32_t *block_ids_out);
/* Pushes the listed ids, in the order given; their contents become undefined.
 * Errors: INVALID, RANGE, DUP, DOUBLE_FREE; on error nothing is freed. */
int lamps_free_blocks(lamps_ctx *ctx, const int32_t *block_ids, int32_t n);
/* Number of free blocks, or a negative status. */
int lamps_num_free(lamps_ctx *ctx);

/* Text of the last error on this context ("" if none).  With ctx == NULL,
 * the last error of a failed lamps_create or lamps_decode_attn_static on this
 * thread. */
const char *lamps_last_error(lamps_ctx *ctx);

#ifdef __cplusplus
}
#endif
#endif /* LAMPS_H */
