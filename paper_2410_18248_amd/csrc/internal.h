// Internal launcher interface between the host half of liblamps (lamps.cpp)
// and its kernels.  Not part of the ABI.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "lamps.h"

namespace lamps {

struct DecodeArgs {
    const void *q;            // [batch][H][D]
    const void *k_pool;       // pool[block][layer][kv_head][tile of block_size * head_dim]
    const void *v_pool;
    const int32_t *block_table;  // [batch][max_blocks]
    const int32_t *ctx_lens;     // [batch]
    const uint8_t *running;      // [batch]
    float *partials;          // fixed partitions: [batch][H][max_parts][D + 2];
                              // balanced: [wave share][2][heads per pass][D + 2]
    size_t partial_capacity;  // bytes behind partials (balanced: bounds the number of shares)
    int4 *share_info;         // balanced: [shares + 1] what each share leaves to the merge kernel
    void *out;                // [batch][H][D]
    int32_t batch, max_batch, layer, num_layers, num_q_heads, num_kv_heads, head_dim;
    int32_t block_size, log2_block_size, max_blocks, num_blocks, part_tokens, max_parts;
    int32_t bf16;             // 0: fp32 storage, 1: bf16 storage
    int32_t heads_per_pass;   // query heads of a kv group that share one pass over K/V
    float scale_log2e;        // softmax scale * log2(e)
    // balanced: which share a wavefront takes (filled in by launch_decode): 0 = in launch
    // order, else gcd(head passes, shares) and the inverse of passes / gcd modulo shares / gcd
    int32_t share_gcd, share_inv;
};

// Query heads of one kv group that share a pass over K/V for this geometry
// (0 if the geometry is not supported); group / result passes re-read K/V.
int decode_heads_per_pass(int bf16, int head_dim, int group);
// Nonzero if the geometry's pools use the tiled (MFMA operand) layout.
int decode_uses_tiled_layout(int bf16, int group);

// Most wavefront shares the balanced scheme uses for a geometry (a multiple of
// 4); its partials are [shares][2][heads_per_pass][head_dim + 2] floats,
// decode_share_bytes per share.
int decode_max_shares(int heads_per_pass, int head_dim);
size_t decode_share_bytes(int heads_per_pass, int head_dim);
constexpr int kMaxDevices = 64;   // devices of one process the per-device tables cover

// Enqueues one layer of decode attention.  part_tokens == 0 selects the balanced
// scheme (then max_parts is ignored), part_tokens > 0 fixed partitions; either
// way a small merge kernel follows unless no request can be split.
hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream);
// The same dispatch; with demand != nullptr nothing is launched and *demand receives the bytes
// of partial slots a balanced launch uses when every resident wavefront takes a share.
hipError_t dispatch(const DecodeArgs &a, hipStream_t stream, size_t *demand);
// Validates cfg as lamps_create does and fills the geometry fields of *a (everything but the
// pointers, batch, layer and partial_capacity).  Returns nullptr or an error text; allocates nothing.
const char *decode_geometry(const lamps_config *cfg, DecodeArgs *a);
// Sets the text lamps_last_error(NULL) returns on this thread (fixed buffer, no allocation).
void set_thread_error(const char *text);

struct AppendArgs {
    const void *k_new, *v_new;   // [batch][H_kv][D]
    void *k_pool, *v_pool;
    const int32_t *block_table;  // [batch][max_blocks]
    int32_t *ctx_lens;           // [batch]; incremented for running requests if advance
    const uint8_t *running;      // [batch] (decode form)
    const int32_t *q_start;      // [batch + 1] (token form): first new-token row of each request
    int32_t batch, layer, num_layers, num_kv_heads, head_dim, block_size, log2_block_size;
    int32_t max_blocks, num_blocks, bf16, advance;
};

// Enqueues the append of one new position per running request in one layer.
hipError_t launch_kv_append(const AppendArgs &a, int tiled, hipStream_t stream);
// Enqueues the append of total_tokens new tokens, q_start[r + 1] - q_start[r] of them at the end
// of request r's context.
hipError_t launch_kv_append_tokens(const AppendArgs &a, int total_tokens, int tiled, hipStream_t stream);

struct PrefillArgs {
    DecodeArgs d;                // q and out are [total_tokens][H][D]; batch = number of requests
    const int32_t *q_start;      // [batch + 1]
    int32_t total_tokens;
    int32_t max_new_tokens;      // upper bound of q_start[r + 1] - q_start[r]
    int32_t force_rows;          // use the one-wavefront-per-token kernel whatever the geometry
};
// Enqueues attention for the new tokens of every request over its paged cache, each token over
// the positions up to and including its own.
hipError_t launch_prefill(const PrefillArgs &a, hipStream_t stream);

// Checks the device-resident arguments of a decode call: for every request r < batch, whether
// ctx_lens[r] is negative or beyond the block-table row, and, for running requests, whether any
// block-table entry its context uses lies outside [0, num_blocks).  result (device, 4 + 2 * batch
// ints): [0] = number of bad requests, [1] = the lowest bad request index (or -1), [2] = what was
// wrong with it (1 = length, 2 = table entry), [3] = the offending value; the rest is scratch.
// Reads nothing but the three arrays.
hipError_t launch_validate(const int32_t *block_table, const int32_t *ctx_lens, const uint8_t *running,
                           int32_t batch, int32_t max_blocks, int32_t block_size, int32_t num_blocks,
                           int32_t *result, hipStream_t stream);

// Gather: staging image i (key bytes then value bytes of block ids[i]) <- pools.
// Scatter: the reverse.  `half_bytes` = bytes of one block in one pool, a
// multiple of 16.  `ids` must be readable by the device.
hipError_t launch_gather(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                         size_t half_bytes, void *staging, hipStream_t stream);
hipError_t launch_scatter(void *k_pool, void *v_pool, const int32_t *ids, int32_t n,
                          size_t half_bytes, const void *staging, hipStream_t stream);
// The same image written to / read from `host` directly: pinned host memory at its device
// address, 16-byte aligned.  `workgroups` (1..1024) bounds what the copy occupies of the chip.
hipError_t launch_gather_host(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                              size_t half_bytes, void *host, int32_t workgroups, hipStream_t stream);
hipError_t launch_scatter_host(void *k_pool, void *v_pool, const int32_t *ids, int32_t n, size_t half_bytes,
                               const void *host, int32_t workgroups, hipStream_t stream);
// The same for `nl` layers starting at `layer0` only; staging (and the host image of the
// layer-major swap calls) is [layer - layer0][i][keys | values] with layer_bytes each.
hipError_t launch_gather_layers(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                                size_t half_bytes, size_t layer_bytes, int32_t layer0, int32_t nl,
                                void *staging, hipStream_t stream);
hipError_t launch_scatter_layers(void *k_pool, void *v_pool, const int32_t *ids, int32_t n,
                                 size_t half_bytes, size_t layer_bytes, int32_t layer0, int32_t nl,
                                 const void *staging, hipStream_t stream);

}  // namespace lamps
