// KV append: the step before attention in every decode iteration.
//
// arXiv 2410.18248, Section 2.2 / 2.2.1: each iteration produces one key and
// one value vector per layer (and kv head) for the token being generated and
// adds them to the request's cache, which is why the cache -- the M bytes per
// token of equations (1)-(3) -- grows with every iteration.  Here the new
// vectors of all running requests are written into the paged pools at cached
// position ctx_lens[r], i.e. slot ctx_lens[r] % block_size of physical block
// block_table[r][ctx_lens[r] / block_size], in the tile layout the decode
// kernels read (plain or tiled, see lamps.h).  Requests outside the running
// batch (Algorithm 1) append nothing.
//
// One workgroup per request (decode) or per token (many tokens at once).  In
// the decode form all threads read the request's context length, meet at a
// barrier, then scatter; with `advance` thread 0 stores length + 1 after the
// barrier, so nobody can read the new value.  A position outside the
// block-table row, or a block id outside the pool, writes nothing.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

constexpr int kAppendThreads = 256;

// Writes the key and value vectors kn, vn ([H_kv][D]) of one token at cached
// position t of request r.  Called by a whole workgroup.  A position outside the
// block-table row, or a block id outside the pool, writes nothing.
template <typename T, bool TILED>
__device__ __forceinline__ bool scatter_token(const AppendArgs &a, int r, int t, const T *kn, const T *vn)
{
    const int D = a.head_dim, Hkv = a.num_kv_heads, bs = a.block_size;
    const int lb = t >> a.log2_block_size, slot = t & (bs - 1);
    if (t < 0 || lb >= a.max_blocks) return false;
    const int block = a.block_table[(size_t)r * a.max_blocks + lb];
    if (block < 0 || block >= a.num_blocks) return false;
    const size_t tile = (size_t)bs * D;
    T *kt = static_cast<T *>(a.k_pool) + (((size_t)block * a.num_layers + a.layer) * Hkv) * tile;
    T *vt = static_cast<T *>(a.v_pool) + (((size_t)block * a.num_layers + a.layer) * Hkv) * tile;
    // 16 bytes at a time wherever 16 bytes of a vector stay together in the tile: keys in
    // both layouts (8 dims of a key are contiguous), values in the plain layout
    constexpr int V16 = 16 / (int)sizeof(T);
    for (int i = threadIdx.x * V16; i < Hkv * D; i += kAppendThreads * V16) {
        const int g = i / D, d = i - g * D;           // d is a multiple of V16, and V16 divides D
        const size_t ko = TILED ? (size_t)(slot >> 4) * 16 * D + (size_t)((d >> 3) * 16 + (slot & 15)) * 8
                                : (size_t)slot * D + d;
        *reinterpret_cast<uint4 *>(kt + g * tile + ko) = *reinterpret_cast<const uint4 *>(kn + i);
        if (!TILED) {
            *reinterpret_cast<uint4 *>(vt + g * tile + ko) = *reinterpret_cast<const uint4 *>(vn + i);
        } else {
            const size_t base = (size_t)(slot >> 4) * 16 * D;
            const int s16 = slot & 15;
#pragma unroll
            for (int e = 0; e < V16; ++e) {
                const int dd = d + e;
                const size_t vo = base +
                                  (size_t)(((((dd >> 5) * 4 + (s16 >> 2)) * 16 + (dd & 15)) * 2 + ((dd & 31) >> 4)) * 4) +
                                  (s16 & 3);
                vt[g * tile + vo] = vn[i + e];
            }
        }
    }
    return true;
}

template <typename T, bool TILED>
__global__ __launch_bounds__(kAppendThreads) void kv_append(const AppendArgs a)
{
    const int r = blockIdx.x;
    if (!a.running[r]) return;                        // uniform over the workgroup
    const int t = a.ctx_lens[r];
    __syncthreads();
    const size_t row = (size_t)r * a.num_kv_heads * a.head_dim;
    const bool ok = scatter_token<T, TILED>(a, r, t, static_cast<const T *>(a.k_new) + row,
                                            static_cast<const T *>(a.v_new) + row);
    if (ok && a.advance && threadIdx.x == 0) a.ctx_lens[r] = t + 1;
}

// Several new tokens per request (a prompt, a recomputed context, an API
// response): token row n of k_new / v_new belongs to the request r with
// q_start[r] <= n < q_start[r + 1] and goes to position
// ctx_lens[r] - (q_start[r + 1] - q_start[r]) + (n - q_start[r]), ctx_lens
// already counting the new tokens.  One workgroup per token.
template <typename T, bool TILED>
__global__ __launch_bounds__(kAppendThreads) void kv_append_tokens(const AppendArgs a)
{
    const int n = blockIdx.x;
    int lo = 0, hi = a.batch;                         // last r with q_start[r] <= n
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (a.q_start[mid] <= n) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int first = a.q_start[r], count = a.q_start[r + 1] - first;
    if (n >= first + count) return;                   // q_start[batch] is less than the grid
    const int t = a.ctx_lens[r] - count + (n - first);
    const size_t row = (size_t)n * a.num_kv_heads * a.head_dim;
    scatter_token<T, TILED>(a, r, t, static_cast<const T *>(a.k_new) + row,
                            static_cast<const T *>(a.v_new) + row);
}

}  // namespace

hipError_t launch_kv_append(const AppendArgs &a, int tiled, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    dim3 grid((unsigned)a.batch), block(kAppendThreads);
    if (a.bf16) {
        if (tiled)
            hipLaunchKernelGGL((kv_append<uint16_t, true>), grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL((kv_append<uint16_t, false>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((kv_append<float, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

hipError_t launch_kv_append_tokens(const AppendArgs &a, int total_tokens, int tiled, hipStream_t stream)
{
    if (a.batch == 0 || total_tokens == 0) return hipSuccess;
    dim3 grid((unsigned)total_tokens), block(kAppendThreads);
    if (a.bf16) {
        if (tiled)
            hipLaunchKernelGGL((kv_append_tokens<uint16_t, true>), grid, block, 0, stream, a);
        else
            hipLaunchKernelGGL((kv_append_tokens<uint16_t, false>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((kv_append_tokens<float, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace lamps
