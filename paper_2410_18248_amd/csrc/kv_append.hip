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
// One workgroup per request.  All threads read the request's context length,
// meet at a barrier, then scatter; with `advance` thread 0 stores length + 1
// after the barrier, so nobody can read the new value.  A position outside the
// block-table row, or a block id outside the pool, writes nothing.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

constexpr int kAppendThreads = 256;

template <typename T, bool TILED>
__global__ __launch_bounds__(kAppendThreads) void kv_append(const AppendArgs a)
{
    const int r = blockIdx.x;
    if (!a.running[r]) return;                        // uniform over the workgroup
    const int t = a.ctx_lens[r];
    __syncthreads();
    const int D = a.head_dim, Hkv = a.num_kv_heads, bs = a.block_size;
    const int lb = t >> a.log2_block_size, slot = t & (bs - 1);
    if (t < 0 || lb >= a.max_blocks) return;
    const int block = a.block_table[(size_t)r * a.max_blocks + lb];
    if (block < 0 || block >= a.num_blocks) return;
    const size_t tile = (size_t)bs * D;
    T *kt = static_cast<T *>(a.k_pool) + (((size_t)block * a.num_layers + a.layer) * Hkv) * tile;
    T *vt = static_cast<T *>(a.v_pool) + (((size_t)block * a.num_layers + a.layer) * Hkv) * tile;
    const T *kn = static_cast<const T *>(a.k_new) + (size_t)r * Hkv * D;
    const T *vn = static_cast<const T *>(a.v_new) + (size_t)r * Hkv * D;
    for (int i = threadIdx.x; i < Hkv * D; i += kAppendThreads) {
        const int g = i / D, d = i - g * D;
        size_t ko, vo;
        if (TILED) {                                  // the element orders of lamps.h
            const size_t base = (size_t)(slot >> 4) * 16 * D;
            const int s16 = slot & 15;
            ko = base + (size_t)((d >> 3) * 16 + s16) * 8 + (d & 7);
            vo = base + (size_t)(((((d >> 5) * 4 + (s16 >> 2)) * 16 + (d & 15)) * 2 + ((d & 31) >> 4)) * 4) +
                 (s16 & 3);
        } else {
            ko = vo = (size_t)slot * D + d;
        }
        kt[g * tile + ko] = kn[i];
        vt[g * tile + vo] = vn[i];
    }
    if (a.advance && threadIdx.x == 0) a.ctx_lens[r] = t + 1;
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

}  // namespace lamps
