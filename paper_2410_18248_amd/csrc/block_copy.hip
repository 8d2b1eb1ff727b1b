// KV block gather / scatter for the Swap handling strategy (arXiv 2410.18248,
// Section 1 and Section 4.2): the blocks of a request that enters an API call
// are scattered over the pool; they are packed into one contiguous staging
// area so that a single DMA moves them to pinned host memory, and unpacked the
// other way when the API returns.
//
// Staging image i = key-pool bytes of block ids[i] (all layers) followed by its
// value-pool bytes; the layer-major variant packs [layer][i][keys | values] of a
// range of layers instead, so that a swap can move one layer after the other.
// Pure 16-byte copies, bit-exact; grid.y walks (block, pool) pairs, grid.x and a
// stride loop walk the bytes of one such half.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

constexpr int kCopyThreads = 256;

// Every byte is touched once: non-temporal loads and stores keep the copy from displacing what
// the decode kernels stream through the caches next to it (decode under swap 1.046x -> 1.041x
// of decode alone).
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ void copy16(uint4 *dst, const uint4 *src)
{
    __builtin_nontemporal_store(__builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(src)),
                                reinterpret_cast<u32x4 *>(dst));
}

template <bool GATHER>
__global__ __launch_bounds__(kCopyThreads) void block_copy(uint4 *k_pool, uint4 *v_pool,
                                                           const int32_t *ids, size_t half_vecs,
                                                           uint4 *staging)
{
    const int i = blockIdx.y >> 1, which = blockIdx.y & 1;
    const size_t b = (size_t)ids[i];
    uint4 *pool = (which ? v_pool : k_pool) + b * half_vecs;
    uint4 *img = staging + ((size_t)i * 2 + which) * half_vecs;
    for (size_t x = (size_t)blockIdx.x * kCopyThreads + threadIdx.x; x < half_vecs;
         x += (size_t)gridDim.x * kCopyThreads) {
        if (GATHER)
            copy16(&img[x], &pool[x]);
        else
            copy16(&pool[x], &img[x]);
    }
}

template <bool GATHER>
hipError_t launch(void *k_pool, void *v_pool, const int32_t *ids, int32_t n, size_t half_bytes,
                  void *staging, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    if (n < 0 || 2 * (int64_t)n > 65535 || half_bytes % 16 != 0) return hipErrorInvalidValue;
    const size_t half_vecs = half_bytes / 16;
    // four 16-byte copies per thread per pass keeps loads in flight without a huge grid
    size_t gx = (half_vecs + kCopyThreads * 4 - 1) / (kCopyThreads * 4);
    if (gx < 1) gx = 1;
    if (gx > 256) gx = 256;
    dim3 grid((unsigned)gx, (unsigned)(2 * n));
    hipLaunchKernelGGL(block_copy<GATHER>, grid, dim3(kCopyThreads), 0, stream,
                       static_cast<uint4 *>(k_pool), static_cast<uint4 *>(v_pool), ids, half_vecs,
                       static_cast<uint4 *>(staging));
    return hipGetLastError();
}

// One layer range of the listed blocks: grid.y walks (block, pool) pairs, grid.z the layers.
template <bool GATHER>
__global__ __launch_bounds__(kCopyThreads) void block_copy_layers(uint4 *k_pool, uint4 *v_pool,
                                                                  const int32_t *ids, int n,
                                                                  size_t half_vecs, size_t layer_vecs,
                                                                  int layer0, uint4 *staging)
{
    const int i = blockIdx.y >> 1, which = blockIdx.y & 1, z = blockIdx.z;
    const size_t b = (size_t)ids[i];
    uint4 *pool = (which ? v_pool : k_pool) + b * half_vecs + (size_t)(layer0 + z) * layer_vecs;
    uint4 *img = staging + (((size_t)z * n + i) * 2 + which) * layer_vecs;
    for (size_t x = (size_t)blockIdx.x * kCopyThreads + threadIdx.x; x < layer_vecs;
         x += (size_t)gridDim.x * kCopyThreads) {
        if (GATHER)
            copy16(&img[x], &pool[x]);
        else
            copy16(&pool[x], &img[x]);
    }
}

template <bool GATHER>
hipError_t launch_layers(void *k_pool, void *v_pool, const int32_t *ids, int32_t n, size_t half_bytes,
                         size_t layer_bytes, int32_t layer0, int32_t nl, void *staging, hipStream_t stream)
{
    if (n == 0 || nl == 0) return hipSuccess;
    if (n < 0 || 2 * (int64_t)n > 65535 || nl < 0 || nl > 65535 || layer0 < 0 || half_bytes % 16 != 0 ||
        layer_bytes % 16 != 0 || (size_t)(layer0 + nl) * layer_bytes > half_bytes)
        return hipErrorInvalidValue;
    const size_t layer_vecs = layer_bytes / 16;
    size_t gx = (layer_vecs + kCopyThreads * 4 - 1) / (kCopyThreads * 4);
    if (gx < 1) gx = 1;
    if (gx > 256) gx = 256;
    dim3 grid((unsigned)gx, (unsigned)(2 * n), (unsigned)nl);
    hipLaunchKernelGGL(block_copy_layers<GATHER>, grid, dim3(kCopyThreads), 0, stream,
                       static_cast<uint4 *>(k_pool), static_cast<uint4 *>(v_pool), ids, (int)n, half_bytes / 16,
                       layer_vecs, (int)layer0, static_cast<uint4 *>(staging));
    return hipGetLastError();
}

// The same block-major image, but the image lives in pinned host memory that the device
// reaches over the host link: `workgroups` workgroups walk all 16-byte units of the list,
// four units in flight per thread (a read over the link takes microseconds).
template <bool GATHER>
__global__ __launch_bounds__(kCopyThreads) void block_copy_host(uint4 *k_pool, uint4 *v_pool,
                                                                const int32_t *ids, size_t half_vecs,
                                                                size_t total_vecs, uint4 *host)
{
    constexpr int kInFlight = 4;
    const size_t stride = (size_t)gridDim.x * kCopyThreads;
    for (size_t v0 = (size_t)blockIdx.x * kCopyThreads + threadIdx.x; v0 < total_vecs;
         v0 += kInFlight * stride) {
        uint4 r[kInFlight];
        uint4 *dev[kInFlight];
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const size_t v = v0 + k * stride;
            if (v >= total_vecs) continue;
            const size_t pair = v / half_vecs, x = v - pair * half_vecs;
            dev[k] = ((pair & 1) ? v_pool : k_pool) + (size_t)ids[pair >> 1] * half_vecs + x;
            r[k] = GATHER ? *dev[k] : host[v];
        }
#pragma unroll
        for (int k = 0; k < kInFlight; ++k) {
            const size_t v = v0 + k * stride;
            if (v >= total_vecs) continue;
            if (GATHER)
                host[v] = r[k];
            else
                *dev[k] = r[k];
        }
    }
}

template <bool GATHER>
hipError_t launch_host(void *k_pool, void *v_pool, const int32_t *ids, int32_t n, size_t half_bytes,
                       void *host, int32_t workgroups, hipStream_t stream)
{
    if (n == 0) return hipSuccess;
    if (n < 0 || workgroups < 1 || workgroups > 1024 || half_bytes % 16 != 0) return hipErrorInvalidValue;
    const size_t half_vecs = half_bytes / 16;
    hipLaunchKernelGGL(block_copy_host<GATHER>, dim3((unsigned)workgroups), dim3(kCopyThreads), 0, stream,
                       static_cast<uint4 *>(k_pool), static_cast<uint4 *>(v_pool), ids, half_vecs,
                       (size_t)n * 2 * half_vecs, static_cast<uint4 *>(host));
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gather_host(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                              size_t half_bytes, void *host, int32_t workgroups, hipStream_t stream)
{
    return launch_host<true>(const_cast<void *>(k_pool), const_cast<void *>(v_pool), ids, n, half_bytes, host,
                             workgroups, stream);
}

hipError_t launch_scatter_host(void *k_pool, void *v_pool, const int32_t *ids, int32_t n, size_t half_bytes,
                               const void *host, int32_t workgroups, hipStream_t stream)
{
    return launch_host<false>(k_pool, v_pool, ids, n, half_bytes, const_cast<void *>(host), workgroups, stream);
}

hipError_t launch_gather_layers(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                                size_t half_bytes, size_t layer_bytes, int32_t layer0, int32_t nl,
                                void *staging, hipStream_t stream)
{
    return launch_layers<true>(const_cast<void *>(k_pool), const_cast<void *>(v_pool), ids, n, half_bytes,
                               layer_bytes, layer0, nl, staging, stream);
}

hipError_t launch_scatter_layers(void *k_pool, void *v_pool, const int32_t *ids, int32_t n,
                                 size_t half_bytes, size_t layer_bytes, int32_t layer0, int32_t nl,
                                 const void *staging, hipStream_t stream)
{
    return launch_layers<false>(k_pool, v_pool, ids, n, half_bytes, layer_bytes, layer0, nl,
                                const_cast<void *>(staging), stream);
}

hipError_t launch_gather(const void *k_pool, const void *v_pool, const int32_t *ids, int32_t n,
                         size_t half_bytes, void *staging, hipStream_t stream)
{
    return launch<true>(const_cast<void *>(k_pool), const_cast<void *>(v_pool), ids, n, half_bytes,
                        staging, stream);
}

hipError_t launch_scatter(void *k_pool, void *v_pool, const int32_t *ids, int32_t n,
                          size_t half_bytes, const void *staging, hipStream_t stream)
{
    return launch<false>(k_pool, v_pool, ids, n, half_bytes, const_cast<void *>(staging), stream);
}

}  // namespace lamps
