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

// The same for the tiled layout (bf16), where the 16-byte unit of a value tile is four
// consecutive positions of two dims: one token alone can only write it 16 bits at a time.
// One workgroup per (request, 16-position sub-tile that holds new tokens, kv head): keys are
// copied 16 bytes at a time as above; for values a thread takes four consecutive positions
// and 2 x 2 dims, transposes them in registers and stores two whole units; only the
// positions of a quad that is not entirely new -- at most one at each end of a request's
// range -- fall back to 16-bit stores.
// Workgroup w belongs to the last request r with (q_start[r] >> 4) + 2 r <= w: request r
// touches at most (count >> 4) + 2 sub-tiles, and the keys of consecutive requests are at
// least that far apart.
__global__ __launch_bounds__(kAppendThreads) void kv_append_tokens_tiled(const AppendArgs a)
{
    typedef uint16_t T;
    const int w = blockIdx.x;
    int lo = 0, hi = a.batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((a.q_start[mid] >> 4) + 2 * mid <= w) lo = mid; else hi = mid;
    }
    const int r = lo;
    const int first = a.q_start[r], count = a.q_start[r + 1] - first;
    const int p0 = a.ctx_lens[r] - count;             // position of the request's first new token
    if (count <= 0 || p0 < 0) return;
    const int sub = (p0 >> 4) + (w - ((first >> 4) + 2 * r));     // sub-tile of the request's context
    const int t_lo = max(p0, sub * 16), t_hi = min(p0 + count, sub * 16 + 16);
    if (t_lo >= t_hi) return;
    const int D = a.head_dim, Hkv = a.num_kv_heads, bs = a.block_size;
    const int lb = (sub * 16) >> a.log2_block_size;
    if (lb >= a.max_blocks) return;
    const int block = a.block_table[(size_t)r * a.max_blocks + lb];
    if (block < 0 || block >= a.num_blocks) return;
    const size_t tile = (size_t)bs * D;
    const size_t at = (((size_t)block * a.num_layers + a.layer) * Hkv) * tile + (size_t)(((sub * 16) & (bs - 1)) >> 4) * 16 * D;
    T *kt = static_cast<T *>(a.k_pool) + at;
    T *vt = static_cast<T *>(a.v_pool) + at;
    const T *kn = static_cast<const T *>(a.k_new), *vn = static_cast<const T *>(a.v_new);
    const int row = Hkv * D;                          // elements of one token's keys (or values)

    const int g = blockIdx.y;                         // kv head
    kt += g * tile; vt += g * tile;
    kn += g * D; vn += g * D;

    const int c8 = D / 8;                             // keys: (position, 8 dims) -> one 16-byte unit
    for (int i = threadIdx.x; i < (t_hi - t_lo) * c8; i += kAppendThreads) {
        const int c = i % c8, t = t_lo + i / c8;
        *reinterpret_cast<uint4 *>(kt + (size_t)(c * 16 + (t & 15)) * 8) =
            *reinterpret_cast<const uint4 *>(kn + (size_t)(first + (t - p0)) * row + c * 8);
    }

    // values: (quad of positions, 32-dim group, dims 2 j, 2 j + 1 of its first 16 and of its last 16)
    for (int i = threadIdx.x; i < 4 * (D / 32) * 8; i += kAppendThreads) {
        const int j = i & 7, i32 = (i >> 3) % (D / 32), q = i / (8 * (D / 32));
        const int t0 = sub * 16 + 4 * q;              // the quad's first position
        if (t0 + 4 <= t_lo || t0 >= t_hi) continue;
        const int d0 = 32 * i32 + 2 * j;
        T *dst = vt + (size_t)((i32 * 4 + q) * 16 + 2 * j) * 8;   // unit of dim d0; dim d0 + 1's follows
        if (t0 >= t_lo && t0 + 4 <= t_hi) {
            uint32_t lo2[4], hi2[4];                  // [position]: dims d0, d0 + 1 and d0 + 16, d0 + 17
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const T *src = vn + (size_t)(first + (t0 + k - p0)) * row + d0;
                lo2[k] = *reinterpret_cast<const uint32_t *>(src);
                hi2[k] = *reinterpret_cast<const uint32_t *>(src + 16);
            }
#pragma unroll
            for (int e = 0; e < 2; ++e) {
                const int sh = 16 * e;
                uint4 u;
                u.x = ((lo2[0] >> sh) & 0xFFFFu) | ((lo2[1] >> sh) << 16);
                u.y = ((lo2[2] >> sh) & 0xFFFFu) | ((lo2[3] >> sh) << 16);
                u.z = ((hi2[0] >> sh) & 0xFFFFu) | ((hi2[1] >> sh) << 16);
                u.w = ((hi2[2] >> sh) & 0xFFFFu) | ((hi2[3] >> sh) << 16);
                *reinterpret_cast<uint4 *>(dst + e * 8) = u;
            }
        } else {
            for (int k = 0; k < 4; ++k) {
                const int t = t0 + k;
                if (t < t_lo || t >= t_hi) continue;
                const T *src = vn + (size_t)(first + (t - p0)) * row + d0;
#pragma unroll
                for (int e = 0; e < 2; ++e) {
                    dst[e * 8 + k] = src[e];
                    dst[e * 8 + 4 + k] = src[16 + e];
                }
            }
        }
    }
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
            hipLaunchKernelGGL(kv_append_tokens_tiled, dim3((unsigned)((total_tokens >> 4) + 2 * a.batch), (unsigned)a.num_kv_heads),
                               block, 0, stream, a);
        else
            hipLaunchKernelGGL((kv_append_tokens<uint16_t, false>), grid, block, 0, stream, a);
    } else {
        hipLaunchKernelGGL((kv_append_tokens<float, false>), grid, block, 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace lamps
