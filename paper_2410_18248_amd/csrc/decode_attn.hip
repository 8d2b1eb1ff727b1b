// Paged single-query decode attention for gfx950 (MI355X).
//
// Computes, for every running request r and query head h, the Section 2.2
// equation of arXiv 2410.18248,  out = softmax(q K^T * scale) V,  over the
// first ctx_lens[r] cached positions of r, with K and V reached through the
// block table (paged attention, Section 7).  The context is cut into
// partitions of `part_tokens` tokens; one workgroup reduces one
// (request, kv head, partition) to (max, sum, weighted value sum) with an
// online softmax, and a second small kernel merges the partitions of a request
// (skipped when the configuration has a single partition per request).
//
// Mapping to the hardware.  The path is a stream over K and V (every byte is
// used once: ~1 flop/byte), so it is HBM-bound and runs on the vector ALUs, not
// on MFMA.  A (block, layer, kv head) tile is block_size*head_dim contiguous
// elements; a wavefront reads it with fully coalesced 16-byte-per-lane loads:
// LPT = head_dim*sizeof/16 lanes cover one token, 64/LPT tokens per load.  Each
// lane keeps its 16-byte slice of q for all heads of the kv group in
// registers, so the G query heads of a group share every K/V byte that is
// loaded.  The dot product is finished with DPP adds inside the LPT lanes (no
// LDS).  Each group of LPT lanes ("row") carries its own running max / sum /
// accumulator over the tokens it sees, so there is no cross-lane traffic in
// the main loop beyond the dot-product reduction; rows are merged by shuffles
// and the four waves through LDS once per workgroup.
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

constexpr int kWaves = 4;               // wavefronts per workgroup
constexpr int kThreads = 64 * kWaves;
// wave-wide 16-byte loads per chunk and pool; a chunk (loads * tokens per load)
// must fit in the smallest block (16 tokens)
constexpr int loads_per_chunk(int lpt) { return lpt == 8 ? 2 : 4; }
#ifndef LAMPS_HALVES
#define LAMPS_HALVES 2
#endif
constexpr int kHalves = LAMPS_HALVES;   // half-chunks in flight per wave for 1- and 2-head groups
constexpr float kLowest = -3.0e38f;     // finite stand-in for "no score seen yet"

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;

// K and V are read exactly once per launch: a non-temporal 16-byte load keeps
// the stream from displacing anything in the caches (measurably faster here).
__device__ __forceinline__ uint4 load_stream16(const char *p)
{
    u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(t.x, t.y, t.z, t.w);
}

template <int CTRL>
__device__ __forceinline__ float dpp_add(float x)
{
    int y = __builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true);
    return x + __int_as_float(y);
}

// Sum over the LPT consecutive lanes that hold one token; every lane gets the
// same bits (each step adds the same two numbers on both sides).
template <int LPT>
__device__ __forceinline__ float sum_token_lanes(float x)
{
    x = dpp_add<0xB1>(x);                       // quad_perm [1,0,3,2]
    x = dpp_add<0x4E>(x);                       // quad_perm [2,3,0,1]
    if (LPT >= 8) x = dpp_add<0x141>(x);        // row_half_mirror
    if (LPT >= 16) x = dpp_add<0x140>(x);       // row_mirror
    if (LPT >= 32) x += __shfl_xor(x, 16);
    if (LPT >= 64) x += __shfl_xor(x, 32);
    return x;
}

__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// fp32 -> bf16 bits, round to nearest even.
__device__ __forceinline__ uint16_t to_bf16_rne(float f)
{
    uint32_t b = __float_as_uint(f);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0;
    return (uint16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}

template <bool BF16>
__device__ __forceinline__ void store_out(void *out, size_t i, float o)
{
    if (BF16)
        static_cast<uint16_t *>(out)[i] = to_bf16_rne(o);
    else
        static_cast<float *>(out)[i] = o;
}

// Partial dot product of a lane's 16 bytes of q and K.
template <bool BF16>
__device__ __forceinline__ float dot16(const uint4 &q, const uint4 &k)
{
    if (BF16) {
        float s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.x),
                                                  __builtin_bit_cast(bf16x2, k.x), 0.0f, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.y),
                                            __builtin_bit_cast(bf16x2, k.y), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.z),
                                            __builtin_bit_cast(bf16x2, k.z), s, false);
        s = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, q.w),
                                            __builtin_bit_cast(bf16x2, k.w), s, false);
        return s;
    } else {
        float s = __uint_as_float(q.x) * __uint_as_float(k.x);
        s = fmaf(__uint_as_float(q.y), __uint_as_float(k.y), s);
        s = fmaf(__uint_as_float(q.z), __uint_as_float(k.z), s);
        s = fmaf(__uint_as_float(q.w), __uint_as_float(k.w), s);
        return s;
    }
}

// A lane's 16 bytes of V as floats.
template <bool BF16, int VEC>
__device__ __forceinline__ void unpack(const uint4 &v, float (&f)[VEC])
{
    if constexpr (BF16) {
        f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
        f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
        f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
        f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
    } else {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
}

// (m, l, acc) <- merge of (m, l, acc) and (mo, lo, acco), both in exp2 domain.
template <int VEC>
__device__ __forceinline__ void merge_state(float &m, float &l, float (&acc)[VEC], float mo,
                                            float lo, const float (&acco)[VEC])
{
    float mn = fmaxf(m, mo);
    float fa = fast_exp2(m - mn), fb = fast_exp2(mo - mn);
    l = l * fa + lo * fb;
#pragma unroll
    for (int e = 0; e < VEC; ++e) acc[e] = acc[e] * fa + acco[e] * fb;
    m = mn;
}

// One workgroup: one (partition, request, kv head / head chunk), decoded from a
// 1-D grid.  GH query heads of the kv group share the K/V stream.
template <bool BF16, int LPT, int GH, int NH>
__global__ __launch_bounds__(kThreads) void decode_partial(const DecodeArgs a)
{
    constexpr int VEC = BF16 ? 8 : 4;          // elements per 16-byte load
    constexpr int D = LPT * VEC;
    constexpr int TPW = 64 / LPT;              // tokens per wave-wide load
    constexpr int kLoads = loads_per_chunk(LPT);
    constexpr int HT = TPW * kLoads;           // tokens per half-chunk (<= 16 <= block_size)
    constexpr int NL = NH * kLoads;            // wave-wide loads per chunk and pool
    constexpr int CT = HT * NH;                // tokens per chunk

    // Workgroups are handed to the eight XCDs round-robin in launch order, so the
    // index that varies fastest must be one along which the work is even: the
    // kv head (and head chunk), then the request, then the partition.  (With the
    // partition fastest and eight partitions, all first partitions -- most of
    // the work -- would land on one XCD.)
    const int G = a.num_q_heads / a.num_kv_heads;
    const int chunks_per_group = G / GH;
    const int hc_count = a.num_kv_heads * chunks_per_group;
    const int hc = blockIdx.x % hc_count;
    const int r = (blockIdx.x / hc_count) % a.batch;
    const int part = blockIdx.x / (hc_count * a.batch);
    if (!a.running[r]) return;                 // Preserve / Swap / Discard: not in the batch
    const int C = a.ctx_lens[r];
    const int t_begin = part * a.part_tokens;
    if (t_begin >= C && part != 0) return;     // partition 0 of an empty context writes zeros
    const int t_end = min(C, t_begin + a.part_tokens);
    const int n_parts = max(1, (C + a.part_tokens - 1) / a.part_tokens);
    const int g = hc / chunks_per_group;
    const int h0 = g * G + (hc % chunks_per_group) * GH;

    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int row = lane / LPT;                // which of the TPW tokens of a load
    const int col = lane % LPT;                // which 16-byte slice of the head vector

    // q slices of the GH heads, kept in registers for the whole partition.
    uint4 qv[GH];
#pragma unroll
    for (int h = 0; h < GH; ++h)
        qv[h] = *reinterpret_cast<const uint4 *>(
            static_cast<const char *>(a.q) + (((size_t)r * a.num_q_heads + h0 + h) * D + col * VEC) *
                                                 (BF16 ? 2 : 4));

    float m[GH], l[GH], acc[GH][VEC];
#pragma unroll
    for (int h = 0; h < GH; ++h) {
        m[h] = kLowest;
        l[h] = 0.0f;
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[h][e] = 0.0f;
    }

    const int n_chunks = (t_end - t_begin + CT - 1) / CT;
    const int32_t *table = a.block_table + (size_t)r * a.max_blocks;
    const size_t tile_bytes = (size_t)a.block_size * D * (BF16 ? 2 : 4);
    const size_t block_stride = (size_t)a.num_layers * a.num_kv_heads * tile_bytes;
    const size_t head_off = ((size_t)a.layer * a.num_kv_heads + g) * tile_bytes;
    const char *kp = static_cast<const char *>(a.k_pool) + head_off + lane * 16;
    const char *vp = static_cast<const char *>(a.v_pool) + head_off + lane * 16;

    // A chunk is NH half-chunks of HT tokens; a half-chunk never straddles a
    // block (HT <= 16 <= block_size), so it needs one block-table entry.  All
    // NH * kLoads K loads and as many V loads of a chunk are issued before any
    // is consumed.
    int ch = w;
    int pb[NH], pbn[NH];
#pragma unroll
    for (int f = 0; f < NH; ++f) {
        const int th = t_begin + ch * CT + f * HT;
        pb[f] = (ch < n_chunks && th < t_end) ? table[th >> a.log2_block_size] : -1;
    }
    while (ch < n_chunks) {
        const int t0 = t_begin + ch * CT;
        uint4 kx[NL], vx[NL];
#pragma unroll
        for (int f = 0; f < NH; ++f) {
            if (pb[f] >= 0) {                  // wave-uniform: half-chunks past the context are skipped
                const size_t off = (size_t)pb[f] * block_stride +
                                   (size_t)((t0 + f * HT) & (a.block_size - 1)) * D * (BF16 ? 2 : 4);
#pragma unroll
                for (int i = 0; i < kLoads; ++i) kx[f * kLoads + i] = load_stream16(kp + off + i * 1024);
#pragma unroll
                for (int i = 0; i < kLoads; ++i) vx[f * kLoads + i] = load_stream16(vp + off + i * 1024);
            } else {
#pragma unroll
                for (int i = 0; i < kLoads; ++i) {
                    kx[f * kLoads + i] = make_uint4(0, 0, 0, 0);
                    vx[f * kLoads + i] = make_uint4(0, 0, 0, 0);
                }
            }
        }

        // physical blocks of this wave's next chunk, fetched while the tiles arrive
        const int chn = ch + kWaves;
#pragma unroll
        for (int f = 0; f < NH; ++f) {
            const int th = t_begin + chn * CT + f * HT;
            pbn[f] = (chn < n_chunks && th < t_end) ? table[th >> a.log2_block_size] : -1;
        }

        float s[GH][NL];
#pragma unroll
        for (int h = 0; h < GH; ++h)
#pragma unroll
            for (int i = 0; i < NL; ++i)
                s[h][i] = sum_token_lanes<LPT>(dot16<BF16>(qv[h], kx[i])) * a.scale_log2e;

        if (t0 + CT > t_end) {                 // ragged tail: slots at or past ctx_len never count
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                if (t0 + i * TPW + row >= t_end) {
#pragma unroll
                    for (int h = 0; h < GH; ++h) s[h][i] = -INFINITY;
                    vx[i] = make_uint4(0, 0, 0, 0);
                }
            }
        }

#pragma unroll
        for (int h = 0; h < GH; ++h) {
            float mn = m[h];
#pragma unroll
            for (int i = 0; i < NL; ++i) mn = fmaxf(mn, s[h][i]);
            const float sc = fast_exp2(m[h] - mn);
            float ps = 0.0f;
#pragma unroll
            for (int i = 0; i < NL; ++i) {
                s[h][i] = fast_exp2(s[h][i] - mn);   // now the weight p
                ps += s[h][i];
            }
            l[h] = l[h] * sc + ps;
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[h][e] *= sc;
            m[h] = mn;
        }
#pragma unroll
        for (int i = 0; i < NL; ++i) {
            float vf[VEC];
            unpack<BF16, VEC>(vx[i], vf);
#pragma unroll
            for (int h = 0; h < GH; ++h)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[h][e] = fmaf(s[h][i], vf[e], acc[h][e]);
        }
        ch = chn;
#pragma unroll
        for (int f = 0; f < NH; ++f) pb[f] = pbn[f];
    }

    // rows of a wave -> one state per wave
#pragma unroll
    for (int h = 0; h < GH; ++h) {
#pragma unroll
        for (int stride = LPT; stride < 64; stride *= 2) {
            float mo = __shfl_xor(m[h], stride), lo = __shfl_xor(l[h], stride);
            float ao[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) ao[e] = __shfl_xor(acc[h][e], stride);
            merge_state<VEC>(m[h], l[h], acc[h], mo, lo, ao);
        }
    }

    // waves -> one state per workgroup, through LDS
    __shared__ float sm_acc[kWaves][GH][D];
    __shared__ float sm_m[kWaves][GH], sm_l[kWaves][GH];
    if (row == 0) {
#pragma unroll
        for (int h = 0; h < GH; ++h) {
#pragma unroll
            for (int e = 0; e < VEC; ++e) sm_acc[w][h][col * VEC + e] = acc[h][e];
            if (col == 0) {
                sm_m[w][h] = m[h];
                sm_l[w][h] = l[h];
            }
        }
    }
    __syncthreads();

    const size_t rh0 = (size_t)r * a.num_q_heads + h0;
    for (int idx = threadIdx.x; idx < GH * D; idx += kThreads) {
        const int h = idx / D, d = idx % D;
        float M = sm_m[0][h];
#pragma unroll
        for (int ww = 1; ww < kWaves; ++ww) M = fmaxf(M, sm_m[ww][h]);
        float L = 0.0f, A = 0.0f;
#pragma unroll
        for (int ww = 0; ww < kWaves; ++ww) {
            float f = fast_exp2(sm_m[ww][h] - M);
            L += sm_l[ww][h] * f;
            A += sm_acc[ww][h][d] * f;
        }
        if (n_parts == 1) {
            store_out<BF16>(a.out, (rh0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
        } else {
            float *pp = a.partials + ((rh0 + h) * a.max_parts + part) * (D + 2);
            pp[d] = A;
            if (d == 0) {
                pp[D] = M;
                pp[D + 1] = L;
            }
        }
    }
}

// Merge of the partitions of one (request, query head), always in partition
// order; block = head_dim threads.  A separate launch on purpose: a kernel
// boundary makes the partials visible across the eight XCDs' L2s once, whereas
// a device-scope fence per workgroup writes back and invalidates an L2 each time.
template <bool BF16>
__global__ void decode_merge(const DecodeArgs a)
{
    const int r = blockIdx.y, h = blockIdx.x, d = threadIdx.x;
    if (!a.running[r]) return;
    const int C = a.ctx_lens[r];
    const int n_parts = (C + a.part_tokens - 1) / a.part_tokens;
    if (n_parts <= 1) return;                  // written by the partial kernel already
    const int D = a.head_dim;
    const size_t rh = (size_t)r * a.num_q_heads + h;
    const float *pp = a.partials + rh * a.max_parts * (D + 2);
    float M = kLowest;
    for (int p = 0; p < n_parts; ++p) M = fmaxf(M, pp[(size_t)p * (D + 2) + D]);
    float L = 0.0f, A = 0.0f;
    for (int p = 0; p < n_parts; ++p) {
        const float *x = pp + (size_t)p * (D + 2);
        float f = fast_exp2(x[D] - M);
        L += x[D + 1] * f;
        A += x[d] * f;
    }
    store_out<BF16>(a.out, rh * D + d, L > 0.0f ? A / L : 0.0f);
}

template <bool BF16, int LPT>
hipError_t launch_partial(const DecodeArgs &a, int gh, dim3 grid, hipStream_t s)
{
    switch (gh) {
    case 1: hipLaunchKernelGGL((decode_partial<BF16, LPT, 1, kHalves>), grid, dim3(kThreads), 0, s, a); break;
    case 2: hipLaunchKernelGGL((decode_partial<BF16, LPT, 2, kHalves>), grid, dim3(kThreads), 0, s, a); break;
    case 4: hipLaunchKernelGGL((decode_partial<BF16, LPT, 4, 1>), grid, dim3(kThreads), 0, s, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace

int decode_heads_per_group(int bf16, int head_dim, int group)
{
    const int lpt = head_dim * (bf16 ? 2 : 4) / 16;
    if (head_dim * (bf16 ? 2 : 4) % 16 != 0 || (lpt != 8 && lpt != 16 && lpt != 32)) return 0;
    if (group <= 0) return 0;
    if (group % 4 == 0) return 4;
    if (group % 2 == 0) return 2;
    return 1;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int gh = decode_heads_per_group(a.bf16, a.head_dim, G);
    if (gh == 0) return hipErrorInvalidValue;
    const int lpt = a.head_dim * (a.bf16 ? 2 : 4) / 16;
    dim3 grid((unsigned)((size_t)a.max_parts * a.num_kv_heads * (G / gh) * a.batch));
    hipError_t e = hipErrorInvalidValue;
    if (a.bf16) {
        if (lpt == 8) e = launch_partial<true, 8>(a, gh, grid, stream);
        if (lpt == 16) e = launch_partial<true, 16>(a, gh, grid, stream);
        if (lpt == 32) e = launch_partial<true, 32>(a, gh, grid, stream);
    } else {
        if (lpt == 8) e = launch_partial<false, 8>(a, gh, grid, stream);
        if (lpt == 16) e = launch_partial<false, 16>(a, gh, grid, stream);
        if (lpt == 32) e = launch_partial<false, 32>(a, gh, grid, stream);
    }
    if (e != hipSuccess || a.max_parts == 1) return e;
    dim3 mg(a.num_q_heads, a.batch);
    if (a.bf16)
        hipLaunchKernelGGL(decode_merge<true>, mg, dim3(a.head_dim), 0, stream, a);
    else
        hipLaunchKernelGGL(decode_merge<false>, mg, dim3(a.head_dim), 0, stream, a);
    return hipGetLastError();
}

}  // namespace lamps
