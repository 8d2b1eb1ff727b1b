// Per-wavefront attention reducers shared by the decode and the prefill kernels:
// the online-softmax pass of one wavefront over a token range of one request's
// paged K/V (arXiv 2410.18248, Section 2.2 equation; paging as in Section 7),
// on the vector ALUs (ValuReducer) or on the matrix cores (MfmaReducer).
// Device code; include from a .hip file only.
#pragma once
#include <hip/hip_runtime.h>

#include "internal.h"

namespace lamps {
namespace {

constexpr int kWaves = 4;               // wavefronts per workgroup
constexpr int kThreads = 64 * kWaves;
// wave-wide 16-byte loads per half-chunk and pool; a half-chunk (loads * tokens
// per load) must fit in the smallest block (16 tokens)
constexpr int loads_per_chunk(int lpt) { return lpt == 8 ? 2 : 4; }
constexpr int kHalves = 2;              // half-chunks per chunk on the 1-2 head vector-ALU paths
constexpr float kLowest = -3.0e38f;     // finite stand-in for "no score seen yet"
constexpr int kMaxShares = 16384;       // most wave shares the balanced scheme ever uses
constexpr size_t kPartialBudget = (size_t)64 << 20;   // bytes of partial slots it may need
// The context length of request r as the kernels use it: never beyond the block-table row (a
// longer value is the caller's mistake; clamped, it cannot send a lookup past the row).
__device__ __forceinline__ int ctx_len(const DecodeArgs &a, int r)
{
    return min(a.ctx_lens[r], a.max_blocks * a.block_size);
}

constexpr int kShareOwner = 1, kShareSlot1 = 2, kShareEmpty = 4;   // flags in share_info[].w
constexpr int kWideShares = 16;         // shares one block of the piece-parallel merge looks at

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(4))) float f32x4;
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

__device__ __forceinline__ void store_partial(float *pp, int D, int d, float M, float L, float A)
{
    pp[d] = A;
    if (d == 0) {
        pp[D] = M;
        pp[D + 1] = L;
    }
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

// ---------------------------------------------------------------- vector-ALU reducer

// Plain pool layout, GH query heads of the group per pass (GH == 1 for bf16).
template <bool BF16, int LPT, int GH, int NH>
struct ValuReducer {
    static constexpr bool kBF16 = BF16;
    static constexpr int VEC = BF16 ? 8 : 4;          // elements per 16-byte load
    static constexpr int D = LPT * VEC;
    static constexpr int ES = BF16 ? 2 : 4;           // element bytes
    static constexpr int TPW = 64 / LPT;              // tokens per wave-wide load
    static constexpr int kLoads = loads_per_chunk(LPT);
    static constexpr int HT = TPW * kLoads;           // tokens per half-chunk (<= 16 <= block_size)
    static constexpr int NL = NH * kLoads;            // wave-wide loads per chunk and pool
    static constexpr int CT = HT * NH;                // tokens per chunk

    // One wavefront reduces cached positions [t_begin, t_end) of request r (kv
    // head g, query heads h0 .. h0+GH-1), chunk after chunk, then calls
    // sink(h, d, M, L, A) once for every (head, dim): M = running max (log2
    // domain), L = sum of weights, A = weighted sum of V[:, d].  t_begin is a
    // multiple of CT.  No barrier, no LDS: waves of a workgroup are independent.
    // q is row `qrow` of a.q ([rows][H][D]); the block table row is r (decode: the same).
    template <typename Sink>
    static __device__ __forceinline__ void run(const DecodeArgs &a, int r, size_t qrow, int g, int h0, int,
                                               int t_begin, int t_end, Sink sink)
    {
        const int lane = threadIdx.x & 63;
        const int row = lane / LPT;                // which of the TPW tokens of a load
        const int col = lane % LPT;                // which 16-byte slice of the head vector

        // q slices of the GH heads, kept in registers for the whole range
        uint4 qv[GH];
#pragma unroll
        for (int h = 0; h < GH; ++h)
            qv[h] = *reinterpret_cast<const uint4 *>(
                static_cast<const char *>(a.q) +
                ((qrow * a.num_q_heads + h0 + h) * D + col * VEC) * ES);

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
        const size_t tile_bytes = (size_t)a.block_size * D * ES;
        const size_t block_stride = (size_t)a.num_layers * a.num_kv_heads * tile_bytes;
        const size_t head_off = ((size_t)a.layer * a.num_kv_heads + g) * tile_bytes;
        const char *kp = static_cast<const char *>(a.k_pool) + head_off + lane * 16;
        const char *vp = static_cast<const char *>(a.v_pool) + head_off + lane * 16;

        // A chunk is NH half-chunks of HT tokens; a half-chunk never straddles a
        // block (HT <= 16 <= block_size), so it needs one block-table entry.  All
        // NH * kLoads K loads and as many V loads of a chunk are issued before
        // any is consumed (a deeper software pipeline brought nothing here: with
        // up to eight waves per SIMD the other waves' loads fill the gaps).
        int ch = 0;
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
                // wave-uniform: half-chunks past the context are skipped, and so is a table entry
                // that does not name a block of the pool (the caller's mistake must not become a
                // wild read; the row it belongs to is then meaningless)
                if ((unsigned)pb[f] < (unsigned)a.num_blocks) {
                    const size_t off = (size_t)pb[f] * block_stride +
                                       (size_t)((t0 + f * HT) & (a.block_size - 1)) * D * ES;
                    if (t0 + (f + 1) * HT <= t_end) {
#pragma unroll
                        for (int i = 0; i < kLoads; ++i)
                            kx[f * kLoads + i] = load_stream16(kp + off + i * 1024);
#pragma unroll
                        for (int i = 0; i < kLoads; ++i)
                            vx[f * kLoads + i] = load_stream16(vp + off + i * 1024);
                    } else {                   // the context ends inside: loads wholly past it are skipped too
#pragma unroll
                        for (int i = 0; i < kLoads; ++i) {
                            const bool in = t0 + f * HT + i * TPW < t_end;
                            kx[f * kLoads + i] = in ? load_stream16(kp + off + i * 1024) : make_uint4(0, 0, 0, 0);
                            vx[f * kLoads + i] = in ? load_stream16(vp + off + i * 1024) : make_uint4(0, 0, 0, 0);
                        }
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < kLoads; ++i) {
                        kx[f * kLoads + i] = make_uint4(0, 0, 0, 0);
                        vx[f * kLoads + i] = make_uint4(0, 0, 0, 0);
                    }
                }
            }

            // physical blocks of the next chunk, fetched while the tiles arrive
            const int chn = ch + 1;
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

            if (t0 + CT > t_end) {             // ragged tail: slots at or past ctx_len never count
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

        if (row == 0) {
#pragma unroll
            for (int h = 0; h < GH; ++h)
#pragma unroll
                for (int e = 0; e < VEC; ++e) sink(h, col * VEC + e, m[h], l[h], acc[h][e]);
        }
    }
};

// ---------------------------------------------------------------- MFMA reducer

// bf16, tiled pool layout, up to 16 query heads of one kv group per pass.
// Per 16-token sub-tile (a chunk): scores^T[token][head] = K . q^T with D/32
// 16x16x32 MFMAs (A = a coalesced K load as it arrives, B = q slices held in
// registers); the result leaves each lane with 4 consecutive tokens of head
// lane%16, which after the softmax step is, converted to bf16, already the B
// operand p^T[token][head] of the 16x16x16 MFMAs that accumulate
// out^T[dim][head] += V^T . p^T (A = a coalesced V load).  So every statistic of
// head j lives in the lanes with lane%16 == j, and the only cross-lane step per
// sub-tile is the max over the four token groups (two shuffles).
template <int DIM>
struct MfmaReducer {
    static constexpr bool kBF16 = true;
    static constexpr int D = DIM;
    static constexpr int CT = 16;                     // tokens per chunk = one sub-tile
    static constexpr int NK = D / 32;                 // K loads = score MFMAs per sub-tile
    static constexpr int NS = D / 32;                 // V loads per sub-tile (two 16-dim slabs each)

    template <typename Sink>
    static __device__ __forceinline__ void run(const DecodeArgs &a, int r, size_t qrow, int g, int h0, int heads,
                                               int t_begin, int t_end, Sink sink)
    {
        const int lane = threadIdx.x & 63;
        const int j = lane & 15;                   // head (B / result column); dim in slab (V rows)
        const int qd = lane >> 4;                  // token group of 4 (results) / k slice (operands)

        // B operands of the score MFMAs: q[h0 + j][32 i + 8 qd .. + 8]; zero rows pad to 16 heads
        bf16x8 qb[NK];
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            uint4 t = make_uint4(0, 0, 0, 0);
            if (j < heads)
                t = *reinterpret_cast<const uint4 *>(
                    static_cast<const char *>(a.q) +
                    ((qrow * a.num_q_heads + h0 + j) * D + 32 * i + 8 * qd) * 2);
            qb[i] = __builtin_bit_cast(bf16x8, t);
        }

        float m = kLowest, l = 0.0f;               // m is the same in the 4 lanes of a head
        f32x4 o[2 * NS];                           // out^T: dims 16 s + 4 qd + e, head j
#pragma unroll
        for (int s = 0; s < 2 * NS; ++s) o[s] = f32x4{0.f, 0.f, 0.f, 0.f};

        const int n_chunks = (t_end - t_begin + CT - 1) / CT;
        const int32_t *table = a.block_table + (size_t)r * a.max_blocks;
        const size_t tile_bytes = (size_t)a.block_size * D * 2;
        const size_t block_stride = (size_t)a.num_layers * a.num_kv_heads * tile_bytes;
        const size_t head_off = ((size_t)a.layer * a.num_kv_heads + g) * tile_bytes;
        const char *kp = static_cast<const char *>(a.k_pool) + head_off + lane * 16;
        const char *vp = static_cast<const char *>(a.v_pool) + head_off + lane * 16;

        // Software pipeline: the loads of chunk ch + 1 are issued before chunk ch is
        // consumed, and the block-table entry of chunk ch + 2 is fetched with them,
        // so a wave always has a sub-tile of K and V in flight while it computes.
        auto entry = [&](int c) -> int {
            return c < n_chunks ? table[(t_begin + c * CT) >> a.log2_block_size] : 0;
        };
        auto issue = [&](int c, int block, uint4 (&kx)[NK], uint4 (&vx)[NS]) {
            // sub-tile (t % block_size) / 16 of the block's tile: 16 * D elements each
            const int t = t_begin + c * CT;
            const size_t off = (size_t)block * block_stride +
                               (size_t)((t & (a.block_size - 1)) >> 4) * (16 * D * 2);
            // (wave-uniform) a table entry that does not name a block of the pool is the caller's
            // mistake; it must not become a wild read: the sub-tile counts as zeros and the row it
            // belongs to is meaningless
            if ((unsigned)block < (unsigned)a.num_blocks) {
#pragma unroll
                for (int i = 0; i < NK; ++i) kx[i] = load_stream16(kp + off + i * 1024);
#pragma unroll
                for (int i = 0; i < NS; ++i) vx[i] = load_stream16(vp + off + i * 1024);
            } else {
#pragma unroll
                for (int i = 0; i < NK; ++i) kx[i] = make_uint4(0, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < NS; ++i) vx[i] = make_uint4(0, 0, 0, 0);
            }
        };
        uint4 kx[NK], vx[NS], kn[NK], vn[NS];
        int ch = 0;
        int pb1 = entry(1);
        if (n_chunks > 0) issue(0, entry(0), kx, vx);
        while (ch < n_chunks) {
            const int t0 = t_begin + ch * CT;
            const int pb2 = entry(ch + 2);
            if (ch + 1 < n_chunks) issue(ch + 1, pb1, kn, vn);
            pb1 = pb2;

            f32x4 s = {0.f, 0.f, 0.f, 0.f};        // tokens t0 + 4 qd + e, head j
#pragma unroll
            for (int i = 0; i < NK; ++i)
                s = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, kx[i]), qb[i],
                                                            s, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] *= a.scale_log2e;

            if (t0 + CT > t_end) {                 // ragged tail: slots at or past ctx_len never count
                const int valid = min(4, max(0, t_end - (t0 + 4 * qd)));   // of this lane's 4 tokens
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (e >= valid) s[e] = -INFINITY;
                // a V load holds tokens 4 qd + {0,1} in .x/.z and + {2,3} in .y/.w (16 bits each)
                const uint32_t m01 = valid >= 2 ? 0xFFFFFFFFu : (valid == 1 ? 0x0000FFFFu : 0u);
                const uint32_t m23 = valid >= 4 ? 0xFFFFFFFFu : (valid == 3 ? 0x0000FFFFu : 0u);
#pragma unroll
                for (int i = 0; i < NS; ++i) {
                    vx[i].x &= m01; vx[i].z &= m01;
                    vx[i].y &= m23; vx[i].w &= m23;
                }
            }

            float mx = fmaxf(fmaxf(s[0], s[1]), fmaxf(s[2], s[3]));
            mx = fmaxf(mx, __shfl_xor(mx, 16));
            mx = fmaxf(mx, __shfl_xor(mx, 32));
            const float mn = fmaxf(m, mx);
            const float sc = fast_exp2(m - mn);
            m = mn;
            float p[4], ps = 0.0f;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                p[e] = fast_exp2(s[e] - mn);
                ps += p[e];
            }
            l = l * sc + ps;
            // p as a bf16 pair: high part and (exactly computed) remainder
            union { s16x4 v; uint16_t u[4]; } ph, pl;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                ph.u[e] = to_bf16_rne(p[e]);
                pl.u[e] = to_bf16_rne(p[e] - __uint_as_float((uint32_t)ph.u[e] << 16));
            }
#pragma unroll
            for (int sidx = 0; sidx < 2 * NS; ++sidx) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[sidx][e] *= sc;
            }
#pragma unroll
            for (int i = 0; i < NS; ++i) {
                union { uint2 u; s16x4 v; } a0, a1;    // V^T rows: dim 32 i + j, and 32 i + 16 + j
                a0.u = make_uint2(vx[i].x, vx[i].y);
                a1.u = make_uint2(vx[i].z, vx[i].w);
                o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0.v, ph.v, o[2 * i], 0, 0, 0);
                o[2 * i] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a0.v, pl.v, o[2 * i], 0, 0, 0);
                o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1.v, ph.v, o[2 * i + 1], 0, 0, 0);
                o[2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x16bf16_1k(a1.v, pl.v, o[2 * i + 1], 0, 0, 0);
            }
            ++ch;
#pragma unroll
            for (int i = 0; i < NK; ++i) kx[i] = kn[i];
#pragma unroll
            for (int i = 0; i < NS; ++i) vx[i] = vn[i];
        }

        // the weight sum was kept per token group: add the four groups of a head
        l += __shfl_xor(l, 16);
        l += __shfl_xor(l, 32);

        if (j < heads) {
#pragma unroll
            for (int sidx = 0; sidx < 2 * NS; ++sidx)
#pragma unroll
                for (int e = 0; e < 4; ++e) sink(j, 16 * sidx + 4 * qd + e, m, l, o[sidx][e]);
        }
    }
};

}  // namespace
}  // namespace lamps
