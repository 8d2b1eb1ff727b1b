// Paged single-query decode attention for gfx950 (MI355X).
//
// Computes, for every running request r and query head h, the Section 2.2
// equation of arXiv 2410.18248,  out = softmax(q K^T * scale) V,  over the
// first ctx_lens[r] cached positions of r, with K and V reached through the
// block table (paged attention, Section 7).
//
// Work decomposition.  The unit of work is a chunk of CT tokens of one
// (request, kv head, pass over GH query heads of the group).  Two schemes share
// the same inner loops:
//   balanced (default): all chunks of all running requests form one flat
//     sequence; as many wavefronts as the chip holds at once each take an equal
//     contiguous share of it, so every wavefront ends within a chunk of the
//     others however skewed the context lengths are.  A share is at most: the
//     tail of one (request, head), some whole ones, and the head of another;
//     whole ones are written out directly, the two partial ends go to
//     per-share slots that a small second kernel merges.
//   fixed partitions (part_tokens > 0): the context is cut every part_tokens
//     tokens, one wavefront per (partition, request, kv head) in a dense grid.
// A wavefront works alone (no LDS, no barrier in the main path): with many short
// requests there are far more (request, head) ranges than workgroups, and four
// waves cooperating on each would spend their time in start-up and hand-over.
// Partitions are merged by a separate launch on purpose: a kernel boundary
// makes the partials visible across the eight XCDs' L2s once, whereas a
// device-scope fence per workgroup writes back and invalidates an L2 each time.
//
// Inner loops.  The path is a stream over K and V: every byte is used once, by
// the G query heads of its group.
//   G == 1 (and all fp32): ~1 flop per byte, a matrix-vector product.  Vector
//     ALUs, no MFMA: a tile is block_size*head_dim contiguous elements read
//     with coalesced non-temporal 16-byte-per-lane loads, LPT = head_dim*size/16
//     lanes per token; q slices stay in registers; the dot product ends with
//     DPP adds inside the LPT lanes; each group of LPT lanes ("row") carries
//     its own running max / sum / accumulator, rows are merged by shuffles.
//   bf16 with G >= 2: the group's heads make q a G x d_h matrix and both
//     products real (skinny) contractions, and on the vector ALUs their cost
//     grows with G until it co-limits with HBM.  They go to MFMA instead
//     (16x16x32 for K q^T, 16x16x16 for V^T p^T, up to 16 heads per pass), and
//     the pools use the tiled layout of lamps.h so that a coalesced 16-byte
//     load IS an MFMA operand: no LDS staging, no shuffles.  The weights p are
//     fed as a bf16 pair (high part + remainder), which keeps fp32-grade
//     weights at the price of a second, nearly free, MFMA.
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
constexpr int kShareOwner = 1, kShareSlot1 = 2, kShareEmpty = 4;   // flags in share_info[].w
constexpr int kMergeList = 64;          // pieces whose slots are resolved per pass of the balanced merge

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
    template <typename Sink>
    static __device__ __forceinline__ void run(const DecodeArgs &a, int r, int g, int h0, int,
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
                (((size_t)r * a.num_q_heads + h0 + h) * D + col * VEC) * ES);

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
                if (pb[f] >= 0) {              // wave-uniform: half-chunks past the context are skipped
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
    static __device__ __forceinline__ void run(const DecodeArgs &a, int r, int g, int h0, int heads,
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
                    (((size_t)r * a.num_q_heads + h0 + j) * D + 32 * i + 8 * qd) * 2);
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
#pragma unroll
            for (int i = 0; i < NK; ++i) kx[i] = load_stream16(kp + off + i * 1024);
#pragma unroll
            for (int i = 0; i < NS; ++i) vx[i] = load_stream16(vp + off + i * 1024);
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

// ---------------------------------------------------------------- fixed partitions

// One wavefront: one (partition, request, kv head / pass), decoded from a 1-D
// index.  The heads of one pass share the K/V stream.
template <typename R>
__global__ __launch_bounds__(kThreads) void decode_partial(const DecodeArgs a)
{
    constexpr int D = R::D;
    // Workgroups are handed to the eight XCDs round-robin in launch order, so the
    // index that varies fastest must be one along which the work is even: the
    // kv head (and pass), then the request, then the partition.  (With the
    // partition fastest and eight partitions, all first partitions -- most of
    // the work -- would land on one XCD.)
    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int hc_count = a.num_kv_heads * passes;
    const long long item = (long long)blockIdx.x * kWaves +
                           __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= (long long)a.max_parts * hc_count * a.batch) return;
    const int hc = (int)(item % hc_count);
    const int r = (int)((item / hc_count) % a.batch);
    const int part = (int)(item / ((long long)hc_count * a.batch));
    const int running = a.running[r];          // both loads are in flight together
    const int C = a.ctx_lens[r];
    if (!running) return;                      // Preserve / Swap / Discard: not in the batch
    const int t_begin = part * a.part_tokens;
    if (t_begin >= C && part != 0) return;     // partition 0 of an empty context writes zeros
    const int t_end = min(C, t_begin + a.part_tokens);
    const int n_parts = max(1, (C + a.part_tokens - 1) / a.part_tokens);
    const int g = hc / passes;
    const int h0 = g * G + (hc % passes) * GH;
    const size_t rh0 = (size_t)r * a.num_q_heads + h0;

    R::run(a, r, g, h0, GH, t_begin, t_end, [&](int h, int d, float M, float L, float A) {
        if (n_parts == 1)
            store_out<R::kBF16>(a.out, (rh0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
        else
            store_partial(a.partials + ((rh0 + h) * a.max_parts + part) * (D + 2), D, d, M, L, A);
    });
}

// Merge of the partitions of one (request, query head), always in partition
// order; block = head_dim threads.
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
    float M = kLowest, L = 0.0f, A = 0.0f;
    for (int p0 = 0; p0 < n_parts; p0 += 8) {         // eight partitions' loads in flight together
        float mo[8], lo[8], ao[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const bool ok = p0 + k < n_parts;
            const float *x = pp + (size_t)(ok ? p0 + k : 0) * (D + 2);
            mo[k] = ok ? x[D] : kLowest;
            lo[k] = ok ? x[D + 1] : 0.0f;
            ao[k] = ok ? x[d] : 0.0f;
        }
        float Mn = M;
#pragma unroll
        for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, mo[k]);
        const float f0 = fast_exp2(M - Mn);
        L *= f0;
        A *= f0;
        M = Mn;
#pragma unroll
        for (int k = 0; k < 8; ++k) {
            const float f = fast_exp2(mo[k] - M);
            L += lo[k] * f;
            A += ao[k] * f;
        }
    }
    store_out<BF16>(a.out, rh * D + d, L > 0.0f ? A / L : 0.0f);
}

// ---------------------------------------------------------------- balanced shares

// Position x of the flat chunk sequence belongs to the share w with
// floor(w * total / P) <= x < floor((w + 1) * total / P).
__device__ __forceinline__ long long share_of(long long x, long long total, int P)
{
    return ((x + 1) * P - 1) / total;
}

// Chunks a running request contributes per (kv head, pass): an empty context
// still gets one (empty) chunk so that its zero row is written.
__device__ __forceinline__ int chunks_of(int running, int C, int CT)
{
    return running ? max(1, (C + CT - 1) / CT) : 0;
}

// gridDim.x * 4 wavefronts, each an equal contiguous share of the flat chunk
// sequence ordered (request, kv head / pass, chunk).  prefix[] (dynamic LDS,
// batch + 1 ints) holds the running chunk count per request; every workgroup
// computes it for itself from ctx_lens / running (a few hundred loads that hit
// in L2), which costs less than a dependent launch.
template <typename R>
__global__ __launch_bounds__(kThreads) void decode_balanced(const DecodeArgs a)
{
    constexpr int D = R::D, CT = R::CT;
    extern __shared__ int prefix[];
    __shared__ int wave_total[kWaves];

    const int B = a.batch;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int per = (B + kThreads - 1) / kThreads;   // consecutive requests per thread
    int mine = 0;
    for (int i = 0; i < per; ++i) {
        const int r = tid * per + i;
        if (r < B) mine += chunks_of(a.running[r], a.ctx_lens[r], CT);
    }
    int incl = mine;                                  // inclusive scan inside the wave
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt *= 2) {
        const int up = __shfl_up(incl, dlt);
        if (lane >= dlt) incl += up;
    }
    if (lane == 63) wave_total[wv] = incl;
    __syncthreads();
    int run = incl - mine;
    for (int ww = 0; ww < wv; ++ww) run += wave_total[ww];
    if (tid == 0) prefix[0] = 0;
    for (int i = 0; i < per; ++i) {
        const int r = tid * per + i;
        if (r < B) {
            run += chunks_of(a.running[r], a.ctx_lens[r], CT);
            prefix[r + 1] = run;
        }
    }
    __syncthreads();

    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int HC = a.num_kv_heads * passes;
    const long long total = (long long)HC * prefix[B];
    // from here on every wave is on its own: no barrier below
    const int share = blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(wv);
    const int P = gridDim.x * kWaves;
    // What the merge kernel needs to know about this share: whether it is empty,
    // and the (request, head) range it starts but does not finish, if any (only
    // its last range can be one): request, head/pass, last share of the range,
    // and the slot this share's piece went to.
    int4 owned = make_int4(0, 0, 0, 0);
    const long long x_begin = (long long)share * total / P;
    const long long x_end = (long long)(share + 1) * total / P;
    if (x_begin >= x_end) {
        if (lane == 0) a.share_info[share] = make_int4(0, 0, 0, kShareEmpty);
        return;
    }

    // request that holds position x_begin: the last r with HC * prefix[r] <= x_begin
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if ((long long)HC * prefix[mid] <= x_begin) lo = mid; else hi = mid;
    }
    int r = __builtin_amdgcn_readfirstlane(lo);
    long long x = x_begin;
    while (x < x_end) {
        const int base = __builtin_amdgcn_readfirstlane(prefix[r]);
        const int nr = __builtin_amdgcn_readfirstlane(prefix[r + 1]) - base;   // > 0 here
        const long long rem = x - (long long)HC * base;
        const int hc = (int)(rem / nr), c0 = (int)(rem % nr);
        const int len = (int)min((long long)(nr - c0), x_end - x);
        const int C = a.ctx_lens[r];
        const int g = hc / passes;
        const int h0 = g * G + (hc % passes) * GH;
        const bool whole = (c0 == 0 && len == nr);
        // a share's first range goes to slot 0, a later partial one (its last) to slot 1
        float *slot = a.partials + ((size_t)share * 2 + (x == x_begin ? 0 : 1)) * GH * (D + 2);
        const size_t rh0 = (size_t)r * a.num_q_heads + h0;
        R::run(a, r, g, h0, GH, c0 * CT, min(C, (c0 + len) * CT),
               [&](int h, int d, float M, float L, float A) {
                   if (whole)
                       store_out<R::kBF16>(a.out, (rh0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
                   else
                       store_partial(slot + (size_t)h * (D + 2), D, d, M, L, A);
               });
        if (c0 == 0 && len < nr)
            owned = make_int4(r, hc, (int)share_of(x + nr - 1, total, P),
                              kShareOwner | (x == x_begin ? 0 : kShareSlot1));
        x += len;
        if (c0 + len == nr && hc == HC - 1) {         // request finished: next one with work
            ++r;
            while (r < B && prefix[r + 1] == prefix[r]) ++r;
        }
    }
    if (lane == 0) a.share_info[share] = owned;
}

// Merges the pieces of every (request, kv head / pass) that was split over
// several shares, in share order (= token order).  One block per share and slice
// of 256 (head, dim) outputs: the share that holds the start of a split range
// merges it (most blocks find nothing to do and leave after one load).
template <bool BF16>
__global__ __launch_bounds__(256) void decode_merge_balanced(const DecodeArgs a)
{
    const int4 owned = a.share_info[blockIdx.x];
    if (!(owned.w & kShareOwner)) return;
    const int r = owned.x, hc = owned.y;
    const int D = a.head_dim;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int w_first = blockIdx.x, w_last = owned.z;
    const int g = hc / passes;
    const size_t rh0 = (size_t)r * a.num_q_heads + g * G + (hc % passes) * GH;
    const int idx = blockIdx.y * 256 + threadIdx.x;
    const bool live = idx < GH * D;
    const int h = live ? idx / D : 0, d = live ? idx % D : 0;
    // The pieces' slots are looked up once per block, kMergeList at a time; each list
    // is then reduced eight pieces at a time.
    __shared__ int piece[kMergeList];
    float M = kLowest, L = 0.0f, A = 0.0f;
    for (int w0 = w_first; w0 <= w_last; w0 += kMergeList) {
        const int cnt = min(kMergeList, w_last - w0 + 1);
        __syncthreads();
        if ((int)threadIdx.x < cnt) {
            const int w = w0 + threadIdx.x;        // the first share knows its slot; later ones start
            const int f = w == w_first ? owned.w : a.share_info[w].w;   // inside the range: slot 0
            piece[threadIdx.x] = (f & kShareEmpty) ? -1 : w * 2 + ((w == w_first && (f & kShareSlot1)) ? 1 : 0);
        }
        __syncthreads();
        for (int i0 = 0; i0 < cnt; i0 += 8) {          // share order = token order
            float mo[8], lo[8], ao[8];                 // eight pieces' loads in flight together
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const int pc = i0 + k < cnt ? piece[i0 + k] : -1;
                const float *x = a.partials + ((size_t)max(pc, 0) * GH + h) * (D + 2);
                mo[k] = pc >= 0 ? x[D] : kLowest;
                lo[k] = pc >= 0 ? x[D + 1] : 0.0f;
                ao[k] = pc >= 0 ? x[d] : 0.0f;
            }
            float Mn = M;
#pragma unroll
            for (int k = 0; k < 8; ++k) Mn = fmaxf(Mn, mo[k]);
            const float f0 = fast_exp2(M - Mn);
            L *= f0;
            A *= f0;
            M = Mn;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                const float f = fast_exp2(mo[k] - M);
                L += lo[k] * f;
                A += ao[k] * f;
            }
        }
    }
    if (live) store_out<BF16>(a.out, (rh0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
}

// ---------------------------------------------------------------- launchers

template <typename R>
hipError_t launch_one(const DecodeArgs &a, hipStream_t s)
{
    const int G = a.num_q_heads / a.num_kv_heads;
    const int HC = a.num_kv_heads * (G / a.heads_per_pass);
    if (a.part_tokens > 0) {
        const long long items = (long long)a.max_parts * HC * a.batch;
        dim3 grid((unsigned)((items + kWaves - 1) / kWaves));
        hipLaunchKernelGGL(decode_partial<R>, grid, dim3(kThreads), 0, s, a);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess || a.max_parts == 1) return e;
        hipLaunchKernelGGL(decode_merge<R::kBF16>, dim3(a.num_q_heads, a.batch), dim3(a.head_dim), 0,
                           s, a);
        return hipGetLastError();
    }
    // balanced: as many workgroups as the chip holds at once for this kernel (fewer
    // if the partial slots of that many wave shares would not fit the workspace)
    static int resident = 0;                          // per instantiation; one device per process
    if (resident == 0) {
        int dev = 0, cus = 0, per_cu = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e == hipSuccess) e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_balanced<R>, kThreads,
                                                             (a.max_batch + 1) * sizeof(int));
        if (e != hipSuccess) return e;
        if (cus < 1 || per_cu < 1) return hipErrorInvalidValue;
        resident = cus * per_cu;
    }
    const int wgs = min(resident, decode_max_shares(a.heads_per_pass, a.head_dim) / kWaves);
    const size_t lds = (size_t)(a.batch + 1) * sizeof(int);
    hipLaunchKernelGGL(decode_balanced<R>, dim3(wgs), dim3(kThreads), lds, s, a);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const int slices = (a.heads_per_pass * a.head_dim + 255) / 256;
    hipLaunchKernelGGL(decode_merge_balanced<R::kBF16>, dim3(wgs * kWaves, slices), dim3(256), 0, s, a);
    return hipGetLastError();
}

template <bool BF16, int LPT>
hipError_t launch_valu(const DecodeArgs &a, hipStream_t s)
{
    switch (a.heads_per_pass) {
    case 1: return launch_one<ValuReducer<BF16, LPT, 1, kHalves>>(a, s);
    case 2:
        if constexpr (!BF16) return launch_one<ValuReducer<BF16, LPT, 2, kHalves>>(a, s);
        break;                                 // grouped bf16 heads take the MFMA path
    case 4:
        if constexpr (!BF16) return launch_one<ValuReducer<BF16, LPT, 4, 1>>(a, s);
        break;
    }
    return hipErrorInvalidValue;
}

template <int D>
hipError_t launch_mfma(const DecodeArgs &a, hipStream_t s)
{
    if (a.heads_per_pass > 16) return hipErrorInvalidValue;
    return launch_one<MfmaReducer<D>>(a, s);
}

}  // namespace

int decode_uses_tiled_layout(int bf16, int group) { return bf16 && group >= 2; }

int decode_heads_per_pass(int bf16, int head_dim, int group)
{
    const int lpt = head_dim * (bf16 ? 2 : 4) / 16;
    if (head_dim * (bf16 ? 2 : 4) % 16 != 0 || (lpt != 8 && lpt != 16 && lpt != 32)) return 0;
    if (group <= 0) return 0;
    if (decode_uses_tiled_layout(bf16, group)) {      // MFMA path: the largest divisor <= 16
        for (int gh = 16; gh >= 1; --gh)
            if (group % gh == 0) return gh;
    }
    if (group % 4 == 0) return 4;
    if (group % 2 == 0) return 2;
    return 1;
}

int decode_max_shares(int heads_per_pass, int head_dim)
{
    const size_t per_share = (size_t)2 * heads_per_pass * (head_dim + 2) * sizeof(float);
    size_t n = kPartialBudget / per_share;
    if (n > (size_t)kMaxShares) n = kMaxShares;
    return (int)(n / kWaves) * kWaves;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    const int G = a.num_q_heads / a.num_kv_heads;
    if (a.heads_per_pass != decode_heads_per_pass(a.bf16, a.head_dim, G) || a.heads_per_pass == 0)
        return hipErrorInvalidValue;
    const int lpt = a.head_dim * (a.bf16 ? 2 : 4) / 16;
    if (decode_uses_tiled_layout(a.bf16, G)) {
        if (a.head_dim == 64) return launch_mfma<64>(a, stream);
        if (a.head_dim == 128) return launch_mfma<128>(a, stream);
        if (a.head_dim == 256) return launch_mfma<256>(a, stream);
    } else if (a.bf16) {
        if (lpt == 8) return launch_valu<true, 8>(a, stream);
        if (lpt == 16) return launch_valu<true, 16>(a, stream);
        if (lpt == 32) return launch_valu<true, 32>(a, stream);
    } else {
        if (lpt == 8) return launch_valu<false, 8>(a, stream);
        if (lpt == 16) return launch_valu<false, 16>(a, stream);
        if (lpt == 32) return launch_valu<false, 32>(a, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace lamps
