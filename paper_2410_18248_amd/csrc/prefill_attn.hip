// Attention for several new tokens per request over the paged cache: what the
// Discard strategy's recompute, a new request's prompt and the processing of
// an API response need (arXiv 2410.18248, Section 1, Section 4.2: "Discard and
// Recompute"; Section 2.2 equation per token, each token over the cached
// positions up to and including its own).  The keys and values of the new
// tokens are already in the cache (lamps_kv_append_tokens).
#include <hip/hip_runtime.h>

#include "attn_reducers.h"
#include "internal.h"

namespace lamps {
namespace {

// Last request r with q_start[r] <= n.
__device__ __forceinline__ int request_of(const int32_t *q_start, int batch, int n)
{
    int lo = 0, hi = batch;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (q_start[mid] <= n) lo = mid; else hi = mid;
    }
    return lo;
}

// One wavefront per (new token, kv head / pass): the decode reducer over the
// token's own prefix.  Every K/V byte is read once per new token, so this form
// is for few new tokens per request and for the geometries the matrix-core
// kernel does not cover.
template <typename R>
__global__ __launch_bounds__(kThreads) void prefill_rows(const PrefillArgs p)
{
    constexpr int D = R::D;
    const DecodeArgs &a = p.d;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int hc_count = a.num_kv_heads * passes;
    const long long item = (long long)blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (item >= (long long)p.total_tokens * hc_count) return;
    const int hc = (int)(item % hc_count);
    const int n = (int)(item / hc_count);
    const int r = __builtin_amdgcn_readfirstlane(request_of(p.q_start, a.batch, n));
    const int first = p.q_start[r], count = p.q_start[r + 1] - first;
    if (n >= first + count) return;
    const int t_end = a.ctx_lens[r] - count + (n - first) + 1;     // its own position included
    const int g = hc / passes;
    const int h0 = g * G + (hc % passes) * GH;
    const size_t row0 = (size_t)n * a.num_q_heads + h0;
    R::run(a, r, (size_t)n, g, h0, GH, 0, max(t_end, 0), [&](int h, int d, float M, float L, float A) {
        store_out<R::kBF16>(a.out, (row0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
    });
}

// ---------------------------------------------------------------- matrix cores

// bf16, up to 64 query heads per kv head.  With many new tokens per request both
// products of the Section 2.2 equation are real contractions: for one kv head,
// the (token, head-of-group) pairs are the columns of a query matrix, and every
// 32 cached positions cost 2 D/32 + D/16 MFMAs (16x16x32) per 16 columns.
//
// One workgroup = one (request, kv head, tile of new tokens); its four waves each
// own kCols = 32 columns (kCols / G tokens x G heads) as blocks of 16.  K and V
// are streamed 32 positions at a time: all 256 threads load the next stage from
// the paged pools into registers while the current one, in LDS, is consumed;
// every wave reads each K / V operand from LDS once per stage and uses it for
// its four column blocks.  Scores come out transposed (lane: four consecutive
// positions of one column), which is the operand layout the second product
// wants for the weights, so nothing is shuffled between the two; the positions of
// a stage's two 16-position halves share one 32-deep MFMA (the contraction index
// may be permuted as long as both operands agree).
//
// LDS holds the pool tiles as they are for the tiled layout (16-byte runs are
// operands already).  For the plain layout K rows are padded by 16 bytes so that
// the 16 rows of a K operand fall in different banks, and V -- whose row-major
// order would need a transposition at every operand read -- is scattered into
// the tiled order once, 16 bits at a time, when the stage is written to LDS.
constexpr int kMaxCols = 32;             // columns per wave: two blocks of 16 keep a wave under 256 registers,
                                         // so two workgroups share a CU and cover each other's stalls
constexpr int kStage = 32;               // cached positions per LDS stage
constexpr float kSlack = 8.0f;           // log2 of the largest weight before the reference moves

typedef __attribute__((ext_vector_type(8))) unsigned short u16x8;

template <int D, bool TILED, int kCols>
__global__ __launch_bounds__(kThreads) void prefill_mfma(const PrefillArgs p)
{
    constexpr int kColBlocks = kCols / 16;
    constexpr int NK = D / 32;                       // score MFMAs per 16 positions
    constexpr int NS = D / 16;                       // 16-dim slabs of the output
    constexpr int U = D * 2;                         // 16-byte units of one 16-position sub-tile
    constexpr int LPT = (2 * U) / kThreads;          // units per thread, pool and stage
    constexpr int ROWB = D * 2 + 16;                 // plain layout: padded row, bytes
    constexpr int SUBB = TILED ? 16 * D * 2 : 16 * ROWB;   // K sub-tile in LDS
    // V sub-tile in LDS: always the tiled order, each 1 KiB group of 32 dims shifted by 16
    // bytes so that the scattered 16-bit writes of the plain layout spread over the banks
    constexpr int SUBV = 16 * D * 2 + (D / 32) * 16;
    static_assert(LPT >= 1 && (2 * U) % kThreads == 0, "head_dim");
    __shared__ __align__(16) char lds_k[2 * SUBB];
    __shared__ __align__(16) char lds_v[2 * SUBV];

    const DecodeArgs &a = p.d;
    const int r = blockIdx.z, g = blockIdx.y;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int TW = kCols / G;                        // new tokens per wave (G <= kCols)
    const int WT = kWaves * TW;                      // ... per workgroup
    const int first = p.q_start[r], n_new = p.q_start[r + 1] - first;
    const int tile = gridDim.x - 1 - blockIdx.x;     // the longest tiles start first
    if (tile * WT >= n_new) return;
    const int C = a.ctx_lens[r];
    const int base_pos = C - n_new;                  // position of the request's first new token
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int j = lane & 15, qd = lane >> 4;

    // this lane's column in each block: (token, head), its position, its q slices
    int pos[kColBlocks];                             // -1: no such column
    size_t orow[kColBlocks];                         // element offset of its output row
    bf16x8 qb[kColBlocks][NK];
    int wave_maxpos = -1, wave_minpos = 0x7fffffff;  // over the wave's valid columns
#pragma unroll
    for (int b = 0; b < kColBlocks; ++b) {
        const int c = b * 16 + j;
        const int tl = c / G, hd = c - tl * G;
        const int tok = tile * WT + wv * TW + tl;
        const bool ok = c < TW * G && tok < n_new;
        pos[b] = ok ? base_pos + tok : -1;
        orow[b] = ((size_t)(first + (ok ? tok : 0)) * a.num_q_heads + g * G + hd) * D;
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            uint4 t = make_uint4(0, 0, 0, 0);
            if (ok) t = *reinterpret_cast<const uint4 *>(static_cast<const char *>(a.q) + (orow[b] + 32 * i + 8 * qd) * 2);
            qb[b][i] = __builtin_bit_cast(bf16x8, t);
        }
        wave_maxpos = max(wave_maxpos, pos[b]);
        if (ok) wave_minpos = min(wave_minpos, pos[b]);
    }
#pragma unroll
    for (int dlt = 32; dlt >= 1; dlt >>= 1) {
        wave_maxpos = max(wave_maxpos, __shfl_xor(wave_maxpos, dlt));
        wave_minpos = min(wave_minpos, __shfl_xor(wave_minpos, dlt));
    }
    const int wg_maxpos = base_pos + min(n_new, (tile + 1) * WT) - 1;
    const int n_stages = wg_maxpos / kStage + 1;

    float m[kColBlocks], l[kColBlocks];
    f32x4 o[kColBlocks][NS];                          // out^T: dims 16 s + 4 qd + e, this lane's column
#pragma unroll
    for (int b = 0; b < kColBlocks; ++b) {
        m[b] = kLowest;
        l[b] = 0.0f;
#pragma unroll
        for (int s = 0; s < NS; ++s) o[b][s] = f32x4{0.f, 0.f, 0.f, 0.f};
    }

    const int32_t *table = a.block_table + (size_t)r * a.max_blocks;
    const size_t tile_bytes = (size_t)a.block_size * D * 2;
    const size_t block_stride = (size_t)a.num_layers * a.num_kv_heads * tile_bytes;
    const size_t head_off = ((size_t)a.layer * a.num_kv_heads + g) * tile_bytes;
    const char *kp = static_cast<const char *>(a.k_pool) + head_off;
    const char *vp = static_cast<const char *>(a.v_pool) + head_off;

    // stage st -> registers: unit x of the stage is sub-tile x / U, 16-byte unit x % U of it
    uint4 kreg[LPT], vreg[LPT];
    auto fetch = [&](int st) {
#pragma unroll
        for (int k = 0; k < LPT; ++k) {
            const int x = tid + kThreads * k;
            const int t = st * kStage + 16 * (x / U);
            kreg[k] = vreg[k] = make_uint4(0, 0, 0, 0);
            if (st < n_stages && t <= wg_maxpos) {
                const size_t off = (size_t)table[t >> a.log2_block_size] * block_stride +
                                   (size_t)((t & (a.block_size - 1)) >> 4) * (16 * D * 2) + (size_t)(x % U) * 16;
                kreg[k] = *reinterpret_cast<const uint4 *>(kp + off);
                vreg[k] = *reinterpret_cast<const uint4 *>(vp + off);
            }
        }
    };
    // registers -> LDS; value slots at or past the context's end are zeroed (they may hold
    // anything, and a zero weight does not silence a NaN)
    auto stash = [&](int st) {
#pragma unroll
        for (int k = 0; k < LPT; ++k) {
            const int x = tid + kThreads * k;
            const int u = x / U, unit = x % U;
            const int t = st * kStage + 16 * u;
            uint4 v = vreg[k];
            if (TILED) {
                const size_t where = (size_t)u * SUBB + (size_t)unit * 16;
                const int valid = C - (t + 4 * ((unit >> 4) & 3));     // of the unit's four positions
                if (valid < 4) {
                    const uint32_t m01 = valid >= 2 ? 0xFFFFFFFFu : (valid == 1 ? 0x0000FFFFu : 0u);
                    const uint32_t m23 = valid >= 4 ? 0xFFFFFFFFu : (valid == 3 ? 0x0000FFFFu : 0u);
                    v.x &= m01; v.z &= m01;
                    v.y &= m23; v.w &= m23;
                }
                *reinterpret_cast<uint4 *>(lds_k + where) = kreg[k];
                *reinterpret_cast<uint4 *>(lds_v + (size_t)u * SUBV + (size_t)unit * 16 + (size_t)(unit >> 6) * 16) = v;
            } else {
                const int row = unit / (D / 8), c16 = unit % (D / 8);     // position t + row, dims 8 c16 ..
                *reinterpret_cast<uint4 *>(lds_k + (size_t)u * SUBB + (size_t)row * ROWB + (size_t)c16 * 16) = kreg[k];
                if (t + row >= C) v = make_uint4(0, 0, 0, 0);
                const uint32_t w[4] = {v.x, v.y, v.z, v.w};
                // element (row, d) of the sub-tile goes where the tiled layout of lamps.h puts it
                uint16_t *dst = reinterpret_cast<uint16_t *>(lds_v + (size_t)u * SUBV);
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int d = 8 * c16 + e;
                    const int at = ((((d >> 5) * 4 + (row >> 2)) * 16 + (d & 15)) * 2 + ((d & 31) >> 4)) * 4 + (row & 3) +
                                   (d >> 5) * 8;
                    dst[at] = (uint16_t)(w[e >> 1] >> (16 * (e & 1)));
                }
            }
        }
    };

    fetch(0);
    for (int st = 0; st < n_stages; ++st) {
        __syncthreads();                              // everyone is done with the previous stage
        stash(st);
        __syncthreads();
        fetch(st + 1);                                // in flight while this stage is consumed
        const int t0 = st * kStage;
        if (t0 > wave_maxpos) continue;               // wave-uniform: nothing here for this wave's columns

        // Operand-major order: every K / V operand is read from LDS once and used at once
        // for all column blocks (independent MFMAs back to back, few operand registers
        // alive), so the accumulators can stay in the accumulation registers for the
        // whole loop and only the scores and weights pass through the vector ALUs.
        f32x4 sc0[kColBlocks], sc1[kColBlocks];        // positions t0 (+16) + 4 qd + e of the lane's column
#pragma unroll
        for (int b = 0; b < kColBlocks; ++b) sc0[b] = sc1[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NK; ++i) {
            // K rows: position t0 + 16 u + j, dims 32 i + 8 qd ..
            const size_t where = TILED ? (size_t)((4 * i + qd) * 16 + j) * 16
                                       : (size_t)j * ROWB + (size_t)(32 * i + 8 * qd) * 2;
            const bf16x8 k0 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(lds_k + where));
            const bf16x8 k1 = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(lds_k + SUBB + where));
#pragma unroll
            for (int b = 0; b < kColBlocks; ++b) {
                sc0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k0, qb[b][i], sc0[b], 0, 0, 0);
                sc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(k1, qb[b][i], sc1[b], 0, 0, 0);
            }
        }

        bf16x8 pw[kColBlocks];                         // weights, transposed: the second product's operand
        const bool all_visible = t0 + kStage - 1 <= wave_minpos;   // wave-uniform
#pragma unroll
        for (int b = 0; b < kColBlocks; ++b) {
            float sc[8];                              // raw scores; scale_log2e > 0 is applied in the exponent
            float mx = -INFINITY;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float x = e < 4 ? sc0[b][e] : sc1[b][e - 4];
                const int t = t0 + 16 * (e >> 2) + 4 * qd + (e & 3);
                sc[e] = (all_visible || t <= pos[b]) ? x : -INFINITY;   // a token sees the positions up to its own
                mx = fmaxf(mx, sc[e]);
            }
            mx *= a.scale_log2e;
            // The reference point of the exponentials follows the running maximum lazily:
            // it moves only when a score exceeds it by more than kSlack, so weights stay
            // below 2^kSlack, the four lanes that share a column compare notes only then,
            // and the accumulators (which live in accumulation registers the vector ALUs
            // cannot touch without moving them) are rescaled a handful of times per column.
            float f = 1.0f;
            if (__any(mx - m[b] > kSlack)) {          // wave-uniform, rare after the first stages
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float mn = mx - m[b] > kSlack ? mx : m[b];
                f = fast_exp2(m[b] - mn);
                m[b] = mn;
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[b][s][e] *= f;
            }
            const float mn = m[b];
            float ps = 0.0f;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const float w = fast_exp2(fmaf(sc[e], a.scale_log2e, -mn));
                ps += w;
                pw[b][e] = (__bf16)w;
            }
            l[b] = l[b] * f + ps;
        }

#pragma unroll
        for (int i = 0; i < NS / 2; ++i) {
            // V^T rows: dims 32 i + j (x, y) and 32 i + 16 + j (z, w), positions 4 qd .. of each half
            const size_t where = (size_t)((i * 4 + qd) * 16 + j) * 16 + (size_t)i * 16;
            const uint4 v0 = *reinterpret_cast<const uint4 *>(lds_v + where);
            const uint4 v1 = *reinterpret_cast<const uint4 *>(lds_v + SUBV + where);
            const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4(v0.x, v0.y, v1.x, v1.y));
            const bf16x8 vb = __builtin_bit_cast(bf16x8, make_uint4(v0.z, v0.w, v1.z, v1.w));
#pragma unroll
            for (int b = 0; b < kColBlocks; ++b) {
                o[b][2 * i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, pw[b], o[b][2 * i], 0, 0, 0);
                o[b][2 * i + 1] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vb, pw[b], o[b][2 * i + 1], 0, 0, 0);
            }
        }
    }

#pragma unroll
    for (int b = 0; b < kColBlocks; ++b) {
        float lt = l[b];                              // kept per position group: add the four
        lt += __shfl_xor(lt, 16);
        lt += __shfl_xor(lt, 32);
        if (pos[b] < 0) continue;
        const float inv = lt > 0.0f ? 1.0f / lt : 0.0f;
        uint16_t *dst = static_cast<uint16_t *>(a.out) + orow[b];
#pragma unroll
        for (int s = 0; s < NS; ++s) {
            uint2 w;
            w.x = (uint32_t)to_bf16_rne(o[b][s][0] * inv) | ((uint32_t)to_bf16_rne(o[b][s][1] * inv) << 16);
            w.y = (uint32_t)to_bf16_rne(o[b][s][2] * inv) | ((uint32_t)to_bf16_rne(o[b][s][3] * inv) << 16);
            *reinterpret_cast<uint2 *>(dst + 16 * s + 4 * qd) = w;
        }
    }
}

template <int D, bool TILED>
hipError_t launch_mfma_prefill(const PrefillArgs &p, hipStream_t s)
{
    constexpr int kCols = kMaxCols;
    const int G = p.d.num_q_heads / p.d.num_kv_heads;
    const int WT = kWaves * (kCols / G);
    const int tiles = (p.max_new_tokens + WT - 1) / WT;
    if (tiles < 1 || p.d.num_kv_heads > 65535 || p.d.batch > 65535) return hipErrorInvalidValue;
    hipLaunchKernelGGL((prefill_mfma<D, TILED, kCols>), dim3((unsigned)tiles, (unsigned)p.d.num_kv_heads, (unsigned)p.d.batch),
                       dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

template <typename R>
hipError_t launch_rows(const PrefillArgs &p, hipStream_t s)
{
    const int G = p.d.num_q_heads / p.d.num_kv_heads;
    const long long items = (long long)p.total_tokens * p.d.num_kv_heads * (G / p.d.heads_per_pass);
    if (items > 0x7fffffffLL * kWaves) return hipErrorInvalidValue;
    hipLaunchKernelGGL(prefill_rows<R>, dim3((unsigned)((items + kWaves - 1) / kWaves)), dim3(kThreads), 0, s, p);
    return hipGetLastError();
}

template <bool BF16, int LPT>
hipError_t launch_rows_valu(const PrefillArgs &p, hipStream_t s)
{
    switch (p.d.heads_per_pass) {
    case 1: return launch_rows<ValuReducer<BF16, LPT, 1, kHalves>>(p, s);
    case 2:
        if constexpr (!BF16) return launch_rows<ValuReducer<BF16, LPT, 2, kHalves>>(p, s);
        break;
    case 4:
        if constexpr (!BF16) return launch_rows<ValuReducer<BF16, LPT, 4, 1>>(p, s);
        break;
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t launch_prefill(const PrefillArgs &p, hipStream_t stream)
{
    const DecodeArgs &a = p.d;
    if (a.batch == 0 || p.total_tokens == 0) return hipSuccess;
    const int G = a.num_q_heads / a.num_kv_heads;
    if (a.heads_per_pass != decode_heads_per_pass(a.bf16, a.head_dim, G) || a.heads_per_pass == 0)
        return hipErrorInvalidValue;
    const int lpt = a.head_dim * (a.bf16 ? 2 : 4) / 16;
    if (a.bf16 && G <= kMaxCols && !p.force_rows) {     // matrix cores
        const bool tiled = decode_uses_tiled_layout(a.bf16, G);
        if (a.head_dim == 64) return tiled ? launch_mfma_prefill<64, true>(p, stream) : launch_mfma_prefill<64, false>(p, stream);
        if (a.head_dim == 128) return tiled ? launch_mfma_prefill<128, true>(p, stream) : launch_mfma_prefill<128, false>(p, stream);
        if (a.head_dim == 256) return tiled ? launch_mfma_prefill<256, true>(p, stream) : launch_mfma_prefill<256, false>(p, stream);
    }
    if (decode_uses_tiled_layout(a.bf16, G)) {
        if (a.heads_per_pass > 16) return hipErrorInvalidValue;
        if (a.head_dim == 64) return launch_rows<MfmaReducer<64>>(p, stream);
        if (a.head_dim == 128) return launch_rows<MfmaReducer<128>>(p, stream);
        if (a.head_dim == 256) return launch_rows<MfmaReducer<256>>(p, stream);
    } else if (a.bf16) {
        if (lpt == 8) return launch_rows_valu<true, 8>(p, stream);
        if (lpt == 16) return launch_rows_valu<true, 16>(p, stream);
        if (lpt == 32) return launch_rows_valu<true, 32>(p, stream);
    } else {
        if (lpt == 8) return launch_rows_valu<false, 8>(p, stream);
        if (lpt == 16) return launch_rows_valu<false, 16>(p, stream);
        if (lpt == 32) return launch_rows_valu<false, 32>(p, stream);
    }
    return hipErrorInvalidValue;
}

}  // namespace lamps
