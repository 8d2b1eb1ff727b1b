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
    const int C = a.ctx_lens[r];
    // a context shorter than its new tokens, or longer than the block-table row, is the caller's
    // mistake: nothing is read or written for it
    if (C - count < 0 || C > a.max_blocks * a.block_size) return;
    const int t_end = C - count + (n - first) + 1;    // its own position included
    const int g = hc / passes;
    const int h0 = g * G + (hc % passes) * GH;
    const size_t row0 = (size_t)n * a.num_q_heads + h0;
    R::run(a, r, (size_t)n, g, h0, GH, 0, max(t_end, 0), [&](int h, int d, float M, float L, float A) {
        store_out<R::kBF16>(a.out, (row0 + h) * D + d, L > 0.0f ? A / L : 0.0f);
    });
}

// ---------------------------------------------------------------- matrix cores

// bf16, up to 32 query heads per kv head.  With many new tokens per request both
// products of the Section 2.2 equation are real contractions: for one kv head,
// the (token, head-of-group) pairs are the columns of a query matrix, and every
// 32 cached positions cost 2 D/32 + D/16 + 1 MFMAs (16x16x32) per 16 columns.
//
// One workgroup = one (request, kv head, tile of new tokens); its four waves each
// own kCols = 32 columns (kCols / G tokens x G heads) as blocks of 16.  K and V
// are streamed 32 positions at a time through LDS: while stage s is consumed,
// stage s + 1 arrives in the other of two LDS buffers, straight from the pools (loads
// that write LDS directly: no registers, no LDS-write instructions), one barrier
// per stage -- or per two stages, loaded and published together, when a request has
// several tiles of new tokens and two such groups fit the 64 KiB of a workgroup.  Every wave reads each K / V operand from LDS
// once per stage and uses it for both column blocks.  Scores come out transposed
// (lane: four consecutive positions of one column), which is the operand layout
// the second product wants for the weights, so nothing is shuffled between the
// two; the positions of a stage's two 16-position halves share one 32-deep MFMA
// (the contraction index may be permuted as long as both operands agree).
//
// The loop is software-pipelined around its one barrier: a stage's V operands are
// read from LDS before its scores are computed and used after the barrier, the
// next stage's K operands are read right after the barrier and used at the top of
// the next iteration, so LDS latency is behind MFMA or softmax work both times.
//
// The vector ALUs are the scarce unit (an exponential costs as much issue time as
// a quarter of an MFMA), so everything that is not the softmax itself is kept off
// them: block-table entries are looked up one stage ahead through the scalar
// unit, the causal mask is applied only in the stages that straddle a column's own
// position, the weights' sums come from one more MFMA against a vector of ones
// (they accumulate, like the outputs, in registers and need no cross-lane sum at
// the end), and V reaches the second product without any shuffling in registers.
//
// LDS layouts of a stage: the pools' tiles as they are.  Tiled pool layout: a K unit
// is an operand already, a V operand is the first or the second 8 bytes of the same
// unit of the stage's two sub-tiles.  Plain layout: K and V row-major; rows cannot
// be padded on the way in, so the 16-byte units of a row are permuted instead (unit
// s of row r sits in slot s ^ r, or s ^ 2 r for V) and the rows an operand read
// touches fall in different banks; V^T operands come out of the transposing LDS
// read of gfx950 (ds_read_b64_tr_b16: the 16 lanes of a group read four rows of 16
// dims, lane j receives dim j of the four rows).
constexpr int kMaxCols = 32;             // columns per wave: two blocks of 16 keep a wave under 256 registers,
                                         // so two workgroups share a CU and cover each other's stalls
constexpr int kStage = 32;               // cached positions per LDS stage
constexpr float kSlack = 8.0f;           // log2 of the largest weight before the reference moves

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((address_space(4))) const int32_t *table_ptr;   // read-only: scalar loads

template <int D, bool TILED, int kCols, int GRP>
__global__ __launch_bounds__(kThreads, (D >= 256 && kCols <= 16) ? 2 : 1) void prefill_mfma(const PrefillArgs p, const int tiles, const int full_groups)
{
    constexpr int kColBlocks = kCols / 16;
    constexpr int NK = D / 32;                       // score MFMAs per 16 positions
    constexpr int NS = D / 16;                       // 16-dim slabs of the output
    constexpr int U = D * 2;                         // 16-byte units of one 16-position sub-tile
    constexpr int LPT = (2 * U) / kThreads;          // units per thread, pool and stage
    // The pool's tiles go to LDS as they are, by loads that write LDS directly
    // (global_load_lds_dwordx4: lane l of a wave writes 16 bytes at base + 16 l, read from any
    // address); two stage buffers (64 KiB at head_dim 256).
    constexpr int NB = 2;                            // stage buffers
    constexpr int NU = D / 8;                        // 16-byte units of one row (plain layout)
    constexpr int SUBB = 16 * D * 2;                 // one 16-position sub-tile of K or V
    constexpr int VOFF = 2 * SUBB;                   // V follows the two K sub-tiles
    constexpr int STAGE = 4 * SUBB;
    // Stages are loaded, and published by a barrier, GRP at a time: with two, half as many
    // barriers and waits for loads, and a group's loads have twice as long to arrive.
    constexpr int GSTAGE = GRP * STAGE;
    static_assert(NB * GSTAGE <= 65536, "LDS of one workgroup");
    static_assert(LPT >= 1 && (2 * U) % kThreads == 0, "head_dim");
    __shared__ __align__(16) char lds[NB * GSTAGE];

    const DecodeArgs &a = p.d;
    // All tiles of one (request, kv head) run on one XCD (workgroups are dealt to the 8 XCDs
    // round-robin in launch order), so its K/V stream is fetched into one L2 and shared there;
    // consecutive kv heads go to different XCDs; the longest tiles of a pair start first.  That
    // holds for the pairs that fill whole groups of 8; the (pair, tile) items of the remaining
    // 1..7 pairs are dealt round-robin over all XCDs instead of leaving some of them empty.
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int pairs = a.num_kv_heads * a.batch;
    int pair, t;
    if (slot < full_groups * tiles) {
        pair = xcd + 8 * (slot / tiles);
        t = slot % tiles;
    } else {
        const int rest = pairs - 8 * full_groups;    // 1..7 here: the grid has no such slots otherwise
        const int item = (slot - full_groups * tiles) * 8 + xcd;
        pair = 8 * full_groups + item % rest;
        t = item / rest;
        if (t >= tiles) return;
    }
    const int tile = tiles - 1 - t;
    const int r = pair / a.num_kv_heads, g = pair - r * a.num_kv_heads;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int TW = kCols / G;                        // new tokens per wave (G <= kCols)
    const int WT = kWaves * TW;                      // ... per workgroup
    const int first = p.q_start[r], n_new = p.q_start[r + 1] - first;
    if (tile * WT >= n_new) return;
    const int C = a.ctx_lens[r];
    const int base_pos = C - n_new;                  // position of the request's first new token
    // a context shorter than its new tokens, or longer than the block-table row, is the caller's
    // mistake: nothing is read or written for it
    if (base_pos < 0 || C > a.max_blocks * a.block_size) return;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    wave_maxpos = __builtin_amdgcn_readfirstlane(wave_maxpos);
    wave_minpos = __builtin_amdgcn_readfirstlane(wave_minpos);
    const int wg_maxpos = base_pos + min(n_new, (tile + 1) * WT) - 1;
    const int n_stages = wg_maxpos / kStage + 1;

    float m[kColBlocks];
    f32x4 o[kColBlocks][NS];                          // out^T: dims 16 s + 4 qd + e, this lane's column
    f32x4 l[kColBlocks];                              // the column's sum of weights, four copies
#pragma unroll
    for (int b = 0; b < kColBlocks; ++b) {
        m[b] = kLowest;
        l[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < NS; ++s) o[b][s] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
    const bf16x8 ones = __builtin_bit_cast(bf16x8, make_uint4(0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u));

    const table_ptr table = (table_ptr)(uintptr_t)(a.block_table + (size_t)r * a.max_blocks);
    const uint32_t tile_bytes = (uint32_t)a.block_size * D * 2;
    // bytes from one block to the next; the launcher has checked that they fit 32 bits
    const uint32_t block_stride = (uint32_t)a.num_layers * a.num_kv_heads * tile_bytes;
    const size_t head_off = ((size_t)a.layer * a.num_kv_heads + g) * tile_bytes;
    const char *kp = static_cast<const char *>(a.k_pool) + head_off;
    const char *vp = static_cast<const char *>(a.v_pool) + head_off;

    // Block-table entries of a group's sub-tiles: wave-uniform, through the scalar unit, and
    // looked up one iteration before the loads that use them so that nobody waits for them.
    uint32_t ent[2 * GRP];
    const uint32_t last_entry = (uint32_t)wg_maxpos >> a.log2_block_size;   // nothing past it is looked up
    const uint32_t last_block = (uint32_t)a.num_blocks - 1;
    auto lookup = [&](int grp) {
        const uint32_t t0 = (uint32_t)(grp * GRP * kStage);
#pragma unroll
        for (int i = 0; i < 2 * GRP; ++i)               // (an entry that names no block of the pool is the caller's
            ent[i] = min((uint32_t)table[min((t0 + 16 * i) >> a.log2_block_size, last_entry)], last_block);   // mistake: it reads the last block instead of memory outside the pools)
    };
    // This lane's part of a load's address: unit x of a sub-tile as it lies in the pool goes to
    // LDS slot x (tiled layout), or, plain layout (rows of NU units, which cannot be padded on the
    // way in), slot s of row r takes unit s ^ (r mod NU) of a K row and s ^ (2 r mod NU) of a V
    // row, so that the rows an operand read touches fall in different banks.
    uint32_t lane_k[LPT], lane_v[LPT];
#pragma unroll
    for (int k = 0; k < LPT; ++k) {
        const int x = (kThreads * k + 64 * wv) % U + lane;   // the lane's LDS slot within the sub-tile
        const int row = x / NU, sl = x % NU;
        lane_k[k] = (uint32_t)(TILED ? x : row * NU + (sl ^ (row & (NU - 1)))) * 16;
        lane_v[k] = (uint32_t)(TILED ? x : row * NU + (sl ^ ((2 * row) & (NU - 1)))) * 16;
    }
    // The stage's tiles from the pools straight into LDS buffer `buf`, each wave instruction one
    // run of 64 units (1 KiB).  Sub-tiles past the workgroup's last position are not loaded (LDS is
    // cleared once at the start, and every column's weight for those positions is zero).  Nothing
    // waits here: the caller waits for vmcnt before the barrier that publishes the stage.
    // The address is a scalar base (pool + block + sub-tile, all on the scalar unit, 32 x 32 -> 64
    // bit) plus the lane's constant 32-bit offset: no vector arithmetic per load.
    auto dma = [&](int st, char *buf, uint32_t e0, uint32_t e1) {
#pragma unroll
        for (int k = 0; k < LPT; ++k) {
            const int x0 = kThreads * k + 64 * wv;    // the wave's first unit: sub-tile x0 / U, unit x0 % U
            // (known at compile time where a sub-tile is at least as large as a pass of the workgroup)
            const int sub = U >= kThreads ? (kThreads * k) / U : x0 / U;
            const int t = st * kStage + 16 * sub;
            if (t <= wg_maxpos) {
                const uint64_t off = (uint64_t)(sub ? e1 : e0) * block_stride +
                                     (uint32_t)(((t & (a.block_size - 1)) >> 4) * (16 * D * 2));
                // (written as assembly: the compiler would make every later LDS read wait for these loads;
                // m0, the LDS base of such a load, is a register the compiler reserves and sets itself
                // before any instruction of its own that reads it)
                typedef __attribute__((address_space(3))) char *lptr;
                const uint32_t lk = (uint32_t)(uintptr_t)(lptr)(buf + x0 * 16), lv = lk + VOFF;
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lk), "v"(lane_k[k]),
                             "s"(kp + off) : "memory");
                asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lv), "v"(lane_v[k]),
                             "s"(vp + off) : "memory");
            }
        }
    };
    // Value slots at or past the context's end are zeroed once the stage is in LDS (they may hold
    // anything, and a zero weight does not silence a NaN).
    auto zero_tail = [&](int st, char *buf) {
#pragma unroll
        for (int k = 0; k < LPT; ++k) {
            const int x = tid + kThreads * k, u = x / U, unit = x % U;
            if (!TILED) {                             // a slot is part of one row: position 16 u + unit / NU
                if (st * kStage + 16 * u + unit / NU >= C)
                    *reinterpret_cast<uint4 *>(buf + VOFF + x * 16) = make_uint4(0, 0, 0, 0);
                continue;
            }
            const int valid = C - (st * kStage + 16 * u + 4 * ((unit >> 4) & 3));
            if (valid < 4) {
                uint4 *slot = reinterpret_cast<uint4 *>(buf + VOFF + x * 16);
                uint4 v = *slot;
                const uint32_t m01 = valid >= 2 ? 0xFFFFFFFFu : (valid == 1 ? 0x0000FFFFu : 0u);
                const uint32_t m23 = valid == 3 ? 0x0000FFFFu : 0u;
                v.x &= m01; v.z &= m01;
                v.y &= m23; v.w &= m23;
                *slot = v;
            }
        }
    };

    // per-lane operand offsets in a stage buffer, tiled layout
    const int koff = qd * 256 + j * 16;               // + i * 1024, + SUBB for the second half
    const int voff = VOFF + (qd * 16 + j) * 16;       // + (s / 2) * 1024 + (s % 2) * 8, + SUBB for the second half
    // plain layout, tiles as they are: the swizzled slots of this lane's operands
    int kslot[NK], vslot[NS];
#pragma unroll
    for (int i = 0; i < NK; ++i) kslot[i] = (j * NU + ((4 * i + qd) ^ (j & (NU - 1)))) * 16;   // row j, dims 32 i + 8 qd ..
#pragma unroll
    for (int s2 = 0; s2 < NS; ++s2) {                 // row 4 qd + j / 4, dims 16 s + 4 (j % 4) ..
        const int rv = 4 * qd + (j >> 2);
        vslot[s2] = VOFF + (rv * NU + ((2 * s2 + ((j & 3) >> 1)) ^ ((2 * rv) & (NU - 1)))) * 16 + (j & 1) * 8;
    }

    bf16x8 kop[NK][2];                                // K rows: position (16 h +) j, dims 32 i + 8 qd ..
    bf16x8 vop[NS];                                   // V^T rows: dim 16 s + j, positions 4 qd .. of both halves
    auto read_k = [&](const char *buf) {
#pragma unroll
        for (int i = 0; i < NK; ++i)
#pragma unroll
            for (int h = 0; h < 2; ++h)
                kop[i][h] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const uint4 *>(
                    buf + (TILED ? koff + i * 1024 : kslot[i]) + h * SUBB));
    };
    auto read_v = [&](const char *buf) {
        if constexpr (TILED) {
            // the two sub-tiles' units as they lie in the pool: dims 32 i + j in bytes 0..7, 32 i + 16 + j in 8..15
#pragma unroll
            for (int s = 0; s < NS; ++s) {
                const char *at = buf + voff + (s >> 1) * 1024 + (s & 1) * 8;
                const uint2 h0 = *reinterpret_cast<const uint2 *>(at), h1 = *reinterpret_cast<const uint2 *>(at + SUBB);
                vop[s] = __builtin_bit_cast(bf16x8, make_uint4(h0.x, h0.y, h1.x, h1.y));
            }
        } else {
#pragma unroll
            for (int s = 0; s < NS; ++s) {            // four rows of 16 dims, transposed on the way
                typedef __attribute__((address_space(3))) s16x4 *lds_ptr;
                const s16x4 h0 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(buf + vslot[s]));
                const s16x4 h1 = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_ptr)(buf + vslot[s] + SUBB));
                vop[s] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(h0, h1, 0, 1, 2, 3, 4, 5, 6, 7));
            }
        }
    };

    f32x4 sc0[kColBlocks], sc1[kColBlocks];            // scores: positions t0 (+16) + 4 qd + e of the lane's column
    bf16x8 pw[kColBlocks];                             // weights, transposed: the second product's operand
    // Operand-major order: every K / V operand is used at once for both column blocks
    // (independent MFMAs back to back).
    auto scores = [&]() {
#pragma unroll
        for (int b = 0; b < kColBlocks; ++b) sc0[b] = sc1[b] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < NK; ++i)
#pragma unroll
            for (int b = 0; b < kColBlocks; ++b) {
                sc0[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[i][0], qb[b][i], sc0[b], 0, 0, 0);
                sc1[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(kop[i][1], qb[b][i], sc1[b], 0, 0, 0);
            }
    };
    auto softmax = [&](int t0) {
        const bool masked = t0 + kStage - 1 > wave_minpos;   // wave-uniform: some column does not see the whole stage
#pragma unroll
        for (int b = 0; b < kColBlocks; ++b) {
            float sc[8];                              // raw scores; scale_log2e > 0 is applied in the exponent
#pragma unroll
            for (int e = 0; e < 8; ++e) sc[e] = e < 4 ? sc0[b][e] : sc1[b][e - 4];
            if (masked) {                             // a token sees the positions up to its own
                const int lim = pos[b] - t0 - 4 * qd;
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    if (16 * (e >> 2) + (e & 3) > lim) sc[e] = -INFINITY;
            }
            float mx = sc[0];                         // median with +inf = maximum, without fmaxf's NaN quieting moves
#pragma unroll
            for (int e = 1; e < 8; ++e) mx = __builtin_amdgcn_fmed3f(mx, sc[e], INFINITY);
            mx *= a.scale_log2e;
            // The reference point of the exponentials follows the running maximum lazily:
            // it moves only when a score exceeds it by more than kSlack, so weights stay
            // below 2^kSlack, the four lanes that share a column compare notes only then,
            // and the accumulators are rescaled a handful of times per column.
            if (__any(mx - m[b] > kSlack)) {          // wave-uniform, rare after the first stages
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float mn = mx - m[b] > kSlack ? mx : m[b];
                const float f = fast_exp2(m[b] - mn);
                m[b] = mn;
#pragma unroll
                for (int e = 0; e < 4; ++e) l[b][e] *= f;
#pragma unroll
                for (int s = 0; s < NS; ++s)
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[b][s][e] *= f;
            }
            const float mn = m[b];
#pragma unroll
            for (int e = 0; e < 8; ++e) pw[b][e] = (__bf16)fast_exp2(fmaf(sc[e], a.scale_log2e, -mn));
        }
    };
    auto accumulate = [&]() {
#pragma unroll
        for (int b = 0; b < kColBlocks; ++b) l[b] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ones, pw[b], l[b], 0, 0, 0);
#pragma unroll
        for (int s = 0; s < NS; ++s)
#pragma unroll
            for (int b = 0; b < kColBlocks; ++b) o[b][s] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(vop[s], pw[b], o[b][s], 0, 0, 0);
    };

    auto dma_group = [&](int grp, char *buf) {
#pragma unroll
        for (int h = 0; h < GRP; ++h) dma(grp * GRP + h, buf + h * STAGE, ent[2 * h], ent[2 * h + 1]);
    };
    lookup(0);
    // what is never loaded (sub-tiles past the workgroup's last position) reads as zero
    for (int i = tid; i < NB * GSTAGE / 16; i += kThreads) reinterpret_cast<uint4 *>(lds)[i] = make_uint4(0, 0, 0, 0);
    __syncthreads();
    dma_group(0, lds);
    lookup(1);
    dma_group(1, lds + GSTAGE);
    lookup(2);
    __builtin_amdgcn_s_waitcnt(0x0F70);               // vmcnt(0): both groups have landed
    __syncthreads();
    // At head_dim 256 the K and V operands of a stage are 64 registers each.  With 16 columns per
    // wave they are read one after the other, K right before the scores and V behind them: the
    // wave then stays under 256 registers and two workgroups share a CU here as well.
    constexpr bool kLean = D >= 256 && kCols <= 16;
    if (!kLean) read_k(lds);
    const int n_groups = (n_stages + GRP - 1) / GRP;
    for (int grp = 0; grp < n_groups; ++grp) {
        char *cur = lds + (grp & 1) * GSTAGE, *nxt = lds + ((grp + 1) & 1) * GSTAGE;
        if ((grp + 1) * GRP * kStage > C) {           // the group holds the context's last stage: uniform
#pragma unroll
            for (int h = 0; h < GRP; ++h)
                if ((grp * GRP + h) * kStage + kStage > C) zero_tail(grp * GRP + h, cur + h * STAGE);
            __syncthreads();
        }
#pragma unroll
        for (int h = 0; h < GRP; ++h) {
            const int st = grp * GRP + h;
            char *at = cur + h * STAGE;
            const bool live = st * kStage <= wave_maxpos;   // wave-uniform: this wave's columns see the stage
            if (live) {
                if (kLean) read_k(at);
                else read_v(at);                      // needed after the next K operands are asked for
                scores();
                if (kLean) read_v(at);
                softmax(st * kStage);
            }
            if (h == GRP - 1) {
                __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): group grp + 1, on its way since the last barrier
                __syncthreads();                      // ... is in LDS for everyone; this group's operands are in registers
                dma_group(grp + 2, cur);              // in flight until the next barrier (a third buffer and
                lookup(grp + 3);                      // loads two barriers ahead were measured: slower)
            }
            if (!kLean && st + 1 < n_stages) read_k(h == GRP - 1 ? nxt : at + STAGE);   // needed at the top of the next stage
            if (live) accumulate();
        }
    }

#pragma unroll
    for (int b = 0; b < kColBlocks; ++b) {
        if (pos[b] < 0) continue;
        const float lt = l[b][0];
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

template <int D, bool TILED, int kCols = kMaxCols>
hipError_t launch_mfma_prefill(const PrefillArgs &p, hipStream_t s)
{
    const int G = p.d.num_q_heads / p.d.num_kv_heads;
    const int WT = kWaves * (kCols / G);
    const long long tiles = (p.max_new_tokens + WT - 1) / WT;
    const long long pairs = (long long)p.d.num_kv_heads * p.d.batch;
    const long long full = pairs / 8, rest = pairs % 8;   // whole groups of 8 pairs, and the pairs left over
    const long long grid = full * tiles * 8 + (rest * tiles + 7) / 8 * 8;
    if (tiles < 1 || grid > 0x7fffffffLL) return hipErrorInvalidValue;
    // Two stages per barrier where they fit and a request has many new tokens (the matrix cores
    // bind: +2-5 %); with one tile per request the kernel is a stream over the cache, and the
    // finer grain is the faster one (+3 %).
    constexpr bool kFits = 2 * 2 * (4 * 16 * D * 2) <= 65536;
    if (kFits && tiles > 1)
        hipLaunchKernelGGL((prefill_mfma<D, TILED, kCols, kFits ? 2 : 1>), dim3((unsigned)grid), dim3(kThreads), 0, s, p,
                           (int)tiles, (int)full);
    else
        hipLaunchKernelGGL((prefill_mfma<D, TILED, kCols, 1>), dim3((unsigned)grid), dim3(kThreads), 0, s, p, (int)tiles,
                           (int)full);
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
    // (the matrix-core kernel keeps the distance between two blocks of a pool in 32 bits)
    const unsigned long long stride = 2ull * a.num_layers * a.num_kv_heads * a.block_size * a.head_dim;
    if (a.bf16 && G <= kMaxCols && !p.force_rows && stride <= 0xffffffffull) {     // matrix cores
        const bool tiled = decode_uses_tiled_layout(a.bf16, G);
        if (a.head_dim == 64) return tiled ? launch_mfma_prefill<64, true>(p, stream) : launch_mfma_prefill<64, false>(p, stream);
        if (a.head_dim == 128) return tiled ? launch_mfma_prefill<128, true>(p, stream) : launch_mfma_prefill<128, false>(p, stream);
        // head_dim 256: 32 columns per wave need more than 256 registers (one workgroup per CU); without
        // head groups 16 columns and two workgroups per CU are faster (measured: +9 %), with groups not
        if (a.head_dim == 256) return tiled ? launch_mfma_prefill<256, true>(p, stream) : launch_mfma_prefill<256, false, 16>(p, stream);
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
