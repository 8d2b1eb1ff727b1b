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
//     sequence (head outermost, then request, then position); as many
//     wavefronts as the chip holds at once each take an equal
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

#include <atomic>

#include "attn_reducers.h"
#include "internal.h"
#include "lamps.h"

namespace lamps {
namespace {

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
    const int C = ctx_len(a, r);
    if (!running) return;                      // Preserve / Swap / Discard: not in the batch
    const int t_begin = part * a.part_tokens;
    if (t_begin >= C && part != 0) return;     // partition 0 of an empty context writes zeros
    const int t_end = min(C, t_begin + a.part_tokens);
    const int n_parts = max(1, (C + a.part_tokens - 1) / a.part_tokens);
    const int g = hc / passes;
    const int h0 = g * G + (hc % passes) * GH;
    const size_t rh0 = (size_t)r * a.num_q_heads + h0;

    R::run(a, r, (size_t)r, g, h0, GH, t_begin, t_end, [&](int h, int d, float M, float L, float A) {
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
    const int C = ctx_len(a, r);
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
// sequence ordered (kv head / pass, request, chunk).  prefix[] (dynamic LDS,
// batch + 1 ints) holds the running chunk count per request; every workgroup
// computes it for itself from ctx_lens / running (a few hundred loads that hit
// in L2), which costs less than a dependent launch.
//
// Which share a wavefront takes: with the heads outermost, the shares that read
// the same blocks for different heads lie shares / heads apart.  Workgroups go to
// the eight XCDs in turn, each XCD translates addresses for itself, and a block's
// heads share its pages; so the shares are handed out in the order of their
// position inside a head's stretch, XCD 0 first: the waves that walk the same
// blocks at the same time then sit on one XCD, next to each other.  With pools of
// 100 GB and more this is worth several per cent; with small pools it is neutral.
template <typename R>
__global__ __launch_bounds__(kThreads) void decode_balanced(const DecodeArgs a)
{
    constexpr int D = R::D, CT = R::CT;
    extern __shared__ int prefix[];
    __shared__ int wave_total[kWaves], wave_longest[kWaves];

    const int B = a.batch;
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int per = (B + kThreads - 1) / kThreads;   // consecutive requests per thread
    int mine = 0, longest = 0;
    for (int i = 0; i < per; ++i) {
        const int r = tid * per + i;
        if (r < B) {
            const int n = chunks_of(a.running[r], ctx_len(a, r), CT);
            mine += n;
            longest = max(longest, n);
        }
    }
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt *= 2) longest = max(longest, __shfl_xor(longest, dlt));
    int incl = mine;                                  // inclusive scan inside the wave
#pragma unroll
    for (int dlt = 1; dlt < 64; dlt *= 2) {
        const int up = __shfl_up(incl, dlt);
        if (lane >= dlt) incl += up;
    }
    if (lane == 63) {
        wave_total[wv] = incl;
        wave_longest[wv] = longest;
    }
    __syncthreads();
#pragma unroll
    for (int ww = 0; ww < kWaves; ++ww) longest = max(longest, wave_longest[ww]);
    int run = incl - mine;
    for (int ww = 0; ww < wv; ++ww) run += wave_total[ww];
    if (tid == 0) prefix[0] = 0;
    for (int i = 0; i < per; ++i) {
        const int r = tid * per + i;
        if (r < B) {
            run += chunks_of(a.running[r], ctx_len(a, r), CT);
            prefix[r + 1] = run;
        }
    }
    __syncthreads();

    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int HC = a.num_kv_heads * passes;
    // (values that are the same in every lane are told so: the compiler cannot see it
    // through LDS and the shuffles, and would keep the range arithmetic in vector registers)
    const int T = __builtin_amdgcn_readfirstlane(prefix[B]);   // chunks per head / pass
    const long long total = (long long)HC * T;
    longest = __builtin_amdgcn_readfirstlane(longest);
    // from here on every wave is on its own: no barrier below
    int P = gridDim.x * kWaves;
    int share = blockIdx.x * kWaves + __builtin_amdgcn_readfirstlane(wv);
    // A launch with little work and a long range in it: equal shares over all wavefronts would
    // cut that range into hundreds of pieces of a chunk each, and the merge of one range is a
    // chain of dependent loads (a 40 000-token request among 70 short ones, 2 heads: 10 us of
    // attention, 200 us of merge).  Then only as many shares are used as gives each 2, 4 or
    // 8 chunks -- for a longest range of 256, 512, 1024 chunks and more -- and the rest stay
    // empty.
    const int log2_share_chunks = longest >= 1024 ? 3 : longest >= 512 ? 2 : longest >= 256 ? 1 : 0;
    const long long wanted = (total + (1 << log2_share_chunks) - 1) >> log2_share_chunks;
    if (wanted < P) {
        P = __builtin_amdgcn_readfirstlane(max(1, (int)wanted));
        if (share >= P) {
            if (lane == 0) a.share_info[share] = make_int4(0, 0, 0, kShareEmpty);
            return;
        }
    } else if (a.share_gcd > 0) {
        // rank = (share * HC mod P) + share / (P / gcd) orders the shares by where they
        // start inside a head's stretch; this wave takes the share of rank
        // (XCD, index inside the XCD), found by inverting that
        const int rank = (blockIdx.x & 7) * (P >> 3) + (blockIdx.x >> 3) * kWaves +
                         __builtin_amdgcn_readfirstlane(wv);
        const int tie = rank % a.share_gcd, period = P / a.share_gcd;
        share = (int)((long long)(rank / a.share_gcd) * a.share_inv % period) + tie * period;
    }
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

    // request that holds position x_begin of its head: the last r with prefix[r] <= it
    const int first_pos = (int)(x_begin % T);
    int lo = 0, hi = B;
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (prefix[mid] <= first_pos) lo = mid; else hi = mid;
    }
    int r = __builtin_amdgcn_readfirstlane(lo);
    long long x = x_begin;
    while (x < x_end) {
        const int base = __builtin_amdgcn_readfirstlane(prefix[r]);
        const int nr = __builtin_amdgcn_readfirstlane(prefix[r + 1]) - base;   // > 0 here
        const int hc = (int)(x / T), c0 = (int)(x % T) - base;
        const int len = (int)min((long long)(nr - c0), x_end - x);
        const int C = ctx_len(a, r);
        const int g = hc / passes;
        const int h0 = g * G + (hc % passes) * GH;
        const bool whole = (c0 == 0 && len == nr);
        // a share's first range goes to slot 0, a later partial one (its last) to slot 1
        float *slot = a.partials + ((size_t)share * 2 + (x == x_begin ? 0 : 1)) * GH * (D + 2);
        const size_t rh0 = (size_t)r * a.num_q_heads + h0;
        R::run(a, r, (size_t)r, g, h0, GH, c0 * CT, min(C, (c0 + len) * CT),
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
        if (c0 + len == nr) {                         // request finished: next one with work,
            do {                                      // after the last one the next head's first
                if (++r == B) r = 0;
            } while (prefix[r + 1] == prefix[r]);
        }
    }
    if (lane == 0) a.share_info[share] = owned;
}

// N pieces of a split range, their loads in flight together, folded into the running
// (M, L, A0, A1) of the lane's two outputs.  slot holds one piece per lane (-1: an empty
// share); i0 and cnt are the same in every lane.
template <int N>
__device__ __forceinline__ void merge_pieces(const float *partials, int slot, int i0, int cnt, int GH, int h,
                                             int D, int d, float &M, float &L, float &A0, float &A1)
{
    float2 ml[N], ao[N];                               // rows of the partials are 8-byte aligned
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const int pc = __builtin_amdgcn_readlane(slot, min(i0 + k, 63));
        const bool have = i0 + k < cnt && pc >= 0;
        const float2 *x = reinterpret_cast<const float2 *>(partials + ((size_t)max(pc, 0) * GH + h) * (D + 2));
        ml[k] = have ? x[D / 2] : make_float2(kLowest, 0.0f);
        ao[k] = have ? x[d / 2] : make_float2(0.0f, 0.0f);
    }
    float Mn = M;
#pragma unroll
    for (int k = 0; k < N; ++k) Mn = fmaxf(Mn, ml[k].x);
    const float f0 = fast_exp2(M - Mn);
    L *= f0;
    A0 *= f0;
    A1 *= f0;
    M = Mn;
#pragma unroll
    for (int k = 0; k < N; ++k) {
        const float f = fast_exp2(ml[k].x - M);
        L += ml[k].y * f;
        A0 += ao[k].x * f;
        A1 += ao[k].y * f;
    }
}

// Merges the pieces of every (request, kv head / pass) that was split over
// several shares, in share order (= token order).  One wavefront per share and
// slice of 128 (head, dim) outputs, two outputs per lane: the share that holds the
// start of a split range merges it, eight pieces' loads in flight at a time (most
// waves find nothing to do and leave after one load).  A wave works alone: the
// piece list lives in a register, one piece per lane, and is read with readlane.
// The grid is small on purpose (the launcher also folds up to 16 wavefronts into a
// workgroup): launching a workgroup that leaves at once costs
// about a nanosecond, and a block per share and 256 outputs spent most of this
// kernel's time on that.
template <bool BF16>
__global__ __launch_bounds__(1024) void decode_merge_balanced(const DecodeArgs a)
{
    const int lane = threadIdx.x & 63;
    const int w_first = __builtin_amdgcn_readfirstlane(blockIdx.x * (blockDim.x >> 6) + (threadIdx.x >> 6));
    const int4 owned = a.share_info[w_first];
    if (!(owned.w & kShareOwner)) return;
    const int r = __builtin_amdgcn_readfirstlane(owned.x), hc = __builtin_amdgcn_readfirstlane(owned.y);
    const int w_last = __builtin_amdgcn_readfirstlane(owned.z);
    const int first_flags = __builtin_amdgcn_readfirstlane(owned.w);
    const int D = a.head_dim;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const size_t rh0 = (size_t)r * a.num_q_heads + (hc / passes) * G + (hc % passes) * GH;
    const int idx = blockIdx.y * 128 + 2 * lane;       // the lane's two outputs: same head, d even
    const bool live = idx < GH * D;
    const int h = live ? idx / D : 0, d = live ? idx % D : 0;
    float M = kLowest, L = 0.0f, A0 = 0.0f, A1 = 0.0f;
    // lane i: where piece i of a pass of 64 lies.  The first share knows its slot; later ones
    // start inside the range: slot 0.
    auto slots_of = [&](int w0) {
        const int w = w0 + lane;
        if (w > w_last) return -1;
        const int f = w == w_first ? first_flags : a.share_info[w].w;
        return (f & kShareEmpty) ? -1 : w * 2 + ((w == w_first && (f & kShareSlot1)) ? 1 : 0);
    };
    int slot_next = slots_of(w_first);
    for (int w0 = w_first; w0 <= w_last; w0 += 64) {
        const int cnt = min(64, w_last - w0 + 1);
        const int slot = slot_next;
        slot_next = slots_of(w0 + 64);                 // asked for together with this pass's pieces
        for (int i0 = 0; i0 < cnt; i0 += 8)            // share order = token order
            merge_pieces<8>(a.partials, slot, i0, cnt, GH, h, D, d, M, L, A0, A1);
    }
    if (live) {
        store_out<BF16>(a.out, (rh0 + h) * D + d, L > 0.0f ? A0 / L : 0.0f);
        store_out<BF16>(a.out, (rh0 + h) * D + d + 1, L > 0.0f ? A1 / L : 0.0f);
    }
}

// The same merge for a small batch of long contexts.  A range then has hundreds of
// pieces, and one lane per output pair walking them eight at a time is a long serial
// chain.  Here a block looks at 16 shares and, for each owner among them (there are
// few), takes 32 outputs of one query head of its range: 32 groups of 8 threads,
// four outputs per thread; group j merges the pieces j, j + 32, ... eight in flight
// per thread, so one pass covers the 256 pieces that the piece list resolves at a
// time; the groups' states are merged by a fixed tree through LDS at the end.
template <bool BF16, int D>
__global__ __launch_bounds__(256) void decode_merge_wide(const DecodeArgs a)
{
    constexpr int QUADS = 8, GROUPS = 32, INFL = 8;
    const int tid = threadIdx.x, j = tid / QUADS, q = tid % QUADS;
    const int G = a.num_q_heads / a.num_kv_heads;
    const int GH = a.heads_per_pass;
    const int passes = G / GH;
    const int h = blockIdx.y;                          // query head of the pass
    const int d0 = blockIdx.z * 32 + 4 * q;            // first of this thread's four outputs
    __shared__ int4 owners[kWideShares];
    __shared__ int piece[256];
    __shared__ float state[GROUPS][QUADS][6];
    if (tid < kWideShares) owners[tid] = a.share_info[blockIdx.x * kWideShares + tid];
    __syncthreads();
    for (int s = 0; s < kWideShares; ++s) {
        const int4 owned = owners[s];
        if (!(owned.w & kShareOwner)) continue;        // the same for the whole block
        const int r = owned.x, hc = owned.y;
        const int w_first = blockIdx.x * kWideShares + s, w_last = owned.z;
        const size_t row = (size_t)r * a.num_q_heads + (hc / passes) * G + (hc % passes) * GH + h;
        float M = kLowest, L = 0.0f, A[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        for (int w0 = w_first; w0 <= w_last; w0 += 256) {
            const int cnt = min(256, w_last - w0 + 1);
            __syncthreads();
            if (tid < cnt) {
                const int w = w0 + tid;
                const int f = w == w_first ? owned.w : a.share_info[w].w;
                piece[tid] = (f & kShareEmpty) ? -1 : w * 2 + ((w == w_first && (f & kShareSlot1)) ? 1 : 0);
            }
            __syncthreads();
            float2 ml[INFL], ao[INFL][2];              // rows of the partials are 8-byte aligned
#pragma unroll
            for (int k = 0; k < INFL; ++k) {
                const int i = j + k * GROUPS;
                const int pc = i < cnt ? piece[i] : -1;
                const float2 *x = reinterpret_cast<const float2 *>(
                    a.partials + ((size_t)max(pc, 0) * GH + h) * (D + 2));
                ml[k] = pc >= 0 ? x[D / 2] : make_float2(kLowest, 0.0f);
                ao[k][0] = pc >= 0 ? x[d0 / 2] : make_float2(0.0f, 0.0f);
                ao[k][1] = pc >= 0 ? x[d0 / 2 + 1] : make_float2(0.0f, 0.0f);
            }
            float Mn = M;
#pragma unroll
            for (int k = 0; k < INFL; ++k) Mn = fmaxf(Mn, ml[k].x);
            const float f0 = fast_exp2(M - Mn);
            L *= f0;
#pragma unroll
            for (int e = 0; e < 4; ++e) A[e] *= f0;
            M = Mn;
#pragma unroll
            for (int k = 0; k < INFL; ++k) {
                const float f = fast_exp2(ml[k].x - M);
                L += ml[k].y * f;
                A[0] += ao[k][0].x * f;
                A[1] += ao[k][0].y * f;
                A[2] += ao[k][1].x * f;
                A[3] += ao[k][1].y * f;
            }
        }
        __syncthreads();                               // the state of the owner before is read
        float *mine = state[j][q];
        mine[0] = M;
        mine[1] = L;
#pragma unroll
        for (int e = 0; e < 4; ++e) mine[2 + e] = A[e];
        __syncthreads();
        for (int half = GROUPS / 2; half >= 1; half /= 2) {   // a fixed tree over the groups
            if (j < half) {
                const float *t = state[j + half][q];
                const float Mn = fmaxf(M, t[0]);
                const float f0 = fast_exp2(M - Mn), f1 = fast_exp2(t[0] - Mn);
                L = L * f0 + t[1] * f1;
#pragma unroll
                for (int e = 0; e < 4; ++e) A[e] = A[e] * f0 + t[2 + e] * f1;
                M = Mn;
            }
            __syncthreads();
            if (j >= half / 2 && j < half) {           // the upper half of the next level publishes
                mine[0] = M;
                mine[1] = L;
#pragma unroll
                for (int e = 0; e < 4; ++e) mine[2 + e] = A[e];
            }
            __syncthreads();
        }
        if (j == 0) {
#pragma unroll
            for (int e = 0; e < 4; ++e)
                store_out<BF16>(a.out, row * D + d0 + e, L > 0.0f ? A[e] / L : 0.0f);
        }
    }
}

// ---------------------------------------------------------------- launchers

// Workgroups the chip holds at once for decode_balanced<R>, per device (asked once per device and
// instantiation; every thread that asks computes the same).
template <typename R>
hipError_t resident_workgroups(const DecodeArgs &a, int *out)
{
    static std::atomic<int> resident_on[kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    int resident = resident_on[dev].load(std::memory_order_relaxed);
    if (resident == 0) {
        int cus = 0, per_cu = 0;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e == hipSuccess)
            e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, decode_balanced<R>, kThreads,
                                                             (a.max_batch + 1) * sizeof(int));
        if (e != hipSuccess) return e;
        if (cus < 1 || per_cu < 1) return hipErrorInvalidValue;
        resident = cus * per_cu;
        resident_on[dev].store(resident, std::memory_order_relaxed);
    }
    *out = resident;
    return hipSuccess;
}

// demand != nullptr: nothing is launched; *demand receives the bytes of partial slots the
// balanced launch would use with every resident wavefront taking a share.
template <typename R>
hipError_t launch_one(const DecodeArgs &a, hipStream_t s, size_t *demand)
{
    const int G = a.num_q_heads / a.num_kv_heads;
    const int HC = a.num_kv_heads * (G / a.heads_per_pass);
    if (a.part_tokens > 0) {
        if (demand) return hipErrorInvalidValue;
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
    // if the partial slots of that many wave shares would not fit behind a.partials)
    int resident = 0;
    hipError_t e = resident_workgroups<R>(a, &resident);
    if (e != hipSuccess) return e;
    const size_t per_share = decode_share_bytes(a.heads_per_pass, a.head_dim);
    if (demand) {
        *demand = (size_t)min(resident, kMaxShares / kWaves) * kWaves * per_share;
        return hipSuccess;
    }
    const size_t fit = min((size_t)kMaxShares, a.partial_capacity / per_share);
    const int wgs = min(resident, (int)(fit / kWaves));
    if (wgs < 1) return hipErrorInvalidValue;
    const size_t lds = (size_t)(a.batch + 1) * sizeof(int);
    DecodeArgs b = a;
    b.share_gcd = b.share_inv = 0;                    // shares in launch order
    if (wgs % 8 == 0) {                               // whole rounds over the XCDs: ranked shares
        const int P = wgs * kWaves;
        int g = HC, t = P;
        while (t) { const int m = g % t; g = t; t = m; }
        // inverse of HC / g modulo P / g (the two are coprime), by the extended Euclidean algorithm
        const int period = P / g;
        long long r0 = period, r1 = HC / g % period, t0 = 0, t1 = 1;
        while (r1 > 1) {
            const long long q = r0 / r1, r2 = r0 - q * r1, t2 = t0 - q * t1;
            r0 = r1; r1 = r2; t0 = t1; t1 = t2;
        }
        b.share_gcd = g;
        b.share_inv = period > 1 ? (int)((t1 % period + period) % period) : 0;
    }
    hipLaunchKernelGGL(decode_balanced<R>, dim3(wgs), dim3(kThreads), lds, s, b);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    // a batch so small that its ranges average 64 pieces and more: pieces in parallel
    const int P = wgs * kWaves;
    if ((long long)a.batch * HC * 64 <= P && P % kWideShares == 0) {
        hipLaunchKernelGGL((decode_merge_wide<R::kBF16, R::D>),
                           dim3(P / kWideShares, a.heads_per_pass, R::D / 32), dim3(256), 0, s, a);
        return hipGetLastError();
    }
    const int slices = (a.heads_per_pass * a.head_dim + 127) / 128;
    // (workgroups of 16 wavefronts where the share count allows: fewer, larger workgroups launch faster)
    const int fold = wgs % 4 == 0 ? 4 : wgs % 2 == 0 ? 2 : 1;
    hipLaunchKernelGGL(decode_merge_balanced<R::kBF16>, dim3(wgs / fold, slices), dim3(256 * fold), 0, s, a);
    return hipGetLastError();
}

template <bool BF16, int LPT>
hipError_t launch_valu(const DecodeArgs &a, hipStream_t s, size_t *demand)
{
    switch (a.heads_per_pass) {
    case 1: return launch_one<ValuReducer<BF16, LPT, 1, kHalves>>(a, s, demand);
    case 2:
        if constexpr (!BF16) return launch_one<ValuReducer<BF16, LPT, 2, kHalves>>(a, s, demand);
        break;                                 // grouped bf16 heads take the MFMA path
    case 4:
        if constexpr (!BF16) return launch_one<ValuReducer<BF16, LPT, 4, 1>>(a, s, demand);
        break;
    }
    return hipErrorInvalidValue;
}

template <int D>
hipError_t launch_mfma(const DecodeArgs &a, hipStream_t s, size_t *demand)
{
    if (a.heads_per_pass > 16) return hipErrorInvalidValue;
    return launch_one<MfmaReducer<D>>(a, s, demand);
}

// Picks the instantiation for the geometry; launches, or (demand != nullptr) only asks.
hipError_t dispatch_impl(const DecodeArgs &a, hipStream_t stream, size_t *demand)
{
    const int G = a.num_q_heads / a.num_kv_heads;
    if (a.heads_per_pass != decode_heads_per_pass(a.bf16, a.head_dim, G) || a.heads_per_pass == 0)
        return hipErrorInvalidValue;
    const int lpt = a.head_dim * (a.bf16 ? 2 : 4) / 16;
    if (decode_uses_tiled_layout(a.bf16, G)) {
        if (a.head_dim == 64) return launch_mfma<64>(a, stream, demand);
        if (a.head_dim == 128) return launch_mfma<128>(a, stream, demand);
        if (a.head_dim == 256) return launch_mfma<256>(a, stream, demand);
    } else if (a.bf16) {
        if (lpt == 8) return launch_valu<true, 8>(a, stream, demand);
        if (lpt == 16) return launch_valu<true, 16>(a, stream, demand);
        if (lpt == 32) return launch_valu<true, 32>(a, stream, demand);
    } else {
        if (lpt == 8) return launch_valu<false, 8>(a, stream, demand);
        if (lpt == 16) return launch_valu<false, 16>(a, stream, demand);
        if (lpt == 32) return launch_valu<false, 32>(a, stream, demand);
    }
    return hipErrorInvalidValue;
}

}  // namespace

hipError_t dispatch(const DecodeArgs &a, hipStream_t stream, size_t *demand) { return dispatch_impl(a, stream, demand); }

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

size_t decode_share_bytes(int heads_per_pass, int head_dim)
{
    return (size_t)2 * heads_per_pass * (head_dim + 2) * sizeof(float);
}

int decode_max_shares(int heads_per_pass, int head_dim)
{
    size_t n = kPartialBudget / decode_share_bytes(heads_per_pass, head_dim);
    if (n > (size_t)kMaxShares) n = kMaxShares;
    return (int)(n / kWaves) * kWaves;
}

hipError_t launch_decode(const DecodeArgs &a, hipStream_t stream)
{
    if (a.batch == 0) return hipSuccess;
    return dispatch(a, stream, nullptr);
}

}  // namespace lamps

// ---------------------------------------------------------------- decode without a workspace
//
// The balanced scheme's scratch memory -- the partial slots of split ranges and one int4 per
// share -- in a file-scope device array instead of the caller's workspace.  Every device the
// library runs on holds its own copy of the array, at its own address, until the process ends.
namespace {

constexpr size_t kStaticPartialBytes = (size_t)LAMPS_STATIC_SCRATCH_BYTES - ((size_t)1 << 20);
constexpr size_t kStaticInfoBytes = (size_t)(lamps::kMaxShares + 1) * sizeof(int4);
static_assert(kStaticInfoBytes <= ((size_t)1 << 20), "share records must fit the last MiB");
static_assert(kStaticPartialBytes % 256 == 0, "the share records start 256-byte aligned");

static __device__ __align__(256) unsigned char scratch[LAMPS_STATIC_SCRATCH_BYTES];

// Device address of `scratch` on the current device.  The array's name is only a handle in host
// code: the address comes from hipGetSymbolAddress, once per device, with that device current.
hipError_t static_scratch(unsigned char **base)
{
    static std::atomic<unsigned char *> scratch_on[lamps::kMaxDevices];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= lamps::kMaxDevices) return hipErrorInvalidDevice;
    unsigned char *ptr = scratch_on[dev].load(std::memory_order_acquire);
    if (!ptr) {
        e = hipGetSymbolAddress((void **)&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        scratch_on[dev].store(ptr, std::memory_order_release);   // every thread finds the same address
    }
    *base = ptr;
    return hipSuccess;
}

int static_fail(int code, const char *text)
{
    lamps::set_thread_error(text);
    return code;
}

}  // namespace

extern "C" int lamps_decode_attn_static(const lamps_config *cfg, void *compute_stream, int32_t layer,
                                        int32_t batch, const void *q, const void *k_pool, const void *v_pool,
                                        const int32_t *block_table, const int32_t *ctx_lens,
                                        const uint8_t *running_mask, void *out)
{
    lamps::DecodeArgs a;
    if (const char *why = lamps::decode_geometry(cfg, &a)) return static_fail(LAMPS_ERR_INVALID, why);
    if (cfg->part_tokens != 0)
        return static_fail(LAMPS_ERR_INVALID, "lamps_decode_attn_static: part_tokens must be 0 (balanced shares only)");
    if (!q || !k_pool || !v_pool || !block_table || !ctx_lens || !running_mask || !out)
        return static_fail(LAMPS_ERR_INVALID, "lamps_decode_attn_static: null argument");
    if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)q | (uintptr_t)out) & 15)
        return static_fail(LAMPS_ERR_INVALID, "lamps_decode_attn_static: pools, q and out must be 16-byte aligned");
    if (layer < 0 || layer >= cfg->num_layers)
        return static_fail(LAMPS_ERR_RANGE, "lamps_decode_attn_static: layer out of range");
    if (batch < 0 || batch > cfg->max_batch)
        return static_fail(LAMPS_ERR_RANGE, "lamps_decode_attn_static: batch out of range");
    if (batch == 0) return LAMPS_OK;
    unsigned char *base = nullptr;
    hipError_t e = static_scratch(&base);
    if (e != hipSuccess) return static_fail(LAMPS_ERR_HIP, hipGetErrorString(e));
    a.q = q;
    a.k_pool = k_pool;
    a.v_pool = v_pool;
    a.block_table = block_table;
    a.ctx_lens = ctx_lens;
    a.running = running_mask;
    a.out = out;
    a.batch = batch;
    a.layer = layer;
    a.partials = reinterpret_cast<float *>(base);
    a.partial_capacity = kStaticPartialBytes;
    a.share_info = reinterpret_cast<int4 *>(base + kStaticPartialBytes);
    size_t demand = 0;
    if ((e = lamps::dispatch(a, nullptr, &demand)) != hipSuccess)
        return static_fail(LAMPS_ERR_HIP, hipGetErrorString(e));
    if (demand > kStaticPartialBytes)
        return static_fail(LAMPS_ERR_RANGE,
                           "lamps_decode_attn_static: this geometry's partial slots (two records of heads per "
                           "pass x (head_dim + 2) floats per resident wavefront) exceed the static scratch buffer");
    // every launch writes the share record of every wavefront it starts and reads only those,
    // and reads only the partial slots those records name: nothing has to start at zero
    if ((e = lamps::dispatch(a, static_cast<hipStream_t>(compute_stream), nullptr)) != hipSuccess)
        return static_fail(LAMPS_ERR_HIP, hipGetErrorString(e));
    return LAMPS_OK;
}
