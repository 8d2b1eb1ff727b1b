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
