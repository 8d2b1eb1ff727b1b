// Host half of liblamps: the C ABI of include/lamps.h.
//
// Owns what the paper's engine keeps per model replica around "Execute
// runningBatch" (arXiv 2410.18248, Algorithm 1): the free list of KV blocks
// (Discard frees, Swap frees after its copy, an API return allocates), and the
// ordering between the swap copies and the decode steps.  All data memory and
// the streams belong to the caller; kernels are in decode_attn.hip and
// block_copy.hip.
#include "lamps.h"

#include <hip/hip_runtime.h>

#include <algorithm>
#include <chrono>
#include <cmath>
#include <cstdio>
#include <cstring>
#include <deque>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "internal.h"

namespace {

// Error text of calls that have no context to keep it in (a failed lamps_create, the
// workspace-free decode call): a fixed per-thread buffer, so that setting it allocates nothing.
thread_local char g_thread_error[256] = "";

size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

struct Derived {
    size_t elem = 0, half_bytes = 0, block_bytes = 0, pool_bytes = 0;
    size_t partial_bytes = 0, prefix_bytes = 0, aux_bytes = 0, staging_bytes = 0, workspace_bytes = 0;
    int part_tokens = 0, max_parts = 0, log2_bs = 0, blocks_per_chunk = 0;
    bool direct_copy = false;           // blocks are large enough to be copied one by one, unstaged
    int zero_copy = 0;                  // > 0: workgroups of the kernel that copies to / from host memory
    float scale_log2e = 0.f;
};

// Validates a config and derives the sizes; returns an error text or nullptr.
const char *derive(const lamps_config *c, Derived *d)
{
    if (!c) return "config is null";
    if (c->dtype != LAMPS_F32 && c->dtype != LAMPS_BF16) return "dtype must be LAMPS_F32 or LAMPS_BF16";
    if (c->num_layers < 1 || c->num_q_heads < 1 || c->num_kv_heads < 1 || c->head_dim < 1 ||
        c->num_blocks < 1 || c->max_blocks_per_req < 1 || c->max_batch < 1)
        return "sizes must be positive";
    if (c->num_q_heads % c->num_kv_heads != 0) return "num_q_heads must be a multiple of num_kv_heads";
    const int bf16 = c->dtype == LAMPS_BF16;
    if (lamps::decode_heads_per_pass(bf16, c->head_dim, c->num_q_heads / c->num_kv_heads) == 0)
        return "unsupported head_dim for this dtype (bf16: 64/128/256, f32: 32/64/128)";
    if (c->block_size < 16 || (c->block_size & (c->block_size - 1)) != 0)
        return "block_size must be a power of two >= 16";
    if ((int64_t)c->max_blocks_per_req * c->block_size > (int64_t)1 << 30) return "context too long";
    d->elem = bf16 ? 2 : 4;
    d->log2_bs = 0;
    while ((1 << d->log2_bs) < c->block_size) ++d->log2_bs;
    d->half_bytes = (size_t)c->num_layers * c->num_kv_heads * c->block_size * c->head_dim * d->elem;
    d->block_bytes = 2 * d->half_bytes;
    d->pool_bytes = d->half_bytes * (size_t)c->num_blocks;
    d->part_tokens = c->part_tokens;
    if (d->part_tokens < 0 || d->part_tokens % c->block_size != 0)
        return "part_tokens must be 0 or a positive multiple of block_size";
    if (c->max_batch > 8192) return "max_batch is limited to 8192";
    const int group = c->num_q_heads / c->num_kv_heads;
    const int gh = lamps::decode_heads_per_pass(bf16, c->head_dim, group);
    if (d->part_tokens > 0) {
        const int64_t max_ctx = (int64_t)c->max_blocks_per_req * c->block_size;
        d->max_parts = (int)((max_ctx + d->part_tokens - 1) / d->part_tokens);
        const int64_t wgs = (int64_t)d->max_parts * c->max_batch * c->num_kv_heads * (group / gh);
        if (wgs > 0x7fffffff) return "too many partitions; raise part_tokens";
        d->partial_bytes = (size_t)c->max_batch * c->num_q_heads * d->max_parts * (c->head_dim + 2) * 4;
    } else {
        d->max_parts = 0;
        d->partial_bytes = (size_t)lamps::decode_max_shares(gh, c->head_dim) * 2 * gh * (c->head_dim + 2) * 4;
    }
    d->prefix_bytes = (size_t)(lamps::decode_max_shares(gh, c->head_dim) + 1) * 16;   // share_info
    if (c->staging_bytes < 0) return "staging_bytes is negative";
    size_t st = c->staging_bytes ? (size_t)c->staging_bytes : (size_t)64 << 20;
    if (c->staging_bytes == 0 && st < d->block_bytes) st = d->block_bytes;
    if (st < d->block_bytes) return "staging_bytes is smaller than one block image";
    size_t bpc = st / d->block_bytes;
    if (bpc > 16384) bpc = 16384;               // keeps the copy grid's y dimension legal
    if (bpc > (size_t)c->num_blocks) bpc = c->num_blocks;
    d->blocks_per_chunk = (int)bpc;
    d->staging_bytes = bpc * d->block_bytes;
    d->aux_bytes = (size_t)(4 + 2 * c->max_batch) * sizeof(int32_t);          // lamps_validate_args
    d->workspace_bytes = align256(d->partial_bytes) + align256(d->prefix_bytes) + align256(d->aux_bytes) +
                         2 * align256(d->staging_bytes);
    // 0 = the default: blocks of 4 MiB and more per pool are contiguous runs long enough for the
    // copy engines as they are (measured: a little slower over the link than the staged path,
    // but the decode step next to it slows by 2 % instead of 8 %); zero-copy takes precedence
    const int64_t direct_from = c->direct_copy_bytes != 0 ? c->direct_copy_bytes
                                                          : (c->zero_copy_workgroups > 0 ? -1 : (int64_t)4 << 20);
    d->direct_copy = direct_from > 0 && (int64_t)d->half_bytes >= direct_from;
    if (c->zero_copy_workgroups < 0 || c->zero_copy_workgroups > 1024)
        return "zero_copy_workgroups must be in [0, 1024]";
    if (c->max_swaps_in_flight < 0) return "max_swaps_in_flight is negative";
    if (c->zero_copy_workgroups > 0 && c->direct_copy_bytes > 0)
        return "zero_copy_workgroups and direct_copy_bytes exclude each other";
    d->zero_copy = c->zero_copy_workgroups;
    const float scale = c->softmax_scale != 0.f ? c->softmax_scale : 1.0f / std::sqrt((float)c->head_dim);
    d->scale_log2e = scale * 1.4426950408889634f;
    return nullptr;
}

void thread_error(const char *a, const char *b = "")
{
    std::snprintf(g_thread_error, sizeof g_thread_error, "%s%s", a, b);
}

struct Ticket {
    hipEvent_t ev;
    size_t ring_slots;
    const char *host_lo, *host_hi;   // host bytes the copy writes (swap-out) or reads (swap-in)
    bool is_out;
    std::vector<hipEvent_t> step_ev; // layer-major copies: one event per step of layers_per_step layers
    int32_t layers_per_step = 0;
};

}  // namespace

struct lamps_ctx {
    lamps_config cfg;
    Derived d;
    char *k_pool, *v_pool;
    float *partials;
    int4 *share_info;
    int32_t *aux;                               // scratch of the argument checker
    char *stage_out, *stage_in;
    hipStream_t cs, os, is;

    std::vector<int32_t> free_stack;
    std::vector<uint8_t> allocated;
    std::vector<uint64_t> out_guard, in_guard;  // last swap-out / swap-in ticket per block, 0 = none
    std::vector<uint32_t> mark;                 // duplicate detection, by epoch
    uint32_t epoch = 0;

    std::deque<Ticket> tickets;                 // tickets[i] has id base_ticket + i
    uint64_t base_ticket = 1;
    std::vector<hipEvent_t> spare_events;
    hipEvent_t fence = nullptr;
    int32_t *ring = nullptr;                    // pinned; id lists read by the copy kernels
    size_t ring_cap = 0;
    uint64_t ring_head = 0, ring_tail = 0;      // monotonic slot counters
    bool swap_fence = true;                     // swap calls order themselves behind the compute stream
    std::mutex err_lock;                        // the compute-stream calls may fail next to a swap call
    std::string err;
};

namespace {

void fill_geometry(const lamps_config &cfg, const Derived &d, lamps::DecodeArgs *pa)
{
    lamps::DecodeArgs &a = *pa;
    a.max_batch = cfg.max_batch;
    a.num_layers = cfg.num_layers;
    a.num_q_heads = cfg.num_q_heads;
    a.num_kv_heads = cfg.num_kv_heads;
    a.head_dim = cfg.head_dim;
    a.block_size = cfg.block_size;
    a.log2_block_size = d.log2_bs;
    a.max_blocks = cfg.max_blocks_per_req;
    a.num_blocks = cfg.num_blocks;
    a.part_tokens = d.part_tokens;
    a.max_parts = d.max_parts;
    a.bf16 = cfg.dtype == LAMPS_BF16;
    a.heads_per_pass = lamps::decode_heads_per_pass(a.bf16, a.head_dim, a.num_q_heads / a.num_kv_heads);
    a.scale_log2e = d.scale_log2e;
    a.share_gcd = a.share_inv = 0;
}

void fill_decode_args(lamps_ctx *c, lamps::DecodeArgs *pa, int32_t layer, int32_t batch, const void *q,
                      const int32_t *block_table, const int32_t *ctx_lens, const uint8_t *running_mask,
                      void *out)
{
    lamps::DecodeArgs &a = *pa;
    fill_geometry(c->cfg, c->d, pa);
    a.q = q;
    a.k_pool = c->k_pool;
    a.v_pool = c->v_pool;
    a.block_table = block_table;
    a.ctx_lens = ctx_lens;
    a.running = running_mask;
    a.partials = c->partials;
    a.partial_capacity = c->d.partial_bytes;
    a.share_info = c->share_info;
    a.out = out;
    a.batch = batch;
    a.layer = layer;
}

int fail(lamps_ctx *c, int code, const std::string &msg)
{
    if (c) {
        std::lock_guard<std::mutex> hold(c->err_lock);
        c->err = msg;
    }
    return code;
}

int hip_fail(lamps_ctx *c, const char *what, hipError_t e)
{
    return fail(c, LAMPS_ERR_HIP, std::string(what) + ": " + hipGetErrorString(e));
}

// No exception crosses the C ABI: host containers may throw std::bad_alloc.  The texts are
// short enough for the string's in-place buffer, so reporting them allocates nothing.
#define LAMPS_CATCH(ctx)                                                             \
    catch (const std::bad_alloc &) { return fail(ctx, LAMPS_ERR_NOMEM, "out of memory"); } \
    catch (...) { return fail(ctx, LAMPS_ERR_INVALID, "C++ exception"); }
#define LAMPS_CATCH_NOCTX                                                \
    catch (const std::bad_alloc &) { thread_error("out of host memory"); return LAMPS_ERR_NOMEM; } \
    catch (...) { thread_error("C++ exception"); return LAMPS_ERR_INVALID; }

#define LAMPS_HIP(call)                                        \
    do {                                                       \
        hipError_t e_ = (call);                                \
        if (e_ != hipSuccess) return hip_fail(c, #call, e_);   \
    } while (0)

// Retires finished tickets from the front; releases their events and ring slots.
void retire_finished(lamps_ctx *c)
{
    while (!c->tickets.empty() && hipEventQuery(c->tickets.front().ev) == hipSuccess) {
        c->spare_events.push_back(c->tickets.front().ev);
        for (hipEvent_t e : c->tickets.front().step_ev) c->spare_events.push_back(e);
        c->ring_tail += c->tickets.front().ring_slots;
        c->tickets.pop_front();
        ++c->base_ticket;
    }
}

// Blocks until the oldest ticket has finished, then retires it.
int retire_oldest(lamps_ctx *c)
{
    LAMPS_HIP(hipEventSynchronize(c->tickets.front().ev));
    retire_finished(c);
    return LAMPS_OK;
}

bool ticket_known(const lamps_ctx *c, uint64_t t)
{
    return t >= 1 && t < c->base_ticket + c->tickets.size();
}

bool ticket_done(lamps_ctx *c, uint64_t t)
{
    if (t < c->base_ticket) return true;
    retire_finished(c);
    if (t < c->base_ticket) return true;
    return hipEventQuery(c->tickets[t - c->base_ticket].ev) == hipSuccess;
}

hipEvent_t ticket_event(lamps_ctx *c, uint64_t t) { return c->tickets[t - c->base_ticket].ev; }

int ensure_runtime(lamps_ctx *c)
{
    if (!c->fence) LAMPS_HIP(hipEventCreateWithFlags(&c->fence, hipEventDisableTiming));
    if (!c->ring) {
        c->ring_cap = (size_t)c->cfg.num_blocks * 2;
        if (c->ring_cap < 1024) c->ring_cap = 1024;
        void *p = nullptr;
        LAMPS_HIP(hipHostMalloc(&p, c->ring_cap * sizeof(int32_t), hipHostMallocDefault));
        c->ring = static_cast<int32_t *>(p);
    }
    return LAMPS_OK;
}

int new_event(lamps_ctx *c, hipEvent_t *ev)
{
    if (!c->spare_events.empty()) {
        *ev = c->spare_events.back();
        c->spare_events.pop_back();
        return LAMPS_OK;
    }
    LAMPS_HIP(hipEventCreateWithFlags(ev, hipEventDisableTiming));
    return LAMPS_OK;
}

// Backpressure (lamps_config.max_swaps_in_flight): waits, polling, until fewer than the limit
// of this direction's copies are unfinished.  Copies of one direction finish in ticket order, so
// the oldest unfinished one is the one to watch.
int wait_for_room(lamps_ctx *c, bool out)
{
    const int limit = c->cfg.max_swaps_in_flight;
    if (limit <= 0) return LAMPS_OK;
    for (;;) {
        retire_finished(c);
        int busy = 0;
        hipEvent_t oldest = nullptr;
        for (const Ticket &t : c->tickets)
            if (t.is_out == out && hipEventQuery(t.ev) != hipSuccess) {
                if (!oldest) oldest = t.ev;
                ++busy;
            }
        if (busy < limit) return LAMPS_OK;
        while (hipEventQuery(oldest) == hipErrorNotReady) std::this_thread::sleep_for(std::chrono::microseconds(50));
        const hipError_t e = hipEventQuery(oldest);
        if (e != hipSuccess) return hip_fail(c, "hipEventQuery", e);
    }
}

// Reserves n contiguous ring slots; *slots is what the ticket must give back.
int ring_reserve(lamps_ctx *c, int32_t n, int32_t **where, size_t *slots)
{
    for (;;) {
        size_t pos = (size_t)(c->ring_head % c->ring_cap);
        size_t pad = pos + (size_t)n > c->ring_cap ? c->ring_cap - pos : 0;
        if (c->ring_head + pad + n - c->ring_tail <= c->ring_cap) {
            c->ring_head += pad;
            *where = c->ring + (size_t)(c->ring_head % c->ring_cap);
            c->ring_head += n;
            *slots = pad + n;
            return LAMPS_OK;
        }
        if (c->tickets.empty()) return fail(c, LAMPS_ERR_NOMEM, "id ring too small for this list");
        int rc = retire_oldest(c);
        if (rc != LAMPS_OK) return rc;
    }
}

// Checks an id list: range, duplicates, and that every block is allocated.
int check_ids(lamps_ctx *c, const int32_t *ids, int32_t n, const char *who)
{
    if (n < 0) return fail(c, LAMPS_ERR_INVALID, std::string(who) + ": n is negative");
    if (n > 0 && !ids) return fail(c, LAMPS_ERR_INVALID, std::string(who) + ": block_ids is null");
    if (++c->epoch == 0) {
        std::fill(c->mark.begin(), c->mark.end(), 0u);
        c->epoch = 1;
    }
    for (int32_t i = 0; i < n; ++i) {
        const int32_t b = ids[i];
        if (b < 0 || b >= c->cfg.num_blocks)
            return fail(c, LAMPS_ERR_RANGE, std::string(who) + ": block id out of range");
        if (c->mark[b] == c->epoch)
            return fail(c, LAMPS_ERR_DUP, std::string(who) + ": duplicate block id");
        c->mark[b] = c->epoch;
    }
    for (int32_t i = 0; i < n; ++i)
        if (!c->allocated[ids[i]])
            return fail(c, LAMPS_ERR_DOUBLE_FREE, std::string(who) + ": block is not allocated");
    return LAMPS_OK;
}

// Makes `stream` wait for every unfinished ticket named in guard[ids[*]].  A guard array holds
// tickets of one direction only, and the copies of one direction run on one stream in ticket
// order: waiting for the newest of them covers all the others.
int wait_guards(lamps_ctx *c, hipStream_t stream, const std::vector<uint64_t> &guard,
                const int32_t *ids, int32_t n)
{
    uint64_t newest = 0;
    for (int32_t i = 0; i < n; ++i) newest = std::max(newest, guard[ids[i]]);
    if (newest >= c->base_ticket && !ticket_done(c, newest))
        LAMPS_HIP(hipStreamWaitEvent(stream, ticket_event(c, newest), 0));
    return LAMPS_OK;
}

// Orders `stream` after every unfinished copy of the other direction that
// touches host bytes [lo, hi): a swap-in may be enqueued right after the
// swap-out that fills its buffer, and the other way round.  The newest such copy
// stands for all of them (same stream, ticket order).
int wait_host_overlap(lamps_ctx *c, hipStream_t stream, const char *lo, const char *hi,
                      bool other_is_out)
{
    for (size_t k = c->tickets.size(); k-- > 0;) {
        Ticket &t = c->tickets[k];
        if (t.is_out == other_is_out && t.host_lo < hi && lo < t.host_hi) {
            if (hipEventQuery(t.ev) != hipSuccess) LAMPS_HIP(hipStreamWaitEvent(stream, t.ev, 0));
            break;
        }
    }
    return LAMPS_OK;
}

// The device address of the pinned, mapped host range [host, host + bytes), for the copy
// kernel that reaches it over the host link; anything else must not get near a kernel.
int mapped_host(lamps_ctx *c, const void *host, size_t bytes, const char *who, void **dev)
{
    *dev = nullptr;
    if (bytes == 0) return LAMPS_OK;
    if ((uintptr_t)host & 15)
        return fail(c, LAMPS_ERR_INVALID, std::string(who) + ": host_buf must be 16-byte aligned for the zero-copy path");
    const char *ends[2] = {static_cast<const char *>(host), static_cast<const char *>(host) + bytes - 1};
    for (int k = 0; k < 2; ++k) {
        hipPointerAttribute_t at;
        std::memset(&at, 0, sizeof at);
        if (hipPointerGetAttributes(&at, ends[k]) != hipSuccess || at.type != hipMemoryTypeHost ||
            at.devicePointer == nullptr) {
            (void)hipGetLastError();
            return fail(c, LAMPS_ERR_INVALID,
                        std::string(who) + ": host_buf is not pinned host memory mapped into the device");
        }
        if (k == 0) *dev = at.devicePointer;
    }
    return LAMPS_OK;
}

// A swap copy reads (out) or overwrites (in) blocks that compute-stream work enqueued before the
// call may still write or read: unless the caller has taken that ordering into its own hands,
// the swap stream waits for everything the compute stream holds at this moment.
int fence_behind_compute(lamps_ctx *c, hipStream_t st)
{
    if (!c->swap_fence) return LAMPS_OK;
    LAMPS_HIP(hipEventRecord(c->fence, c->cs));
    LAMPS_HIP(hipStreamWaitEvent(st, c->fence, 0));
    return LAMPS_OK;
}

// Last step of every swap call.  The ticket is filed whether or not the enqueue went through,
// so that its events and ring slots come back when the stream has passed it; a failed call
// hands no ticket to the caller and leaves the guards alone.
int file_ticket(lamps_ctx *c, int enqueue_rc, hipStream_t st, Ticket &t, std::vector<uint64_t> &guard,
                const int32_t *block_ids, int32_t n, uint64_t *ticket)
{
    const hipError_t e = hipEventRecord(t.ev, st);
    c->tickets.push_back(t);
    if (enqueue_rc != LAMPS_OK) return enqueue_rc;
    if (e != hipSuccess) return hip_fail(c, "hipEventRecord", e);
    const uint64_t id = c->base_ticket + c->tickets.size() - 1;
    for (int32_t i = 0; i < n; ++i) guard[block_ids[i]] = id;
    *ticket = id;
    return LAMPS_OK;
}

// Enqueues the steps of a layer-major swap on `st`, one event per step into t->step_ev:
// whole layers per step while a layer of the list fits the staging area (several when they
// are small, so that a copy is at least about 8 MiB), else one layer in chunks of blocks.
int enqueue_layer_steps(lamps_ctx *c, bool out, char *host, const int32_t *ids, int32_t n, hipStream_t st,
                        Ticket *t)
{
    const int32_t L = c->cfg.num_layers;
    const size_t layer_bytes = c->d.half_bytes / L;           // one block, one pool, one layer
    const size_t unit = 2 * layer_bytes;                       // keys + values of one block, one layer
    const size_t slice = (size_t)n * unit;                     // one layer of the whole list
    const bool whole = slice <= c->d.staging_bytes && n <= 16384;   // 16384: the copy grid's y limit
    char *stage = out ? c->stage_out : c->stage_in;
    int32_t nl = 1;
    if (whole) {
        const size_t want = (size_t)8 << 20;
        nl = (int32_t)std::min<size_t>({(size_t)L, c->d.staging_bytes / slice, (want + slice - 1) / slice});
        if (nl < 1) nl = 1;
    }
    const int32_t bpc = whole ? n : (int32_t)std::min<size_t>({(size_t)n, c->d.staging_bytes / unit, (size_t)16384});
    t->layers_per_step = nl;
    for (int32_t l0 = 0; l0 < L; l0 += nl) {
        const int32_t cnt_l = std::min<int32_t>(nl, L - l0);
        for (int32_t done = 0; done < n; done += bpc) {
            const int32_t cnt = std::min<int32_t>(bpc, n - done);
            char *himg = host + (size_t)l0 * slice + (size_t)done * unit;
            const size_t bytes = (size_t)cnt_l * cnt * unit;
            if (out) {
                LAMPS_HIP(lamps::launch_gather_layers(c->k_pool, c->v_pool, ids + done, cnt, c->d.half_bytes,
                                                      layer_bytes, l0, cnt_l, stage, st));
                LAMPS_HIP(hipMemcpyAsync(himg, stage, bytes, hipMemcpyDeviceToHost, st));
            } else {
                LAMPS_HIP(hipMemcpyAsync(stage, himg, bytes, hipMemcpyHostToDevice, st));
                LAMPS_HIP(lamps::launch_scatter_layers(c->k_pool, c->v_pool, ids + done, cnt, c->d.half_bytes,
                                                       layer_bytes, l0, cnt_l, stage, st));
            }
        }
        hipEvent_t se;
        const int rc = new_event(c, &se);
        if (rc != LAMPS_OK) return rc;
        t->step_ev.push_back(se);
        LAMPS_HIP(hipEventRecord(se, st));
    }
    return LAMPS_OK;
}

// The layer-major swap, both directions.
int swap_layered(lamps_ctx *c, bool out, char *host, const int32_t *block_ids, int32_t n, uint64_t *ticket,
                 const char *who)
{
    if (!ticket || (n > 0 && !host)) return fail(c, LAMPS_ERR_INVALID, std::string(who) + ": null argument");
    int rc = check_ids(c, block_ids, n, who);
    if (rc != LAMPS_OK) return rc;
    if ((rc = ensure_runtime(c)) != LAMPS_OK) return rc;
    if ((rc = wait_for_room(c, out)) != LAMPS_OK) return rc;
    retire_finished(c);
    int32_t *ids = nullptr;
    size_t slots = 0;
    if ((rc = ring_reserve(c, n, &ids, &slots)) != LAMPS_OK) return rc;
    if (n > 0) std::memcpy(ids, block_ids, (size_t)n * sizeof(int32_t));
    hipEvent_t ev;
    if ((rc = new_event(c, &ev)) != LAMPS_OK) {
        c->ring_head -= slots;                      // nothing reads the reserved slots yet
        return rc;
    }

    hipStream_t st = out ? c->os : c->is;
    const size_t total = (size_t)n * c->d.block_bytes;
    Ticket t{ev, slots, host, host + total, out, {}, 0};
    auto enqueue = [&]() -> int {
        int rc = fence_behind_compute(c, st);
        if (rc != LAMPS_OK) return rc;
        if ((rc = wait_guards(c, st, out ? c->in_guard : c->out_guard, block_ids, n)) != LAMPS_OK) return rc;
        if ((rc = wait_host_overlap(c, st, host, host + total, !out)) != LAMPS_OK) return rc;
        return n > 0 ? enqueue_layer_steps(c, out, host, ids, n, st, &t) : LAMPS_OK;
    };
    return file_ticket(c, enqueue(), st, t, out ? c->out_guard : c->in_guard, block_ids, n, ticket);
}

}  // namespace

namespace lamps {

const char *decode_geometry(const lamps_config *cfg, DecodeArgs *a)
{
    Derived d;
    if (const char *why = derive(cfg, &d)) return why;
    *a = DecodeArgs{};
    fill_geometry(*cfg, d, a);
    return nullptr;
}

void set_thread_error(const char *text) { thread_error(text); }

}  // namespace lamps

extern "C" {

size_t lamps_kv_bytes_per_token(const lamps_config *cfg)
{
    Derived d;
    if (derive(cfg, &d)) return 0;
    return 2 * (size_t)cfg->num_layers * cfg->num_kv_heads * cfg->head_dim * d.elem;
}

int lamps_kv_layout(const lamps_config *cfg)
{
    try {
        Derived d;
        if (derive(cfg, &d)) return LAMPS_ERR_INVALID;
        return lamps::decode_uses_tiled_layout(cfg->dtype == LAMPS_BF16, cfg->num_q_heads / cfg->num_kv_heads)
                   ? LAMPS_LAYOUT_TILED
                   : LAMPS_LAYOUT_PLAIN;
    }
    LAMPS_CATCH_NOCTX
}

size_t lamps_block_bytes(const lamps_config *cfg)
{
    Derived d;
    return derive(cfg, &d) ? 0 : d.block_bytes;
}

size_t lamps_pool_bytes(const lamps_config *cfg)
{
    Derived d;
    return derive(cfg, &d) ? 0 : d.pool_bytes;
}

size_t lamps_workspace_bytes(const lamps_config *cfg)
{
    Derived d;
    return derive(cfg, &d) ? 0 : d.workspace_bytes;
}

int lamps_create(const lamps_config *cfg, void *k_pool, void *v_pool, void *workspace,
                 void *compute_stream, void *swap_out_stream, void *swap_in_stream, lamps_ctx **out)
{
    try {
        Derived d;
        if (!out) {
            thread_error("lamps_create: out is null");
            return LAMPS_ERR_INVALID;
        }
        *out = nullptr;
        if (const char *why = derive(cfg, &d)) {
            thread_error("lamps_create: ", why);
            return LAMPS_ERR_INVALID;
        }
        if (!k_pool || !v_pool || !workspace) {
            thread_error("lamps_create: k_pool, v_pool and workspace must be non-null");
            return LAMPS_ERR_INVALID;
        }
        if (((uintptr_t)k_pool | (uintptr_t)v_pool | (uintptr_t)workspace) & 15) {
            thread_error("lamps_create: pools and workspace must be 16-byte aligned");
            return LAMPS_ERR_INVALID;
        }
        std::unique_ptr<lamps_ctx> c(new (std::nothrow) lamps_ctx());   // freed if a container below throws
        if (!c) {
            thread_error("lamps_create: out of host memory");
            return LAMPS_ERR_NOMEM;
        }
        c->cfg = *cfg;
        c->d = d;
        c->k_pool = static_cast<char *>(k_pool);
        c->v_pool = static_cast<char *>(v_pool);
        char *ws = static_cast<char *>(workspace);
        c->partials = reinterpret_cast<float *>(ws);
        c->share_info = reinterpret_cast<int4 *>(ws + align256(d.partial_bytes));
        c->aux = reinterpret_cast<int32_t *>(ws + align256(d.partial_bytes) + align256(d.prefix_bytes));
        c->stage_out = ws + align256(d.partial_bytes) + align256(d.prefix_bytes) + align256(d.aux_bytes);
        c->stage_in = c->stage_out + align256(d.staging_bytes);
        c->cs = static_cast<hipStream_t>(compute_stream);
        c->os = static_cast<hipStream_t>(swap_out_stream);
        c->is = static_cast<hipStream_t>(swap_in_stream);
        const int nb = cfg->num_blocks;
        c->free_stack.resize(nb);
        for (int i = 0; i < nb; ++i) c->free_stack[i] = nb - 1 - i;   // top of stack = id 0
        c->allocated.assign(nb, 0);
        c->out_guard.assign(nb, 0);
        c->in_guard.assign(nb, 0);
        c->mark.assign(nb, 0);
        *out = c.release();
        g_thread_error[0] = 0;
        return LAMPS_OK;
    }
    LAMPS_CATCH_NOCTX
}

int lamps_destroy(lamps_ctx *c)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        int rc = LAMPS_OK;
        while (!c->tickets.empty()) {
            if (hipEventSynchronize(c->tickets.front().ev) != hipSuccess) rc = LAMPS_ERR_HIP;
            (void)hipEventDestroy(c->tickets.front().ev);
            for (hipEvent_t e : c->tickets.front().step_ev) (void)hipEventDestroy(e);
            c->tickets.pop_front();
        }
        for (hipEvent_t e : c->spare_events) (void)hipEventDestroy(e);
        if (c->fence) (void)hipEventDestroy(c->fence);
        if (c->ring) (void)hipHostFree(c->ring);
        delete c;
        return rc;
    }
    LAMPS_CATCH(c)
}

int lamps_decode_attn(lamps_ctx *c, int32_t layer, int32_t batch, const void *q,
                      const int32_t *block_table, const int32_t *ctx_lens,
                      const uint8_t *running_mask, void *out)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!q || !block_table || !ctx_lens || !running_mask || !out)
            return fail(c, LAMPS_ERR_INVALID, "lamps_decode_attn: null argument");
        if (layer < 0 || layer >= c->cfg.num_layers)
            return fail(c, LAMPS_ERR_RANGE, "lamps_decode_attn: layer out of range");
        if (batch < 0 || batch > c->cfg.max_batch)
            return fail(c, LAMPS_ERR_RANGE, "lamps_decode_attn: batch out of range");
        if (batch == 0) return LAMPS_OK;
        lamps::DecodeArgs a;
        fill_decode_args(c, &a, layer, batch, q, block_table, ctx_lens, running_mask, out);
        LAMPS_HIP(lamps::launch_decode(a, c->cs));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_validate_args(lamps_ctx *c, int32_t batch, const int32_t *block_table, const int32_t *ctx_lens,
                        const uint8_t *running_mask, int32_t *report)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!block_table || !ctx_lens || !running_mask)
            return fail(c, LAMPS_ERR_INVALID, "lamps_validate_args: null argument");
        if (batch < 0 || batch > c->cfg.max_batch)
            return fail(c, LAMPS_ERR_RANGE, "lamps_validate_args: batch out of range");
        int32_t res[4] = {0, -1, 0, 0};
        if (batch > 0) {
            LAMPS_HIP(lamps::launch_validate(block_table, ctx_lens, running_mask, batch, c->cfg.max_blocks_per_req,
                                             c->cfg.block_size, c->cfg.num_blocks, c->aux, c->cs));
            LAMPS_HIP(hipMemcpyAsync(res, c->aux, sizeof res, hipMemcpyDeviceToHost, c->cs));
            LAMPS_HIP(hipStreamSynchronize(c->cs));
        }
        if (report) std::memcpy(report, res, sizeof res);
        if (res[0] == 0) return LAMPS_OK;
        char text[160];
        std::snprintf(text, sizeof text,
                      res[2] == 1 ? "lamps_validate_args: %d bad request(s); request %d has context length %d"
                                  : "lamps_validate_args: %d bad request(s); request %d uses block id %d",
                      res[0], res[1], res[3]);
        return fail(c, LAMPS_ERR_RANGE, text);
    }
    LAMPS_CATCH(c)
}

int lamps_kv_append(lamps_ctx *c, int32_t layer, int32_t batch, const void *k_new,
                    const void *v_new, const int32_t *block_table, int32_t *ctx_lens,
                    const uint8_t *running_mask, int32_t advance)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!k_new || !v_new || !block_table || !ctx_lens || !running_mask)
            return fail(c, LAMPS_ERR_INVALID, "lamps_kv_append: null argument");
        if (((uintptr_t)k_new | (uintptr_t)v_new) & 15)
            return fail(c, LAMPS_ERR_INVALID, "lamps_kv_append: k_new and v_new must be 16-byte aligned");
        if (layer < 0 || layer >= c->cfg.num_layers)
            return fail(c, LAMPS_ERR_RANGE, "lamps_kv_append: layer out of range");
        if (batch < 0 || batch > c->cfg.max_batch)
            return fail(c, LAMPS_ERR_RANGE, "lamps_kv_append: batch out of range");
        if (batch == 0) return LAMPS_OK;
        lamps::AppendArgs a;
        a.k_new = k_new;
        a.v_new = v_new;
        a.k_pool = c->k_pool;
        a.v_pool = c->v_pool;
        a.block_table = block_table;
        a.ctx_lens = ctx_lens;
        a.running = running_mask;
        a.q_start = nullptr;
        a.batch = batch;
        a.layer = layer;
        a.num_layers = c->cfg.num_layers;
        a.num_kv_heads = c->cfg.num_kv_heads;
        a.head_dim = c->cfg.head_dim;
        a.block_size = c->cfg.block_size;
        a.log2_block_size = c->d.log2_bs;
        a.max_blocks = c->cfg.max_blocks_per_req;
        a.num_blocks = c->cfg.num_blocks;
        a.bf16 = c->cfg.dtype == LAMPS_BF16;
        a.advance = advance != 0;
        const int tiled = lamps::decode_uses_tiled_layout(a.bf16, c->cfg.num_q_heads / c->cfg.num_kv_heads);
        LAMPS_HIP(lamps::launch_kv_append(a, tiled, c->cs));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_kv_append_tokens(lamps_ctx *c, int32_t layer, int32_t n_req, int32_t total_tokens,
                           const void *k_new, const void *v_new, const int32_t *q_start,
                           const int32_t *block_table, const int32_t *ctx_lens)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!k_new || !v_new || !q_start || !block_table || !ctx_lens)
            return fail(c, LAMPS_ERR_INVALID, "lamps_kv_append_tokens: null argument");
        if (((uintptr_t)k_new | (uintptr_t)v_new) & 15)
            return fail(c, LAMPS_ERR_INVALID, "lamps_kv_append_tokens: k_new and v_new must be 16-byte aligned");
        if (layer < 0 || layer >= c->cfg.num_layers)
            return fail(c, LAMPS_ERR_RANGE, "lamps_kv_append_tokens: layer out of range");
        if (n_req < 0 || n_req > c->cfg.max_batch || total_tokens < 0)
            return fail(c, LAMPS_ERR_RANGE, "lamps_kv_append_tokens: n_req / total_tokens out of range");
        if (n_req == 0 || total_tokens == 0) return LAMPS_OK;
        lamps::AppendArgs a;
        a.k_new = k_new;
        a.v_new = v_new;
        a.k_pool = c->k_pool;
        a.v_pool = c->v_pool;
        a.block_table = block_table;
        a.ctx_lens = const_cast<int32_t *>(ctx_lens);     // the token form only reads it
        a.running = nullptr;
        a.q_start = q_start;
        a.batch = n_req;
        a.layer = layer;
        a.num_layers = c->cfg.num_layers;
        a.num_kv_heads = c->cfg.num_kv_heads;
        a.head_dim = c->cfg.head_dim;
        a.block_size = c->cfg.block_size;
        a.log2_block_size = c->d.log2_bs;
        a.max_blocks = c->cfg.max_blocks_per_req;
        a.num_blocks = c->cfg.num_blocks;
        a.bf16 = c->cfg.dtype == LAMPS_BF16;
        a.advance = 0;
        const int tiled = lamps::decode_uses_tiled_layout(a.bf16, c->cfg.num_q_heads / c->cfg.num_kv_heads);
        LAMPS_HIP(lamps::launch_kv_append_tokens(a, total_tokens, tiled, c->cs));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_prefill_attn(lamps_ctx *c, int32_t layer, int32_t n_req, int32_t total_tokens,
                       int32_t max_new_tokens, const void *q, const int32_t *q_start,
                       const int32_t *block_table, const int32_t *ctx_lens, void *out)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!q || !q_start || !block_table || !ctx_lens || !out)
            return fail(c, LAMPS_ERR_INVALID, "lamps_prefill_attn: null argument");
        if (((uintptr_t)q | (uintptr_t)out) & 15)
            return fail(c, LAMPS_ERR_INVALID, "lamps_prefill_attn: q and out must be 16-byte aligned");
        if (layer < 0 || layer >= c->cfg.num_layers)
            return fail(c, LAMPS_ERR_RANGE, "lamps_prefill_attn: layer out of range");
        if (n_req < 0 || n_req > c->cfg.max_batch || total_tokens < 0)
            return fail(c, LAMPS_ERR_RANGE, "lamps_prefill_attn: n_req / total_tokens out of range");
        if (n_req == 0 || total_tokens == 0) return LAMPS_OK;
        lamps::PrefillArgs p;
        fill_decode_args(c, &p.d, layer, n_req, q, block_table, ctx_lens, nullptr, out);
        p.q_start = q_start;
        p.total_tokens = total_tokens;
        p.max_new_tokens = max_new_tokens > 0 && max_new_tokens < total_tokens ? max_new_tokens : total_tokens;
        p.force_rows = max_new_tokens < 0;
        LAMPS_HIP(lamps::launch_prefill(p, c->cs));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_swap_out(lamps_ctx *c, const int32_t *block_ids, int32_t n, void *host_buf,
                   uint64_t *ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket || (n > 0 && !host_buf))
            return fail(c, LAMPS_ERR_INVALID, "lamps_swap_out: null argument");
        int rc = check_ids(c, block_ids, n, "lamps_swap_out");
        if (rc != LAMPS_OK) return rc;
        void *host_dev = nullptr;
        if (c->d.zero_copy &&
            (rc = mapped_host(c, host_buf, (size_t)n * c->d.block_bytes, "lamps_swap_out", &host_dev)) != LAMPS_OK)
            return rc;
        if ((rc = ensure_runtime(c)) != LAMPS_OK) return rc;
        if ((rc = wait_for_room(c, true)) != LAMPS_OK) return rc;
        retire_finished(c);
        int32_t *ids = nullptr;
        size_t slots = 0;
        if (!c->d.direct_copy) {                        // the gather kernel reads the ids from the pinned ring
            if ((rc = ring_reserve(c, n, &ids, &slots)) != LAMPS_OK) return rc;
            if (n > 0) std::memcpy(ids, block_ids, (size_t)n * sizeof(int32_t));
        }
        hipEvent_t ev;
        if ((rc = new_event(c, &ev)) != LAMPS_OK) {
            c->ring_head -= slots;                      // nothing reads the reserved slots yet
            return rc;
        }

        char *host = static_cast<char *>(host_buf);
        const size_t total = (size_t)n * c->d.block_bytes;
        Ticket t{ev, slots, host, host + total, true, {}, 0};
        auto enqueue = [&]() -> int {
            // the copy reads what the compute stream (and any earlier swap-in) wrote
            int rc = fence_behind_compute(c, c->os);
            if (rc != LAMPS_OK) return rc;
            if ((rc = wait_guards(c, c->os, c->in_guard, block_ids, n)) != LAMPS_OK) return rc;
            if ((rc = wait_host_overlap(c, c->os, host, host + total, false)) != LAMPS_OK) return rc;

            if (c->d.direct_copy) {
                // each block is two long contiguous runs: the copy engines take them as they are
                for (int32_t i = 0; i < n; ++i) {
                    const size_t at = (size_t)block_ids[i] * c->d.half_bytes;
                    LAMPS_HIP(hipMemcpyAsync(host + (size_t)i * c->d.block_bytes, c->k_pool + at, c->d.half_bytes,
                                             hipMemcpyDeviceToHost, c->os));
                    LAMPS_HIP(hipMemcpyAsync(host + (size_t)i * c->d.block_bytes + c->d.half_bytes, c->v_pool + at,
                                             c->d.half_bytes, hipMemcpyDeviceToHost, c->os));
                }
            } else if (c->d.zero_copy) {
                LAMPS_HIP(lamps::launch_gather_host(c->k_pool, c->v_pool, ids, n, c->d.half_bytes, host_dev,
                                                    c->d.zero_copy, c->os));
            } else {
                for (int32_t done = 0; done < n; done += c->d.blocks_per_chunk) {
                    const int32_t cnt = std::min<int32_t>(c->d.blocks_per_chunk, n - done);
                    LAMPS_HIP(lamps::launch_gather(c->k_pool, c->v_pool, ids + done, cnt, c->d.half_bytes,
                                                   c->stage_out, c->os));
                    LAMPS_HIP(hipMemcpyAsync(host + (size_t)done * c->d.block_bytes, c->stage_out,
                                             (size_t)cnt * c->d.block_bytes, hipMemcpyDeviceToHost, c->os));
                }
            }
            return LAMPS_OK;
        };
        return file_ticket(c, enqueue(), c->os, t, c->out_guard, block_ids, n, ticket);
    }
    LAMPS_CATCH(c)
}

int lamps_swap_in(lamps_ctx *c, const void *host_buf, const int32_t *block_ids, int32_t n,
                  uint64_t *ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket || (n > 0 && !host_buf))
            return fail(c, LAMPS_ERR_INVALID, "lamps_swap_in: null argument");
        int rc = check_ids(c, block_ids, n, "lamps_swap_in");
        if (rc != LAMPS_OK) return rc;
        void *host_dev = nullptr;
        if (c->d.zero_copy &&
            (rc = mapped_host(c, host_buf, (size_t)n * c->d.block_bytes, "lamps_swap_in", &host_dev)) != LAMPS_OK)
            return rc;
        if ((rc = ensure_runtime(c)) != LAMPS_OK) return rc;
        if ((rc = wait_for_room(c, false)) != LAMPS_OK) return rc;
        retire_finished(c);
        int32_t *ids = nullptr;
        size_t slots = 0;
        if (!c->d.direct_copy) {
            if ((rc = ring_reserve(c, n, &ids, &slots)) != LAMPS_OK) return rc;
            if (n > 0) std::memcpy(ids, block_ids, (size_t)n * sizeof(int32_t));
        }
        hipEvent_t ev;
        if ((rc = new_event(c, &ev)) != LAMPS_OK) {
            c->ring_head -= slots;                      // nothing reads the reserved slots yet
            return rc;
        }

        const char *host = static_cast<const char *>(host_buf);
        const size_t total = (size_t)n * c->d.block_bytes;
        Ticket t{ev, slots, host, host + total, false, {}, 0};
        auto enqueue = [&]() -> int {
            // the scatter overwrites blocks: earlier compute-stream readers and an
            // unfinished swap-out of the same blocks go first
            int rc = fence_behind_compute(c, c->is);
            if (rc != LAMPS_OK) return rc;
            if ((rc = wait_guards(c, c->is, c->out_guard, block_ids, n)) != LAMPS_OK) return rc;
            if ((rc = wait_host_overlap(c, c->is, host, host + total, true)) != LAMPS_OK) return rc;

            if (c->d.direct_copy) {
                for (int32_t i = 0; i < n; ++i) {
                    const size_t at = (size_t)block_ids[i] * c->d.half_bytes;
                    LAMPS_HIP(hipMemcpyAsync(c->k_pool + at, host + (size_t)i * c->d.block_bytes, c->d.half_bytes,
                                             hipMemcpyHostToDevice, c->is));
                    LAMPS_HIP(hipMemcpyAsync(c->v_pool + at, host + (size_t)i * c->d.block_bytes + c->d.half_bytes,
                                             c->d.half_bytes, hipMemcpyHostToDevice, c->is));
                }
            } else if (c->d.zero_copy) {
                LAMPS_HIP(lamps::launch_scatter_host(c->k_pool, c->v_pool, ids, n, c->d.half_bytes, host_dev,
                                                     c->d.zero_copy, c->is));
            } else {
                for (int32_t done = 0; done < n; done += c->d.blocks_per_chunk) {
                    const int32_t cnt = std::min<int32_t>(c->d.blocks_per_chunk, n - done);
                    LAMPS_HIP(hipMemcpyAsync(c->stage_in, host + (size_t)done * c->d.block_bytes,
                                             (size_t)cnt * c->d.block_bytes, hipMemcpyHostToDevice, c->is));
                    LAMPS_HIP(lamps::launch_scatter(c->k_pool, c->v_pool, ids + done, cnt, c->d.half_bytes,
                                                    c->stage_in, c->is));
                }
            }
            return LAMPS_OK;
        };
        return file_ticket(c, enqueue(), c->is, t, c->in_guard, block_ids, n, ticket);
    }
    LAMPS_CATCH(c)
}

int lamps_swap_out_layered(lamps_ctx *c, const int32_t *block_ids, int32_t n, void *host_buf, uint64_t *ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        return swap_layered(c, true, static_cast<char *>(host_buf), block_ids, n, ticket, "lamps_swap_out_layered");
    }
    LAMPS_CATCH(c)
}

int lamps_swap_in_layered(lamps_ctx *c, const void *host_buf, const int32_t *block_ids, int32_t n,
                          uint64_t *ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        return swap_layered(c, false, const_cast<char *>(static_cast<const char *>(host_buf)), block_ids, n, ticket,
                            "lamps_swap_in_layered");
    }
    LAMPS_CATCH(c)
}

int lamps_compute_wait_layer(lamps_ctx *c, uint64_t ticket, int32_t layer)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket_known(c, ticket)) return fail(c, LAMPS_ERR_RANGE, "lamps_compute_wait_layer: unknown ticket");
        if (layer < 0 || layer >= c->cfg.num_layers)
            return fail(c, LAMPS_ERR_RANGE, "lamps_compute_wait_layer: layer out of range");
        if (ticket_done(c, ticket)) return LAMPS_OK;
        const Ticket &t = c->tickets[ticket - c->base_ticket];
        hipEvent_t e = t.ev;
        if (t.layers_per_step > 0 && (size_t)(layer / t.layers_per_step) < t.step_ev.size())
            e = t.step_ev[layer / t.layers_per_step];
        if (hipEventQuery(e) != hipSuccess) LAMPS_HIP(hipStreamWaitEvent(c->cs, e, 0));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_set_swap_fence(lamps_ctx *c, int32_t enabled)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        c->swap_fence = enabled != 0;
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_swap_wait_compute(lamps_ctx *c)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        int rc = ensure_runtime(c);
        if (rc != LAMPS_OK) return rc;
        LAMPS_HIP(hipEventRecord(c->fence, c->cs));
        LAMPS_HIP(hipStreamWaitEvent(c->os, c->fence, 0));
        LAMPS_HIP(hipStreamWaitEvent(c->is, c->fence, 0));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_ticket_query(lamps_ctx *c, uint64_t ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket_known(c, ticket)) return fail(c, LAMPS_ERR_RANGE, "lamps_ticket_query: unknown ticket");
        return ticket_done(c, ticket) ? LAMPS_OK : LAMPS_ERR_BUSY;
    }
    LAMPS_CATCH(c)
}

int lamps_ticket_wait(lamps_ctx *c, uint64_t ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket_known(c, ticket)) return fail(c, LAMPS_ERR_RANGE, "lamps_ticket_wait: unknown ticket");
        if (ticket >= c->base_ticket) LAMPS_HIP(hipEventSynchronize(ticket_event(c, ticket)));
        retire_finished(c);
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_compute_wait(lamps_ctx *c, uint64_t ticket)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (!ticket_known(c, ticket)) return fail(c, LAMPS_ERR_RANGE, "lamps_compute_wait: unknown ticket");
        if (!ticket_done(c, ticket)) LAMPS_HIP(hipStreamWaitEvent(c->cs, ticket_event(c, ticket), 0));
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_compute_wait_blocks(lamps_ctx *c, const int32_t *block_ids, int32_t n)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        int rc = check_ids(c, block_ids, n, "lamps_compute_wait_blocks");
        if (rc != LAMPS_OK) return rc;
        if ((rc = wait_guards(c, c->cs, c->out_guard, block_ids, n)) != LAMPS_OK) return rc;
        return wait_guards(c, c->cs, c->in_guard, block_ids, n);
    }
    LAMPS_CATCH(c)
}

int lamps_alloc_blocks(lamps_ctx *c, int32_t n, int32_t *block_ids_out)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        if (n < 0 || (n > 0 && !block_ids_out))
            return fail(c, LAMPS_ERR_INVALID, "lamps_alloc_blocks: bad argument");
        if ((size_t)n > c->free_stack.size())
            return fail(c, LAMPS_ERR_NOMEM, "lamps_alloc_blocks: not enough free blocks");
        for (int32_t i = 0; i < n; ++i) {
            block_ids_out[i] = c->free_stack.back();
            c->free_stack.pop_back();
            c->allocated[block_ids_out[i]] = 1;
        }
        // A popped block may still be the source of an unfinished swap-out.  Its
        // guard stays in place: lamps_swap_in orders itself behind it, and a caller
        // that writes the block from the compute stream asks for the same with
        // lamps_compute_wait_blocks.  Nothing is made to wait here, so decode steps
        // of other requests keep running while the copy drains.
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_free_blocks(lamps_ctx *c, const int32_t *block_ids, int32_t n)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        int rc = check_ids(c, block_ids, n, "lamps_free_blocks");
        if (rc != LAMPS_OK) return rc;
        for (int32_t i = 0; i < n; ++i) {
            c->allocated[block_ids[i]] = 0;
            c->free_stack.push_back(block_ids[i]);
        }
        return LAMPS_OK;
    }
    LAMPS_CATCH(c)
}

int lamps_num_free(lamps_ctx *c)
{
    try {
        if (!c) return LAMPS_ERR_INVALID;
        return (int)c->free_stack.size();
    }
    LAMPS_CATCH(c)
}

const char *lamps_last_error(lamps_ctx *c) { return c ? c->err.c_str() : g_thread_error; }

}  // extern "C"
