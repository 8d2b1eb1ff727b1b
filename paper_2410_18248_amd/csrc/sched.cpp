// The LAMPS scheduler (arXiv 2410.18248): equations (1)-(3), the memory-over-time
// rank of Section 4.2 / 4.3 and Algorithm 1, behind the C ABI of lamps_sched.h.
//
// Host code only.  The scheduler owns one small state machine per request
// (new -> waiting <-> in an API call -> done) and is stepped once per decode
// iteration; what an iteration costs comes either from the caller's clock (the
// GPU executed it) or from the linear cost model.  Requests live in one array
// sorted by (arrival, id); the waiting queue and the set of requests in an API
// call are index lists into it, so an iteration touches only those.
#include "lamps_sched.h"

#include <algorithm>
#include <cstring>
#include <new>
#include <unordered_map>
#include <vector>

#include "lamps.h"

namespace {

enum State : int32_t { kNew = 0, kWaiting = 1, kInApi = 2, kDone = 3 };

struct Req {
    int64_t id;
    double arrival, priority;
    int32_t prompt;
    std::vector<lamps_segment> seg;     // handling filled in when decided
    State state = kNew;
    int32_t cur = 0;                    // current segment
    int64_t done_in_seg = 0;
    bool started = false;               // current segment has been admitted once
    int64_t ctx = 0;                    // logical context, tokens
    int64_t held = 0;                   // tokens of it in GPU memory
    int64_t pending_recompute = 0;      // tokens to run through the model before generating
    int64_t pending_swapin = 0;
    double api_end = 0.0;
    int32_t starv = 0;
    bool prioritized = false;
    bool has_score = false;
    double score = 0.0;
    int64_t score_iter = 0;
    double completion = -1.0, first_token = -1.0;
};

// In the worked example's units (Section 3.1) a recomputation takes one iteration and a swap none.
double cost_t_fwd(const lamps_cost_model &c, double C) { return c.unit ? 1.0 : c.fwd_a + c.fwd_b * C; }
double cost_t_swap(const lamps_cost_model &c, double C) { return c.unit ? 0.0 : c.sw_a + c.sw_b * C; }
double cost_iteration(const lamps_cost_model &c, int64_t ctx_tokens, int64_t recomputed, int64_t swapped)
{
    if (c.unit) return 1.0;
    double t = c.it_a + c.it_b * (double)ctx_tokens + c.fwd_b * (double)recomputed;
    if (c.swap_stalls && swapped > 0) t += c.sw_a + c.sw_b * (double)swapped;
    return t;
}

// sum_{j=1..n} (base + j), exact in integers
int64_t ramp(int64_t base, int64_t n) { return n * base + n * (n + 1) / 2; }

}  // namespace

// No exception crosses the C ABI: the request table, the queues and the maps may throw
// std::bad_alloc.
#define LAMPS_SCHED_CATCH                                   \
    catch (const std::bad_alloc &) { return LAMPS_ERR_NOMEM; } \
    catch (...) { return LAMPS_ERR_INVALID; }

struct lamps_sched {
    lamps_sched_config cfg;
    std::vector<Req> reqs;              // sorted by (arrival, id) once the first batch is formed
    std::unordered_map<int64_t, size_t> by_id;
    bool sorted = false;
    size_t next_new = 0;                // first request not yet arrived
    std::vector<size_t> waiting, in_api, batch;
    std::vector<char> in_batch;
    size_t done = 0;
    double now = 0.0;
    int64_t iteration = 0, total_held = 0, peak = 0, preemptions = 0;
    bool batch_pending = false;
    std::vector<int64_t> discarded;     // requests discarded for lack of memory, not yet reported

    // Section 4.2: the handling strategy of a segment's API call is fixed, from the
    // predicted context at the call and the call's duration, before the segment runs.
    void decide(Req &r)
    {
        lamps_segment &s = r.seg[r.cur];
        if (s.api_duration < 0 || s.handling != LAMPS_HANDLING_AUTO) return;
        const int64_t base = r.ctx ? r.ctx : r.pending_recompute;
        const double C = (double)(base + (s.n_out - r.done_in_seg));
        s.handling = lamps_handling_strategy(s.api_duration, C, cfg.c_other, cfg.bytes_per_token,
                                             cost_t_fwd(cfg.cost, C), cost_t_swap(cfg.cost, C));
    }

    void return_from_api(Req &r)
    {
        const lamps_segment &s = r.seg[r.cur];
        if (s.handling == LAMPS_DISCARD)
            r.pending_recompute = r.ctx;            // everything is run through the model again
        else if (s.handling == LAMPS_SWAP)
            r.pending_swapin = r.ctx;
        r.pending_recompute += s.api_response;      // the API's response is new context
        r.ctx += s.api_response;
        ++r.cur;
        r.done_in_seg = 0;
        r.started = false;
        r.has_score = false;
        r.state = kWaiting;
        decide(r);
    }

    int64_t remaining_tokens(const Req &r) const
    {
        int64_t rem = r.pending_recompute + (r.seg[r.cur].n_out - r.done_in_seg);
        for (size_t k = r.cur + 1; k < r.seg.size(); ++k) rem += r.seg[k].n_out;
        return rem;
    }

    double rank(const Req &r) const
    {
        switch (cfg.policy) {
        case LAMPS_POLICY_FCFS: return 0.0;         // ties: arrival, id
        case LAMPS_POLICY_FIXED: return r.priority;
        case LAMPS_POLICY_SJF: return (double)remaining_tokens(r);
        case LAMPS_POLICY_SJF_TOTAL: {
            double api = 0.0;
            for (size_t k = r.cur; k < r.seg.size(); ++k)
                if (r.seg[k].api_duration >= 0) api += r.seg[k].api_duration;
            return (double)remaining_tokens(r) + api / cost_iteration(cfg.cost, 0, 0, 0);
        }
        default: break;
        }
        // memory over time of the current segment, its API call handled as decided, and
        // the tokens that follow the call
        const lamps_segment &s = r.seg[r.cur];
        const int64_t c0 = r.ctx ? r.ctx : r.pending_recompute;
        const int64_t n1 = s.n_out - r.done_in_seg;
        const double tau = cost_iteration(cfg.cost, 0, 0, 0);
        if (s.api_duration < 0)
            return lamps_memory_over_time(LAMPS_PRESERVE, c0, n1, 0.0, 0, 0, tau, 0.0, 0.0);
        const double C = (double)(c0 + n1);
        return lamps_memory_over_time(s.handling, c0, n1, s.api_duration, s.api_response,
                                      r.seg[r.cur + 1].n_out, tau, cost_t_fwd(cfg.cost, C),
                                      cost_t_swap(cfg.cost, C));
    }

    int64_t need(const Req &r) const
    {
        if (!r.started) return r.pending_swapin + r.pending_recompute + (r.seg[r.cur].n_out - r.done_in_seg);
        if (r.pending_recompute > 0) return std::min<int64_t>(cfg.recompute_chunk, r.pending_recompute);
        return 1;
    }
};

extern "C" {

double lamps_waste_preserve(double t_int, double c_i, double m) { return t_int * c_i * m; }

double lamps_waste_discard(double t_fwd_ci, double c_i, double c_other, double m)
{
    return t_fwd_ci * c_i * m + t_fwd_ci * c_other * m;
}

double lamps_waste_swap(double t_swap_ci, double c_batch, double m) { return 2 * t_swap_ci * c_batch * m; }

int lamps_handling_strategy(double t_int, double c_i, double c_other, double m, double t_fwd_ci,
                            double t_swap_ci)
{
    const double w[3] = {lamps_waste_preserve(t_int, c_i, m), lamps_waste_discard(t_fwd_ci, c_i, c_other, m),
                         lamps_waste_swap(t_swap_ci, c_i + c_other, m)};
    int best = 0;
    for (int k = 1; k < 3; ++k)
        if (w[k] < w[best]) best = k;
    return best;
}

double lamps_memory_over_time(int strategy, int64_t c0, int64_t n1, double t_int, int64_t rho, int64_t n2,
                              double tau, double t_fwd_c, double t_swap_c)
{
    const int64_t C = c0 + n1;
    const double pre = tau * (double)ramp(c0, n1);
    const double post = tau * (double)ramp(C + rho, n2);
    double mid;
    if (strategy == LAMPS_PRESERVE)
        mid = t_int * (double)C;
    else if (strategy == LAMPS_DISCARD)
        mid = t_fwd_c * (double)C;
    else
        mid = 2 * t_swap_c * (double)C;
    return pre + mid + post;
}

int lamps_sched_create(const lamps_sched_config *cfg, lamps_sched **out)
{
    try {
        if (!cfg || !out) return LAMPS_ERR_INVALID;
        *out = nullptr;
        if (cfg->policy < LAMPS_POLICY_FCFS || cfg->policy > LAMPS_POLICY_FIXED || cfg->max_batch < 1 ||
            cfg->memory_tokens < 1 || cfg->starvation_threshold < 1 || cfg->score_refresh < 1 ||
            cfg->recompute_chunk < 1 || !(cfg->c_other >= 0) || !(cfg->bytes_per_token > 0))
            return LAMPS_ERR_INVALID;
        if (!cfg->cost.unit && !(cfg->cost.it_a + cfg->cost.it_b > 0)) return LAMPS_ERR_INVALID;
        lamps_sched *s = new (std::nothrow) lamps_sched();
        if (!s) return LAMPS_ERR_NOMEM;
        s->cfg = *cfg;
        *out = s;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_destroy(lamps_sched *s)
{
    try {
        if (!s) return LAMPS_ERR_INVALID;
        delete s;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_add(lamps_sched *s, int64_t id, double arrival, int32_t prompt_tokens,
                    const lamps_segment *segments, int32_t n_segments, double priority)
{
    try {
        if (!s || !segments || n_segments < 1 || prompt_tokens < 0 || s->batch_pending) return LAMPS_ERR_INVALID;
        for (int32_t k = 0; k < n_segments; ++k) {
            const bool last = k == n_segments - 1;
            if (segments[k].n_out < 1 || segments[k].api_response < 0) return LAMPS_ERR_INVALID;
            if (last != (segments[k].api_duration < 0)) return LAMPS_ERR_INVALID;
            if (segments[k].handling < LAMPS_HANDLING_AUTO || segments[k].handling > LAMPS_SWAP)
                return LAMPS_ERR_INVALID;
        }
        if (s->by_id.count(id)) return LAMPS_ERR_DUP;
        if (s->sorted && arrival < s->now) return LAMPS_ERR_INVALID;    // no arrivals in the past
        Req r;
        r.id = id;
        r.arrival = arrival;
        r.priority = priority;
        r.prompt = prompt_tokens;
        r.seg.assign(segments, segments + n_segments);
        r.pending_recompute = prompt_tokens;
        s->reqs.push_back(std::move(r));
        s->by_id[id] = s->reqs.size() - 1;
        s->sorted = false;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_next_batch(lamps_sched *s, lamps_batch_entry *out, int32_t cap, int32_t *n)
{
    try {
        if (!s || !out || !n || s->batch_pending) return LAMPS_ERR_INVALID;
        if (cap < s->cfg.max_batch) return LAMPS_ERR_RANGE;
        if (!s->sorted) {
            // (re)establish the (arrival, id) order; indices held in the lists are remapped
            std::vector<size_t> order(s->reqs.size());
            for (size_t i = 0; i < order.size(); ++i) order[i] = i;
            std::sort(order.begin(), order.end(), [&](size_t a, size_t b) {
                const Req &x = s->reqs[a], &y = s->reqs[b];
                return x.arrival != y.arrival ? x.arrival < y.arrival : x.id < y.id;
            });
            std::vector<size_t> where(order.size());
            std::vector<Req> sorted;
            sorted.reserve(order.size());
            for (size_t i = 0; i < order.size(); ++i) {
                where[order[i]] = i;
                sorted.push_back(std::move(s->reqs[order[i]]));
            }
            s->reqs.swap(sorted);
            for (size_t &w : s->waiting) w = where[w];
            for (size_t &w : s->in_api) w = where[w];
            for (auto &kv : s->by_id) kv.second = where[kv.second];
            s->next_new = 0;
            s->in_batch.assign(s->reqs.size(), 0);
            s->sorted = true;
        }
        const lamps_sched_config &cfg = s->cfg;
        for (;;) {
            if (s->done == s->reqs.size()) {
                *n = 0;
                return LAMPS_OK;
            }
            // new requests get their handling strategy and enter the waiting queue
            // (requests added later with an arrival equal to the current time may sort in
            // front of ones that are already past this stage; those are skipped)
            while (s->next_new < s->reqs.size() &&
                   (s->reqs[s->next_new].state != kNew || s->reqs[s->next_new].arrival <= s->now)) {
                Req &r = s->reqs[s->next_new];
                if (r.state == kNew) {
                    s->decide(r);
                    r.state = kWaiting;
                    s->waiting.push_back(s->next_new);
                }
                ++s->next_new;
            }
            // requests whose API call has finished re-enter it
            for (size_t k = 0; k < s->in_api.size();) {
                Req &r = s->reqs[s->in_api[k]];
                if (r.api_end <= s->now) {
                    s->return_from_api(r);
                    s->waiting.push_back(s->in_api[k]);
                    s->in_api[k] = s->in_api.back();
                    s->in_api.pop_back();
                } else {
                    ++k;
                }
            }
            // scores (cached, refreshed every score_refresh iterations), then the sort
            for (size_t w : s->waiting) {
                Req &r = s->reqs[w];
                if (!r.has_score || s->iteration - r.score_iter >= cfg.score_refresh) {
                    r.score = s->rank(r);
                    r.has_score = true;
                    r.score_iter = s->iteration;
                }
            }
            auto by_rank = [&](size_t a, size_t b) {
                const Req &x = s->reqs[a], &y = s->reqs[b];
                if (x.prioritized != y.prioritized) return x.prioritized;
                if (x.score != y.score) return x.score < y.score;
                if (x.arrival != y.arrival) return x.arrival < y.arrival;
                return x.id < y.id;
            };
            std::sort(s->waiting.begin(), s->waiting.end(), by_rank);
            // the running batch; `count` = this is the pass that moves the starvation counters
            auto form = [&](bool count) {
                int64_t free_tokens = cfg.memory_tokens - s->total_held;
                for (size_t w : s->batch) s->in_batch[w] = 0;
                s->batch.clear();
                for (size_t w : s->waiting) {
                    Req &r = s->reqs[w];
                    const int64_t nd = s->need(r);
                    if ((int32_t)s->batch.size() < cfg.max_batch && nd <= free_tokens) {
                        s->batch.push_back(w);
                        s->in_batch[w] = 1;
                        free_tokens -= nd;
                        if (count) r.starv = 0;
                    } else if (count) {
                        ++r.starv;
                    }
                }
            };
            form(true);
            // Algorithm 1's second loop: a request left out often enough is tagged and goes to the
            // head of the queue for this very iteration (Section 4.4): the batch is formed once more
            bool tagged = false;
            for (size_t w : s->waiting) {
                Req &r = s->reqs[w];
                if (!s->in_batch[w] && !r.prioritized && r.starv >= cfg.starvation_threshold) {
                    r.prioritized = true;
                    r.starv = 0;
                    tagged = true;
                }
            }
            if (tagged) {
                std::sort(s->waiting.begin(), s->waiting.end(), by_rank);
                form(false);
            }
            if (!s->batch.empty()) break;
            // Nothing fits.  If memory is held by waiting requests none of which can grow, the
            // worst-ranked holder is discarded and recomputes once memory is there (Section 4.3 on
            // full memory); otherwise the engine idles until the next arrival or API return.
            Req *victim = nullptr;
            for (size_t k = s->waiting.size(); k-- > 0;)
                if (s->reqs[s->waiting[k]].held > 0) {
                    victim = &s->reqs[s->waiting[k]];
                    break;
                }
            if (victim) {
                s->total_held -= victim->held;
                victim->held = 0;
                victim->pending_swapin = 0;
                victim->pending_recompute = victim->ctx;
                victim->started = false;
                victim->has_score = false;
                ++s->preemptions;
                s->discarded.push_back(victim->id);
                continue;
            }
            bool have = false;
            double nxt = 0.0;
            for (size_t k : s->in_api)
                if (!have || s->reqs[k].api_end < nxt) nxt = s->reqs[k].api_end, have = true;
            if (s->next_new < s->reqs.size() && (!have || s->reqs[s->next_new].arrival < nxt))
                nxt = s->reqs[s->next_new].arrival, have = true;
            if (!have) return LAMPS_ERR_NOMEM;
            s->now = std::max(s->now, nxt);
        }
        *n = (int32_t)s->batch.size();
        for (int32_t i = 0; i < *n; ++i) {
            const Req &r = s->reqs[s->batch[i]];
            out[i].id = r.id;
            out[i].swap_in = r.pending_swapin;
            out[i].recompute = r.pending_recompute > 0 ? std::min<int64_t>(cfg.recompute_chunk, r.pending_recompute) : 0;
            const int64_t held_after = r.held + r.pending_swapin + (out[i].recompute ? out[i].recompute : 1);
            out[i].context = out[i].recompute ? std::max(r.ctx, held_after) : r.ctx + 1;
        }
        s->batch_pending = true;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_commit(lamps_sched *s, double iteration_time, lamps_sched_event *events, int32_t cap,
                       int32_t *n)
{
    try {
        if (!s || !events || !n || !s->batch_pending) return LAMPS_ERR_INVALID;
        if (cap < s->cfg.max_batch) return LAMPS_ERR_RANGE;
        const lamps_sched_config &cfg = s->cfg;
        int64_t recomputed = 0, swapped = 0, ctx_tokens = 0;
        std::vector<size_t> generated;
        for (size_t w : s->batch) {
            Req &r = s->reqs[w];
            r.started = true;
            if (r.pending_swapin) {
                r.held += r.pending_swapin;
                s->total_held += r.pending_swapin;
                swapped += r.pending_swapin;
                r.pending_swapin = 0;
            }
            if (r.pending_recompute > 0) {
                const int64_t k = std::min<int64_t>(cfg.recompute_chunk, r.pending_recompute);
                r.held += k;
                s->total_held += k;
                if (r.ctx < r.held) r.ctx = r.held;
                r.pending_recompute -= k;
                recomputed += k;
            } else {
                ++r.held;
                ++s->total_held;
                ++r.ctx;
                ++r.done_in_seg;
                generated.push_back(w);
            }
            ctx_tokens += r.held;
        }
        s->peak = std::max(s->peak, s->total_held);
        if (s->total_held > cfg.memory_tokens) return LAMPS_ERR_INVALID;      // cannot happen: need() was free
        // requests that reach their API call leave by their handling strategy
        for (size_t w : generated) {
            const Req &r = s->reqs[w];
            const lamps_segment &sg = r.seg[r.cur];
            if (r.done_in_seg == sg.n_out && sg.api_duration >= 0 && sg.handling == LAMPS_SWAP) swapped += r.held;
        }
        s->now += iteration_time >= 0 ? iteration_time : cost_iteration(cfg.cost, ctx_tokens, recomputed, swapped);
        ++s->iteration;
        int32_t ne = 0;
        for (size_t w : generated) {
            Req &r = s->reqs[w];
            if (r.first_token < 0) r.first_token = s->now;
            const lamps_segment &sg = r.seg[r.cur];
            if (r.done_in_seg < sg.n_out) continue;
            events[ne].id = r.id;
            events[ne].context = r.ctx;
            if (sg.api_duration < 0) {                  // finished
                r.state = kDone;
                r.completion = s->now;
                s->total_held -= r.held;
                r.held = 0;
                ++s->done;
                events[ne].what = 1;
                events[ne].handling = LAMPS_PRESERVE;
            } else {
                r.state = kInApi;
                r.api_end = s->now + sg.api_duration;
                r.starv = 0;
                if (sg.handling == LAMPS_DISCARD || sg.handling == LAMPS_SWAP) {
                    s->total_held -= r.held;            // Preserve keeps it
                    r.held = 0;
                }
                s->in_api.push_back(w);
                events[ne].what = 0;
                events[ne].handling = sg.handling;
            }
            ++ne;
        }
        // what left the waiting queue (API call or finished) is dropped from it
        size_t keep = 0;
        for (size_t w : s->waiting)
            if (s->reqs[w].state == kWaiting) s->waiting[keep++] = w;
        s->waiting.resize(keep);
        for (size_t w : s->batch) s->in_batch[w] = 0;
        s->batch.clear();
        s->batch_pending = false;
        *n = ne;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_run(lamps_sched *s)
{
    try {
        if (!s) return LAMPS_ERR_INVALID;
        std::vector<lamps_batch_entry> b(s->cfg.max_batch);
        std::vector<lamps_sched_event> e(s->cfg.max_batch);
        for (;;) {
            int32_t n = 0, ne = 0;
            int rc = lamps_sched_next_batch(s, b.data(), (int32_t)b.size(), &n);
            if (rc != LAMPS_OK) return rc;
            if (n == 0) return LAMPS_OK;
            rc = lamps_sched_commit(s, -1.0, e.data(), (int32_t)e.size(), &ne);
            if (rc != LAMPS_OK) return rc;
        }
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_take_discards(lamps_sched *s, int64_t *ids, int32_t cap, int32_t *n)
{
    try {
        if (!s || !n || cap < 0 || (cap > 0 && !ids)) return LAMPS_ERR_INVALID;
        const size_t take = std::min<size_t>(s->discarded.size(), (size_t)cap);
        for (size_t i = 0; i < take; ++i) ids[i] = s->discarded[i];
        s->discarded.erase(s->discarded.begin(), s->discarded.begin() + take);
        *n = (int32_t)take;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

double lamps_sched_now(const lamps_sched *s) { return s ? s->now : -1.0; }

int lamps_sched_result(const lamps_sched *s, int64_t id, double *completion, double *first_token,
                       int32_t *handling, int32_t n_handling)
{
    try {
        if (!s || n_handling < 0 || (n_handling > 0 && !handling)) return LAMPS_ERR_INVALID;
        auto it = s->by_id.find(id);
        if (it == s->by_id.end()) return LAMPS_ERR_RANGE;
        const Req &r = s->reqs[it->second];
        if (completion) *completion = r.completion;
        if (first_token) *first_token = r.first_token;
        for (int32_t k = 0; k < n_handling && k < (int32_t)r.seg.size(); ++k) handling[k] = r.seg[k].handling;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

int lamps_sched_stats(const lamps_sched *s, int64_t *iterations, int64_t *peak_memory, int64_t *preemptions)
{
    try {
        if (!s) return LAMPS_ERR_INVALID;
        if (iterations) *iterations = s->iteration;
        if (peak_memory) *peak_memory = s->peak;
        if (preemptions) *preemptions = s->preemptions;
        return LAMPS_OK;
    }
    LAMPS_SCHED_CATCH
}

}  // extern "C"
