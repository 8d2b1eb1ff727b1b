"""Plain model of the LAMPS scheduler (test infrastructure, see package doc).

arXiv 2410.18248: equations (1)-(3) (memory waste of the three ways to treat a
request's KV cache during an API call), the memory-over-time rank function of
Section 4.2 / 4.3, and Algorithm 1 (iteration-level scheduling with a
starvation counter), written out step by step in the paper's order.  Slow and
obvious on purpose: lists, sorts, no caching beyond what the paper describes.

Units are the caller's: time in iterations for the paper's worked example
(Section 3.1), seconds for a cost model measured on a GPU; memory in tokens
(M bytes each).

Readings where the paper is silent (also listed in the repository's design
notes):
  * A request is a list of segments, each a number of output tokens followed
    by one API call (duration, response length), the last one without a call
    (the "Multi-API" paragraph of Section 4.2).
  * "runningBatch is not full" means: fewer than max_batch requests, and the
    memory the candidate needs is free.  A request at the start of a segment
    needs room for the whole segment (what it has to bring back -- swapped or
    discarded context, the API response -- plus the segment's tokens): the
    worked example (Section 3.1, FCFS) refuses R3 while R1 is in its API call
    because R3 would still hold its memory when R1 comes back.  A request in
    the middle of a segment needs one token.
  * Every request that is not finished and not in an API call is in the
    waiting queue at the start of every iteration and the batch is formed
    anew (iteration-level scheduling), so a better-ranked request displaces a
    running one; the displaced one keeps its memory.
  * An iteration in which a request recomputes discarded context or processes
    an API response produces no new token for it (the worked example counts
    R2's part after its call as 2 units, one of them the recomputation).
  * Ties in the rank go to the earlier arrival, then the lower id.
  * If nothing can run while waiting requests hold memory (each needs more
    than is free), the worst-ranked of them is discarded and recomputes later
    (Section 4.3 names discard-and-recompute as what happens when memory is
    full); if no waiting request holds memory the engine idles until the next
    arrival or API return (the idle unit of the worked example).
  * A request whose starvation counter reaches the threshold while the batch
    is formed goes to the head of the queue in that same iteration (Section
    4.4 places it there for the current iteration): the batch is formed once
    more with the tagged requests first.  Counters are not incremented a
    second time.
  * In the worked example's units (unit=True) recomputing a discarded context
    takes one iteration, T_fwd = 1 (Section 3.1 counts R2's part after its
    call as two units, one of them the recomputation), and a swap takes no
    time (R3's part after its call is one unit).
"""
PRESERVE, DISCARD, SWAP = 0, 1, 2
FCFS, SJF, SJF_TOTAL, LAMPS, FIXED = 0, 1, 2, 3, 4
NEW, WAITING, IN_API, DONE = 0, 1, 2, 3


# ---------------------------------------------------------------- equations (1)-(3)
def waste_preserve(T_int, C_i, M):
    """Equation (1): the context sits idle for the API call's duration."""
    return T_int * C_i * M


def waste_discard(T_fwd_Ci, C_i, C_other, M):
    """Equation (2): recomputing C_i holds C_i, and stalls the others, for T_fwd(C_i)."""
    return T_fwd_Ci * C_i * M + T_fwd_Ci * C_other * M


def waste_swap(T_swap_Ci, C_batch, M):
    """Equation (3): swapping out and in stalls the whole batch twice."""
    return 2 * T_swap_Ci * C_batch * M


def handling_strategy(T_int, C_i, C_other, M, T_fwd_Ci, T_swap_Ci):
    """The strategy of least waste (Section 4.2); ties go to the earlier of
    Preserve, Discard, Swap."""
    w = (waste_preserve(T_int, C_i, M), waste_discard(T_fwd_Ci, C_i, C_other, M),
         waste_swap(T_swap_Ci, C_i + C_other, M))
    return w.index(min(w))


# ---------------------------------------------------------------- memory over time
def memory_over_time(strategy, c0, n1, T_int, rho, n2, tau, T_fwd_C, T_swap_C):
    """Integral of a request's memory (tokens) over time (Section 4.2, the three
    panels of the memory-over-time figure): it starts with c0 tokens of context,
    generates n1 tokens (tau each), calls an API for T_int, gets rho tokens
    back and generates n2 more.  C = c0 + n1 is the context at the call.
      Preserve: C tokens are held for T_int.
      Discard : nothing is held during the call; C is held while it is
                recomputed, T_fwd(C).
      Swap    : nothing is held during the call; C is held while it is moved
                out and back in, 2 T_swap(C).
    """
    C = c0 + n1
    pre = tau * sum(c0 + j for j in range(1, n1 + 1))
    post = tau * sum(C + rho + j for j in range(1, n2 + 1))
    if strategy == PRESERVE:
        mid = T_int * C
    elif strategy == DISCARD:
        mid = T_fwd_C * C
    else:
        mid = 2 * T_swap_C * C
    return pre + mid + post


# ---------------------------------------------------------------- cost model
class CostModel:
    """Times of the engine the scheduler drives.

    iteration  = it_a + it_b * (context tokens of the running batch)
                 + fwd_b * (tokens recomputed or first processed in it)
                 + (sw_a + sw_b * tokens swapped in or out in it), if swaps stall the batch
    T_fwd(C)   = fwd_a + fwd_b * C          T_swap(C) = sw_a + sw_b * C
    unit=True: every iteration takes exactly 1, swaps cost nothing (the paper's
    worked example)."""

    def __init__(self, it_a=1.0, it_b=0.0, fwd_a=0.0, fwd_b=0.0, sw_a=0.0, sw_b=0.0,
                 swap_stalls=True, unit=False):
        self.it_a, self.it_b, self.fwd_a, self.fwd_b = it_a, it_b, fwd_a, fwd_b
        self.sw_a, self.sw_b, self.swap_stalls, self.unit = sw_a, sw_b, swap_stalls, unit

    def t_fwd(self, C):
        if self.unit:
            return 1.0
        return self.fwd_a + self.fwd_b * C

    def t_swap(self, C):
        if self.unit:
            return 0.0
        return self.sw_a + self.sw_b * C

    def iteration(self, ctx_tokens, recomputed, swapped):
        if self.unit:
            return 1.0
        t = self.it_a + self.it_b * ctx_tokens + self.fwd_b * recomputed
        if self.swap_stalls and swapped > 0:
            t += self.sw_a + self.sw_b * swapped
        return t


class Request:
    """segments: [(n_out, api_duration or None, api_response_tokens), ...]; the
    last segment has api_duration None.  handling: one strategy per segment
    with an API call, or None to let equations (1)-(3) choose."""

    def __init__(self, rid, arrival, prompt, segments, handling=None, priority=0.0):
        self.id, self.arrival, self.prompt = rid, arrival, prompt
        self.segments = [tuple(s) for s in segments]
        assert self.segments and self.segments[-1][1] is None
        assert all(s[1] is not None for s in self.segments[:-1])
        self.handling = list(handling) if handling is not None else [None] * len(self.segments)
        self.priority = priority                       # FIXED policy only
        self.state = NEW
        self.seg = 0
        self.done_in_seg = 0
        self.started = False                           # current segment admitted once
        self.ctx = 0                                   # logical context, tokens
        self.held = 0                                  # tokens of it in GPU memory
        self.pending_recompute = prompt                # tokens to run through the model first
        self.pending_swapin = 0
        self.api_end = None
        self.starv = 0
        self.prioritized = False
        self.score = None
        self.score_iter = 0
        self.completion = None
        self.first_token = None


class Simulator:
    def __init__(self, requests, policy, max_batch, memory_tokens, cost, starvation_threshold=100,
                 score_refresh=1, recompute_chunk=1 << 30, c_other=0.0, bytes_per_token=1.0):
        self.reqs = sorted(requests, key=lambda r: (r.arrival, r.id))
        self.policy, self.max_batch, self.budget, self.cost = policy, max_batch, memory_tokens, cost
        self.starvation_threshold, self.score_refresh = starvation_threshold, score_refresh
        self.recompute_chunk = recompute_chunk
        self.c_other, self.M = c_other, bytes_per_token
        self.now = 0.0
        self.iteration = 0
        self.trace = []                                # (time, [ids run]) per executed iteration
        self.peak_memory = 0
        self.preemptions = 0

    def _context_at_call(self, r):
        """Context length the request will have when it reaches this segment's API call."""
        base = r.ctx if r.ctx else r.pending_recompute
        n_out = r.segments[r.seg][0]
        return base + (n_out - r.done_in_seg)

    def _remaining_tokens(self, r):
        rem = r.pending_recompute + (r.segments[r.seg][0] - r.done_in_seg)
        for s in r.segments[r.seg + 1:]:
            rem += s[0]
        return rem

    def _rank(self, r):
        if self.policy == FCFS:
            return 0.0                                 # ties: arrival, id
        if self.policy == FIXED:
            return r.priority
        if self.policy == SJF:
            return float(self._remaining_tokens(r))
        if self.policy == SJF_TOTAL:
            api = sum(s[1] for s in r.segments[r.seg:] if s[1] is not None)
            return self._remaining_tokens(r) + api / self.cost.iteration(0, 0, 0)
        # LAMPS: memory over time of the current segment, its API call handled as decided,
        # and the tokens that follow the call
        n_out, api, rho = r.segments[r.seg]
        c0 = r.ctx if r.ctx else r.pending_recompute
        n1 = n_out - r.done_in_seg
        tau = self.cost.iteration(0, 0, 0)
        if api is None:
            return memory_over_time(PRESERVE, c0, n1, 0.0, 0, 0, tau, 0.0, 0.0)
        n2 = r.segments[r.seg + 1][0]
        C = c0 + n1
        return memory_over_time(r.handling[r.seg], c0, n1, api, rho, n2, tau, self.cost.t_fwd(C),
                                self.cost.t_swap(C))

    def _need(self, r):
        """Tokens of memory the request must find free to join the batch."""
        if not r.started:
            return r.pending_swapin + r.pending_recompute + (r.segments[r.seg][0] - r.done_in_seg)
        if r.pending_recompute > 0:
            return min(self.recompute_chunk, r.pending_recompute)
        return 1

    def run(self, max_iterations=10 ** 7):
        reqs = self.reqs
        while any(r.state != DONE for r in reqs):
            assert self.iteration < max_iterations, "simulation does not end"
            # Algorithm 1: new requests get their handling strategy and enter the waiting queue
            for r in reqs:
                if r.state == NEW and r.arrival <= self.now:
                    self._decide(r)
                    r.state = WAITING
            # requests whose API call has finished re-enter it
            for r in reqs:
                if r.state == IN_API and r.api_end <= self.now:
                    self._return_from_api(r)
            waiting = [r for r in reqs if r.state == WAITING]
            # scores (cached and refreshed every score_refresh iterations), then the sort
            for r in waiting:
                if r.score is None or self.iteration - r.score_iter >= self.score_refresh:
                    r.score = self._rank(r)
                    r.score_iter = self.iteration
            order = lambda r: (0 if r.prioritized else 1, r.score, r.arrival, r.id)
            waiting.sort(key=order)
            # the running batch
            held_now = sum(r.held for r in reqs)

            def form(count):
                free, chosen = self.budget - held_now, []
                for r in waiting:
                    need = self._need(r)
                    if len(chosen) < self.max_batch and need <= free:
                        chosen.append(r)
                        free -= need
                        if count:
                            r.starv = 0
                    elif count:
                        r.starv += 1
                return chosen
            batch = form(True)
            # Algorithm 1's second loop: a request left out often enough is tagged and goes
            # to the head of the queue for this very iteration
            tagged = False
            for r in waiting:
                if r not in batch and not r.prioritized and r.starv >= self.starvation_threshold:
                    r.prioritized = True
                    r.starv = 0
                    tagged = True
            if tagged:
                waiting.sort(key=order)
                batch = form(False)
            if not batch:
                # Nothing fits.  If memory is held by waiting requests none of which can grow,
                # the worst-ranked holder is discarded and recomputes once memory is there
                # (Section 4.3 on full memory); otherwise the engine idles until the next
                # arrival or API return.
                victims = [r for r in reversed(waiting) if r.held > 0]
                if victims:
                    v = victims[0]
                    v.held = 0
                    v.pending_swapin = 0
                    v.pending_recompute = v.ctx
                    v.started = False
                    v.score = None
                    self.preemptions += 1
                    continue
                nxt = [r.api_end for r in reqs if r.state == IN_API]
                nxt += [r.arrival for r in reqs if r.state == NEW]
                assert nxt, "a request needs more memory than the whole budget"
                self.now = max(self.now, min(nxt))
                continue
            # execute the batch: one iteration
            recomputed = swapped = 0
            generated = []
            for r in batch:
                r.started = True
                if r.pending_swapin:
                    r.held += r.pending_swapin
                    swapped += r.pending_swapin
                    r.pending_swapin = 0
                if r.pending_recompute > 0:
                    k = min(self.recompute_chunk, r.pending_recompute)
                    r.held += k
                    if r.ctx < r.held:
                        r.ctx = r.held
                    r.pending_recompute -= k
                    recomputed += k
                else:
                    r.held += 1
                    r.ctx += 1
                    r.done_in_seg += 1
                    generated.append(r)
            ctx_tokens = sum(r.held for r in batch)
            self.peak_memory = max(self.peak_memory, sum(r.held for r in reqs))
            assert sum(r.held for r in reqs) <= self.budget, "memory budget exceeded"
            # requests that reach their API call leave by their handling strategy
            leaving = [r for r in generated
                       if r.done_in_seg == r.segments[r.seg][0] and r.segments[r.seg][1] is not None]
            swapped += sum(r.held for r in leaving if r.handling[r.seg] == SWAP)
            self.now += self.cost.iteration(ctx_tokens, recomputed, swapped)
            self.iteration += 1
            self.trace.append((self.now, [r.id for r in batch]))
            for r in generated:
                if r.first_token is None:
                    r.first_token = self.now
                if r.done_in_seg < r.segments[r.seg][0]:
                    continue
                if r.segments[r.seg][1] is None:       # finished
                    r.state = DONE
                    r.completion = self.now
                    r.held = 0
                else:
                    r.state = IN_API
                    r.api_end = self.now + r.segments[r.seg][1]
                    r.starv = 0
                    h = r.handling[r.seg]
                    if h == DISCARD or h == SWAP:
                        r.held = 0                     # Preserve keeps it
        return self

    def _decide(self, r):
        """Section 4.2: the handling strategy of a segment's API call is fixed, from the
        predicted context at the call and the call's duration, before the segment runs."""
        n_out, api, _ = r.segments[r.seg]
        if api is not None and r.handling[r.seg] is None:
            C_i = self._context_at_call(r)
            r.handling[r.seg] = handling_strategy(api, C_i, self.c_other, self.M,
                                                  self.cost.t_fwd(C_i), self.cost.t_swap(C_i))

    def _return_from_api(self, r):
        _, _, rho = r.segments[r.seg]
        h = r.handling[r.seg]
        if h == DISCARD:
            r.pending_recompute = r.ctx                # everything is run through the model again
        elif h == SWAP:
            r.pending_swapin = r.ctx
        r.pending_recompute += rho                     # the API's response is new context
        r.ctx += rho
        r.seg += 1
        r.done_in_seg = 0
        r.started = False
        r.score = None
        r.state = WAITING
        self._decide(r)

    # ---- results
    def completion_times(self):
        return {r.id: r.completion - r.arrival for r in self.reqs}

    def mean_completion(self):
        c = self.completion_times()
        return sum(c.values()) / len(c)
