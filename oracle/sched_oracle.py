"""Oracle of the server-side pipeline-aware batch former: TEST INFRASTRUCTURE ONLY.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may import this module; the
product (paper_2505_17052_amd, its C++ scheduler and its replay driver) never does, and this module
imports nothing from the product.

What it models (paper, section "Server-side Pipeline-aware Scheduling"): the server only verifies;
draft blocks from many edge devices arrive over a network with a round-trip time; the server takes
the blocks that have arrived as one batch, verifies them, and every verified request returns to its
edge, which drafts again.  The draft depth is calibrated so that
    server verification time ~= edge drafting time + network round trip.
Everything is written as a plain discrete-event simulation over integer microseconds, one event at
a time, with exact rational arithmetic where a rounding rule is involved.

Readings of the paper (it gives the scheme and one worked example, no pseudo-code):
  * drafts are processed as soon as they come in (the scheduling section's description of the server): a free
    server starts a batch as soon as one block has arrived (min_batch = 1); min_batch / max_wait_us generalise
    this to waiting for a fuller batch.
  * order of service: first come, first served, no overtaking; a batch is capped by a request count
    and by a row (draft token) count.
  * depth calibration: nearest integer to (t_verify - rtt) / t_draft_fwd, halves up.  Pinned by the
    paper's example (section "Pipeline-aware draft depth adjustment"): 94.2 ms verification, about
    11 ms per draft pass, depth 7 / 5 / 4 at 15 / 40 / 50 ms RTT; rounding down would give 4 at 40 ms.
  * the depth is set from times measured while serving (same section): a running estimate
    est += floor((d - est) / 8).
"""
from fractions import Fraction
import heapq
import math


def calibrate_depth(t_verify_us, t_draft_fwd_us, rtt_us, min_depth, max_depth):
    """Depth d that best satisfies t_verify = d * t_draft_fwd + rtt (nearest integer, halves up), clamped."""
    if t_verify_us <= rtt_us:
        return min_depth
    exact = Fraction(t_verify_us - rtt_us, t_draft_fwd_us)
    d = math.floor(exact + Fraction(1, 2))
    return max(min_depth, min(max_depth, d))


def running_estimate(durations):
    """The estimate after each recorded duration: first sample as is, then est += floor((d - est) / 8)."""
    out, est = [], None
    for d in durations:
        est = d if est is None else est + (d - est) // 8
        out.append(est)
    return out


class Former:
    """The batch former: blocks (request, n_draft, arrival) are served in order of (arrival, submission)."""

    def __init__(self, max_batch, max_rows, min_batch=1, max_wait_us=0):
        self.max_batch, self.max_rows, self.min_batch, self.max_wait_us = max_batch, max_rows, min_batch, max_wait_us
        self.blocks = []          # dicts; kept unsorted, ordered when needed
        self.counter = 0

    def submit(self, request, n_draft, arrival_us):
        assert all(b["request"] != request for b in self.blocks)
        assert 1 <= n_draft <= self.max_rows
        self.blocks.append({"request": request, "n": n_draft, "t": arrival_us, "order": self.counter})
        self.counter += 1

    def next_batch(self, now_us):
        """Returns (batch as a list of (request, n_draft), wake time); wake is -1 with an empty queue."""
        if not self.blocks:
            return [], -1
        line = sorted(self.blocks, key=lambda b: (b["t"], b["order"]))
        here = [b for b in line if b["t"] <= now_us]
        if not here:
            return [], line[0]["t"]
        if len(here) < self.min_batch and now_us < here[0]["t"] + self.max_wait_us:
            wake = here[0]["t"] + self.max_wait_us
            if len(line) >= self.min_batch:
                wake = min(wake, line[self.min_batch - 1]["t"])
            return [], wake
        batch, rows = [], 0
        for b in here:
            if len(batch) == self.max_batch or rows + b["n"] > self.max_rows:
                break
            batch.append(b)
            rows += b["n"]
        for b in batch:
            self.blocks.remove(b)
        return [(b["request"], b["n"]) for b in batch], now_us


def simulate(n_draft, draft_us, rtt_us, former, verify, n_batches):
    """Replay of the edge/server loop on a simulated clock.

    Edge e (request e) drafts for draft_us[e], its block of n_draft[e] tokens needs half a round trip to
    reach the server (the first half is rtt // 2), the result needs the other half to come back, and the
    edge drafts again at once.  verify(batch) -> (duration_us, [emitted tokens per request of the batch]).
    The server is an event of its own: whenever it is free it asks the former for a batch.
    Returns {"log": [(start_us, [requests])], "tokens": per-request emitted, "busy_us", "end_us"}.
    """
    E = len(n_draft)
    up = rtt_us // 2
    down = rtt_us - up
    events = []                               # (time, kind, request); kind 0 = block reaches the server
    for e in range(E):
        heapq.heappush(events, (draft_us[e] + up, 0, e))
    tokens = [0] * E
    log, busy, now, done = [], 0, 0, 0
    while done < n_batches:
        # deliver every block that has reached the server by now (the former also accepts future ones,
        # but handing them over only on arrival keeps this simulation independent of that feature)
        while events and events[0][0] <= now:
            t, _, e = heapq.heappop(events)
            former.submit(e, n_draft[e], t)
        batch, wake = former.next_batch(now)
        if not batch:
            nxt = events[0][0] if events else None
            cand = [t for t in (wake if wake >= 0 else None, nxt) if t is not None and t > now]
            assert cand, "nothing left to wait for"
            now = min(cand)
            continue
        dur, emitted = verify([r for r, _ in batch])
        log.append((now, [r for r, _ in batch]))
        busy += dur
        now += dur
        done += 1
        for (r, _), m in zip(batch, emitted):
            tokens[r] += m
            heapq.heappush(events, (now + down + draft_us[r] + up, 0, r))
    return {"log": log, "tokens": tokens, "busy_us": busy, "end_us": now}


def edge_align(parents, tokens, accept_path, bonus_token):
    """Complete draft alignment (paper, "Post-verification update"): the server accepted accept_path and
    emitted bonus_token; if a child of the last accepted node (of the prefix, for an empty path) carries
    that token, the edge keeps that child's subtree.  Written out naively: a node is kept iff walking up
    its parents reaches the matching child.  Returns (kept indices ascending, parents re-indexed into kept)."""
    last = accept_path[-1] if len(accept_path) else -1
    heads = [i for i in range(len(parents)) if parents[i] == last and tokens[i] == bonus_token]
    if not heads:
        return [], []
    head = min(heads)

    def under_head(i):
        while i != -1:
            if i == head:
                return True
            i = parents[i]
        return False
    kept = [i for i in range(len(parents)) if under_head(i)]
    return kept, [-1 if i == head else kept.index(parents[i]) for i in kept]
