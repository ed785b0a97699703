// Server-side pipeline-aware batch former (paper: "Server-side Pipeline-aware Scheduling").
// Host code only: a FIFO of draft blocks ordered by arrival time, the rule that forms the next
// verification batch from the blocks that have arrived, a running estimate of the verification time
// and the draft-depth calibration  t_verify ~= depth * t_draft_fwd + rtt.  Semantics: include/sev_sched.h.
#include <stdint.h>

#include <algorithm>
#include <new>
#include <vector>

#include "../../include/sev.h"
#include "../../include/sev_sched.h"

int sev_fail(int code, const char *fmt, ...);

namespace {
struct Block {
    int64_t arrival;
    uint64_t seq;        // order of submission, breaks ties of equal arrival times
    int32_t request, n_draft;
};
inline bool before(const Block &a, const Block &b) { return a.arrival != b.arrival ? a.arrival < b.arrival : a.seq < b.seq; }
}  // namespace

struct sev_sched {
    sev_sched_desc d;
    std::vector<Block> q;   // sorted by (arrival, seq)
    uint64_t next_seq = 0;
    int64_t est = 0;
    bool have_est = false;
};

extern "C" int sev_sched_create(const sev_sched_desc *desc, sev_sched **out) {
    if (!out) return sev_fail(SEV_EINVAL, "null output handle");
    *out = nullptr;
    if (!desc) return sev_fail(SEV_EINVAL, "null scheduler description");
    if (desc->max_batch < 1 || desc->max_batch > 256) return sev_fail(SEV_EINVAL, "max_batch must be in 1..256");
    if (desc->max_rows < 1) return sev_fail(SEV_EINVAL, "max_rows must be positive");
    if (desc->min_batch < 1 || desc->min_batch > desc->max_batch) return sev_fail(SEV_EINVAL, "min_batch must be in 1..max_batch");
    if (desc->max_wait_us < 0) return sev_fail(SEV_EINVAL, "max_wait_us must not be negative");
    sev_sched *s = new (std::nothrow) sev_sched();
    if (!s) return sev_fail(SEV_ENOSPACE, "host allocation failed");
    s->d = *desc;
    *out = s;
    return SEV_OK;
}

extern "C" int sev_sched_destroy(sev_sched *s) {
    delete s;
    return SEV_OK;
}

extern "C" int sev_sched_submit(sev_sched *s, int32_t request, int32_t n_draft, int64_t arrival_us) {
    if (!s) return sev_fail(SEV_EINVAL, "null scheduler");
    if (request < 0) return sev_fail(SEV_EINVAL, "request id must not be negative");
    if (n_draft < 1 || n_draft > s->d.max_rows) return sev_fail(SEV_EINVAL, "n_draft %d outside 1..max_rows (%d)", n_draft, s->d.max_rows);
    for (const Block &b : s->q)
        if (b.request == request) return sev_fail(SEV_ESTATE, "request %d already has a block waiting", request);
    const Block nb{arrival_us, s->next_seq++, request, n_draft};
    s->q.insert(std::upper_bound(s->q.begin(), s->q.end(), nb, before), nb);
    return SEV_OK;
}

extern "C" int sev_sched_next_batch(sev_sched *s, int64_t now_us, int32_t *requests, int32_t *rows, int32_t *n_out, int64_t *wake_us) {
    if (!s || !requests || !n_out || !wake_us) return sev_fail(SEV_EINVAL, "null argument");
    *n_out = 0;
    *wake_us = -1;
    if (s->q.empty()) return SEV_OK;
    size_t ready = 0;
    while (ready < s->q.size() && s->q[ready].arrival <= now_us) ++ready;
    if (ready == 0) {
        *wake_us = s->q[0].arrival;
        return SEV_OK;
    }
    if ((int)ready < s->d.min_batch) {
        const int64_t deadline = s->q[0].arrival + s->d.max_wait_us;
        if (now_us < deadline) {
            // the batch can start when the min_batch-th block arrives or when the wait runs out
            int64_t wake = deadline;
            if (s->q.size() >= (size_t)s->d.min_batch) wake = std::min(wake, s->q[s->d.min_batch - 1].arrival);
            *wake_us = wake;
            return SEV_OK;
        }
    }
    int n = 0, total = 0;
    while ((size_t)n < ready && n < s->d.max_batch && total + s->q[n].n_draft <= s->d.max_rows) {
        requests[n] = s->q[n].request;
        if (rows) rows[n] = s->q[n].n_draft;
        total += s->q[n].n_draft;
        ++n;
    }
    s->q.erase(s->q.begin(), s->q.begin() + n);
    *n_out = n;
    *wake_us = now_us;
    return SEV_OK;
}

extern "C" int sev_sched_pending(const sev_sched *s) { return s ? (int)s->q.size() : 0; }

extern "C" int sev_sched_record_verify(sev_sched *s, int64_t duration_us) {
    if (!s) return sev_fail(SEV_EINVAL, "null scheduler");
    if (duration_us < 0) return sev_fail(SEV_EINVAL, "negative duration");
    if (!s->have_est) {
        s->est = duration_us;
        s->have_est = true;
    } else {
        const int64_t diff = duration_us - s->est;
        s->est += diff >= 0 ? diff / 8 : -((-diff + 7) / 8);      // floor division
    }
    return SEV_OK;
}

extern "C" int64_t sev_sched_verify_estimate(const sev_sched *s) { return (s && s->have_est) ? s->est : 0; }

extern "C" int sev_sched_calibrate_depth(int64_t t_verify_us, int64_t t_draft_fwd_us, int64_t rtt_us, int32_t min_depth, int32_t max_depth) {
    if (t_draft_fwd_us < 1) return sev_fail(SEV_EINVAL, "t_draft_fwd_us must be positive");
    if (min_depth < 1 || max_depth < min_depth) return sev_fail(SEV_EINVAL, "need 1 <= min_depth <= max_depth");
    if (t_verify_us < 0 || rtt_us < 0) return sev_fail(SEV_EINVAL, "times must not be negative");
    const int64_t budget = t_verify_us - rtt_us;                  // time left for drafting (both terms >= 0: no overflow)
    if (budget <= 0) return min_depth;
    const int64_t whole = budget / t_draft_fwd_us, rem = budget % t_draft_fwd_us;
    const int64_t depth = whole + (rem >= t_draft_fwd_us - rem ? 1 : 0);          // nearest, halves up, without doubling anything
    return (int)std::min<int64_t>(std::max<int64_t>(depth, min_depth), max_depth);
}

extern "C" int sev_edge_align(const int32_t *parents, const int32_t *tokens, int32_t n_nodes, const int32_t *accept_path, int32_t accept_len,
                              int32_t bonus_token, int32_t *kept, int32_t *new_parents, int32_t *n_kept) {
    if (!parents || !tokens || !kept || !new_parents || !n_kept || (accept_len > 0 && !accept_path))
        return sev_fail(SEV_EINVAL, "null argument");
    *n_kept = 0;
    if (n_nodes < 0 || accept_len < 0 || accept_len > n_nodes) return sev_fail(SEV_EINVAL, "bad node or path count");
    for (int i = 0; i < n_nodes; ++i)
        if (parents[i] < -1 || parents[i] >= i) return sev_fail(SEV_EINVAL, "node %d: parent %d does not precede it", i, parents[i]);
    int last = -1;
    for (int j = 0; j < accept_len; ++j) {
        const int c = accept_path[j];
        if (c < 0 || c >= n_nodes || parents[c] != last) return sev_fail(SEV_EINVAL, "accept_path[%d] = %d does not continue the path", j, c);
        last = c;
    }
    int head = -1;
    for (int i = last + 1; i < n_nodes && head < 0; ++i)
        if (parents[i] == last && tokens[i] == bonus_token) head = i;
    if (head < 0) return SEV_OK;
    // parents precede children: one sweep marks the subtree; new index = number of kept nodes before it
    std::vector<int32_t> pos((size_t)n_nodes, -1);
    int n = 0;
    for (int i = head; i < n_nodes; ++i) {
        const bool in = i == head || (parents[i] >= head && pos[parents[i]] >= 0);
        if (!in) continue;
        pos[i] = n;
        kept[n] = i;
        new_parents[n] = i == head ? -1 : pos[parents[i]];
        ++n;
    }
    *n_kept = n;
    return SEV_OK;
}
