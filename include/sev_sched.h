/* sev_sched.h — server-side pipeline-aware batch former (host code only, no GPU calls).
 *
 * What it does (paper: "Server-side Pipeline-aware Scheduling").  The server only verifies.  Draft
 * blocks of many requests arrive from their edge devices at different times; the server verifies
 * whatever has arrived as one batch while the other requests are still drafting, and a verified
 * request goes straight back to its edge.  With about twice as many requests in flight as fit one
 * batch, and the draft depth chosen so that
 *         server verification time  ~=  edge drafting time + network round trip,
 * a new batch is complete exactly when the previous verification ends and the server never idles.
 * This library holds the two decisions of that scheme: which arrived blocks form the next batch,
 * and the draft depth that balances the equation from measured times.  It also holds the edge's side
 * of the protocol after a verification: the draft-alignment check.
 *
 * All times are int64 microseconds on a clock the caller owns (wall clock or a simulated one); the
 * scheduler never reads a clock itself, so a replay is deterministic.
 *
 * Conventions: every call returns 0 (SEV_OK) or a negative sev_status code of sev.h; the message is
 * available from sev_last_error().  All pointers are HOST pointers.  A handle is not thread safe.
 */
#ifndef SEV_SCHED_H
#define SEV_SCHED_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct sev_sched sev_sched;

typedef struct {
    int32_t max_batch;    /* most requests in one verification batch (1 .. 256)                           */
    int32_t max_rows;     /* most draft tokens (GEMM rows) in one batch, summed over its requests (>= 1)    */
    int32_t min_batch;    /* a batch smaller than this waits for more arrivals ... (1 .. max_batch)        */
    int64_t max_wait_us;  /* ... but never longer than this after its oldest block arrived (>= 0)          */
} sev_sched_desc;

int sev_sched_create(const sev_sched_desc *desc, sev_sched **out);
int sev_sched_destroy(sev_sched *s);

/* A draft block of `n_draft` tokens for request `request` (any non-negative id) reaches the server at
 * `arrival_us` (may lie in the future of the caller's clock: a replay submits arrivals ahead).
 * Errors: SEV_EINVAL n_draft < 1 or > max_rows, negative id; SEV_ESTATE the request already has a
 * block waiting (an edge sends its next block only after the previous one was verified). */
int sev_sched_submit(sev_sched *s, int32_t request, int32_t n_draft, int64_t arrival_us);

/* The server is free at `now_us`: form the next batch.
 * Blocks are served strictly in order of arrival (ties: order of submission).  Among the blocks that
 * have arrived by now_us, the batch takes them in that order until max_batch requests or max_rows
 * rows would be exceeded (it stops at the first block that does not fit: no overtaking).  If fewer
 * than min_batch blocks have arrived and the oldest has waited less than max_wait_us, no batch is
 * formed yet.
 * requests[0 .. *n_out) receives the batch (capacity max_batch), rows[] (may be NULL) their n_draft.
 * With *n_out == 0, *wake_us is the earliest time at which calling again can give a different answer
 * (the next arrival that matters or the end of the wait), or -1 if nothing is queued.  With a batch,
 * *wake_us is now_us. */
int sev_sched_next_batch(sev_sched *s, int64_t now_us, int32_t *requests, int32_t *rows, int32_t *n_out, int64_t *wake_us);

/* Number of blocks queued (arrived or not). */
int sev_sched_pending(const sev_sched *s);

/* Measured duration of a verification; keeps a running estimate est += (d - est) / 8 (first sample:
 * est = d; the division rounds toward minus infinity).  sev_sched_verify_estimate returns it (0 if
 * none yet). */
int sev_sched_record_verify(sev_sched *s, int64_t duration_us);
int64_t sev_sched_verify_estimate(const sev_sched *s);

/* Draft depth (number of draft-model forward passes per block) that balances
 *     t_verify ~= depth * t_draft_fwd + rtt :
 * depth = (t_verify - rtt) / t_draft_fwd rounded to nearest (halves up), clamped to
 * [min_depth, max_depth]; min_depth if t_verify <= rtt.  Returns the depth, or a negative status for
 * t_draft_fwd_us < 1, a negative t_verify_us or rtt_us, min_depth < 1 or max_depth < min_depth.  (The paper's example: verification
 * 94.2 ms, 11 ms per draft pass: depth 7 at 15 ms RTT, 5 at 40 ms, 4 at 50 ms.) */
int sev_sched_calibrate_depth(int64_t t_verify_us, int64_t t_draft_fwd_us, int64_t rtt_us, int32_t min_depth, int32_t max_depth);

/* Edge-side post-verification update (paper: "Post-verification update", complete draft alignment).
 * The edge holds a draft tree of n_nodes nodes in topological order (parents[i] in [-1, i), -1 = child
 * of the committed prefix): the nodes it sent for verification and the ones it drafted proactively
 * while the server was busy.  The server answers with the accepted path (node indices, root first) and
 * one additional token.  If the last accepted node (the prefix, if nothing was accepted) has a child
 * whose token equals that additional token, the draft is aligned: the edge keeps that child and
 * everything below it and continues drafting from there; otherwise all drafted work is discarded.
 *   kept[0 .. *n_kept)        indices of the kept nodes in increasing order; kept[0] is the matching
 *                             child (lowest index if several match); *n_kept = 0: no alignment
 *   new_parents[0 .. *n_kept) parent of each kept node as an index into kept[] (-1 for kept[0]): the
 *                             tree to send next, rooted at the token the server just emitted
 * kept and new_parents have room for n_nodes entries.  Errors: SEV_EINVAL for null pointers, parents
 * out of range, an accept_path that is not a root-to-node path of the tree. */
int sev_edge_align(const int32_t *parents, const int32_t *tokens, int32_t n_nodes, const int32_t *accept_path, int32_t accept_len,
                   int32_t bonus_token, int32_t *kept, int32_t *new_parents, int32_t *n_kept);

#ifdef __cplusplus
}
#endif
#endif
