"""Host-side tests of the pipeline-aware batch former (no GPU).

Oracle pins (oracle/sched_oracle.py against what the paper and arithmetic fix):
  * the paper's worked example of the depth calibration (section "Pipeline-aware draft depth adjustment":
    94.2 ms verification, 11 ms per draft pass -> depth 7 / 5 / 4 at 15 / 40 / 50 ms round trip);
  * closed forms of the replay: with B requests in flight and t_verify = t_draft + rtt the server is busy
    half of the time, with 2B it never idles after the first arrival, so the throughput doubles (the
    mechanism behind the paper's "effectively doubles server throughput");
  * invariants of the batch former on random traffic: first come first served, caps respected, nobody lost.
Product: the C++ scheduler (through the C ABI) must take exactly the oracle's decisions, and the replay
driver must produce exactly the oracle simulation's log, on seeded random traffic.
"""
import os

import numpy as np
import pytest

from oracle import sched_oracle as so

GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "depth_calibration.txt")


def _golden_rows():
    rows = []
    for line in open(GOLDEN):
        line = line.split("#")[0].strip()
        if line:
            rows.append([int(x) for x in line.split()])
    return rows


# ---------------------------------------------------------------- oracle pins

def test_oracle_depth_matches_paper_example():
    rows = _golden_rows()
    assert len(rows) == 3
    for t_verify, t_fwd, rtt, depth in rows:
        assert so.calibrate_depth(t_verify, t_fwd, rtt, 1, 64) == depth
    # rounding down instead of to nearest would miss the 40 ms case
    assert (94200 - 40000) // 11000 == 4


def test_oracle_depth_special_cases():
    assert so.calibrate_depth(10000, 1000, 10000, 2, 9) == 2          # no time left for drafting
    assert so.calibrate_depth(10000, 1000, 20000, 1, 9) == 1
    assert so.calibrate_depth(10500, 1000, 0, 1, 64) == 11            # a half rounds up
    assert so.calibrate_depth(10499, 1000, 0, 1, 64) == 10
    assert so.calibrate_depth(10 ** 9, 1000, 0, 1, 64) == 64          # clamped
    for d in range(1, 20):                                            # exact balance gives the depth back
        assert so.calibrate_depth(d * 7000 + 3000, 7000, 3000, 1, 64) == d


def test_oracle_running_estimate():
    assert so.running_estimate([800]) == [800]
    assert so.running_estimate([800, 1600]) == [800, 900]
    assert so.running_estimate([800, 0]) == [800, 700]
    assert so.running_estimate([10, 9]) == [10, 9]                    # floor of -1/8 is -1
    est = so.running_estimate([1000] * 5 + [2000] * 200)
    assert est[4] == 1000 and 1990 <= est[-1] <= 2000                 # converges towards the new level


def _const_verify(v_us, emitted):
    return lambda reqs: (v_us, [emitted] * len(reqs))


def test_oracle_replay_closed_forms():
    B, D, rtt, n = 4, 6000, 2000, 25
    V = D + rtt                                                       # the balance the calibration aims at
    one = so.simulate([8] * B, [D] * B, rtt, so.Former(B, 8 * B), _const_verify(V, 3), n)
    two = so.simulate([8] * (2 * B), [D] * (2 * B), rtt, so.Former(B, 8 * B), _const_verify(V, 3), n)
    t0 = D + rtt // 2                                                 # first arrival
    # B in flight: verify, then wait a full draft + round trip: a batch every 2V
    assert [t for t, _ in one["log"]] == [t0 + 2 * V * j for j in range(n)]
    assert one["end_us"] == t0 + 2 * V * (n - 1) + V and one["busy_us"] == n * V
    # 2B in flight: the second group's blocks are complete exactly when the first verification ends
    assert [t for t, _ in two["log"]] == [t0 + V * j for j in range(n)]
    assert two["end_us"] == t0 + n * V and two["busy_us"] == n * V
    assert all(len(b) == B for _, b in one["log"] + two["log"])
    assert sum(one["tokens"]) == sum(two["tokens"]) == 3 * B * n
    ratio = (sum(two["tokens"]) / two["end_us"]) / (sum(one["tokens"]) / one["end_us"])
    assert ratio == pytest.approx((t0 + (2 * n - 1) * V) / (t0 + n * V)) and ratio > 1.9
    # the two groups alternate
    assert two["log"][0][1] == list(range(B)) and two["log"][1][1] == list(range(B, 2 * B)) and two["log"][2][1] == list(range(B))


def test_oracle_former_invariants_on_random_traffic():
    rng = np.random.default_rng(5)
    for trial in range(40):
        max_batch, max_rows = int(rng.integers(1, 6)), int(rng.integers(8, 40))
        min_batch = int(rng.integers(1, max_batch + 1))
        f = so.Former(max_batch, max_rows, min_batch, int(rng.integers(0, 50)))
        n = 30
        arrivals = np.sort(rng.integers(0, 400, size=n))
        sizes = rng.integers(1, 9, size=n)
        for i in range(n):
            f.submit(i, int(sizes[i]), int(arrivals[i]))
        served, now = [], 0
        while f.blocks:
            batch, wake = f.next_batch(now)
            if not batch:
                assert wake > now
                now = wake
                continue
            assert len(batch) <= max_batch and sum(r for _, r in batch) <= max_rows
            assert all(arrivals[r] <= now for r, _ in batch)
            if len(batch) < min_batch:                                # a short batch only after the wait ran out, or capped by rows
                first = batch[0][0]
                later = [i for i in range(n) if i not in served and i not in [r for r, _ in batch] and arrivals[i] <= now]
                assert now >= arrivals[first] + f.max_wait_us or later
            served += [r for r, _ in batch]
            now += int(rng.integers(1, 30))
        assert served == list(range(n))                               # first come first served (ids were given in arrival order)


# ---------------------------------------------------------------- product against the oracle

def test_library_depth_and_estimate_match_oracle():
    import paper_2505_17052_amd as sev
    for t_verify, t_fwd, rtt, depth in _golden_rows():
        assert sev.calibrate_depth(t_verify, t_fwd, rtt, 1, 64) == depth
    rng = np.random.default_rng(11)
    for _ in range(2000):
        tv, tf, rtt = int(rng.integers(0, 200000)), int(rng.integers(1, 30000)), int(rng.integers(0, 100000))
        lo = int(rng.integers(1, 5)); hi = lo + int(rng.integers(0, 12))
        assert sev.calibrate_depth(tv, tf, rtt, lo, hi) == so.calibrate_depth(tv, tf, rtt, lo, hi)
    with pytest.raises(sev.SevError):
        sev.calibrate_depth(1000, 0, 10)
    s = sev.Scheduler(4, 64)
    ds = [int(x) for x in rng.integers(0, 100000, size=300)]
    got = []
    for d in ds:
        s.record_verify(d)
        got.append(s.verify_estimate())
    assert got == so.running_estimate(ds)


def test_library_batches_match_oracle_on_random_traffic():
    import paper_2505_17052_amd as sev
    rng = np.random.default_rng(23)
    for trial in range(60):
        max_batch, max_rows = int(rng.integers(1, 7)), int(rng.integers(8, 48))
        min_batch, wait = int(rng.integers(1, max_batch + 1)), int(rng.integers(0, 60))
        s, f = sev.Scheduler(max_batch, max_rows, min_batch, wait), so.Former(max_batch, max_rows, min_batch, wait)
        n = 40
        arrivals, sizes = rng.integers(0, 500, size=n), rng.integers(1, 9, size=n)      # unsorted: ties and out-of-order submission
        for i in range(n):
            s.submit(i, int(sizes[i]), int(arrivals[i]))
            f.submit(i, int(sizes[i]), int(arrivals[i]))
        now = 0
        while f.blocks:
            a, b = s.next_batch(now), f.next_batch(now)
            assert a == b, (trial, now, a, b)
            now = b[1] if not b[0] else now + int(rng.integers(0, 40))
        assert s.pending() == 0 and s.next_batch(now) == ([], -1)


def test_library_validation():
    import paper_2505_17052_amd as sev
    for bad in ((0, 8, 1, 0), (257, 8, 1, 0), (4, 0, 1, 0), (4, 8, 5, 0), (4, 8, 0, 0), (4, 8, 1, -1)):
        with pytest.raises(sev.SevError):
            sev.Scheduler(*bad)
    s = sev.Scheduler(2, 8)
    s.submit(3, 8, 10)
    with pytest.raises(sev.SevError):
        s.submit(3, 1, 20)                                            # one block per request at a time
    with pytest.raises(sev.SevError):
        s.submit(4, 9, 20)                                            # larger than a whole batch
    with pytest.raises(sev.SevError):
        s.submit(-1, 1, 20)
    assert s.next_batch(10) == ([(3, 8)], 10)
    s.submit(3, 1, 20)                                                # allowed again once served


def test_replay_driver_matches_oracle_simulation():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd.pipeline import replay
    rng = np.random.default_rng(31)
    for trial in range(25):
        E, max_batch = int(rng.integers(2, 10)), int(rng.integers(1, 6))
        n_draft = [int(x) for x in rng.integers(1, 9, size=E)]
        draft_us = [int(x) for x in rng.integers(500, 9000, size=E)]
        rtt = int(rng.integers(0, 5000))
        min_batch, wait = int(rng.integers(1, max_batch + 1)), int(rng.integers(0, 3000))
        max_rows = 8 * max_batch

        def make_verify(seed):
            r = np.random.default_rng(seed)                           # same stream of durations and acceptances for both sides
            def verify(reqs):
                return int(r.integers(1000, 9000)) + 100 * len(reqs), [int(r.integers(1, 6)) for _ in reqs]
            return verify
        got = replay(n_draft, draft_us, rtt, sev.Scheduler(max_batch, max_rows, min_batch, wait), make_verify(trial), 30)
        want = so.simulate(n_draft, draft_us, rtt, so.Former(max_batch, max_rows, min_batch, wait), make_verify(trial), 30)
        assert got == want, trial


def test_waiting_for_a_fuller_batch_hand_case():
    """min_batch = 3, max_wait 100: worked through by hand; the oracle and the library must both follow it."""
    import paper_2505_17052_amd as sev
    want = [(0, ([], 50)),                       # one block there: wait, the third one is due at 50 (before the deadline 100)
            (50, ([(0, 2), (1, 3), (2, 1)], 50)),
            (60, ([], 500)),                     # only a future block is queued
            (500, ([], 600)),                    # it is alone: wait until it has waited 100
            (599, ([], 600)),
            (600, ([(3, 4)], 600)),
            (601, ([], -1))]
    for make in (lambda: so.Former(4, 16, 3, 100), lambda: sev.Scheduler(4, 16, 3, 100)):
        f = make()
        for r, (n, t) in enumerate([(2, 0), (3, 10), (1, 50), (4, 500)]):
            f.submit(r, n, t)
        for now, expect in want:
            assert f.next_batch(now) == expect, (now, expect)
    # the row cap stops a batch at the first block that does not fit, and nobody overtakes it
    for make in (lambda: so.Former(4, 8), lambda: sev.Scheduler(4, 8)):
        f = make()
        for r, n in enumerate([5, 4, 2]):
            f.submit(r, n, 0)
        assert f.next_batch(0) == ([(0, 5)], 0)            # 5 + 4 > 8: block 1 waits, and block 2 does not jump the queue
        assert f.next_batch(0) == ([(1, 4), (2, 2)], 0)


# ---------------------------------------------------------------- edge-side draft alignment

def test_oracle_edge_align_hand_cases():
    # sent: 0 -> 1 -> 2 (a chain); proactively drafted under the leaf 2: 3 (token 9) -> 4, and 5 (token 7) -> 6 -> 7
    parents = [-1, 0, 1, 2, 3, 2, 5, 6]
    tokens = [10, 11, 12, 9, 20, 7, 21, 22]
    assert so.edge_align(parents, tokens, [0, 1, 2], 7) == ([5, 6, 7], [-1, 0, 1])      # aligned on the second head
    assert so.edge_align(parents, tokens, [0, 1, 2], 9) == ([3, 4], [-1, 0])
    assert so.edge_align(parents, tokens, [0, 1, 2], 8) == ([], [])                       # the extra token was not drafted
    assert so.edge_align(parents, tokens, [0, 1], 7) == ([], [])                          # stopped early: 7 is not a child of node 1
    assert so.edge_align(parents, tokens, [0, 1], 12) == ([2, 3, 4, 5, 6, 7], [-1, 0, 1, 0, 3, 4])
    assert so.edge_align(parents, tokens, [], 10) == (list(range(8)), parents)            # nothing accepted, root matches the emitted token
    assert so.edge_align(parents, tokens, [], 11) == ([], [])


def test_library_edge_align_matches_oracle():
    import paper_2505_17052_amd as sev
    rng = np.random.default_rng(47)
    aligned = 0
    for trial in range(400):
        n = int(rng.integers(1, 40))
        parents = [-1] + [int(rng.integers(-1, i)) for i in range(1, n)]
        tokens = [int(x) for x in rng.integers(0, 6, size=n)]                            # few token values: matches and duplicate siblings happen
        path, cur = [], -1                                                                # a random root-to-node path
        while rng.random() < 0.7:
            kids = [i for i in range(n) if parents[i] == cur]
            if not kids:
                break
            cur = int(rng.choice(kids))
            path.append(cur)
        bonus = int(rng.integers(0, 6))
        got, want = sev.edge_align(parents, tokens, path, bonus), so.edge_align(parents, tokens, path, bonus)
        assert got == want, (trial, parents, tokens, path, bonus)
        aligned += bool(want[0])
    assert 50 < aligned < 350
    with pytest.raises(sev.SevError):
        sev.edge_align([-1, 0, 1], [1, 2, 3], [0, 2], 5)                                 # 2 is not a child of 0
    with pytest.raises(sev.SevError):
        sev.edge_align([-1, 1], [1, 2], [], 5)                                           # a node cannot be its own parent
