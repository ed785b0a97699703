"""Replay of the edge/server pipeline around the verification step (paper: "Server-side Pipeline-aware
Scheduling"): simulated edge devices and network on an integer-microsecond clock, the C++ batch former
(sev_sched_*) deciding the batches, and a caller-supplied verification step (the real GPU call, or a
time model).  Measurement harness: nothing here is on the verification hot path.

    python -m paper_2505_17052_amd.pipeline [--workload 8b-chain-b16k8] [--batches 40]

runs the replay on cuda:0 with the real sev_verify step at three round-trip times and prints, for each,
the calibrated draft depth and the server throughput with B requests in flight and with 2B.
"""
import argparse
import json
import sys
import time

from .binding import Scheduler, calibrate_depth


def replay(n_draft, draft_us, rtt_us, sched: Scheduler, verify, n_batches: int):
    """Runs n_batches verifications.  Request e lives on edge e: it drafts for draft_us[e], its block of
    n_draft[e] tokens reaches the server half a round trip later (first half rtt // 2), the answer takes
    the other half, and the edge drafts again at once.  verify(requests) -> (duration_us, emitted tokens
    per request).  Returns the batch log, emitted tokens per request, server busy time and end time."""
    E = len(n_draft)
    up = rtt_us // 2
    for e in range(E):
        sched.submit(e, n_draft[e], draft_us[e] + up)             # arrivals are submitted ahead of the clock
    tokens = [0] * E
    log, busy, now = [], 0, 0
    while len(log) < n_batches:
        batch, wake = sched.next_batch(now)
        if not batch:
            if wake < 0:
                raise RuntimeError("no block queued and no edge drafting: the replay cannot advance")
            now = wake
            continue
        reqs = [r for r, _ in batch]
        dur, emitted = verify(reqs)
        sched.record_verify(dur)
        log.append((now, reqs))
        busy += dur
        now += dur
        for r, m in zip(reqs, emitted):
            tokens[r] += m
            sched.submit(r, n_draft[r], now + rtt_us + draft_us[r])
    return {"log": log, "tokens": tokens, "busy_us": busy, "end_us": now}


def _gpu_main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", default="8b-chain-b16k8")
    ap.add_argument("--batches", type=int, default=40)
    ap.add_argument("--draft-fwd-us", type=int, default=1000, help="time of one draft-model forward pass on an edge device")
    ap.add_argument("--layers", type=int, default=0)
    args = ap.parse_args()
    import numpy as np
    import torch
    import synth
    from . import binding as sev
    from . import harness

    wl = synth.WORKLOADS[args.workload]
    shape = wl.shape if args.layers <= 0 else wl.shape.with_layers(args.layers)
    B, k = wl.B, wl.k_max
    E = 2 * B                                                   # twice as many requests in flight as fit one batch
    model = harness.build_model(shape, wl.seed)
    reqs = synth.make_requests(wl)
    lens = [reqs[e % B].prefix_len for e in range(E)]
    room = args.batches * (k + 1) + 2 * k + 16
    batch = harness.Batch(model, shape, [P + room for P in lens], max_rows=B * k, seed=wl.seed)
    batch.fill_synthetic(wl.seed, lens, [int(reqs[e % B].prefix_tokens[-1]) for e in range(E)])
    cur = list(lens)
    rng = np.random.default_rng(wl.seed)

    def verify(rs):
        n = len(rs)
        # synthetic edges: the first token is the server's own next token (always accepted), the rest random
        toks = rng.integers(0, shape.vocab, size=(n, k)).astype(np.int32)
        for i, r in enumerate(rs):
            toks[i, 0] = batch.kv.get_state(r)[1]
        d = torch.tensor(toks, device="cuda")
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = sev.verify_ex(model, batch.kv, [cur[r] for r in rs], d, k, slots=rs)
        sev.kv_commit(batch.kv, rs, n)
        torch.cuda.synchronize()
        dur = int((time.perf_counter() - t0) * 1e6)
        a = out["accept_len"].cpu().numpy()
        for i, r in enumerate(rs):
            cur[r] += int(a[i])
        return dur, [int(x) + 1 for x in a]

    for _ in range(3):                                          # warm-up, also the first verification-time samples
        t_verify, _ = verify(list(range(B)))
    out = {"workload": wl.name, "model_shape": shape.name, "B": B, "k": k, "t_verify_us": t_verify, "draft_fwd_us": args.draft_fwd_us, "runs": []}
    for rtt_ms in (15, 40, 50):                                 # the round-trip times of the paper's depth experiment, scaled below
        # the paper's server step takes 94 ms; this one takes milliseconds, so the network is scaled with it
        rtt = int(rtt_ms * 1000 * t_verify / 94200)
        depth = calibrate_depth(t_verify, args.draft_fwd_us, rtt, 1, 64)
        run = {"rtt_us": rtt, "depth": depth}
        for name, n_edges in (("B_in_flight", B), ("2B_in_flight", E)):
            s = Scheduler(B, B * k)
            r = replay([k] * n_edges, [depth * args.draft_fwd_us] * n_edges, rtt, s, verify, args.batches)
            run[name] = {"emitted_tokens_per_s": sum(r["tokens"]) / (r["end_us"] * 1e-6), "server_busy_frac": r["busy_us"] / r["end_us"],
                         "mean_batch": sum(len(b) for _, b in r["log"]) / len(r["log"])}
            s.close()
        run["throughput_ratio"] = run["2B_in_flight"]["emitted_tokens_per_s"] / run["B_in_flight"]["emitted_tokens_per_s"]
        out["runs"].append(run)
        print(f"[pipeline] rtt {rtt} us depth {depth}: " + json.dumps(run), file=sys.stderr, flush=True)
    flags = batch.kv.get_state(0)[2]
    assert flags == 0, f"device error flags {flags}"
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    _gpu_main()
