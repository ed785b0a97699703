#!/usr/bin/env python3
"""Benchmark of the batched verification step on one MI355X.

A step = sev_verify (one target forward over B*k draft tokens against the paged KV prefixes, fused
arg-max, greedy acceptance) + sev_kv_commit + one sev_kv_set_state launch that rewinds the slots so
that every step sees the same input.  Workload: "8b-chain-b16k8" (Llama-3-8B-shaped bf16 model,
random-init; B=16 requests, prefix lengths U[256,2048], 16-token pages, k=8 chain drafts made from
the model's own greedy continuation with corruption p=0.3), all inputs resident in HBM.

Prints ONE JSON line: verified draft tokens/s, the roofline of the dominant kernel (gate/up GEMM,
timed with HIP events on the launch stream) and the CPU oracle timed on a bounded sample.
"""
import argparse
import json
import os
import sys
import time

import numpy as np


def log(msg):
    print(f"[bench] {msg}", file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="8b-chain-b16k8")
    ap.add_argument("--layers", type=int, default=0, help="truncate the model (debugging only; result is then not the headline metric)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--padded-kv", action="store_true",
                    help="comparison run, not the headline: attention walks the longest request's length for every request "
                         "(the paper's padded KV + dense mask); reported under its own metric name")
    ap.add_argument("--stochastic", action="store_true",
                    help="comparison run, not the headline: the accept / resample rule at temperature 0.7 (sev_verify_sample) with "
                         "synthetic edge distributions; reported under its own metric name")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (a kernel of known HBM traffic, for scaling rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no sharding, no collectives); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import synth
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness

    wl = synth.WORKLOADS[args.workload]
    shape = wl.shape if args.layers <= 0 else wl.shape.with_layers(args.layers)
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    t0 = time.time()
    log(f"building {shape.name} ({shape.streamed_params() * 2 / 1e9:.2f} GB of streamed weights)")
    model = harness.build_model(shape, wl.seed, progress=lambda l: log(f"  layer {l} loaded") if l % 8 == 7 else None)
    reqs = synth.make_requests(wl)
    lens = [r.prefix_len for r in reqs]
    B, k = wl.B, wl.k_max
    cap = [(max(lens) if args.padded_kv else P) + k + 16 for P in lens]
    batch = harness.Batch(model, shape, cap, max_rows=B * k, seed=wl.seed)
    log(f"filling caches: B={B}, sum of prefix lengths {sum(lens)}  ({time.time() - t0:.0f}s)")
    batch.fill_synthetic(wl.seed, lens, [int(r.prefix_tokens[-1]) for r in reqs])
    nt0 = [batch.kv.get_state(b)[1] for b in range(B)]

    # drafts: the model's own greedy continuation (k-1 single-token verify+commit rounds through the
    # library), then each position replaced by a random id with probability p
    g = np.zeros((B, k), dtype=np.int32)
    g[:, 0] = nt0
    cur = list(lens)
    for i in range(1, k):
        a, bt = sev.verify(model, batch.kv, cur, torch.tensor(g[:, i - 1:i].copy(), device="cuda"), None, B, 1)
        sev.kv_commit(batch.kv, None, B)
        torch.cuda.synchronize()
        assert int(a.min()) == 1
        g[:, i] = bt.cpu().numpy()
        cur = [c + 1 for c in cur]
    drafts = g.copy()
    for b, r in enumerate(reqs):
        for j in range(k):
            if r.corrupt_draw[j] < r.corrupt_p:
                drafts[b, j] = r.random_tokens[j]
    d_dev = torch.tensor(drafts, device="cuda")
    acc = torch.empty(B, dtype=torch.int32, device="cuda")
    bon = torch.empty(B, dtype=torch.int32, device="cuda")

    if args.stochastic:
        # edge distributions: a softmax of seeded normal scores (scale 3: a few likely ids per row, like a small draft
        # model's output), the drafts drawn greedily from them except node 0 (the server's previous token)
        gen = torch.Generator(device="cuda").manual_seed(wl.seed)
        q_dev = torch.softmax(3.0 * torch.randn(B * k, shape.vocab, device="cuda", generator=gen), dim=-1).contiguous()
        u_acc = torch.rand(B, k, device="cuda", generator=gen)
        u_emit = torch.rand(B, device="cuda", generator=gen)
        batch.kv.set_state(None, lens, nt0)                                # rewind the greedy continuation above
        s_out = sev.verify_sample(model, batch.kv, lens, d_dev, k, q_dev, u_acc, u_emit, 0.7)
        acc = s_out["accept_len"]

    def step():
        if args.stochastic:
            sev.verify_sample(model, batch.kv, lens, d_dev, k, q_dev, u_acc, u_emit, 0.7, out=s_out)
        elif args.padded_kv:
            sev.verify_ex(model, batch.kv, lens, d_dev, k, mode=2, accept_len=acc, bonus_token=bon)
        else:
            sev.verify(model, batch.kv, lens, d_dev, None, B, k, acc, bon)
        sev.kv_commit(batch.kv, None, B)
        batch.kv.set_state(None, lens, nt0)

    if args.calibration_copy:
        src_t = torch.full((1 << 30,), 7, dtype=torch.uint8, device="cuda")
        dst_t = torch.empty_like(src_t)
        for _ in range(3):
            dst_t.copy_(src_t)
        torch.cuda.synchronize()
        del src_t, dst_t
    batch.kv.set_state(None, lens, nt0)
    log(f"warm-up {args.warmup}, timing {args.steps} steps  ({time.time() - t0:.0f}s)")
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    ms_per_step = (t2 - t1) * 1e3 / args.steps
    accept = acc.cpu().numpy()
    flags = batch.kv.get_state(0)[2]
    assert flags == 0, f"device error flags {flags}"

    # per-kernel device time: HIP events on the launch stream around every launch of each class
    classes = batch.kv.profile_classes()
    gu = classes.index("gemm_gate_up_swiglu")
    batch.kv.profile_enable(1 << gu)
    torch.cuda.synchronize()
    t3 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t4 = time.perf_counter()
    gu_ms, gu_n = batch.kv.profile_read()["gemm_gate_up_swiglu"]
    batch.kv.profile_enable((1 << len(classes)) - 1)
    for _ in range(5):
        step()
    torch.cuda.synchronize()
    per_class = {nm: (ms / 5.0) for nm, (ms, n) in batch.kv.profile_read().items()}
    batch.kv.profile_enable(0)

    # what a pair of events reads around an empty interval on the same stream, in the middle of the same queue of
    # kernels: the part of avg_launch_ms that is not the kernel itself (reported, not subtracted)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(64)]
    for a, b in ev:
        step()
        a.record()
        b.record()
    torch.cuda.synchronize()
    empty_ms = float(np.median([a.elapsed_time(b) for a, b in ev]))

    gu_bytes = 2 * shape.d_ffn * shape.d_model * 2                      # gate and up matrices, bf16, read once
    gu_avg_ms = gu_ms / max(gu_n, 1)
    achieved = gu_bytes / (gu_avg_ms * 1e-3) / 1e9
    step_bytes = shape.streamed_params() * 2 + sum(P + k for P in lens) * shape.kv_bytes_per_token()
    tokens = B * k
    # HBM bytes per gate/up launch from the rocprofv3 FETCH_SIZE and WRITE_SIZE runs kept under profiles/
    # (KiB per dispatch x the factor a plain 1 GiB copy gives each counter); they hold for this one launch shape
    traffic = (123035.7 * 2.0 + 7168.0 * 1.0) * 1024.0 if (wl.name == "8b-chain-b16k8" and not os.environ.get("SEV_TUNE_GU")) else None
    out = {
        "metric": ("COMPARISON RUN (accept / resample rule at temperature 0.7): verified draft tokens/sec on 1 MI355X" if args.stochastic else
                   "COMPARISON RUN (padded KV + dense mask): verified draft tokens/sec on 1 MI355X" if args.padded_kv else
                   "verified draft tokens/sec on 1 MI355X (8B-shape bf16, B=16, k=8); % roofline"),
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "emitted_tokens_per_s": float((accept + 1).sum()) / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "model_shape": shape.name, "B": B, "k": k, "rows_per_step": tokens,
                   "sum_prefix_tokens": int(sum(lens)), "page_size": 16,
                   "padded_kv": bool(args.padded_kv), "stochastic": bool(args.stochastic), "mean_accept_len": float(accept.mean()), "precision": "bf16 weights/KV, split-bf16 activations, f32 accumulate"},
        "roofline": {"bound": "hbm", "kernel": "gemm_gate_up_swiglu", "achieved": achieved, "peak": 8000.0, "unit": "GB/s",
                     "frac": achieved / 8000.0, "traffic": traffic, "bytes_per_launch": gu_bytes,
                     "avg_launch_ms": gu_avg_ms, "launches_timed": gu_n, "empty_event_pair_ms": empty_ms,
                     "ms_per_step_with_events": (t4 - t3) * 1e3 / args.steps},
        "step_roofline": {"algorithmic_bytes_per_step": step_bytes, "achieved_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                          "frac_of_8TBps": step_bytes / (ms_per_step * 1e-3) / 8e12,
                          "gemm_flop_per_step": 2 * tokens * shape.streamed_params(),
                          "ms_per_step_by_kernel_class": per_class},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, shape, reqs, lens, drafts, nt0)
    print(json.dumps(out), flush=True)


def cpu_baseline(wl, shape, reqs, lens, drafts, nt0):
    """The CPU oracle's verify step timed on the host cores, on a bounded sample: the first layers of
    the model (all requests, full prefixes, LM head included), extrapolated linearly in depth."""
    import synth
    from oracle import verify_oracle as vo
    sample_layers = (1, 3) if shape.n_layers >= 3 else (shape.n_layers, shape.n_layers)
    times = {}
    src = synth.WeightSource(shape, wl.seed)
    for nl in sample_layers:
        om = vo.Model(nl, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                      shape.rope_base, shape.rms_eps, tensor=src.tensor_f32, dtype=np.float32, kv_bf16=(shape.dtype == "bf16"))
        caches = []
        for b, P in enumerate(lens):
            c = vo.Cache(om, P + wl.k_max)
            for l in range(nl):
                K, V = synth.synthetic_kv(shape, wl.seed, b, l, P)
                c.K[l][:P] = synth.bf16_bits_to_f32(K) if K.dtype == np.uint16 else K
                c.V[l][:P] = synth.bf16_bits_to_f32(V) if V.dtype == np.uint16 else V
            c.length, c.next_tok = P, int(nt0[b])
            caches.append(c)
        for nm in ("embed", "lm_head"):
            om.w(nm)
        for l in range(nl):
            for nm in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
                om.w(nm, l)
        reps = 0
        t = time.perf_counter()
        while reps < 3 or (time.perf_counter() - t < 6.0 and reps < 200):      # about 6 s of oracle work per depth
            vo.verify(om, caches, [drafts[b] for b in range(len(lens))])
            reps += 1
        times[nl] = (time.perf_counter() - t) / reps
        log(f"oracle verify with {nl} layer(s): {times[nl]:.3f}s per pass, {reps} passes")
    a, b = sample_layers
    per_layer = (times[b] - times[a]) / (b - a) if b > a else times[a] / a
    fixed = max(times[a] - a * per_layer, 0.0)
    full = fixed + shape.n_layers * per_layer
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        blas = os.cpu_count()
    return {"value": len(lens) * wl.k_max / full, "unit": "tokens/s", "cores": int(min(blas, len(os.sched_getaffinity(0)))),
            "kind": "oracle", "est_seconds_per_step": full,
            "sample": f"oracle verify of all {len(lens)} requests timed with {a} and {b} of {shape.n_layers} layers "
                      f"(+embedding, LM head, acceptance), about 6 s of repeated passes at each depth; per-layer time "
                      f"extrapolated to full depth"}


if __name__ == "__main__":
    main()
