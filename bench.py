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

    nd = [r.n_draft for r in reqs]                                         # candidates per request (ragged for the interleaved workload)
    ragged = len(set(nd)) > 1
    parents_dev = None
    if wl.draft == "tree":
        # trees: the workload's seeded topologies; node 0 carries the slot's own prediction, the others random ids
        # (acceptance stops early, the forward pass is the same work)
        pars = np.stack([synth.tree_parents(wl.seed, b, k, wl.tree_depth) for b in range(B)]).astype(np.int32)
        parents_dev = torch.tensor(pars, device="cuda")
        drafts = np.stack([r.random_tokens[:k] for r in reqs]).astype(np.int32)
        drafts[:, 0] = nt0
    else:
        # chains: the model's own greedy continuation (k-1 single-token verify+commit rounds through the
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
        elif ragged:
            sev.verify_ex(model, batch.kv, lens, d_dev, k, draft_lens=nd, accept_len=acc, bonus_token=bon)
        else:
            sev.verify(model, batch.kv, lens, d_dev, parents_dev, B, k, acc, bon)
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
    step_bytes = shape.streamed_params() * 2 + sum(P + n for P, n in zip(lens, nd)) * shape.kv_bytes_per_token()
    tokens = sum(nd)
    traffic, traffic_note = traffic_from_profile(wl.name)
    classes_out = kernel_class_table(shape, tokens, lens, nd, per_class, empty_ms)
    out = {
        "metric": ("COMPARISON RUN (accept / resample rule at temperature 0.7): verified draft tokens/sec on 1 MI355X" if args.stochastic else
                   "COMPARISON RUN (padded KV + dense mask): verified draft tokens/sec on 1 MI355X" if args.padded_kv else
                   "verified draft tokens/sec on 1 MI355X (8B-shape bf16, B=16, k=8); % roofline" if wl.name == "8b-chain-b16k8" else
                   f"OTHER WORKLOAD ({wl.name}), not the headline: verified draft tokens/sec on 1 MI355X"),
        "value": tokens / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "emitted_tokens_per_s": float((accept + 1).sum()) / (ms_per_step * 1e-3),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "model_shape": shape.name, "B": B, "k": k, "draft": wl.draft, "rows_per_step": tokens,
                   "sum_prefix_tokens": int(sum(lens)), "page_size": 16,
                   "padded_kv": bool(args.padded_kv), "stochastic": bool(args.stochastic), "mean_accept_len": float(accept.mean()),
                   "accept_len": [int(a) for a in accept], "precision": "bf16 weights/KV, split-bf16 activations, f32 accumulate"},
        "roofline": {"bound": "hbm", "kernel": "gemm_gate_up_swiglu", "achieved": achieved, "peak": 8000.0, "unit": "GB/s",
                     "frac": achieved / 8000.0, "traffic": traffic, "traffic_source": traffic_note, "bytes_per_launch": gu_bytes,
                     "avg_launch_ms": gu_avg_ms, "launches_timed": gu_n, "empty_event_pair_ms": empty_ms,
                     "ms_per_step_with_events": (t4 - t3) * 1e3 / args.steps},
        "step_roofline": {"algorithmic_bytes_per_step": step_bytes, "achieved_GBps": step_bytes / (ms_per_step * 1e-3) / 1e9,
                          "frac_of_8TBps": step_bytes / (ms_per_step * 1e-3) / 8e12,
                          "gemm_flop_per_step": 2 * tokens * shape.streamed_params(),
                          "ms_per_step_by_kernel_class": per_class},
        "kernel_classes": classes_out,
        "paper_context": "context only, other hardware, not a target: the paper reports 2.22x server throughput and 11.24 % lower "
                         "inter-token latency for its whole edge/server system against server-only speculative decoding (server "
                         "NVIDIA A100 40/80 GB, edges RTX 4090, 14.07 ms RTT), and 94.2 ms per verification of a 32B model with a "
                         "32-token tree at batch 1 on an A100 80 GB",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, shape, reqs, lens, drafts, nt0, nd, None if parents_dev is None else pars)
    print(json.dumps(out), flush=True)


SOURCES_FOR_HASH = ("kernels_bf16.hip", "kernels_common.hip", "sev_api.hip", "sev_internal.h", "kv_layout.h")


def kernel_source_hash():
    """sha1 over the kernel and launch sources: ties a stored profile to the code it was taken from."""
    import hashlib
    h = hashlib.sha1()
    root = os.path.join(os.path.dirname(os.path.abspath(__file__)), "paper_2505_17052_amd", "csrc")
    for f in SOURCES_FOR_HASH:
        with open(os.path.join(root, f), "rb") as fh:
            h.update(fh.read())
    return h.hexdigest()[:16]


def traffic_from_profile(workload):
    """HBM bytes per gate/up launch from the committed rocprofv3 counter summary of this workload
    (profiles/gemm_gate_up_swiglu_<workload>_hbm_traffic.txt, line 'sev-traffic ...': FETCH_SIZE and WRITE_SIZE in KiB
    per dispatch and the factors a plain copy of known size gives each counter).  The summary names the hash of the
    sources it was measured on; with other sources the figure would be stale and None is reported instead."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"gemm_gate_up_swiglu_{workload}_hbm_traffic.txt")
    if not os.path.exists(path):
        return None, "no counter summary for this workload under profiles/"
    fields = {}
    for line in open(path):
        if line.startswith("sev-traffic "):
            fields = dict(kv.split("=", 1) for kv in line.split()[1:])
    if not fields:
        return None, "profiles summary has no sev-traffic line"
    if fields.get("source_sha") != kernel_source_hash() or os.environ.get("SEV_TUNE_GU") or os.environ.get("SEV_TUNE_TPB"):
        return None, f"profiles/{os.path.basename(path)} was measured on other sources ({fields.get('source_sha')}): stale, not reported"
    val = (float(fields["fetch_KiB"]) * float(fields["fetch_factor"]) + float(fields["write_KiB"]) * float(fields["write_factor"])) * 1024.0
    return val, f"profiles/{os.path.basename(path)}"


def kernel_class_table(shape, rows, lens, nd, per_class_ms, empty_ms):
    """Per kernel class of one step: algorithmic bytes and FLOP per launch span, event-timed duration, and the fraction
    of both rooflines (HBM 8 TB/s; dense bf16 matrix cores 2.5 PFLOP/s).  'mfma_useful' counts 2*M*N*K once; the
    split-bf16 activations make the matrix cores issue twice that ('mfma_issued').  'binding' is the roofline whose
    ideal time is longer.  A span holds the class's main kernel and its split-K fix-up / chunk merge; the events add
    about empty_event_pair_ms to every span (reported, not subtracted)."""
    d, F, V, L = shape.d_model, shape.d_ffn, shape.vocab, shape.n_layers
    qkv_n = shape.q_dim + 2 * shape.kv_dim
    kv_tokens = sum(P + n for P, n in zip(lens, nd))
    att_bytes = kv_tokens * 2 * shape.kv_dim * 2
    att_flop = 4 * shape.q_dim * sum(n * (P + n) for P, n in zip(lens, nd))
    spec = {
        "gemm_qkv": (qkv_n * d * 2, 2 * rows * qkv_n * d, L),
        "gemm_o": (d * shape.q_dim * 2, 2 * rows * d * shape.q_dim, L),
        "gemm_gate_up_swiglu": (2 * F * d * 2, 2 * rows * 2 * F * d, L),
        "gemm_down": (d * F * 2, 2 * rows * d * F, L),
        "gemm_lm_head_argmax": (V * d * 2, 2 * rows * V * d, 1),
        "attention": (att_bytes, att_flop, L),
    }
    out = {}
    for name, (nbytes, flop, n) in spec.items():
        ms = per_class_ms.get(name)
        if not ms:
            continue
        us = ms * 1e3 / n
        t = us * 1e-6
        hbm, useful = nbytes / t / 8e12, flop / t / 2.5e15
        out[name] = {"launches_per_step": n, "bytes_per_launch": nbytes, "flop_per_launch": flop, "avg_us_event_timed": us,
                     "hbm_frac": hbm, "mfma_useful_frac": useful, "mfma_issued_frac": 2 * useful,
                     "ideal_us_hbm": nbytes / 8e12 * 1e6, "ideal_us_mfma_issued": 2 * flop / 2.5e15 * 1e6,
                     "binding": "hbm" if nbytes / 8e12 >= 2 * flop / 2.5e15 else "mfma"}
    return out


def cpu_baseline(wl, shape, reqs, lens, drafts, nt0, nd, pars):
    """The CPU oracle's verify step (all requests, all layers, LM head, acceptance) timed on the host cores as it stands:
    weights widened to float32 once (not timed), then whole passes with the BLAS threads the process has, and one
    pass with a single thread.  Bounded sample: at most about 15 s of passes per leg."""
    import synth
    from oracle import verify_oracle as vo
    if shape.streamed_params() * 4 > 64e9:
        return {"value": None, "unit": "tokens/s", "cores": 0, "kind": "oracle",
                "sample": "not timed: the float32 oracle weights of this shape do not fit the host memory budget of a bench run"}
    src = synth.WeightSource(shape, wl.seed)
    om = vo.Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn, shape.vocab,
                  shape.rope_base, shape.rms_eps, tensor=src.tensor_f32, dtype=np.float32, kv_bf16=(shape.dtype == "bf16"))
    t0 = time.perf_counter()
    caches = []
    for b, P in enumerate(lens):
        c = vo.Cache(om, P + wl.k_max)
        for l in range(shape.n_layers):
            K, V = synth.synthetic_kv(shape, wl.seed, b, l, P)
            c.K[l][:P] = synth.bf16_bits_to_f32(K) if K.dtype == np.uint16 else K
            c.V[l][:P] = synth.bf16_bits_to_f32(V) if V.dtype == np.uint16 else V
        c.length, c.next_tok = P, int(nt0[b])
        caches.append(c)
    for nm in ("embed", "lm_head"):
        om.w(nm)
    for l in range(shape.n_layers):
        for nm in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            om.w(nm, l)
        if l % 8 == 7:
            log(f"  oracle weights widened up to layer {l}  ({time.perf_counter() - t0:.0f}s)")
    blocks = [drafts[b][:nd[b]] for b in range(len(lens))]
    par_list = None if pars is None else [pars[b] for b in range(len(lens))]

    def timed(budget_s, max_reps):
        reps, t = 0, time.perf_counter()
        while reps < 1 or (time.perf_counter() - t < budget_s and reps < max_reps):
            vo.verify(om, caches, blocks, par_list)
            reps += 1
        return (time.perf_counter() - t) / reps, reps

    vo.verify(om, caches, blocks, par_list)                                  # warm-up (page faults, BLAS thread start)
    full, reps = timed(12.0, 20)
    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        with threadpool_limits(limits=1):
            one, reps1 = timed(0.0, 1)
    except Exception:
        blas, one, reps1 = os.cpu_count(), None, 0
    log(f"oracle verify, full depth: {full:.3f}s per pass on {blas} BLAS threads ({reps} passes); 1 thread: {one}")
    n_tok = int(sum(nd))
    return {"value": n_tok / full, "unit": "tokens/s", "cores": int(min(blas, len(os.sched_getaffinity(0)))),
            "kind": "oracle", "seconds_per_step": full,
            "single_thread": None if one is None else {"value": n_tok / one, "unit": "tokens/s", "cores": 1, "seconds_per_step": one},
            "sample": f"the whole step (oracle verify of all {len(lens)} requests, all {shape.n_layers} layers, LM head, acceptance) "
                      f"measured, not extrapolated: {reps} passes with the BLAS threads of the process, {reps1} pass with one "
                      f"thread; weights widened to float32 beforehand ({time.perf_counter() - t0:.0f}s in all)"}


if __name__ == "__main__":
    main()
