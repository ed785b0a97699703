"""GPU parity of sev_verify_sample (stochastic verification of chains at temperature 0.7) against the
oracle's accept / resample rule, on the float32 tiny model and the bf16 small GQA model.  The random
numbers and the edge distributions are seeded inputs shared by both sides.  A decision is compared
exactly where it is firm: an acceptance test whose two sides differ by more than 1e-3 relative, an
inverse-CDF draw that lands more than 1e-4 (of the total weight) inside its cell; what float32 against
float64 arithmetic can flip is exempt (and counted)."""
import numpy as np
import pytest
import torch

import synth
from oracle import verify_oracle as vo
from tests.helpers import oracle_model, announce, oracle_caches_synthetic

pytestmark = pytest.mark.gpu

T = 0.7


def _uniforms(seed, purpose, n):
    from synth.workload import P_CORRUPT
    return synth.uniform_f64(seed, synth.stream_id(P_CORRUPT, 700 + purpose), n)


def _edge_blocks(om, caches, k, seed, noise):
    """Edge side: candidate 0 = the server's previous token; candidate i >= 1 drawn from q_i = softmax((server
    logits + noise) / T), a perturbed copy of the server distribution (so that some proposals are rejected)."""
    B, V = len(caches), om.vocab
    drafts = np.zeros((B, k), dtype=np.int64)
    q = np.zeros((B, k, V))
    cs = [c.copy() for c in caches]
    for b in range(B):
        drafts[b, 0] = cs[b].next_tok
        q[b, 0] = 1.0 / V
    rng = np.random.default_rng(seed)
    for i in range(1, k):
        lg = vo.extend(om, cs, [np.array([drafts[b, i - 1]]) for b in range(B)])
        for b in range(B):
            q[b, i] = vo.softmax_t(lg[b][0] + noise * rng.standard_normal(V), T)
            u = _uniforms(seed, 10 * b + 1, k)[i]
            drafts[b, i] = vo.inverse_cdf(q[b, i], u)[0]
    return drafts, q


def _run(shape, seed, lens, k, dtype, noise, acc_eps, logit_tol):
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    model = harness.build_model(shape, seed)
    om = oracle_model(shape, seed, dtype=dtype)
    B = len(lens)
    last = [int(synth.uniform_i32(seed, 5000 + b, 1, 0, shape.vocab)[0]) for b in range(B)]
    batch = harness.Batch(model, shape, [P + 80 for P in lens], max_rows=B * k, seed=seed)
    batch.fill_synthetic(seed, lens, last)
    caches = oracle_caches_synthetic(om, shape, seed, lens, last)
    drafts, q = _edge_blocks(om, caches, k, seed, noise)
    u_acc = np.stack([_uniforms(seed, 10 * b + 2, k) for b in range(B)])
    u_emit = np.array([_uniforms(seed, 10 * b + 3, 1)[0] for b in range(B)])
    drafts[B - 1, 0] = (drafts[B - 1, 0] + 1) % shape.vocab          # one edge is out of step: nothing accepted
    for b in range(B):
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_sample(model, batch.kv, lens, torch.tensor(drafts.astype(np.int32), device="cuda"), k,
                            torch.tensor(q.reshape(B * k, -1).astype(np.float32), device="cuda"),
                            torch.tensor(u_acc.astype(np.float32), device="cuda"), torch.tensor(u_emit.astype(np.float32), device="cuda"), T)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    # both sides see the same float32 inputs
    res = vo.verify_sample(om, caches, [drafts[b] for b in range(B)], [q[b].astype(np.float32) for b in range(B)],
                           [u_acc[b].astype(np.float32) for b in range(B)], [np.float32(u_emit[b]) for b in range(B)], T)
    lg = out["logits"].cpu().numpy()
    acc, emi = out["accept_len"].cpu().numpy(), out["emitted_token"].cpu().numpy()
    n_exact = 0
    for b in range(B):
        d = np.abs(lg[b * k:(b + 1) * k] - res[b].logits)
        assert d.max() < logit_tol[0] and d.mean() < logit_tol[1], (b, d.max(), d.mean())
        if res[b].accept_margin > acc_eps:
            assert acc[b] == res[b].accept_len, (b, acc[b], res[b].accept_len)
            if res[b].emit_margin > 1e-4:
                n_exact += 1
                assert emi[b] == res[b].emitted, (b, emi[b], res[b].emitted)
    announce(f"  accept {[r.accept_len for r in res]}, emitted exact-compared {n_exact}/{B}")
    assert acc[B - 1] == 0 and emi[B - 1] == caches[B - 1].next_tok
    assert n_exact >= B // 2
    # commit applies the accepted prefix and the emitted token
    sev.kv_commit(batch.kv, None, B)
    for b in range(B):
        assert batch.kv.get_state(b) == (lens[b] + int(acc[b]), int(emi[b]), 0)


def test_sample_tiny_f32():
    announce("stochastic verification, tiny f32")
    _run(synth.TINY, 23, [40, 64, 17, 5], 6, np.float64, noise=0.7, acc_eps=1e-3, logit_tol=(1e-4, 1e-5))


def test_sample_mini_bf16():
    announce("stochastic verification, mini bf16")
    _run(synth.MINI_BF16, 606, [37, 300, 64, 129, 5], 8, np.float32, noise=0.7, acc_eps=3e-2, logit_tol=(3e-2, 3e-3))


def _edge_trees(om, caches, parents, seed, noise):
    """Edge side for trees: node 0 is the root (the server's previous token); the children of a node are
    independent draws from one q = softmax((server logits at the node + noise) / T).  Built level by level
    with one oracle pass over the tree so far per level."""
    B, V = len(caches), om.vocab
    n = len(parents)
    dep = vo.depths(np.asarray(parents))
    toks = np.zeros((B, n), dtype=np.int64)
    q = np.full((B, n, V), 1.0 / V)
    rng = np.random.default_rng(seed + 1)
    for b in range(B):
        toks[b, 0] = caches[b].next_tok
    for lvl in range(1, int(dep.max()) + 1):
        known = [i for i in range(n) if dep[i] < lvl]
        sub_par = np.asarray([parents[i] for i in known])            # parents precede children and levels are contiguous in index order
        assert known == list(range(len(known)))
        for b in range(B):
            lg = vo.forward_blocks(om, [caches[b]], [toks[b, :len(known)]], [sub_par])[0][0]
            for c in range(n):
                if dep[c] != lvl:
                    continue
                par = parents[c]
                first = min(j for j in range(n) if parents[j] == par and dep[j] == lvl)
                if c == first:
                    q[b, c] = vo.softmax_t(lg[par] + noise * rng.standard_normal(V), T)
                else:
                    q[b, c] = q[b, first]
                toks[b, c] = vo.inverse_cdf(q[b, c], rng.random())[0]
    return toks, q


def _run_tree(shape, seed, lens, dtype, noise, acc_eps, logit_tol):
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    model = harness.build_model(shape, seed)
    om = oracle_model(shape, seed, dtype=dtype)
    B = len(lens)
    # root; three proposals for its successor; two of them continued, one twice
    parents = np.array([-1, 0, 0, 0, 1, 1, 2, 4, 4, 7], dtype=np.int64)
    n = len(parents)
    last = [int(synth.uniform_i32(seed, 6000 + b, 1, 0, shape.vocab)[0]) for b in range(B)]
    batch = harness.Batch(model, shape, [P + 80 for P in lens], max_rows=B * n, seed=seed)
    batch.fill_synthetic(seed, lens, last)
    caches = oracle_caches_synthetic(om, shape, seed, lens, last)
    toks, q = _edge_trees(om, caches, parents, seed, noise)
    u_acc = np.stack([_uniforms(seed, 10 * b + 4, n) for b in range(B)])
    u_emit = np.array([_uniforms(seed, 10 * b + 5, 1)[0] for b in range(B)])
    for b in range(B):
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    pars = np.tile(parents.astype(np.int32), (B, 1))
    out = sev.verify_sample(model, batch.kv, lens, torch.tensor(toks.astype(np.int32), device="cuda"), n,
                            torch.tensor(q.reshape(B * n, -1).astype(np.float32), device="cuda"),
                            torch.tensor(u_acc.astype(np.float32), device="cuda"), torch.tensor(u_emit.astype(np.float32), device="cuda"), T,
                            parents=torch.tensor(pars, device="cuda"))
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify_sample_tree(om, caches, [toks[b] for b in range(B)], [parents] * B, [q[b].astype(np.float32) for b in range(B)],
                                [u_acc[b].astype(np.float32) for b in range(B)], [np.float32(u_emit[b]) for b in range(B)], T)
    lg = out["logits"].cpu().numpy()
    acc, emi = out["accept_len"].cpu().numpy(), out["emitted_token"].cpu().numpy()
    n_exact = 0
    for b in range(B):
        r, path = res[b]
        d = np.abs(lg[b * n:(b + 1) * n] - r.logits)
        assert d.max() < logit_tol[0] and d.mean() < logit_tol[1], (b, d.max(), d.mean())
        if r.accept_margin > acc_eps:
            assert acc[b] == r.accept_len and out["accept_path"][b].cpu().tolist()[:r.accept_len] == path, (b, acc[b], r.accept_len, path)
            if r.emit_margin > 1e-4:
                n_exact += 1
                assert emi[b] == r.emitted, (b, emi[b], r.emitted)
    announce(f"  tree accept {[r.accept_len for r, _ in res]} paths {[p for _, p in res]}, emitted exact-compared {n_exact}/{B}")
    assert n_exact >= B // 2
    sev.kv_commit(batch.kv, None, B)
    for b in range(B):
        assert batch.kv.get_state(b) == (lens[b] + int(acc[b]), int(emi[b]), 0)


def test_sample_tree_tiny_f32():
    announce("stochastic tree verification, tiny f32")
    _run_tree(synth.TINY, 29, [40, 64, 17, 5, 33, 90], np.float64, noise=1.0, acc_eps=1e-3, logit_tol=(1e-4, 1e-5))


def test_sample_tree_mini_bf16():
    announce("stochastic tree verification, mini bf16")
    _run_tree(synth.MINI_BF16, 606, [37, 300, 64, 129], np.float32, noise=1.0, acc_eps=3e-2, logit_tol=(3e-2, 3e-3))
