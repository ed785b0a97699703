"""Glue used by the tests: wraps the seeded weight source as an oracle model and
builds draft blocks from the oracle's own greedy continuation."""
import numpy as np

import synth
from oracle import verify_oracle as vo


def oracle_model(shape: synth.ModelShape, seed: int, dtype=np.float64, cache_weights=True, gains=False) -> vo.Model:
    """gains=True: seeded non-unit RMSNorm gains (synth.WeightSource.gain) instead of ones."""
    src = synth.WeightSource(shape, seed)
    return vo.Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                    shape.d_ffn, shape.vocab, shape.rope_base, shape.rms_eps,
                    tensor=src.tensor_f32, dtype=dtype, cache_weights=cache_weights,
                    kv_bf16=(shape.dtype == "bf16"), gains=src.gain if gains else None)


def corrupt_chain(greedy: np.ndarray, req: synth.workload.Request, n: int) -> np.ndarray:
    """Draft = greedy continuation with position j replaced by a random id iff its draw < p."""
    d = np.array(greedy[:n], dtype=np.int64)
    for j in range(n):
        if req.corrupt_draw[j] < req.corrupt_p:
            d[j] = req.random_tokens[j]
    return d


def decision_gap_ok(res, gap_min: float) -> bool:
    """True iff every arg-max the oracle's acceptance walk relied on (the nodes of its accepted path;
    the last of them also produced the stop decision and the bonus token) has a top-1/top-2 logit gap
    of at least gap_min.  Only such requests are compared bit-exactly."""
    return all(res.top2_gap[i] >= gap_min for i in res.path)


def greedy_in_place(om, caches, k: int):
    """Plain greedy decoding, k single-token forwards from each cache, WITHOUT copying the caches (the large
    shapes' caches are tens of GB): the decoded tokens' K/V are written behind the committed length, which is put
    back afterwards, so the caches end as they started.  Same result as vo.greedy_continuation."""
    state = [(c.length, c.next_tok) for c in caches]
    out = [[c.next_tok] for c in caches]
    for _ in range(k):
        vo.extend(om, caches, [np.array([o[-1]]) for o in out])
        for r, c in enumerate(caches):
            out[r].append(c.next_tok)
    for c, (n, t) in zip(caches, state):
        c.length, c.next_tok, c.pending = n, t, None
    return [np.array(o, dtype=np.int64) for o in out]


def announce(msg: str):
    print(f"[case] {msg}", flush=True)


def oracle_caches_synthetic(om, shape, seed, prefix_lens, last_tokens, extra=80):
    """Oracle-side twin of harness.Batch.fill_synthetic: drawn K/V for positions 0..P-2, then a real
    forward over the last prefix token (position P-1), which also yields next_tok."""
    caches = []
    for b, P in enumerate(prefix_lens):
        c = vo.Cache(om, P + extra)
        if P > 1:
            for l in range(shape.n_layers):
                K, V = synth.synthetic_kv(shape, seed, b, l, P - 1)
                if K.dtype == np.uint16:
                    K, V = synth.bf16_bits_to_f32(K), synth.bf16_bits_to_f32(V)
                c.K[l][:P - 1] = K
                c.V[l][:P - 1] = V
        c.length = P - 1
        caches.append(c)
    vo.extend(om, caches, [np.array([int(t)]) for t in last_tokens])
    return caches


def tree_tokens(om, caches, parents_list, reqs, vocab, p_keep=0.7):
    """Tokens for draft trees, level by level: at every node one designated child receives the target's
    own arg-max with probability p_keep (else a random id); its siblings get distinct random ids.
    Uses one oracle forward per level (the tree so far) to learn the arg-max at the new parents."""
    R = len(caches)
    toks = [np.zeros(len(p), dtype=np.int64) for p in parents_list]
    deps = [vo.depths(np.asarray(p)) for p in parents_list]
    max_d = max(int(d.max()) for d in deps)
    amax = [None] * R
    for lvl in range(max_d + 1):
        for r in range(R):
            par, req = np.asarray(parents_list[r]), reqs[r]
            nodes = [i for i in range(len(par)) if deps[r][i] == lvl]
            by_parent = {}
            for i in nodes:
                by_parent.setdefault(int(par[i]), []).append(i)
            for pnode, kids in by_parent.items():
                want = caches[r].next_tok if pnode < 0 else int(amax[r][pnode])
                used = set()
                for j, i in enumerate(kids):
                    if j == 0 and req.corrupt_draw[i % len(req.corrupt_draw)] < p_keep:
                        t = want
                    else:
                        t = int(req.random_tokens[i % len(req.random_tokens)])
                        while t in used or t == want:
                            t = (t + 1) % vocab
                    used.add(t)
                    toks[r][i] = t
        # arg-max at all nodes placed so far (deeper nodes still hold 0: they do not influence shallower ones)
        lg, _, _ = vo.forward_blocks(om, caches, toks, parents_list)
        amax = [np.argmax(l, axis=-1) for l in lg]
    return toks
