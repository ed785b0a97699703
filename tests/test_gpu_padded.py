"""GPU test of the padded-KV comparison variant (mode | 2 of sev_verify_ex): the paper's handling of a
heterogeneous batch (section 4.3: every sequence padded to the longest one under a per-sequence mask).
Attention then walks the longest sequence's number of cache slots for every request; the results must
be those of the ragged path (same tolerances against the oracle; decisions identical to the ragged run)."""
import numpy as np
import pytest
import torch

import synth
from oracle import verify_oracle as vo
from tests.helpers import oracle_model, corrupt_chain, announce, oracle_caches_synthetic, tree_tokens
from tests.test_gpu_bf16_mini import _compare, _wl, SHAPE, SEED

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    model = harness.build_model(SHAPE, SEED)
    om = oracle_model(SHAPE, SEED, dtype=np.float32)
    return sev, harness, model, om


def _batch(setup, lens, k, cap):
    sev, harness, model, om = setup
    reqs = synth.make_requests(_wl(len(lens), k, "chain", lens))
    last = [int(r.random_tokens[-1]) for r in reqs]
    batch = harness.Batch(model, SHAPE, cap, max_rows=len(lens) * k, seed=SEED)
    batch.fill_synthetic(SEED, lens, last)
    return reqs, batch, oracle_caches_synthetic(om, SHAPE, SEED, lens, last)


def test_padded_chains_equal_ragged(setup):
    sev, harness, model, om = setup
    lens, k = [37, 700, 64, 129, 1], 8                     # the longest request sets everybody's walk: 45 pages
    announce(f"padded KV: chains, lens {lens}")
    reqs, batch, caches = _batch(setup, lens, k, [max(lens) + k + 16] * len(lens))
    gs = vo.greedy_continuation(om, caches, k)
    drafts = np.stack([corrupt_chain(gs[b], reqs[b], k) for b in range(len(lens))]).astype(np.int32)
    drafts[0] = gs[0][:k]
    d = torch.tensor(drafts, device="cuda")
    outs = {}
    for name, mode in (("ragged", 0), ("padded", 2)):
        for b in range(len(lens)):
            batch.kv.set_state(b, lens[b], caches[b].next_tok)
        outs[name] = sev.verify_ex(model, batch.kv, lens, d, k, mode=mode, want_path=True, want_argmax=True, want_logits=True)
        torch.cuda.synchronize()
        assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [drafts[b] for b in range(len(lens))])
    n_exact, worst, mean = _compare(outs["padded"], res, len(lens), k)
    for key in ("accept_len", "bonus_token", "accept_path", "row_argmax"):
        assert torch.equal(outs["ragged"][key], outs["padded"][key]), key
    dl = (outs["ragged"]["logits"] - outs["padded"]["logits"]).abs().max().item()
    announce(f"  exact-compared {n_exact}/{len(lens)}, logits vs oracle max {worst:.2e} mean {mean:.2e}; padded vs ragged max {dl:.2e}")
    assert dl < 5e-3                                        # same arithmetic, different chunking of the softmax sums
    sev.kv_commit(batch.kv, None, len(lens))
    for b in range(len(lens)):
        assert batch.kv.get_state(b) == (lens[b] + int(outs["padded"]["accept_len"][b]), int(outs["padded"]["bonus_token"][b]), 0)


def test_padded_trees_equal_ragged(setup):
    sev, harness, model, om = setup
    lens, n = [150, 18, 333], 16
    announce(f"padded KV: trees of {n} nodes, lens {lens}")
    reqs, batch, caches = _batch(setup, lens, n, [max(lens) + n + 16] * len(lens))
    pars = [synth.tree_parents(SEED, b, n, 5) for b in range(len(lens))]
    toks = tree_tokens(om, caches, pars, reqs, SHAPE.vocab)
    d = torch.tensor(np.stack(toks).astype(np.int32), device="cuda")
    par = torch.tensor(np.stack(pars).astype(np.int32), device="cuda")
    outs = {}
    for name, mode in (("ragged", 0), ("padded", 2)):
        for b in range(len(lens)):
            batch.kv.set_state(b, lens[b], caches[b].next_tok)
        outs[name] = sev.verify_ex(model, batch.kv, lens, d, n, parents=par, mode=mode, want_path=True, want_argmax=True, want_logits=True)
        torch.cuda.synchronize()
        assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, toks, pars)
    n_exact, worst, mean = _compare(outs["padded"], res, len(lens), n)
    for key in ("accept_len", "bonus_token", "accept_path", "row_argmax"):
        assert torch.equal(outs["ragged"][key], outs["padded"][key]), key
    announce(f"  accept {[r.accept_len for r in res]}, exact-compared {n_exact}/{len(lens)}")


def test_padded_needs_pages_up_to_the_longest(setup):
    sev, harness, model, om = setup
    lens, k = [20, 200], 4
    reqs, batch, caches = _batch(setup, lens, k, [P + k + 16 for P in lens])     # the short request's pages end long before 204 tokens
    d = torch.zeros((2, k), dtype=torch.int32, device="cuda")
    with pytest.raises(sev.SevError):
        sev.verify_ex(model, batch.kv, lens, d, k, mode=2)
    sev.verify_ex(model, batch.kv, lens, d, k, mode=0)      # the ragged call is fine
    torch.cuda.synchronize()
