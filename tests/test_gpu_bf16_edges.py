"""GPU parity of the bfloat16 path at the edges of the interface, on the small GQA model:
the largest batch (256 requests of one draft token), the longest chain (64 draft tokens in one
request), prefixes that end exactly on and right after a page boundary, a one-token prefix, rollback
followed by a second verify, and a fork (a block with several roots).  Same tolerances as the other
bf16 tests (logits max-abs 3e-2, mean-abs 3e-3; integers exact where the oracle's decisions are firm)."""
import numpy as np
import pytest
import torch

import synth
from oracle import verify_oracle as vo
from tests.helpers import oracle_model, corrupt_chain, decision_gap_ok, announce, oracle_caches_synthetic
from tests.test_gpu_bf16_mini import _make, _compare, SHAPE, SEED, GAP_MIN

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def setup():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    announce(f"build model {SHAPE.name}")
    model = harness.build_model(SHAPE, SEED)
    om = oracle_model(SHAPE, SEED, dtype=np.float32)
    return sev, harness, model, om


def test_largest_batch_single_token_drafts(setup):
    sev, harness, model, om = setup
    B = 256                                               # SEV_MAX_BATCH
    lens = [1 + (7 * b) % 45 for b in range(B)]           # 1..45 tokens: one to three pages each
    announce(f"edges: B={B}, k=1")
    reqs, batch, caches = _make(setup, lens, 1, B)
    drafts = np.zeros((B, 1), dtype=np.int32)
    for b in range(B):                                    # even requests send the target's own token, odd ones a wrong one
        drafts[b, 0] = caches[b].next_tok if b % 2 == 0 else (caches[b].next_tok + 1) % SHAPE.vocab
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(drafts, device="cuda"), 1, want_path=True, want_argmax=True,
                        want_logits=True)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [drafts[b] for b in range(B)])
    n_exact, worst, mean = _compare(out, res, B, 1)
    announce(f"  exact-compared {n_exact}/{B}, logits max {worst:.2e} mean {mean:.2e}")
    acc = out["accept_len"].cpu().numpy()
    assert np.array_equal(acc, np.array([1 if b % 2 == 0 else 0 for b in range(B)]))   # integer inputs decide this exactly
    assert n_exact >= B // 2


def test_maximum_batch_times_maximum_draft_length(setup):
    """Both interface limits at once: 256 requests (SEV_MAX_BATCH) of up to 64 candidates (SEV_MAX_DRAFT), 15 360 GEMM
    rows in one call, with a ragged tail (every fourth request sends fewer candidates, some only one).  Every
    request is compared with the oracle.  The first candidates continue the oracle's greedy decoding for a while
    (a different number per request), the rest are random ids."""
    sev, harness, model, om = setup
    B, k = 256, 64
    lens = [1 + (11 * b) % 70 for b in range(B)]
    nd = [k if b % 4 else 1 + (5 * b) % k for b in range(B)]
    announce(f"edges: B={B} x k<={k}, {sum(nd)} rows")
    reqs, batch, caches = _make(setup, lens, k, sum(nd))
    from tests.helpers import greedy_in_place
    gs = greedy_in_place(om, caches, 6)
    drafts = np.zeros((B, k), dtype=np.int32)
    for b in range(B):
        good = b % 7                                      # 0..6 tokens of the true continuation, then random ids
        row = np.array(reqs[b].random_tokens[:k], dtype=np.int64)
        row[:good] = gs[b][:good]
        if row[good] == gs[b][good]:
            row[good] = (row[good] + 1) % SHAPE.vocab
        drafts[b, :nd[b]] = row[:nd[b]]
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(drafts, device="cuda"), k, draft_lens=nd, want_path=True,
                        want_argmax=True, want_logits=True)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [drafts[b, :nd[b]] for b in range(B)])
    n_exact, worst, mean = _compare(out, res, B, k)
    acc = out["accept_len"].cpu().numpy()
    announce(f"  exact-compared {n_exact}/{B}, logits max {worst:.2e} mean {mean:.2e}, accept lengths 0..{int(acc.max())}")
    assert n_exact >= B // 3 and int(acc.max()) >= 4
    sev.kv_commit(batch.kv, None, B)
    for b in (0, 1, 37, 128, 255):
        assert batch.kv.get_state(b) == (lens[b] + int(acc[b]), int(out["bonus_token"][b]), 0)


def test_longest_chain_and_page_boundaries(setup):
    sev, harness, model, om = setup
    lens = [16, 17, 15, 32, 1]                            # on, after and before a page boundary; two full pages; one token
    k = 64                                                # SEV_MAX_DRAFT
    announce(f"edges: k={k} chains, lens {lens}")
    reqs, batch, caches = _make(setup, lens, k, 5 * k)
    gs = vo.greedy_continuation(om, caches, k)
    drafts = np.stack([gs[b][:k] for b in range(5)]).astype(np.int32)
    drafts[1, 40] = (drafts[1, 40] + 1) % SHAPE.vocab     # request 1 stops after 40 tokens
    drafts[3, 0] = (drafts[3, 0] + 1) % SHAPE.vocab       # request 3 accepts nothing
    for b in range(5):
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(drafts, device="cuda"), k, want_path=True, want_argmax=True,
                        want_logits=True)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [drafts[b] for b in range(5)])
    n_exact, worst, mean = _compare(out, res, 5, k)
    announce(f"  accept {[r.accept_len for r in res]}, exact-compared {n_exact}/5, logits max {worst:.2e} mean {mean:.2e}")
    assert int(out["accept_len"][3]) == 0 and int(out["bonus_token"][3]) == caches[3].next_tok
    sev.kv_commit(batch.kv, None, 5)
    for b in range(5):
        L, nt, flags = batch.kv.get_state(b)
        assert flags == 0 and L == lens[b] + int(out["accept_len"][b]) and nt == int(out["bonus_token"][b])


def test_rollback_then_verify_again(setup):
    sev, harness, model, om = setup
    lens = [40, 123]
    k = 8
    announce("edges: rollback, then the same block again")
    reqs, batch, caches = _make(setup, lens, k, 2 * k)
    gs = vo.greedy_continuation(om, caches, k)
    drafts = np.stack([corrupt_chain(gs[b], reqs[b], k) for b in range(2)]).astype(np.int32)
    drafts[0] = gs[0][:k]
    for b in range(2):
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    d = torch.tensor(drafts, device="cuda")
    out1 = sev.verify_ex(model, batch.kv, lens, d, k, want_path=True, want_argmax=True, want_logits=True)
    sev.kv_rollback(batch.kv, None, 2)
    torch.cuda.synchronize()
    for b in range(2):                                    # rollback leaves length and next token as they were
        assert batch.kv.get_state(b) == (lens[b], caches[b].next_tok, 0)
    # a different block in between must not leak into the repeat
    other = torch.tensor(((drafts + 5) % SHAPE.vocab).astype(np.int32), device="cuda")
    sev.verify_ex(model, batch.kv, lens, other, k)
    sev.kv_rollback(batch.kv, None, 2)
    out2 = sev.verify_ex(model, batch.kv, lens, d, k, want_path=True, want_argmax=True, want_logits=True)
    torch.cuda.synchronize()
    for key in ("accept_len", "bonus_token", "accept_path", "row_argmax", "logits"):
        assert torch.equal(out1[key], out2[key]), key     # same kernels, same order of operations: bit-identical
    res = vo.verify(om, caches, [drafts[0], drafts[1]])
    _compare(out2, res, 2, k)


def test_fork_with_several_roots(setup):
    sev, harness, model, om = setup
    lens = [70, 18]
    n = 6
    announce("edges: blocks with three roots")
    reqs, batch, caches = _make(setup, lens, n, 2 * n)
    gs = vo.greedy_continuation(om, caches, 3)
    # nodes 0, 1, 2 are children of the prefix; node 3 and 4 follow node 1; node 5 follows node 3
    parents = np.array([[-1, -1, -1, 1, 1, 3]] * 2, dtype=np.int32)
    toks = np.zeros((2, n), dtype=np.int32)
    for b in range(2):
        wrong = [(int(gs[b][0]) + 1 + i) % SHAPE.vocab for i in range(4)]
        toks[b] = [wrong[0], gs[b][0], wrong[1], gs[b][1], wrong[2], gs[b][2]]
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(toks, device="cuda"), n,
                        parents=torch.tensor(parents, device="cuda"), want_path=True, want_argmax=True, want_logits=True)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [toks[0], toks[1]], [parents[0], parents[1]])
    n_exact, worst, mean = _compare(out, res, 2, n)
    announce(f"  accept {[r.accept_len for r in res]} paths {[r.path for r in res]}, exact-compared {n_exact}/2")
    for b in range(2):
        if decision_gap_ok(res[b], GAP_MIN):
            assert res[b].path == [1, 3, 5] and out["accept_path"][b].cpu().tolist()[:3] == [1, 3, 5]
