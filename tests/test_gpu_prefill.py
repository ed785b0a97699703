"""GPU parity of sev_prefill (the step before verification): long token blocks appended under a
causal mask, in chunks, against the oracle's plain prefill.  float32 tiny model: K/V within float32
reassociation error; bf16 small GQA model: K/V within one bf16 rounding step plus the propagated
rounding noise, then a verify on top of the prefilled cache is compared as in the other bf16 tests."""
import numpy as np
import pytest
import torch

import synth
from oracle import verify_oracle as vo
from tests.helpers import oracle_model, corrupt_chain, announce

pytestmark = pytest.mark.gpu

GAP_MIN = 0.05


def _tokens(seed, b, n, vocab):
    from synth.workload import P_PREFIX_TOK
    return synth.uniform_i32(seed, synth.stream_id(P_PREFIX_TOK, 900 + b), n, 0, vocab)


def test_prefill_f32_matches_oracle_and_blockwise_append():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    shape, seed = synth.TINY, 17
    model = harness.build_model(shape, seed)
    om = oracle_model(shape, seed, dtype=np.float64)
    lens = [150, 1, 97]                                   # several chunks, one token, a ragged tail
    prompts = [_tokens(seed, b, n, shape.vocab) for b, n in enumerate(lens)]
    announce(f"prefill f32: lens {lens}, row budget 64 (chunks of 21)")
    batch = harness.Batch(model, shape, [n + 32 for n in lens], max_rows=64, seed=seed)
    batch.prefill(prompts)
    caches = [vo.prefill(om, p, len(p) + 32) for p in prompts]
    for b, n in enumerate(lens):
        L, nt, flags = batch.kv.get_state(b)
        assert (L, flags) == (n, 0)
        for l in range(shape.n_layers):
            k, v = batch.export_kv(b, l, 0, n)
            assert np.max(np.abs(k - caches[b].K[l][:n])) < 5e-5
            assert np.max(np.abs(v - caches[b].V[l][:n])) < 5e-5
        lg = vo.forward_blocks(om, [vo.Cache(om, n)], [prompts[b]], [vo.chain_parents(n)])[0][0]
        t2 = np.sort(lg[-1])[-2:]
        if t2[1] - t2[0] >= 1e-3:
            assert nt == caches[b].next_tok
    # the same prompts appended 64 tokens at a time through sev_verify_ex (mode 1) give the same cache bit for bit
    batch2 = harness.Batch(model, shape, [n + 32 for n in lens], max_rows=64 * 3, seed=seed)
    batch2.append(prompts)
    for b, n in enumerate(lens):
        assert batch2.kv.get_state(b)[:1] == (n,)
        for l in range(shape.n_layers):
            k1, v1 = batch.export_kv(b, l, 0, n)
            k2, v2 = batch2.export_kv(b, l, 0, n)
            # same arithmetic per row; only the float32 attention order over chunk boundaries is shared too
            assert np.max(np.abs(k1 - k2)) < 2e-6 and np.max(np.abs(v1 - v2)) < 2e-6


def test_prefill_bf16_then_verify():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    from tests.test_gpu_bf16_mini import _compare

    def assert_cache_close(got, ref, what):
        """Stored bf16 K/V after a real prefill.  Rounding K/V to bf16 makes the comparison chaotic in the
        small: a float32-level difference flips the rounding of a few per cent of the entries by one step
        (0.4 % of the entry), and those flips feed the next layer's attention, so by layer 2 the values before
        rounding differ by about 1e-4 of the row scale.  Hence: one bf16 step of the entry plus 1e-3 of the
        tensor's rms (entries far smaller than the row scale carry the absolute error), and at most 12 % of
        the entries differing at all.  The bar that matters, the logits of a verify on top of this cache, is
        checked below with the logit tolerances of the bfloat16 path."""
        err = np.abs(got - ref)
        tol = np.abs(ref) * 2.0 ** -7 + 1e-3 * float(np.sqrt(np.mean(ref * ref)))
        bad = int(np.sum(err > tol))
        assert bad == 0, f"{what}: {bad} entries off, worst {float(err.max()):.3e}"
        assert np.mean(got != ref) < 0.12, f"{what}: {np.mean(got != ref):.4f} of entries differ"
    shape, seed = synth.MINI_BF16, 606
    model = harness.build_model(shape, seed)
    om = oracle_model(shape, seed, dtype=np.float32)
    lens = [333, 70, 1]                                   # more than 64 tokens per request and block, chunked by the row budget
    prompts = [_tokens(seed, b, n, shape.vocab) for b, n in enumerate(lens)]
    announce(f"prefill bf16: lens {lens}, row budget 256")
    batch = harness.Batch(model, shape, [n + 80 for n in lens], max_rows=256, seed=seed)
    batch.prefill(prompts)
    caches = [vo.prefill(om, p, len(p) + 80) for p in prompts]
    for b, n in enumerate(lens):
        L, nt, flags = batch.kv.get_state(b)
        assert (L, flags) == (n, 0)
        for l in range(shape.n_layers):
            k, v = batch.export_kv(b, l, 0, n)
            assert_cache_close(k, caches[b].K[l][:n], f"K slot {b} layer {l}")
            assert_cache_close(v, caches[b].V[l][:n], f"V slot {b} layer {l}")
    # verification on top of the prefilled caches
    k = 8
    reqs = synth.make_requests(synth.Workload("mini", shape, 3, k, "chain", 1, 333, "fixed", (k,), 0.3, 0.3, "synthetic", seed))
    gs = vo.greedy_continuation(om, caches, k)
    drafts = np.stack([corrupt_chain(gs[b], reqs[b], k) for b in range(3)]).astype(np.int32)
    drafts[0] = gs[0][:k]
    for b in range(3):
        batch.kv.set_state(b, lens[b], caches[b].next_tok)
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(drafts, device="cuda"), k, want_path=True, want_argmax=True,
                        want_logits=True)
    torch.cuda.synchronize()
    res = vo.verify(om, caches, [drafts[b] for b in range(3)])
    n_exact, worst, mean = _compare(out, res, 3, k)
    announce(f"  verify after prefill: exact-compared {n_exact}/3, logits max {worst:.2e} mean {mean:.2e}")


def test_prefill_error_paths():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    shape, seed = synth.TINY, 17
    model = harness.build_model(shape, seed)
    batch = harness.Batch(model, shape, [40], max_rows=16, seed=seed)
    toks = torch.zeros((1, 64), dtype=torch.int32, device="cuda")
    with pytest.raises(sev.SevError):                     # more tokens than the slot's pages hold
        sev.prefill(model, batch.kv, [0], [64], toks)
    with pytest.raises(sev.SevError):                     # empty block
        sev.prefill(model, batch.kv, [0], [0], toks)
    sev.prefill(model, batch.kv, [5], [4], toks)          # wrong start length: flagged on the device, not a crash
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] & 1
