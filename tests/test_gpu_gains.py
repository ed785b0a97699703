"""GPU parity with non-unit RMSNorm gains, float32 and bfloat16 paths.

The workloads use unit gains, so a gain that is loaded but not applied, applied at the wrong norm
or taken from the wrong layer would pass every other test.  Here every norm of every layer gets its
own seeded gain vector in [0.5, 1.5), loaded through sev_model_load_tensor (kinds NORM_ATTN,
NORM_FFN, NORM_FINAL) and handed to the oracle through its gain callback; the results are compared
at the tolerances of the respective path.  The oracle's own use of the gains is pinned on the CPU
against torch's rms_norm routine (tests/test_oracle_pins.py)."""
import numpy as np
import pytest
import torch

import synth
from oracle import verify_oracle as vo
from tests.helpers import oracle_model, announce, decision_gap_ok

pytestmark = pytest.mark.gpu


def _run(shape, seed, lens, k, dtype, tol, gap_min):
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    model = harness.build_model(shape, seed, gains=True)
    om = oracle_model(shape, seed, dtype=dtype, gains=True)
    om_unit = oracle_model(shape, seed, dtype=dtype)
    B = len(lens)
    prompts = [synth.rng.uniform_i32(seed, 300 + b, P, 0, shape.vocab) for b, P in enumerate(lens)]
    batch = harness.Batch(model, shape, [P + 48 for P in lens], max_rows=256, seed=seed)
    batch.append(prompts)                                    # real cache fill on the GPU: the gains act on every layer's K/V
    caches = [vo.prefill(om, p, len(p) + 48) for p in prompts]
    g = vo.greedy_continuation(om, caches, k)
    drafts = np.stack([x[:k] for x in g]).astype(np.int32)
    drafts[B - 1, k // 2] = (drafts[B - 1, k // 2] + 1) % shape.vocab
    batch.kv.set_state(None, lens, [c.next_tok for c in caches])
    out = sev.verify_ex(model, batch.kv, lens, torch.tensor(drafts, device="cuda"), k, want_path=True, want_argmax=True,
                        want_logits=True)
    torch.cuda.synchronize()
    assert batch.kv.get_state(0)[2] == 0
    res = vo.verify(om, caches, [drafts[b] for b in range(B)])
    lg = out["logits"].cpu().numpy().reshape(B, k, -1)
    am = out["row_argmax"].cpu().numpy().reshape(B, k)
    n_exact, n_firm, worst, mean = 0, 0, 0.0, 0.0
    for b in range(B):
        d = np.abs(lg[b] - res[b].logits)
        worst, mean = max(worst, float(d.max())), max(mean, float(d.mean()))
        firm = res[b].top2_gap >= gap_min
        n_firm += int(firm.sum())
        assert np.array_equal(am[b][firm], res[b].argmax[firm]), f"request {b}: arg-max differs at a firm position"
        if decision_gap_ok(res[b], gap_min):
            n_exact += 1
            assert int(out["accept_len"][b]) == res[b].accept_len and int(out["bonus_token"][b]) == res[b].bonus_token, b
    # the gains matter: the same model with unit gains gives clearly different logits
    unit = vo.forward_blocks(om_unit, [vo.prefill(om_unit, prompts[0], lens[0] + 48)], [drafts[0]], [vo.chain_parents(k)])[0][0]
    sep = float(np.abs(unit - res[0].logits).mean())
    announce(f"  {shape.name} with seeded gains: logits max-abs {worst:.2e} mean-abs {mean:.2e} (unit-gain model differs by {sep:.2e}); "
             f"arg-max compared at {n_firm}/{B * k} firm positions, accept/bonus exactly for {n_exact}/{B} requests")
    assert worst < tol[0] and mean < tol[1], (worst, mean)
    assert sep > 20 * tol[1]
    assert n_firm >= B * k // 4


def test_gains_tiny_f32():
    announce("norm gains, tiny f32")
    _run(synth.TINY, 77, [33, 9, 64], 4, np.float64, (1e-4, 1e-5), 1e-3)


def test_gains_mini_bf16():
    announce("norm gains, mini bf16")
    _run(synth.MINI_BF16, 78, [70, 17, 130], 6, np.float32, (3e-2, 3e-3), 0.05)
