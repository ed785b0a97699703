"""GPU test of the pipeline replay: the C++ batch former drives real sev_verify_ex + sev_kv_commit calls
on the small bf16 model while edges and network run on a simulated clock (the verification time the
clock sees is a fixed model, so the schedule is deterministic and must equal the oracle simulation's;
the acceptances come from the GPU and are fed to the oracle simulation in the same order)."""
import numpy as np
import pytest
import torch

import synth
from oracle import sched_oracle as so
from tests.helpers import announce

pytestmark = pytest.mark.gpu


def test_pipeline_replay_on_gpu():
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness
    from paper_2505_17052_amd.pipeline import replay
    shape, seed = synth.MINI_BF16, 606
    B, k, E, n_batches = 3, 4, 6, 12
    model = harness.build_model(shape, seed)
    lens = [20 + 7 * e for e in range(E)]
    batch = harness.Batch(model, shape, [P + n_batches * (k + 1) + 16 for P in lens], max_rows=B * k, seed=seed)
    batch.fill_synthetic(seed, lens, [int(synth.uniform_i32(seed, 7000 + e, 1, 0, shape.vocab)[0]) for e in range(E)])
    cur = list(lens)
    rng = np.random.default_rng(seed)
    emitted_log = []

    def verify(rs):
        toks = rng.integers(0, shape.vocab, size=(len(rs), k)).astype(np.int32)
        for i, r in enumerate(rs):
            toks[i, 0] = batch.kv.get_state(r)[1]                     # the server's own next token: always accepted
        out = sev.verify_ex(model, batch.kv, [cur[r] for r in rs], torch.tensor(toks, device="cuda"), k, slots=rs)
        sev.kv_commit(batch.kv, rs, len(rs))
        a = out["accept_len"].cpu().numpy()
        assert (a >= 1).all()
        for i, r in enumerate(rs):
            cur[r] += int(a[i])
        em = [int(x) + 1 for x in a]
        emitted_log.append(em)
        return 4000 + 100 * len(rs), em

    announce(f"pipeline replay: {E} edges, batches of {B}, {n_batches} verifications")
    got = replay([k] * E, [3000] * E, 1000, sev.Scheduler(B, B * k), verify, n_batches)
    it = iter(emitted_log)
    want = so.simulate([k] * E, [3000] * E, 1000, so.Former(B, B * k), lambda rs: (4000 + 100 * len(rs), next(it)), n_batches)
    assert got == want
    for e in range(E):                                                # the caches advanced by exactly the accepted tokens
        L, _, flags = batch.kv.get_state(e)
        assert flags == 0 and L == cur[e] and L - lens[e] == got["tokens"][e] - sum(1 for _, b in got["log"] if e in b)
    announce(f"  server busy {got['busy_us'] / got['end_us']:.2f} of the time, {sum(got['tokens'])} tokens emitted")
