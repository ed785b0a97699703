"""sev_verify_sample_static (the entry point that allocates nothing: logits in the library's static device scratch)
against sev_verify_sample (caller-provided logits workspace) through the C ABI: same inputs, same integers out, same
cache state after commit — on two calls in a row, the second with a smaller input, so that the second call finds the
first call's contents in the scratch.  Runs alone in a fresh process and after the other GPU tests."""
import ctypes as C

import numpy as np
import pytest
import torch

import synth
from tests.helpers import announce

pytestmark = pytest.mark.gpu

T = 0.7


def _inputs(sev, model, batch, lens, nts, k, gen):
    """Candidate blocks with plausible edge distributions: a first pass gives the server's logits for random blocks;
    the edge distributions are perturbed copies of them and the candidates are drawn from those."""
    B, V = len(lens), model.desc.vocab
    d0 = torch.randint(0, V, (B, k), device="cuda", generator=gen, dtype=torch.int32)
    d0[:, 0] = torch.tensor(nts, device="cuda", dtype=torch.int32)
    q0 = torch.softmax(torch.randn(B * k, V, device="cuda", generator=gen), dim=-1).contiguous()
    u_acc = torch.rand(B, k, device="cuda", generator=gen)
    u_emit = torch.rand(B, device="cuda", generator=gen)
    batch.kv.set_state(None, lens, nts)
    lg = sev.verify_sample(model, batch.kv, lens, d0, k, q0, u_acc, u_emit, T)["logits"].view(B, k, V)
    q = torch.softmax((lg + 0.7 * torch.randn(B, k, V, device="cuda", generator=gen)) / T, dim=-1)
    q = torch.cat([q0.view(B, k, V)[:, :1], q[:, :-1]], dim=1).contiguous()        # row i: the distribution candidate i was drawn from
    d = d0.clone()
    d[:, 1:] = torch.multinomial(q[:, 1:].reshape(-1, V), 1, generator=gen).view(B, k - 1).to(torch.int32)
    d[B - 1, 0] = (d[B - 1, 0] + 1) % V                                            # one request out of step
    torch.cuda.synchronize()
    return d.contiguous(), q.view(B * k, V).contiguous(), u_acc, u_emit


def _pair(sev, model, batch, lens, nts, k, gen, what):
    B = len(lens)
    d, q, u_acc, u_emit = _inputs(sev, model, batch, lens, nts, k, gen)
    batch.kv.set_state(None, lens, nts)
    ref = sev.verify_sample(model, batch.kv, lens, d, k, q, u_acc, u_emit, T)
    sev.kv_commit(batch.kv, None, B)
    torch.cuda.synchronize()
    st_ref = [batch.kv.get_state(b) for b in range(B)]
    out = {"accept_len": torch.full((B,), -9, dtype=torch.int32, device="cuda"),
           "emitted_token": torch.full((B,), -9, dtype=torch.int32, device="cuda"),
           "accept_path": torch.full((B, k), -9, dtype=torch.int32, device="cuda")}
    batch.kv.set_state(None, lens, nts)
    torch.cuda.synchronize()
    mem0 = torch.cuda.memory_allocated()
    sev.verify_sample_static(model, batch.kv, lens, d, k, q, u_acc, u_emit, T, out)
    sev.kv_commit(batch.kv, None, B)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == mem0
    st = [batch.kv.get_state(b) for b in range(B)]
    announce(f"  {what}: accept {ref['accept_len'].tolist()} emitted {ref['emitted_token'].tolist()}")
    for key in ("accept_len", "emitted_token", "accept_path"):
        assert torch.equal(out[key], ref[key]), (what, key, out[key].tolist(), ref[key].tolist())
    assert st == st_ref and all(s[2] == 0 for s in st), (what, st, st_ref)
    assert int(ref["accept_len"].max()) >= 1 and int(ref["accept_len"][B - 1]) == 0


@pytest.mark.parametrize("shape", [synth.TINY, synth.MINI_BF16], ids=["tiny-f32", "mini-bf16"])
def test_static_scratch_entry_point_matches_workspace_entry_point(shape):
    import paper_2505_17052_amd as sev
    from paper_2505_17052_amd import harness, binding
    seed = 515
    announce(f"allocation-free entry point, {shape.name}")
    model = harness.build_model(shape, seed)
    lens = [40, 300, 17, 64, 129, 5]
    batch = harness.Batch(model, shape, [P + 80 for P in lens], max_rows=len(lens) * 8, seed=seed)
    last = [int(synth.uniform_i32(seed, 8000 + b, 1, 0, shape.vocab)[0]) for b in range(len(lens))]
    batch.fill_synthetic(seed, lens, last)
    nts = [batch.kv.get_state(b)[1] for b in range(len(lens))]
    gen = torch.Generator(device="cuda").manual_seed(seed)
    _pair(sev, model, batch, lens, nts, 8, gen, "first call, 6 requests x 8 candidates")
    _pair(sev, model, batch, lens[:3], nts[:3], 5, gen, "second call, 3 requests x 5 candidates")
    # limits and misuse are refused on the host, before anything is launched
    L = binding.lib()
    B, k = 63, 64                                                                   # 4032 rows of logits: beyond the scratch for this vocabulary?
    need = B * k * shape.vocab * 4
    pl = np.zeros(B, dtype=np.int32)
    a = binding.SampleArgs(B, k, None, C.c_void_p(pl.ctypes.data), None, None, None, None, None, None, T, None, None, None, None)
    rc = L.sev_verify_sample_static(model.handle, batch.kv.handle, C.byref(a), None)
    assert rc == (-3 if need > (64 << 20) else -1), (rc, L.sev_last_error())
    ws = torch.empty(16, device="cuda")
    a = binding.SampleArgs(1, 1, None, C.c_void_p(pl.ctypes.data), None, None, None, None, None, None, T, C.c_void_p(ws.data_ptr()), None, None, None)
    assert L.sev_verify_sample_static(model.handle, batch.kv.handle, C.byref(a), None) == -1 and b"logits_ws must be NULL" in L.sev_last_error()
