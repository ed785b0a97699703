"""Workload plumbing for tests, the smoke check and the benchmark: uploads seeded weights and
cache contents from `synth` into the library's handles.  No arithmetic of the method happens
here; every model step runs inside libsev."""
import numpy as np
import torch

import synth
from . import binding as sev


def _to_device(arr: np.ndarray, device) -> torch.Tensor:
    if arr.dtype == np.uint16:                       # bf16 bit patterns
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def build_model(shape: synth.ModelShape, seed: int, device="cuda:0", progress=None, gains=False) -> sev.Model:
    """Creates a model and loads every matrix from the seeded weight source, one tensor at a time
    (host generation -> staging tensor -> sev_model_load_tensor), so peak staging is one tensor.
    gains=True also loads the source's seeded non-unit norm gains (the default gains are 1)."""
    dt = sev.SEV_F32 if shape.dtype == "f32" else sev.SEV_BF16
    m = sev.Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim, shape.d_ffn,
                  shape.vocab, shape.rope_base, shape.rms_eps, dt, device)
    src = synth.WeightSource(shape, seed)
    for name in ("embed", "lm_head"):
        m.load_tensor(name, 0, _to_device(src.tensor(name), m.device))
    for l in range(shape.n_layers):
        for name in ("wq", "wk", "wv", "wo", "wg", "wu", "wd"):
            m.load_tensor(name, l, _to_device(src.tensor(name, l), m.device))
        if gains:
            for name in ("norm_attn", "norm_ffn"):
                m.load_tensor(name, l, _to_device(src.gain(name, l), m.device))
        if progress:
            progress(l)
    if gains:
        m.load_tensor("norm_final", 0, _to_device(src.gain("norm_final"), m.device))
    torch.cuda.synchronize()
    return m


class Batch:
    """A set of request slots with pages assigned, ready for verify calls."""

    def __init__(self, model: sev.Model, shape: synth.ModelShape, capacities, max_rows: int, seed: int = 0,
                 spare_pages: int = 0):
        self.model, self.shape = model, shape
        self.B = len(capacities)
        lists, n_pages = synth.page_lists(seed, capacities, 16, spare_pages)
        self.kv = sev.KVCache(model, self.B, max_rows, max(n_pages, 1))
        self.page_lists = lists
        for b, pl in enumerate(lists):
            self.kv.set_pages(b, pl)
        self.lens = [0] * self.B

    def import_kv(self, slot: int, layer: int, start: int, K: np.ndarray, V: np.ndarray):
        """Writes plain [n][Hkv][hd] arrays (model dtype; uint16 = bf16 bits) into the paged cache."""
        k, v = _to_device(np.ascontiguousarray(K), self.model.device), _to_device(np.ascontiguousarray(V), self.model.device)
        self.kv.copy_tokens(slot, layer, start, K.shape[0], k, v, True)

    def export_kv(self, slot: int, layer: int, start: int, n: int):
        s = self.shape
        k = torch.empty(n, s.n_kv_heads, s.head_dim, dtype=self.model.torch_dtype, device=self.model.device)
        v = torch.empty_like(k)
        self.kv.copy_tokens(slot, layer, start, n, k, v, False)
        torch.cuda.synchronize()
        return k.float().cpu().numpy(), v.float().cpu().numpy()

    def append(self, token_lists, slots=None):
        """Teacher-forced append (cache fill): runs the forward over the given tokens of each listed
        slot in blocks of at most 64, keeps all of them, and leaves next_tok = arg-max after the last."""
        slots = list(range(self.B)) if slots is None else list(slots)
        todo = [np.asarray(t, dtype=np.int32) for t in token_lists]
        at = [0] * len(slots)
        while any(at[i] < len(todo[i]) for i in range(len(slots))):
            act = [i for i in range(len(slots)) if at[i] < len(todo[i])]
            ns = [min(64, len(todo[i]) - at[i]) for i in act]
            kmax = max(ns)
            toks = np.zeros((len(act), kmax), dtype=np.int32)
            for r, i in enumerate(act):
                toks[r, :ns[r]] = todo[i][at[i]:at[i] + ns[r]]
            sl = [slots[i] for i in act]
            sev.verify_ex(self.model, self.kv, [self.lens[s] for s in sl], torch.from_numpy(toks).to(self.model.device),
                          kmax, slots=sl, draft_lens=ns, mode=1)
            sev.kv_commit(self.kv, sl, len(sl))
            for r, i in enumerate(act):
                at[i] += ns[r]
                self.lens[slots[i]] += ns[r]
        torch.cuda.synchronize()

    def prefill(self, token_lists, slots=None):
        """sev_prefill over whole token lists (any length the slots' pages can hold)."""
        slots = list(range(self.B)) if slots is None else list(slots)
        ns = [len(t) for t in token_lists]
        toks = np.zeros((len(slots), max(ns)), dtype=np.int32)
        for r, t in enumerate(token_lists):
            toks[r, :ns[r]] = np.asarray(t, dtype=np.int32)
        sev.prefill(self.model, self.kv, [self.lens[s] for s in slots], ns, torch.from_numpy(toks).to(self.model.device),
                    slots=slots)
        for r, s_ in enumerate(slots):
            self.lens[s_] += ns[r]
        torch.cuda.synchronize()

    def fill_synthetic(self, seed: int, prefix_lens, last_tokens):
        """Drawn K/V for positions 0..P-2 of every slot, then a real forward over the last prefix
        token so that position P-1 and next_tok come from the model."""
        for b, P in enumerate(prefix_lens):
            if P > 1:
                for l in range(self.shape.n_layers):
                    K, V = synth.synthetic_kv(self.shape, seed, b, l, P - 1)
                    self.import_kv(b, l, 0, K, V)
            self.kv.set_state(b, P - 1, -1)
            self.lens[b] = P - 1
        torch.cuda.synchronize()
        self.append([[int(t)] for t in last_tokens])
