"""ctypes binding of include/sev.h.  Argument marshalling only."""
import ctypes as C
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
SEV_F32, SEV_BF16 = 0, 1
W_KINDS = {"embed": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "wg": 5, "wu": 6, "wd": 7, "lm_head": 8,
           "norm_attn": 9, "norm_ffn": 10, "norm_final": 11}


class SevError(RuntimeError):
    pass


class ModelDesc(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
                ("head_dim", C.c_int32), ("d_ffn", C.c_int32), ("vocab", C.c_int32), ("rope_base", C.c_float),
                ("rms_eps", C.c_float), ("dtype", C.c_int32)]


class VerifyArgs(C.Structure):
    _fields_ = [("B", C.c_int32), ("k_max", C.c_int32), ("slots", C.c_void_p), ("prefix_lens", C.c_void_p),
                ("draft_lens", C.c_void_p), ("draft_tokens", C.c_void_p), ("parents", C.c_void_p), ("mode", C.c_int32),
                ("accept_len", C.c_void_p), ("bonus_token", C.c_void_p), ("accept_path", C.c_void_p),
                ("row_argmax", C.c_void_p), ("logits", C.c_void_p)]


class SampleArgs(C.Structure):
    _fields_ = [("B", C.c_int32), ("k_max", C.c_int32), ("slots", C.c_void_p), ("prefix_lens", C.c_void_p),
                ("draft_lens", C.c_void_p), ("draft_tokens", C.c_void_p), ("parents", C.c_void_p), ("draft_probs", C.c_void_p),
                ("u_accept", C.c_void_p), ("u_emit", C.c_void_p), ("temperature", C.c_float),
                ("logits_ws", C.c_void_p), ("accept_len", C.c_void_p), ("emitted_token", C.c_void_p), ("accept_path", C.c_void_p)]


class SchedDesc(C.Structure):
    _fields_ = [("max_batch", C.c_int32), ("max_rows", C.c_int32), ("min_batch", C.c_int32), ("max_wait_us", C.c_int64)]


def lib_path() -> str:
    return os.path.join(_HERE, "libsev.so")


_lib = None


def lib():
    """Loads libsev.so (building it first only if it has never been built)."""
    global _lib
    if _lib is not None:
        return _lib
    path = lib_path()
    if not os.path.exists(path):
        from . import build as _build
        _build.build()
    L = C.CDLL(path)
    vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
    sig = {
        "sev_model_arena_bytes": (sz, [C.POINTER(ModelDesc)]),
        "sev_model_create": (i32, [C.POINTER(ModelDesc), vp, sz, C.POINTER(vp)]),
        "sev_model_destroy": (i32, [vp]),
        "sev_model_load_tensor": (i32, [vp, i32, i32, vp, vp]),
        "sev_kv_pool_bytes": (sz, [vp, i64, i32]),
        "sev_kv_create": (i32, [vp, i32, i32, i64, i32, vp, sz, C.POINTER(vp)]),
        "sev_kv_destroy": (i32, [vp]),
        "sev_kv_set_pages": (i32, [vp, i32, vp, i32, vp]),
        "sev_kv_set_state": (i32, [vp, vp, vp, vp, i32, vp]),
        "sev_kv_copy_tokens": (i32, [vp, i32, i32, i32, i32, vp, vp, i32, vp]),
        "sev_kv_get_state": (i32, [vp, i32, C.POINTER(C.c_int32), C.POINTER(C.c_int32), C.POINTER(C.c_uint32), vp]),
        "sev_verify": (i32, [vp, vp, vp, vp, vp, i32, i32, vp, vp, vp]),
        "sev_verify_ex": (i32, [vp, vp, C.POINTER(VerifyArgs), vp]),
        "sev_verify_sample": (i32, [vp, vp, C.POINTER(SampleArgs), vp]),
        "sev_verify_sample_static": (i32, [vp, vp, C.POINTER(SampleArgs), vp]),
        "sev_prefill": (i32, [vp, vp, vp, vp, vp, vp, i32, i32, vp]),
        "sev_kv_commit": (i32, [vp, vp, i32, vp]),
        "sev_kv_rollback": (i32, [vp, vp, i32, vp]),
        "sev_last_error": (C.c_char_p, []),
        "sev_profile_enable": (i32, [vp, C.c_uint]),
        "sev_profile_read": (i32, [vp, i32, C.POINTER(C.c_double), C.POINTER(C.c_int64)]),
        "sev_profile_name": (C.c_char_p, [i32]),
        "sev_sched_create": (i32, [C.POINTER(SchedDesc), C.POINTER(vp)]),
        "sev_sched_destroy": (i32, [vp]),
        "sev_sched_submit": (i32, [vp, i32, i32, i64]),
        "sev_sched_next_batch": (i32, [vp, i64, vp, vp, C.POINTER(C.c_int32), C.POINTER(C.c_int64)]),
        "sev_sched_pending": (i32, [vp]),
        "sev_sched_record_verify": (i32, [vp, i64]),
        "sev_sched_verify_estimate": (i64, [vp]),
        "sev_sched_calibrate_depth": (i32, [i64, i64, i64, i32, i32]),
        "sev_edge_align": (i32, [vp, vp, i32, vp, i32, i32, vp, vp, C.POINTER(C.c_int32)]),
    }
    for name, (res, args) in sig.items():
        f = getattr(L, name)
        f.restype, f.argtypes = res, args
    _lib = L
    return L


def _check(rc: int, what: str):
    if rc != 0:
        raise SevError(f"{what} failed ({rc}): {lib().sev_last_error().decode()}")


def _stream_ptr():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _host_i32(x):
    """A C-contiguous int32 host array (kept alive by the caller for the duration of the call)."""
    if x is None:
        return None
    return np.ascontiguousarray(np.asarray(x, dtype=np.int32))


def _hp(a):
    return None if a is None else C.c_void_p(a.ctypes.data)


def _dp(t):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


class Model:
    """sev_model over a torch-allocated weight arena."""

    def __init__(self, n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps, dtype,
                 device="cuda:0"):
        if not torch.cuda.is_available():
            raise SevError("no GPU: the sev library has no CPU path")
        self.desc = ModelDesc(n_layers, d_model, n_q_heads, n_kv_heads, head_dim, d_ffn, vocab, rope_base, rms_eps, dtype)
        self.device = torch.device(device)
        nbytes = lib().sev_model_arena_bytes(C.byref(self.desc))
        if nbytes == 0:
            raise SevError("unsupported model description: " + lib().sev_last_error().decode())
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        h = C.c_void_p()
        _check(lib().sev_model_create(C.byref(self.desc), _dp(self.arena), nbytes, C.byref(h)), "sev_model_create")
        self.handle = h
        self.torch_dtype = torch.float32 if dtype == SEV_F32 else torch.bfloat16

    def load_tensor(self, kind, layer, src: torch.Tensor):
        k = W_KINDS[kind] if isinstance(kind, str) else kind
        _check(lib().sev_model_load_tensor(self.handle, k, layer, _dp(src), _stream_ptr()), "sev_model_load_tensor")

    def close(self):
        if self.handle:
            lib().sev_model_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class KVCache:
    """sev_kv over a torch-allocated page pool."""

    def __init__(self, model: Model, max_requests: int, max_rows: int, n_pages: int, page_size: int = 16):
        self.model = model
        nbytes = lib().sev_kv_pool_bytes(model.handle, n_pages, page_size)
        if nbytes == 0:
            raise SevError("bad pool geometry")
        self.pool = torch.zeros(nbytes, dtype=torch.uint8, device=model.device)
        h = C.c_void_p()
        _check(lib().sev_kv_create(model.handle, max_requests, max_rows, n_pages, page_size, _dp(self.pool), nbytes,
                                   C.byref(h)), "sev_kv_create")
        self.handle = h
        self.n_pages, self.page_size = n_pages, page_size

    def set_pages(self, slot: int, page_ids):
        a = _host_i32(page_ids)
        _check(lib().sev_kv_set_pages(self.handle, slot, _hp(a), len(a), _stream_ptr()), "sev_kv_set_pages")

    def set_state(self, slot, seq_len, next_tok):
        """Scalars (one slot) or equal-length sequences (several slots; slot may be None for 0..B-1)."""
        if np.isscalar(seq_len):
            slot, seq_len, next_tok = [slot], [seq_len], [next_tok]
        sl, ln, nt = _host_i32(slot), _host_i32(seq_len), _host_i32(next_tok)
        _check(lib().sev_kv_set_state(self.handle, _hp(sl), _hp(ln), _hp(nt), len(ln), _stream_ptr()), "sev_kv_set_state")

    def get_state(self, slot: int):
        a, b, f = C.c_int32(), C.c_int32(), C.c_uint32()
        _check(lib().sev_kv_get_state(self.handle, slot, C.byref(a), C.byref(b), C.byref(f), _stream_ptr()),
               "sev_kv_get_state")
        return a.value, b.value, f.value

    def copy_tokens(self, slot, layer, start, n_tokens, k: torch.Tensor, v: torch.Tensor, to_cache: bool):
        _check(lib().sev_kv_copy_tokens(self.handle, slot, layer, start, n_tokens, _dp(k), _dp(v), int(to_cache),
                                        _stream_ptr()), "sev_kv_copy_tokens")

    def profile_enable(self, class_mask: int):
        _check(lib().sev_profile_enable(self.handle, int(class_mask)), "sev_profile_enable")

    def profile_classes(self):
        out, i = [], 0
        while lib().sev_profile_name(i) is not None:
            out.append(lib().sev_profile_name(i).decode())
            i += 1
        return out

    def profile_read(self):
        out, i = {}, 0
        while True:
            nm = lib().sev_profile_name(i)
            if nm is None:
                break
            ms, n = C.c_double(), C.c_int64()
            _check(lib().sev_profile_read(self.handle, i, C.byref(ms), C.byref(n)), "sev_profile_read")
            out[nm.decode()] = (ms.value, n.value)
            i += 1
        return out

    def close(self):
        if self.handle:
            lib().sev_kv_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def verify(model: Model, kv: KVCache, prefix_lens, draft_tokens: torch.Tensor, draft_mask, B: int, k: int,
           accept_len: torch.Tensor = None, bonus_token: torch.Tensor = None):
    """sev_verify: returns (accept_len, bonus_token) device int32 tensors (valid after a stream sync)."""
    pl = _host_i32(prefix_lens)
    if accept_len is None:
        accept_len = torch.empty(B, dtype=torch.int32, device=model.device)
    if bonus_token is None:
        bonus_token = torch.empty(B, dtype=torch.int32, device=model.device)
    _check(lib().sev_verify(model.handle, kv.handle, _hp(pl), _dp(draft_tokens), _dp(draft_mask), B, k,
                            _dp(accept_len), _dp(bonus_token), _stream_ptr()), "sev_verify")
    return accept_len, bonus_token


def verify_ex(model: Model, kv: KVCache, prefix_lens, draft_tokens: torch.Tensor, k_max: int, slots=None,
              draft_lens=None, parents: torch.Tensor = None, mode: int = 0, want_path=False, want_argmax=False,
              want_logits=False, accept_len: torch.Tensor = None, bonus_token: torch.Tensor = None):
    """sev_verify_ex: returns a dict of device tensors (accept_len, bonus_token and the requested extras)."""
    pl, sl, dl = _host_i32(prefix_lens), _host_i32(slots), _host_i32(draft_lens)
    B = len(pl)
    rows = int(dl.sum()) if dl is not None else B * k_max
    dev = model.device
    out = {"accept_len": accept_len if accept_len is not None else torch.empty(B, dtype=torch.int32, device=dev),
           "bonus_token": bonus_token if bonus_token is not None else torch.empty(B, dtype=torch.int32, device=dev)}
    if want_path:
        out["accept_path"] = torch.empty(B, k_max, dtype=torch.int32, device=dev)
    if want_argmax:
        out["row_argmax"] = torch.empty(rows, dtype=torch.int32, device=dev)
    if want_logits:
        out["logits"] = torch.empty(rows, model.desc.vocab, dtype=torch.float32, device=dev)
    a = VerifyArgs(B, k_max, _hp(sl), _hp(pl), _hp(dl), _dp(draft_tokens), _dp(parents), mode,
                   _dp(out["accept_len"]), _dp(out["bonus_token"]), _dp(out.get("accept_path")),
                   _dp(out.get("row_argmax")), _dp(out.get("logits")))
    _check(lib().sev_verify_ex(model.handle, kv.handle, C.byref(a), _stream_ptr()), "sev_verify_ex")
    return out


def verify_sample(model: Model, kv: KVCache, prefix_lens, draft_tokens: torch.Tensor, k_max: int, draft_probs: torch.Tensor,
                  u_accept: torch.Tensor, u_emit: torch.Tensor, temperature: float, slots=None, draft_lens=None,
                  parents: torch.Tensor = None, out: dict = None):
    """sev_verify_sample: returns a dict of device tensors (accept_len, emitted_token, accept_path, logits); a dict
    returned by an earlier call of the same shape can be passed back as `out` to reuse its tensors."""
    pl, sl, dl = _host_i32(prefix_lens), _host_i32(slots), _host_i32(draft_lens)
    B = len(pl)
    rows = int(dl.sum()) if dl is not None else B * k_max
    dev = model.device
    out = out if out is not None else {
           "accept_len": torch.empty(B, dtype=torch.int32, device=dev),
           "emitted_token": torch.empty(B, dtype=torch.int32, device=dev),
           "accept_path": torch.empty(B, k_max, dtype=torch.int32, device=dev),
           "logits": torch.empty(rows, model.desc.vocab, dtype=torch.float32, device=dev)}
    assert draft_probs.dtype == torch.float32 and tuple(draft_probs.shape) == (rows, model.desc.vocab) and draft_probs.is_contiguous()
    assert u_accept.dtype == torch.float32 and tuple(u_accept.shape) == (B, k_max) and u_emit.dtype == torch.float32
    a = SampleArgs(B, k_max, _hp(sl), _hp(pl), _hp(dl), _dp(draft_tokens), _dp(parents), _dp(draft_probs), _dp(u_accept), _dp(u_emit),
                   float(temperature), _dp(out["logits"]), _dp(out["accept_len"]), _dp(out["emitted_token"]),
                   _dp(out["accept_path"]))
    _check(lib().sev_verify_sample(model.handle, kv.handle, C.byref(a), _stream_ptr()), "sev_verify_sample")
    return out


def verify_sample_static(model: Model, kv: KVCache, prefix_lens, draft_tokens: torch.Tensor, k_max: int, draft_probs: torch.Tensor,
                         u_accept: torch.Tensor, u_emit: torch.Tensor, temperature: float, out: dict, slots=None, draft_lens=None,
                         parents: torch.Tensor = None):
    """sev_verify_sample_static: as verify_sample, with the logits in the library's static scratch.  `out` holds the
    caller's output tensors (accept_len, emitted_token, accept_path): this call allocates nothing on the device."""
    pl, sl, dl = _host_i32(prefix_lens), _host_i32(slots), _host_i32(draft_lens)
    a = SampleArgs(len(pl), k_max, _hp(sl), _hp(pl), _hp(dl), _dp(draft_tokens), _dp(parents), _dp(draft_probs), _dp(u_accept), _dp(u_emit),
                   float(temperature), None, _dp(out["accept_len"]), _dp(out["emitted_token"]), _dp(out["accept_path"]))
    _check(lib().sev_verify_sample_static(model.handle, kv.handle, C.byref(a), _stream_ptr()), "sev_verify_sample_static")
    return out


def prefill(model: Model, kv: KVCache, start_lens, n_tokens, tokens: torch.Tensor, slots=None):
    """sev_prefill: appends n_tokens[b] tokens (device int32 [B][t_max]) to each slot under a causal mask."""
    st, nt, sl = _host_i32(start_lens), _host_i32(n_tokens), _host_i32(slots)
    B, t_max = int(tokens.shape[0]), int(tokens.shape[1])
    _check(lib().sev_prefill(model.handle, kv.handle, _hp(sl), _hp(st), _hp(nt), _dp(tokens), B, t_max, _stream_ptr()),
           "sev_prefill")


def kv_commit(kv: KVCache, slots, B: int):
    sl = _host_i32(slots)
    _check(lib().sev_kv_commit(kv.handle, _hp(sl), B, _stream_ptr()), "sev_kv_commit")


def kv_rollback(kv: KVCache, slots, B: int):
    sl = _host_i32(slots)
    _check(lib().sev_kv_rollback(kv.handle, _hp(sl), B, _stream_ptr()), "sev_kv_rollback")


class Scheduler:
    """Handle of the server-side batch former (sev_sched_*): host code, needs no GPU."""

    def __init__(self, max_batch: int, max_rows: int, min_batch: int = 1, max_wait_us: int = 0):
        self.desc = SchedDesc(max_batch, max_rows, min_batch, max_wait_us)
        self.h = C.c_void_p()
        _check(lib().sev_sched_create(C.byref(self.desc), C.byref(self.h)), "sev_sched_create")
        self._req = np.zeros(max(max_batch, 1), dtype=np.int32)
        self._rows = np.zeros(max(max_batch, 1), dtype=np.int32)

    def submit(self, request: int, n_draft: int, arrival_us: int):
        _check(lib().sev_sched_submit(self.h, request, n_draft, arrival_us), "sev_sched_submit")

    def next_batch(self, now_us: int):
        """Returns ([(request, n_draft)], wake_us)."""
        n, wake = C.c_int32(0), C.c_int64(0)
        _check(lib().sev_sched_next_batch(self.h, now_us, _hp(self._req), _hp(self._rows), C.byref(n), C.byref(wake)), "sev_sched_next_batch")
        return [(int(self._req[i]), int(self._rows[i])) for i in range(n.value)], wake.value

    def pending(self) -> int:
        return lib().sev_sched_pending(self.h)

    def record_verify(self, duration_us: int):
        _check(lib().sev_sched_record_verify(self.h, duration_us), "sev_sched_record_verify")

    def verify_estimate(self) -> int:
        return lib().sev_sched_verify_estimate(self.h)

    def close(self):
        if self.h:
            lib().sev_sched_destroy(self.h)
            self.h = C.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def calibrate_depth(t_verify_us: int, t_draft_fwd_us: int, rtt_us: int, min_depth: int = 1, max_depth: int = 64) -> int:
    d = lib().sev_sched_calibrate_depth(t_verify_us, t_draft_fwd_us, rtt_us, min_depth, max_depth)
    if d < 0:
        _check(d, "sev_sched_calibrate_depth")
    return d


def edge_align(parents, tokens, accept_path, bonus_token: int):
    """sev_edge_align: returns (kept node indices, their parents as indices into kept); both empty without alignment."""
    par, tok, path = _host_i32(parents), _host_i32(tokens), _host_i32(accept_path)
    n = len(par)
    kept, newp, nk = np.zeros(max(n, 1), dtype=np.int32), np.zeros(max(n, 1), dtype=np.int32), C.c_int32(0)
    _check(lib().sev_edge_align(_hp(par), _hp(tok), n, _hp(path), len(path), int(bonus_token), _hp(kept), _hp(newp), C.byref(nk)),
           "sev_edge_align")
    return kept[:nk.value].tolist(), newp[:nk.value].tolist()
