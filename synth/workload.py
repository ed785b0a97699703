"""Shape tables and seeded request generators for the verification workloads.

Nothing here evaluates the model: the functions only draw lengths, token ids,
cache contents, page placements and draft-tree topologies from the
counter-based generator, so the CPU oracle and the GPU library can be fed the
same inputs.
"""
from dataclasses import dataclass, replace
from typing import Optional, Tuple

import numpy as np

from . import rng

# ---------------------------------------------------------------------------
# model shapes
# ---------------------------------------------------------------------------


@dataclass(frozen=True)
class ModelShape:
    name: str
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    dtype: str            # "f32" or "bf16": storage type of weights and KV cache
    rms_eps: float = 1e-5
    init_std: float = 0.02

    def with_layers(self, n: int) -> "ModelShape":
        return replace(self, n_layers=n, name=f"{self.name}-L{n}")

    @property
    def q_dim(self) -> int:
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self) -> int:
        return self.n_kv_heads * self.head_dim

    def streamed_params(self) -> int:
        """Weight elements one forward pass must read (the embedding table is gathered, not streamed)."""
        per_layer = self.d_model * (self.q_dim + 2 * self.kv_dim) + self.q_dim * self.d_model \
            + 3 * self.d_model * self.d_ffn
        return self.n_layers * per_layer + self.d_model * self.vocab

    def kv_bytes_per_token(self) -> int:
        esz = 4 if self.dtype == "f32" else 2
        return 2 * self.kv_dim * esz * self.n_layers


TINY = ModelShape("tiny", 2, 256, 4, 4, 64, 688, 1024, 10000.0, "f32")
LLAMA8B = ModelShape("llama3-8b-shape", 32, 4096, 32, 8, 128, 14336, 128256, 500000.0, "bf16")
LLAMA70B = ModelShape("llama3-70b-shape", 80, 8192, 64, 8, 128, 28672, 128256, 500000.0, "bf16")
# A small bf16 model with the same head geometry as the large shapes (GQA 4:1,
# head_dim 128) whose forward the CPU oracle finishes in well under a second.
MINI_BF16 = ModelShape("mini-bf16", 3, 512, 8, 2, 128, 1408, 4224, 500000.0, "bf16")

# weight tensor kinds; canonical layout is [out_features, in_features], row-major
_KINDS = {"embed": 0, "wq": 1, "wk": 2, "wv": 3, "wo": 4, "wg": 5, "wu": 6, "wd": 7, "lm_head": 8}

# stream purposes (upper bits of the stream id keep them disjoint from weights)
P_WEIGHT, P_LEN, P_PREFIX_TOK, P_KV, P_CORRUPT, P_RAND_TOK, P_TREE, P_PAGES, P_KDRAW, P_PDRAW = range(10)


def stream_id(purpose: int, a: int = 0, b: int = 0, c: int = 0) -> int:
    """Pack (purpose, a, b, c) into one 64-bit stream number."""
    assert 0 <= purpose < 256 and 0 <= a < (1 << 24) and 0 <= b < (1 << 16) and 0 <= c < (1 << 8)
    return (purpose << 48) | (a << 24) | (b << 8) | c


class WeightSource:
    """Random-init weights N(0, init_std) regenerated on demand from (seed, tensor, layer).

    For "bf16" shapes the values are bfloat16 (round-to-nearest-even of the normal
    draw) and are returned as uint16 bit patterns; for "f32" shapes as float32.
    The workloads use unit norm gains and no biases; `gain` draws non-unit gains for
    the tests that check that the gains are applied.
    """

    def __init__(self, shape: ModelShape, seed: int):
        self.shape = shape
        self.seed = seed

    def dims(self, name: str) -> Tuple[int, int]:
        s = self.shape
        return {
            "embed": (s.vocab, s.d_model), "lm_head": (s.vocab, s.d_model),
            "wq": (s.q_dim, s.d_model), "wk": (s.kv_dim, s.d_model), "wv": (s.kv_dim, s.d_model),
            "wo": (s.d_model, s.q_dim), "wg": (s.d_ffn, s.d_model), "wu": (s.d_ffn, s.d_model),
            "wd": (s.d_model, s.d_ffn),
        }[name]

    def tensor(self, name: str, layer: int = 0, out: Optional[np.ndarray] = None) -> np.ndarray:
        rows, cols = self.dims(name)
        st = stream_id(P_WEIGHT, layer, _KINDS[name])
        n = rows * cols
        if self.shape.dtype == "bf16":
            flat = rng.normal_bf16(self.seed, st, n, self.shape.init_std,
                                   out=None if out is None else out.reshape(-1))
        else:
            flat = rng.normal_f32(self.seed, st, n, self.shape.init_std,
                                  out=None if out is None else out.reshape(-1))
        return flat.reshape(rows, cols)

    def gain(self, name: str, layer: int = 0) -> np.ndarray:
        """Seeded RMSNorm gain vector [d_model], float32, uniform in [0.5, 1.5);
        name in {norm_attn, norm_ffn, norm_final} (layer ignored for norm_final)."""
        kind = {"norm_attn": 9, "norm_ffn": 10, "norm_final": 11}[name]
        st = stream_id(P_WEIGHT, 0 if name == "norm_final" else layer, kind)
        return (0.5 + rng.uniform_f64(self.seed, st, self.shape.d_model)).astype(np.float32)

    def tensor_f32(self, name: str, layer: int = 0) -> np.ndarray:
        """The tensor's values as float32 (bf16 shapes are widened exactly)."""
        t = self.tensor(name, layer)
        return rng.bf16_bits_to_f32(t) if t.dtype == np.uint16 else t


# ---------------------------------------------------------------------------
# workloads
# ---------------------------------------------------------------------------


@dataclass(frozen=True)
class Workload:
    name: str
    shape: ModelShape
    B: int
    k_max: int                       # draft nodes per request (upper bound when ragged)
    draft: str                       # "chain" or "tree"
    prefix_lo: int
    prefix_hi: int                   # inclusive
    prefix_dist: str                 # "fixed", "uniform" or "loguniform"
    k_choices: Tuple[int, ...]       # per-request draft length is drawn from these
    corrupt_lo: float
    corrupt_hi: float
    cache_fill: str                  # "prefill": run the model over prefix tokens; "synthetic": drawn K/V
    seed: int
    page_size: int = 16
    tree_depth: int = 8

    def scaled(self, **kw) -> "Workload":
        return replace(self, **kw)


WORKLOADS = {
    # 1: tiny fp32 model, true prefill of 64 random ids, k=4 chain
    "tiny-chain": Workload("tiny-chain", TINY, 1, 4, "chain", 64, 64, "fixed", (4,), 0.3, 0.3, "prefill", 1001),
    # 2: headline: 8B shape, B=16, k=8 chains, prefix U[256,2048], paged KV
    "8b-chain-b16k8": Workload("8b-chain-b16k8", LLAMA8B, 16, 8, "chain", 256, 2048, "uniform", (8,), 0.3, 0.3,
                               "synthetic", 2002),
    # 3: 8B shape, B=8 trees of 64 nodes, depth 8, prefix U[512,4096]
    "8b-tree-b8n64": Workload("8b-tree-b8n64", LLAMA8B, 8, 64, "tree", 512, 4096, "uniform", (64,), 0.3, 0.3,
                              "synthetic", 3003),
    # 4: 8B shape, B=64 ragged chains k in {2,4,8}, prefix log-uniform [128,8192], p ~ U[0.1,0.5]
    "8b-ragged-b64": Workload("8b-ragged-b64", LLAMA8B, 64, 8, "chain", 128, 8192, "loguniform", (2, 4, 8), 0.1, 0.5,
                              "synthetic", 4004),
    # 5: 70B shape, B=32, k=8 chains, prefix U[1024,4096]
    "70b-chain-b32k8": Workload("70b-chain-b32k8", LLAMA70B, 32, 8, "chain", 1024, 4096, "uniform", (8,), 0.3, 0.3,
                                "synthetic", 5005),
}


@dataclass
class Request:
    index: int
    prefix_len: int                  # P: committed positions 0..P-1 before the verify
    n_draft: int                     # number of draft nodes in this request's block
    corrupt_p: float
    prefix_tokens: np.ndarray        # int32[P]; for "synthetic" fill only the last id is ever fed to the model
    corrupt_draw: np.ndarray         # float64[k_max] uniform: position j is corrupted iff draw < corrupt_p
    random_tokens: np.ndarray        # int32[k_max] replacement ids (also sibling filler for trees)


def make_requests(wl: Workload):
    """Draw every per-request quantity of a workload from its seed."""
    B, V = wl.B, wl.shape.vocab
    u = rng.uniform_f64(wl.seed, stream_id(P_LEN), B)
    if wl.prefix_dist == "fixed":
        lens = np.full(B, wl.prefix_lo, dtype=np.int64)
    elif wl.prefix_dist == "uniform":
        lens = wl.prefix_lo + np.floor(u * (wl.prefix_hi - wl.prefix_lo + 1)).astype(np.int64)
    elif wl.prefix_dist == "loguniform":
        lens = np.floor(np.exp(np.log(wl.prefix_lo) + u * (np.log(wl.prefix_hi + 1) - np.log(wl.prefix_lo)))).astype(np.int64)
    else:
        raise ValueError(wl.prefix_dist)
    lens = np.clip(lens, wl.prefix_lo, wl.prefix_hi)
    kd = rng.uniform_i32(wl.seed, stream_id(P_KDRAW), B, 0, len(wl.k_choices))
    pd = rng.uniform_f64(wl.seed, stream_id(P_PDRAW), B)
    reqs = []
    for b in range(B):
        P = int(lens[b])
        reqs.append(Request(
            index=b, prefix_len=P, n_draft=int(wl.k_choices[kd[b]]),
            corrupt_p=float(wl.corrupt_lo + pd[b] * (wl.corrupt_hi - wl.corrupt_lo)),
            prefix_tokens=rng.uniform_i32(wl.seed, stream_id(P_PREFIX_TOK, b), P, 0, V),
            corrupt_draw=rng.uniform_f64(wl.seed, stream_id(P_CORRUPT, b), wl.k_max),
            random_tokens=rng.uniform_i32(wl.seed, stream_id(P_RAND_TOK, b), 4 * wl.k_max, 0, V),
        ))
    return reqs


def synthetic_kv(shape: ModelShape, seed: int, request: int, layer: int, n_tokens: int):
    """Drawn cache contents for positions 0..n_tokens-1 of one request and layer.

    Returns (K, V), each [n_tokens, n_kv_heads, head_dim]; entries are
    N(0, (init_std*sqrt(d_model))^2), the scale a projection of a unit-RMS
    vector through N(0, init_std) weights has.  bf16 shapes get bf16 values
    (uint16 bit patterns), f32 shapes float32.
    """
    n = n_tokens * shape.kv_dim
    scale = shape.init_std * np.sqrt(shape.d_model)
    out = []
    for which in (0, 1):
        st = stream_id(P_KV, request, layer, which)
        flat = rng.normal_bf16(seed, st, n, scale) if shape.dtype == "bf16" else rng.normal_f32(seed, st, n, scale)
        out.append(flat.reshape(n_tokens, shape.n_kv_heads, shape.head_dim))
    return out[0], out[1]


def page_lists(seed: int, tokens_needed, page_size: int = 16, spare_pages: int = 0):
    """Shuffled, non-contiguous physical page ids for each request.

    tokens_needed[b] is the capacity request b must hold.  Returns (lists, n_pages).
    """
    counts = [(int(t) + page_size - 1) // page_size for t in tokens_needed]
    total = sum(counts) + spare_pages
    keys = rng.uniform_f64(seed, stream_id(P_PAGES), total)
    perm = np.argsort(keys, kind="stable").astype(np.int32)
    lists, at = [], 0
    for c in counts:
        lists.append(perm[at:at + c].copy())
        at += c
    return lists, total


def tree_parents(seed: int, request: int, n_nodes: int = 64, depth: int = 8) -> np.ndarray:
    """Topology of one draft tree as a parent-index array (−1 = child of the committed prefix).

    A spine of `depth` nodes guarantees the stated depth; then nodes are visited in
    creation order and each draws a branching factor from {1,2,3,4} and receives
    children until it has that many (nodes on the last level get none), until
    n_nodes exist.  Nodes are finally relabelled in breadth-first order, so every
    parent index is smaller than its child's.
    """
    assert n_nodes >= depth
    draws = rng.uniform_i32(seed, stream_id(P_TREE, request), 4 * n_nodes, 1, 5)
    parent = [-1] + list(range(depth - 1))          # the spine: node i has parent i-1
    level = list(range(depth))
    n_child = [1] * (depth - 1) + [0]
    visit = 0
    while len(parent) < n_nodes and visit < len(parent):
        want = int(draws[visit])
        while n_child[visit] < want and level[visit] < depth - 1 and len(parent) < n_nodes:
            parent.append(visit)
            level.append(level[visit] + 1)
            n_child.append(0)
            n_child[visit] += 1
        visit += 1
    # if the draw sequence ran dry before n_nodes (every open node saturated), hang the rest under the root level
    while len(parent) < n_nodes:
        parent.append(-1)
        level.append(0)
        n_child.append(0)
    order = sorted(range(n_nodes), key=lambda i: (level[i], i))      # breadth-first relabelling
    new_of = {old: new for new, old in enumerate(order)}
    out = np.empty(n_nodes, dtype=np.int32)
    for old in range(n_nodes):
        out[new_of[old]] = -1 if parent[old] < 0 else new_of[parent[old]]
    return out
