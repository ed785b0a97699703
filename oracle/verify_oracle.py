"""CPU oracle for batched speculative verification.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition that the GPU library is checked
against.  Nothing in the product path may import it; it shares no code with
the HIP kernels.  Only tests, the smoke check and the CPU-baseline leg of the
benchmark call it.

What it defines (paper: section 4.1, the draft/verify cycle; section 4.3,
"Processing heterogeneous requests"; section 4.2, "Post-verification update"):

  * the server holds, per request, the target model's KV cache of the
    committed sequence;
  * an edge sends n candidate tokens (a chain, or a tree given by parent
    indices); the server scores all of them in ONE forward pass in which each
    candidate attends only to its own request's cache and to its own
    ancestors in the block (per-sequence masking, no cross-request
    interaction);
  * the server returns the accepted candidates plus one additional token that
    its own forward pass produced, and its cache is brought in line with the
    accepted tokens.

The acceptance rule is greedy exact match (the temperature -> 0 case of the
distribution-preserving rule the paper inherits from speculative decoding):
a candidate is accepted iff it equals the target model's arg-max prediction
for its position given its accepted ancestors.

Model: decoder-only pre-norm transformer, RMSNorm, rotary embedding on
half-split pairs, grouped-query attention, SwiGLU feed-forward, untied output
head, no biases.  All arithmetic is carried out in `model.dtype` (float64 by
default; float32 for the large shapes, where weights are bf16-valued and only
reassociation error is at stake).

Readings of points the paper leaves open (all conventions, parity unpinned
against any external implementation): RoPE pairs element i with i+hd/2 and uses
angle pos * base**(-2i/hd); RMSNorm epsilon sits inside the square root;
a model whose KV cache is bfloat16 (`kv_bf16`) rounds every key (after the
rotation) and value to nearest-even bfloat16 where it enters the cache, and the
block's own attention reads those stored values - the cache format is part of
the model, everything else stays in `model.dtype`;
arg-max ties go to the lowest token id; the first candidate of a block is
checked against `next_tok`, the target's own prediction after the committed
prefix, which the cache carries from the previous step; a tree node sits at
position P + depth(node).
"""
from dataclasses import dataclass, field
from typing import Callable, List, Optional, Sequence

import numpy as np


# ---------------------------------------------------------------------------
# model description
# ---------------------------------------------------------------------------


@dataclass
class Model:
    """Shape of the target model plus a callable that yields weight tensors.

    tensor(name, layer) returns a float array in canonical [out_features,
    in_features] layout for name in {embed, lm_head, wq, wk, wv, wo, wg, wu, wd}
    (layer is ignored for embed / lm_head).  gains(name, layer), if given, returns
    the RMSNorm gain vector [d_model] for name in {norm_attn, norm_ffn, norm_final}
    (layer ignored for norm_final); without it every gain is 1.
    """
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ffn: int
    vocab: int
    rope_base: float
    rms_eps: float
    tensor: Callable[[str, int], np.ndarray]
    dtype: type = np.float64
    cache_weights: bool = True
    kv_bf16: bool = False            # the KV cache stores bfloat16 (round-to-nearest-even on write)
    gains: Optional[Callable[[str, int], np.ndarray]] = None
    _memo: dict = field(default_factory=dict, repr=False)

    def w(self, name: str, layer: int = 0) -> np.ndarray:
        key = (name, layer)
        if key in self._memo:
            return self._memo[key]
        t = np.asarray(self.tensor(name, layer)).astype(self.dtype, copy=False)
        if self.cache_weights:
            self._memo[key] = t
        return t

    def g(self, name: str, layer: int = 0):
        """RMSNorm gain vector (1.0 when the model has unit gains)."""
        if self.gains is None:
            return 1.0
        return np.asarray(self.gains(name, layer)).astype(self.dtype, copy=False)


class Cache:
    """KV cache of ONE request: dense, contiguous, positions 0..length-1 valid."""

    def __init__(self, model: Model, capacity: int):
        shp = (capacity, model.n_kv_heads, model.head_dim)
        self.K = [np.zeros(shp, dtype=model.dtype) for _ in range(model.n_layers)]
        self.V = [np.zeros(shp, dtype=model.dtype) for _ in range(model.n_layers)]
        self.length = 0
        self.next_tok = -1            # target's arg-max prediction for position `length`
        self.pending = None           # draft block awaiting commit / rollback

    def copy(self) -> "Cache":
        c = Cache.__new__(Cache)
        c.K = [k.copy() for k in self.K]
        c.V = [v.copy() for v in self.V]
        c.length, c.next_tok, c.pending = self.length, self.next_tok, None
        return c


@dataclass
class Pending:
    new_k: List[np.ndarray]           # per layer [n, Hkv, hd], rotated keys of the block's nodes
    new_v: List[np.ndarray]
    path: List[int]                   # accepted node indices, root to leaf
    bonus: int


@dataclass
class VerifyResult:
    accept_len: int
    bonus_token: int
    path: List[int]                   # block-local indices of the accepted nodes, in order
    logits: np.ndarray                # [n, vocab] target logits at every node
    argmax: np.ndarray                # [n]
    top2_gap: np.ndarray              # [n] top-1 minus top-2 logit
    next_tok_in: int                  # the prediction the first candidate was checked against


# ---------------------------------------------------------------------------
# primitives
# ---------------------------------------------------------------------------


def rmsnorm(x: np.ndarray, gain, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * gain, row-wise."""
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * gain


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate x[n, H, hd] by position: pair (i, i+hd/2), angle pos * base**(-2i/hd)."""
    n, H, hd = x.shape
    half = hd // 2
    theta = np.float64(base) ** (-2.0 * np.arange(half, dtype=np.float64) / hd)
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]
    c = np.cos(ang).astype(x.dtype)[:, None, :]
    s = np.sin(ang).astype(x.dtype)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def softmax_rows(s: np.ndarray) -> np.ndarray:
    m = np.max(s, axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, mask: np.ndarray) -> np.ndarray:
    """softmax(q K^T / sqrt(hd) + mask) V with grouped-query head sharing.

    q [n, Hq, hd]; K, V [T, Hkv, hd]; mask [n, T] boolean (True = may attend).
    Query head j reads KV head floor(j * Hkv / Hq).
    """
    n, Hq, hd = q.shape
    Hkv = K.shape[1]
    out = np.empty_like(q)
    neg = np.array(-np.inf, dtype=q.dtype)
    for j in range(Hq):
        g = (j * Hkv) // Hq
        s = (q[:, j, :] @ K[:, g, :].T) / np.sqrt(np.array(hd, dtype=q.dtype))
        s = np.where(mask, s, neg)
        out[:, j, :] = softmax_rows(s) @ V[:, g, :]
    return out


def round_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned in x's dtype.

    bfloat16 keeps the sign, the 8-bit exponent and the top 7 fraction bits of a
    float32.  float64 input is rounded in ONE step to those 7 fraction bits (valid
    for magnitudes inside bfloat16's normal range, or exactly zero)."""
    if x.dtype == np.float64:
        a = np.abs(x)
        assert np.all((a == 0) | ((a > 1.2e-38) & (a < 3.3e38))), "outside bfloat16 normal range"
        u = np.ascontiguousarray(x).view(np.uint64)
        drop = np.uint64(45)                               # 52 fraction bits -> 7
        r = (u + np.uint64((1 << 44) - 1) + ((u >> drop) & np.uint64(1))) >> drop << drop
        return r.view(np.float64).reshape(x.shape)
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16) << np.uint32(16)
    return r.view(np.float32).reshape(x.shape).astype(x.dtype)


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def depths(parents: np.ndarray) -> np.ndarray:
    """Depth of every node (0 for children of the prefix); parents must precede children."""
    d = np.zeros(len(parents), dtype=np.int64)
    for i, p in enumerate(parents):
        if p >= 0:
            assert p < i, "parent index must be smaller than the child's"
            d[i] = d[p] + 1
    return d


def ancestor_mask(parents: np.ndarray) -> np.ndarray:
    """m[i, j] is True iff node j is node i or one of its ancestors."""
    n = len(parents)
    m = np.zeros((n, n), dtype=bool)
    for i in range(n):
        j = i
        while j >= 0:
            m[i, j] = True
            j = int(parents[j])
    return m


def chain_parents(n: int) -> np.ndarray:
    return np.arange(-1, n - 1, dtype=np.int64)


# ---------------------------------------------------------------------------
# forward pass over a batch of blocks
# ---------------------------------------------------------------------------


def forward_blocks(model: Model, caches: Sequence[Cache], tokens: Sequence[np.ndarray],
                   parents: Sequence[np.ndarray], want_logits: bool = True):
    """One target forward over a block of new tokens per request.

    Request r contributes tokens[r] (n_r ids) with tree structure parents[r];
    node i sits at position caches[r].length + depth(i) and attends to the whole
    cached prefix and to its ancestors-or-self in the block.  Rows of all
    requests are stacked for the position-wise operations (norm, projections,
    feed-forward); attention, the only operation that mixes rows, is done per
    request, so requests cannot influence each other.

    Returns (logits per request [n_r, vocab] or None, new_k, new_v) where
    new_k[r][l] / new_v[r][l] are the block's keys/values [n_r, Hkv, hd].
    Caches are not modified.
    """
    m = model
    R = len(caches)
    ns = [len(t) for t in tokens]
    offs = np.concatenate([[0], np.cumsum(ns)]).astype(np.int64)
    all_tok = np.concatenate([np.asarray(t, dtype=np.int64) for t in tokens])
    pos = np.concatenate([caches[r].length + depths(np.asarray(parents[r])) for r in range(R)])
    masks = []
    for r in range(R):
        P = caches[r].length
        masks.append(np.concatenate([np.ones((ns[r], P), dtype=bool), ancestor_mask(np.asarray(parents[r]))], axis=1))

    h = m.w("embed")[all_tok].astype(m.dtype)
    new_k = [[None] * m.n_layers for _ in range(R)]
    new_v = [[None] * m.n_layers for _ in range(R)]
    M = len(all_tok)
    for l in range(m.n_layers):
        x = rmsnorm(h, m.g("norm_attn", l), m.rms_eps)
        q = (x @ m.w("wq", l).T).reshape(M, m.n_q_heads, m.head_dim)
        k = (x @ m.w("wk", l).T).reshape(M, m.n_kv_heads, m.head_dim)
        v = (x @ m.w("wv", l).T).reshape(M, m.n_kv_heads, m.head_dim)
        q = rope(q, pos, m.rope_base)
        k = rope(k, pos, m.rope_base)
        if m.kv_bf16:
            k, v = round_bf16(k), round_bf16(v)
        o = np.empty_like(q)
        for r in range(R):
            a, b = offs[r], offs[r + 1]
            P = caches[r].length
            Kall = np.concatenate([caches[r].K[l][:P], k[a:b]], axis=0)
            Vall = np.concatenate([caches[r].V[l][:P], v[a:b]], axis=0)
            o[a:b] = attention(q[a:b], Kall, Vall, masks[r])
            new_k[r][l] = k[a:b].copy()
            new_v[r][l] = v[a:b].copy()
        h = h + o.reshape(M, -1) @ m.w("wo", l).T
        x = rmsnorm(h, m.g("norm_ffn", l), m.rms_eps)
        act = silu(x @ m.w("wg", l).T) * (x @ m.w("wu", l).T)
        h = h + act @ m.w("wd", l).T
    logits = None
    if want_logits:
        full = rmsnorm(h, m.g("norm_final"), m.rms_eps) @ m.w("lm_head").T
        logits = [full[offs[r]:offs[r + 1]] for r in range(R)]
    return logits, new_k, new_v


def _argmax_and_gap(logits: np.ndarray):
    am = np.argmax(logits, axis=-1)                    # first (lowest id) maximum
    top2 = np.partition(logits, -2, axis=-1)[:, -2:]
    return am, top2[:, 1] - top2[:, 0]


# ---------------------------------------------------------------------------
# cache filling
# ---------------------------------------------------------------------------


def extend(model: Model, caches: Sequence[Cache], tokens: Sequence[np.ndarray]):
    """Append known tokens to each cache (prefill, or teacher-forced decode).

    Runs the causal forward over the new tokens, stores their K/V at positions
    length.., and sets next_tok to the arg-max after the last appended token.
    Returns the logits per request.
    """
    pars = [chain_parents(len(t)) for t in tokens]
    logits, nk, nv = forward_blocks(model, caches, tokens, pars)
    for r, c in enumerate(caches):
        n = len(tokens[r])
        for l in range(model.n_layers):
            c.K[l][c.length:c.length + n] = nk[r][l]
            c.V[l][c.length:c.length + n] = nv[r][l]
        c.length += n
        c.next_tok = int(np.argmax(logits[r][-1]))
        c.pending = None
    return logits


def prefill(model: Model, prompt: np.ndarray, capacity: int) -> Cache:
    c = Cache(model, capacity)
    extend(model, [c], [np.asarray(prompt)])
    return c


def greedy_continuation(model: Model, caches: Sequence[Cache], k: int):
    """Plain autoregressive greedy decoding, one token per forward, from each cache.

    Returns g[r] = [g_0 .. g_k] with g_0 = next_tok and g_{i+1} the arg-max after
    feeding g_i (k single-token decodes).  Works on copies; caches are untouched.
    """
    cs = [c.copy() for c in caches]
    out = [[c.next_tok] for c in cs]
    for _ in range(k):
        extend(model, cs, [np.array([o[-1]]) for o in out])
        for r, c in enumerate(cs):
            out[r].append(c.next_tok)
    return [np.array(o, dtype=np.int64) for o in out]


# ---------------------------------------------------------------------------
# acceptance
# ---------------------------------------------------------------------------


def accept_chain(draft: np.ndarray, next_tok: int, argmax: np.ndarray):
    """Longest prefix of the chain that matches the target's predictions.

    y_0 = next_tok, y_{i+1} = argmax[i]; accept_len = max j with draft[i] == y_i
    for all i < j; bonus = y_{accept_len}.
    """
    a, want = 0, int(next_tok)
    while a < len(draft) and int(draft[a]) == want:
        want = int(argmax[a])
        a += 1
    return a, want, list(range(a))


def accept_tree(draft: np.ndarray, parents: np.ndarray, next_tok: int, argmax: np.ndarray):
    """Greedy descent: from the prefix, step to the child whose token equals the
    target's prediction (lowest node index if several), until no child matches.

    With distinct sibling tokens this is the longest root-to-leaf path all of
    whose tokens match the target arg-max.  Returns (accept_len, bonus, path).
    """
    cur, want, path = -1, int(next_tok), []
    while True:
        nxt = -1
        for c in range(len(draft)):
            if int(parents[c]) == cur and int(draft[c]) == want:
                nxt = c
                break
        if nxt < 0:
            break
        path.append(nxt)
        cur, want = nxt, int(argmax[nxt])
    return len(path), want, path


# ---------------------------------------------------------------------------
# verify / commit / rollback
# ---------------------------------------------------------------------------


def verify(model: Model, caches: Sequence[Cache], drafts: Sequence[np.ndarray],
           parents: Optional[Sequence[Optional[np.ndarray]]] = None) -> List[VerifyResult]:
    """Batched verification: one forward over every request's draft block, then
    greedy acceptance.  Leaves each cache PENDING (commit or rollback decides)."""
    R = len(caches)
    pars = []
    for r in range(R):
        p = None if parents is None else parents[r]
        pars.append(chain_parents(len(drafts[r])) if p is None else np.asarray(p, dtype=np.int64))
    logits, nk, nv = forward_blocks(model, caches, drafts, pars)
    res = []
    for r, c in enumerate(caches):
        am, gap = _argmax_and_gap(logits[r])
        if parents is None or parents[r] is None:
            a, bonus, path = accept_chain(np.asarray(drafts[r]), c.next_tok, am)
        else:
            a, bonus, path = accept_tree(np.asarray(drafts[r]), pars[r], c.next_tok, am)
        c.pending = Pending(nk[r], nv[r], path, bonus)
        res.append(VerifyResult(a, bonus, path, logits[r], am, gap, c.next_tok))
    return res


def commit(model: Model, cache: Cache) -> None:
    """Keep the accepted nodes' K/V at positions length..length+a-1, drop the rest."""
    p = cache.pending
    assert p is not None, "commit without a pending verify"
    for l in range(model.n_layers):
        for j, node in enumerate(p.path):
            cache.K[l][cache.length + j] = p.new_k[l][node]
            cache.V[l][cache.length + j] = p.new_v[l][node]
    cache.length += len(p.path)
    cache.next_tok = p.bonus
    cache.pending = None


def rollback(cache: Cache) -> None:
    """Discard the pending draft block; length and next_tok stay as they were."""
    cache.pending = None


# ---------------------------------------------------------------------------
# stochastic verification (chains): the distribution-preserving rule
# ---------------------------------------------------------------------------
# The paper states that the draft/verify cycle preserves the server model's output
# distribution exactly (section 4.1, citing speculative sampling) and runs every model at
# temperature 0.7 (section 5, setup).  The rule of that cited method, written out:
#   a candidate x drawn by the edge from its distribution q is accepted with probability
#   min(1, p(x)/q(x)), p being the server's distribution for that position; at the first
#   rejection the server emits a token drawn from the normalised residual max(0, p - q);
#   if every candidate is accepted it emits one more token drawn from p.
# Conventions of this build (readings; the paper does not spell them out): the first
# candidate of a block is the token the server itself emitted in the previous step
# (`next_tok`), which has no K/V yet; it is accepted iff it equals next_tok and no random
# number is spent on it.  Candidate i >= 1 is judged with the server distribution computed
# at candidate i-1.  All random numbers are inputs: u_acc[i] decides candidate i
# (accept iff u_acc[i] * q_i(x_i) < p_{i-1}(x_i)), u_emit picks the emitted token by inverse
# CDF in token-id order.


def softmax_t(logits: np.ndarray, temperature: float) -> np.ndarray:
    z = np.asarray(logits, dtype=np.float64) / float(temperature)
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def inverse_cdf(weights: np.ndarray, u: float):
    """Index i with cum[i-1] <= u * total < cum[i] (token-id order), and the distance of u * total to
    the nearest boundary of that cell, relative to the total (how firm the draw is)."""
    w = np.asarray(weights, dtype=np.float64)
    cum = np.cumsum(w)
    total = cum[-1]
    t = u * total
    i = int(np.searchsorted(cum, t, side="right"))
    i = min(i, len(w) - 1)
    while w[i] == 0.0 and i > 0:          # u * total == a boundary shared with empty cells
        i -= 1
    lo = cum[i] - w[i]
    margin = min(t - lo, cum[i] - t) / total if total > 0 else 0.0
    return i, float(margin)


@dataclass
class SampleResult:
    accept_len: int
    emitted: int               # the one additional token (resampled at a rejection, or drawn from p after full acceptance)
    accept_margin: float       # smallest |u*q - p| / max(p, u*q) over the decisions taken (how firm they were)
    emit_margin: float         # see inverse_cdf
    logits: np.ndarray


def accept_sample_chain(draft: np.ndarray, next_tok: int, p_rows: np.ndarray, q_rows: np.ndarray,
                        u_acc: np.ndarray, u_emit: float):
    """p_rows[i] = server distribution after candidate i; q_rows[i] = edge distribution candidate i was
    drawn from (q_rows[0] is unused: candidate 0 is the server's own previous token)."""
    n = len(draft)
    if int(draft[0]) != int(next_tok):
        # the edge is out of step with the server: nothing can be accepted; the server re-sends its token
        return 0, int(next_tok), 1.0, 1.0
    a, margin = 1, 1.0
    for i in range(1, n):
        x = int(draft[i])
        p, q = float(p_rows[i - 1][x]), float(q_rows[i][x])
        lhs = float(u_acc[i]) * q
        margin = min(margin, abs(lhs - p) / max(p, lhs, 1e-300))
        if lhs < p:
            a += 1
        else:
            res = np.maximum(p_rows[i - 1] - q_rows[i], 0.0)
            if res.sum() <= 0.0:           # p == q everywhere: a rejection has probability zero; fall back to p
                res = p_rows[i - 1]
            tok, em = inverse_cdf(res, u_emit)
            return a, tok, margin, em
    tok, em = inverse_cdf(p_rows[n - 1], u_emit)
    return a, tok, margin, em


def verify_sample(model: Model, caches: Sequence[Cache], drafts: Sequence[np.ndarray], q_rows: Sequence[np.ndarray],
                  u_acc: Sequence[np.ndarray], u_emit: Sequence[float], temperature: float) -> List[SampleResult]:
    """Batched stochastic verification of chains: one forward over every request's block, then the
    accept / resample rule above.  Leaves each cache PENDING with the accepted prefix and the emitted
    token as its next token."""
    R = len(caches)
    pars = [chain_parents(len(d)) for d in drafts]
    logits, nk, nv = forward_blocks(model, caches, drafts, pars)
    res = []
    for r, c in enumerate(caches):
        p_rows = np.stack([softmax_t(row, temperature) for row in logits[r]])
        a, tok, m1, m2 = accept_sample_chain(np.asarray(drafts[r]), c.next_tok, p_rows, np.asarray(q_rows[r], dtype=np.float64),
                                             np.asarray(u_acc[r]), float(u_emit[r]))
        c.pending = Pending(nk[r], nv[r], list(range(a)), tok)
        res.append(SampleResult(a, tok, m1, m2, logits[r]))
    return res


# Trees under the stochastic rule (multi-step speculative sampling, the tree generalisation used by the
# tree-based methods the paper builds on, section 2): at the current node the children are tried in
# index order; child c with token x, drawn by the edge from q_c, is accepted with probability
# min(1, p(x)/q_c(x)), p being the CURRENT server distribution at that node; a rejection replaces p by
# the normalised residual max(0, p - q_c) before the next sibling is tried; when a child is accepted
# the walk moves there and p becomes the server distribution computed at that child; when no child is
# left the emitted token is drawn from the current p.  The rule preserves the server distribution when
# the siblings of a node are independent draws from the same q.  Readings as for chains: the block's
# root is the token the server emitted in the previous step (a node with parent -1 whose token equals
# next_tok, lowest index first; without one nothing is accepted).


def accept_sample_tree(draft: np.ndarray, parents: np.ndarray, next_tok: int, p_rows: np.ndarray, q_rows: np.ndarray,
                       u_acc: np.ndarray, u_emit: float):
    n = len(draft)
    roots = [c for c in range(n) if parents[c] == -1 and int(draft[c]) == int(next_tok)]
    if not roots:
        return 0, int(next_tok), [], 1.0, 1.0
    cur = roots[0]
    path, margin = [cur], 1.0
    p = np.asarray(p_rows[cur], dtype=np.float64)
    while True:
        moved = False
        for c in range(cur + 1, n):
            if parents[c] != cur:
                continue
            x = int(draft[c])
            px, qx = float(p[x]), float(q_rows[c][x])
            lhs = float(u_acc[c]) * qx
            margin = min(margin, abs(lhs - px) / max(px, lhs, 1e-300))
            if lhs < px:
                cur = c
                path.append(c)
                p = np.asarray(p_rows[c], dtype=np.float64)
                moved = True
                break
            res = np.maximum(p - q_rows[c], 0.0)
            if res.sum() > 0.0:
                p = res / res.sum()
        if not moved:
            tok, em = inverse_cdf(p, u_emit)
            return len(path), tok, path, margin, em


def verify_sample_tree(model: Model, caches: Sequence[Cache], drafts: Sequence[np.ndarray], parents: Sequence[np.ndarray],
                       q_rows: Sequence[np.ndarray], u_acc: Sequence[np.ndarray], u_emit: Sequence[float], temperature: float):
    """Batched stochastic verification of trees; returns (SampleResult, path) per request and leaves the
    caches PENDING with the accepted path."""
    pars = [np.asarray(p, dtype=np.int64) for p in parents]
    logits, nk, nv = forward_blocks(model, caches, drafts, pars)
    out = []
    for r, c in enumerate(caches):
        p_rows = np.stack([softmax_t(row, temperature) for row in logits[r]])
        a, tok, path, m1, m2 = accept_sample_tree(np.asarray(drafts[r]), pars[r], c.next_tok, p_rows,
                                                  np.asarray(q_rows[r], dtype=np.float64), np.asarray(u_acc[r]), float(u_emit[r]))
        c.pending = Pending(nk[r], nv[r], path, tok)
        out.append((SampleResult(a, tok, m1, m2, logits[r]), path))
    return out
