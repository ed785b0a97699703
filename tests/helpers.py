"""Glue used by the tests: wraps the seeded weight source as an oracle model and
builds draft blocks from the oracle's own greedy continuation."""
import numpy as np

import synth
from oracle import verify_oracle as vo


def oracle_model(shape: synth.ModelShape, seed: int, dtype=np.float64, cache_weights=True) -> vo.Model:
    src = synth.WeightSource(shape, seed)
    return vo.Model(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.head_dim,
                    shape.d_ffn, shape.vocab, shape.rope_base, shape.rms_eps,
                    tensor=src.tensor_f32, dtype=dtype, cache_weights=cache_weights,
                    kv_bf16=(shape.dtype == "bf16"))


def corrupt_chain(greedy: np.ndarray, req: synth.workload.Request, n: int) -> np.ndarray:
    """Draft = greedy continuation with position j replaced by a random id iff its draw < p."""
    d = np.array(greedy[:n], dtype=np.int64)
    for j in range(n):
        if req.corrupt_draw[j] < req.corrupt_p:
            d[j] = req.random_tokens[j]
    return d


def decision_gap_ok(res, gap_min: float) -> bool:
    """True iff every arg-max the oracle's acceptance walk relied on (the nodes of its accepted path;
    the last of them also produced the stop decision and the bonus token) has a top-1/top-2 logit gap
    of at least gap_min.  Only such requests are compared bit-exactly."""
    return all(res.top2_gap[i] >= gap_min for i in res.path)


def announce(msg: str):
    print(f"[case] {msg}", flush=True)
