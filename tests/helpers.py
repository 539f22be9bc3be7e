"""Glue used by the tests only: turns generated torch weights into the oracle's fp64 numpy dicts."""
import numpy as np
import torch

from oracle import prism_oracle as O
from paper_2510_15620_amd import workloads as W


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to("cpu").to(torch.float64).numpy()


def oracle_weights(wt: W.Weights, layers=None) -> dict:
    return {
        "embed": to_f64(wt.embed), "final_norm": to_f64(wt.final_norm),
        "w_yes": to_f64(wt.w_yes), "w_no": to_f64(wt.w_no),
        "layers": [None if (l is None or (layers is not None and i not in layers))
                   else {k: to_f64(v) for k, v in l.items()} for i, l in enumerate(wt.layers)],
    }


def oracle_model(m: W.ModelShape, operand: str = None) -> O.Model:
    """operand: precision of the contraction operands, "exact" unless a test asks for a rounded one."""
    operand = operand or "exact"
    return O.Model(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab,
                   m.rms_eps, m.rope_base, m.qk_norm, operand)


def oracle_select(w: W.Workload, wt=None, tokens=None, **over):
    wt = wt if wt is not None else W.make_weights(w)
    q, cands = tokens if tokens is not None else W.make_tokens(w)
    kw = dict(checkpoints=w.checkpoints, n_clusters=w.n_clusters, tau=w.cv_threshold, mode=O.MODE_DROP_ONLY)
    kw.update(over)
    K = kw.pop("K", w.K)
    operand = kw.pop("operand", None)
    return O.select(q, cands, K, oracle_weights(wt), oracle_model(w.model, operand), **kw)
