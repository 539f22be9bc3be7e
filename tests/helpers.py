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


# --------------------------------------------------------------------------- full-size goldens and the margin rule

import json
import os
from types import SimpleNamespace

GOLDEN_DIR = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def golden_path(workload: str, mode: str) -> str:
    return os.path.join(GOLDEN_DIR, f"fullsize_{workload}_{mode}.json")


def load_fullsize_golden(workload: str, mode: str):
    """A complete oracle run written by tests/golden/make_fullsize_goldens.py: events (layer, live, scores, fate, keep)
    and the returned top-K."""
    d = json.load(open(golden_path(workload, mode)))
    ev = [SimpleNamespace(layer=e["layer"], live=np.array(e["live"], np.int64), scores=np.array([float(s) for s in e["scores"]]),
                          gate=e["gate"], pruned=e["pruned"],
                          fate=None if e["fate"] is None else np.array(e["fate"], np.int8),
                          keep=None if e["keep"] is None else np.array(e["keep"], bool)) for e in d["events"]]
    return SimpleNamespace(events=ev, idx=np.array(d["idx"], np.int64), scores=np.array([float(s) for s in d["scores"]]),
                           layers_run=d["layers_run"], token_layers=d["token_layers"], K=d["K"], n_cands=d["n_cands"],
                           n_clusters=d["n_clusters"], tau=d["tau"], checkpoints=d["checkpoints"])


def _partition_costs_k3(ranked: np.ndarray):
    """Within-cluster sum of squares of every partition of the ranked scores into three runs: C[s1, s2], inf where
    s1 >= s2.  Direct prefix-sum evaluation (the margins below need the runner-up, which the oracle does not keep)."""
    n = len(ranked)
    P = np.concatenate([[0.0], np.cumsum(ranked)])
    Q = np.concatenate([[0.0], np.cumsum(ranked * ranked)])
    i = np.arange(n + 1)
    with np.errstate(divide="ignore", invalid="ignore"):
        run = (Q[None, :] - Q[:, None]) - (P[None, :] - P[:, None]) ** 2 / (i[None, :] - i[:, None])      # run[a, b] = cost of ranked[a:b]
    s1, s2 = np.meshgrid(np.arange(n + 1), np.arange(n + 1), indexing="ij")
    ok = (s1 >= 1) & (s2 > s1) & (s2 <= n - 1)
    C = np.full((n + 1, n + 1), np.inf)
    C[ok] = run[0, s1[ok]] + run[s1[ok], s2[ok]] + run[s2[ok], n]
    return C


def checkpoint_margins(scores, K_rem: int, n_clusters: int, tau: float, tol: float) -> dict:
    """Is the outcome of a pruning check on these (oracle) scores immune to perturbing every score by up to tol?
    Three margins, all of which must hold for the check to count as pinned:
      gate     |std - tau |mean|| > (1 + tau) tol            (std and mean move by at most tol each)
      split    every two rank-adjacent scores on either side of a cluster split differ by more than 2 tol
      cost     SSE(second-best partition) - SSE(best) > 4 tol sum |x - mean of its cluster| + 2 n tol^2
    Only k = 3 clusters on more than three distinct scores is classified; anything else reports unpinned."""
    s = np.asarray(scores, np.float64)
    n = len(s)
    mean, std = float(np.mean(s)), float(np.std(s))
    out = {"gate": abs(std - tau * abs(mean)) > (1 + tau) * tol, "split": False, "cost": False}
    ranked = np.sort(s)[::-1]
    if n_clusters == 3 and len(np.unique(ranked)) > 3 and n > K_rem:
        C = _partition_costs_k3(ranked)
        flat = np.sort(C[np.isfinite(C)])
        a, b = np.unravel_index(np.argmin(C), C.shape)
        out["split"] = bool(ranked[a - 1] - ranked[a] > 2 * tol and ranked[b - 1] - ranked[b] > 2 * tol)
        dev = 0.0
        for lo, hi in ((0, a), (a, b), (b, n)):
            dev += float(np.sum(np.abs(ranked[lo:hi] - np.mean(ranked[lo:hi]))))
        out["cost"] = bool(flat[1] - flat[0] > 4 * tol * dev + 2 * n * tol * tol)
        out["splits"] = (int(a), int(b))
    out["pinned"] = bool(out["gate"] and out["split"] and out["cost"])
    return out
