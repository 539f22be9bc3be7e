"""CPU oracle for the monolithic-forwarding reranker hot path.  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 numpy implementation of what the HIP library computes: one
forward of a decoder-only cross-encoder reranker over every (query, candidate)
sequence, with progressive cluster pruning between layers, written from the
paper (Sec. 3.3 monolithic forwarding, Sec. 4.1 progressive cluster pruning,
Sec. 4.5 working example, Sec. 7 drop-only variant) and from the layer recipe
of the benchmark configurations (pre-norm RMSNorm, GQA causal attention with
per-head q/k RMSNorm and rotate-half RoPE, SwiGLU FFN, no biases, score =
logit(yes) - logit(no) at the last token).

It shares no code with the HIP path and must never be imported by it.  Only the
tests, the smoke check and the benchmark's cpu_baseline leg call it.  There is no
blocking, fusion or reordering here: every function is the textbook definition
or the paper's step, so it can be read against the paper by eye.  numpy's matmul
and argsort are the only library primitives used as steps.

Readings taken where the paper is silent (each is also listed in the design notes):
  * intermediate score = final RMSNorm, then the yes/no head rows, exactly as
    after the last layer (Sec. 4.1 "the model's classifier");
  * CV uses the population standard deviation; the gate test is written
    division-free, std > tau * |mean|, so mean = 0 opens it and std = 0 closes it;
  * K-Means (Sec. 4.1) on scalars is taken as the exact optimum of the
    within-cluster sum of squares over contiguous partitions of the ranked
    scores; ties between partitions go to the lexicographically smallest split
    positions in rank order; with fewer distinct scores than clusters the number
    of clusters is reduced, with one distinct score nothing is pruned;
  * ranking: score descending, ties by lower original index;
  * number of clusters: an option, default 3;
  * operand precision: Model.operand = "exact" keeps every value in fp64.  "bf16" / "f16" round the
    operands of the matrix-core contractions to that type (round-to-nearest-even): the normalised
    GEMM inputs, q and k after RoPE, v, the attention output and the SwiGLU output - the weights are
    already of that type.  Accumulation, softmax (including the probabilities), norms and the
    residual stream stay in fp64.  This is the arithmetic a 16-bit-operand forward defines, whatever
    its blocking; it is not a model of any particular kernel.  Every parity bar of the device path
    is against "exact"; the rounded modes exist to measure what operand rounding alone costs
    (tests/test_oracle_operand_precision.py) and to compare the bf16-operand device variant with a
    forward of the same operand precision.

Parity status: the numeric score values on the synthetic workloads are "parity
unpinned" by the paper (it prints no scores and ships no weights); they are
pinned by the invariants in tests/test_oracle_*.py.  The dispersion-threshold
value is unpinned as well (the paper shows it only in a figure).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence

import numpy as np

F64 = np.float64

# fates at a pruning event (Sec. 4.1: selected / deferred / dropped)
SELECTED, DEFERRED, DROPPED = 2, 1, 0
# modes
MODE_DROP_ONLY, MODE_THREE_WAY, MODE_NO_PRUNING = 0, 1, 2


# --------------------------------------------------------------------------- layer math

def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    """x / sqrt(mean(x^2) + eps) * g over the last axis."""
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(g, F64)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate-half rotary embedding.  x [L, heads, hd]; pos [L].
    Pair (i, i + hd/2) is rotated by the angle pos * base^(-2i/hd)."""
    x = np.asarray(x, F64)
    hd = x.shape[-1]
    half = hd // 2
    theta = F64(base) ** (-2.0 * np.arange(half, dtype=F64) / hd)
    ang = np.asarray(pos, F64)[:, None] * theta[None, :]          # [L, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def causal_gqa_attention(q: np.ndarray, k: np.ndarray, v: np.ndarray) -> np.ndarray:
    """softmax(q k^T / sqrt(hd), keys j <= i) v for one sequence.
    q [L, nq, hd]; k, v [L, nkv, hd]; query head h reads KV head h // (nq / nkv)."""
    q, k, v = np.asarray(q, F64), np.asarray(k, F64), np.asarray(v, F64)
    L, nq, hd = q.shape
    group = nq // k.shape[1]
    out = np.empty_like(q)
    future = np.triu(np.ones((L, L), dtype=bool), 1)
    for h in range(nq):
        kh, vh = k[:, h // group, :], v[:, h // group, :]
        s = q[:, h, :] @ kh.T / np.sqrt(F64(hd))
        s[future] = -np.inf
        p = np.exp(s - s.max(axis=1, keepdims=True))
        p /= p.sum(axis=1, keepdims=True)
        out[:, h, :] = p @ vh
    return out


def silu(x: np.ndarray) -> np.ndarray:
    return x / (1.0 + np.exp(-x))


def round_operand(x: np.ndarray, kind: str) -> np.ndarray:
    """Value of x after rounding to the operand type (round-to-nearest-even), returned as fp64."""
    if kind == "exact":
        return x
    if kind == "f16":
        return np.asarray(x, F64).astype(np.float16).astype(F64)
    if kind == "bf16":
        f = np.ascontiguousarray(np.asarray(x, F64).astype(np.float32))
        u = f.view(np.uint32).astype(np.uint64)
        u = ((u + 0x7FFF + ((u >> 16) & 1)) >> 16) << 16          # nearest, ties to even, on the top 16 bits
        return u.astype(np.uint32).view(np.float32).reshape(f.shape).astype(F64)
    raise ValueError(kind)


@dataclass
class Model:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    rms_eps: float = 1e-6
    rope_base: float = 1e6
    qk_norm: bool = True
    operand: str = "exact"          # "exact" | "bf16" | "f16": precision of the contraction operands


def attention_block(X: np.ndarray, lw: Dict[str, np.ndarray], m: Model) -> np.ndarray:
    """X + Attn(RMSNorm(X)) W_o^T for one sequence X [L, hidden]; positions 0..L-1."""
    L = X.shape[0]
    rnd = lambda t: round_operand(t, m.operand)
    xn = rnd(rmsnorm(X, lw["attn_norm"], m.rms_eps))
    q = (xn @ lw["wq"].T).reshape(L, m.n_q_heads, m.head_dim)
    k = (xn @ lw["wk"].T).reshape(L, m.n_kv_heads, m.head_dim)
    v = rnd((xn @ lw["wv"].T).reshape(L, m.n_kv_heads, m.head_dim))
    if m.qk_norm:
        q = rmsnorm(q, lw["q_norm"], m.rms_eps)
        k = rmsnorm(k, lw["k_norm"], m.rms_eps)
    pos = np.arange(L)
    q, k = rnd(rope(q, pos, m.rope_base)), rnd(rope(k, pos, m.rope_base))
    a = rnd(causal_gqa_attention(q, k, v).reshape(L, m.n_q_heads * m.head_dim))
    return X + a @ lw["wo"].T


def ffn_block(X: np.ndarray, lw: Dict[str, np.ndarray], m: Model) -> np.ndarray:
    """X + (silu(Xn W_g^T) * (Xn W_u^T)) W_d^T with Xn = RMSNorm(X)."""
    xn = round_operand(rmsnorm(X, lw["ffn_norm"], m.rms_eps), m.operand)
    act = round_operand(silu(xn @ lw["w_gate"].T) * (xn @ lw["w_up"].T), m.operand)
    return X + act @ lw["w_down"].T


def layer_forward(X: np.ndarray, lw: Dict[str, np.ndarray], m: Model) -> np.ndarray:
    return ffn_block(attention_block(X, lw, m), lw, m)


def embed(tokens: np.ndarray, table: np.ndarray) -> np.ndarray:
    return np.asarray(table[np.asarray(tokens, np.int64)], F64)


def head_score(h_last: np.ndarray, final_norm: np.ndarray, w_yes: np.ndarray, w_no: np.ndarray,
               eps: float) -> float:
    """logit(yes) - logit(no) of the normalised last-token state (Sec. 4.1: the model's
    own classifier applied to an intermediate layer's output)."""
    z = rmsnorm(h_last, final_norm, eps)
    return float(z @ np.asarray(w_yes, F64) - z @ np.asarray(w_no, F64))


# --------------------------------------------------------------------------- pruning rule

def coefficient_of_variation(scores: np.ndarray) -> float:
    """CV = |std / mean| (Sec. 4.1), population std.  inf when mean = 0 and std > 0."""
    mean, std = _mean_std(scores)
    if mean == 0.0:
        return float("inf") if std > 0.0 else 0.0
    return abs(std / mean)


def _mean_std(scores) -> tuple:
    # Sequential sums in index order, so that any implementation that adds in the
    # same order gets the same bits.
    n = len(scores)
    tot = 0.0
    for s in scores:
        tot = tot + float(s)
    mean = tot / float(n)
    acc = 0.0
    for s in scores:
        d = float(s) - mean
        acc = acc + d * d
    return mean, math.sqrt(acc / float(n))


def gate_open(scores: np.ndarray, tau: float) -> bool:
    """Prune only when the dispersion exceeds the threshold: CV > tau, tested as
    std > tau * |mean|."""
    mean, std = _mean_std(scores)
    return bool(std > float(tau) * abs(mean))


def rank_order(scores: np.ndarray) -> np.ndarray:
    """Candidate positions from rank 1 to rank n: score descending, lower index first on ties."""
    s = np.asarray(scores, F64)
    return np.lexsort((np.arange(len(s)), -s))


def kmeans_1d_splits(ranked: np.ndarray, k: int) -> List[int]:
    """Exact k-means of scalars already in rank (descending) order.

    Every optimum of the within-cluster sum of squares of scalars is a partition
    into runs of consecutive ranked values, so the search is over split positions
    0 < s_1 < ... < s_{k-1} < n; cluster c is ranked[s_{c-1}:s_c].
    cost(i, j) = sum x^2 - (sum x)^2 / (j - i) over ranked[i:j], from prefix sums.
    E[m][i] = best cost of cutting ranked[i:] into m runs
            = min over s of cost(i, s) + E[m-1][s];  the smallest minimising s is
    kept, which yields the lexicographically smallest split vector among ties.
    Returns the k-1 split positions.
    """
    x = [float(v) for v in ranked]           # Python floats are IEEE doubles
    n = len(x)
    assert 1 <= k <= n
    P = [0.0] * (n + 1)
    Q = [0.0] * (n + 1)
    for i in range(n):                       # sequential prefix sums
        P[i + 1] = P[i] + x[i]
        Q[i + 1] = Q[i] + x[i] * x[i]

    def cost(i, j):
        sp = P[j] - P[i]
        return (Q[j] - Q[i]) - sp * sp / float(j - i)

    INF = float("inf")
    E = [[INF] * (n + 1) for _ in range(k + 1)]
    arg = [[0] * (n + 1) for _ in range(k + 1)]
    for i in range(n):
        E[1][i] = cost(i, n)
    for m in range(2, k + 1):
        # the last stage is only ever read at i = 0
        for i in ([0] if m == k else range(0, n - m + 1)):
            best, best_s = INF, -1
            for s in range(i + 1, n - (m - 1) + 1):
                c = cost(i, s) + E[m - 1][s]
                if c < best:
                    best, best_s = c, s
            E[m][i], arg[m][i] = best, best_s
    splits, i = [], 0
    for m in range(k, 1, -1):
        i = arg[m][i]
        splits.append(i)
    return splits


@dataclass
class RouteResult:
    gate: bool                      # dispersion gate fired
    pruned: bool                    # clustering ran and produced fates
    fate: np.ndarray                # per live candidate (input order): SELECTED / DEFERRED / DROPPED
    cluster: np.ndarray             # per live candidate: cluster number in rank order (0 = best), -1 if not clustered
    n_clusters: int
    mean: float
    std: float
    terminate: bool = False         # three-way mode: |deferred| equals the remaining top-K slots


def route(scores: Sequence[float], K_rem: int, n_clusters: int = 3, tau: float = 0.0) -> RouteResult:
    """One pruning check on the live candidates' provisional scores (Sec. 4.1, Sec. 4.5).

    Gate on the coefficient of variation; cluster; the boundary cluster is the one
    that holds the K_rem-th ranked candidate; clusters with a higher mean are
    selected, with a lower mean dropped, the boundary cluster (and any cluster of
    exactly equal mean) deferred.  With n_live <= K_rem nothing may be dropped, so
    the check is skipped.
    """
    s = np.asarray(scores, F64)
    n = len(s)
    mean, std = _mean_std(s) if n else (0.0, 0.0)
    res = RouteResult(False, False, np.full(n, DEFERRED, np.int8), np.full(n, -1, np.int32), 0, mean, std)
    if n <= K_rem or n == 0:
        return res
    res.gate = gate_open(s, tau)
    if not res.gate:
        return res
    order = rank_order(s)
    ranked = s[order]
    k = min(int(n_clusters), len(np.unique(ranked)))
    if k <= 1:
        return res
    splits = [0] + kmeans_1d_splits(ranked, k) + [n]
    means = []
    for c in range(k):
        tot = 0.0
        for r in range(splits[c], splits[c + 1]):
            tot = tot + float(ranked[r])
        means.append(tot / float(splits[c + 1] - splits[c]))
    b = next(c for c in range(k) if splits[c] <= K_rem - 1 < splits[c + 1])
    for c in range(k):
        fate = SELECTED if means[c] > means[b] else (DROPPED if means[c] < means[b] else DEFERRED)
        for r in range(splits[c], splits[c + 1]):
            res.fate[order[r]] = fate
            res.cluster[order[r]] = c
    res.pruned = True
    res.n_clusters = k
    n_sel = int(np.sum(res.fate == SELECTED))
    res.terminate = int(np.sum(res.fate == DEFERRED)) == K_rem - n_sel
    return res


def keep_mask(r: RouteResult, mode: int) -> np.ndarray:
    """Who stays in the batch after the check.  Drop-only (Sec. 7: only hopeless
    candidates are pruned, contenders run to full depth) keeps selected and deferred;
    three-way keeps only deferred."""
    if mode == MODE_DROP_ONLY:
        return r.fate != DROPPED
    return r.fate == DEFERRED


# --------------------------------------------------------------------------- whole path

@dataclass
class Event:
    layer: int                      # scores taken from the output of this layer (1-indexed); n_layers = final
    live: np.ndarray                # original candidate indices scored, in batch order
    scores: np.ndarray              # fp64, aligned with live
    gate: bool = False
    pruned: bool = False
    fate: Optional[np.ndarray] = None
    cluster: Optional[np.ndarray] = None
    keep: Optional[np.ndarray] = None
    mean: float = 0.0
    std: float = 0.0


@dataclass
class Selection:
    idx: np.ndarray                 # original indices of the top-K, best first
    scores: np.ndarray              # their scores (three-way mode: exit-time scores for early-selected ones)
    events: List[Event] = field(default_factory=list)
    layers_run: int = 0
    token_layers: int = 0           # sum over layers of live tokens (work actually done)


def select(query_tokens, cand_tokens: Sequence, K: int, weights, m: Model, *,
           checkpoints: Sequence[int] = (), n_clusters: int = 3, tau: float = 0.0,
           mode: int = MODE_DROP_ONLY, progress=None) -> Selection:
    """Top-K of the candidates for the query (Sec. 2.1 problem statement), by monolithic
    forwarding with progressive cluster pruning.

    weights: dict with "embed" [V, H], "final_norm" [H], "w_yes" [H], "w_no" [H] and
    "layers": list of dicts (see attention_block / ffn_block) - any float dtype.
    Every live candidate advances one layer at a time together (Sec. 3.3); the pruning
    check on layer l's output happens before layer l+1 runs (Sec. 3.4, Sec. 4.5).
    """
    n = len(cand_tokens)
    K = min(K, n)
    ckpt = set(int(c) for c in checkpoints)
    X = {c: embed(np.concatenate([query_tokens, cand_tokens[c]]), weights["embed"]) for c in range(n)}
    live = list(range(n))
    out = Selection(np.zeros(0, np.int64), np.zeros(0, F64))
    early_idx: List[int] = []
    early_scores: List[float] = []
    K_rem = K

    def score_live():
        return np.array([head_score(X[c][-1], weights["final_norm"], weights["w_yes"], weights["w_no"],
                                    m.rms_eps) for c in live], F64)

    terminated = False
    for l in range(1, m.n_layers + 1):
        lw = weights["layers"][l - 1]
        for c in live:
            X[c] = layer_forward(X[c], lw, m)
            out.token_layers += X[c].shape[0]
        out.layers_run = l
        if progress is not None:
            progress(l, len(live))
        if l in ckpt and l < m.n_layers and mode != MODE_NO_PRUNING and len(live) > K_rem:
            s = score_live()
            r = route(s, K_rem, n_clusters, tau)
            ev = Event(l, np.array(live), s, r.gate, r.pruned, r.fate, r.cluster, None, r.mean, r.std)
            keep = keep_mask(r, mode) if r.pruned else np.ones(len(live), bool)
            ev.keep = keep
            out.events.append(ev)
            if r.pruned and mode == MODE_THREE_WAY:
                sel = [i for i in rank_order(s) if r.fate[i] == SELECTED]
                early_idx += [live[i] for i in sel]
                early_scores += [float(s[i]) for i in sel]
                K_rem -= len(sel)
                if r.terminate:
                    terminated = True
            for i, c in enumerate(live):
                if not keep[i]:
                    del X[c]
            live = [c for i, c in enumerate(live) if keep[i]]
            if terminated:
                # Sec. 4.1 / 4.5: the deferred set fills the remaining slots exactly, so the
                # forward stops here; the set is ordered by its current scores
                final_s = s[keep]
                break
    if not terminated:
        final_s = score_live()
        out.events.append(Event(m.n_layers, np.array(live), final_s))
    order = rank_order(final_s)[:K_rem]
    out.idx = np.array(early_idx + [live[i] for i in order], np.int64)
    out.scores = np.array(early_scores + [float(final_s[i]) for i in order], F64)
    return out


def score_trajectory(query_tokens, cand, weights, m: Model, at_layers: Sequence[int], progress=None) -> Dict[int, float]:
    """Provisional score of ONE candidate after each layer in at_layers (1-indexed), run to
    the deepest of them.  Candidates never interact (Sec. 2.2), so this equals what select()
    sees for that candidate while it is live."""
    X = embed(np.concatenate([query_tokens, cand]), weights["embed"])
    out = {}
    for l in range(1, max(at_layers) + 1):
        X = layer_forward(X, weights["layers"][l - 1], m)
        if progress is not None:
            progress(l, 1)
        if l in at_layers:
            out[l] = head_score(X[-1], weights["final_norm"], weights["w_yes"], weights["w_no"], m.rms_eps)
    return out


W4_GROUP = 128


def quantize_w4(W: np.ndarray, group: int = W4_GROUP):
    """4-bit weights, 16-bit activations (the quantised variant evaluated in Sec. 6).  The paper names the format only;
    the reading taken here: symmetric codes q in [-7, 7] for groups of `group` consecutive input features of one output
    row, one scale per group, scale = max|w| / 7 rounded to bf16 (1 if the group is all zero), q = w / scale rounded
    to nearest (ties to even) and clamped.  With a bf16 scale and |q| <= 7 the product q * scale has at most 11
    significant bits, so the dequantised weight is exact in IEEE half and in fp32.
    Every step is in fp32, as on the device.  Returns (codes int8 [N, K], scales float32 [N, K / group])."""
    W = np.asarray(W, np.float32)
    N, K = W.shape
    assert K % group == 0
    g = W.reshape(N, K // group, group)
    amax = np.max(np.abs(g), axis=2)
    scale = round_operand(amax / np.float32(7.0), "bf16").astype(np.float32)
    scale = np.where(scale == 0, np.float32(1.0), scale).astype(np.float32)
    q = np.rint(g / scale[:, :, None])                       # fp32 division, round half to even
    q = np.clip(q, -7, 7).astype(np.int8)
    return q.reshape(N, K), scale


def dequantize_w4(codes: np.ndarray, scales: np.ndarray, group: int = W4_GROUP) -> np.ndarray:
    """w' = q * scale, exact (see quantize_w4); fp64."""
    N, K = codes.shape
    return (codes.reshape(N, K // group, group).astype(F64) * scales.astype(F64)[:, :, None]).reshape(N, K)


class LruRowCache:
    """Embedding-table cache of Sec. 4.4: a fixed number of table rows kept by least-recently-used replacement.
    Textbook LRU over the stream of token ids, in the order the tokens are embedded (sequence by sequence, position by
    position); the cache persists from one request to the next.  `access` returns True on a hit."""

    def __init__(self, capacity: int):
        assert capacity >= 1
        self.capacity = capacity
        self.order: List[int] = []          # least recently used first

    def access(self, token: int) -> bool:
        hit = token in self.order
        if hit:
            self.order.remove(token)
        elif len(self.order) == self.capacity:
            self.order.pop(0)
        self.order.append(token)
        return hit

    def run(self, tokens: Sequence[int]) -> tuple:
        """(hits, misses) of a token stream, updating the cache."""
        hits = sum(self.access(int(t)) for t in tokens)
        return hits, len(tokens) - hits


def goodman_kruskal_gamma(a: Sequence[float], b: Sequence[float]) -> float:
    """(N_c - N_d) / (N_c + N_d) over candidate pairs (Sec. 3.1): concordant pairs keep
    their relative order between score vectors a and b, discordant pairs reverse it."""
    nc = nd = 0
    for i in range(len(a)):
        for j in range(i + 1, len(a)):
            t = (a[i] - a[j]) * (b[i] - b[j])
            nc += t > 0
            nd += t < 0
    return (nc - nd) / (nc + nd) if nc + nd else 0.0
