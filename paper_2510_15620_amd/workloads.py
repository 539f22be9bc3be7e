"""Seeded synthetic workloads for the reranker hot path.

This module only *draws inputs* (weights, token ids, lengths).  It contains none
of the method's arithmetic and is the single piece shared by the CPU oracle's
tests and the HIP library's tests / benchmark.

Every value is a pure function of (seed, tensor name, element index): a 32-bit
counter hash picks a 16-bit quantile index and a 65 536-entry normal-quantile
table (built once on the CPU in fp64) turns it into a Gaussian draw.  The device
side of the generator is integer arithmetic plus one table gather, so a tensor
generated on the GPU is bit-identical to the same tensor generated on the CPU.

The workloads stand in for the retrieval pools the paper evaluates on
(Sec. 6.1: short dense sequences of at most a few hundred tokens, tens of
candidates per query); only their shapes are taken.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Tuple

import numpy as np
import torch

_M32 = 0xFFFFFFFF
_MULT = 0x45D9F3B


def _mix32_int(x: int) -> int:
    x &= _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    return ((x >> 16) ^ x) & _M32


def _mix32(x: torch.Tensor) -> torch.Tensor:
    """Same mixer on an int64 tensor whose values stay below 2**32 (no overflow:
    a 32-bit value times a 27-bit constant fits in 63 bits)."""
    x = (((x >> 16) ^ x) * _MULT) & _M32
    x = (((x >> 16) ^ x) * _MULT) & _M32
    return (x >> 16) ^ x


def _stream_keys(seed: int, name: str) -> Tuple[int, int]:
    h = _mix32_int(seed * 0x9E3779B1 + 0x7F4A7C15)
    for ch in name.encode():
        h = _mix32_int(h * 31 + ch + 1)
    return h, _mix32_int(h ^ 0xA5A5A5A5)


def hash_u32(seed: int, name: str, start: int, count: int, device="cpu") -> torch.Tensor:
    """32-bit hash of element indices start..start+count-1 of stream (seed, name)."""
    k1, k2 = _stream_keys(seed, name)
    i = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix32((_mix32(i ^ k1) + k2) & _M32)


_QUANTILES: Optional[np.ndarray] = None


def normal_quantiles() -> np.ndarray:
    """Phi^-1((j + 1/2) / 65536), j = 0..65535, in fp64 (computed on the CPU only)."""
    global _QUANTILES
    if _QUANTILES is None:
        from scipy.special import ndtri
        _QUANTILES = ndtri((np.arange(65536, dtype=np.float64) + 0.5) / 65536.0)
    return _QUANTILES


def gaussian(seed: int, name: str, shape, mean: float, std: float, dtype: torch.dtype,
             device="cpu", block: int = 1 << 26) -> torch.Tensor:
    """Tensor of draws mean + std * z, z ~ N(0,1) (65 536-level quantile table),
    rounded to `dtype` (round-to-nearest-even for bf16) on the CPU table."""
    table = torch.from_numpy(mean + std * normal_quantiles()).to(torch.float32).to(dtype).to(device)
    n = int(np.prod(shape))
    out = torch.empty(n, dtype=dtype, device=device)
    for s in range(0, n, block):
        c = min(block, n - s)
        out[s:s + c] = table[hash_u32(seed, name, s, c, device) >> 16]
    return out.view(*shape)


def gaussian_rows(seed: int, name: str, rows, row_len: int, mean: float, std: float, dtype: torch.dtype) -> torch.Tensor:
    """Rows `rows` of the [*, row_len] tensor that gaussian() draws for (seed, name), without drawing the rest (a value
    depends on its element index only).  CPU."""
    table = torch.from_numpy(mean + std * normal_quantiles()).to(torch.float32).to(dtype)
    out = torch.empty(len(rows), row_len, dtype=dtype)
    for i, r in enumerate(rows):
        out[i] = table[hash_u32(seed, name, int(r) * row_len, row_len) >> 16]
    return out


def uniform_int(seed: int, name: str, count: int, lo: int, hi: int) -> np.ndarray:
    """count integers i.i.d. uniform on the closed range [lo, hi] (host side)."""
    h = hash_u32(seed, name, 0, count).numpy()
    return (lo + h % (hi - lo + 1)).astype(np.int32)


@dataclass
class ModelShape:
    n_layers: int
    hidden: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    ffn: int
    vocab: int
    dtype: str = "bf16"            # "fp32" or "bf16": storage type of weights, compute type of the GEMMs
    rms_eps: float = 1e-6
    rope_base: float = 1e6
    qk_norm: bool = True

    @property
    def q_dim(self):
        return self.n_q_heads * self.head_dim

    @property
    def kv_dim(self):
        return self.n_kv_heads * self.head_dim

    def gemm_flops_per_token_layer(self) -> int:
        h, f = self.hidden, self.ffn
        return 2 * (h * (self.q_dim + 2 * self.kv_dim) + self.q_dim * h + 3 * h * f)

    def attn_flops_per_seq_layer(self, L: int) -> int:
        return 2 * self.n_q_heads * self.head_dim * L * (L + 1)


@dataclass
class Workload:
    name: str
    model: ModelShape
    query_len: int
    n_cands: int
    doc_len: Tuple            # ("uniform", lo, hi) | ("const", n) | ("lognormal", median, sigma, lo, hi)
    K: int
    checkpoints: List[int]    # 1-indexed "after layer l"
    n_clusters: int = 3
    cv_threshold: float = 0.0
    chunk_cands: int = 0
    stream_weights: bool = False
    hbm_cap_bytes: int = 0
    seed: int = 0
    weights_name: str = ""    # stream name of the weight tensors; "" = the workload's own name

    @property
    def wname(self) -> str:
        return self.weights_name or self.name


def _every(n_layers, stride):
    return [l for l in range(stride, n_layers, stride)]


WORKLOADS: Dict[str, Workload] = {
    # benchmark configuration 1: tiny fp32 model
    "cfg1_tiny": Workload("cfg1_tiny", ModelShape(2, 256, 4, 2, 64, 688, 1000, "fp32"),
                          16, 8, ("uniform", 16, 48), 3, [1]),
    # benchmark configuration 2: 0.6B-shaped
    "cfg2_0p6b": Workload("cfg2_0p6b", ModelShape(28, 1024, 16, 8, 128, 3072, 151936),
                          32, 40, ("uniform", 128, 480), 10, _every(28, 4)),
    # benchmark configuration 3: 4B-shaped
    "cfg3_4b": Workload("cfg3_4b", ModelShape(36, 2560, 32, 8, 128, 9728, 151936),
                        32, 100, ("uniform", 256, 992), 10, _every(36, 4)),
    # benchmark configuration 4: 8B-shaped headline, every sequence exactly 1024 tokens (64 + 960)
    "cfg4_8b": Workload("cfg4_8b", ModelShape(36, 4096, 32, 8, 128, 12288, 151936),
                        64, 100, ("const", 960), 10, _every(36, 4)),
    # benchmark configuration 5: 8B-shaped, weights streamed from pinned host memory, chunks of 64
    "cfg5_8b_stream": Workload("cfg5_8b_stream", ModelShape(36, 4096, 32, 8, 128, 12288, 151936),
                               64, 500, ("lognormal", 400.0, 0.6, 32, 2048), 20, _every(36, 4),
                               chunk_cands=64, stream_weights=True, hbm_cap_bytes=24 * 10**9,
                               weights_name="cfg4_8b"),       # "8B-shaped reranker as in the previous config"
    # small cases for element-by-element parity (not benchmark configurations)
    "mini_bf16": Workload("mini_bf16", ModelShape(4, 512, 8, 2, 128, 1408, 2048),
                          24, 13, ("uniform", 20, 300), 4, [1, 2, 3]),
    "mini_fp32": Workload("mini_fp32", ModelShape(3, 192, 6, 3, 32, 400, 500, "fp32"),
                          9, 11, ("uniform", 5, 70), 3, [1, 2]),
}


def doc_lengths(w: Workload) -> np.ndarray:
    kind = w.doc_len[0]
    if kind == "const":
        return np.full(w.n_cands, w.doc_len[1], dtype=np.int32)
    if kind == "uniform":
        return uniform_int(w.seed, w.name + "/doc_len", w.n_cands, w.doc_len[1], w.doc_len[2])
    if kind == "lognormal":
        _, median, sigma, lo, hi = w.doc_len
        u = hash_u32(w.seed, w.name + "/doc_len", 0, w.n_cands).numpy() >> 16
        z = normal_quantiles()[u]
        return np.clip(np.rint(median * np.exp(sigma * z)), lo, hi).astype(np.int32)
    raise ValueError(kind)


def make_tokens(w: Workload):
    """-> (query_tokens int32[query_len], [cand_tokens int32[len_c]] * n_cands)."""
    v = w.model.vocab
    q = uniform_int(w.seed, w.name + "/query", w.query_len, 0, v - 1)
    lens = doc_lengths(w)
    cands = [uniform_int(w.seed, f"{w.name}/cand{c}", int(lens[c]), 0, v - 1) for c in range(w.n_cands)]
    return q, cands


LAYER_TENSORS = ("attn_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


def layer_tensor_shapes(m: ModelShape) -> Dict[str, Tuple[int, ...]]:
    """Row-major [out_features, in_features] matrices (y = x W^T) and gain vectors."""
    return {
        "attn_norm": (m.hidden,), "wq": (m.q_dim, m.hidden), "wk": (m.kv_dim, m.hidden),
        "wv": (m.kv_dim, m.hidden), "q_norm": (m.head_dim,), "k_norm": (m.head_dim,),
        "wo": (m.hidden, m.q_dim), "ffn_norm": (m.hidden,), "w_gate": (m.ffn, m.hidden),
        "w_up": (m.ffn, m.hidden), "w_down": (m.hidden, m.ffn),
    }


def torch_dtype(m: ModelShape) -> torch.dtype:
    return torch.float32 if m.dtype == "fp32" else torch.bfloat16


def make_layer(w: Workload, layer: int, device="cpu") -> Dict[str, torch.Tensor]:
    """Matrices ~ N(0, 0.02); RMSNorm gains ~ 1 + N(0, 0.02) so that a dropped gain shows."""
    dt = torch_dtype(w.model)
    out = {}
    for name, shape in layer_tensor_shapes(w.model).items():
        mean = 1.0 if len(shape) == 1 else 0.0
        out[name] = gaussian(w.seed, f"{w.wname}/L{layer}/{name}", shape, mean, 0.02, dt, device)
    return out


@dataclass
class Weights:
    embed: torch.Tensor                       # [vocab, hidden]
    layers: List[Dict[str, torch.Tensor]]
    final_norm: torch.Tensor                  # [hidden]
    yes_id: int = 1                           # tied head: w_yes = embed[1], w_no = embed[0]
    no_id: int = 0

    @property
    def w_yes(self):
        return self.embed[self.yes_id]

    @property
    def w_no(self):
        return self.embed[self.no_id]


def make_weights(w: Workload, device="cpu", layers: Optional[List[int]] = None) -> Weights:
    """All tensors of the model (or only the listed layers; others are left out as None)."""
    dt = torch_dtype(w.model)
    m = w.model
    embed = gaussian(w.seed, w.wname + "/embed", (m.vocab, m.hidden), 0.0, 0.02, dt, device)
    final_norm = gaussian(w.seed, w.wname + "/final_norm", (m.hidden,), 1.0, 0.02, dt, device)
    ls = [make_layer(w, l, device) if (layers is None or l in layers) else None for l in range(m.n_layers)]
    return Weights(embed, ls, final_norm)
