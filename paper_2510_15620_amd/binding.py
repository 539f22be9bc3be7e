"""ctypes binding of libprism.so: argument marshalling only - every step of the path runs in the
library's HIP kernels.  Function names follow include/prism.h.  PyTorch tensors are used as
device-memory handles (data_ptr) and for the caller's stream."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass, field
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libprism.so")

OK, EINVAL, ECAP, EHIP, ENOMEM, EUNSUPPORTED = 0, -1, -2, -3, -4, -5
WFMT_PLAIN, WFMT_W4G128 = 0, 1
DTYPE_FP32, DTYPE_BF16, DTYPE_F16 = 0, 1, 2
MODE_DROP_ONLY, MODE_THREE_WAY, MODE_NO_PRUNING = 0, 1, 2
EPI_STORE, EPI_RESIDUAL, EPI_SWIGLU, EPI_STORE_F32 = 0, 1, 2, 3
FATE_NOT_LIVE, FATE_DROPPED, FATE_DEFERRED, FATE_SELECTED = -1, 0, 1, 2
KIND_TRANSFERS = 8          # bit of prism_report.kind_mask that asks for ms_transfers (PRISM_KIND_MASK_TRANSFERS)
MAX_CANDS, MAX_CLUSTERS, MAX_SEQ = 4096, 8, 8192

EXPORTS = ["prism_create", "prism_select", "prism_set_forced_keep", "prism_destroy", "prism_strerror",
           "prism_last_error", "prism_op_embed", "prism_op_rmsnorm", "prism_op_gemm", "prism_op_qkv_finish", "prism_op_qkv_project", "prism_w4_bytes", "prism_op_quantize_w4", "prism_op_dequantize_w4",
           "prism_op_attention", "prism_op_score", "prism_op_route", "prism_op_route_static", "prism_op_compact", "prism_op_topk", "prism_vt_column_of_key"]


class PrismError(RuntimeError):
    def __init__(self, code: int, detail: str):
        super().__init__(f"prism error {code}: {detail}")
        self.code = code


class prism_model(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("n_layers", "hidden", "n_q_heads", "n_kv_heads", "head_dim", "ffn", "vocab")] + \
               [("rms_eps", C.c_float), ("rope_base", C.c_float), ("dtype", C.c_int32), ("qk_norm", C.c_int32)]


LAYER_FIELDS = ("attn_norm", "wq", "wk", "wv", "q_norm", "k_norm", "wo", "ffn_norm", "w_gate", "w_up", "w_down")


class prism_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in LAYER_FIELDS]


class prism_weights(C.Structure):
    _fields_ = [("embed", C.c_void_p), ("layers", C.POINTER(prism_layer_weights)), ("final_norm", C.c_void_p),
                ("w_yes", C.c_void_p), ("w_no", C.c_void_p), ("layer_residency", C.c_int32), ("embed_residency", C.c_int32), ("layer_format", C.c_int32)]


class prism_options(C.Structure):
    _fields_ = [("checkpoint_layers", C.POINTER(C.c_int32)), ("n_checkpoints", C.c_int32), ("cv_threshold", C.c_float),
                ("n_clusters", C.c_int32), ("mode", C.c_int32), ("chunk_cands", C.c_int32), ("hbm_cap_bytes", C.c_int64),
                ("stream", C.c_void_p), ("operand", C.c_int32), ("offload_hidden", C.c_int32), ("embed_cache_rows", C.c_int32), ("stream_slots", C.c_int32),
                ("no_query_sharing", C.c_int32), ("single_pass_checks", C.c_int32)]


class prism_report(C.Structure):
    _fields_ = [("cap_events", C.c_int32), ("n_cands", C.c_int32), ("n_events", C.c_int32),
                ("ev_layer", C.POINTER(C.c_int32)), ("ev_n_before", C.POINTER(C.c_int32)),
                ("ev_n_after", C.POINTER(C.c_int32)), ("ev_tokens_after", C.POINTER(C.c_int32)),
                ("ev_gate", C.POINTER(C.c_int32)), ("ev_n_clusters", C.POINTER(C.c_int32)),
                ("ev_mean", C.POINTER(C.c_double)), ("ev_std", C.POINTER(C.c_double)),
                ("ev_scores", C.POINTER(C.c_float)), ("ev_fate", C.POINTER(C.c_int8)),
                ("ms_total", C.c_double), ("ms_layers", C.c_double), ("ms_checks", C.c_double),
                ("token_layers", C.c_int64), ("peak_hbm_bytes", C.c_int64), ("bytes_streamed", C.c_int64),
                ("layers_run", C.c_int32), ("kind_launches", C.c_int32 * 6), ("kind_ms", C.c_double * 6),
                ("kind_flops", C.c_double * 6), ("bytes_hidden_moved", C.c_int64), ("embed_rows_hit", C.c_int64),
                ("embed_rows_missed", C.c_int64), ("span_cap", C.c_int32), ("n_spans", C.c_int32),
                ("span_kind", C.POINTER(C.c_int32)), ("span_rows", C.POINTER(C.c_int32)), ("span_ms", C.POINTER(C.c_float)),
                ("span_flops", C.POINTER(C.c_double)), ("kind_mask", C.c_int32), ("ms_transfers", C.c_double)]


_lib = None


def lib() -> C.CDLL:
    """The HIP library.  There is no fallback: a missing library is an error."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise PrismError(EHIP, f"{LIB_PATH} is not built; run `python -m paper_2510_15620_amd.build`")
        # PyTorch ships its own copy of the HIP runtime.  Streams and device pointers cross between it and this library,
        # so both must use ONE runtime instance: load PyTorch's first and let the library bind to it.  (Loaded the other
        # way round, the second copy finds no device.)
        import torch  # noqa: F401
        _lib = C.CDLL(LIB_PATH)
        _lib.prism_strerror.restype = C.c_char_p
        _lib.prism_last_error.restype = C.c_char_p
        _lib.prism_destroy.restype = None
        vp, i32, f32 = C.c_void_p, C.c_int32, C.c_float
        _lib.prism_create.argtypes = [C.POINTER(prism_model), C.POINTER(prism_weights), C.POINTER(prism_options), C.POINTER(vp)]
        _lib.prism_select.argtypes = [vp, C.POINTER(i32), i32, C.POINTER(C.POINTER(i32)), C.POINTER(i32), i32, i32,
                                      C.POINTER(i32), C.POINTER(f32), C.POINTER(i32), C.POINTER(prism_report)]
        _lib.prism_set_forced_keep.argtypes = [vp, C.POINTER(C.c_int8), i32, i32]
        _lib.prism_destroy.argtypes = [vp]
        _lib.prism_strerror.argtypes = [i32]
        _lib.prism_op_embed.argtypes = [vp, i32, vp, i32, i32, vp, vp]
        _lib.prism_op_rmsnorm.argtypes = [vp, vp, i32, i32, f32, i32, vp, vp]
        _lib.prism_op_gemm.argtypes = [i32, i32, vp, vp, vp, i32, i32, i32, vp]
        _lib.prism_op_qkv_finish.argtypes = [i32, vp, vp, i32, vp, vp, i32, i32, i32, i32, f32, f32, i32, vp, vp, vp, C.c_int64, vp]
        _lib.prism_op_qkv_project.argtypes = [i32, vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, f32, f32, i32, vp, vp, vp,
                                              C.c_int64, vp]
        _lib.prism_op_attention.argtypes = [i32, vp, vp, C.c_int64, C.POINTER(i32), C.POINTER(i32), i32, i32, i32, i32, vp, vp]
        _lib.prism_op_score.argtypes = [vp, vp, i32, i32, vp, vp, vp, i32, f32, vp, vp]
        _lib.prism_op_route.argtypes = [vp, i32, i32, i32, f32, vp, vp, vp]
        _lib.prism_op_route_static.argtypes = [vp, i32, i32, i32, f32, vp, vp, vp]
        _lib.prism_op_compact.argtypes = [vp, vp, vp, vp, vp, i32, i32, vp]
        _lib.prism_op_topk.argtypes = [vp, i32, i32, vp, vp, vp]
        _lib.prism_w4_bytes.restype = C.c_int64
        _lib.prism_w4_bytes.argtypes = [i32, i32]
        _lib.prism_op_quantize_w4.argtypes = [vp, i32, i32, vp, vp]
        _lib.prism_op_dequantize_w4.argtypes = [vp, i32, i32, i32, vp, vp]
    return _lib


def _check(rc: int):
    if rc != OK:
        l = lib()
        raise PrismError(rc, f"{l.prism_strerror(rc).decode()}: {l.prism_last_error().decode()}")


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _i32_array(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(C.POINTER(C.c_int32))


@dataclass
class Report:
    layer: np.ndarray
    n_before: np.ndarray
    n_after: np.ndarray
    tokens_after: np.ndarray
    gate: np.ndarray
    n_clusters: np.ndarray
    mean: np.ndarray
    std: np.ndarray
    scores: np.ndarray          # [n_events, n_cands], NaN where not live
    fate: np.ndarray            # [n_events, n_cands]
    ms_total: float
    ms_layers: float
    ms_checks: float
    token_layers: int
    peak_hbm_bytes: int
    bytes_streamed: int
    layers_run: int
    kind_launches: List[int] = field(default_factory=list)   # QKV, O, gate/up, down GEMMs, attention, elementwise
    kind_ms: List[float] = field(default_factory=list)
    kind_flops: List[float] = field(default_factory=list)
    bytes_hidden_moved: int = 0
    embed_rows_hit: int = 0
    embed_rows_missed: int = 0
    ms_transfers: float = 0.0   # side-stream time spent copying streamed layer weights
    spans: Optional[np.ndarray] = None   # per launch, in order: structured array (kind, rows, ms, flops); None unless asked for


class Prism:
    """prism_create / prism_select / prism_set_forced_keep / prism_destroy."""

    def __init__(self, model, weights, *, checkpoints: Sequence[int] = (), cv_threshold: float = 0.0, n_clusters: int = 3,
                 mode: int = MODE_DROP_ONLY, chunk_cands: int = 0, hbm_cap_bytes: int = 0, stream_weights: bool = False,
                 stream: Optional[int] = None, operand: str = "f16", offload_hidden: bool = False, embed_on_host: bool = False,
                 embed_cache_rows: int = 0, w4: bool = False, stream_slots: int = 0, share_query: bool = True,
                 two_pass_checks: bool = True):
        """model: object with n_layers, hidden, n_q_heads, n_kv_heads, head_dim, ffn, vocab, rms_eps, rope_base,
        qk_norm, dtype ("fp32" | "bf16": storage type of the weights).  operand ("f16" | "bf16"): 16-bit type of the
        matrix-core operands when the weights are bf16.  weights: object with embed, final_norm, w_yes, w_no (device tensors) and
        layers: list of dicts of tensors (device, or pinned host when stream_weights).  embed_on_host: weights.embed is a
        pinned host tensor (w_yes / w_no stay device tensors) read through a device LRU cache of embed_cache_rows rows.
        offload_hidden: the residual stream lives in pinned host memory, three chunks at a time on the device.
        w4: the seven matrices of every layer dict are uint8 blobs from quantize_w4 (gains stay bf16).
        share_query=False: every sequence carries its own copy of the query (prism_options.no_query_sharing).
        two_pass_checks=False: a checked layer runs completely before its check (prism_options.single_pass_checks)."""
        self._ctx = C.c_void_p()
        m = prism_model(model.n_layers, model.hidden, model.n_q_heads, model.n_kv_heads, model.head_dim, model.ffn,
                        model.vocab, model.rms_eps, model.rope_base, DTYPE_FP32 if model.dtype == "fp32" else DTYPE_BF16,
                        int(model.qk_norm))
        layers = (prism_layer_weights * model.n_layers)()
        for l, lw in enumerate(weights.layers):
            for n in LAYER_FIELDS:
                setattr(layers[l], n, _ptr(lw[n]))
        self._keep = (weights, layers)      # borrowed by the library for the context's lifetime
        w = prism_weights(_ptr(weights.embed), layers, _ptr(weights.final_norm), _ptr(weights.w_yes), _ptr(weights.w_no),
                          1 if stream_weights else 0, 1 if embed_on_host else 0, WFMT_W4G128 if w4 else WFMT_PLAIN)
        ck, ckp = _i32_array(list(checkpoints))
        o = prism_options(ckp, len(ck), cv_threshold, n_clusters, mode, chunk_cands, hbm_cap_bytes,
                          _stream() if stream is None else stream, DTYPE_BF16 if operand == "bf16" else DTYPE_F16,
                          int(offload_hidden), embed_cache_rows, stream_slots, 0 if share_query else 1,
                          0 if two_pass_checks else 1)
        self.n_checkpoints = len(ck)
        _check(lib().prism_create(C.byref(m), C.byref(w), C.byref(o), C.byref(self._ctx)))

    def select(self, query_tokens, cand_tokens: Sequence, K: int, report: bool = True, spans: int = 0, kinds=None):
        """spans: capacity of the per-launch detail of the report (0 = none).  kinds: the kernel kinds that get event spans
        (iterable of kind numbers; None = all); KIND_TRANSFERS in it additionally times the streamed layers' copies."""
        q, qp = _i32_array(query_tokens)
        cands = [np.ascontiguousarray(c, dtype=np.int32) for c in cand_tokens]
        n = len(cands)
        cptrs = (C.POINTER(C.c_int32) * max(n, 1))(*[c.ctypes.data_as(C.POINTER(C.c_int32)) for c in cands])
        lens, lp = _i32_array([len(c) for c in cands])
        kk = max(K, 1)
        out_idx = np.full(kk, -1, np.int32)
        out_scores = np.full(kk, np.nan, np.float32)
        count = C.c_int32(0)
        rep = None
        if report:
            cap = self.n_checkpoints + 1
            arrs = {k: np.zeros(cap, np.int32) for k in ("layer", "n_before", "n_after", "tokens_after", "gate", "n_clusters")}
            arrs["mean"], arrs["std"] = np.zeros(cap, np.float64), np.zeros(cap, np.float64)
            arrs["scores"] = np.zeros((cap, max(n, 1)), np.float32)
            arrs["fate"] = np.zeros((cap, max(n, 1)), np.int8)
            P = lambda a, t: a.ctypes.data_as(C.POINTER(t))
            rep = prism_report(cap, max(n, 1), 0, P(arrs["layer"], C.c_int32), P(arrs["n_before"], C.c_int32),
                               P(arrs["n_after"], C.c_int32), P(arrs["tokens_after"], C.c_int32), P(arrs["gate"], C.c_int32),
                               P(arrs["n_clusters"], C.c_int32), P(arrs["mean"], C.c_double), P(arrs["std"], C.c_double),
                               P(arrs["scores"], C.c_float), P(arrs["fate"], C.c_int8))
            if spans > 0:
                sp = {"kind": np.zeros(spans, np.int32), "rows": np.zeros(spans, np.int32), "ms": np.zeros(spans, np.float32),
                      "flops": np.zeros(spans, np.float64)}
                rep.span_cap = spans
                rep.span_kind, rep.span_rows = P(sp["kind"], C.c_int32), P(sp["rows"], C.c_int32)
                rep.span_ms, rep.span_flops = P(sp["ms"], C.c_float), P(sp["flops"], C.c_double)
            if kinds is not None:
                rep.kind_mask = sum(1 << int(k) for k in kinds)
        _check(lib().prism_select(self._ctx, qp, len(q), cptrs, lp, n, K, out_idx.ctypes.data_as(C.POINTER(C.c_int32)),
                                  out_scores.ctypes.data_as(C.POINTER(C.c_float)), C.byref(count),
                                  C.byref(rep) if rep is not None else None))
        k = count.value
        r = None
        if rep is not None:
            e = rep.n_events
            r = Report(arrs["layer"][:e], arrs["n_before"][:e], arrs["n_after"][:e], arrs["tokens_after"][:e],
                       arrs["gate"][:e].astype(bool), arrs["n_clusters"][:e], arrs["mean"][:e], arrs["std"][:e],
                       arrs["scores"][:e], arrs["fate"][:e], rep.ms_total, rep.ms_layers, rep.ms_checks,
                       rep.token_layers, rep.peak_hbm_bytes, rep.bytes_streamed, rep.layers_run,
                       list(rep.kind_launches), list(rep.kind_ms), list(rep.kind_flops), rep.bytes_hidden_moved,
                       rep.embed_rows_hit, rep.embed_rows_missed, rep.ms_transfers)
            if spans > 0:
                n = rep.n_spans
                r.spans = np.rec.fromarrays([sp["kind"][:n], sp["rows"][:n], sp["ms"][:n], sp["flops"][:n]],
                                            names="kind,rows,ms,flops")
        return out_idx[:k].copy(), out_scores[:k].copy(), r

    def set_forced_keep(self, masks: Optional[np.ndarray]):
        if masks is None:
            _check(lib().prism_set_forced_keep(self._ctx, None, 0, 0))
            return
        m = np.ascontiguousarray(masks, dtype=np.int8)
        _check(lib().prism_set_forced_keep(self._ctx, m.ctypes.data_as(C.POINTER(C.c_int8)), m.shape[0], m.shape[1]))

    def destroy(self):
        if self._ctx:
            lib().prism_destroy(self._ctx)
            self._ctx = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


# ---- kernel-level entry points (device tensors in, device tensors out) ---------------------------------------------

def _dt(t) -> int:
    import torch
    return {torch.float32: DTYPE_FP32, torch.bfloat16: DTYPE_BF16, torch.float16: DTYPE_F16}[t.dtype]


def op_embed(tokens, table, X):
    _check(lib().prism_op_embed(_ptr(tokens), tokens.numel(), _ptr(table), table.shape[1], _dt(table), _ptr(X), _stream()))


def op_rmsnorm(X, gain, eps, out):
    _check(lib().prism_op_rmsnorm(_ptr(X), _ptr(gain), X.shape[0], X.shape[1], eps, _dt(gain), _ptr(out), _stream()))


def op_gemm(epilogue, A, W, out):
    _check(lib().prism_op_gemm(_dt(A), epilogue, _ptr(A), _ptr(W), _ptr(out), A.shape[0], W.shape[0], A.shape[1], _stream()))


def op_qkv_finish(dtype, QKV, pos, max_pos, q_gain, k_gain, nq, nkv, hd, eps, base, qk_norm, QK=None, Vt=None,
                  vt_col=None, vt_stride=0):
    _check(lib().prism_op_qkv_finish(dtype, _ptr(QKV), _ptr(pos), max_pos, _ptr(q_gain), _ptr(k_gain), QKV.shape[0],
                                     nq, nkv, hd, eps, base, int(qk_norm), _ptr(QK), _ptr(Vt), _ptr(vt_col), vt_stride,
                                     _stream()))


def op_qkv_project(Xn, Wqkv, pos, max_pos, q_gain, k_gain, nq, nkv, hd, eps, base, qk_norm, QK, Vt, vt_col, vt_stride):
    _check(lib().prism_op_qkv_project(_dt(Xn), _ptr(Xn), _ptr(Wqkv), _ptr(pos), max_pos, _ptr(q_gain), _ptr(k_gain),
                                      Xn.shape[0], Xn.shape[1], nq, nkv, hd, eps, base, int(qk_norm), _ptr(QK), _ptr(Vt),
                                      _ptr(vt_col), vt_stride, _stream()))


def w4_bytes(N: int, K: int) -> int:
    return int(lib().prism_w4_bytes(N, K))


def quantize_w4(W):
    """W [N, K] bf16 device tensor -> uint8 device tensor holding the 4-bit blob (codes, then bf16 scales)."""
    import torch
    N, K = W.shape
    blob = torch.empty(w4_bytes(N, K), dtype=torch.uint8, device=W.device)
    _check(lib().prism_op_quantize_w4(_ptr(W), N, K, _ptr(blob), _stream()))
    return blob


def dequantize_w4(blob, N: int, K: int, out):
    _check(lib().prism_op_dequantize_w4(_ptr(blob), N, K, _dt(out), _ptr(out), _stream()))


MATRICES = ("wq", "wk", "wv", "wo", "w_gate", "w_up", "w_down")


def quantize_layers_w4(layers):
    """Layer dicts with the seven matrices replaced by their 4-bit blobs (device tensors in, device tensors out)."""
    return [{k: (quantize_w4(v) if k in MATRICES else v) for k, v in l.items()} for l in layers]


def vt_column_of_key(p):
    """Column, relative to its sequence's first, of the key at position p in the transposed V buffer: the library's
    prism_vt_column_of_key applied to an int or elementwise to an integer array (its 16 values per group, tiled)."""
    perm = np.array([lib().prism_vt_column_of_key(i) for i in range(16)], dtype=np.int64)
    p = np.asarray(p)
    out = (p & ~15) | perm[p & 15]
    return int(out) if out.ndim == 0 else out.astype(p.dtype)


def op_attention(dtype, QK, Vt, vt_stride, cu_seqlens, vt_col0, nq, nkv, hd, out):
    cu, cup = _i32_array(cu_seqlens)
    c0, c0p = _i32_array(vt_col0 if vt_col0 is not None else np.zeros(len(cu) - 1))
    _check(lib().prism_op_attention(dtype, _ptr(QK), _ptr(Vt), vt_stride, cup, c0p, len(cu) - 1, nq, nkv, hd, _ptr(out),
                                    _stream()))


def op_score(X, last_row, final_norm, w_yes, w_no, eps, scores):
    _check(lib().prism_op_score(_ptr(X), _ptr(last_row), last_row.numel(), X.shape[1], _ptr(final_norm), _ptr(w_yes),
                                _ptr(w_no), _dt(final_norm), eps, _ptr(scores), _stream()))


def op_route(scores, K_rem, n_clusters, tau, fate, stats):
    _check(lib().prism_op_route(_ptr(scores), scores.numel(), K_rem, n_clusters, tau, _ptr(fate), _ptr(stats), _stream()))


def op_route_static(scores, K_rem, n_clusters, tau, fate, stats):
    """prism_op_route on the library's static workspace: allocates nothing and does not synchronise."""
    _check(lib().prism_op_route_static(_ptr(scores), scores.numel(), K_rem, n_clusters, tau, _ptr(fate), _ptr(stats), _stream()))


def op_compact(X_src, X_dst, src_start, dst_start, length):
    _check(lib().prism_op_compact(_ptr(X_src), _ptr(X_dst), _ptr(src_start), _ptr(dst_start), _ptr(length),
                                  length.numel(), X_src.shape[1], _stream()))


def op_topk(scores, K, out_pos, out_scores):
    _check(lib().prism_op_topk(_ptr(scores), scores.numel(), K, _ptr(out_pos), _ptr(out_scores), _stream()))
