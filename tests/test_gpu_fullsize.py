"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (IEEE half operands),
against the exact (fp64) oracle.

The 0.6B-shaped workload is compared with a complete oracle run.  For the 4B- and 8B-shaped workloads a
complete oracle run would take hours, so the comparison is on sampled outputs the oracle can compute one
by one (candidates never interact, Sec. 2.2): the provisional scores of sampled candidates at every
checkpoint they are live at and, for a survivor, the final full-depth score; plus properties that hold
at any size: the device's routing equals the oracle's route() of the device's own scores at every
checkpoint, survivors' final scores are bit-identical to the unpruned run's, and the returned top-K is
the ranking of the final scores.
"""
import os
import time

import numpy as np
import pytest
import torch

from oracle import prism_oracle as O
from paper_2510_15620_amd import binding as B
from paper_2510_15620_amd import workloads as W
from tests.helpers import oracle_model, oracle_select, to_f64
from tests.test_gpu_select import check_against_oracle

pytestmark = pytest.mark.gpu
TOL = 2e-2


def _progress(msg):
    """Long oracle loops leave a trace so that a quiet run is not mistaken for a hung one (PRISM_PROGRESS_DIR, else a
    scratch folder beside the tests)."""
    d = os.environ.get("PRISM_PROGRESS_DIR") or os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "gpurun_out")
    try:
        os.makedirs(d, exist_ok=True)
        with open(os.path.join(d, "progress.log"), "a") as f:
            f.write(f"{time.strftime('%H:%M:%S')} {msg}\n")
    except OSError:
        pass


def test_cfg2_full_oracle_parity():
    w = W.WORKLOADS["cfg2_0p6b"]
    wt = W.make_weights(w, "cuda")
    q, cands = W.make_tokens(w)
    p = B.Prism(w.model, wt, checkpoints=w.checkpoints)
    idx, scores, rep = p.select(q, cands, w.K)
    p.destroy()
    _progress("cfg2: gpu done, oracle starts")
    ref = oracle_select(w, wt, (q, cands), progress=lambda l, n: _progress(f"cfg2 oracle layer {l} live {n}"))
    check_against_oracle(w, idx, scores, rep, ref, TOL)
    worst = max(float(np.max(np.abs(rep.scores[e][ev.live] - ev.scores))) for e, ev in enumerate(ref.events))
    _progress(f"cfg2: worst |gpu - oracle| {worst:.3e}")


def _rule1_and_topk(w, idx, scores, rep):
    """Properties that need no oracle forward: routing of the device's own scores, final ranking."""
    for e in range(len(rep.layer) - 1):
        live = np.where(~np.isnan(rep.scores[e]))[0]
        r = O.route(rep.scores[e][live].astype(np.float64), w.K, w.n_clusters, float(np.float32(w.cv_threshold)))
        assert np.array_equal(rep.fate[e][live], r.fate), rep.layer[e]
        assert rep.n_after[e] == (int(O.keep_mask(r, O.MODE_DROP_ONLY).sum()) if r.pruned else len(live))
        nxt = np.where(~np.isnan(rep.scores[e + 1]))[0]
        assert np.array_equal(nxt, live[O.keep_mask(r, O.MODE_DROP_ONLY)] if r.pruned else live)
    fin = rep.scores[-1]
    live = np.where(~np.isnan(fin))[0]
    order = live[O.rank_order(fin[live].astype(np.float64))[:w.K]]
    assert idx.tolist() == order.tolist()
    assert np.array_equal(scores, fin[order])


def _oracle_trajectories(w, wt, q, cands, sample, depth, tag):
    """Layer-major oracle pass over the sampled candidates: layer l is drawn on the GPU by the input
    generator, copied to the host as fp64, and every sampled candidate still short of its depth advances."""
    om = oracle_model(w.model)
    fn, wy, wn = to_f64(wt.final_norm), to_f64(wt.w_yes), to_f64(wt.w_no)
    X = {c: to_f64(wt.embed[torch.from_numpy(np.concatenate([q, cands[c]]).astype(np.int64)).cuda()]) for c in sample}
    out = {c: {} for c in sample}
    for l in range(1, max(depth.values()) + 1):
        lw = {k: to_f64(v) for k, v in W.make_layer(w, l - 1, "cuda").items()}
        for c in sample:
            if l <= depth[c]:
                X[c] = O.layer_forward(X[c], lw, om)
                if l in w.checkpoints or l == w.model.n_layers:
                    out[c][l] = O.head_score(X[c][-1], fn, wy, wn, om.rms_eps)
        _progress(f"{tag}: oracle layer {l} done")
    return out


class _HostTable:
    """The same weights with the embedding table in pinned host memory (the two head rows stay on the device)."""
    def __init__(self, wt):
        self.embed = wt.embed.cpu().pin_memory()
        self.layers, self.final_norm = wt.layers, wt.final_norm
        self.w_yes, self.w_no = wt.w_yes.clone(), wt.w_no.clone()


def _run_gpu(w, wt, mode=B.MODE_DROP_ONLY, operand="f16", lean=False, hbm_cap_bytes=None):
    """lean: hidden-state offload and the embedding-table cache on top of the workload's own options."""
    q, cands = W.make_tokens(w)
    weights = wt
    if w.stream_weights:
        host = [{k: v.to("cpu").pin_memory() for k, v in l.items()} for l in wt.layers]
        weights = W.Weights(wt.embed, host, wt.final_norm)
    if lean:
        weights = _HostTable(weights)
    p = B.Prism(w.model, weights, checkpoints=w.checkpoints, mode=mode, chunk_cands=w.chunk_cands,
                hbm_cap_bytes=w.hbm_cap_bytes if hbm_cap_bytes is None else hbm_cap_bytes, stream_weights=w.stream_weights,
                operand=operand, offload_hidden=lean, embed_on_host=lean)
    out = p.select(q, cands, w.K)
    p.destroy()
    return out


def _sampled_check(w, wt, n_survivors=1):
    q, cands = W.make_tokens(w)
    idx, scores, rep = _run_gpu(w, wt)
    _progress(f"{w.name}: pruned gpu run done, survivors {rep.n_after.tolist()}")
    _rule1_and_topk(w, idx, scores, rep)
    assert rep.n_after[-1] < w.n_cands                                   # the workload really prunes
    # sample: the best survivor(s) to full depth, and the first candidate dropped at the first pruning event
    first = next(e for e in range(len(rep.layer)) if rep.n_after[e] < rep.n_before[e])
    dropped = int(np.where(rep.fate[first] == B.FATE_DROPPED)[0][0])
    sample = [int(i) for i in idx[:n_survivors]] + [dropped]
    depth = {c: w.model.n_layers for c in sample}
    depth[dropped] = int(rep.layer[first])
    traj = _oracle_trajectories(w, wt, q, cands, sample, depth, w.name)
    worst = 0.0
    for c in sample:
        for l, s in traj[c].items():
            e = int(np.where(rep.layer == l)[0][0]) if l in rep.layer.tolist() else None
            if e is None or np.isnan(rep.scores[e][c]):
                continue                                                # checkpoint skipped (n_live <= K)
            worst = max(worst, abs(float(rep.scores[e][c]) - s))
            assert abs(float(rep.scores[e][c]) - s) <= TOL, (w.name, c, l, float(rep.scores[e][c]), s)
    _progress(f"{w.name}: worst |gpu - oracle| over sampled scores {worst:.3e}")
    return idx, scores, rep, traj


def _bf16_operand_variant(w, wt, traj):
    """The bf16-operand variant at full size: the properties hold exactly; its distance to the exact oracle
    is inherent to 8-bit significands (a forward with bf16-rounded operands, in any arithmetic, differs from
    the exact one by up to ~0.1 in score on these random-weight models), so it is logged and only bounded
    loosely here."""
    idx, scores, rep = _run_gpu(w, wt, operand="bf16")
    _rule1_and_topk(w, idx, scores, rep)
    worst = 0.0
    for c, tr in traj.items():
        for l, s in tr.items():
            if l in rep.layer.tolist():
                g = rep.scores[int(np.where(rep.layer == l)[0][0])][c]
                if not np.isnan(g):
                    worst = max(worst, abs(float(g) - s))
    _progress(f"{w.name}: bf16 operands: worst |gpu - exact oracle| over sampled scores {worst:.3e}")
    assert worst < 0.3


@pytest.fixture(scope="module")
def weights_8b():
    return W.make_weights(W.WORKLOADS["cfg4_8b"], "cuda")


def test_cfg3_sampled_oracle_parity_and_properties():
    w = W.WORKLOADS["cfg3_4b"]
    wt = W.make_weights(w, "cuda")
    idx, scores, rep, traj = _sampled_check(w, wt)
    idx0, s0, rep0 = _run_gpu(w, wt, B.MODE_NO_PRUNING)
    live = ~np.isnan(rep.scores[-1])
    assert np.array_equal(rep.scores[-1][live], rep0.scores[-1][live])   # drop-only survivors = full-depth scores


def test_cfg4_headline_sampled_oracle_parity_and_properties(weights_8b):
    w = W.WORKLOADS["cfg4_8b"]
    idx, scores, rep, traj = _sampled_check(w, weights_8b, n_survivors=2)
    idx0, s0, rep0 = _run_gpu(w, weights_8b, B.MODE_NO_PRUNING)
    live = ~np.isnan(rep.scores[-1])
    assert np.array_equal(rep.scores[-1][live], rep0.scores[-1][live])
    assert rep.ms_total < rep0.ms_total                                  # pruning cuts the top-K latency
    _bf16_operand_variant(w, weights_8b, traj)


def test_cfg5_streamed_chunked_under_the_hbm_cap(weights_8b):
    """500 candidates, log-normal lengths, weights streamed from pinned host memory one layer ahead,
    chunks of 64 candidates, 24 GB cap on library-owned device memory."""
    w = W.WORKLOADS["cfg5_8b_stream"]
    idx, scores, rep, traj = _sampled_check(w, weights_8b)
    assert rep.peak_hbm_bytes <= w.hbm_cap_bytes
    per_layer = 2 * (w.model.gemm_flops_per_token_layer() // 2)          # bf16 bytes of the matrices of one layer
    assert rep.bytes_streamed >= w.model.n_layers * per_layer


def test_cfg5_offload_and_embedding_cache_are_bit_identical_and_leaner(weights_8b):
    """The 500-candidate pool again with the residual stream in pinned host memory (three chunks on the device) and the
    embedding table behind a device cache of a tenth of its rows: same numbers, a fraction of the device memory."""
    w = W.WORKLOADS["cfg5_8b_stream"]
    idx0, sc0, rep0 = _run_gpu(w, weights_8b)
    cap = 8 * 2 ** 30
    idx1, sc1, rep1 = _run_gpu(w, weights_8b, lean=True, hbm_cap_bytes=cap)
    assert idx0.tolist() == idx1.tolist() and np.array_equal(sc0, sc1)
    assert np.array_equal(rep0.scores, rep1.scores, equal_nan=True) and np.array_equal(rep0.fate, rep1.fate)
    _progress(f"cfg5 lean: peak {rep1.peak_hbm_bytes / 2**30:.2f} GiB vs {rep0.peak_hbm_bytes / 2**30:.2f} GiB, "
              f"hidden bytes moved {rep1.bytes_hidden_moved / 1e9:.1f} GB, embed rows hit/missed "
              f"{rep1.embed_rows_hit}/{rep1.embed_rows_missed}, {rep1.ms_total:.0f} ms vs {rep0.ms_total:.0f} ms")
    assert rep1.peak_hbm_bytes <= cap < rep0.peak_hbm_bytes
    q, cands = W.make_tokens(w)
    lru = O.LruRowCache(w.model.vocab // 10)
    sample = np.concatenate([np.concatenate([q, c]) for c in cands[:40]])     # the oracle's list-based LRU is slow
    assert rep1.embed_rows_hit + rep1.embed_rows_missed == sum(len(q) + len(c) for c in cands)
    # the first 40 sequences of the stream, replayed by the oracle, give a lower bound on misses of the full stream's prefix
    assert rep1.embed_rows_missed >= lru.run(sample)[1]


def test_cfg5_with_4bit_layers_streams_a_quarter_of_the_bytes(weights_8b):
    """The 500-candidate pool with every layer matrix as a 4-bit blob in pinned host memory.  The numbers differ from
    the bf16 run (other weights), so what is checked is what holds for any weights: the routing rule at every check, the
    final ranking, and the bytes that travelled."""
    w = W.WORKLOADS["cfg5_8b_stream"]
    q, cands = W.make_tokens(w)

    class Q4:
        pass
    q4 = Q4()
    q4.embed, q4.final_norm, q4.w_yes, q4.w_no = weights_8b.embed, weights_8b.final_norm, weights_8b.w_yes, weights_8b.w_no
    q4.layers = [{k: v.cpu().pin_memory() for k, v in l.items()} for l in B.quantize_layers_w4(weights_8b.layers)]
    p = B.Prism(w.model, q4, checkpoints=w.checkpoints, chunk_cands=w.chunk_cands, hbm_cap_bytes=w.hbm_cap_bytes,
                stream_weights=True, w4=True)
    idx, scores, rep = p.select(q, cands, w.K)
    p.destroy()
    _rule1_and_topk(w, idx, scores, rep)
    plain = w.model.n_layers * sum(v.numel() * 2 for v in weights_8b.layers[0].values())
    assert 0.25 * plain < rep.bytes_streamed < 0.27 * plain
    assert rep.peak_hbm_bytes <= w.hbm_cap_bytes
    _progress(f"cfg5 w4: {rep.ms_total:.0f} ms, streamed {rep.bytes_streamed / 1e9:.2f} GB of {plain / 1e9:.2f} GB, survivors {rep.n_after.tolist()}")
