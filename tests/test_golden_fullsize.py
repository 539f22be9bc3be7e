"""The stored complete oracle runs of the 4B- and 8B-shaped workloads (tests/golden/fullsize_*.json, written by
tests/golden/make_fullsize_goldens.py) are internally consistent: every stored pruning decision is what the oracle's
route() gives for the stored scores, live sets chain from one event to the next, and the stored top-K is the ranking of
the stored scores.  Guards against a damaged or hand-edited file; also prints which checks the margin rule pins."""
import json
import os

import numpy as np
import pytest

from oracle import prism_oracle as O
from paper_2510_15620_amd import workloads as W
from tests.helpers import GOLDEN_DIR, checkpoint_margins, load_fullsize_golden

CASES = [("cfg3_4b", "drop_only"), ("cfg3_4b", "three_way"), ("cfg4_8b", "drop_only"), ("cfg4_8b", "three_way"),
         ("cfg5_8b_stream", "drop_only"), ("cfg5_8b_stream", "three_way"), ("cfg4_8b", "drop_only_w4"),
         ("cfg5_8b_stream", "drop_only_w4")]


@pytest.mark.parametrize("workload,mode", CASES)
def test_stored_oracle_run_is_self_consistent(workload, mode):
    g = load_fullsize_golden(workload, mode)
    w = W.WORKLOADS[workload]
    assert (g.K, g.n_cands, g.n_clusters, g.tau, g.checkpoints) == (w.K, w.n_cands, w.n_clusters, w.cv_threshold, list(w.checkpoints))
    omode = O.MODE_DROP_ONLY if mode.startswith("drop_only") else O.MODE_THREE_WAY
    live = np.arange(w.n_cands)
    K_rem, early, early_scores, lens = w.K, [], [], (W.doc_lengths(w) + w.query_len)
    token_layers, prev_layer = 0, 0
    pinned = []
    for ev in g.events:
        assert np.array_equal(ev.live, live), ev.layer
        token_layers += int(lens[live].sum()) * (ev.layer - prev_layer)
        prev_layer = ev.layer
        if ev.fate is None:                                   # final scoring
            assert ev.layer == w.model.n_layers and ev is g.events[-1]
            break
        assert ev.layer in w.checkpoints and len(live) > K_rem
        r = O.route(ev.scores, K_rem, w.n_clusters, w.cv_threshold)
        assert np.array_equal(r.fate, ev.fate) and r.gate == ev.gate and r.pruned == ev.pruned
        keep = O.keep_mask(r, omode) if r.pruned else np.ones(len(live), bool)
        assert np.array_equal(keep, ev.keep)
        pinned.append((ev.layer, checkpoint_margins(ev.scores, K_rem, w.n_clusters, w.cv_threshold, 2e-2)["pinned"]))
        if omode == O.MODE_THREE_WAY and r.pruned:
            sel = [i for i in O.rank_order(ev.scores) if ev.fate[i] == O.SELECTED]
            early += [int(live[i]) for i in sel]
            early_scores += [float(ev.scores[i]) for i in sel]
            K_rem -= len(sel)
            if r.terminate:
                d = np.where(keep)[0]
                o = O.rank_order(ev.scores[d])[:K_rem]
                early += [int(live[d][i]) for i in o]
                early_scores += [float(ev.scores[d][i]) for i in o]
                live = live[keep]
                K_rem = 0
                break
        live = live[keep]
    if K_rem:
        fin = g.events[-1]
        o = O.rank_order(fin.scores)[:K_rem]
        early += [int(fin.live[i]) for i in o]
        early_scores += [float(fin.scores[i]) for i in o]
    assert g.idx.tolist() == early and g.scores.tolist() == early_scores
    assert g.token_layers == token_layers and g.layers_run == prev_layer
    print(f"{workload} {mode}: checks (layer, pinned by the 2e-2 margins) {pinned}; live sizes {[len(e.live) for e in g.events]}")


def test_half_operand_noise_file_agrees_with_the_complete_run():
    """tests/golden/half_operand_noise_cfg5_8b_stream_w4.json (three candidates forwarded alone, exact and with half operands):
    its exact scores are the complete run's final scores of those candidates - the oracle forwards every candidate on
    its own (Sec. 3.3), so the pool around it changes nothing - and half operands alone move each by less than the 2e-2 bar."""
    d = json.load(open(os.path.join(GOLDEN_DIR, "half_operand_noise_cfg5_8b_stream_w4.json")))
    fin = load_fullsize_golden(d["workload"], "drop_only_w4").events[-1]
    for c, e, h in zip(d["cands"], d["exact"], d["half"]):
        i = int(np.where(fin.live == c)[0][0])
        assert abs(float(e) - fin.scores[i]) <= 1e-12
        assert 0 < abs(float(h) - float(e)) <= 2e-2
