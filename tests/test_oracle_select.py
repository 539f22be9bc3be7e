"""Whole-path invariants of the oracle on small seeded workloads (CPU only)."""
import numpy as np
import pytest

from oracle import prism_oracle as O
from paper_2510_15620_amd import workloads as W
from tests.helpers import oracle_model, oracle_select, oracle_weights


@pytest.fixture(scope="module")
def tiny():
    w = W.WORKLOADS["cfg1_tiny"]
    wt = W.make_weights(w)
    return w, wt, W.make_tokens(w)


def _full_depth_scores(w, wt, tokens):
    q, cands = tokens
    ow, om = oracle_weights(wt), oracle_model(w.model)
    return np.array([O.score_trajectory(q, c, ow, om, [w.model.n_layers])[w.model.n_layers] for c in cands])


def test_no_pruning_topk_is_the_full_depth_ranking(tiny):
    w, wt, tokens = tiny
    full = _full_depth_scores(w, wt, tokens)
    sel = oracle_select(w, wt, tokens, mode=O.MODE_NO_PRUNING)
    order = O.rank_order(full)[:w.K]
    assert list(sel.idx) == list(order)
    assert np.allclose(sel.scores, full[order], atol=1e-12)
    assert len(sel.events) == 1 and sel.events[0].layer == w.model.n_layers


def test_drop_only_survivors_keep_their_full_depth_scores(tiny):
    """Sequences never interact (Sec. 2.2), so a survivor's final score is what the unpruned
    model gives it (Sec. 7: contenders undergo full inference)."""
    w, wt, tokens = tiny
    full = _full_depth_scores(w, wt, tokens)
    sel = oracle_select(w, wt, tokens)
    ev = sel.events[0]
    assert ev.layer == 1 and ev.pruned and 0 < ev.keep.sum() < w.n_cands      # the case really prunes
    final = sel.events[-1]
    assert list(final.live) == [c for c, k in zip(ev.live, ev.keep) if k]
    assert np.array_equal(final.scores, full[final.live])
    assert list(sel.idx) == [final.live[i] for i in O.rank_order(final.scores)[:w.K]]
    # work accounting: dropped candidates do not run layer 2
    lens = np.array([w.query_len + len(c) for c in tokens[1]])
    assert sel.token_layers == lens.sum() + lens[final.live].sum()


def test_candidate_permutation_permutes_outputs_only(tiny):
    w, wt, (q, cands) = tiny
    base = oracle_select(w, wt, (q, cands))
    perm = np.random.default_rng(0).permutation(len(cands))
    sel = oracle_select(w, wt, (q, [cands[p] for p in perm]))
    assert set(perm[sel.idx]) == set(base.idx)
    assert np.allclose(np.sort(sel.scores), np.sort(base.scores), atol=1e-12)
    assert set(perm[sel.events[-1].live]) == set(base.events[-1].live)


def test_duplicates_single_candidate_and_k_ge_n(tiny):
    w, wt, (q, cands) = tiny
    sel = oracle_select(w, wt, (q, [cands[0], cands[1], cands[0]]), K=3)
    s = dict(zip(sel.idx, sel.scores))
    assert s[0] == s[2] and list(sel.idx).index(0) < list(sel.idx).index(2)   # tie: lower index first
    one = oracle_select(w, wt, (q, [cands[3]]), K=1)
    assert list(one.idx) == [0] and len(one.events) == 1
    alln = oracle_select(w, wt, (q, cands), K=50)                             # K >= N: no pruning, all sorted
    assert len(alln.idx) == len(cands) and len(alln.events) == 1
    assert np.all(np.diff(alln.scores) <= 0)


def test_three_way_mode_stops_early_and_orders_groups():
    """Three-way routing (Sec. 4.1): selected leave with their exit-time score, deferred run on,
    and the forward ends when the deferred set fills the remaining slots."""
    w = W.WORKLOADS["mini_fp32"]
    wt, tokens = W.make_weights(w), W.make_tokens(w)
    sel = oracle_select(w, wt, tokens, mode=O.MODE_THREE_WAY, K=4)
    assert len(sel.idx) == 4 and len(set(sel.idx)) == 4
    n_sel = 0
    for ev in sel.events:
        if ev.pruned:
            picked = [ev.live[i] for i in O.rank_order(ev.scores) if ev.fate[i] == O.SELECTED]
            assert list(sel.idx[n_sel:n_sel + len(picked)]) == picked
            n_sel += len(picked)
    # every returned candidate was selected early or survived to the end
    last = sel.events[-1]
    tail = set(last.live if not last.pruned else last.live[last.keep])
    assert set(sel.idx[n_sel:]) <= tail


def test_workload_shapes_match_the_benchmark_configs():
    for name, w in W.WORKLOADS.items():
        lens = W.doc_lengths(w)
        assert len(lens) == w.n_cands and lens.min() >= 1
    assert (W.doc_lengths(W.WORKLOADS["cfg4_8b"]) + 64 == 1024).all()
    l5 = W.doc_lengths(W.WORKLOADS["cfg5_8b_stream"])
    assert l5.min() >= 32 and l5.max() <= 2048 and 330 < np.median(l5) < 480
    l2 = W.doc_lengths(W.WORKLOADS["cfg2_0p6b"])
    assert l2.min() >= 128 and l2.max() <= 480
    m = W.WORKLOADS["cfg4_8b"].model
    assert abs(m.gemm_flops_per_token_layer() / 1e6 - 385.9) < 0.1          # flops per live token per layer
    assert abs(W.WORKLOADS["cfg2_0p6b"].model.gemm_flops_per_token_layer() / 2 / 1e6 - 15.7) < 0.1


def test_generator_is_counter_based_and_gaussian():
    a = W.gaussian(0, "t", (1000, 64), 0.0, 0.02, __import__("torch").float32)
    b = W.gaussian(0, "t", (1000, 64), 0.0, 0.02, __import__("torch").float32, block=777)
    assert (a == b).all()                                                   # independent of blocking
    assert abs(float(a.std()) - 0.02) < 3e-4 and abs(float(a.mean())) < 3e-4
    c = W.gaussian(1, "t", (1000, 64), 0.0, 0.02, __import__("torch").float32)
    assert not (a == c).all()
