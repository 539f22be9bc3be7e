"""Edges of prism_select on the device against the oracle: the largest pool and the longest sequence the library accepts,
one more of each refused, a pool of identical candidates (every score equal: nothing may be pruned, ties go to the lower
index), a single candidate, ragged pools with one-token documents."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import prism_oracle as O
from paper_2510_15620_amd import binding as B
from paper_2510_15620_amd import workloads as W
from tests.helpers import oracle_select
from tests.test_gpu_select import check_against_oracle

pytestmark = pytest.mark.gpu
MAX_CANDS, MAX_SEQ = 4096, 8192


def _tokens(seed, lens, vocab):
    rng = np.random.default_rng(seed)
    return [rng.integers(0, vocab, size=int(l), dtype=np.int32) for l in lens]


def test_largest_pool():
    w = dataclasses.replace(W.WORKLOADS["cfg1_tiny"], K=5)
    wt = W.make_weights(w, "cuda")
    q = _tokens(1, [3], w.model.vocab)[0]
    cands = _tokens(2, np.random.default_rng(3).integers(1, 4, size=MAX_CANDS), w.model.vocab)     # 1..3 tokens each
    p = B.Prism(w.model, wt, checkpoints=w.checkpoints)
    idx, scores, rep = p.select(q, cands, w.K)
    ref = oracle_select(w, wt, (q, cands))
    check_against_oracle(w, idx, scores, rep, ref, 1e-4)
    assert rep.n_before[0] == MAX_CANDS
    with pytest.raises(B.PrismError) as e:
        p.select(q, cands + cands[:1], w.K)
    assert e.value.code == B.EINVAL
    p.destroy()


@pytest.mark.parametrize("name,tol", [("cfg1_tiny", 1e-4), ("mini_bf16", 2e-2)])
def test_longest_sequence(name, tol):
    """One candidate that fills the longest sequence exactly (no pruning with a single candidate: the check is the
    score after every layer's attention over 8192 keys), next to a one-token one."""
    w = dataclasses.replace(W.WORKLOADS[name], K=2)
    wt = W.make_weights(w, "cuda")
    q = _tokens(4, [7], w.model.vocab)[0]
    cands = _tokens(5, [MAX_SEQ - 7, 1], w.model.vocab)
    p = B.Prism(w.model, wt, checkpoints=w.checkpoints)
    idx, scores, rep = p.select(q, cands, w.K)
    ref = oracle_select(w, wt, (q, cands))
    assert idx.tolist() == ref.idx.tolist()
    assert np.max(np.abs(scores - ref.scores)) <= tol
    with pytest.raises(B.PrismError) as e:
        p.select(q, _tokens(6, [MAX_SEQ - 6], w.model.vocab), 1)
    assert e.value.code == B.EINVAL
    p.destroy()


@pytest.mark.parametrize("name", ["mini_fp32", "mini_bf16"])
def test_identical_candidates_and_single_candidate(name):
    w = W.WORKLOADS[name]
    wt = W.make_weights(w, "cuda")
    q, cands = W.make_tokens(w)
    same = [cands[0].copy() for _ in range(9)]
    p = B.Prism(w.model, wt, checkpoints=w.checkpoints)
    idx, scores, rep = p.select(q, same, 3)
    assert idx.tolist() == [0, 1, 2]                           # equal scores: lower index first
    assert np.all(scores == scores[0])                         # rows of a batch do not influence each other
    assert np.all(rep.n_after == 9) and not rep.gate.any()     # zero dispersion: the gate stays closed
    idx1, scores1, rep1 = p.select(q, same[:1], 3)             # K >= N
    assert idx1.tolist() == [0] and scores1[0] == scores[0]
    p.destroy()


def test_ragged_pool_with_one_token_documents():
    w = dataclasses.replace(W.WORKLOADS["mini_bf16"], K=3)
    wt = W.make_weights(w, "cuda")
    q = _tokens(7, [1], w.model.vocab)[0]
    cands = _tokens(8, [1, 300, 1, 63, 64, 65, 1, 129, 2, 1], w.model.vocab)
    p = B.Prism(w.model, wt, checkpoints=w.checkpoints)
    idx, scores, rep = p.select(q, cands, w.K)
    p.destroy()
    check_against_oracle(w, idx, scores, rep, oracle_select(w, wt, (q, cands)), 2e-2)
