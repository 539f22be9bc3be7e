"""Properties of the oracle's pruning rule (Sec. 4.1: dispersion gate, clustering of the scores, routing around the
cluster that holds the K-th ranked candidate) that hold for any input, checked on generated score vectors.  Scores are
small integers over a power of two, so that scaling by a power of two, shifting by an integer and permuting are exact
in floating point and "the same partition" can be demanded literally."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle import prism_oracle as O

scores_st = st.lists(st.integers(-400, 400), min_size=2, max_size=40).map(lambda v: np.array(v, np.float64) / 16.0)


@settings(max_examples=300, deadline=None, derandomize=True)
@given(scores_st, st.integers(1, 12), st.integers(2, 6))
def test_fates_are_monotone_in_the_score_and_the_top_k_is_never_dropped(s, K, k):
    r = O.route(s, K, k, 0.0)
    if not r.pruned:
        assert len(s) <= K or len(set(s.tolist())) == 1 or not r.gate
        return
    order = O.rank_order(s)
    # a better score never gets a worse fate, equal scores get equal fates
    f = r.fate[order]
    assert all(f[i] >= f[i + 1] for i in range(len(f) - 1))
    for i in range(len(s)):
        for j in range(len(s)):
            if s[i] == s[j]:
                assert r.fate[i] == r.fate[j]
    # the K best are kept in both modes' union (selected or deferred), and the K-th ranked one is deferred
    assert (r.fate[order[:K]] != O.DROPPED).all()
    assert r.fate[order[K - 1]] == O.DEFERRED
    # selected candidates alone never fill the K slots (the boundary cluster still has to be resolved)
    assert int((r.fate == O.SELECTED).sum()) < K
    # clusters are numbered best first and are contiguous in rank order
    c = r.cluster[order]
    assert all(c[i] <= c[i + 1] for i in range(len(c) - 1)) and c[0] == 0 and c[-1] == r.n_clusters - 1


@settings(max_examples=200, deadline=None, derandomize=True)
@given(scores_st, st.integers(1, 12), st.integers(2, 6), st.integers(-3, 3), st.integers(-50, 50), st.randoms(use_true_random=False))
def test_partition_is_invariant_under_scaling_shifting_and_permuting(s, K, k, e, shift, rnd):
    r = O.route(s, K, k, 0.0)
    # tau = 0: the gate only asks for std > 0, which scaling and shifting keep
    r2 = O.route(s * 2.0 ** e + shift, K, k, 0.0)
    assert r.pruned == r2.pruned
    if r.pruned:
        assert np.array_equal(r.fate, r2.fate) and np.array_equal(r.cluster, r2.cluster)
    perm = list(range(len(s)))
    rnd.shuffle(perm)
    perm = np.array(perm)
    r3 = O.route(s[perm], K, k, 0.0)
    assert r.pruned == r3.pruned
    if r.pruned:
        assert np.array_equal(r.fate[perm], r3.fate) and np.array_equal(r.cluster[perm], r3.cluster)


@settings(max_examples=200, deadline=None, derandomize=True)
@given(scores_st, st.integers(2, 6))
def test_splits_minimise_the_within_cluster_cost_among_neighbouring_splits(s, k):
    """Moving any single split position by one never lowers the cost (a necessary condition of the optimum that does not
    share the oracle's recurrence)."""
    ranked = np.sort(s)[::-1]
    k = min(k, len(set(ranked.tolist())))
    if k < 2:
        return
    splits = O.kmeans_1d_splits(ranked, k)

    def cost(sp):
        b = [0] + list(sp) + [len(ranked)]
        return sum(float(((ranked[a:z] - ranked[a:z].mean()) ** 2).sum()) for a, z in zip(b[:-1], b[1:]))
    assert len(splits) == k - 1 and all(0 < a < len(ranked) for a in splits) and list(splits) == sorted(set(splits))
    best = cost(splits)
    for i in range(len(splits)):
        for d in (-1, 1):
            sp = list(splits)
            sp[i] += d
            if 0 < sp[i] < len(ranked) and sp == sorted(set(sp)):
                assert cost(sp) >= best - 1e-9
