"""Pins for the oracle's pruning rule (Sec. 4.1, Sec. 4.5): closed forms, brute force, the
paper's worked-example counts.  CPU only."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import prism_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_cv_closed_form():
    # {1,2,3,4}: mean 2.5, population variance 1.25
    assert abs(O.coefficient_of_variation([1, 2, 3, 4]) - math.sqrt(1.25) / 2.5) < 1e-15
    assert abs(O.coefficient_of_variation([1, 2, 3, 4]) - 0.4472135955) < 1e-9
    assert abs(O.coefficient_of_variation([-1, -2, -3, -4]) - 0.4472135955) < 1e-9   # absolute value


def test_gate_branches():
    assert O.gate_open([1, 2, 3, 4], 0.44) and not O.gate_open([1, 2, 3, 4], 0.45)
    assert not O.gate_open([2.5, 2.5, 2.5], 0.0)             # no dispersion: nothing to separate
    assert O.gate_open([-1.0, 1.0], 100.0)                   # mean 0, std > 0: CV is infinite
    assert O.gate_open([1, 2, 3, 4], 0.0)


def test_rank_order_ties_prefer_lower_index():
    assert list(O.rank_order([1.0, 3.0, 3.0, 2.0, 3.0])) == [1, 2, 4, 3, 0]


def _sse(groups):
    return sum(sum((x - sum(g) / len(g)) ** 2 for x in g) for g in groups if g)


def _splits_to_groups(x, splits):
    b = [0] + list(splits) + [len(x)]
    return [list(x[b[i]:b[i + 1]]) for i in range(len(b) - 1)]


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("k", [2, 3, 4])
def test_kmeans_matches_brute_force_over_contiguous_splits(seed, k):
    r = np.random.default_rng(seed)
    n = int(r.integers(k, 13))
    x = np.sort(r.normal(size=n) * (1 + 3 * (r.random(n) > 0.5)))[::-1]
    best = min(itertools.combinations(range(1, n), k - 1), key=lambda s: (round(_sse(_splits_to_groups(x, s)), 12), s))
    got = O.kmeans_1d_splits(x, k)
    assert abs(_sse(_splits_to_groups(x, got)) - _sse(_splits_to_groups(x, best))) < 1e-10
    assert tuple(got) == best


@pytest.mark.parametrize("seed", range(4))
def test_contiguous_optimum_is_the_global_kmeans_optimum(seed):
    """All k^n labelings for n <= 8: no non-contiguous clustering has a lower SSE."""
    r = np.random.default_rng(100 + seed)
    n, k = 8, 3
    x = np.sort(r.normal(size=n))[::-1]
    best = math.inf
    for lab in itertools.product(range(k), repeat=n):
        if len(set(lab)) < k:
            continue
        best = min(best, _sse([[x[i] for i in range(n) if lab[i] == c] for c in range(k)]))
    got = _sse(_splits_to_groups(x, O.kmeans_1d_splits(x, k)))
    assert abs(got - best) < 1e-12


@pytest.mark.parametrize("seed,n,spread", [(0, 200, 50), (1, 237, 9), (2, 160, 3), (3, 64, 1)])
def test_kmeans_at_working_sizes_against_exact_rational_enumeration(seed, n, spread):
    """k = 3 at the pool sizes the checks run at (hundreds of scores, many exact duplicates): every one of the
    C(n-1, 2) contiguous partitions is costed in exact rational arithmetic from integer scores (within-cluster sum of
    squares = sum x^2 - (sum x)^2 / size), the minimum taken, and among exactly tied partitions the lexicographically
    smallest pair of split positions.  Integer scores keep the oracle's fp64 prefix sums exact, so its tie rule is
    exercised on true ties."""
    from fractions import Fraction
    r = np.random.default_rng(100 + seed)
    x = np.sort(r.integers(-spread, spread + 1, size=n))[::-1].astype(np.int64)      # rank order: descending
    P = [0] * (n + 1)
    Q = [0] * (n + 1)
    for i, v in enumerate(x):
        P[i + 1] = P[i] + int(v)
        Q[i + 1] = Q[i] + int(v) * int(v)
    cost = lambda i, j: Fraction(Q[j] - Q[i]) - Fraction((P[j] - P[i]) ** 2, j - i)
    head = [cost(0, s) for s in range(n + 1) if s > 0]                                # head[s - 1] = cost(0, s)
    tail = [cost(s, n) for s in range(n)]                                             # tail[s] = cost(s, n)
    best, best_splits = None, None
    for s1 in range(1, n - 1):
        for s2 in range(s1 + 1, n):
            c = head[s1 - 1] + cost(s1, s2) + tail[s2]
            if best is None or c < best:                                              # strict: the first (smallest) pair wins ties
                best, best_splits = c, [s1, s2]
    assert O.kmeans_1d_splits(x.astype(np.float64), 3) == best_splits


def test_kmeans_two_blobs_split_at_the_gap_and_tie_rule():
    x = np.array([10.2, 10.1, 9.9, 9.8, 1.2, 1.0, 0.9])
    assert O.kmeans_1d_splits(x, 2) == [4]
    # {2 | 1 0} and {2 1 | 0} have the same SSE: smallest split position wins
    assert O.kmeans_1d_splits(np.array([2.0, 1.0, 0.0]), 2) == [1]
    assert O.kmeans_1d_splits(np.array([5.0, 4.0, 3.0]), 3) == [1, 2]
    assert O.kmeans_1d_splits(np.array([5.0, 4.0, 3.0]), 1) == []


def test_kmeans_agrees_with_library_lloyd_on_separated_data():
    """Special case where an iterative library K-Means reaches the optimum: three far-apart blobs."""
    from sklearn.cluster import KMeans
    r = np.random.default_rng(7)
    x = np.concatenate([r.normal(8, .3, 5), r.normal(0, .3, 9), r.normal(-7, .3, 6)])
    x = np.sort(x)[::-1]
    lab = KMeans(3, n_init=10, random_state=0).fit(x[:, None]).labels_
    lib_splits = [i for i in range(1, len(x)) if lab[i] != lab[i - 1]]
    assert O.kmeans_1d_splits(x, 3) == lib_splits == [5, 14]


def _golden_events():
    out = []
    for line in open(os.path.join(GOLDEN, "working_example_sec4_5.txt")):
        if line.startswith("#") or not line.strip():
            continue
        name, k, tau, scores, counts, gate, term = [f.strip() for f in line.split("|")]
        out.append((name, int(k), float(tau), [float(s) for s in scores.split()],
                    [int(c) for c in counts.split()], bool(int(gate)), bool(int(term))))
    return out


@pytest.mark.parametrize("ev", _golden_events(), ids=lambda e: e[0])
def test_paper_worked_example_counts(ev):
    name, K_rem, tau, scores, (n_sel, n_def, n_drop), gate, term = ev
    r = O.route(scores, K_rem, 3, tau)
    assert r.gate == gate
    assert int((r.fate == O.SELECTED).sum()) == n_sel
    assert int((r.fate == O.DEFERRED).sum()) == n_def
    assert int((r.fate == O.DROPPED).sum()) == n_drop
    assert (r.terminate and r.pruned) == term
    # drop-only keeps selected + deferred, three-way keeps only deferred
    assert int(O.keep_mask(r, O.MODE_DROP_ONLY).sum()) == n_sel + n_def
    assert int(O.keep_mask(r, O.MODE_THREE_WAY).sum()) == n_def


def test_route_fates_follow_cluster_means_and_rank():
    s = [0.1, 5.0, 0.2, 9.0, 5.1, 0.0, 4.9]
    r = O.route(s, 2, 3, 0.0)                    # rank 2 is 5.1 -> boundary = {5.1, 5.0, 4.9}
    assert list(r.fate) == [O.DROPPED, O.DEFERRED, O.DROPPED, O.SELECTED, O.DEFERRED, O.DROPPED, O.DEFERRED]
    assert list(r.cluster) == [2, 1, 2, 0, 1, 2, 1]
    r = O.route(s, 1, 3, 0.0)                    # rank 1 is in the top cluster: nothing is selected
    assert (r.fate == O.SELECTED).sum() == 0 and (r.fate == O.DEFERRED).sum() == 1
    r = O.route(s, 5, 3, 0.0)                    # boundary is the lowest cluster: nothing dropped
    assert (r.fate == O.DROPPED).sum() == 0 and (r.fate == O.SELECTED).sum() == 4


def test_route_degenerate_cases():
    assert not O.route([1.0, 2.0, 3.0], 3, 3, 0.0).pruned          # n_live <= K: nothing may be dropped
    assert not O.route([4.0, 4.0, 4.0, 4.0], 2, 3, 0.0).pruned     # a single distinct score
    r = O.route([4.0, 4.0, 1.0, 1.0, 1.0], 1, 3, 0.0)              # two distinct scores -> two clusters
    assert r.pruned and r.n_clusters == 2 and list(r.fate) == [1, 1, 0, 0, 0]
    # a planted mistake must be caught: K-th rank is 1-indexed (K = 2 of [9 | 5 5 | 1]) -> 9 selected
    assert list(O.route([9.0, 5.0, 5.1, 1.0], 2, 3, 0.0).fate) == [O.SELECTED, O.DEFERRED, O.DEFERRED, O.DROPPED]


def test_gamma_formula():
    a = [1, 2, 3, 4]
    assert O.goodman_kruskal_gamma(a, [10, 20, 30, 40]) == 1.0
    assert O.goodman_kruskal_gamma(a, [4, 3, 2, 1]) == -1.0
    # pairs: 6; swapping the two middle ones reverses exactly one pair -> (5 - 1) / 6
    assert abs(O.goodman_kruskal_gamma(a, [1, 3, 2, 4]) - 4 / 6) < 1e-15


# ---- embedding-table cache (Sec. 4.4): the oracle's LRU against hand-worked traces and what any LRU must satisfy

def test_lru_hand_worked_trace():
    c = O.LruRowCache(2)
    # 1 miss, 2 miss, 1 hit (2 is now the oldest), 3 miss evicts 2, 2 miss evicts 1, 3 hit
    assert [c.access(t) for t in (1, 2, 1, 3, 2, 3)] == [False, False, True, False, False, True]
    assert c.order == [2, 3]


def test_lru_invariants():
    rng = np.random.default_rng(3)
    toks = rng.integers(0, 40, size=500).tolist()
    # capacity >= distinct tokens: one miss per distinct token
    assert O.LruRowCache(40).run(toks) == (500 - len(set(toks)), len(set(toks)))
    # capacity 1: a hit only when a token repeats immediately
    rep = sum(a == b for a, b in zip(toks[:-1], toks[1:]))
    assert O.LruRowCache(1).run(toks) == (rep, 500 - rep)
    # inclusion property of LRU: a larger cache never misses more
    misses = [O.LruRowCache(k).run(toks)[1] for k in (1, 2, 5, 10, 20, 40)]
    assert misses == sorted(misses, reverse=True)
    # brute force against the definition: hit iff fewer than `capacity` distinct other tokens since the last use
    cap = 7
    c = O.LruRowCache(cap)
    for i, t in enumerate(toks):
        prev = max((j for j in range(i) if toks[j] == t), default=None)
        expect = prev is not None and len(set(toks[prev + 1:i])) < cap
        assert c.access(t) == expect
    # state carries over between requests
    c2 = O.LruRowCache(3)
    c2.run([5, 6, 7])
    # 7, 6, 5 hit (5 newest); 8 evicts 7, the oldest; 7 misses again
    assert c2.run([7, 6, 5, 8, 7]) == (3, 2)


# ---- 4-bit weights (Sec. 6, the quantised variant): the oracle's quantiser against a hand-worked group and its invariants

def test_w4_hand_worked_group():
    w = np.zeros((1, 128), np.float32)
    w[0, :5] = [0.7, -0.35, 0.1, -0.05, 0.0499]
    codes, scales = O.quantize_w4(w)
    # 0.7 / 7 = 0.1 -> bf16 0.10009765625 (0x3DCD); 0.7 / s = 6.993 -> 7; -0.35 / s = -3.4966 -> -3; 0.1 / s = 0.999 -> 1;
    # -0.05 / s = -0.4995 -> 0; 0.0499 / s = 0.4985 -> 0
    assert scales.shape == (1, 1) and float(scales[0, 0]) == 0.10009765625
    assert codes[0, :5].tolist() == [7, -3, 1, 0, 0] and not codes[0, 5:].any()
    back = O.dequantize_w4(codes, scales)
    assert back[0, :3].tolist() == [7 * 0.10009765625, -3 * 0.10009765625, 0.10009765625]


def test_w4_invariants():
    rng = np.random.default_rng(11)
    w = O.round_operand(rng.normal(0, 0.02, size=(24, 512)), "bf16").astype(np.float32)
    w[3, 128:256] = 0                                         # an all-zero group
    codes, scales = O.quantize_w4(w)
    assert codes.min() >= -7 and codes.max() <= 7
    assert np.all(scales > 0) and np.array_equal(O.round_operand(scales, "bf16"), scales.astype(np.float64))
    assert float(scales[3, 1]) == 1.0 and not codes[3, 128:256].any()
    back = O.dequantize_w4(codes, scales)
    # nearest code: the error is at most half a step, except where the largest element was clamped to +-7
    err = np.abs(back - w).reshape(24, 4, 128)
    step = scales[:, :, None].astype(np.float64)
    assert np.all(err <= 0.5 * step * (1 + 2 ** -20) + np.abs(w).reshape(24, 4, 128) * 2 ** -7)
    # the largest element of every non-zero group sits on the outermost code
    amax = np.argmax(np.abs(w).reshape(24, 4, 128), axis=2)
    top = np.take_along_axis(codes.reshape(24, 4, 128), amax[:, :, None], axis=2)[:, :, 0]
    nz = np.abs(w).reshape(24, 4, 128).max(axis=2) > 0
    assert np.all(np.abs(top[nz]) == 7)
    # the dequantised weights are exact in half precision and quantise to themselves
    assert np.array_equal(back.astype(np.float16).astype(np.float64), back)
    c2, s2 = O.quantize_w4(back.astype(np.float32))
    assert np.array_equal(c2, codes) and np.array_equal(s2, scales)
