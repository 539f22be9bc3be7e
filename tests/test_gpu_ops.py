"""Parity of each HIP kernel with the oracle's function for the same step, element by element, on
seeded inputs spanning several tiles and ragged tails.  All calls go through the C ABI."""
import math

import numpy as np
import pytest
import torch

from oracle import prism_oracle as O
from paper_2510_15620_amd import binding as B

pytestmark = pytest.mark.gpu

DEV = "cuda"


def _rand(shape, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    return (torch.randn(*shape, generator=g) * scale).to(dtype)


def _f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def _tol(dtype):
    return dict(rtol=2e-5, atol=2e-5) if dtype == torch.float32 else dict(rtol=1.2e-2, atol=1e-2)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_embed(dtype):
    table = _rand((300, 256), dtype, 1)
    tok = torch.randint(0, 300, (777,), generator=torch.Generator().manual_seed(2), dtype=torch.int32)
    X = torch.empty(777, 256, dtype=torch.float32, device=DEV)
    B.op_embed(tok.to(DEV), table.to(DEV), X)
    assert np.array_equal(X.cpu().numpy().astype(np.float64), O.embed(tok.numpy(), _f64(table)))


@pytest.mark.parametrize("dtype,hidden", [(torch.float32, 256), (torch.float32, 192), (torch.bfloat16, 4096), (torch.bfloat16, 512)])
def test_rmsnorm(dtype, hidden):
    X = _rand((333, hidden), torch.float32, 3, 2.5)
    g = (1 + _rand((hidden,), torch.float32, 4, 0.1)).to(dtype)
    out = torch.empty(333, hidden, dtype=dtype, device=DEV)
    B.op_rmsnorm(X.to(DEV), g.to(DEV), 1e-6, out)
    ref = O.rmsnorm(_f64(X), _f64(g), 1e-6)
    tol = dict(rtol=1e-5, atol=1e-6) if dtype == torch.float32 else dict(rtol=2 ** -8, atol=1e-6)
    np.testing.assert_allclose(_f64(out), ref, **tol)


GEMM_SHAPES = [  # M, N (rows of W), K
    (1, 64, 64), (77, 200, 128), (300, 384, 256), (513, 1024, 192), (1000, 2560, 1408), (4100, 6144, 1024),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
@pytest.mark.parametrize("shape", GEMM_SHAPES)
def test_gemm(dtype, epi, shape):
    M, N, K = shape
    if dtype == torch.float32:
        K += 3; N += 2                                   # the fp32 kernel takes any shape
    A = _rand((M, K), dtype, 10 + M, 1.0)
    Wt = _rand((N, K), dtype, 20 + N, 1.0 / math.sqrt(K))
    ref = _f64(A) @ _f64(Wt).T
    if epi == B.EPI_STORE:
        out = torch.zeros(M, N, dtype=dtype, device=DEV)
    elif epi == B.EPI_RESIDUAL:
        X0 = _rand((M, N), torch.float32, 30, 1.0)
        out = X0.to(DEV).clone()
        ref = _f64(X0) + ref
    else:
        F = N // 2
        out = torch.zeros(M, F, dtype=dtype, device=DEV)
        ref = O.silu(ref[:, :F]) * ref[:, F:]
    B.op_gemm(epi, A.to(DEV), Wt.to(DEV), out)
    torch.cuda.synchronize()
    if dtype == torch.float32:
        np.testing.assert_allclose(_f64(out), ref, rtol=1e-4, atol=1e-4)
    elif epi == B.EPI_RESIDUAL:
        np.testing.assert_allclose(_f64(out), ref, rtol=1e-4, atol=1e-4)       # fp32 accumulate, fp32 out
    else:
        np.testing.assert_allclose(_f64(out), ref, rtol=2 ** -8, atol=2e-3)    # one bf16 rounding of the result


@pytest.mark.parametrize("dtype,nq,nkv,hd", [(torch.float32, 4, 2, 64), (torch.float32, 6, 3, 32), (torch.bfloat16, 8, 2, 128)])
@pytest.mark.parametrize("qk_norm", [True, False])
def test_qknorm_rope(dtype, nq, nkv, hd, qk_norm):
    lens = [5, 130, 1, 64, 299]
    T = sum(lens)
    pos = np.concatenate([np.arange(l) for l in lens]).astype(np.int32)
    QKV = _rand((T, (nq + 2 * nkv) * hd), dtype, 40, 1.5)
    gq, gk = (1 + _rand((hd,), torch.float32, 41, 0.1)).to(dtype), (1 + _rand((hd,), torch.float32, 42, 0.1)).to(dtype)
    d = QKV.to(DEV).clone()
    B.op_qknorm_rope(d, torch.from_numpy(pos).to(DEV), 512, gq.to(DEV), gk.to(DEV), nq, nkv, hd, 1e-6, 1e6, qk_norm)
    x = _f64(QKV).reshape(T, nq + 2 * nkv, hd)
    q, k, v = x[:, :nq], x[:, nq:nq + nkv], x[:, nq + nkv:]
    if qk_norm:
        q, k = O.rmsnorm(q, _f64(gq), 1e-6), O.rmsnorm(k, _f64(gk), 1e-6)
    ref = np.concatenate([O.rope(q, pos, 1e6), O.rope(k, pos, 1e6), v], axis=1).reshape(T, -1)
    tol = dict(rtol=1e-5, atol=2e-5) if dtype == torch.float32 else dict(rtol=2 ** -7, atol=2e-2)
    np.testing.assert_allclose(_f64(d), ref, **tol)
    assert np.array_equal(_f64(d).reshape(T, -1, hd)[:, nq + nkv:], v)          # v untouched


ATTN_CASES = [
    (torch.float32, 4, 2, 64, [1, 17, 64, 100]),
    (torch.float32, 6, 3, 32, [33, 2]),
    (torch.bfloat16, 8, 2, 128, [1, 63, 64, 65, 130, 300]),      # G = 4
    (torch.bfloat16, 16, 8, 128, [200, 129, 31]),                # G = 2
    (torch.bfloat16, 8, 8, 128, [257, 5]),                       # G = 1
    (torch.bfloat16, 8, 1, 128, [97, 32]),                       # G = 8
]


@pytest.mark.parametrize("dtype,nq,nkv,hd,lens", ATTN_CASES)
def test_attention(dtype, nq, nkv, hd, lens):
    T = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    QKV = _rand((T, (nq + 2 * nkv) * hd), dtype, 50 + T, 1.0)
    out = torch.zeros(T, nq * hd, dtype=dtype, device=DEV)
    B.op_attention(QKV.to(DEV), cu, nq, nkv, hd, out)
    x = _f64(QKV).reshape(T, nq + 2 * nkv, hd)
    ref = np.concatenate([O.causal_gqa_attention(x[a:b, :nq], x[a:b, nq:nq + nkv], x[a:b, nq + nkv:]).reshape(b - a, -1)
                          for a, b in zip(cu[:-1], cu[1:])])
    tol = dict(rtol=1e-4, atol=1e-5) if dtype == torch.float32 else dict(rtol=2e-2, atol=1.5e-2)
    np.testing.assert_allclose(_f64(out), ref, **tol)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_score(dtype):
    H, T = 1024, 500
    X = _rand((T, H), torch.float32, 60, 3.0)
    g = (1 + _rand((H,), torch.float32, 61, 0.05)).to(dtype)
    wy, wn = _rand((H,), dtype, 62, 0.02), _rand((H,), dtype, 63, 0.02)
    rows = np.array([0, 17, 499, 250, 17], np.int32)
    s = torch.zeros(len(rows), dtype=torch.float32, device=DEV)
    B.op_score(X.to(DEV), torch.from_numpy(rows).to(DEV), g.to(DEV), wy.to(DEV), wn.to(DEV), 1e-6, s)
    ref = [O.head_score(_f64(X)[r], _f64(g), _f64(wy), _f64(wn), 1e-6) for r in rows]
    np.testing.assert_allclose(_f64(s), ref, rtol=1e-5, atol=2e-6)


def _route_case(scores, K, k, tau):
    s = torch.tensor(scores, dtype=torch.float32)
    fate = torch.full((len(scores),), 9, dtype=torch.int8, device=DEV)
    stats = torch.zeros(4, dtype=torch.float64, device=DEV)
    B.op_route(s.to(DEV), K, k, tau, fate, stats)
    r = O.route(s.numpy().astype(np.float64), K, k, float(np.float32(tau)))
    st = stats.cpu().numpy()
    assert np.array_equal(fate.cpu().numpy(), r.fate), (scores[:8], K, k, tau)
    assert st[0] == r.mean and st[1] == r.std and bool(st[2]) == r.gate and int(st[3]) == r.n_clusters


def test_route_hand_cases_and_degenerate_inputs():
    _route_case([0.1, 5.0, 0.2, 9.0, 5.1, 0.0, 4.9], 2, 3, 0.0)
    _route_case([0.1, 5.0, 0.2, 9.0, 5.1, 0.0, 4.9], 5, 3, 0.0)
    _route_case([1.0, 2.0, 3.0], 3, 3, 0.0)                # n <= K
    _route_case([4.0, 4.0, 4.0, 4.0], 2, 3, 0.0)           # one distinct value
    _route_case([4.0, 4.0, 1.0, 1.0, 1.0], 1, 3, 0.0)      # two distinct values, k = 3
    _route_case([2.0, 1.0, 0.0], 1, 2, 0.0)                # SSE tie between the two splits
    _route_case([1, 2, 3, 4], 2, 3, 0.45)                  # gate closed
    _route_case([1, 2, 3, 4], 2, 3, 0.44)                  # gate open
    _route_case([5.0], 1, 3, 0.0)


@pytest.mark.parametrize("seed", range(12))
def test_route_random_matches_oracle_bit_for_bit(seed):
    r = np.random.default_rng(seed)
    n = int(r.choice([4, 9, 40, 100, 257, 500]))
    k = int(r.integers(2, 6))
    K = int(r.integers(1, n))
    s = r.normal(size=n) * r.choice([0.3, 1.0, 3.0]) + r.choice([0.0, 2.0])
    if seed % 3 == 0:
        s = np.round(s, 1)                                 # many exact duplicates
    _route_case(s.astype(np.float32).tolist(), K, k, float(r.choice([0.0, 0.5])))


def test_route_large_n():
    r = np.random.default_rng(99)
    _route_case(r.normal(size=1500).astype(np.float32).tolist(), 20, 3, 0.0)


def test_compact_and_topk():
    H = 512
    lens = np.array([5, 130, 1, 64, 299, 40], np.int32)
    start = np.concatenate([[0], np.cumsum(lens)])[:-1].astype(np.int32)
    X = _rand((int(lens.sum()), H), torch.float32, 70)
    keep = np.array([1, 0, 1, 1, 0, 1], bool)
    kl = lens[keep]
    dst = np.concatenate([[0], np.cumsum(kl)])[:-1].astype(np.int32)
    Xd = torch.full((int(kl.sum()) + 3, H), 7.0, dtype=torch.float32, device=DEV)
    T = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    B.op_compact(X.to(DEV), Xd, T(start[keep]), T(dst), T(kl))
    ref = np.concatenate([X.numpy()[s:s + l] for s, l in zip(start[keep], kl)])
    assert np.array_equal(Xd.cpu().numpy()[:len(ref)], ref) and (Xd.cpu().numpy()[len(ref):] == 7.0).all()

    s = np.array([0.5, 2.0, -1.0, 2.0, 0.5, 3.5, 2.0], np.float32)
    pos = torch.zeros(4, dtype=torch.int32, device=DEV)
    sc = torch.zeros(4, dtype=torch.float32, device=DEV)
    B.op_topk(T(s), 4, pos, sc)
    order = O.rank_order(s.astype(np.float64))[:4]
    assert pos.cpu().numpy().tolist() == order.tolist() == [5, 1, 3, 6]
    assert np.array_equal(sc.cpu().numpy(), s[order])
