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


SIXTEEN = [torch.bfloat16, torch.float16]
EPS16 = {torch.bfloat16: 2.0 ** -8, torch.float16: 2.0 ** -11}      # half an ulp, relative
OPERAND = {torch.bfloat16: "bf16", torch.float16: "f16"}


@pytest.mark.parametrize("dtype,hidden", [(torch.float32, 256), (torch.float32, 192), (torch.bfloat16, 4096), (torch.bfloat16, 512),
                                          (torch.float16, 4096), (torch.float16, 1024)])
def test_rmsnorm(dtype, hidden):
    X = _rand((333, hidden), torch.float32, 3, 2.5)
    g = (1 + _rand((hidden,), torch.float32, 4, 0.1)).to(dtype)
    out = torch.empty(333, hidden, dtype=dtype, device=DEV)
    B.op_rmsnorm(X.to(DEV), g.to(DEV), 1e-6, out)
    ref = O.rmsnorm(_f64(X), _f64(g), 1e-6)
    tol = dict(rtol=1e-5, atol=1e-6) if dtype == torch.float32 else dict(rtol=EPS16[dtype] * 1.01, atol=1e-6)
    np.testing.assert_allclose(_f64(out), ref, **tol)


GEMM_SHAPES = [  # M, N (rows of W), K
    (1, 64, 64), (77, 200, 128), (300, 384, 256), (513, 1024, 192), (1000, 2560, 1408), (4100, 6144, 1024),
]


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16, torch.float16])
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
        np.testing.assert_allclose(_f64(out), ref, rtol=EPS16[dtype] * 1.01, atol=2e-3 * EPS16[dtype] * 256)    # one 16-bit rounding of the result


def _gemm_16_case(dtype, epi, M, N, K):
    A = _rand((M, K), dtype, 10 + M + K, 1.0)
    Wt = _rand((N, K), dtype, 20 + N + K, 1.0 / math.sqrt(K))
    ref = _f64(A) @ _f64(Wt).T
    if epi == B.EPI_RESIDUAL:
        X0 = _rand((M, N), torch.float32, 30, 1.0)
        out = X0.to(DEV).clone()
        ref = _f64(X0) + ref
    elif epi == B.EPI_SWIGLU:
        out = torch.zeros(M, N // 2, dtype=dtype, device=DEV)
        ref = O.silu(ref[:, :N // 2]) * ref[:, N // 2:]
    else:
        out = torch.zeros(M, N, dtype=dtype, device=DEV)
    B.op_gemm(epi, A.to(DEV), Wt.to(DEV), out)
    torch.cuda.synchronize()
    if epi == B.EPI_RESIDUAL:
        np.testing.assert_allclose(_f64(out), ref, rtol=1e-4, atol=1e-4)
    else:
        np.testing.assert_allclose(_f64(out), ref, rtol=EPS16[dtype] * 1.01, atol=2e-3 * EPS16[dtype] * 256)


@pytest.mark.parametrize("dtype", SIXTEEN)
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
@pytest.mark.parametrize("K", [64, 128, 192, 320, 448])
def test_gemm_16_big_tile_with_few_and_odd_slice_counts(dtype, epi, K):
    """4100 x 6144 outputs are 17 x 24 tiles of 256 x 256 (SwiGLU: 17 x 24 of 256 x 128), enough for the launcher to pick
    the big tile, whose K loop is scheduled by hand two 64-deep slices per iteration: 1, 2, 3, 5 and 7 slices exercise
    its prologue-only, single-iteration and mid-iteration exits."""
    _gemm_16_case(dtype, epi, 4100, 6144, K)


@pytest.mark.parametrize("dtype", SIXTEEN)
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_16_big_tile_with_a_ragged_last_column_tile(dtype, epi):
    """N = 6144 + 128: the last column tile of the 256 x 256 path is half outside the matrix (SwiGLU: N / 2 = 3136 =
    24.5 tiles of 128 output columns)."""
    _gemm_16_case(dtype, epi, 4100, 6144 + 128, 320)


@pytest.mark.parametrize("dtype", SIXTEEN)
@pytest.mark.parametrize("epi", [B.EPI_STORE, B.EPI_RESIDUAL, B.EPI_SWIGLU])
def test_gemm_16_rows_beyond_whole_rounds_go_to_small_tiles_with_the_same_bits(dtype, epi):
    """2900 x 6144 outputs are 12 x 24 = 288 tiles of 256 x 256: one round of 256 compute units and a few tiles more.  The
    launcher gives the first 10 row tiles (240 tiles, one round) to the big tile and the last 340 rows to a second launch
    with 128 x 128 tiles.  Checked against the oracle, and bit for bit against the same rows computed by the small tile
    alone (2560 rows are 240 big tiles, too few for the big tile: that launch takes the small one)."""
    M, N, K, cut = 2900, 6144, 320, 2560
    _gemm_16_case(dtype, epi, M, N, K)
    A = _rand((M, K), dtype, 10 + M + K, 1.0).to(DEV)
    Wt = _rand((N, K), dtype, 20 + N + K, 1.0 / math.sqrt(K)).to(DEV)
    cols = N // 2 if epi == B.EPI_SWIGLU else N

    def fresh(rows):
        if epi == B.EPI_RESIDUAL:
            return _rand((M, N), torch.float32, 30, 1.0)[rows].to(DEV).clone()
        return torch.zeros(len(range(M)[rows]), cols, dtype=dtype, device=DEV)
    whole = fresh(slice(0, M))
    B.op_gemm(epi, A, Wt, whole)
    top, bottom = fresh(slice(0, cut)), fresh(slice(cut, M))
    B.op_gemm(epi, A[:cut].contiguous(), Wt, top)
    B.op_gemm(epi, A[cut:].contiguous(), Wt, bottom)
    torch.cuda.synchronize()
    assert torch.equal(whole[:cut], top) and torch.equal(whole[cut:], bottom)


@pytest.mark.parametrize("dtype", SIXTEEN)
def test_gemm_16_fp32_output(dtype):
    M, N, K = 700, 6144, 1024
    A, Wt = _rand((M, K), dtype, 5), _rand((N, K), dtype, 6, 1.0 / math.sqrt(K))
    out = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    B.op_gemm(B.EPI_STORE_F32, A.to(DEV), Wt.to(DEV), out)
    np.testing.assert_allclose(_f64(out), _f64(A) @ _f64(Wt).T, rtol=1e-4, atol=1e-4)


def test_gemm_16_row_panels_beyond_4gib():
    """A has more than 4 GiB of bytes: the launcher cuts it into row panels (the kernel addresses with 32-bit offsets).
    Sampled rows on both sides of the cut against the oracle's plain product."""
    K, N = 12288, 512
    M = ((1 << 32) // (K * 2) // 256 + 3) * 256                  # three row tiles past the first panel
    g = torch.Generator(device=DEV).manual_seed(7)
    A = torch.randn(M, K, device=DEV, generator=g, dtype=torch.float32).to(torch.float16)
    Wt = (torch.randn(N, K, device=DEV, generator=g, dtype=torch.float32) / math.sqrt(K)).to(torch.float16)
    out = torch.zeros(M, N, dtype=torch.float32, device=DEV)
    B.op_gemm(B.EPI_STORE_F32, A, Wt, out)
    torch.cuda.synchronize()
    cut = (1 << 32) // (K * 2) // 256 * 256
    rows = [0, 1, 255, cut - 1, cut, cut + 1, cut + 300, M - 1]
    ref = _f64(A[rows]) @ _f64(Wt).T
    np.testing.assert_allclose(_f64(out[rows]), ref, rtol=1e-4, atol=1e-4)
    assert out.abs().sum(dim=1).min().item() > 0                 # no row was left unwritten


def _vt_layout(lens):
    """Column of every token in the transposed V buffer: sequences start at multiples of 64; within every group of 16
    positions the columns follow the order 0-3, 8-11, 4-7, 12-15 (the header's prism_vt_column_of_key)."""
    col0 = np.concatenate([[0], np.cumsum([(l + 63) // 64 * 64 for l in lens])]).astype(np.int32)
    vt_col = np.concatenate([col0[i] + B.vt_column_of_key(np.arange(l)) for i, l in enumerate(lens)]).astype(np.int32)
    return col0[:-1], vt_col, int(col0[-1])


@pytest.mark.parametrize("dtype,nq,nkv,hd", [(torch.float32, 4, 2, 64), (torch.float32, 6, 3, 32), (torch.bfloat16, 8, 2, 128),
                                             (torch.float16, 8, 2, 128)])
@pytest.mark.parametrize("qk_norm", [True, False])
def test_qkv_finish(dtype, nq, nkv, hd, qk_norm):
    lens = [5, 130, 1, 64, 299]
    T = sum(lens)
    pos = np.concatenate([np.arange(l) for l in lens]).astype(np.int32)
    QKV = _rand((T, (nq + 2 * nkv) * hd), torch.float32, 40, 1.5)
    gq, gk = (1 + _rand((hd,), torch.float32, 41, 0.1)).to(dtype), (1 + _rand((hd,), torch.float32, 42, 0.1)).to(dtype)
    x = _f64(QKV).reshape(T, nq + 2 * nkv, hd)
    q, k, v = x[:, :nq], x[:, nq:nq + nkv], x[:, nq + nkv:]
    if qk_norm:
        q, k = O.rmsnorm(q, _f64(gq), 1e-6), O.rmsnorm(k, _f64(gk), 1e-6)
    q, k = O.rope(q, pos, 1e6), O.rope(k, pos, 1e6)
    d = QKV.to(DEV).clone()
    dpos = torch.from_numpy(pos).to(DEV)
    if dtype == torch.float32:
        B.op_qkv_finish(B.DTYPE_FP32, d, dpos, 512, gq.to(DEV), gk.to(DEV), nq, nkv, hd, 1e-6, 1e6, qk_norm)
        ref = np.concatenate([q, k, v], axis=1).reshape(T, -1)
        np.testing.assert_allclose(_f64(d), ref, rtol=1e-5, atol=2e-5)
        return
    col0, vt_col, ncol = _vt_layout(lens)
    QK = torch.zeros(T, (nq + nkv) * hd, dtype=dtype, device=DEV)
    Vt = torch.zeros(nkv, hd, ncol, dtype=torch.float16, device=DEV)
    B.op_qkv_finish(B._dt(QK), d, dpos, 512, gq.to(DEV), gk.to(DEV), nq, nkv, hd, 1e-6, 1e6, qk_norm,
                    QK, Vt, torch.from_numpy(vt_col).to(DEV), ncol)
    ref_qk = np.concatenate([q, k], axis=1).reshape(T, -1)
    got = _f64(QK)
    # one rounding to bf16 of a value computed in fp32: within one bf16 ulp of the oracle's rounded value,
    # and equal to it except where fp32 arithmetic lands on the other side of a rounding boundary
    np.testing.assert_allclose(got, ref_qk, rtol=EPS16[dtype] * 1.01, atol=1e-6)
    assert np.mean(got != O.round_operand(ref_qk, OPERAND[dtype])) < 0.02
    vt = _f64(Vt)
    ref_v = np.transpose(O.round_operand(v, OPERAND[dtype]), (1, 2, 0))
    diff = np.abs(vt[:, :, vt_col] - ref_v)
    # exact (rounding + layout), except that half cannot hold bf16 values below 2^-17 exactly
    assert diff.max() <= 2.0 ** -25 and np.all(diff[np.abs(ref_v) >= 2.0 ** -14] == 0), (diff.max(), int((diff > 0).sum()))
    pad = np.setdiff1d(np.arange(ncol), vt_col)
    assert (vt[:, :, pad] == 0).all()


@pytest.mark.parametrize("dtype", SIXTEEN)
@pytest.mark.parametrize("qk_norm", [True, False])
def test_qkv_project_fused(dtype, qk_norm):
    """Projection + norm + RoPE + V transposition in one kernel against the oracle's separate steps, several row
    tiles with a ragged last one, and against the unfused device path."""
    nq, nkv, hd, H = 32, 8, 128, 256
    lens = [700, 1, 1024, 64, 911]
    T = sum(lens)
    pos = np.concatenate([np.arange(l) for l in lens]).astype(np.int32)
    Xn, Wt = _rand((T, H), dtype, 50), _rand(((nq + 2 * nkv) * hd, H), dtype, 51, 1.0 / math.sqrt(H))
    gq, gk = (1 + _rand((hd,), torch.float32, 52, 0.1)).to(dtype), (1 + _rand((hd,), torch.float32, 53, 0.1)).to(dtype)
    x = (_f64(Xn) @ _f64(Wt).T).reshape(T, nq + 2 * nkv, hd)
    q, k, v = x[:, :nq], x[:, nq:nq + nkv], x[:, nq + nkv:]
    if qk_norm:
        q, k = O.rmsnorm(q, _f64(gq), 1e-6), O.rmsnorm(k, _f64(gk), 1e-6)
    q, k = O.rope(q, pos, 1e6), O.rope(k, pos, 1e6)
    col0, vt_col, ncol = _vt_layout(lens)
    dpos, dcol = torch.from_numpy(pos).to(DEV), torch.from_numpy(vt_col).to(DEV)
    QK = torch.zeros(T, (nq + nkv) * hd, dtype=dtype, device=DEV)
    Vt = torch.zeros(nkv, hd, ncol, dtype=torch.float16, device=DEV)
    B.op_qkv_project(Xn.to(DEV), Wt.to(DEV), dpos, 1024, gq.to(DEV), gk.to(DEV), nq, nkv, hd, 1e-6, 1e6, qk_norm, QK, Vt, dcol, ncol)
    ref_qk = np.concatenate([q, k], axis=1).reshape(T, -1)
    got = _f64(QK)
    # fp32 accumulation over 256 products, fp32 norm and rotation, then ONE 16-bit rounding
    np.testing.assert_allclose(got, ref_qk, rtol=EPS16[dtype] * 1.01, atol=2e-6)
    assert np.mean(got != O.round_operand(ref_qk, OPERAND[dtype])) < 0.02
    vt = _f64(Vt)
    ref_v = np.transpose(v, (1, 2, 0))
    np.testing.assert_allclose(vt[:, :, vt_col], ref_v, rtol=EPS16[dtype] * 1.01, atol=2e-6)
    pad = np.setdiff1d(np.arange(ncol), vt_col)
    assert (vt[:, :, pad] == 0).all()
    # the unfused device path: same arithmetic except the order of the sum of squares
    QKV = torch.zeros(T, (nq + 2 * nkv) * hd, dtype=torch.float32, device=DEV)
    B.op_gemm(B.EPI_STORE_F32, Xn.to(DEV), Wt.to(DEV), QKV)
    QK2, Vt2 = torch.zeros_like(QK), torch.zeros_like(Vt)
    B.op_qkv_finish(B._dt(QK), QKV, dpos, 1024, gq.to(DEV), gk.to(DEV), nq, nkv, hd, 1e-6, 1e6, qk_norm, QK2, Vt2, dcol, ncol)
    assert torch.equal(Vt, Vt2)
    assert (QK != QK2).float().mean().item() < 1e-3
    np.testing.assert_allclose(_f64(QK), _f64(QK2), rtol=2 * EPS16[dtype] * 1.01, atol=2e-6)   # neighbouring 16-bit values at most


def test_qkv_project_rejects_small_problems():
    Xn, Wt = torch.zeros(100, 256, dtype=torch.float16, device=DEV), torch.zeros(48 * 128, 256, dtype=torch.float16, device=DEV)
    z = torch.zeros(128, dtype=torch.float16, device=DEV)
    with pytest.raises(B.PrismError) as e:
        B.op_qkv_project(Xn, Wt, torch.zeros(100, dtype=torch.int32, device=DEV), 16, z, z, 32, 8, 128, 1e-6, 1e6, True,
                         torch.zeros(100, 40 * 128, dtype=torch.float16, device=DEV), torch.zeros(8, 128, 128, dtype=torch.float16, device=DEV),
                         torch.zeros(100, dtype=torch.int32, device=DEV), 128)
    assert e.value.code == B.EUNSUPPORTED


ATTN_CASES = [
    (torch.float32, 4, 2, 64, [1, 17, 64, 100]),
    (torch.float32, 6, 3, 32, [33, 2]),
    (torch.bfloat16, 8, 2, 128, [1, 63, 64, 65, 130, 300]),      # G = 4
    (torch.bfloat16, 16, 8, 128, [200, 129, 31]),                # G = 2
    (torch.bfloat16, 8, 8, 128, [257, 5]),                       # G = 1
    (torch.bfloat16, 8, 1, 128, [97, 32]),                       # G = 8
    (torch.bfloat16, 32, 8, 128, [1024, 700]),                   # the 8B head shape at its sequence length
    (torch.float16, 32, 8, 128, [1024, 700]),
    (torch.float16, 16, 8, 128, [200, 129, 31]),
    (torch.float16, 8, 2, 128, [1, 63, 64, 65, 130, 300]),
]


@pytest.mark.parametrize("dtype,nq,nkv,hd,lens", ATTN_CASES)
def test_attention(dtype, nq, nkv, hd, lens):
    T = sum(lens)
    cu = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    QKV = _rand((T, (nq + 2 * nkv) * hd), dtype, 50 + T, 1.0)
    out = torch.zeros(T, nq * hd, dtype=dtype, device=DEV)
    x = _f64(QKV).reshape(T, nq + 2 * nkv, hd)
    if dtype == torch.float32:
        B.op_attention(B.DTYPE_FP32, QKV.to(DEV), None, 0, cu, None, nq, nkv, hd, out)
    else:
        col0, vt_col, ncol = _vt_layout(lens)
        QK = QKV[:, :(nq + nkv) * hd].contiguous().to(DEV)
        Vt = torch.zeros(nkv, hd, ncol, dtype=torch.float16)
        Vt[:, :, torch.from_numpy(vt_col.astype(np.int64))] = QKV.view(T, -1, hd)[:, nq + nkv:].permute(1, 2, 0).to(torch.float16)
        B.op_attention(B._dt(QK), QK, Vt.to(DEV), ncol, cu, col0, nq, nkv, hd, out)
    ref = np.concatenate([O.causal_gqa_attention(x[a:b, :nq], x[a:b, nq:nq + nkv], x[a:b, nq + nkv:]).reshape(b - a, -1)
                          for a, b in zip(cu[:-1], cu[1:])])
    # bf16 mode: exact operands, f16 probabilities, fp32 accumulation, one bf16 rounding of the output
    tol = dict(rtol=1e-4, atol=1e-5) if dtype == torch.float32 else dict(rtol=2 ** -8 if dtype == torch.bfloat16 else 2 ** -9, atol=2e-3)
    np.testing.assert_allclose(_f64(out), ref, **tol)


def test_attention_refuses_a_transposed_v_stride_beyond_its_32_bit_offsets():
    """The 16-bit kernel addresses the 128 rows of a KV head's V^T with 32-bit byte offsets: a row stride of 2^24 columns
    (128 rows x 2 bytes = 4 GiB) is refused before anything is launched (the buffers here are tiny and never touched)."""
    nq, nkv, hd = 8, 2, 128
    QK = torch.zeros(4, (nq + nkv) * hd, dtype=torch.float16, device=DEV)
    Vt = torch.zeros(nkv, hd, 64, dtype=torch.float16, device=DEV)
    out = torch.zeros(4, nq * hd, dtype=torch.float16, device=DEV)
    with pytest.raises(B.PrismError) as e:
        B.op_attention(B.DTYPE_F16, QK, Vt, 1 << 24, np.array([0, 4], np.int32), np.array([0], np.int32), nq, nkv, hd, out)
    assert e.value.code == B.EUNSUPPORTED


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
