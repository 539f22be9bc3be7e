"""Pins for the oracle's layer arithmetic: closed forms, hand values, brute force and an
independently structured padded/batched forward.  CPU only."""
import math

import numpy as np
import pytest
import torch

from oracle import prism_oracle as O

rng = np.random.default_rng(1234)


def test_rmsnorm_hand_values_and_gain():
    out = O.rmsnorm(np.array([3.0, 4.0]), np.array([1.0, 1.0]), 0.0)
    assert np.allclose(out, [3 / math.sqrt(12.5), 4 / math.sqrt(12.5)], atol=1e-15)
    out = O.rmsnorm(np.array([3.0, 4.0]), np.array([2.0, 0.5]), 0.0)
    assert np.allclose(out, [6 / math.sqrt(12.5), 2 / math.sqrt(12.5)], atol=1e-15)
    # eps sits inside the square root, added to the mean square
    out = O.rmsnorm(np.array([0.0, 0.0, 2.0, 0.0]), np.ones(4), 3.0)
    assert np.allclose(out, [0, 0, 2 / math.sqrt(1.0 + 3.0), 0])


def test_rmsnorm_unit_rms_and_scale_invariance():
    x = rng.normal(size=(5, 64))
    g = 1 + 0.1 * rng.normal(size=64)
    y = O.rmsnorm(x, g, 0.0) / g
    assert np.allclose(np.sqrt((y * y).mean(-1)), 1.0, atol=1e-14)
    assert np.allclose(O.rmsnorm(7.5 * x, g, 0.0), O.rmsnorm(x, g, 0.0), atol=1e-13)


def test_rope_is_plane_rotation_with_rotate_half_pairing():
    # hd = 2: a single pair, frequency base^0 = 1: counter-clockwise rotation by pos radians
    x = np.array([[[1.0, 0.0]], [[1.0, 0.0]], [[0.0, 1.0]]])
    y = O.rope(x, np.array([0.0, math.pi / 2, math.pi / 2]), 10000.0)
    assert np.allclose(y[0, 0], [1, 0], atol=1e-15)          # position 0 is the identity
    assert np.allclose(y[1, 0], [0, 1], atol=1e-15)
    assert np.allclose(y[2, 0], [-1, 0], atol=1e-15)
    # hd = 4: dimension 0 pairs with 2 (frequency 1), dimension 1 with 3 (frequency base^-1/2)
    base = 100.0
    x = np.zeros((1, 1, 4)); x[0, 0, 0] = 1.0; x[0, 0, 1] = 1.0
    y = O.rope(x, np.array([3.0]), base)
    assert np.allclose(y[0, 0], [math.cos(3.0), math.cos(0.3), math.sin(3.0), math.sin(0.3)], atol=1e-15)


def test_rope_relative_property_and_norm():
    hd = 16
    q, k = rng.normal(size=(1, 1, hd)), rng.normal(size=(1, 1, hd))
    def dot(m, n):
        return float((O.rope(q, np.array([m]), 1e6) * O.rope(k, np.array([n]), 1e6)).sum())
    assert abs(dot(5, 2) - dot(13, 10)) < 1e-12
    assert abs(dot(5, 2) - dot(3, 0)) < 1e-12
    assert abs(dot(5, 2) - dot(2, 5)) > 1e-6                 # direction matters
    assert np.allclose(np.linalg.norm(O.rope(q, np.array([77]), 1e6)), np.linalg.norm(q))


def _attention_loops(q, k, v):
    """Pure-Python definition: for each query i and head h, softmax over keys j <= i."""
    L, nq, hd = q.shape
    g = nq // k.shape[1]
    out = np.zeros_like(q)
    for i in range(L):
        for h in range(nq):
            logits = [sum(q[i, h, d] * k[j, h // g, d] for d in range(hd)) / math.sqrt(hd) for j in range(i + 1)]
            mx = max(logits)
            w = [math.exp(t - mx) for t in logits]
            z = sum(w)
            for d in range(hd):
                out[i, h, d] = sum(w[j] * v[j, h // g, d] for j in range(i + 1)) / z
    return out


def test_attention_matches_brute_force_loops():
    q, k, v = rng.normal(size=(7, 4, 6)), rng.normal(size=(7, 2, 6)), rng.normal(size=(7, 2, 6))
    assert np.allclose(O.causal_gqa_attention(q, k, v), _attention_loops(q, k, v), atol=1e-13)


def test_attention_special_cases():
    L, nq, nkv, hd = 9, 4, 2, 8
    q, v = rng.normal(size=(L, nq, hd)), rng.normal(size=(L, nkv, hd))
    # identical keys -> uniform weights -> running mean of the values
    k = np.tile(rng.normal(size=(1, nkv, hd)), (L, 1, 1))
    out = O.causal_gqa_attention(q, k, v)
    run_mean = np.cumsum(v, axis=0) / np.arange(1, L + 1)[:, None, None]
    for h in range(nq):
        assert np.allclose(out[:, h], run_mean[:, h // 2], atol=1e-13)
    # first position only sees itself
    k = rng.normal(size=(L, nkv, hd))
    out = O.causal_gqa_attention(q, k, v)
    assert np.allclose(out[0, 3], v[0, 1])
    # GQA == MHA with the KV heads replicated
    out_mha = O.causal_gqa_attention(q, np.repeat(k, 2, axis=1), np.repeat(v, 2, axis=1))
    assert np.allclose(out, out_mha, atol=1e-14)


def test_attention_causality():
    L, nq, nkv, hd = 10, 2, 1, 4
    q, k, v = rng.normal(size=(L, nq, hd)), rng.normal(size=(L, nkv, hd)), rng.normal(size=(L, nkv, hd))
    a = O.causal_gqa_attention(q, k, v)
    k2, v2 = k.copy(), v.copy()
    k2[6] += 1.0; v2[6] -= 2.0
    b = O.causal_gqa_attention(q, k2, v2)
    assert np.array_equal(a[:6], b[:6]) and not np.allclose(a[6:], b[6:])


def test_silu_values():
    assert O.silu(np.array([0.0]))[0] == 0.0
    assert abs(O.silu(np.array([1.0]))[0] - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    h = 1e-6
    assert abs((O.silu(np.array([h]))[0] - O.silu(np.array([-h]))[0]) / (2 * h) - 0.5) < 1e-9
    assert abs(O.silu(np.array([-20.0]))[0]) < 1e-7 and abs(O.silu(np.array([20.0]))[0] - 20.0) < 1e-7


def _tiny_model(**kw):
    d = dict(n_layers=2, hidden=12, n_q_heads=4, n_kv_heads=2, head_dim=4, ffn=10, vocab=30)
    d.update(kw)
    return O.Model(**d)


def _tiny_weights(m, seed=0):
    r = np.random.default_rng(seed)
    qd, kd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    def layer():
        return {"attn_norm": 1 + .1 * r.normal(size=m.hidden), "wq": .3 * r.normal(size=(qd, m.hidden)),
                "wk": .3 * r.normal(size=(kd, m.hidden)), "wv": .3 * r.normal(size=(kd, m.hidden)),
                "q_norm": 1 + .1 * r.normal(size=m.head_dim), "k_norm": 1 + .1 * r.normal(size=m.head_dim),
                "wo": .3 * r.normal(size=(m.hidden, qd)), "ffn_norm": 1 + .1 * r.normal(size=m.hidden),
                "w_gate": .3 * r.normal(size=(m.ffn, m.hidden)), "w_up": .3 * r.normal(size=(m.ffn, m.hidden)),
                "w_down": .3 * r.normal(size=(m.hidden, m.ffn))}
    emb = r.normal(size=(m.vocab, m.hidden))
    return {"embed": emb, "final_norm": 1 + .1 * r.normal(size=m.hidden), "w_yes": emb[1], "w_no": emb[0],
            "layers": [layer() for _ in range(m.n_layers)]}


def test_ffn_block_against_three_loop_products():
    m = _tiny_model()
    w = _tiny_weights(m)["layers"][0]
    X = rng.normal(size=(3, m.hidden))
    out = O.ffn_block(X, w, m)
    for t in range(3):
        ms = sum(X[t, i] ** 2 for i in range(m.hidden)) / m.hidden
        xn = [X[t, i] / math.sqrt(ms + m.rms_eps) * w["ffn_norm"][i] for i in range(m.hidden)]
        act = []
        for f in range(m.ffn):
            g = sum(xn[i] * w["w_gate"][f, i] for i in range(m.hidden))
            u = sum(xn[i] * w["w_up"][f, i] for i in range(m.hidden))
            act.append(g / (1 + math.exp(-g)) * u)
        for o in range(m.hidden):
            ref = X[t, o] + sum(act[f] * w["w_down"][o, f] for f in range(m.ffn))
            assert abs(out[t, o] - ref) < 1e-12


def _padded_forward_torch(tokens_list, w, m):
    """Independent structure: one right-padded batch, all sequences at once, key masking,
    heads handled by einsum.  Checks 'packed equals padded' and the attention block's wiring."""
    B, Lmax = len(tokens_list), max(len(t) for t in tokens_list)
    T = lambda a: torch.tensor(np.asarray(a), dtype=torch.float64)
    ids = torch.zeros(B, Lmax, dtype=torch.long)
    valid = torch.zeros(B, Lmax, dtype=torch.bool)
    for b, t in enumerate(tokens_list):
        ids[b, :len(t)] = torch.tensor(np.asarray(t), dtype=torch.long); valid[b, :len(t)] = True
    X = T(w["embed"])[ids]
    def norm(x, g):
        return x * torch.rsqrt((x * x).mean(-1, keepdim=True) + m.rms_eps) * T(g)
    pos = torch.arange(Lmax, dtype=torch.float64)
    half = m.head_dim // 2
    inv = m.rope_base ** (-torch.arange(half, dtype=torch.float64) * 2 / m.head_dim)
    ang = pos[:, None] * inv[None, :]
    cos, sin = torch.cos(ang)[None, :, None, :], torch.sin(ang)[None, :, None, :]
    def rot(x):
        a, b = x[..., :half], x[..., half:]
        return torch.cat([a * cos - b * sin, b * cos + a * sin], -1)
    causal = torch.tril(torch.ones(Lmax, Lmax, dtype=torch.bool))
    mask = causal[None, None] & valid[:, None, None, :]
    rep = m.n_q_heads // m.n_kv_heads
    for lw in w["layers"]:
        xn = norm(X, lw["attn_norm"])
        q = (xn @ T(lw["wq"]).T).view(B, Lmax, m.n_q_heads, m.head_dim)
        k = (xn @ T(lw["wk"]).T).view(B, Lmax, m.n_kv_heads, m.head_dim)
        v = (xn @ T(lw["wv"]).T).view(B, Lmax, m.n_kv_heads, m.head_dim)
        if m.qk_norm:
            q, k = norm(q, lw["q_norm"]), norm(k, lw["k_norm"])
        q, k = rot(q), rot(k)
        k, v = k.repeat_interleave(rep, 2), v.repeat_interleave(rep, 2)
        s = torch.einsum("bihd,bjhd->bhij", q, k) / math.sqrt(m.head_dim)
        s = s.masked_fill(~mask, float("-inf"))
        a = torch.einsum("bhij,bjhd->bihd", torch.softmax(s, -1), v).reshape(B, Lmax, -1)
        X = X + a @ T(lw["wo"]).T
        xn = norm(X, lw["ffn_norm"])
        X = X + (torch.nn.functional.silu(xn @ T(lw["w_gate"]).T) * (xn @ T(lw["w_up"]).T)) @ T(lw["w_down"]).T
    last = torch.stack([X[b, len(t) - 1] for b, t in enumerate(tokens_list)])
    z = norm(last, w["final_norm"])
    return (z @ (T(w["w_yes"]) - T(w["w_no"]))).numpy()


@pytest.mark.parametrize("qk_norm", [True, False])
def test_packed_per_sequence_forward_equals_padded_batch(qk_norm):
    m = _tiny_model(qk_norm=qk_norm)
    w = _tiny_weights(m, 3)
    r = np.random.default_rng(5)
    query = r.integers(0, m.vocab, 4)
    cands = [r.integers(0, m.vocab, n) for n in (3, 9, 1, 6)]
    seqs = [np.concatenate([query, c]) for c in cands]
    ref = _padded_forward_torch(seqs, w, m)
    got = np.array([O.score_trajectory(query, c, w, m, [m.n_layers])[m.n_layers] for c in cands])
    assert np.allclose(got, ref, atol=1e-11)


def test_query_prefix_states_do_not_depend_on_candidate():
    m = _tiny_model()
    w = _tiny_weights(m, 4)
    r = np.random.default_rng(6)
    query = r.integers(0, m.vocab, 5)
    outs = []
    for n in (2, 7):
        X = O.embed(np.concatenate([query, r.integers(0, m.vocab, n)]), w["embed"])
        for lw in w["layers"]:
            X = O.layer_forward(X, lw, m)
        outs.append(X[:5])
    assert np.allclose(outs[0], outs[1], atol=1e-13)


def test_head_score_hand_value():
    h = np.array([1.0, -1.0, 1.0, -1.0])           # rms = 1
    g = np.array([1.0, 2.0, 1.0, 1.0])
    yes, no = np.array([1.0, 0, 0, 0]), np.array([0, 1.0, 0, 0])
    # z = h * g = [1, -2, 1, -1]; yes - no = 1 - (-2) = 3
    assert abs(O.head_score(h, g, yes, no, 0.0) - 3.0) < 1e-14


def test_operand_rounding_is_round_to_nearest_even():
    # bf16 keeps 8 significand bits: spacing 2^-7 in [1, 2)
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, 1.0 + 3 * 2 ** -8, -(1.0 + 2 ** -8), 3.14159265, 1e-3])
    got = O.round_operand(x, "bf16")
    assert got[0] == 1.0 and got[1] == 1.0                      # tie -> even (1.0)
    assert got[2] == 1.0 + 2 ** -7                              # just above the tie -> up
    assert got[3] == 1.0 + 2 ** -6 and got[4] == -1.0           # tie -> even (1 + 2/128); sign symmetric
    assert got[5] == 3.140625 and abs(got[6] - 1e-3) < 1e-3 * 2 ** -8
    ref = torch.tensor(x, dtype=torch.float64).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(got, ref)                             # library conversion agrees
    r = np.random.default_rng(0).normal(size=4096) * 10.0 ** np.random.default_rng(1).integers(-6, 6, 4096)
    assert np.array_equal(O.round_operand(r, "bf16"),
                          torch.tensor(r).to(torch.float32).to(torch.bfloat16).to(torch.float64).numpy())
    assert np.array_equal(O.round_operand(r, "f16"), torch.tensor(r).to(torch.float16).to(torch.float64).numpy())
    assert O.round_operand(r, "exact") is r


def test_operand_rounding_enters_only_at_contraction_operands():
    m = _tiny_model()
    w = _tiny_weights(m, 8)
    r = np.random.default_rng(9)
    toks = r.integers(0, m.vocab, 9)
    exact = O.score_trajectory(toks[:4], toks[4:], w, m, [2])[2]
    import dataclasses
    for kind, eps in (("bf16", 2 ** -8), ("f16", 2 ** -11)):
        got = O.score_trajectory(toks[:4], toks[4:], w, dataclasses.replace(m, operand=kind), [2])[2]
        assert got != exact and abs(got - exact) < 60 * eps     # a perturbation of the size of the rounding
