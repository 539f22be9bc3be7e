"""Seeded differential test of prism_select against the oracle over the option space: pool size, ragged lengths, K,
routing mode, number of clusters, dispersion threshold, checkpoint subset, chunk size, and the memory modes (hidden-state
offload, embedding cache, layers streamed from pinned host memory through a ring of 2 to 5 buffers), which must not change
any number.  Small models so that the oracle finishes in a fraction of a second per case."""
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


class _HostEmbed:
    def __init__(self, wt, layers):
        self.embed = wt.embed.cpu().pin_memory()
        self.layers, self.final_norm = layers, wt.final_norm
        self.w_yes, self.w_no = wt.w_yes.clone(), wt.w_no.clone()


_WEIGHTS, _HOST_LAYERS = {}, {}


def _host_layers(name):
    if name not in _HOST_LAYERS:
        _HOST_LAYERS[name] = [{k: v.cpu().pin_memory() for k, v in l.items()} for l in _weights(name).layers]
    return _HOST_LAYERS[name]


def _weights(name):
    if name not in _WEIGHTS:
        _WEIGHTS[name] = W.make_weights(W.WORKLOADS[name], "cuda")
    return _WEIGHTS[name]


@pytest.mark.parametrize("seed", range(48))
def test_random_options_match_the_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    name, tol = (("mini_fp32", 1e-4), ("mini_bf16", 2e-2))[seed % 2]
    base = W.WORKLOADS[name]
    m = base.model
    n = int(rng.integers(1, 15))
    qlen = int(rng.integers(1, 20))
    lens = rng.integers(1, 120, size=n)
    q = rng.integers(0, m.vocab, size=qlen, dtype=np.int32)
    cands = [rng.integers(0, m.vocab, size=int(l), dtype=np.int32) for l in lens]
    K = int(rng.integers(1, n + 2))
    mode = int(rng.choice([B.MODE_DROP_ONLY, B.MODE_DROP_ONLY, B.MODE_THREE_WAY, B.MODE_NO_PRUNING]))
    layers = list(range(1, m.n_layers))
    ck = sorted(rng.choice(layers, size=int(rng.integers(0, len(layers) + 1)), replace=False).tolist())
    tau = float(rng.choice([0.0, 0.2, 0.6]))
    k = int(rng.integers(2, 6))
    chunk = int(rng.choice([0, 1, 3, 50]))
    offload = bool(rng.integers(0, 2)) and chunk > 0
    cache = bool(rng.integers(0, 2))
    w = dataclasses.replace(base, K=K, checkpoints=ck, cv_threshold=tau, n_clusters=k)
    wt = _weights(name)
    cache_rows = int(rng.integers(1, 40)) if cache else 0
    stream = bool(rng.integers(0, 2))                     # (drawn last: the cases above keep their earlier options)
    slots = int(rng.choice([0, 3, 5]))
    layers_arg = _host_layers(name) if stream else wt.layers
    weights = _HostEmbed(wt, layers_arg) if cache else (W.Weights(wt.embed, layers_arg, wt.final_norm) if stream else wt)
    p = B.Prism(m, weights, checkpoints=ck, cv_threshold=tau, n_clusters=k, mode=mode, chunk_cands=chunk, offload_hidden=offload,
                embed_on_host=cache, embed_cache_rows=cache_rows, stream_weights=stream, stream_slots=slots)
    idx, scores, rep = p.select(q, cands, K)
    p.destroy()
    ref = oracle_select(w, wt, (q, cands), mode=mode)
    desc = dict(n=n, K=K, mode=mode, ck=ck, tau=tau, k=k, chunk=chunk, offload=offload, cache=cache, stream=stream, slots=slots)
    assert len(idx) == min(K, n), desc
    if mode == B.MODE_THREE_WAY:
        assert sorted(idx.tolist()) == sorted(ref.idx.tolist()), desc
        got = dict(zip(idx.tolist(), scores.tolist()))
        for i, s in zip(ref.idx.tolist(), ref.scores.tolist()):
            assert abs(got[i] - s) <= tol, desc
        assert len(rep.layer) == len(ref.events), desc
    else:
        check_against_oracle(w, idx, scores, rep, ref, tol)
