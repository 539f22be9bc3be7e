"""4-bit layer weights on the device (the paper's quantised variant, Sec. 6; format: this build's reading, stated in the
header).  Integer work is compared bit for bit: the device quantiser against the oracle's, the expansion against
q * scale.  End to end, a context fed 4-bit blobs must agree with the oracle run on the dequantised weights (from the oracle's own
quantiser) within the usual tolerance, and the resident and the streamed form must agree bit for bit."""
import numpy as np
import pytest
import torch

from oracle import prism_oracle as O
from paper_2510_15620_amd import binding as B
from paper_2510_15620_amd import workloads as W
from tests.helpers import oracle_select
from tests.test_gpu_select import check_against_oracle

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _unpack(blob, N, K):
    b = blob.cpu().numpy()
    codes = b[:N * K // 2].reshape(N, K // 2)
    q = np.empty((N, K), np.int8)
    q[:, 0::2] = (codes & 15).astype(np.int8) - 8
    q[:, 1::2] = (codes >> 4).astype(np.int8) - 8
    sc = b[N * K // 2:].view(np.uint16).astype(np.uint32) << 16
    return q, sc.view(np.float32).reshape(N, K // 128)


@pytest.mark.parametrize("N,K,scale", [(7, 128, 0.02), (300, 1408, 0.02), (64, 512, 5.0), (33, 256, 1e-4)])
def test_quantiser_is_the_oracles(N, K, scale):
    g = torch.Generator().manual_seed(N * 1000 + K)
    Wt = (torch.randn(N, K, generator=g) * scale).to(torch.bfloat16)
    Wt[0, :128] = 0                                            # an all-zero group
    Wt[1 % N, 5] = Wt[1 % N].abs().max() * 4                   # one dominant element
    blob = B.quantize_w4(Wt.to(DEV))
    assert blob.numel() == B.w4_bytes(N, K) == N * K // 2 + N * (K // 128) * 2
    q, sc = _unpack(blob, N, K)
    rq, rsc = O.quantize_w4(Wt.float().numpy())
    assert np.array_equal(sc, rsc)
    assert np.array_equal(q, rq)
    for dt in (torch.float16, torch.bfloat16):
        out = torch.zeros(N, K, dtype=dt, device=DEV)
        B.dequantize_w4(blob, N, K, out)
        ref = torch.from_numpy(O.dequantize_w4(rq, rsc)).to(dt)          # exact in half; rounded once in bf16
        assert torch.equal(out.cpu(), ref)


class _Weights:
    def __init__(self, wt, layers):
        self.embed, self.layers, self.final_norm = wt.embed, layers, wt.final_norm
        self.w_yes, self.w_no = wt.w_yes, wt.w_no


def _dequantised_layers(layers):
    """What the 4-bit layers stand for, as fp64 arrays (oracle side) from the oracle's own quantiser."""
    out = []
    for l in layers:
        d = {}
        for k, v in l.items():
            a = v.float().cpu().numpy()
            d[k] = O.dequantize_w4(*O.quantize_w4(a)) if k in B.MATRICES else a.astype(np.float64)
        out.append(d)
    return out


@pytest.mark.parametrize("streamed", [False, True])
@pytest.mark.parametrize("mode", [B.MODE_DROP_ONLY, B.MODE_THREE_WAY])
def test_select_with_4bit_layers(streamed, mode):
    w = W.WORKLOADS["mini_bf16"]
    wt = W.make_weights(w, DEV)
    q, cands = W.make_tokens(w)
    ql = B.quantize_layers_w4(wt.layers)
    if streamed:
        ql = [{k: v.cpu().pin_memory() for k, v in l.items()} for l in ql]
    p = B.Prism(w.model, _Weights(wt, ql), checkpoints=w.checkpoints, mode=mode, w4=True, stream_weights=streamed)
    out = p.select(q, cands, w.K)
    out_again = p.select(q, cands, w.K)                        # the two slots are refilled from the blobs every call
    p.destroy()
    assert out[0].tolist() == out_again[0].tolist() and np.array_equal(out[1], out_again[1])
    # oracle on the dequantised weights
    deq = _dequantised_layers(wt.layers)
    ow = W.Weights(wt.embed.cpu(), [{k: torch.from_numpy(v) for k, v in l.items()} for l in deq], wt.final_norm.cpu())
    ref = oracle_select(w, ow, (q, cands), mode=mode)
    if mode == B.MODE_DROP_ONLY:
        check_against_oracle(w, out[0], out[1], out[2], ref, 2e-2)
    else:
        assert out[0].tolist() == ref.idx.tolist()
        assert np.max(np.abs(out[1] - ref.scores)) <= 2e-2
    if not streamed:
        assert out[2].bytes_streamed == 0
    else:
        per_layer = sum(B.w4_bytes(*v.shape) if k in B.MATRICES else v.numel() * 2 for k, v in wt.layers[0].items())
        assert out[2].bytes_streamed == per_layer * w.model.n_layers
        plain = sum(v.numel() * 2 for v in wt.layers[0].values())
        assert out[2].bytes_streamed < 0.3 * plain * w.model.n_layers


def test_resident_and_streamed_4bit_agree_bit_for_bit():
    w = W.WORKLOADS["mini_bf16"]
    wt = W.make_weights(w, DEV)
    q, cands = W.make_tokens(w)
    ql = B.quantize_layers_w4(wt.layers)
    outs = []
    for streamed in (False, True):
        layers = [{k: v.cpu().pin_memory() for k, v in l.items()} for l in ql] if streamed else ql
        p = B.Prism(w.model, _Weights(wt, layers), checkpoints=w.checkpoints, w4=True, stream_weights=streamed)
        outs.append(p.select(q, cands, w.K))
        p.destroy()
    assert outs[0][0].tolist() == outs[1][0].tolist() and np.array_equal(outs[0][1], outs[1][1])
    assert np.array_equal(outs[0][2].scores, outs[1][2].scores, equal_nan=True)


def test_4bit_layers_with_offload_cache_and_deep_ring_agree_bit_for_bit():
    """Every memory mode on top of streamed 4-bit layers: hidden-state offload, embedding cache, a ring of three buffers."""
    w = W.WORKLOADS["mini_bf16"]
    wt = W.make_weights(w, DEV)
    q, cands = W.make_tokens(w)
    ql = [{k: v.cpu().pin_memory() for k, v in l.items()} for l in B.quantize_layers_w4(wt.layers)]
    p = B.Prism(w.model, _Weights(wt, ql), checkpoints=w.checkpoints, w4=True, stream_weights=True, chunk_cands=3)
    ref = p.select(q, cands, w.K)
    p.destroy()

    class Lean(_Weights):
        def __init__(self, wt, layers):
            super().__init__(wt, layers)
            self.embed = wt.embed.cpu().pin_memory()
            self.w_yes, self.w_no = wt.w_yes.clone(), wt.w_no.clone()
    p = B.Prism(w.model, Lean(wt, ql), checkpoints=w.checkpoints, w4=True, stream_weights=True, chunk_cands=3,
                offload_hidden=True, embed_on_host=True, embed_cache_rows=50, stream_slots=3)
    out = p.select(q, cands, w.K)
    p.destroy()
    assert out[0].tolist() == ref[0].tolist() and np.array_equal(out[1], ref[1])
    assert np.array_equal(out[2].scores, ref[2].scores, equal_nan=True) and np.array_equal(out[2].fate, ref[2].fate)


def test_4bit_needs_bf16_model_and_aligned_shapes():
    w = W.WORKLOADS["cfg1_tiny"]                               # fp32 model
    wt = W.make_weights(w, DEV)
    with pytest.raises(B.PrismError) as e:
        B.Prism(w.model, wt, checkpoints=w.checkpoints, w4=True)
    assert e.value.code == B.EUNSUPPORTED
