"""Writes tests/golden/fullsize_<workload>_<mode>.json: complete runs of the CPU oracle's select() on the
4B- and 8B-shaped benchmark workloads.  CPU only; calls nothing but oracle/ and the seeded input generator.

    python tests/golden/make_fullsize_goldens.py cfg3_4b drop_only
    python tests/golden/make_fullsize_goldens.py cfg3_4b three_way
    python tests/golden/make_fullsize_goldens.py cfg4_8b drop_only
    python tests/golden/make_fullsize_goldens.py cfg4_8b three_way
    python tests/golden/make_fullsize_goldens.py cfg5_8b_stream drop_only
    python tests/golden/make_fullsize_goldens.py cfg5_8b_stream three_way
    python tests/golden/make_fullsize_goldens.py cfg4_8b drop_only_w4
    python tests/golden/make_fullsize_goldens.py cfg5_8b_stream drop_only_w4
    python tests/golden/make_fullsize_goldens.py cfg5_8b_stream half_noise_w4 211,420,146

Each takes 10 to 70 minutes on eight host cores.  What is stored, per scoring event (every evaluated pruning
check of Sec. 4.1, plus the final scoring): the layer, the live candidates, their fp64 scores, the fates
(2 selected / 1 deferred / 0 dropped) and who continues; then the returned top-K with its scores.  Floats are
written with repr(), so they read back bit for bit.

The oracle walks one layer at a time over every live candidate (Sec. 3.3), so only one layer's fp64 weights
need to exist at once: the weights handed to it are sequences that draw a layer, or a set of embedding rows,
when it is asked for.

A mode name ending in _w4 runs the oracle on the weights that the 4-bit layer format stands for: each of a layer's
seven matrices goes through the oracle's own quantiser and back (Sec. 6 names the quantised variant; the format is this
build's reading of it), norm gains and the embedding table stay as drawn.

half_noise[_w4] <candidates> writes tests/golden/half_operand_noise_<workload>[_w4].json instead: the full-depth scores
of the listed candidates (no pruning; every candidate is forwarded independently, Sec. 3.3) once exact and once with every
contraction operand rounded to IEEE half, i.e. how far half operands alone move a score on this workload.
"""
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from oracle import prism_oracle as O                     # noqa: E402
from paper_2510_15620_amd import workloads as W          # noqa: E402

MODES = {"drop_only": O.MODE_DROP_ONLY, "three_way": O.MODE_THREE_WAY}


class LazyLayers:
    """weights["layers"][l]: the fp64 tensors of layer l, drawn when asked for; the previous layer is released."""

    def __init__(self, w, w4=False):
        self.w, self.at, self.cur, self.w4 = w, -1, None, w4

    def __len__(self):
        return self.w.model.n_layers

    def __getitem__(self, l):
        if l != self.at:
            self.cur = None
            if self.w4:                                      # matrices (2-D) as code x scale, gains (1-D) as drawn
                self.cur = {k: (O.dequantize_w4(*O.quantize_w4(v.float().numpy())) if v.ndim == 2
                                else v.to(torch.float64).numpy()) for k, v in W.make_layer(self.w, l).items()}
            else:
                self.cur = {k: v.to(torch.float64).numpy() for k, v in W.make_layer(self.w, l).items()}
            self.at = l
        return self.cur


class RowTable:
    """weights["embed"][tokens]: rows of the (16-bit) table as fp64, without an fp64 copy of the whole table."""

    def __init__(self, table):
        self.table = table

    def __getitem__(self, tokens):
        return self.table[torch.from_numpy(np.asarray(tokens, np.int64))].to(torch.float64).numpy()


def golden_path(workload: str, mode: str) -> str:
    return os.path.join(os.path.dirname(os.path.abspath(__file__)), f"fullsize_{workload}_{mode}.json")


def _weights(w, w4):
    m = w.model
    dt = W.torch_dtype(m)
    table = W.gaussian(w.seed, w.wname + "/embed", (m.vocab, m.hidden), 0.0, 0.02, dt)
    final_norm = W.gaussian(w.seed, w.wname + "/final_norm", (m.hidden,), 1.0, 0.02, dt)
    f64 = lambda t: t.to(torch.float64).numpy()
    return {"embed": RowTable(table), "final_norm": f64(final_norm), "w_yes": f64(table[1]), "w_no": f64(table[0]),
            "layers": LazyLayers(w, w4)}


def half_noise(workload: str, w4: bool, which):
    w = W.WORKLOADS[workload]
    m = w.model
    t0 = time.time()
    weights = _weights(w, w4)
    q, cands = W.make_tokens(w)
    scores = {}
    for operand in ("exact", "f16"):
        om = O.Model(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab, m.rms_eps, m.rope_base,
                     m.qk_norm, operand)
        sel = O.select(q, [cands[c] for c in which], len(which), weights, om, mode=O.MODE_NO_PRUNING,
                       progress=lambda l, n: print(f"[{time.time() - t0:7.0f} s] {operand}: layer {l} done", flush=True))
        by = {which[int(i)]: float(s) for i, s in zip(sel.idx, sel.scores)}
        scores[operand] = [by[c] for c in which]
    out = {
        "_about": "Full-depth scores from oracle/prism_oracle.py select() without pruning, operand = exact and operand = f16 "
                  "(every contraction operand rounded to IEEE half, everything else fp64); written by "
                  "tests/golden/make_fullsize_goldens.py.  Scores are repr() of fp64 values.",
        "workload": workload, "w4": w4, "seed": w.seed, "cands": [int(c) for c in which],
        "exact": [repr(x) for x in scores["exact"]], "half": [repr(x) for x in scores["f16"]],
        "oracle_seconds": round(time.time() - t0),
    }
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), f"half_operand_noise_{workload}{'_w4' if w4 else ''}.json")
    with open(path, "w") as f:
        f.write("{\n" + ",\n".join(f"{json.dumps(k)}: {json.dumps(v)}" for k, v in out.items()) + "\n}\n")
    print(f"wrote {path}: half - exact = {[f'{h - e:+.3e}' for h, e in zip(scores['f16'], scores['exact'])]}")


def main(workload: str, mode: str):
    w4 = mode.endswith("_w4")
    routing = mode[:-3] if w4 else mode
    w = W.WORKLOADS[workload]
    m = w.model
    t0 = time.time()
    say = lambda s: print(f"[{time.time() - t0:7.0f} s] {s}", flush=True)
    weights = _weights(w, w4)
    q, cands = W.make_tokens(w)
    om = O.Model(m.n_layers, m.hidden, m.n_q_heads, m.n_kv_heads, m.head_dim, m.ffn, m.vocab, m.rms_eps, m.rope_base,
                 m.qk_norm, "exact")
    say(f"{workload} {mode}: inputs drawn, {sum(len(q) + len(c) for c in cands)} tokens")
    sel = O.select(q, cands, w.K, weights, om, checkpoints=w.checkpoints, n_clusters=w.n_clusters, tau=w.cv_threshold,
                   mode=MODES[routing], progress=lambda l, n: say(f"layer {l} done, {n} live"))
    events = []
    for ev in sel.events:
        events.append({
            "layer": int(ev.layer), "live": [int(c) for c in ev.live], "scores": [repr(float(s)) for s in ev.scores],
            "gate": bool(ev.gate), "pruned": bool(ev.pruned),
            "fate": None if ev.fate is None else [int(f) for f in ev.fate],
            "keep": None if ev.keep is None else [int(k) for k in ev.keep],
        })
    out = {
        "_about": "Complete run of oracle/prism_oracle.py select() (fp64, operand = exact) on the seeded synthetic "
                  "workload; written by tests/golden/make_fullsize_goldens.py, which calls only the oracle and the "
                  "input generator.  Scores are repr() of fp64 values.",
        "workload": workload, "mode": mode, "seed": w.seed, "K": w.K, "n_cands": w.n_cands,
        "checkpoints": list(w.checkpoints), "n_clusters": w.n_clusters, "tau": w.cv_threshold,
        "layers_run": int(sel.layers_run), "token_layers": int(sel.token_layers),
        "events": events, "idx": [int(i) for i in sel.idx], "scores": [repr(float(s)) for s in sel.scores],
        "oracle_seconds": round(time.time() - t0),
    }
    with open(golden_path(workload, mode), "w") as f:           # one key per line, one event per line
        f.write("{\n")
        for k, v in out.items():
            if k == "events":
                f.write('"events": [\n' + ",\n".join(json.dumps(e) for e in v) + "\n],\n")
            else:
                f.write(f"{json.dumps(k)}: {json.dumps(v)}" + (",\n" if k != "oracle_seconds" else "\n"))
        f.write("}\n")
    say(f"wrote {golden_path(workload, mode)}: survivors {[int(np.sum(e['keep'])) for e in events if e['keep']]}, "
        f"top-K {out['idx']}")


if __name__ == "__main__":
    if len(sys.argv) > 3 and sys.argv[2].startswith("half_noise"):
        half_noise(sys.argv[1], sys.argv[2].endswith("_w4"), [int(c) for c in sys.argv[3].split(",")])
    else:
        main(sys.argv[1], sys.argv[2] if len(sys.argv) > 2 else "drop_only")
