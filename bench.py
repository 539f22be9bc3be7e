#!/usr/bin/env python3
"""Benchmark of the monolithic-forwarding hot path on one MI355X.

One "step" is one prism_select over the whole synthetic workload (pack + embed, every layer over the
live candidates, every pruning checkpoint, compaction, final top-K).  Weights and the context are
resident in HBM before the timed region; the tokens are handed over as host arrays, as the C ABI
defines (a few hundred KB).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4_8b]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA peak
KIND_NAMES = ["gemm_qkv", "gemm_o", "gemm_gate_up_swiglu", "gemm_down", "attention", "elementwise"]


def cpu_baseline(w, wt_dev, q, cands, token_layers_job: int, n_cands: int):
    """The oracle as it stands, timed on a bounded sample (about 15 s): eight candidates of median length through the
    first four layers plus their scoring, extrapolated by token-layers to the job the GPU ran (same pruning schedule)."""
    import numpy as np
    from oracle import prism_oracle as O
    from tests.helpers import oracle_model, to_f64
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    n_layers = min(4, w.model.n_layers)
    med = np.median([len(y) for y in cands])
    picks = [int(i) for i in np.argsort([abs(len(x) - med) for x in cands])[:8]]
    ow = {"embed": None, "final_norm": to_f64(wt_dev.final_norm), "w_yes": to_f64(wt_dev.w_yes), "w_no": to_f64(wt_dev.w_no),
          "layers": [{k: to_f64(v) for k, v in wt_dev.layers[l].items()} for l in range(n_layers)]}
    toks = [np.concatenate([q, cands[c]]) for c in picks]
    emb_rows = [to_f64(wt_dev.embed[t.tolist()]) for t in toks]
    om = oracle_model(w.model)
    t0 = time.perf_counter()
    for X in emb_rows:
        for l in range(n_layers):
            X = O.layer_forward(X, ow["layers"][l], om)
        O.head_score(X[-1], ow["final_norm"], ow["w_yes"], ow["w_no"], om.rms_eps)
    dt = time.perf_counter() - t0
    sample_token_layers = sum(len(t) for t in toks) * n_layers
    job_seconds = dt * token_layers_job / sample_token_layers
    return {"value": n_cands / job_seconds, "unit": "candidates/s", "cores": int(cores), "kind": "oracle",
            "sample": f"fp64 numpy oracle, candidates {picks} ({sum(len(t) for t in toks)} tokens) through layers 1-{n_layers} "
                      f"+ scoring: {dt:.2f} s, scaled by token-layers ({token_layers_job} in the pruned job / "
                      f"{sample_token_layers} in the sample)"}


def stored_traffic(workload: str, kernel: str):
    """HBM-side bytes per launch of the dominant kernel from the committed rocprofv3 counter summary, if the summary is
    for this workload and kernel; (None, reason) otherwise.  bench.py cannot run the profiler itself, so this is a STORED
    figure: the second return value says where it comes from."""
    rel = os.path.join("profiles", f"{workload}_gate_up_gemm_traffic.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, f"no stored counter summary ({rel})"
    kv = dict(l.split(":", 1) for l in open(path) if ":" in l and not l.startswith("#"))
    kv = {k.strip(): v.strip() for k, v in kv.items()}
    if kv.get("kernel") != kernel or kv.get("workload") != workload:
        return None, f"{rel} is for {kv.get('kernel')} on {kv.get('workload')}"
    return int(kv["fetch_bytes_per_launch"]) + int(kv["write_bytes_per_launch"]), \
        f"stored, not measured in this run: {rel} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of {kv.get('measured', 'unknown date')})"


def golden_scores(workload: str, mode: str):
    """Every scoring event of the oracle's complete run of this workload (tests/golden/, written by the oracle alone):
    {layer: {candidate: fp64 score}}, or None if no such run is stored."""
    path = os.path.join(ROOT, "tests", "golden", f"fullsize_{workload}_{mode}.json")
    if not os.path.exists(path):
        return None
    d = json.load(open(path))
    return {e["layer"]: {c: float(x) for c, x in zip(e["live"], e["scores"])} for e in d["events"]}, d["idx"]


def parity_record(rep, idx, gold):
    """Worst |device - oracle| over every score of every event that both runs took, and whether the top-K agrees."""
    if gold is None:
        return None
    by_layer, gold_idx = gold
    import numpy as np
    worst, n = 0.0, 0
    for e, layer in enumerate(rep.layer.tolist()):
        for c, ref in by_layer.get(layer, {}).items():
            g = rep.scores[e][c]
            if not np.isnan(g):
                worst = max(worst, abs(float(g) - ref))
                n += 1
    return {"worst_abs_score_err_vs_oracle": round(worst, 5), "scores_compared": n,
            "topk_equals_oracle": [int(i) for i in idx] == [int(i) for i in gold_idx],
            "oracle": "complete fp64 run stored under tests/golden/"}


def kind_table(reps):
    kinds = {}
    for k, name in enumerate(KIND_NAMES):
        ms = sum(r.kind_ms[k] for r in reps)
        fl = sum(r.kind_flops[k] for r in reps)
        n = sum(r.kind_launches[k] for r in reps)
        kinds[name] = {"launches": n, "ms": round(ms, 3), "tflops": round(fl / ms / 1e9, 1) if ms > 0 and fl > 0 else None}
    return kinds


def utilisation(reps):
    gemm_ms = sum(r.kind_ms[k] for r in reps for k in range(4))
    gemm_fl = sum(r.kind_flops[k] for r in reps for k in range(4))
    attn_ms = sum(r.kind_ms[4] for r in reps)
    attn_fl = sum(r.kind_flops[4] for r in reps)
    return {"layer_gemms": round(gemm_fl / gemm_ms / 1e9 / PEAK_BF16_TFLOPS, 4) if gemm_ms else None,
            "attention": round(attn_fl / attn_ms / 1e9 / PEAK_BF16_TFLOPS, 4) if attn_ms else None}


def by_pool_size(reps, tokens_per_cand=None):
    """Per-kind TFLOP/s of the layer kernels split by the rows (live tokens) a launch covered: the pool shrinks at every
    pruning event, so the same kernel runs at several sizes within one call."""
    import numpy as np
    out = {}
    for k in range(5):
        rows = {}
        for r in reps:
            sp = r.spans
            if sp is None:
                continue
            for m in np.unique(sp.rows[(sp.kind == k) & (sp.rows > 0)]):
                sel = (sp.kind == k) & (sp.rows == m) & (sp.flops > 0)
                if sel.any():
                    a = rows.setdefault(int(m), [0, 0.0, 0.0])
                    a[0] += int(sel.sum()); a[1] += float(sp.ms[sel].sum()); a[2] += float(sp.flops[sel].sum())
        out[KIND_NAMES[k]] = {(f"{m} rows" if not tokens_per_cand else f"{m // tokens_per_cand} candidates"):
                              {"launches": v[0], "avg_us": round(v[1] / v[0] * 1e3, 1), "tflops": round(v[2] / v[1] / 1e9, 1)}
                              for m, v in sorted(rows.items(), reverse=True) if v[1] > 0}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="cfg4_8b")
    ap.add_argument("--operand", default="f16", choices=["f16", "bf16"],
                    help="16-bit type of the matrix-core operands when the weights are bf16")
    ap.add_argument("--checkpoints", default="workload", choices=["workload", "every"],
                    help="pruning checks after the workload's layers (every 4th) or after every layer (Sec. 4.5)")
    ap.add_argument("--mode", default="drop-only", choices=["drop-only", "three-way"],
                    help="routing: drop-only (Sec. 7, the headline) or three-way with early termination (Sec. 4.1)")
    ap.add_argument("--tau", type=float, default=None, help="dispersion threshold (default: the workload's, 0)")
    ap.add_argument("--lean", action="store_true",
                    help="hidden-state offload + embedding-table cache (needs a chunked workload, e.g. cfg5_8b_stream)")
    ap.add_argument("--stream-slots", type=int, default=0, help="layer buffers of the streaming ring (default 2, as in the paper)")
    ap.add_argument("--w4", action="store_true", help="4-bit layer weights (quantised on the device before the timed region)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-unpruned", action="store_true")
    ap.add_argument("--no-bf16", action="store_true", help="skip the bf16-operand sub-record")
    ap.add_argument("--no-cfg5", action="store_true", help="skip the streamed + chunked 500-candidate sub-record (cfg4_8b only)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU; --gpus must be 1 (the path would shard by candidate: sequences never interact)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2510_15620_amd import binding as B
    from paper_2510_15620_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    w = W.WORKLOADS[args.workload]
    if args.checkpoints == "every" or args.tau is not None:
        import dataclasses
        w = dataclasses.replace(w, checkpoints=list(range(1, w.model.n_layers)) if args.checkpoints == "every" else w.checkpoints,
                                cv_threshold=w.cv_threshold if args.tau is None else args.tau)
    m = w.model
    t_gen = time.perf_counter()
    if w.stream_weights:
        dev = W.make_weights(w, "cuda")
        host_layers = [{k: v.to("cpu").pin_memory() for k, v in l.items()} for l in dev.layers]
        wt = W.Weights(dev.embed, host_layers, dev.final_norm)
        wt_for_oracle = dev
    else:
        wt = wt_for_oracle = W.make_weights(w, "cuda")
    if args.w4:
        class Q4:                             # the same weights with every layer matrix as a 4-bit blob
            pass
        q4 = Q4()
        q4.embed, q4.final_norm, q4.w_yes, q4.w_no = wt.embed, wt.final_norm, wt_for_oracle.w_yes, wt_for_oracle.w_no
        q4.layers = B.quantize_layers_w4(wt_for_oracle.layers)
        if w.stream_weights:
            q4.layers = [{k: v.to("cpu").pin_memory() for k, v in l.items()} for l in q4.layers]
        wt = q4
    if args.lean:
        class HostTable:                      # embedding table in pinned host memory, the two head rows on the device
            pass
        ht = HostTable()
        ht.embed, ht.layers, ht.final_norm = wt.embed.cpu().pin_memory(), wt.layers, wt.final_norm
        ht.w_yes, ht.w_no = wt_for_oracle.w_yes.clone(), wt_for_oracle.w_no.clone()
        wt = ht
    q, cands = W.make_tokens(w)
    torch.cuda.synchronize()
    t_gen = time.perf_counter() - t_gen
    opts = dict(checkpoints=w.checkpoints, cv_threshold=w.cv_threshold, n_clusters=w.n_clusters, chunk_cands=w.chunk_cands,
                hbm_cap_bytes=w.hbm_cap_bytes, stream_weights=w.stream_weights, operand=args.operand,
                offload_hidden=args.lean, embed_on_host=args.lean, w4=args.w4, stream_slots=args.stream_slots,
                mode=B.MODE_THREE_WAY if args.mode == "three-way" else B.MODE_DROP_ONLY)
    p = B.Prism(m, wt, **opts)

    for _ in range(args.warmup):
        p.select(q, cands, w.K, report=False)
    torch.cuda.synchronize()
    # Timed region: HIP-event spans only around the dominant kernel's launches (every span costs two event records on
    # the compute stream; with all kinds on that is about 1 % of the call).  The per-kind breakdown comes from extra,
    # untimed selects right after.
    DOM = 2        # the gate/up GEMM with the SwiGLU epilogue carries more than half of all flops
    dom_reps, step_ms = [], []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        ts = time.perf_counter()
        idx, scores, rep = p.select(q, cands, w.K, report=True, kinds=[DOM])      # synchronous: results are on the host
        step_ms.append((time.perf_counter() - ts) * 1e3)
        dom_reps.append(rep)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_step = wall / args.steps * 1e3
    rep = dom_reps[-1]
    reps = [p.select(q, cands, w.K, report=True, spans=4096)[2] for _ in range(2)]      # all kinds, not timed

    unpruned_ms = None
    if not args.no_unpruned:
        p0 = B.Prism(m, wt, **{**opts, "mode": B.MODE_NO_PRUNING})
        p0.select(q, cands, w.K, report=False)
        t1 = time.perf_counter()
        p0.select(q, cands, w.K, report=False)
        unpruned_ms = (time.perf_counter() - t1) * 1e3
        p0.destroy()

    # per-kernel-kind totals (HIP events around each launch on the compute stream): the dominant kernel over the timed
    # steps, all kinds over the two selects that follow them
    kinds = kind_table(reps)
    dom_ms = sum(r.kind_ms[DOM] for r in dom_reps)
    dom_fl = sum(r.kind_flops[DOM] for r in dom_reps)
    dom_n = sum(r.kind_launches[DOM] for r in dom_reps)
    achieved = dom_fl / dom_ms / 1e9
    op_t = "float" if m.dtype == "fp32" else args.operand
    traffic, traffic_source = stored_traffic(w.name, f"gemm_16_kernel<{op_t},256,256,2,2,2>")
    roofline = {"bound": "mfma", "kernel": f"gemm_16_kernel<{op_t},256,256,2,2,SWIGLU>", "achieved": round(achieved, 1),
                "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": round(achieved / PEAK_BF16_TFLOPS, 4),
                "traffic": traffic, "traffic_source": traffic_source,
                "flops_per_launch": dom_fl / dom_n, "avg_launch_ms": round(dom_ms / dom_n, 4), "launches": dom_n}
    mode_name = "three_way" if args.mode == "three-way" else "drop_only"
    plain_run = not args.w4 and args.checkpoints == "workload" and args.tau is None
    gold = golden_scores(w.name, mode_name) if plain_run else None
    const_len = len(set(len(c) for c in cands)) == 1

    # ---- the same workload with bf16 matrix-core operands (the headline runs IEEE half operands)
    bf16_rec = None
    if not args.no_bf16 and m.dtype != "fp32" and args.operand != "bf16":
        pb = B.Prism(m, wt, **{**opts, "operand": "bf16"})
        pb.select(q, cands, w.K, report=False)
        torch.cuda.synchronize()
        tb = time.perf_counter()
        breps = []
        for _ in range(2):
            bidx, bscores, brep = pb.select(q, cands, w.K, report=True, spans=4096)
            breps.append(brep)
        torch.cuda.synchronize()
        b_ms = (time.perf_counter() - tb) / 2 * 1e3
        pb.destroy()
        bf16_rec = {"topk_latency_ms": round(b_ms, 3), "candidates_per_s": round(w.n_cands / (b_ms / 1e3), 2), "steps": 2,
                    "kernels": kind_table(breps), "mfma_utilisation": utilisation(breps),
                    "survivors": brep.n_after.tolist(), "topk": bidx.tolist(), "parity": parity_record(brep, bidx, gold)}

    # ---- cfg 5: the same model streamed from pinned host memory, 500 candidates in chunks of 64, 24 GB cap
    cfg5_rec = None
    if args.workload == "cfg4_8b" and not args.no_cfg5 and plain_run and not args.lean:
        w5 = W.WORKLOADS["cfg5_8b_stream"]
        host_layers = [{k: v.to("cpu").pin_memory() for k, v in l.items()} for l in wt_for_oracle.layers]
        wt5 = W.Weights(wt_for_oracle.embed, host_layers, wt_for_oracle.final_norm)
        q5, cands5 = W.make_tokens(w5)
        p5 = B.Prism(w5.model, wt5, checkpoints=w5.checkpoints, cv_threshold=w5.cv_threshold, n_clusters=w5.n_clusters,
                     chunk_cands=w5.chunk_cands, hbm_cap_bytes=w5.hbm_cap_bytes, stream_weights=True, operand=args.operand)
        p5.select(q5, cands5, w5.K, report=False)
        torch.cuda.synchronize()
        t5 = time.perf_counter()
        reps5 = []
        step_ms5 = []
        for _ in range(2):
            ts = time.perf_counter()
            idx5, scores5, rep5 = p5.select(q5, cands5, w5.K, report=True)
            reps5.append(rep5)
            step_ms5.append(round((time.perf_counter() - ts) * 1e3, 1))
        torch.cuda.synchronize()
        ms5 = (time.perf_counter() - t5) / 2 * 1e3
        # one more select, not timed, with the copies of the streamed layers bracketed by events on the side stream
        rep5x = p5.select(q5, cands5, w5.K, report=True, kinds=[B.KIND_TRANSFERS])[2]
        p5.destroy()
        caller = int(wt_for_oracle.embed.numel() * 2 + wt_for_oracle.final_norm.numel() * 2)
        cfg5_rec = {"workload": f"cfg5_8b_stream: {w5.n_cands} candidates, {int(sum(len(c) + len(q5) for c in cands5))} tokens, "
                                f"layers streamed from pinned host memory ({'2' if not args.stream_slots else args.stream_slots} "
                                f"buffers), chunks of {w5.chunk_cands} candidates, K={w5.K}",
                    "topk_latency_ms": round(ms5, 3), "candidates_per_s": round(w5.n_cands / (ms5 / 1e3), 2), "steps": 2, "step_ms": step_ms5,
                    "stream_GBps": round(rep5.bytes_streamed / rep5.ms_total / 1e6, 1), "bytes_streamed": int(rep5.bytes_streamed),
                    # the host link while it is in use (HIP events on the side stream around each layer's copies), next to
                    # PCIe Gen5 x16's 64 GB/s; stream_GBps above is the same bytes over the whole call
                    "host_link": {"GBps_while_copying": round(rep5x.bytes_streamed / max(rep5x.ms_transfers, 1e-9) / 1e6, 1),
                                  "peak_GBps": 64.0, "ms_copying": round(rep5x.ms_transfers, 1),
                                  "measured_on": "one more select after the timed ones"},
                    "peak_hbm_bytes_library": int(rep5.peak_hbm_bytes), "caller_device_bytes": caller,
                    "hbm_cap_bytes": int(w5.hbm_cap_bytes), "under_cap": bool(rep5.peak_hbm_bytes + caller <= w5.hbm_cap_bytes),
                    "survivors": rep5.n_after.tolist(), "kernels": kind_table(reps5), "mfma_utilisation": utilisation(reps5),
                    "parity": parity_record(rep5, idx5, golden_scores(w5.name, "drop_only"))}
        del host_layers, wt5

    out = {
        "metric": "candidates/sec + top-K latency (ms), 8B-shaped reranker, 100 cands x 1024 tok"
                  if args.workload == "cfg4_8b" else f"candidates/sec + top-K latency (ms), {args.workload}",
        "value": round(w.n_cands / (ms_per_step / 1e3), 2), "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 3),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32" if m.dtype == "fp32" else args.operand,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: {m.n_layers} layers, hidden {m.hidden}, {m.n_q_heads}/{m.n_kv_heads} heads x {m.head_dim}, "
                               f"ffn {m.ffn}, vocab {m.vocab}; query {w.query_len} tok, {w.n_cands} candidates, "
                               f"{int(sum(len(c) + len(q) for c in cands))} tokens in all; K={w.K}; "
                               f"checkpoints after layers {w.checkpoints}; k={w.n_clusters} clusters, tau={w.cv_threshold}, {args.mode}; "
                               f"weights {'4-bit (groups of 128) expanded to ' + op_t if args.w4 else m.dtype}, matrix-core operands {op_t}, "
                               f"fp32 accumulation and residual",
                   "n_cands": w.n_cands, "K": w.K, "seed": w.seed, "chunk_cands": w.chunk_cands, "stream_weights": w.stream_weights},
        "topk_latency_ms": round(ms_per_step, 3), "topk_latency_ms_median": round(float(np.median(step_ms)), 3),
        "topk_latency_ms_min": round(min(step_ms), 3),
        "unpruned_latency_ms": None if unpruned_ms is None else round(unpruned_ms, 3),
        "gpu_ms": {"total": round(rep.ms_total, 3), "layers": round(rep.ms_layers, 3), "checks": round(rep.ms_checks, 3)},
        "survivors": {"layer": rep.layer.tolist(), "n_before": rep.n_before.tolist(), "n_after": rep.n_after.tolist()},
        "layers_run": int(rep.layers_run), "token_layers": int(rep.token_layers), "peak_hbm_bytes": int(rep.peak_hbm_bytes), "bytes_streamed": int(rep.bytes_streamed),
        "topk": idx.tolist(),
        "kernels_measured_on": "2 selects with spans on every kind, run right after the timed steps (the timed steps carry spans on the roofline kernel only)",
        "kernels": kinds,
        "kernels_by_pool_size": by_pool_size(reps, len(q) + len(cands[0]) if const_len else None),
        "mfma_utilisation": utilisation(reps),
        "roofline": roofline,
        "parity": parity_record(rep, idx, gold),
        "bf16_operands": bf16_rec,
        "cfg5": cfg5_rec,
        "weights_gen_s": round(t_gen, 1),
    }
    if args.lean:
        out["lean"] = {"bytes_hidden_moved": int(rep.bytes_hidden_moved), "embed_rows_hit": int(rep.embed_rows_hit),
                       "embed_rows_missed": int(rep.embed_rows_missed)}
    if w.stream_weights and rep.ms_total > 0:
        out["stream_GBps"] = round(rep.bytes_streamed / rep.ms_total / 1e6, 1)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, wt_for_oracle, q, cands, int(rep.token_layers), w.n_cands)
    p.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
