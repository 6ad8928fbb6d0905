#!/usr/bin/env python3
"""Benchmark of the Top-K+phi decode step on one MI355X.

Workload: the Llama-3.2-3B-shaped single layer at 128K context and a 1 % budget
(24 query / 8 KV heads, head_dim 128, d_phi 128, 4 sink + 64 tail anchors, K = 1310), bf16
K/V with fp32 accumulation, synthetic seeded inputs.  One "step" is one tkphi_decode call
on one layer (score pass over the mid-region, Top-K selection, exact branch + subtraction sums
over the retrieved tokens, phi_q and the summary terms, merge).  The steps rotate over several distinct resident layers so that the keys
are really streamed from HBM and not served by the 256 MB last-level cache.  The summary
build (prefill side, once per prefix) is timed separately and reported under "build".

Prints one JSON line (rank 0; this build is single-GPU).
"""
from __future__ import annotations

import argparse
import concurrent.futures
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16
PROFILE = os.path.join(ROOT, "profiles", "decode_and_build_l3b_128k.md")


def measured_traffic(workload: str, budget_bp: int, kernel: str):
    """HBM bytes per launch of the dominant kernel as the tracked rocprofv3 --pmc summary states them (a line
    `TRAFFIC <workload> <budget_bp> <kernel> fetched=<bytes> written=<bytes>`), or None if it has no such line."""
    try:
        with open(PROFILE) as f:
            for line in f:
                t = line.split()
                if len(t) >= 6 and t[0] == "TRAFFIC" and t[1] == workload and t[2] == str(budget_bp) and t[3] == kernel:
                    kv = dict(x.split("=") for x in t[4:6])
                    return float(kv["fetched"]) + float(kv["written"])
    except (OSError, ValueError, KeyError):
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="l3b_128k")
    ap.add_argument("--budget-bp", type=int, default=100)
    ap.add_argument("--rotate", type=int, default=8, help="distinct resident layers the steps rotate over")
    ap.add_argument("--cache-features", action="store_true",
                    help="build stores the key features, decode gathers them instead of recomputing (not the headline)")
    ap.add_argument("--mlp-d-emb", type=int, default=0,
                    help="width of the one-block ReZero MLP feature maps (512 in the paper's appendix); 0 = the "
                         "exp-affine maps of the headline.  Implies the feature cache unless --mlp-recompute")
    ap.add_argument("--mlp-recompute", action="store_true",
                    help="MLP maps without a feature cache: decode recomputes the features of the retrieved keys")
    ap.add_argument("--select-mode", type=int, default=0, choices=[0, 1, 2],
                    help="tkphi_tuning::select_mode: 0 = the library's choice, 1 = spill pipeline, 2 = filtered pipeline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run plain 256 MiB device copies (a known-size kernel to scale rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters with)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; --gpus N with N > 1 is not supported "
              "(no collectives or sharding are part of it).", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2604_05438_amd import binding as B
    from paper_2604_05438_amd import harness as H
    from paper_2604_05438_amd import inputs as I

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = I.WORKLOADS[args.workload]
    cfg = H.config_of(w, cache_features=(not args.mlp_recompute) if args.mlp_d_emb else args.cache_features, d_emb=args.mlp_d_emb,
                      tuning={"select_mode": args.select_mode} if args.select_mode else None)
    esz = 2 if w.dtype == "bf16" else 4

    # ---- inputs, resident in HBM before anything is timed --------------------------------
    # single-layer workloads: `rotate` distinct layers, one problem per call;
    # model-level workloads: every (sequence, layer) problem of the model in ONE call.
    t0 = time.time()
    model_level = w.n_layers > 1
    if model_level:
        lens = I.ragged_lengths(w)
        pairs = [(layer, seq) for layer in range(w.n_layers) for seq in range(w.n_seqs)]
        Ls = [int(lens[seq]) for _, seq in pairs]
    else:
        pairs = [(r, 0) for r in range(args.rotate)]
        Ls = [w.L] * len(pairs)
    Ks = [I.mid_budget(L, args.budget_bp, w.n_sink, w.n_tail) for L in Ls]
    n_keep = 1 if model_level else len(pairs)           # host copies kept for the CPU baseline
    layers, dev_layers = [], []
    with concurrent.futures.ThreadPoolExecutor(max_workers=8) as ex:
        def make(a):
            P = I.make_layer(w, layer=a[0][0], seq=a[0][1], L=a[1])
            if args.mlp_d_emb:
                P["mlp"] = I.make_mlp_phi(w, layer=a[0][0], d_emb=args.mlp_d_emb)
            return P

        gen = ex.map(make, zip(pairs, Ls))
        for P in gen:
            if len(layers) < n_keep:
                layers.append(P)
            dev_layers.append({k: (H.to_device(v) if isinstance(v, np.ndarray) and k != "needle_pos" else v)
                               for k, v in P.items()})
    if model_level:
        batches = [H.Batch(cfg, dev_layers, Ks, diag=True)]
        probs_per_step = len(pairs)
    else:
        batches = [H.Batch(cfg, [P], [k], diag=True) for P, k in zip(dev_layers, Ks)]
        probs_per_step = 1
    del dev_layers
    L, K = Ls[0], Ks[0]
    mids = [max(0, l - w.n_sink - w.n_tail) for l in Ls]
    n_mid = sum(mids) if model_level else mids[0]       # mid tokens scanned by one step
    sum_K = sum(Ks) if model_level else K
    t_gen = time.time() - t0
    stream = torch.cuda.current_stream()

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- build (prefill side), timed on its own ------------------------------------------
    for b in batches:
        b.build()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record(stream)
    for b in batches:
        b.build()
    e1.record(stream)
    torch.cuda.synchronize()
    build_ms = e0.elapsed_time(e1) / len(batches)                      # per call
    build_bytes = w.n_kv_heads * n_mid * w.d_head * esz * 2            # K and V rows of M, once
    build_flops = w.n_kv_heads * n_mid * (2 * w.d_phi * w.d_head + 2 * w.d_phi * (w.d_head + 1))
    if args.mlp_d_emb:      # stem, two hidden contractions, output layer, then Phi^T [V 1]; one bf16 pass each
        E = args.mlp_d_emb
        build_flops = w.n_kv_heads * n_mid * (2 * (w.d_head * E + 2 * E * E + w.d_phi * E) + 2 * w.d_phi * (w.d_head + 1))

    # ---- decode: W warm-up steps, then exactly K timed steps ------------------------------
    for i in range(args.warmup):
        batches[i % len(batches)].decode()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    t_wall = time.perf_counter()
    e0.record(stream)
    for i in range(args.steps):
        batches[i % len(batches)].decode()
    e1.record(stream)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t_wall) * 1e3
    ms_per_step = e0.elapsed_time(e1) / args.steps
    assert all(b.status() == 0 for b in batches)

    # ---- spread of single steps (each between its own pair of events; not what `value` is made of) ------
    pairs_ev = [(ev(), ev()) for _ in range(args.steps)]
    for i, (a, b_) in enumerate(pairs_ev):
        a.record(stream)
        batches[i % len(batches)].decode()
        b_.record(stream)
    torch.cuda.synchronize()
    single = np.array([a.elapsed_time(b_) * 1e3 for a, b_ in pairs_ev])
    step_us_dist = {"median": float(np.median(single)), "p10": float(np.percentile(single, 10)),
                    "p90": float(np.percentile(single, 90)), "n": int(single.size)}

    # ---- cache-warm figure: the same resident problem(s) every step (the 256 MB last-level cache keeps what fits) ----
    for i in range(max(args.warmup, 2)):
        batches[0].decode()
    torch.cuda.synchronize()
    c0, c1 = ev(), ev()
    c0.record(stream)
    for i in range(args.steps):
        batches[0].decode()
    c1.record(stream)
    torch.cuda.synchronize()
    cache_warm_step_us = c0.elapsed_time(c1) / args.steps * 1e3

    # ---- the same steps replayed from HIP graphs (one graph per resident batch) -------------------------
    graph_replay_us = None
    try:
        graphs = []
        for b in batches:
            gr = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gr):
                b.decode()
            graphs.append(gr)
        for i in range(max(args.warmup, len(graphs))):
            graphs[i % len(graphs)].replay()
        torch.cuda.synchronize()
        g0, g1 = ev(), ev()
        g0.record(stream)
        for i in range(args.steps):
            graphs[i % len(graphs)].replay()
        g1.record(stream)
        torch.cuda.synchronize()
        graph_replay_us = g0.elapsed_time(g1) / args.steps * 1e3
        assert all(b.status() == 0 for b in batches)
        del graphs
    except RuntimeError as exc:                        # (capture refused: reported, not fatal)
        print(f"bench.py: graph capture failed: {exc}", file=sys.stderr)

    # ---- per-stage kernel durations: HIP events on the launch stream, same steps ---------
    stage = np.zeros(len(B.STAGES))
    for i in range(args.steps):
        stage += np.array(batches[i % len(batches)].decode_stage_times())
    stage /= args.steps
    stage_us = {n: float(v * 1e3) for n, v in zip(B.STAGES, stage)}

    # ---- how sharp / diffuse the synthetic attention is (by-products of the score pass; untimed) ----
    batches[0].decode(B.TKPHI_MODE_SUB | B.TKPHI_FLAG_DIAG)
    torch.cuda.synchronize()
    dg = np.stack([batches[0].result(i, "diag") for i in range(min(batches[0].n, 16))]).reshape(-1, B.TKPHI_DIAG_STRIDE)
    diagnostics = {"heads": int(dg.shape[0]), "H_mid_mean": float(dg[:, 0].mean()), "C_mid_mean": float(dg[:, 2].mean()),
                   "rho_res_mean": float(dg[:, 3].mean()), "rho_res_star_mean": float(dg[:, 4].mean()),
                   "log_Z_err_mean": float(np.nanmean(dg[:, 5]))}

    # algorithmic bytes of one step (what the method must move)
    bytes_scan = w.n_kv_heads * n_mid * w.d_head * esz                  # every mid key row, once per KV head
    bytes_gather = w.n_q_heads * sum_K * 2 * w.d_head * esz             # k and v rows of the retrieved tokens
    bytes_anchor = probs_per_step * w.n_kv_heads * (w.n_sink + w.n_tail) * 2 * w.d_head * esz
    bytes_const = probs_per_step * (w.n_kv_heads * w.d_phi * (w.d_head + 1) * 4          # S, u
                                    + (w.n_q_heads + w.n_kv_heads) * w.d_phi * w.d_head * esz)   # Wq, Wk
    bytes_step = bytes_scan + bytes_gather + bytes_anchor + bytes_const
    scan_kernel = "score_filtered_kernel" if stage_us.get("prep", 0.0) > 0 else "score_mid_kernel"
    scan_s = stage_us["score_mid"] * 1e-6
    achieved = bytes_scan / scan_s / 1e9

    out = {
        "metric": "mid_kv_tokens_per_s",
        "value": n_mid / (ms_per_step * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "decode_step_us": ms_per_step * 1e3,
        "step_us_dist": step_us_dist,
        "graph_replay_us": graph_replay_us,
        "cache_warm_step_us": cache_warm_step_us,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if w.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.n_q_heads}q/{w.n_kv_heads}kv heads, head_dim {w.d_head}, "
                               f"d_phi {w.d_phi}, sink {w.n_sink} + tail {w.n_tail}, budget {args.budget_bp} bp "
                               f"of the mid-region, "
                               + (f"{len(pairs)} (sequence, layer) problems per step ({w.n_seqs} sequences x "
                                  f"{w.n_layers} layers), L {min(Ls)}..{max(Ls)}, K {min(Ks)}..{max(Ks)}"
                                  if model_level else f"L {L}, K {K}, one layer per step"),
                   "rotating_layers": 0 if model_level else args.rotate, "problems_per_step": probs_per_step,
                   "budget_bp": args.budget_bp, "K": K, "L": L, "cache_features": bool(cfg.cache_features),
                   "select_mode": args.select_mode,
                   "phi": f"one-block ReZero MLP, d_emb {args.mlp_d_emb}" if args.mlp_d_emb else "exp-affine"},
        "step_hbm": {"algorithmic_bytes": bytes_step, "achieved_GBs": bytes_step / (ms_per_step * 1e-3) / 1e9,
                     "frac_of_peak": bytes_step / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS},
        "stage_us": stage_us,
        "wall_ms_per_step": wall_ms / args.steps,
        "roofline": {"kernel": scan_kernel, "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(w.name, args.budget_bp, scan_kernel),
                     "algorithmic_bytes_per_launch": bytes_scan},
        "build": {"ms_per_call": build_ms, "problems_per_call": probs_per_step, "algorithmic_bytes": build_bytes, "flops": build_flops,
                  "hbm_GBs": build_bytes / (build_ms * 1e-3) / 1e9,
                  "hbm_frac": build_bytes / (build_ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                  "mfma_TFLOPs": build_flops / (build_ms * 1e-3) / 1e12,
                  "mfma_frac": build_flops / (build_ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS},
        "diagnostics": diagnostics,
        "input_gen_s": t_gen,
    }

    # ---- CPU baseline: the float64 oracle, as it stands, on a bounded sample --------------
    if not args.no_cpu_baseline:
        sys.path.insert(0, os.path.join(ROOT, "tests"))
        import parity_utils as PU
        from oracle import tkphi_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        # sample: whole layer-steps (every query head) of the first layers of the rotation
        t_build = t_dec = 0.0
        n_done = 0
        worst = 0.0
        n_mid_done = 0
        for li, P in enumerate(layers):
            O = PU.oracle_inputs(P)
            t0 = time.perf_counter()
            fq, fk = PU.mlp_feature_fns(P)
            S, u = orc.build_summaries(O["K"], O["V"], O["Wk"], O["bk"], w.phi_in_scale, w.phi_norm_coef,
                                       w.n_sink, w.n_tail, phi_k_fns=fk)
            t_build += time.perf_counter() - t0
            t0 = time.perf_counter()
            res = orc.decode_layer(O["q"], O["K"], O["V"], S, u, O["Wq"], O["bq"], O["Wk"], O["bk"],
                                   w.phi_in_scale, w.phi_norm_coef, w.score_scale, w.n_sink, w.n_tail, Ks[li],
                                   phi_q_fns=fq, phi_k_fns=fk)
            t_dec += time.perf_counter() - t0
            n_done += 1
            n_mid_done += mids[li]
            bi, pi = (0, li) if model_level else (li, 0)
            batches[bi].decode()
            torch.cuda.synchronize()
            y = batches[bi].result(pi, "out")
            worst = max([worst] + [float(np.abs(y[g] - r["y"]).max()) for g, r in enumerate(res)])
            del O
            if t_dec + t_build > 20.0:
                break
        out["cpu_baseline"] = {
            "value": n_mid_done / t_dec, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"float64 numpy oracle, {n_done} whole layer-step(s) (all {w.n_q_heads} query heads) of the same "
                      f"workload: decode {t_dec:.2f} s (value = layers x mid tokens / decode seconds); the summary "
                      f"build of those layers took {t_build:.2f} s and is not in value",
            "decode_s": t_dec, "build_s": t_build,
        }
        out["parity_max_abs_vs_oracle"] = worst
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        src.fill_(1)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": 256 << 20, "bytes_written": 256 << 20, "copies": 4}
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
