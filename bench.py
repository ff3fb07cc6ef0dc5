#!/usr/bin/env python3
"""Benchmark of the MoE FFN layer forward over a verification batch of
T = B*(gamma+1) tokens on one MI355X.

A step is one pass of the whole hot path (route, permute, grouped gate/up +
SwiGLU, grouped down, shared expert, combine) over one batch of synthetic
tokens, with the weights already resident in HBM.  The default workload is the
largest benchmark shape, the DeepSeek-V3-shaped layer (256 experts, top-8,
22.6 GB of bf16 weights) at B=16, gamma=3 (T=64).  Weights are kept cold by
rotating over several replicas of the layer, as consecutive layers of a real
model would be.  The same line carries the other benchmark shapes at T=64, the
skewed-routing variant, every shape's (B, gamma) sweep and the compute-bound
extension points.

Prints ONE JSON line on stdout; progress goes to stderr.
"""
from __future__ import annotations

import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0      # MI355X HBM3E
MFMA_BF16_PEAK_TF = 2500.0  # MI355X dense bf16


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def layer_bytes(shape, n_active, T):
    """Algorithmic HBM bytes of one layer call: every activated weight once, plus
    the tokens in and out.  Intermediates are not counted."""
    w = n_active * shape.expert_bytes + shape.shared_bytes + shape.router_bytes
    return w + 2 * T * shape.d * 2


def gate_up_bytes(shape, n_active, T):
    """Algorithmic bytes of the gate/up kernel: the gate and up matrices of the
    activated experts and of the shared expert once, tokens in, activations out."""
    esz = shape.weight_bytes_per_element
    w = (n_active * 2 * shape.d * shape.inter + 2 * shape.d * shape.shared_inter) * esz
    if esz == 1:   # one fp32 scale per weight row
        w += (n_active * 2 * shape.inter + 2 * shape.shared_inter) * 4
    act = T * shape.d * 2 + (T * shape.top_k * shape.inter + T * shape.shared_inter) * 2
    return w + act


def down_bytes(shape, n_active, T):
    esz = shape.weight_bytes_per_element
    w = (n_active * shape.d * shape.inter + shape.d * shape.shared_inter) * esz
    if esz == 1:
        w += (n_active * shape.d + (shape.d if shape.shared_inter else 0)) * 4
    act = (T * shape.top_k * shape.inter + T * shape.shared_inter) * 2 \
        + (T * shape.top_k * shape.d + (T * shape.d if shape.shared_inter else 0)) * 4
    return w + act


def layer_flops(shape, T):
    return 6 * T * shape.top_k * shape.d * shape.inter + 6 * T * shape.d * shape.shared_inter \
        + 2 * T * shape.E * shape.d


class Runner:
    """Device-resident replicas of one layer plus per-T buffers."""

    def __init__(self, shape, host_w, n_rep):
        import torch
        import paper_2505_19645_amd as moesd
        self.torch, self.moesd, self.shape = torch, moesd, shape
        self.desc = moesd.make_desc(shape)
        import numpy as np
        dev = "cuda:0"
        base = {}
        for k, v in host_w.items():
            if v is None:
                base[k] = None
            elif k == "router_bias" or k.endswith("_scale"):
                base[k] = torch.from_numpy(v.astype(np.float32)).to(dev)
            elif v.dtype == np.uint8:                      # E4M3 codes
                base[k] = torch.from_numpy(np.ascontiguousarray(v)).to(dev)
            else:
                base[k] = torch.from_numpy(np.ascontiguousarray(v).view(np.int16)).to(dev)
        self.reps = [base]
        for _ in range(1, n_rep):
            self.reps.append({k: (None if v is None else v.clone()) for k, v in base.items()})
        self.wstructs = [moesd.make_weights(r) for r in self.reps]
        self.stream = torch.cuda.current_stream().cuda_stream

    def prepare(self, x_np):
        torch, moesd, s = self.torch, self.moesd, self.shape
        import numpy as np
        T = x_np.shape[0]
        self.T = T
        self.x = torch.from_numpy(np.ascontiguousarray(x_np).view(np.int16)).to("cuda:0")
        self.ws = torch.empty(moesd.moesd_workspace_bytes(self.desc, T), dtype=torch.uint8, device="cuda:0")
        self.out = torch.empty((T, s.d), dtype=torch.int16, device="cuda:0")
        self.n_active = torch.zeros(1, dtype=torch.int32, device="cuda:0")
        self.counts = torch.zeros(s.E, dtype=torch.int32, device="cuda:0")

    def step(self, i, events=None):
        self.moesd.moesd_moe_forward(self.desc, self.wstructs[i % len(self.wstructs)], self.x, self.T,
                                     self.out, self.ws, counts=self.counts, n_active=self.n_active,
                                     stream=self.stream, events=events)

    def time_steps(self, steps, warmup):
        """-> mean ms per step over exactly `steps` steps (events on our stream)."""
        from paper_2505_19645_amd.hiputil import Event
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        e0, e1 = Event(), Event()
        e0.record(self.stream)
        for i in range(steps):
            self.step(warmup + i)
        e1.record(self.stream)
        torch.cuda.synchronize()
        return e0.elapsed_ms(e1) / steps

    def time_stages(self, steps, warmup):
        """Same steps again with events at the stage boundaries of every forward.
        -> dict of mean ms: route_permute, gate_up, down, combine, total."""
        from paper_2505_19645_amd.hiputil import Event
        torch = self.torch
        evs = [[Event() for _ in range(5)] for _ in range(steps)]
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        for i in range(steps):
            self.step(warmup + i, events=[e.handle for e in evs[i]])
        torch.cuda.synchronize()
        names = ["route_permute", "gate_up", "down", "combine"]
        acc = {n: 0.0 for n in names}
        tot = 0.0
        for row in evs:
            for j, n in enumerate(names):
                acc[n] += row[j].elapsed_ms(row[j + 1])
            tot += row[0].elapsed_ms(row[4])
        out = {n: acc[n] / steps for n in names}
        out["total"] = tot / steps
        # per-forward samples for the spread (first to last event of each forward, and its gate/up stage)
        self.samples_ms = {"layer": [row[0].elapsed_ms(row[4]) for row in evs],
                           "gate_up": [row[1].elapsed_ms(row[2]) for row in evs]}
        return out


def pick_replicas(shape, T, budget_gb=24.0):
    import paper_2505_19645_amd as moesd
    n_exp = moesd.moesd_expected_active_experts(shape.E, shape.top_k, T)
    active = n_exp * shape.expert_bytes + shape.shared_bytes
    full = shape.E * shape.expert_bytes + shape.shared_bytes
    want = int(math.ceil(1.5e9 / max(active, 1.0))) + 1     # >= 1.5 GB of other weights between visits
    cap = max(2, int(budget_gb * 1e9 // full))
    return max(2, min(want, cap, 12))


SHORT_CURVE = [(1, 0), (2, 0), (4, 0), (8, 0), (16, 0), (8, 3), (16, 3), (32, 3), (64, 3), (128, 3), (128, 4)]
# compute-bound extension points outside the benchmark's own sweeps (rows per expert above the ridge)
MFMA_POINTS = {"mixtral-8x7b": (2048, 4096, 8192), "qwen2-57b-a14b": (2048, 4096, 8192)}


PAPER_BATCH_SIZES = [1, 2, 4, 8, 12, 16, 20, 24, 28, 32, 36, 40, 44, 48, 52, 56, 60, 80, 100]   # Appendix C.1


def layer_times(run, shape, Ts, steps, point_base):
    """Mean us per layer for each T (fresh token batch per T); -> {T: (us, n_active)}."""
    from paper_2505_19645_amd import synth
    out = {}
    for t in Ts:
        run.prepare(synth.make_tokens(shape, t, point=point_base + t))
        m = run.time_steps(steps, max(5, steps // 3))
        out[t] = (m * 1e3, int(run.n_active.item()))
    return out


def efficiency_rows(times, Bs, gammas):
    """Layer-level target efficiency t(B) / t(B*(gamma+1)) (Sec. 3.1) where both are measured."""
    rows = []
    for g in gammas:
        for b in Bs:
            if b in times and b * (g + 1) in times:
                rows.append({"B": b, "gamma": g, "target_efficiency": round(times[b][0] / times[b * (g + 1)][0], 4)})
    return rows


def peak_of(rows, g):
    cand = [r for r in rows if r["gamma"] == g]
    return max(cand, key=lambda r: r["target_efficiency"]) if cand else None


def mode_dense(args, shape, torch, moesd, synth):
    """Sec. 4.2 / Fig. 2(c) at layer level: the MoE layer against a dense FFN with the same
    activated flops (E = K = 1, intermediate size K * I), same kernels."""
    import dataclasses
    dense = dataclasses.replace(shape, name=shape.name + "-dense-equivalent", E=1, top_k=1,
                                inter=shape.top_k * shape.inter)
    Bs = [1, 2, 4, 8, 16, 32, 64, 128]
    gammas = (1, 3)
    Ts = sorted({b * (g + 1) for b in Bs for g in gammas} | set(Bs))
    res = {}
    for sh in (shape, dense):
        w = synth.make_layer(sh, threads=min(16, os.cpu_count() or 1))
        run = Runner(sh, w, pick_replicas(sh, 1))
        times = layer_times(run, sh, Ts, args.curve_steps, 7000)
        res[sh.name] = {"times_us": {str(t): round(v[0], 2) for t, v in times.items()},
                        "rows": efficiency_rows(times, Bs, gammas)}
        for g in gammas:
            pk = peak_of(res[sh.name]["rows"], g)
            log(f"[bench] {sh.name}: gamma={g} target efficiency peaks at B={pk['B']} ({pk['target_efficiency']:.2f}); "
                + " ".join(f"{r['B']}:{r['target_efficiency']:.2f}" for r in res[sh.name]["rows"] if r["gamma"] == g))
        del run, w
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "layer-level target efficiency t(B)/t(B*(gamma+1)), MoE vs dense FFN of equal activated flops",
                      "unit": "ratio", "n_gpus": 1, "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"{shape.name}-shaped MoE layer vs dense equivalent (E=K=1, I={dense.inter})"},
                      "moe": res[shape.name], "dense": res[dense.name]}))


def mode_ksweep(args, shape, torch, moesd, synth):
    """Sec. 4.3 / Fig. 3 at layer level: the same layer with K experts per token, K in
    {1, 2, 4, 8, 16, 32}, gamma in {2, 4}, the paper's 19 batch sizes."""
    import dataclasses
    gammas = (2, 4)
    Ts = sorted({b * (g + 1) for b in PAPER_BATCH_SIZES for g in gammas} | set(PAPER_BATCH_SIZES))
    w = synth.make_layer(shape, threads=min(16, os.cpu_count() or 1))
    run = Runner(shape, w, 2)
    out = []
    for K in (1, 2, 4, 8, 16, 32):
        if K > shape.E:
            continue
        sk = dataclasses.replace(shape, top_k=K)
        run.shape, run.desc = sk, moesd.make_desc(sk)
        times = layer_times(run, sk, Ts, args.curve_steps, 9000 + 100000 * K)
        rows = efficiency_rows(times, PAPER_BATCH_SIZES, gammas)
        entry = {"K": K, "rho": round(K / shape.E, 4), "T_thres_tau0.95": int(moesd.moesd_token_threshold(shape.E, K, 0.95)),
                 "rows": rows, "times_us": {str(t): round(v[0], 2) for t, v in times.items()}}
        for g in gammas:
            pk = peak_of(rows, g)
            entry[f"peak_gamma{g}"] = {"B": pk["B"], "target_efficiency": pk["target_efficiency"]}
        out.append(entry)
        log(f"[bench] K={K} (rho={K / shape.E:.3f}, T_thres={entry['T_thres_tau0.95']}): "
            + ", ".join(f"gamma={g}: peak at B={entry[f'peak_gamma{g}']['B']} "
                        f"({entry[f'peak_gamma{g}']['target_efficiency']:.2f})" for g in gammas))
    print(json.dumps({"metric": "layer-level target efficiency vs sparsity (K sweep)", "unit": "ratio", "n_gpus": 1,
                      "data": "synthetic", "dtype": "bf16",
                      "config": {"workload": f"{shape.name}-shaped MoE layer, K in 1..32, gamma in (2, 4), 19 batch sizes"},
                      "sweep": out}))


def mode_routing(args, shape, torch, moesd, synth):
    """Activated experts under routing variants, router only (moesd_route + moesd_permute): unconstrained,
    group-limited (8 groups, 4 kept, when E allows) and a skewed router; the measured mean count over independent
    batches against Eq. N(t) (Sec. 3.2) and against its per-expert form with probabilities measured on a
    separate sample."""
    import dataclasses
    import numpy as np
    dev = "cuda:0"
    variants = [("uniform", shape, 0.0)]
    if shape.E % 8 == 0 and shape.top_k <= 4 * (shape.E // 8):
        variants.append(("group-limited 8/4", dataclasses.replace(shape, n_group=8, topk_group=4), 0.0))
    variants.append(("skewed (bias std 1.0)", shape, 1.0))
    Ts = (1, 4, 16, 64, 256)
    n_sample, per_T = 8192, 4096
    out = []
    for label, sh, skew in variants:
        r = synth.make_router(sh, skew)
        desc = moesd.make_desc(sh)
        wr = torch.from_numpy(r["w_router"].view(np.int16)).to(dev)
        bias = None if r["router_bias"] is None else torch.from_numpy(r["router_bias"]).to(dev)

        def route(n, point):
            x = torch.from_numpy(synth.make_tokens(sh, n, point=point).view(np.int16)).to(dev)
            ids = torch.empty((n, sh.top_k), dtype=torch.int32, device=dev)
            w = torch.empty((n, sh.top_k), dtype=torch.float32, device=dev)
            ws = torch.empty(max(moesd.moesd_workspace_bytes(desc, n), 256), dtype=torch.uint8, device=dev)
            moesd.moesd_route(desc, x, wr, bias, n, ids, w, ws)
            return ids.cpu().numpy()

        p = np.bincount(route(n_sample, 7001).ravel(), minlength=sh.E) / float(n_sample)
        ids = route(per_T, 7002)
        rows = []
        for T in Ts:
            nb = per_T // T
            n_act = np.array([len(np.unique(ids[i * T:(i + 1) * T])) for i in range(nb)], np.float64)
            rows.append({"T": T, "batches": nb, "n_active_mean": round(float(n_act.mean()), 3),
                         "n_active_sem": round(float(n_act.std(ddof=1) / np.sqrt(nb)), 3) if nb > 1 else None,
                         "N_uniform": round(moesd.moesd_expected_active_experts(sh.E, sh.top_k, T), 3),
                         "N_measured_p": round(moesd.moesd_expected_active_experts_p(p.tolist(), T), 3)})
        out.append({"variant": label, "p_min": round(float(p.min()), 5), "p_max": round(float(p.max()), 5),
                    "p_uniform": round(sh.top_k / sh.E, 5), "rows": rows})
        log(f"[bench] {label}: " + ", ".join(f"T={r_['T']}: {r_['n_active_mean']} (uniform {r_['N_uniform']}, "
                                             f"per-expert {r_['N_measured_p']})" for r_ in rows))
    print(json.dumps({"metric": "activated experts vs Eq. N(t) under routing variants", "unit": "experts", "n_gpus": 1,
                      "data": "synthetic", "dtype": "f64",
                      "config": {"workload": f"{shape.name}-shaped router, {per_T} tokens cut into batches of T"},
                      "variants": out}))


def stored_traffic(key):
    """HBM bytes per launch of the expert kernels from earlier `rocprofv3 --pmc` runs of this command
    (FETCH_SIZE, WRITE_SIZE; summaries under profiles/): counters cannot be read from inside the run."""
    try:
        with open(os.path.join(ROOT, "paper_2505_19645_amd", "measured_traffic.json")) as f:
            return json.load(f).get(key)
    except OSError:
        return None


def measure_point(run, shape, B, gamma, steps, warmup, point=None, stages=True):
    """One (B, gamma) point of one layer: mean us per layer (cold weights), the stage times of a second,
    identical set of forwards, and the fractions of the HBM peak they amount to."""
    from paper_2505_19645_amd import synth
    T = B * (gamma + 1)
    x = synth.make_tokens(shape, T, point=100 * B + gamma if point is None else point)
    run.prepare(x)
    ms = run.time_steps(steps, warmup)
    n_active = int(run.n_active.item())
    lb = layer_bytes(shape, n_active, T)
    fl = layer_flops(shape, T)
    roof = max(lb / (HBM_PEAK_GBS * 1e9), fl / (MFMA_BF16_PEAK_TF * 1e12))
    out = {"B": B, "gamma": gamma, "T": T, "us": round(ms * 1e3, 2), "n_active": n_active,
           "N_model": round(run.moesd.moesd_expected_active_experts(shape.E, shape.top_k, T), 2),
           "max_rows_per_expert": int(run.counts.max().item()),
           "layer_bytes": lb, "layer_GBps": round(lb / (ms * 1e-3) / 1e9, 1),
           "layer_hbm_frac": round(lb / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
           "roofline_us": round(roof * 1e6, 2), "roofline_frac": round(roof / (ms * 1e-3), 4)}
    if stages:
        st = run.time_stages(steps, warmup)
        gub, dnb = gate_up_bytes(shape, n_active, T), down_bytes(shape, n_active, T)
        out["stages_us"] = {k: round(v * 1e3, 2) for k, v in st.items()}
        out["gate_up"] = {"bytes": gub, "GBps": round(gub / (st["gate_up"] * 1e-3) / 1e9, 1),
                          "hbm_frac": round(gub / (st["gate_up"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        out["down"] = {"bytes": dnb, "GBps": round(dnb / (st["down"] * 1e-3) / 1e9, 1),
                       "hbm_frac": round(dnb / (st["down"] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        out["routing_share"] = round(st["route_permute"] / st["total"], 4)
    return out, x


SWEEP_FIELDS = ["sweep", "B", "gamma", "T", "us", "n_active", "N_model", "Texp_model", "layer_hbm_frac", "roofline_us",
                "roofline_frac"]


class SweepLog:
    """Optional CSV of every sweep point, written as the run goes; a later run with the same file takes the
    points it already holds from it instead of measuring them again (an interrupted sweep resumes)."""

    def __init__(self, path):
        import csv
        self.path, self.have = path, {}
        if path and os.path.exists(path):
            with open(path, newline="") as f:
                for r in csv.DictReader(f):
                    self.have[(r["sweep"], int(r["B"]), int(r["gamma"]))] = r
        if path and not self.have:
            with open(path, "w", newline="") as f:
                csv.writer(f).writerow(SWEEP_FIELDS)

    def get(self, key, b, g):
        r = self.have.get((key, b, g))
        if r is None:
            return None
        out = {k: (int(r[k]) if k in ("B", "gamma", "T", "n_active") else float(r[k])) for k in SWEEP_FIELDS[1:]}
        return out

    def put(self, key, row):
        if not self.path:
            return
        import csv
        with open(self.path, "a", newline="") as f:
            csv.writer(f).writerow([key] + [row[k] for k in SWEEP_FIELDS[1:]])


def sweep(run, shape, pts, steps, log_csv=None, key=None):
    """Layer time over a (B, gamma) grid: us, measured and modelled activated experts, roofline fraction,
    and the layer-level target efficiency t(B) / t(B (gamma + 1)) (Sec. 3.1) where the gamma = 0 point exists."""
    rows = []
    key = key or shape.name
    for (b, g) in pts:
        r = log_csv.get(key, b, g) if log_csv else None
        if r is None:
            r, _ = measure_point(run, shape, b, g, steps, max(5, steps // 3), stages=False)
            r["Texp_model"] = round(run.moesd.moesd_expected_tokens_per_expert(shape.E, shape.top_k, r["T"]), 2)
            for k in ("layer_bytes", "layer_GBps", "max_rows_per_expert"):
                r.pop(k)
            if log_csv:
                log_csv.put(key, r)
        rows.append(r)
    by = {(c["B"], c["gamma"]): c["us"] for c in rows}
    for c in rows:
        if c["gamma"] > 0 and (c["B"], 0) in by:
            c["target_efficiency"] = round(by[(c["B"], 0)] / c["us"], 4)
    log(f"[bench] {shape.name} sweep, {len(rows)} points: "
        + " ".join(f"T={c['T']}:{c['us']:.0f}us({c['roofline_frac']:.2f})" for c in rows if c["gamma"] in (0, 3)))
    return rows


def fit_models(shape, rows, moesd):
    """The paper's forward-time form restricted to one layer (Sec. 3.3, Appendix C.2) fitted to a sweep, and
    the speed-up model of Sec. 3.1 / Alg. 1 fitted to layer-level speed-ups built from it."""
    from paper_2505_19645_amd import sdmodel
    out = {}
    ridge = MFMA_BF16_PEAK_TF * 1e12 / (HBM_PEAK_GBS * 1e9)
    k2_min_us = shape.expert_bytes / (HBM_PEAK_GBS * 1e9) * 1e6
    if len(rows) >= 6:
        mf = sdmodel.fit_layer_curve([c["T"] for c in rows], [c["n_active"] for c in rows], [c["us"] for c in rows],
                                     shape.E, shape.top_k, k2_min_us, ridge)
        out["model_fit"] = mf
        log(f"[bench] {shape.name}: t = c0 + c2*N + c3*G(Texp): c0={mf['c0_us']:.1f} us, c2={mf['c2_us_per_expert']:.2f} "
            f"us/expert ({mf['c2_over_k2_min']:.2f} x k2_min), c3={mf['c3_us']:.2f}, mean rel err {mf['mean_rel_err']:.3f}")
    times_by_T = {}
    for c in rows:
        times_by_T.setdefault(c["T"], c["us"])
    if len(times_by_T) >= 8:
        assume = {"alpha": 0.8, "draft_over_target": 0.1, "reject_over_target": 0.01, "verify_tokens": "B*(gamma+1)"}
        pts = sdmodel.layer_speedups_from_curve(times_by_T, gammas=(1, 3), alpha=assume["alpha"],
                                                draft_ratio=assume["draft_over_target"],
                                                reject_ratio=assume["reject_over_target"])
        if len(pts) >= 10:
            bias_min = (shape.shared_bytes + shape.router_bytes) / (HBM_PEAK_GBS * 1e9) * 1e6
            fit = sdmodel.fit_speedup([r["B"] for r in pts], [r["gamma"] for r in pts], shape.top_k, shape.E,
                                      [r["sigma"] for r in pts], [r["speedup"] for r in pts], ridge,
                                      bias_min=max(bias_min, 1e-3), k2_min=k2_min_us, t_rej_max=max(times_by_T.values()))
            best = {}
            for r, pr in zip(pts, fit["pred"]):
                r["model"] = round(float(pr), 4)
                for k in ("speedup", "sigma", "target_efficiency"):
                    r[k] = round(r[k], 4)
                g = r["gamma"]
                if g not in best or r["target_efficiency"] > best[g]["target_efficiency"]:
                    best[g] = r
            out["sd_speedup_model"] = {
                "assumptions": assume, "points": pts, "params": {k: round(v, 5) for k, v in fit["params"].items()},
                "mean_rel_err": round(fit["mean_rel_err"], 4), "max_rel_err": round(fit["max_rel_err"], 4),
                "best_target_efficiency": {str(g): {"B": r["B"], "value": r["target_efficiency"]} for g, r in best.items()},
                "T_thres_tau0.95": int(moesd.moesd_token_threshold(shape.E, shape.top_k, 0.95))}
            log(f"[bench] {shape.name}: speed-up model over {len(pts)} (B, gamma) points, mean rel err "
                f"{fit['mean_rel_err']:.3f}; " + ", ".join(f"gamma={g}: target efficiency peaks at B={r['B']} "
                                                          f"({r['target_efficiency']:.2f})" for g, r in sorted(best.items())))
    return out


def device_fp8_weights(shape, torch, synth, np):
    """E4M3 expert weights drawn on the device (timing only: values do not affect time); the router, which
    decides the routing, is the canonical one.  Gaussian draws scaled so that a row's 3.5-sigma lands on 448."""
    dev = "cuda:0"
    g = torch.Generator(device=dev)
    g.manual_seed(shape.seed + 8)
    r = synth.make_router(shape)
    sh = synth.make_shared(dataclasses_replace(shape, shared_inter=0))
    w = {"w_router": torch.from_numpy(r["w_router"].view(np.int16)).to(dev), "router_bias": None,
         "w_shared_gate": None}
    if shape.shared_gate:
        w["w_shared_gate"] = torch.from_numpy(synth.normal_bf16(shape.seed, "w_shared_gate", 0, (shape.d,), 0.02)
                                              .view(np.int16)).to(dev)

    def codes(rows, cols):
        out = torch.empty((rows, cols), dtype=torch.uint8, device=dev)
        step = max(1, (1 << 26) // cols)
        for r0 in range(0, rows, step):
            n = min(step, rows - r0)
            out[r0:r0 + n] = (torch.randn(n, cols, device=dev, generator=g) * 128.0).clamp_(-448.0, 448.0) \
                .to(torch.float8_e4m3fn).view(torch.uint8)
        return out

    E, I, d, S = shape.E, shape.inter, shape.d, shape.shared_inter
    for name, rows, cols, fan in (("w_gate", E * I, d, d), ("w_up", E * I, d, d), ("w_down", E * d, I, I),
                                  ("ws_gate", S, d, d), ("ws_up", S, d, d), ("ws_down", d, S, S)):
        if rows == 0 or cols == 0:
            w[name] = w[name + "_scale"] = None
            continue
        w[name] = codes(rows, cols)
        w[name + "_scale"] = torch.full((rows,), float(fan) ** -0.5 / 128.0, dtype=torch.float32, device=dev)
    del sh
    return w


def dataclasses_replace(shape, **kw):
    import dataclasses
    return dataclasses.replace(shape, **kw)


def fp8_points(shape, torch, moesd, synth, np, Ts, steps, bf16_us):
    """The same layer with its expert weights as E4M3 codes and one fp32 scale per output row: layer time against
    the bf16 layer's and against the floor of the expert-loading term at one byte per weight (Appendix C.2)."""
    q = dataclasses_replace(shape, name=shape.name + "-fp8", weight_format=1)
    dw = device_fp8_weights(q, torch, synth, np)
    run = Runner.__new__(Runner)
    run.torch, run.moesd, run.shape = torch, moesd, q
    run.desc = moesd.make_desc(q)
    n_rep = 2 if q.E * q.expert_bytes > 4e9 else 3
    run.reps = [dw] + [{k: (None if v is None else v.clone()) for k, v in dw.items()} for _ in range(n_rep - 1)]
    run.wstructs = [moesd.make_weights(r) for r in run.reps]
    run.stream = torch.cuda.current_stream().cuda_stream
    rows = []
    for T in Ts:
        r, _ = measure_point(run, q, T, 0, steps, max(5, steps // 3), point=100 * T)
        r.pop("B"), r.pop("gamma")
        r["bf16_us"] = bf16_us.get(T)
        if r["bf16_us"]:
            r["speedup_over_bf16"] = round(r["bf16_us"] / r["us"], 3)
        rows.append(r)
    out = {"workload": f"{shape.name}-shaped layer, E4M3 expert weights with row scales (router from the seeded "
                       "generator, expert codes drawn on the device: timing only)",
           "k2_min_us_per_expert": round(q.expert_bytes / (HBM_PEAK_GBS * 1e9) * 1e6, 3), "points": rows}
    if len(rows) >= 2 and rows[-1]["n_active"] > rows[0]["n_active"]:
        k2 = (rows[-1]["us"] - rows[0]["us"]) / (rows[-1]["n_active"] - rows[0]["n_active"])
        out["k2_us_per_expert"] = round(k2, 3)
        out["k2_over_k2_min"] = round(k2 / out["k2_min_us_per_expert"], 3)
    log(f"[bench] {q.name}: " + ", ".join(f"T={r['T']}: {r['us']:.0f} us (bf16 {r['bf16_us']}, layer {r['layer_hbm_frac']:.2f} "
                                            f"of the HBM peak on 1-byte weights)" for r in rows)
        + (f"; k2 = {out['k2_us_per_expert']} us per expert = {out['k2_over_k2_min']} x its floor" if "k2_us_per_expert" in out else ""))
    del run, dw
    torch.cuda.empty_cache()
    return out


def mfma_points(run, shape, Ts, steps=8, warmup=3):
    """Compute-bound points: layer and gate/up kernel against the bf16 MFMA peak."""
    from paper_2505_19645_amd import synth
    rows = []
    for T in Ts:
        run.prepare(synth.make_tokens(shape, T, point=T))
        ms = run.time_steps(steps, warmup)
        st = run.time_stages(steps, warmup)
        fl = layer_flops(shape, T)
        gu_fl = 4 * T * shape.top_k * shape.d * shape.inter + 4 * T * shape.d * shape.shared_inter
        dn_fl = 2 * T * shape.top_k * shape.d * shape.inter + 2 * T * shape.d * shape.shared_inter
        rows.append({"T": T, "us_per_layer": round(ms * 1e3, 1),
                     "layer_TFLOPs": round(fl / (ms * 1e-3) / 1e12, 1),
                     "layer_frac_of_peak": round(fl / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, 4),
                     "gate_up_us": round(st["gate_up"] * 1e3, 1),
                     "gate_up_TFLOPs": round(gu_fl / (st["gate_up"] * 1e-3) / 1e12, 1),
                     "gate_up_frac_of_peak": round(gu_fl / (st["gate_up"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, 4),
                     "down_us": round(st["down"] * 1e3, 1),
                     "down_frac_of_peak": round(dn_fl / (st["down"] * 1e-3) / 1e12 / MFMA_BF16_PEAK_TF, 4),
                     "n_active": int(run.n_active.item()), "max_rows_per_expert": int(run.counts.max().item())})
        log(f"[bench] {shape.name} T={T}: {rows[-1]['us_per_layer']} us/layer, {rows[-1]['layer_TFLOPs']} TFLOP/s "
            f"({rows[-1]['layer_frac_of_peak']:.1%} of bf16 peak); gate/up kernel {rows[-1]['gate_up_frac_of_peak']:.1%}, "
            f"down {rows[-1]['down_frac_of_peak']:.1%}")
    return rows


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--mode", choices=["headline", "dense", "ksweep", "routing"], default="headline",
                    help="headline: the benchmark line; dense: MoE vs dense-equivalent target efficiency; "
                         "ksweep: target efficiency for K = 1..32 (use --config qwen2-57b-a14b); "
                         "routing: activated experts under routing variants (use --config deepseek-v3)")
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", default="deepseek-v3", help="the headline shape")
    ap.add_argument("--B", type=int, default=16)
    ap.add_argument("--gamma", type=int, default=3)
    ap.add_argument("--skew", type=float, default=0.0, help="std of the per-expert logit bias of the headline shape")
    ap.add_argument("--others", choices=["all", "none"], default="all",
                    help="all: also the other benchmark shapes at the same (B, gamma), the skewed variant, "
                         "every shape's sweep and the compute-bound points; none: the headline shape only")
    ap.add_argument("--curve", choices=["none", "short", "full"], default="full",
                    help="the (B, gamma) sweep of each shape: the benchmark's full grid, a short one, or none")
    ap.add_argument("--curve-steps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--replicas", type=int, default=0)
    ap.add_argument("--no-mfma-point", action="store_true", help="skip the compute-bound extension points")
    ap.add_argument("--no-fp8", action="store_true", help="skip the points with E4M3 expert weights")
    ap.add_argument("--sweep-csv", default="", help="write every sweep point to this CSV as the run goes; points the "
                                                    "file already holds are not measured again (resume)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 1 GiB device copy (known traffic) for scaling rocprofv3 --pmc byte counters")
    args = ap.parse_args()

    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU; the layer is not sharded across GPUs "
            "(how it would shard by expert parallelism is described in the design notes only). Use --gpus 1.")
        sys.exit(2)

    import dataclasses
    import numpy as np
    import torch
    import paper_2505_19645_amd as moesd
    from paper_2505_19645_amd import synth

    if not torch.cuda.is_available():
        log("bench.py: no GPU visible; the HIP path has no CPU fallback")
        sys.exit(3)
    moesd.lib()
    shape = synth.PRESETS[args.config]
    T = args.B * (args.gamma + 1)
    log(f"[bench] {shape.name}: d={shape.d} E={shape.E} K={shape.top_k} I={shape.inter} "
        f"S={shape.shared_inter}; B={args.B} gamma={args.gamma} T={T} on {torch.cuda.get_device_name(0)}")

    if args.mode == "dense":
        return mode_dense(args, shape, torch, moesd, synth)
    if args.mode == "ksweep":
        return mode_ksweep(args, shape, torch, moesd, synth)
    if args.mode == "routing":
        return mode_routing(args, shape, torch, moesd, synth)

    threads = min(16, os.cpu_count() or 1)
    t_start = time.time()
    sweep_log = SweepLog(args.sweep_csv) if args.sweep_csv else None

    def curve_points(sh):
        if args.curve == "none":
            return []
        if args.curve == "full":
            return synth.sweep_points(sh.name)
        return [(t, 0) for t in (1, 4, 16, 64, 256)] if sh.name == "mixtral-8x7b" else SHORT_CURVE

    def open_layer(sh, skew):
        t0 = time.time()
        host_w = synth.make_layer(sh, skew_std=skew, threads=threads)
        pts = curve_points(sh)
        t_min = min([T] + [b * (g + 1) for b, g in pts])
        n_rep = args.replicas or pick_replicas(sh, t_min, budget_gb=100.0)
        run = Runner(sh, host_w, n_rep)
        log(f"[bench] {sh.name}: weights generated and uploaded in {time.time() - t0:.1f}s, {n_rep} replicas resident "
            f"({n_rep * (sh.E * sh.expert_bytes + sh.shared_bytes) / 1e9:.1f} GB)")
        return run, host_w, n_rep, pts

    if args.calibrate_copy:
        src = torch.ones(1 << 29, dtype=torch.int16, device="cuda:0")   # 1 GiB read + 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- headline point -------------------------------------------------------
    run, host_w, n_rep, pts = open_layer(shape, args.skew)
    head, x = measure_point(run, shape, args.B, args.gamma, args.steps, args.warmup)
    ms = head["us"] * 1e-3
    log(f"[bench] T={T}: {head['us']:.1f} us/layer, n_active={head['n_active']}, max m_e={head['max_rows_per_expert']}; "
        f"layer {head['layer_hbm_frac']:.3f} of the HBM peak; stages (us): "
        + ", ".join(f"{k}={v:.1f}" for k, v in head["stages_us"].items()))
    tr = stored_traffic(f"{shape.name}/B{args.B}/g{args.gamma}/skew{args.skew}")
    traffic = tr["gate_up"] if tr else None
    roofline = {"bound": "hbm", "kernel": "expert_stream_kernel<gate_up>", "achieved": head["gate_up"]["GBps"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": head["gate_up"]["hbm_frac"],
                "traffic": None if traffic is None else round(traffic["fetch_bytes"] + traffic["write_bytes"]),
                "traffic_source": None if traffic is None else "earlier rocprofv3 --pmc runs of this command (profiles/pmc_traffic_*)",
                "traffic_detail": traffic, "algorithmic_bytes": head["gate_up"]["bytes"],
                "avg_launch_us": head["stages_us"]["gate_up"],
                "layer_frac": head["layer_hbm_frac"], "down_kernel_frac": head["down"]["hbm_frac"]}

    def spread(xs):
        xs = sorted(xs)
        pick = lambda q: xs[min(len(xs) - 1, int(q * len(xs)))]
        return {"p10": round(pick(0.10) * 1e3, 2), "median": round(pick(0.50) * 1e3, 2),
                "p90": round(pick(0.90) * 1e3, 2)}
    spread_us = {k: spread(v) for k, v in run.samples_ms.items()}
    layer = {"bytes": head["layer_bytes"], "flops": layer_flops(shape, T), "hbm_roofline_us": head["roofline_us"],
             "achieved_GBps": head["layer_GBps"], "hbm_frac": head["layer_hbm_frac"], "n_active": head["n_active"],
             "n_active_model": head["N_model"],
             "k2_min_us_per_expert": round(shape.expert_bytes / (HBM_PEAK_GBS * 1e9) * 1e6, 3)}

    # ---- CPU baseline: the oracle as it stands, one forward of the same batch ----
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import moe as oracle
        oracle.lib()
        cores = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", os.cpu_count() or 1)))
        n_tok = T if layer_flops(shape, T) <= 4e11 else max(1, int(T * 4e11 / layer_flops(shape, T)))  # <= ~20 s of work
        log(f"[bench] oracle on the host ({cores} threads): routing of all {T} tokens, layer output of {n_tok} ...")
        t0 = time.time()
        ref = oracle.moe_forward(shape, host_w, x, tokens=None if n_tok == T else list(range(n_tok)))
        dt = time.time() - t0
        cpu = {"value": round(dt / n_tok * T * 1e6, 1), "unit": "us/layer", "cores": cores, "kind": "oracle",
               "sample": (f"one full forward of the same batch (T={T}, all tokens)" if n_tok == T else
                          f"routing of the whole batch (T={T}) and the layer output of its first {n_tok} tokens, "
                          f"scaled by {T}/{n_tok}") + f": {dt:.2f} s measured; fp64 plain C + OpenMP",
               "measured_s": round(dt, 3)}
        log(f"[bench] oracle: {dt:.2f}s for {n_tok} of {T} tokens; n_active={ref['n_active']}")
        assert ref["n_active"] == head["n_active"]

    # ---- the headline shape's sweep, then the other shapes -------------------------
    configs, sweeps, fits, mfma, fp8 = [], {}, {}, {}, {}
    FP8_TS = (1, 16, 64, 256)

    def bf16_times(run_, sh_, rows_):
        """bf16 layer times at the token counts of the fp8 comparison (from the sweep where it has them)."""
        have = {}
        for c in rows_ or []:
            if c["gamma"] == 0:
                have[c["T"]] = c["us"]
        for t in FP8_TS:
            if t not in have:
                have[t] = measure_point(run_, sh_, t, 0, args.curve_steps, 6, stages=False)[0]["us"]
        return have

    if pts:
        sweeps[shape.name] = sweep(run, shape, pts, args.curve_steps, sweep_log)
        fits[shape.name] = fit_models(shape, sweeps[shape.name], moesd)
    if shape.name in MFMA_POINTS and not args.no_mfma_point:
        mfma[shape.name] = mfma_points(run, shape, MFMA_POINTS[shape.name])
    head_bf16 = bf16_times(run, shape, sweeps.get(shape.name)) if not args.no_fp8 else None
    del run, host_w
    torch.cuda.empty_cache()
    if not args.no_fp8:
        fp8[shape.name] = fp8_points(shape, torch, moesd, synth, np, FP8_TS, args.curve_steps, head_bf16)

    if args.others == "all":
        for name in synth.PRESET_ORDER[1:]:
            sh = synth.PRESETS[name]
            if name == shape.name and args.skew == 0.0:
                continue
            orun, ow, onrep, opts = open_layer(sh, 0.0)
            c, _ = measure_point(orun, sh, args.B, args.gamma, args.steps, args.warmup)
            c.update(workload=f"{name}-shaped MoE layer, B={args.B}, gamma={args.gamma}, T={T}", weight_replicas=onrep,
                     k2_min_us_per_expert=round(sh.expert_bytes / (HBM_PEAK_GBS * 1e9) * 1e6, 3))
            configs.append(c)
            log(f"[bench] {name} T={T}: {c['us']:.1f} us/layer, layer {c['layer_hbm_frac']:.3f}, gate/up "
                f"{c['gate_up']['hbm_frac']:.3f}, down {c['down']['hbm_frac']:.3f} of the HBM peak, routing "
                f"{c['routing_share']:.1%} of the layer")
            if opts:
                sweeps[name] = sweep(orun, sh, opts, args.curve_steps, sweep_log)
                fits[name] = fit_models(sh, sweeps[name], moesd)
            if name == "qwen2-57b-a14b":
                # the skewed-routing variant: per-expert logit bias N(0, 1.5), same weights otherwise
                bias = synth.make_router(sh, 1.5)["router_bias"]
                bdev = torch.from_numpy(bias.astype(np.float32)).to("cuda:0")
                keep = [(r["router_bias"], wsx) for r, wsx in zip(orun.reps, orun.wstructs)]
                for r in orun.reps:
                    r["router_bias"] = bdev
                orun.wstructs = [moesd.make_weights(r) for r in orun.reps]
                c2, _ = measure_point(orun, sh, args.B, args.gamma, args.steps, args.warmup, point=9000 + T)
                c2.update(workload=f"{name}-shaped MoE layer, router bias N(0, 1.5) (skewed loads), B={args.B}, "
                                   f"gamma={args.gamma}, T={T}", weight_replicas=onrep)
                configs.append(c2)
                log(f"[bench] {name} skewed T={T}: {c2['us']:.1f} us/layer, n_active={c2['n_active']} "
                    f"(uniform model {c2['N_model']}), layer {c2['layer_hbm_frac']:.3f} of the HBM peak")
                if opts:
                    sk_pts = [(b, g) for (b, g) in opts if g in (0, 3)]
                    sweeps[name + "/skew1.5"] = sweep(orun, sh, sk_pts, args.curve_steps, sweep_log, key=name + "/skew1.5")
                for r, (b0, w0) in zip(orun.reps, keep):
                    r["router_bias"] = b0
                orun.wstructs = [k[1] for k in keep]
            if name in MFMA_POINTS and not args.no_mfma_point:
                mfma[name] = mfma_points(orun, sh, MFMA_POINTS[name])
            o_bf16 = bf16_times(orun, sh, sweeps.get(name)) if not args.no_fp8 else None
            del orun, ow
            torch.cuda.empty_cache()
            if not args.no_fp8:
                fp8[name] = fp8_points(sh, torch, moesd, synth, np, FP8_TS, args.curve_steps, o_bf16)
    log(f"[bench] whole run {time.time() - t_start:.0f}s")

    result = {
        "metric": "MoE-layer us at T=B*(gamma+1)", "value": head["us"], "unit": "us/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": f"{shape.name}-shaped MoE layer, B={args.B}, gamma={args.gamma}, T={T}",
                   "d": shape.d, "E": shape.E, "top_k": shape.top_k, "inter": shape.inter,
                   "shared_inter": shape.shared_inter, "skew_std": args.skew,
                   "weight_replicas": n_rep, "cold_weights": True},
        "roofline": roofline, "cpu_baseline": cpu, "layer": layer, "stages_us": head["stages_us"],
        "routing_share": head["routing_share"], "spread_us": spread_us,
        "configs": configs, "sweeps": sweeps, "fits": fits, "mfma_points": mfma, "fp8_weights": fp8,
    }
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
