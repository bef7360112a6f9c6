#!/usr/bin/env python3
"""Benchmark of the MoE++ layer forward on one MI355X.

One "step" is one pass of the whole hot path (router + gating residual,
softmax/top-k, permutation, grouped SwiGLU FFN, combine with the
zero-computation experts) over one batch of seeded synthetic tokens that is
already resident in HBM.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload large]

The default workload is the large bf16 layer (T = 8 x 4096 tokens, D = 4096,
F = 5632, 16 FFN + 1 zero + 1 copy + 2 constant experts, top-2), the one the
roofline targets are quoted on.  The same shape with the zero-computation
experts disabled (vanilla MoE, 20 and 16 FFN experts) is timed right after it
for the throughput ratio, and the CPU oracle is timed on a bounded sample of
the same tokens as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import numpy as np

PEAK_BF16_MFMA_TFLOPS = 2500.0     # MI355X dense bf16, published
PEAK_HBM_GBS = 8000.0              # MI355X HBM3E, published
RIDGE = PEAK_BF16_MFMA_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)     # flop per byte


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def run_gpu(shape, inp, steps, warmup, capacity=None):
    """Timed steps of moepp_layer_forward on cuda:0.  Returns a dict.
    capacity = (gamma, tau): expert capacities of Eq.8 and the statistics of Eq.7 on."""
    import torch
    from paper_2410_07348_amd.torch_util import make_layer, to_device
    dev = to_device(shape, inp)
    L = make_layer(shape)
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"]) if shape.n_ffn else None
    for k in ("w1", "w3", "w2"):          # only the packed copy is needed from here on
        dev[k] = None
    L.set_router_bias(dev.get("bias"))
    cap = None
    if capacity:
        cap = L.capacity(shape.T, capacity[0], capacity[1])
        L.set_capacity(cap)
        L.set_balance(capacity[1])
    cv = dev["const_vecs"] if shape.n_const else None
    wc = dev["W_c"] if shape.n_const else None
    out = torch.empty((shape.T, shape.D), dtype=L.act_dtype, device=L.device)
    out_gate = torch.empty((shape.T, shape.N), dtype=torch.float32, device=L.device)

    def step():
        L.layer_forward(dev["x"], dev.get("prev_gate"), dev["W_g"], dev.get("W_res"), packed, cv,
                        wc, k=shape.k, out=out, out_gate=out_gate)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    L.set_timing(True)                    # HIP events around every kernel, on the launch stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern = L.get_timing()                 # per-kernel average over the timed steps (last 64)
    L.set_timing(False)
    # the same steps once more without the per-kernel events (two event records per
    # kernel cost about 20 us per step: 5 % of the T = 64 step, 0.4 % of the large one)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    plain = (time.perf_counter() - t1) / steps * 1e3
    r = L.get_routing()
    counts = r["counts"].cpu().numpy().copy()
    R = int(r["offsets"][-1].item()) if shape.n_ffn else 0
    res = {"ms_per_step": wall / steps * 1e3, "ms_per_step_no_events": plain, "kernel_ms": kern, "R": R,
           "counts": counts.tolist(), "cap": cap,
           "kept": L.get_kept().cpu().numpy().tolist(),
           "loss": float(L.get_balance()["loss"].item()) if capacity else None,
           "topk_idx": r["topk_idx"].cpu().numpy().copy(),
           "out": out, "layer": L, "dev": dev}
    return res


def run_chain(shape, inp, n_layers, steps, warmup):
    """n_layers layers back to back (the same weights, G(x^j) of one layer is the
    gating residual input of the next, Eq.6; the first has none), eagerly and as one
    HIP graph: what the launch overhead of the seven kernels per layer costs."""
    import torch
    from paper_2410_07348_amd.torch_util import make_layer, to_device
    dev = to_device(shape, inp)
    L = make_layer(shape)
    packed = L.pack_experts(dev["w1"], dev["w3"], dev["w2"]) if shape.n_ffn else None
    L.set_router_bias(dev.get("bias"))
    cv = dev["const_vecs"] if shape.n_const else None
    wc = dev["W_c"] if shape.n_const else None
    out = torch.empty((shape.T, shape.D), dtype=L.act_dtype, device=L.device)
    gates = [torch.empty((shape.T, shape.N), dtype=torch.float32, device=L.device) for _ in range(2)]

    def chain():
        for j in range(n_layers):
            L.layer_forward(dev["x"], gates[(j - 1) % 2] if j else None, dev["W_g"],
                            dev["W_res"] if j else None, packed, cv, wc, k=shape.k, out=out,
                            out_gate=gates[j % 2])

    def timed(fn):
        for _ in range(warmup):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    eager = timed(chain)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        chain()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            chain()
    torch.cuda.current_stream().wait_stream(side)
    replay = timed(graph.replay)
    return {"layers": n_layers, "eager_ms_per_layer": eager / n_layers,
            "graph_ms_per_layer": replay / n_layers}


def tau_sweep(model, steps, warmup):
    """Expert-forward time of one layer of a paper model (Tab.2 shape) against tau, with
    the expert capacities of Eq.8 and a router bias under which the zero-computation
    experts take N_ZC / (tau N_FFN + N_ZC) of the assignments, next to the vanilla MoE
    layer with the same FFN experts: the shape of the paper's Tab.3 on this GPU."""
    import torch
    from workloads import PAPER_MODELS, make_inputs
    base = PAPER_MODELS[model]
    rows = []
    van = base.with_(name=base.name + "_vanilla", n_zero=0, n_copy=0, n_const=0)
    gv = run_gpu(van, make_inputs(van), steps, warmup)
    kv = gv["kernel_ms"]
    t_van = kv["gemm1"] + kv["gemm2"] + kv["combine"]
    van_layer = gv["ms_per_step"]
    del gv
    torch.cuda.empty_cache()
    for tau in (0.1, 0.25, 0.5, 0.75, 1.0):
        s = base.with_(bias="tau%g" % tau)
        g = run_gpu(s, make_inputs(s), steps, warmup, capacity=(1.1, tau))
        k = g["kernel_ms"]
        t = k["gemm1"] + k["gemm2"] + k["combine"]
        slots = s.T * s.k
        rows.append({"tau": tau, "expert_forward_ms": t, "layer_ms": g["ms_per_step"],
                     "ffn_rows_fraction": g["R"] / slots,
                     "tab1_fraction": tau * s.n_ffn / (tau * s.n_ffn + s.n_zc),
                     "dropped_fraction": 1.0 - sum(g["kept"]) / slots,
                     "expert_throughput_increase_pct": 100.0 * (t_van / t - 1.0),
                     "layer_throughput_increase_pct": 100.0 * (van_layer / g["ms_per_step"] - 1.0)})
        log("tau", rows[-1])
        del g
        torch.cuda.empty_cache()
    return {"model": model, "T": base.T, "D": base.D, "F": base.F, "n_ffn": base.n_ffn,
            "n_zc": base.n_zc, "gamma": 1.1, "vanilla_expert_forward_ms": t_van,
            "vanilla_layer_ms": van_layer, "rows": rows,
            "paper_context": "Tab.3 (other hardware, whole models): 1B/(16+4)E expert-forward "
                             "throughput +111 % / +59 % / +30 % / +22 % / +15 % at tau = 0.1 / "
                             "0.25 / 0.5 / 0.75 / 1"}


def roofline_numbers(shape, g):
    """Algorithmic work per launch / measured duration, per kernel."""
    T, D, F, N, K, R = shape.T, shape.D, shape.F, shape.N, shape.k, g["R"]
    b = 2 if shape.act == "bf16" else 4
    km = g["kernel_ms"]
    out = {}
    if km["gemm1"] > 0:
        fl1, fl2 = 4.0 * D * F * R, 2.0 * D * F * R
        out["gemm1_tflops"] = fl1 / (km["gemm1"] * 1e-3) / 1e12
        out["gemm2_tflops"] = fl2 / (km["gemm2"] * 1e-3) / 1e12
        out["ffn_tflops"] = (fl1 + fl2) / ((km["gemm1"] + km["gemm2"]) * 1e-3) / 1e12
        # algorithmic bytes of GEMM1: W1 and W3 of the experts that received rows, the
        # gathered rows of x, h; below the ridge point the weight stream bounds the kernel
        touched = sum(1 for c in g["counts"][:shape.n_ffn] if c > 0)
        by1 = touched * 2 * F * D * b + R * D * b + R * F * b
        out["gemm1_bytes"] = by1
        # both GEMMs: every weight of the touched experts once, x rows, h twice, yffn
        out["ffn_bytes"] = touched * 3 * F * D * b + R * D * b + 2 * R * F * b + R * D * b
        out["gemm1_gbs"] = by1 / (km["gemm1"] * 1e-3) / 1e9
        out["gemm1_flop_per_byte"] = fl1 / by1
    router_bytes = T * (D * b + (N * 4 if shape.residual else 0) + N * 4 + K * 8 + shape.n_const * 4)
    out["router_gbs"] = router_bytes / (km["router"] * 1e-3) / 1e9
    # combine: one yffn row per FFN slot, x only for the tokens with a copy or constant
    # slot (the kernel does not read it otherwise), out once, 12 bytes of routing per slot
    need_x = int((g["topk_idx"] >= shape.n_ffn + shape.n_zero).any(axis=1).sum())
    combine_bytes = (R + need_x + T) * D * b + T * K * 12
    out["combine_bytes"] = combine_bytes
    out["combine_gbs"] = combine_bytes / (km["combine"] * 1e-3) / 1e9
    out["permute_us"] = (km["perm_hist"] + km["perm_scan"] + km["perm_scatter"]) * 1e3
    return out


def source_digest():
    """Digest of the HIP sources: the stored counter figures belong to the kernels of one
    state of the sources and say nothing about any other."""
    import hashlib
    h = hashlib.sha256()
    d = os.path.join(ROOT, "paper_2410_07348_amd", "csrc")
    for fn in sorted(os.listdir(d)):
        if fn.endswith((".hip", ".h")):
            with open(os.path.join(d, fn), "rb") as f:
                h.update(fn.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def profiled_traffic(workload):
    """HBM bytes per launch of each kernel, from the committed rocprofv3 --pmc
    summary (FETCH_SIZE / WRITE_SIZE scaled by the copy kernel of known size);
    counters cannot be read from inside this process, so this is the stored
    figure for the same workload, and only while the HIP sources are the ones
    that were profiled.  Returns (dict, note)."""
    path = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    try:
        with open(path) as f:
            allt = json.load(f)
    except OSError:
        return {}, "no stored counter summary"
    if allt.get("source_digest") != source_digest():
        return {}, ("the HIP sources changed since profiles/hbm_traffic.json was recorded "
                    "(digest %s, now %s): traffic not reported" % (allt.get("source_digest"), source_digest()))
    return allt.get(workload, {}), None


def cpu_baseline(shape, inp, target_s=15.0):
    """The CPU oracle timed on a bounded sample of the workload's tokens."""
    import oracle

    def timed(n):
        toks = np.arange(n, dtype=np.int32)          # the first n tokens of the seeded batch
        sub = shape.with_(T=n)
        t0 = time.perf_counter()
        r = oracle.route(sub, inp["x"][:n], None if inp["prev_gate"] is None else inp["prev_gate"][:n],
                         inp["W_g"], inp["W_res"], inp["bias"])
        oracle.permute(sub, r["topk_idx"])
        oracle.experts(sub, inp["x"][:n], r["topk_idx"], r["topk_w"], inp["w1"], inp["w3"],
                       inp["w2"], inp["const_vecs"], inp["W_c"], tok_list=toks)
        return time.perf_counter() - t0

    cores = oracle.threads()
    n0 = min(shape.T, max(cores * 2, 32))
    t_probe = timed(n0)
    n = int(min(shape.T, max(n0, n0 * target_s / max(t_probe, 1e-3))))
    n = max(cores, n // cores * cores)
    t = timed(n) if n > n0 else t_probe
    return {"value": n / t, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": "first %d of %d tokens of the same seeded batch, full layer "
                      "(route + permute + experts), %.1f s wall" % (n, shape.T, t)}


def summary_line(shape, g, rf, args, ceiling, traffic, traffic_note):
    """The JSON object of the benchmark workload: the contract's fields, per-kernel
    times and the roofline of the dominant kernel."""
    km = g["kernel_ms"]
    expert_ms = km["gemm1"] + km["gemm2"] + km["combine"]
    result = {
        "metric": "moepp_layer_forward_tokens_per_s",
        "value": shape.T / (g["ms_per_step"] * 1e-3),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": g["ms_per_step"],
        "ms_per_step_no_events": g["ms_per_step_no_events"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if shape.act == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": shape.name, "T": shape.T, "D": shape.D, "F": shape.F,
                   "n_ffn": shape.n_ffn, "n_zero": shape.n_zero, "n_copy": shape.n_copy,
                   "n_const": shape.n_const, "top_k": shape.k, "bias": shape.bias,
                   "gating_residual": shape.residual, "ffn_rows_R": g["R"],
                   "weights": "expert weights packed once before timing"},
        "kernel_ms": km,
        "expert_forward_tokens_per_s": shape.T / (expert_ms * 1e-3) if expert_ms > 0 else None,
        "pct_bf16_mfma_peak_ffn": 100.0 * rf.get("ffn_tflops", 0.0) / PEAK_BF16_MFMA_TFLOPS,
        "router_gbs": rf["router_gbs"], "combine_gbs": rf["combine_gbs"],
        "permute_us": rf["permute_us"],
        "gemm2_tflops": rf.get("gemm2_tflops"),
    }
    ridge = RIDGE
    if "gemm1_tflops" in rf and rf["gemm1_flop_per_byte"] < ridge:
        # few rows per expert (decoding): GEMM1 streams the expert weights
        result["roofline"] = {"kernel": "k_grouped_gemm<SwiGLU> (GEMM1: W1/W3 + SwiGLU)",
                              "bound": "hbm", "achieved": rf["gemm1_gbs"], "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": rf["gemm1_gbs"] / PEAK_HBM_GBS,
                              "traffic": traffic.get("gemm1"),
                              "flop_per_byte": rf["gemm1_flop_per_byte"], "ridge_flop_per_byte": ridge}
    elif "gemm1_tflops" in rf:
        result["roofline"] = {"kernel": "k_grouped_gemm<SwiGLU> (GEMM1: W1/W3 + SwiGLU)",
                              "bound": "mfma", "achieved": rf["gemm1_tflops"],
                              "peak": PEAK_BF16_MFMA_TFLOPS, "unit": "TFLOP/s",
                              "frac": rf["gemm1_tflops"] / PEAK_BF16_MFMA_TFLOPS,
                              "traffic": traffic.get("gemm1"),
                              "measured_mfma_ceiling_tflops": ceiling,
                              "frac_of_measured_ceiling":
                                  rf["gemm1_tflops"] / ceiling if ceiling else None}
    else:
        result["roofline"] = {"kernel": "k_combine", "bound": "hbm",
                              "achieved": rf["combine_gbs"], "peak": PEAK_HBM_GBS,
                              "unit": "GB/s", "frac": rf["combine_gbs"] / PEAK_HBM_GBS,
                              "traffic": None}

    if traffic_note:
        result["roofline"]["traffic_note"] = traffic_note
    result["combine_frac_hbm_peak"] = rf["combine_gbs"] / PEAK_HBM_GBS
    result["router_frac_hbm_peak"] = rf["router_gbs"] / PEAK_HBM_GBS
    return result


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="large")
    ap.add_argument("--no-vanilla", action="store_true")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-others", action="store_true",
                    help="skip the one-run summaries of the small, mid, skew and smallbatch workloads")
    ap.add_argument("--tau-sweep", default="",
                    help="also time a paper model's layer (e.g. '1B/(16+4)E') against tau")
    ap.add_argument("--chain", type=int, default=0,
                    help="also time this many layers back to back, eagerly and as one HIP graph")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs the layer on one GPU only; --gpus %d is not "
                 "supported (tokens are independent: shard T, or the FFN experts, across GPUs)" % args.gpus)

    import torch
    from workloads import WORKLOADS, make_inputs, ffn_work_fraction
    import paper_2410_07348_amd as M
    M.load_library()
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    shape = WORKLOADS[args.workload]
    log("generating", shape)
    inp = make_inputs(shape)
    g = run_gpu(shape, inp, args.steps, args.warmup)
    rf = roofline_numbers(shape, g)
    log("moe++  ms/step %.3f" % g["ms_per_step"], g["kernel_ms"], rf)
    km = g["kernel_ms"]
    expert_ms = km["gemm1"] + km["gemm2"] + km["combine"]

    ceiling = M.mfma_ceiling() if shape.act == "bf16" else None
    log("measured MFMA-only ceiling (random bf16 operands): %s TFLOP/s" % ceiling)
    stream_read, stream_copy = M.stream_ceiling(0), M.stream_ceiling(1)
    log("measured streaming ceilings: read %.0f GB/s, copy %.0f GB/s" % (stream_read, stream_copy))
    traffic, traffic_note = profiled_traffic(shape.name)

    result = summary_line(shape, g, rf, args, ceiling, traffic, traffic_note)
    # what kernels that only read 1 GiB / copy 0.5 GiB reach on this GPU, beside the published 8 TB/s
    result["measured_stream_read_gbs"] = stream_read
    result["measured_stream_copy_gbs"] = stream_copy

    # ---- the other workloads, one timed run each --------------------------------
    if not args.no_others and shape.name == "large":
        for k_ in ("layer", "dev", "out"):
            g.pop(k_, None)
        torch.cuda.empty_cache()
        others = {}
        for name in ("small", "mid", "skew", "smallbatch"):
            so = WORKLOADS[name]
            log("generating", so.name)
            go = run_gpu(so, make_inputs(so), args.steps, args.warmup)
            ro = roofline_numbers(so, go)
            ko = go["kernel_ms"]
            eo = ko["gemm1"] + ko["gemm2"] + ko["combine"]
            o = {"T": so.T, "D": so.D, "F": so.F, "ffn_rows_R": go["R"],
                 "ms_per_step": go["ms_per_step"], "ms_per_step_no_events": go["ms_per_step_no_events"],
                 "tokens_per_s": so.T / (go["ms_per_step"] * 1e-3),
                 "tokens_per_s_no_events": so.T / (go["ms_per_step_no_events"] * 1e-3),
                 "expert_forward_tokens_per_s": so.T / (eo * 1e-3), "kernel_ms": ko,
                 "pct_bf16_mfma_peak_ffn": 100.0 * ro.get("ffn_tflops", 0.0) / PEAK_BF16_MFMA_TFLOPS,
                 "gemm1_tflops": ro.get("gemm1_tflops"), "gemm2_tflops": ro.get("gemm2_tflops"),
                 "router_gbs": ro["router_gbs"], "combine_gbs": ro["combine_gbs"],
                 "permute_us": ro["permute_us"]}
            if ro.get("gemm1_flop_per_byte", 1e9) < RIDGE:
                # few rows per expert: the GEMMs stream the expert weights, HBM is their roofline
                o["gemm1_hbm_gbs"] = ro["gemm1_gbs"]
                o["gemm1_frac_hbm_peak"] = ro["gemm1_gbs"] / PEAK_HBM_GBS
                o["ffn_weight_stream_floor_us"] = 1e6 * ro["ffn_bytes"] / (PEAK_HBM_GBS * 1e9)
                o["ffn_us"] = 1e3 * (ko["gemm1"] + ko["gemm2"])
            others[name] = o
            log(name, o)
            del go
            torch.cuda.empty_cache()
        result["other_workloads"] = others

    # ---- vanilla MoE: same T/D/F/k, zero-computation experts disabled --------
    if not args.no_vanilla and shape.n_zc > 0 and shape.name == "large":
        for k_ in ("layer", "dev", "out"):
            g.pop(k_, None)
        torch.cuda.empty_cache()
        van = {}
        for vname in ("large_vanilla16", "large_vanilla20"):
            vs = WORKLOADS[vname]
            log("generating", vs.name)
            if vs.n_ffn == shape.n_ffn:
                # same seed -> the same expert weights; only the router side differs
                vin = dict(make_inputs(vs.with_(F=8)), w1=inp["w1"], w3=inp["w3"], w2=inp["w2"])
            else:
                vin = make_inputs(vs)
            gv = run_gpu(vs, vin, args.steps, args.warmup)
            kv = gv["kernel_ms"]
            van[vname] = {"ms_per_step": gv["ms_per_step"], "R": gv["R"], "kernel_ms": kv,
                          "tokens_per_s": vs.T / (gv["ms_per_step"] * 1e-3),
                          "ratio_layer": gv["ms_per_step"] / g["ms_per_step"],
                          "ratio_expert": (kv["gemm1"] + kv["gemm2"] + kv["combine"]) / expert_ms}
            log(vname, van[vname])
            del gv, vin
            torch.cuda.empty_cache()
        result["vanilla"] = van
        result["ideal_ratio_rows"] = shape.T * shape.k / max(g["R"], 1)
        result["tab1_fraction_tau1"] = ffn_work_fraction(1.0, shape.n_ffn, shape.n_zc)
        result["paper_context"] = "paper Tab.3: 1.1-2.1x expert forward throughput vs vanilla MoE " \
                                  "(A100 cluster, other shapes); context only"

    # ---- the same layer with the paper's expert capacities (Sec. 3.3) ----------
    if not args.no_vanilla and shape.n_ffn > 0:
        for k in ("layer", "dev", "out"):
            g.pop(k, None)
        torch.cuda.empty_cache()
        gamma, tau = 1.1, 0.75               # the paper's capacity factor and default tau
        gc = run_gpu(shape, inp, args.steps, args.warmup, capacity=(gamma, tau))
        slots = shape.T * shape.k
        result["with_capacity"] = {
            "gamma": gamma, "tau": tau, "ms_per_step": gc["ms_per_step"], "R": gc["R"],
            "tokens_per_s": shape.T / (gc["ms_per_step"] * 1e-3),
            "dropped_fraction": 1.0 - sum(gc["kept"]) / slots,
            "capacity_ffn": gc["cap"][0], "capacity_zc": gc["cap"][-1] if shape.n_zc else None,
            "load_balance_loss": gc["loss"], "kernel_ms": gc["kernel_ms"]}
        log("with capacity", result["with_capacity"])
        del gc
        torch.cuda.empty_cache()

    if args.tau_sweep:
        for k_ in ("layer", "dev", "out"):
            g.pop(k_, None)
        torch.cuda.empty_cache()
        result["tau_sweep"] = tau_sweep(args.tau_sweep, args.steps, args.warmup)

    if args.chain > 0 and shape.residual:
        for k_ in ("layer", "dev", "out"):
            g.pop(k_, None)
        torch.cuda.empty_cache()
        result["chain"] = run_chain(shape, inp, args.chain, args.steps, args.warmup)
        log("chain", result["chain"])

    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a sample")
        result["cpu_baseline"] = cpu_baseline(shape, inp)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
