#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

A step = one pass of the whole path over one synthetic batch that already sits in HBM: radius graph,
embedding, L message-passing layers, pooling, per-source heads, and the reverse pass of all of them.
Prints ONE JSON line. Default workload: config 4 (mixed five-source batch, ~40k atoms, ~1.2M edges,
H=256, 6 layers, bf16 matrix-core operands).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0
PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}


def kernel_work(tag, N, E, H, dtype, dsum_in_edge_kernel=False):
    """Algorithmic work of ONE launch of a kernel class: (flops on the matrix cores, HBM bytes).

    Bytes are what the method has to move for that kernel: every edge tensor it streams once (b bytes
    per element, b = 2 for bf16 operands, 4 for fp32), the per-edge index/scalar arrays, and the node
    tensors it gathers counted once (compulsory traffic; re-reads are cache traffic)."""
    b = 2 if dtype == "bf16" else 4
    EH, NH = float(E) * H, float(N) * H
    # a1 is recomputed by the W2-gradient kernel instead of stored: bf16 pairs (H = 256), fp32 operands at H = 128
    pairs = (dtype == "bf16" and H == 256) or (dtype == "f32" and H == 128)
    if tag == "edge_fused_fwd":      # out: z2 (and a1 unless recomputed); in: dst, col, d2; gathers P|Q
        return 2.0 * EH * H, (1 if pairs else 2) * EH * b + 12.0 * E + 2 * NH * b
    if tag == "edge_fused_bwd":      # in: z2, dst, col, d2, c; out: g_z2, g_z1; gathers P|Q, g_M
        # where the kernel also sums g_z1 per destination (no separate pass over g_z1 for that): out g_P as well
        return 4.0 * EH * H, 3 * EH * b + 16.0 * E + 3 * NH * b + (NH * 4 if dsum_in_edge_kernel else 0.0)
    if tag == "wgrad_edge":          # in: g_z2 and a1 (or dst, col, d2 and gathers of P|Q to recompute a1); out: H x H
        if pairs:
            return 2.0 * EH * H, EH * b + 12.0 * E + 2 * NH * b + 4.0 * H * H
        return 2.0 * EH * H, 2 * EH * b + 4.0 * H * H
    if tag == "seg_fwd":             # in: z2, rvec, row_ptr; out: M, v
        return 0.0, EH * b + 12.0 * E + 4.0 * (N + 1) + (NH + 6.0 * N) * 4
    if tag in ("segsum_dst", "segsum_src"):
        # (where the edge kernel forms the destination sums, the source-sorted launch also adds the per-unit partials
        # of the rows that cross units: not algorithmic bytes)
        return 0.0, EH * b + 4.0 * (N + 1) + NH * 4 + (4.0 * E if tag == "segsum_src" else 0.0)
    if tag == "gemm_node":           # one H x H block product per atom row, fp32 in / out
        return 2.0 * NH * H, 2 * NH * 4
    if tag == "wgrad_node":
        return 2.0 * NH * H, 2 * NH * 4
    if tag == "colsum":
        return 0.0, NH * 4
    # widths other than 64 / 128 / 256 (fragment-GEMM path, bf16): per-edge products run as plain GEMMs over materialised tensors
    if tag == "frag_gemm_edge":      # in: a1 (or g_z2) + W2; out: z2 (or g_a1)
        return 2.0 * EH * H, 2 * EH * b + 2.0 * H * H
    if tag == "frag_wgrad_edge":     # in: a1, g_z2; out: H x H. The class has two launches per product (the split
        # product and the ordered sum of its partials): the product's work is spread over both
        return EH * H, (2 * EH * b + 4.0 * H * H) / 2.0
    if tag == "edge_elementwise":    # three kernels per layer: a1 (out 2 copies), g_z2 (in z2, out 2 copies), g_z1 (in g_a1,
        # out 1 copy) = 7 edge tensors, 36 B of per-edge scalars and 5 gathered atom tensors over 3 launches
        return 0.0, (7 * EH * b + 36.0 * E + 5 * NH * b) / 3.0
    if tag.startswith("neigh"):      # whole graph build: in pos; out col, shift, d2, rvec, dst, permT, offsets
        return 0.0, 12.0 * N + 31.0 * E + 12.0 * N
    return 0.0, 0.0


def roofline_of(tag, avg_s, N, E, H, dtype, traffic=None, dsum_in_edge_kernel=False):
    flops, nbytes = kernel_work(tag, N, E, H, dtype, dsum_in_edge_kernel)
    mfma_dtype = dtype
    if dtype == "f32" and tag in ("edge_fused_fwd", "edge_fused_bwd", "wgrad_edge"):
        # fp32 operands of the per-edge products are split into three bf16 terms each: six bf16 products on the
        # matrix cores per fp32 product; the executed bf16 flops are what is held against the bf16 peak
        flops, mfma_dtype = 6.0 * flops, "bf16"
    t_mfma = flops / (PEAK_TFLOPS[mfma_dtype] * 1e12)
    t_hbm = nbytes / (PEAK_HBM_GBS * 1e9)
    if t_mfma > t_hbm:
        ach, peak, unit, bound, work = flops / avg_s / 1e12, PEAK_TFLOPS[mfma_dtype], "TFLOP/s", "mfma", flops
    else:
        ach, peak, unit, bound, work = nbytes / avg_s / 1e9, PEAK_HBM_GBS, "GB/s", "hbm", nbytes
    return {"kernel": tag, "bound": bound, "achieved": ach, "peak": peak, "unit": unit, "frac": ach / peak,
            "traffic": traffic, "avg_launch_ms": avg_s * 1e3, "work_per_launch": work,
            "flops_per_launch": flops, "algorithmic_bytes_per_launch": nbytes}


def read_traffic(config, tag):
    """HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (see profiles/)."""
    path = os.path.join(ROOT, "profiles", f"traffic_{config}.txt")
    if not os.path.exists(path):
        return None
    for line in open(path):
        f = line.split()
        if len(f) >= 2 and f[0] == tag:
            return float(f[1])
    return None


def calib_copy():
    """A plain device-to-device copy of known size, for calibrating the FETCH_SIZE / WRITE_SIZE counters."""
    import torch
    n = 1 << 28   # 1 GiB of float32 read + 1 GiB written per copy
    a = torch.ones(n, dtype=torch.float32, device="cuda")
    b = torch.empty_like(a)
    for _ in range(5):
        b.copy_(a)
    torch.cuda.synchronize()
    print(json.dumps({"calib_copy_bytes_read": n * 4, "calib_copy_bytes_written": n * 4, "copies": 5}))


def cpu_model():
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                return line.split(":", 1)[1].strip()
    except OSError:
        pass
    return "unknown"


def cpu_baseline(P, target_edges=150000):
    """The oracle, as it stands (numpy float64), on a bounded sample of the same batch: the first graphs with about
    target_edges edges with every host thread numpy's BLAS takes, and an eighth of that sample on one thread."""
    import numpy as np
    sys.path.insert(0, os.path.join(ROOT, "tests"))   # only this leg uses the oracle (through the tests' helpers)
    from hgnn_inputs import sub_batch
    from parity_util import oracle_graph, oracle_step
    b = P["batch"]

    def run(target):
        # grow the sample until the oracle graph has about `target` edges (degree estimate ~30)
        k, atoms = 0, 0
        while k < b.G and atoms < target / 30.0:
            atoms += int(b.graph_off[k + 1] - b.graph_off[k])
            k += 1
        sb = sub_batch(b, np.arange(k))
        Ps = dict(P, batch=sb, gE=P["gE"][:k], gF=P["gF"][:sb.N])
        t0 = time.perf_counter()
        og = oracle_graph(Ps)
        alpha = 1.0 / max(1.0, og["E"] / sb.N)
        oracle_step(Ps, og, alpha)
        dt = time.perf_counter() - t0
        return og["E"] / dt, f"first {k} graphs ({sb.N} atoms, {og['E']} edges), graph + fwd + bwd, {dt:.1f} s"

    try:
        from threadpoolctl import threadpool_info, threadpool_limits
        cores = max([d.get("num_threads", 1) for d in threadpool_info()] + [1])
    except Exception:
        threadpool_limits, cores = None, os.cpu_count() or 1
    rate, what = run(target_edges)
    out = {"value": rate, "unit": "edges/s", "cores": int(cores), "kind": "oracle", "cpu": cpu_model(),
           "precision": "float64 (the oracle as the parity tests use it)", "sample": what}
    if threadpool_limits is not None:
        with threadpool_limits(limits=1):
            r1, w1 = run(target_edges / 8)
        out["single_thread"] = {"value": r1, "unit": "edges/s", "cores": 1, "sample": w1}
    return out


def measure(name, steps, warmup, rbf=0, move=False, pos_grad=False, hip_graph=False, adamw=False):
    """Time whole steps of one workload; returns (figures, problem). A step = radius graph + routing plan + forward +
    backward on a batch that already sits in HBM."""
    import torch
    from hgnn_inputs import problem_from_config
    from paper_2506_21788_amd import binding as B
    from paper_2506_21788_amd.step import HotPath

    P = problem_from_config(name, rbf_k=rbf or None, move=move, pos_grad=pos_grad)
    b, hp = P["batch"], P["hp"]
    hot = HotPath.from_problem(P)
    gE = torch.as_tensor(P["gE"]).cuda()
    gF = torch.as_tensor(P["gF"]).cuda()

    for _ in range(max(1, warmup)):
        hot.step(gE, gF)
    torch.cuda.synchronize()
    E, N, G, H, L = hot.graph.E, b.N, b.G, hp["H"], hp["L"]

    # which kernel class dominates? All classes are timed over two untimed steps with the library's side stream
    # switched off, so that every class is timed alone (with it on, kernels of two streams share the GPU and
    # their event times include each other). The timed region below runs the default configuration again; the
    # dominant class of this workload is not overlapped with side-stream work (the library drains it first).
    ntags = B.profile_num_tags()
    side_was_on = B.set_side_stream(False)
    B.profile_begin((1 << ntags) - 1)
    for _ in range(2):
        hot.step(gE, gF)
    B.profile_end()
    B.set_side_stream(side_was_on)
    split = {}
    for t in range(ntags):
        n, ms = B.profile_read(t)
        if n:
            split[B.profile_tag_name(t)] = {"launches_per_step": n / 2, "ms_per_step": ms / 2}
    dom = max(split, key=lambda k: split[k]["ms_per_step"])
    dom_id = [t for t in range(ntags) if B.profile_tag_name(t) == dom][0]

    # timed region: whole steps, with HIP events around the dominant kernel class only
    B.profile_begin(1 << dom_id)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        hot.step(gE, gF)
    torch.cuda.synchronize()
    t_full = (time.perf_counter() - t0) / steps
    B.profile_end()
    dom_n, dom_ms = B.profile_read(dom_id)

    # message passing only (graph and routing plan prebuilt), for reference
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        hot.step(gE, gF, with_graph=False)
    torch.cuda.synchronize()
    t_mp = (time.perf_counter() - t0) / steps

    avg_s = dom_ms / max(dom_n, 1) * 1e-3
    # no launch of the destination-sorted sum in the split <=> the reverse edge kernel formed those sums itself
    dsum = "segsum_dst" not in split and "edge_fused_bwd" in split
    roofline = roofline_of(dom, avg_s, N, E, H, hp["dtype"], read_traffic(name, dom), dsum)
    roofline["launches_per_step"] = dom_n / steps
    if roofline["traffic"] is not None:
        roofline["traffic_source"] = (f"profiles/traffic_{name}.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of this "
                                      "kernel, measured in runs of their own (see profiles/), not in this run")

    out = {
        "ms_per_step": t_full * 1e3, "edges_per_s": E / t_full, "edge_layers_per_s": E * L / t_full,
        "graphs_per_s": G / t_full, "dtype": hp["dtype"],
        "config": {"workload": f"{name}: {hp['desc']}" + (f" + {rbf} radial-basis edge attributes" if rbf else "")
                   + (" + moving atoms" if move else "") + (" + position gradients" if move or pos_grad else ""),
                   "atoms": N, "graphs": G, "edges": E, "H": H,
                   "layers": L, "sources": hp["S"], "cutoff": hp["rc"], "alpha": hot.alpha,
                   "head_width": hp.get("Hh", H), "head_hidden_layers": hp.get("D", 1)},
        "ms_per_step_graph_prebuilt": t_mp * 1e3, "edges_per_s_graph_prebuilt": E / t_mp,
        "roofline": roofline,
        "kernel_split_ms_per_step": {k: round(v["ms_per_step"], 4) for k, v in
                                     sorted(split.items(), key=lambda kv: -kv[1]["ms_per_step"])},
        "_split": split, "_shape": (N, E, H),
    }

    if adamw:
        # AdamW update of every weight buffer (not part of `value`: the metric is the message-passing step). The
        # step's own weights are left alone: copies are updated, with the gradients of the last step.
        params = [(w.clone(), g) for w, g in zip([*hot.W, hot.Whead, hot.emb], [*hot.gW, hot.gWhead, hot.g_emb])]
        moments = [(torch.zeros_like(w), torch.zeros_like(w)) for w, _ in params]
        n_params = sum(w.numel() for w, _ in params)
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for t in range(1, 4):
            for (w, g), (m, v) in zip(params, moments):
                B.adamw_step(w, g, m, v, t)
        ev0.record()
        for t in range(4, 4 + steps):
            for (w, g), (m, v) in zip(params, moments):
                B.adamw_step(w, g, m, v, t)
        ev1.record()
        torch.cuda.synchronize()
        adamw_ms = ev0.elapsed_time(ev1) / steps
        out["adamw"] = {"parameters": n_params, "buffers": len(params), "ms_per_update": adamw_ms,
                        "GB_per_s": 28.0 * n_params / (adamw_ms * 1e-3) / 1e9,
                        "note": "separate from value; 28 B per parameter (read w, g, m, v; write w, m, v)"}

    # the same forward + backward as one HIP graph (graph prebuilt), for launch-bound workloads
    if hip_graph:
        graph = hot.capture(gE, gF)
        for _ in range(3):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            graph.replay()
        torch.cuda.synchronize()
        out["ms_per_step_graph_prebuilt_hip_graph"] = (time.perf_counter() - t0) / steps * 1e3
    del hot
    torch.cuda.empty_cache()
    return out, P


def print_breakdown(name, m):
    N, E, H = m["_shape"]
    print(f"--- {name}: {m['ms_per_step']:.3f} ms/step", file=sys.stderr)
    for k, v in sorted(m["_split"].items(), key=lambda kv: -kv[1]["ms_per_step"]):
        per = v["ms_per_step"] / v["launches_per_step"] * 1e-3
        r = roofline_of(k, per, N, E, H, m["dtype"], None, "segsum_dst" not in m["_split"])
        print(f"{k:18s} {v['launches_per_step']:6.1f} launches  {v['ms_per_step']:9.3f} ms/step  "
              f"{r['achieved']:10.1f} {r['unit']:8s} {100 * r['frac']:5.1f} % of {r['bound']} peak", file=sys.stderr)


def public(m):
    return {k: v for k, v in m.items() if not k.startswith("_")}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", default="cfg4", help="the workload `value` is quoted on")
    ap.add_argument("--only", action="store_true", help="skip the short runs of the other configs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--breakdown", action="store_true", help="print the per-kernel-class split to stderr")
    ap.add_argument("--hip-graph", action="store_true",
                    help="also time forward + backward replayed as one HIP graph (graph prebuilt)")
    ap.add_argument("--rbf", type=int, default=0, metavar="K",
                    help="K radial-basis edge attributes in place of d2 (2..16)")
    ap.add_argument("--pos-grad", action="store_true",
                    help="the reverse pass also gives the gradient with respect to positions")
    ap.add_argument("--move", action="store_true",
                    help="the atoms move between layers (edge geometry recomputed per layer; implies --pos-grad)")
    ap.add_argument("--calib-copy", action="store_true", help="only run a 1 GiB copy kernel (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; no figure at several GPUs exists (--gpus 1 only)",
              file=sys.stderr)
        sys.exit(2)

    if args.calib_copy:
        calib_copy()
        return
    import torch
    assert torch.cuda.is_available(), "bench.py needs a GPU"

    head, P = measure(args.config, args.steps, args.warmup, rbf=args.rbf, move=args.move, pos_grad=args.pos_grad,
                      hip_graph=args.hip_graph, adamw=True)
    if args.breakdown:
        print_breakdown(args.config, head)
    out = {
        "metric": "message-passing edges/s (fwd+bwd), whole step incl. neighbour search, 1 MI355X",
        "value": head["edges_per_s"], "unit": "edges/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": head["ms_per_step"], "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": head["dtype"], "data": "synthetic", "config": head["config"],
        "edge_layers_per_s": head["edge_layers_per_s"], "graphs_per_s": head["graphs_per_s"],
        "ms_per_step_graph_prebuilt": head["ms_per_step_graph_prebuilt"],
        "edges_per_s_graph_prebuilt": head["edges_per_s_graph_prebuilt"],
        "ms_per_step_graph_prebuilt_hip_graph": head.get("ms_per_step_graph_prebuilt_hip_graph"),
        "roofline": head["roofline"], "adamw": head["adamw"],
        "kernel_split_note": "per kernel class, timed alone (side stream off), over 2 untimed steps",
        "kernel_split_ms_per_step": head["kernel_split_ms_per_step"],
    }
    # the other workloads of the benchmark set, a few steps each: throughput and the roofline of their dominant kernel
    if not args.only and not (args.rbf or args.move or args.pos_grad):
        others = {}
        for name in ("cfg1", "cfg2", "cfg3", "cfg4", "cfg5"):
            if name == args.config:
                others[name] = {k: v for k, v in public(head).items() if k != "adamw"}
                continue
            m, _ = measure(name, max(3, min(args.steps, 10)), 2)
            if args.breakdown:
                print_breakdown(name, m)
            others[name] = public(m)
        out["configs"] = others
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(P)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
