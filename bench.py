#!/usr/bin/env python3
"""Benchmark of the virtual-node training step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload C2] [--accumulate staged|fused]
                    [--streams 2|1] [--launch eager|graph] [--fold-window 8]

A "step" is one pass of the whole hot path over one synthetic batch already resident in HBM:
partition, V sequential node passes (forward, loss, backward), the size-weighted fold of each
node's gradient into the fp32 gradient buffer, one optimizer update.  Prints ONE JSON line.
Everything runs on one GPU; --gpus above 1 is refused.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16 matrix cores
FP32_VECTOR_PEAK_TFLOPS = 157.3


def algorithmic_work(wl, P, fused=False, window=1, group=1):
    """Per step, per kernel tag: (bytes, flops, launches) the method itself needs.
    Bytes count each operand once per launch (fp32 = 4, bf16 = 2).  With the fused fold the
    weight-gradient kernels read and write the gradient buffer once per fold window of `window`
    nodes (the first window only writes it) and there is no accumulate kernel."""
    V, B = wl.n_nodes, wl.batch
    esz = 2 if wl.dtype == "bf16" else 4
    work = {} if fused else {"accumulate": ((12 * V - 4) * P, 2 * V * P, V)}
    # With node groups a launch takes a unit of several nodes at once and needs the weights once:
    # the bytes counted are those of the launches as they are made (weights once per unit), not
    # the node-by-node stream of Section 3.2 (weights once per node), which a grouped launch does
    # not perform -- credited with it, a launch would "exceed" the HBM peak.
    U = pass_units(wl, group)                     # units that go through the passes
    nwin = -(-U // window) if fused else V        # passes over the gradient buffer per step
    wg = (8 * nwin - 4) if fused else 4 * V       # fp32 bytes per matrix entry per step
    opt_bytes = (20 if wl.optimizer == "sgdm" else 28) * P
    work["optimizer"] = (opt_bytes, 4 * P, 1)
    if wl.kind == "mlp":
        mats = [(wl.dims[i], wl.dims[i + 1]) for i in range(len(wl.dims) - 1)]
        W = sum(k * n for k, n in mats)
        fwd_fl = 2 * B * W
        dgr_fl = 2 * B * sum(k * n for k, n in mats[1:])
        act = sum(b * (k * esz + n * 4) for b in wl.node_sizes for k, n in mats)
        work["gemm_fwd"] = (U * W * esz + act, fwd_fl, U * len(mats))
        work["gemm_dgrad"] = (U * sum(k * n for k, n in mats[1:]) * esz + act, dgr_fl, U * (len(mats) - 1))
        work["gemm_wgrad"] = (wg * W + act, fwd_fl, nwin * len(mats))
        work["cast_weight"] = (W * (4 + 2 * esz), 0, len(mats))
    elif wl.kind == "conv":
        # a 3x3 convolution as a product over patch rows: per position 2 * 9 Cin * Cout flops; the
        # method needs the activations in (bf16) and out (fp32) once and the filters once per launch
        HW, C = wl.img * wl.img, wl.width
        convs = [(wl.in_ch, C)] + [(C, C)] * (2 * wl.n_blocks)
        R = B * HW
        fl = sum(2 * R * 9 * ci * co for ci, co in convs)
        fl_d = sum(2 * R * 9 * ci * co for ci, co in convs[1:])
        wbytes = sum(9 * ci * co * esz for ci, co in convs)
        act = sum(R * (ci * esz + co * 4) for ci, co in convs)
        act_d = sum(R * (co * esz + ci * 4) for ci, co in convs[1:])
        work["gemm_fwd"] = (V * wbytes + act, fl, V * len(convs))
        work["gemm_dgrad"] = (V * wbytes + act_d, fl_d, V * (len(convs) - 1))
        work["gemm_wgrad"] = (sum(R * (ci + co) * esz for ci, co in convs) + wg * sum(9 * ci * co for ci, co in convs),
                              fl, V * len(convs))
        # element-wise passes over [positions, C]: statistics + apply forward, reduce + apply backward
        work["bn_apply"] = (R * C * (4 + esz) * len(convs), 0, V * len(convs))
        work["bn_bwd"] = (R * C * (2 * (4 + 4 + esz) + esz) * len(convs), 0, V * len(convs))
    else:
        d, f, T, Vc, m, nl = wl.d_model, wl.d_ffn, wl.seq_len, wl.vocab, wl.n_masked, wl.n_layers
        R, Rm = B * T, B * m                       # tokens and masked rows per step
        Wl = 4 * d * d + 2 * d * f                 # matrix entries of one block
        lin_fl = 2 * R * Wl * nl                   # one pass over the four Linears of all blocks
        act_f = nl * R * (2 * d + 3 * d + d + f + f + d) * esz   # operands read / written once
        work["gemm_fwd"] = (U * nl * Wl * esz + act_f, lin_fl, U * nl * 4)
        work["gemm_dgrad"] = (U * nl * Wl * esz + act_f, lin_fl, U * nl * 4)
        work["gemm_wgrad"] = (wg * nl * Wl + act_f, lin_fl, U * nl * 4)
        head_fl = 2 * Rm * d * Vc
        work["gemm_head"] = (U * d * Vc * esz + Rm * Vc * 4, head_fl, U)
        work["gemm_head_dgrad"] = (U * d * Vc * esz + Rm * Vc * esz, head_fl, U)
        work["gemm_head_wgrad"] = (wg * d * Vc + Rm * Vc * esz, head_fl, U)
        att = 2 * T * T * d * B * nl               # one [T,T,d_head] product over all heads, all blocks
        for tag in ("attn_scores", "attn_pv", "attn_bwd_dp", "attn_bwd_dv", "attn_bwd_dq", "attn_bwd_dk"):
            work[tag] = (nl * (3 * R * d * esz + B * wl.n_heads * T * T * 4), att, U * nl)
        # fused matrix-core kernels: 2 products forward, 4 backward, per head
        work["attn_fwd"] = (nl * (4 * R * d * esz + B * wl.n_heads * T * T * esz), 2 * att, U * nl)
        work["attn_bwd"] = (nl * (6 * R * d * esz + R * d * 4 + B * wl.n_heads * T * T * esz), 4 * att, U * nl)
        work["cast_weight"] = ((nl * Wl + d * Vc) * (4 + 2 * esz), 0, 4 * nl + 1)
    return work


def pass_units(wl, group):
    """Units that go through the passes of a step: the nodes, or (the library's rule) runs of up to
    `group` consecutive nodes where the model takes groups -- bf16 MLP: nodes of at most 128 rows, a
    multiple of 8, of any mix of sizes; encoder: 2 or 4 nodes of one size."""
    sizes, units, i = list(wl.node_sizes), 0, 0
    mlp = wl.kind == "mlp" and wl.dtype == "bf16"
    enc = wl.kind == "encoder"
    while i < len(sizes):
        take = 1
        if group > 1 and mlp and sizes[i] <= 128 and sizes[i] % 8 == 0:
            while i + take < len(sizes) and take < group and sizes[i + take] <= 128 and sizes[i + take] % 8 == 0:
                take += 1
        elif group > 1 and enc:
            run, most = 1, min(group, 4)
            while i + run < len(sizes) and run < most and sizes[i + run] == sizes[i]:
                run += 1
            take = 4 if run >= 4 else (2 if run >= 2 else 1)
        units += 1
        i += take
    return units


def roofline_for(tag, work, avg_ms):
    r = _roofline_for(tag, work, avg_ms)
    flops, launches = work[tag][1], work[tag][2]
    if flops and tag.startswith(("gemm", "attn_fwd", "attn_bwd")):
        # matrix-core rate of every product, whichever roof binds it
        r["mfma_tflops"] = flops / launches / (avg_ms * 1e-3) / 1e12
        r["mfma_frac"] = r["mfma_tflops"] / MFMA_BF16_PEAK_TFLOPS
    return r


def _roofline_for(tag, work, avg_ms):
    bytes_, flops, launches = work[tag]
    b_per, f_per = bytes_ / launches, flops / launches
    t_hbm = b_per / (HBM_PEAK_GBS * 1e9)
    t_mfma = f_per / (MFMA_BF16_PEAK_TFLOPS * 1e12)
    if tag.startswith("attn_") and tag not in ("attn_fwd", "attn_bwd"):
        # these products run on the fp32 vector ALUs (no matrix-core version yet)
        ach = f_per / (avg_ms * 1e-3) / 1e12
        return {"kernel": tag, "bound": "alu", "achieved": ach, "peak": FP32_VECTOR_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": ach / FP32_VECTOR_PEAK_TFLOPS, "traffic": None,
                "avg_launch_ms": avg_ms, "algorithmic_flops_per_launch": f_per}
    if t_hbm >= t_mfma:
        ach = b_per / (avg_ms * 1e-3) / 1e9
        return {"kernel": tag, "bound": "hbm", "achieved": ach, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": ach / HBM_PEAK_GBS, "traffic": None, "avg_launch_ms": avg_ms,
                "algorithmic_bytes_per_launch": b_per}
    ach = f_per / (avg_ms * 1e-3) / 1e12
    return {"kernel": tag, "bound": "mfma", "achieved": ach, "peak": MFMA_BF16_PEAK_TFLOPS,
            "unit": "TFLOP/s", "frac": ach / MFMA_BF16_PEAK_TFLOPS, "traffic": None,
            "avg_launch_ms": avg_ms, "algorithmic_flops_per_launch": f_per}


def measured_traffic(workload, accumulate, tag):
    """HBM bytes per launch of kernel `tag` from the committed hardware-counter summary
    (profiles/<workload>_hbm_traffic.txt: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
    script, scaled by the plain-copy dispatch), or None when no summary covers this case."""
    path = os.path.join(ROOT, "profiles", f"{workload.lower()}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                parts = line.split()
                if len(parts) >= 4 and parts[0] == "traffic" and parts[1] == accumulate and parts[2] == tag:
                    return float(parts[3])
    except OSError:
        pass
    return None


def cpu_baseline(wl, theta, x, y, budget_s=12.0):
    """The oracle as it stands, timed node by node on the host cores until about
    `budget_s` seconds of work are done (at least one node; the nodes again from the first when
    one pass over them is quicker than that)."""
    import numpy as np
    import oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.perf_counter()
    done = 0
    samples = 0
    while time.perf_counter() - t0 < budget_s:          # whole passes over the nodes, again if they are quick
        for i in range(wl.n_nodes):
            O.oracle_step(wl, theta, x, y, nodes=[i])
            done += 1
            samples += wl.node_sizes[i]
            if time.perf_counter() - t0 >= budget_s:
                break
    dt = time.perf_counter() - t0
    return {"value": samples / dt, "unit": "samples/s", "cores": int(cores), "kind": "oracle",
            "threads": "cores = the BLAS threads of the NumPy float64 oracle (threadpoolctl); its Python parts run on one",
            "sample": f"{done} virtual-node passes ({samples} samples; the workload has {wl.n_nodes} nodes) of "
                      f"workload {wl.name}, each with the combine and one optimizer update, {dt:.1f} s",
            "seconds": dt}


def mode_flags(vf, args):
    return (vf.VF_FLAG_NO_GRAPH if args.launch == "eager" else 0) | \
           (vf.VF_FLAG_OVERLAP if args.streams == 2 else 0)


def time_steps(vf, torch, wl, theta, x, y, flags, steps, warmup, max_node_size=None, fold_window=1, node_group=1):
    """(ms per step, workspace bytes) of `wl` on the device."""
    from paper_2009_09523_amd.binding import config_from_workload
    stream = torch.cuda.Stream()
    eng = vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, max_node_size=max_node_size,
                                                  fold_window=fold_window, node_group=node_group))
    params = torch.from_numpy(theta).cuda()
    xt = torch.from_numpy(x).cuda()
    if wl.kind in ("mlp", "conv") and wl.dtype == "bf16":
        xt = xt.to(torch.bfloat16)
    yt = torch.from_numpy(y).cuda()
    sizes = list(wl.node_sizes)
    for _ in range(warmup):
        eng.step(params, xt, yt, sizes)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        eng.step(params, xt, yt, sizes)
    stream.synchronize()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    ws = eng.workspace_bytes
    eng.close()
    return ms, ws


def vsweep(args):
    """Synthetic analogue of the paper's microbenchmark of virtual node processing on one
    accelerator (Section 6.6, Figures 13 and 14): (a) node size fixed, batch growing with the
    number of virtual nodes -- throughput and memory relative to one node; (b) batch fixed (it
    already fits), split into more and more nodes -- throughput relative to no virtual nodes."""
    from dataclasses import replace
    import numpy as np
    import torch
    import paper_2009_09523_amd as vf
    import vf_inputs as I
    base = I.workload(args.workload)
    flags = (vf.VF_FLAG_FUSED_ACCUMULATE if args.accumulate == "fused" else 0) | mode_flags(vf, args)
    b = max(base.node_sizes)
    grow, fits = [], []
    literal = []
    for V in (1, 2, 4, 8, 16, 32, 64, 128):
        wl = replace(base, node_sizes=(b,) * V)
        theta = I.make_params(wl)
        x, y = I.make_batch(wl)
        ms, ws = time_steps(vf, torch, wl, theta, x, y, flags, args.steps, args.warmup, fold_window=args.fold_window, node_group=args.node_group)
        grow.append({"V": V, "batch": b * V, "ms_per_step": ms, "samples_per_s": b * V / (ms * 1e-3),
                     "workspace_bytes": ws})
        if V in (1, 8, 64):
            # the same node after node (units of one node, window 1): the workspace of the method as the paper states it
            ms1, ws1 = time_steps(vf, torch, wl, theta, x, y, flags, args.steps, args.warmup, fold_window=1, node_group=1)
            literal.append({"V": V, "batch": b * V, "ms_per_step": ms1, "samples_per_s": b * V / (ms1 * 1e-3),
                            "workspace_bytes": ws1})
    B = base.batch
    theta = I.make_params(base)
    x, y = I.make_batch(base)
    V = 1
    while B // V >= 16 and B % V == 0:
        wl = replace(base, node_sizes=(B // V,) * V)
        ms, ws = time_steps(vf, torch, wl, theta, x, y, flags, args.steps, args.warmup, fold_window=args.fold_window, node_group=args.node_group)
        fits.append({"V": V, "node_size": B // V, "ms_per_step": ms, "samples_per_s": B / (ms * 1e-3),
                     "workspace_bytes": ws})
        V *= 2
    for rows in (grow, fits, literal):
        for r in rows:
            r["throughput_vs_V1"] = r["samples_per_s"] / rows[0]["samples_per_s"]
            r["workspace_vs_V1"] = r["workspace_bytes"] / rows[0]["workspace_bytes"]
    print(json.dumps({"mode": "vsweep", "workload": base.name, "accumulate": args.accumulate,
                      "fold_window": args.fold_window, "node_group": args.node_group,
                      "growing_batch_fixed_node_size": grow, "growing_batch_node_after_node": literal,
                      "fixed_batch": fits,
                      "paper_context": "Section 6.6 on one RTX 2080 Ti, normalised to TensorFlow: throughput "
                                       "-4.2 % to +31.4 % as virtual nodes are added at growing batch; at "
                                       "least 88.4 % when the batch already fits; memory overhead constant "
                                       "beyond two nodes"}))


def het_profile(args):
    """Offline profile of Section 5.1.1 on this accelerator (time of one virtual-node pass against
    node batch size, power-of-2 and power-of-2-like sizes), then the split solver of Section 5.1.2
    on a synthetic mix: 2 accelerators with the measured curve and 8 of a type 4x as slow (the
    paper's V100 : P100 ratio), global batch 8192."""
    from dataclasses import replace
    import torch
    import paper_2009_09523_amd as vf
    import vf_inputs as I
    base = I.workload(args.workload)
    flags = (vf.VF_FLAG_FUSED_ACCUMULATE if args.accumulate == "fused" else 0) | mode_flags(vf, args)
    V = 4                                   # several nodes per step so that the update is amortised
    sizes = [16, 24, 32, 48, 64, 96, 128, 192, 256]
    curve = []
    for b in sizes:
        wl = replace(base, node_sizes=(b,) * V)
        theta = I.make_params(wl)
        x, y = I.make_batch(wl)
        ms, _ = time_steps(vf, torch, wl, theta, x, y, flags, args.steps, args.warmup, fold_window=args.fold_window, node_group=args.node_group)
        curve.append({"node_batch": b, "ms_per_node": ms / V, "samples_per_s": b * V / (ms * 1e-3)})
    fast = [c["ms_per_node"] for c in curve]
    slow = [4.0 * t for t in fast]
    mix = [(2, sizes, fast), (8, sizes, slow)]
    b_het, v_het, t_het = vf.vf_solve_split(mix, 8192, 0.0)
    b_hom, v_hom, t_hom = vf.vf_solve_split(mix[:1], 8192, 0.0)
    print(json.dumps({"mode": "het-profile", "workload": base.name, "profile": curve,
                      "synthetic_mix": {"types": [{"n": 2, "speed": "measured"}, {"n": 8, "speed": "measured / 4"}],
                                        "global_batch": 8192,
                                        "split": {"batch_per_device": b_het, "nodes_per_device": v_het,
                                                  "ms_per_step": t_het},
                                        "fast_type_only": {"batch_per_device": b_hom, "nodes_per_device": v_hom,
                                                           "ms_per_step": t_hom},
                                        "throughput_gain": t_hom / t_het - 1.0},
                      "paper_context": "Table 4 / Section 6.5: 2 V100 + 8 P100 at 2048 / 512 per GPU, "
                                       "+42 % throughput over V100 only"}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=None,
                    help="the workload `value` is measured on (default C5: the largest configuration that one "
                         "GPU holds)")
    ap.add_argument("--also", default="C2,C4",
                    help="comma-separated workloads measured as well and reported under other_workloads "
                         "(default C2,C4; empty: none)")
    ap.add_argument("--accumulate", choices=["staged", "fused"], default="fused",
                    help="fused (default): weight-gradient epilogues fold w_i*g_i into the gradient buffer; "
                         "staged: per-node staging vector + the accumulate kernel")
    ap.add_argument("--no-alt", action="store_true", help="skip the timing of the other accumulate mode")
    ap.add_argument("--streams", type=int, choices=[1, 2], default=2,
                    help="2 (default): the forward passes on one stream, the backward passes and weight "
                         "gradients on a second one, so that node i+1's forward pass runs beside node i's "
                         "backward pass (bf16 MLP; other models run on one stream); 1: everything in line")
    ap.add_argument("--launch", choices=["eager", "graph"], default="eager",
                    help="eager (default): kernels launched one by one; graph: the captured launch "
                         "sequence replayed as HIP graphs")
    ap.add_argument("--fold-window", type=int, default=8,
                    help="fused fold: the weight gradients of this many consecutive nodes (1..8) are folded "
                         "into the gradient buffer in one pass (nodes of one size: one product over the "
                         "window's rows; the workspace keeps that many nodes' transposed bf16 operands)")
    ap.add_argument("--node-group", type=int, choices=[1, 2, 4, 8, 16, 32], default=32,
                    help="up to this many consecutive nodes go through their passes together "
                         "(one operand of every product, so the weights are read once per group; BatchNorm "
                         "statistics, node losses and weights stay per node); 1: node after node")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-profile", action="store_true")
    ap.add_argument("--vsweep", action="store_true",
                    help="instead of the benchmark line: throughput and memory against the number of "
                         "virtual nodes (the paper's Section 6.6 microbenchmark, synthetic)")
    ap.add_argument("--het-profile", action="store_true",
                    help="instead of the benchmark line: the offline profile (time per virtual node "
                         "against node batch size) and the heterogeneous split it gives on a synthetic mix")
    args = ap.parse_args()
    if args.workload is None:     # the sweeps are defined on the configuration whose step takes about 1 ms
        args.workload = "C2" if (args.vsweep or args.het_profile) else "C5"
    if args.gpus != 1:
        print("bench.py: this build runs the virtual-node step on ONE GPU; --gpus above 1 is not "
              "supported (no collectives are part of it).", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2009_09523_amd as vf
    import vf_inputs as I
    from paper_2009_09523_amd.binding import config_from_workload

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    if args.vsweep:
        vsweep(args)
        return
    if args.het_profile:
        het_profile(args)
        return
    out = bench_workload(args.workload, args, primary=True)
    # the other named configurations that fit one GPU, each with its own roofline and floor
    # (never `value`): C2 is the one whose weights stay cache resident, C4 the one where the
    # matrix cores are the binding roof
    others = [w for w in args.also.split(",") if w and w != args.workload]
    if others:
        out["other_workloads"] = {w: bench_workload(w, args, primary=False) for w in others}
    print(json.dumps(out))


def bench_workload(name, args, primary):
    """One benchmark record of workload `name` (see the module docstring for what a step is)."""
    import numpy as np
    import torch
    import paper_2009_09523_amd as vf
    import vf_inputs as I
    from paper_2009_09523_amd.binding import config_from_workload
    wl = I.workload(name)
    # a secondary record of a small workload is timed over more steps (its step takes about 1 ms)
    steps = args.steps if primary or name in ("C4", "C5") else max(args.steps, 50)
    warmup = args.warmup
    theta = I.make_params(wl)
    x, y = I.make_batch(wl)
    stream = torch.cuda.Stream()
    mode = mode_flags(vf, args)
    flags = (vf.VF_FLAG_FUSED_ACCUMULATE if args.accumulate == "fused" else 0) | mode
    eng = vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, fold_window=args.fold_window, node_group=args.node_group))
    P = eng.num_params
    window = eng.fold_window                      # the window in effect (1 where no windowed path exists)
    params = torch.from_numpy(theta).cuda()
    xt = torch.from_numpy(x).cuda()
    if wl.kind in ("mlp", "conv") and wl.dtype == "bf16":
        xt = xt.to(torch.bfloat16)
    yt = torch.from_numpy(y).cuda()
    sizes = list(wl.node_sizes)
    torch.cuda.synchronize()

    # One plain copy of known size (P floats read, P floats written; first-node form of the
    # accumulate kernel with weight 1): the reference dispatch that hardware-counter runs use
    # to scale FETCH_SIZE / WRITE_SIZE.  Not part of the timed region.
    cal_src = torch.ones(P, device="cuda")
    cal_dst = torch.empty(P, device="cuda")
    vf.vf_accumulate(cal_dst, cal_src, 1.0, first=True, stream=stream)
    stream.synchronize()
    del cal_src, cal_dst

    for _ in range(warmup):
        eng.step(params, xt, yt, sizes)
    stream.synchronize()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        eng.step(params, xt, yt, sizes)
    stream.synchronize()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt * 1e3 / steps
    loss = eng.loss()

    out = {
        "metric": "samples/sec per training step at V virtual nodes on 1 MI355X",
        "value": wl.batch / (ms_per_step * 1e-3), "unit": "samples/s", "n_gpus": 1,
        "steps": steps, "warmup": warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if wl.dtype == "bf16" else "f32", "data": "synthetic",
        "config": {"workload": wl.name, "model": wl.kind, "dims": list(wl.dims) if wl.kind == "mlp" else None,
                   "batchnorm": bool(wl.batchnorm),
                   "encoder": None if wl.kind != "encoder" else {"layers": wl.n_layers, "d_model": wl.d_model,
                                                                 "heads": wl.n_heads, "d_ffn": wl.d_ffn,
                                                                 "seq_len": wl.seq_len, "vocab": wl.vocab,
                                                                 "masked_per_seq": wl.n_masked},
                   "conv": None if wl.kind != "conv" else {"img": wl.img, "in_ch": wl.in_ch, "width": wl.width,
                                                           "blocks": wl.n_blocks, "classes": wl.classes},
                   "global_batch": wl.batch, "virtual_nodes": wl.n_nodes,
                   "node_sizes": sizes if len(set(sizes)) > 1 else f"{wl.n_nodes}x{sizes[0]}",
                   "optimizer": wl.optimizer, "params": P, "accumulate": args.accumulate,
                   "fold_window": window, "workspace_bytes": eng.workspace_bytes,
                   "streams": eng.streams, "launch": args.launch,
                   "node_group": args.node_group, "pass_units": pass_units(wl, args.node_group),
                   "value_is": ("%d units of up to %d nodes go through the passes one after another "
                                "(a group's rows are one operand of every product; BatchNorm statistics, losses "
                                "and weights b_i/B per node); fused fold with a window of %d units: the weight "
                                "gradients of a window are ONE product over its rows (the weighted sum of "
                                "Section 5.2).  alt_window_1 is the same step node after node (groups of 1, "
                                "window 1), alt the form with the stand-alone accumulate kernel of Section 3.2 "
                                "step 3" % (pass_units(wl, args.node_group), args.node_group, window))},
        "loss": loss,
    }

    work = algorithmic_work(wl, P, fused=args.accumulate == "fused", window=window, group=args.node_group)
    total_bytes = sum(v[0] for v in work.values())
    total_flops = sum(v[1] for k, v in work.items() if k.startswith(("gemm", "attn")))
    floor_ms = max(total_bytes / (HBM_PEAK_GBS * 1e9), total_flops / (MFMA_BF16_PEAK_TFLOPS * 1e12)) * 1e3
    out["step_floor"] = {"algorithmic_bytes": total_bytes, "gemm_flops": total_flops, "floor_ms": floor_ms,
                         "frac": floor_ms / ms_per_step,
                         "gemm_tflops_achieved": total_flops / (ms_per_step * 1e-3) / 1e12}

    if not args.no_kernel_profile:
        # The same steps again on ONE stream, launched one by one with an event pair around every
        # kernel: each kernel's duration with nothing running beside it (with two streams a
        # kernel's own time also holds what it loses to its neighbour, which says nothing about
        # the kernel).
        engp, pp = eng, params
        if eng.streams == 2:
            engp = vf.VirtualNodeStep(config_from_workload(wl, flags=flags & ~vf.VF_FLAG_OVERLAP, stream=stream,
                                                           fold_window=args.fold_window, node_group=args.node_group))
            pp = params.clone()
            for _ in range(warmup):
                engp.step(pp, xt, yt, sizes)
        engp.profile_start()
        for _ in range(steps):
            engp.step(pp, xt, yt, sizes)
        prof = engp.profile_stop()
        if engp is not eng:
            engp.close()
            del pp
        out["kernels_mode"] = "one stream, launched one by one, an event pair around every kernel"
        tot = sum(v["total_ms"] for v in prof.values())
        kernels = {k: {"launches_per_step": v["launches"] / steps,
                       "avg_launch_ms": v["total_ms"] / v["launches"],
                       "ms_per_step": v["total_ms"] / steps,
                       "share": v["total_ms"] / tot} for k, v in prof.items()}
        out["kernels"] = kernels
        units = pass_units(wl, args.node_group)
        if wl.kind == "mlp" and "gemm_dgrad_bn" in kernels and "gemm_dgrad" not in kernels:
            # every input-gradient product took the BatchNorm / ReLU backward pass in its epilogue: the
            # product's flops; weights and incoming gradient in (bf16), the layer's pre-activations in
            # (fp32), the gradient at the pre-activation and its transposed copy out (bf16)
            esz = 2
            mats = [(wl.dims[i], wl.dims[i + 1]) for i in range(len(wl.dims) - 1)]
            fused_bytes = units * sum(k * n for k, n in mats[1:]) * esz + sum(
                b * (n * esz + k * 4 + 2 * k * esz) for b in wl.node_sizes for k, n in mats[1:])
            work["gemm_dgrad_bn"] = (fused_bytes, work["gemm_dgrad"][1], work["gemm_dgrad"][2])
        if wl.kind == "mlp" and "gemm_fwd_bn" in kernels and kernels["gemm_fwd_bn"]["launches_per_step"] == units * (len(wl.dims) - 2):
            # every hidden layer's forward product took BatchNorm + ReLU in its epilogue: weights and input in
            # (bf16), pre-activations out (fp32), activation and its transposed copy out (bf16); gemm_fwd is
            # then the last layer's product alone
            esz = 2
            mats = [(wl.dims[i], wl.dims[i + 1]) for i in range(len(wl.dims) - 1)]
            hid, last = mats[:-1], mats[-1:]
            hb = units * sum(k * n for k, n in hid) * esz + sum(
                b * (k * esz + n * 4 + 2 * n * esz) for b in wl.node_sizes for k, n in hid)
            work["gemm_fwd_bn"] = (hb, 2 * wl.batch * sum(k * n for k, n in hid), units * len(hid))
            lb = units * sum(k * n for k, n in last) * esz + sum(b * (k * esz + n * 4) for b in wl.node_sizes for k, n in last)
            work["gemm_fwd"] = (lb, 2 * wl.batch * sum(k * n for k, n in last), units)
        dom = max((k for k in kernels if k in work), key=lambda k: kernels[k]["ms_per_step"])
        out["roofline"] = roofline_for(dom, work, kernels[dom]["avg_launch_ms"])
        out["roofline"]["traffic"] = measured_traffic(wl.name, args.accumulate, dom)
        if units != wl.n_nodes:
            out["roofline"]["note"] = (
                f"a launch takes a unit of {wl.n_nodes // units} nodes and reads the weights once: bytes and flops "
                "are those of the launch as made (node by node, the same weights would be streamed once per node)")
        if dom == "gemm_fwd_bn":
            out["roofline"]["note"] = out["roofline"].get("note", "") + (
                "; gemm_fwd_bn is a hidden layer's forward product WITH BatchNorm + ReLU in its epilogue (pre-activations, "
                "activation and its transposed copy written, statistics per node; no kernel of its own for that pass): its "
                "duration holds both, its flops are the product's alone.  The pure products are gemm_wgrad (and the last "
                "layer's gemm_fwd) in roofline_all")
        if dom == "gemm_dgrad_bn":
            out["roofline"]["note"] = out["roofline"].get("note", "") + (
                "; gemm_dgrad_bn is the input-gradient product WITH the BatchNorm / ReLU backward pass of the layer it "
                "arrives at in its epilogue (the layer's fp32 pre-activations read, the bf16 gradient and its transposed "
                "copy written; no kernel of its own for that pass): its duration holds both, its flops are the "
                "product's alone.  The pure products are gemm_wgrad (and gemm_fwd where present) in roofline_all")
        out["roofline_all"] = {k: {kk: vv for kk, vv in roofline_for(k, work, kernels[k]["avg_launch_ms"]).items()
                                   if kk in ("bound", "achieved", "peak", "unit", "frac", "mfma_tflops", "mfma_frac")}
                               for k in kernels if k in work}
    eng.close()

    if not args.no_alt and window > 1:
        # the same fused fold node by node (window 1), for comparison (never `value`)
        ms1, ws1 = time_steps(vf, torch, wl, theta, x, y, flags, steps, warmup)
        out["alt_window_1"] = {"fold_window": 1, "ms_per_step": ms1, "value": wl.batch / (ms1 * 1e-3),
                               "workspace_bytes": ws1}

    if primary and not args.no_alt and (args.streams != 1 or args.launch != "graph"):
        # one stream, the whole step replayed as one HIP graph, for comparison (never `value`)
        gflags = flags & ~(vf.VF_FLAG_NO_GRAPH | vf.VF_FLAG_OVERLAP)
        msg, wsg = time_steps(vf, torch, wl, theta, x, y, gflags, steps, warmup, fold_window=args.fold_window, node_group=args.node_group)
        out["alt_one_stream_graph"] = {"streams": 1, "launch": "graph", "ms_per_step": msg,
                                       "value": wl.batch / (msg * 1e-3), "workspace_bytes": wsg}

    if primary and not args.no_alt:
        # the other accumulate mode, same workload, for comparison (never `value`)
        alt_mode = "staged" if args.accumulate == "fused" else "fused"
        aflags = (vf.VF_FLAG_FUSED_ACCUMULATE if alt_mode == "fused" else 0) | mode
        eng2 = vf.VirtualNodeStep(config_from_workload(wl, flags=aflags, stream=stream))
        p2 = torch.from_numpy(theta).cuda()
        for _ in range(warmup):
            eng2.step(p2, xt, yt, sizes)
        stream.synchronize()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(steps):
            eng2.step(p2, xt, yt, sizes)
        stream.synchronize()
        torch.cuda.synchronize()
        ams = (time.perf_counter() - t1) * 1e3 / steps
        alt = {"accumulate": alt_mode, "ms_per_step": ams, "value": wl.batch / (ams * 1e-3)}
        if alt_mode == "staged" and not args.no_kernel_profile:
            eng2.profile_start()
            for _ in range(steps):
                eng2.step(p2, xt, yt, sizes)
            pr = eng2.profile_stop()
            w2 = algorithmic_work(wl, P, fused=False)
            if "accumulate" in pr:
                avg = pr["accumulate"]["total_ms"] / pr["accumulate"]["launches"]
                alt["accumulate_kernel"] = {k: v for k, v in roofline_for("accumulate", w2, avg).items()
                                            if k in ("bound", "achieved", "peak", "unit", "frac", "avg_launch_ms")}
        out["alt"] = alt
        eng2.close()
        del p2

    if primary and not args.no_alt:
        # The same steps with every batch coming from pinned host memory through the prefetching
        # entry points (copy of batch t+1 beside step t): the PCIe-inclusive rate, never `value`.
        eng3 = vf.VirtualNodeStep(config_from_workload(wl, flags=flags, stream=stream, fold_window=args.fold_window, node_group=args.node_group))
        p3 = torch.from_numpy(theta).cuda()
        hx, hy = xt.cpu().pin_memory(), yt.cpu().pin_memory()
        eng3.prefetch(hx, hy)
        for _ in range(warmup):
            eng3.step_prefetched(p3, sizes)
            eng3.prefetch(hx, hy)
        stream.synchronize()
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(steps):
            eng3.step_prefetched(p3, sizes)
            eng3.prefetch(hx, hy)
        stream.synchronize()
        torch.cuda.synchronize()
        pms = (time.perf_counter() - t2) * 1e3 / steps
        out["host_input"] = {"ms_per_step": pms, "value": wl.batch / (pms * 1e-3),
                             "bytes_per_step": hx.numel() * hx.element_size() + hy.numel() * hy.element_size(),
                             "note": "batch copied from pinned host memory by vf_prefetch while the previous step runs"}
        eng3.close()
        del p3

    if primary and not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, theta, x, y)
    return out


if __name__ == "__main__":
    main()
