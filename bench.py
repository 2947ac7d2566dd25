#!/usr/bin/env python3
"""Benchmark of the tree-masked SSD verification pass on one MI355X.

A step is one pass of the whole hot path (tree index, tree conv, tree scan,
state commit) over one batch of synthetic input, on the 64-node / 80-head
configuration at batch 16 (Mamba2-2.7B layer shape, bf16 io, fp32 state).  Two
call sequences do that work and both are timed:
  separate: stree_tree_conv -> stree_tree_ssd -> stree_commit_state
            (the tree is committed right after it is scanned)
  fused:    stree_tree_conv_replay -> stree_tree_ssd_replay
            (the previous iteration's tree is committed inside this iteration's
            two kernels, as in Alg. 1: its conv tail while the conv rows are
            staged, its state while the state is loaded for the scan -- one pass
            over the state per iteration instead of two)
`value` is the faster of the two; both are in the JSON line.  Inputs are resident in HBM before the timed region; the
step rotates over several buffer sets so that the working set exceeds the
256 MB Infinity Cache and the scan really streams from HBM.  The other
configurations (cfg0, cfg1, cfg3, cfg4) are measured kernel by kernel, HBM-cold
and cache-warm, under the `configs` key.

Prints ONE JSON line on stdout (metric = tree-nodes/s per SSD layer).  Details
(per-kernel times, cache-warm numbers) go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0     # MI355X published HBM3E bandwidth
N_SETS = 6                # rotating buffer sets (about 117 MB each)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def algorithmic_bytes_tree_ssd(B, N, H, P, S, G, se=4):
    """Each operand once: x, y (bf16), B, C (bf16), dt (f32), h0 (se bytes per element: f32, or the bf16
    variant of the state), parent."""
    per_seq = N * H * P * 2 * 2 + 2 * N * G * S * 2 + N * H * 4 + H * P * S * se + N * 4
    return B * per_seq + 2 * H * 4


def algorithmic_bytes_replay(B, N, Np, H, P, S, G, path_nodes, se=4):
    """The scan's operands plus the replayed state written once, the previous tree's parent /
    accepted / dt, and the x and B rows of the accepted paths (path_nodes = their total length)."""
    extra = B * H * P * S * se + B * (Np * 4 + 4 + Np * H * 4) + path_nodes * (H * P + G * S) * 2
    return algorithmic_bytes_tree_ssd(B, N, H, P, S, G, se) + extra


def algorithmic_bytes_conv(B, N, H, P, S, G, W, e=2):
    """Pre-conv rows read, conv output written, conv state read, weights and bias."""
    Cc = H * P + 2 * G * S
    return B * (2 * N * Cc + (W - 1) * Cc) * e + Cc * (W + 1) * e


def algorithmic_bytes_commit(B, N, H, P, S, G, W, path_nodes, e=2, se=4):
    """State read and written once, parent / accepted / dt, the x and B rows of the accepted paths,
    and (W > 0) the conv tail: W-1 rows read and written per sequence."""
    Cc = H * P + 2 * G * S
    tail = B * 2 * (W - 1) * Cc * e if W else 0
    return 2 * B * H * P * S * se + B * (N * 4 + 4 + N * H * 4) + path_nodes * (H * P + G * S) * e + tail


def algorithmic_flops_tree_ssd(B, N, H, P, S, G):
    """C B^T once per group, (L o CB^T) X and C h0^T per head, dense-masked."""
    return B * (G * 2 * N * N * S + H * (2 * N * N * P + 2 * N * S * P))


def read_traffic(kernel_tag):
    """(HBM bytes per launch, source) from the committed rocprofv3 --pmc summary of this kernel and
    workload -- a figure measured in a profiler run of its own, not by this run -- or (None, None)."""
    rel = os.path.join("profiles", f"{kernel_tag}_pmc.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    m = re.search(r"^traffic_bytes_per_launch:\s*([0-9.eE+]+)", open(path).read(), flags=re.M)
    return (float(m.group(1)), rel) if m else (None, None)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1200)
    ap.add_argument("--warmup", type=int, default=120)
    ap.add_argument("--no-graph", action="store_true", help="launch each kernel from Python instead of HIP graphs")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--only-ssd", type=int, default=0, metavar="K",
                    help="profiling aid: run K tree-scan launches and exit")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the kernel-by-kernel table of the other configurations")
    ap.add_argument("--only-config", type=int, default=-1, metavar="C",
                    help="profiling aid: measure configuration C kernel by kernel and exit")
    ap.add_argument("--only-fused", type=int, default=0, metavar="K",
                    help="profiling aid: run K fused replay + scan launches and exit")
    ap.add_argument("--only-gate", type=int, default=0, metavar="K",
                    help="profiling aid: run K gate + norm launches and exit")
    ap.add_argument("--prefix", action="store_true",
                    help="the 4096-token prefix pass of the prefix-then-tree configuration: the chunked linear "
                         "scan kernel against 16 chain-tree calls (prints its own JSON line)")
    ap.add_argument("--batches", action="store_true",
                    help="the scan and the replay + scan kernels at batch 8 .. 128 of the headline shape: how far "
                         "the fill and drain of a 2-3 unit run are from the steady state (prints its own JSON line)")
    ap.add_argument("--latency", action="store_true",
                    help="the step at batch 1, 2, 4 on the paper's tree sizes (single-sequence decoding)")
    ap.add_argument("--sweep", action="store_true",
                    help="second workload: the paper's tree shapes, packed tree scan against the same scan on the "
                         "tree unrolled into one chain per leaf (prints its own JSON line)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build is single-GPU; run with --gpus 1 (no collectives or sharding are built)")

    import torch
    from paper_2505_14969_amd import binding as st
    from paper_2505_14969_amd import synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    st.load()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if args.sweep:
        return sweep(st, synth, torch, dev)
    if args.prefix:
        return prefix(st, synth, torch, dev)
    if args.latency:
        return latency(st, synth, torch, dev)
    if args.batches:
        return batches(st, synth, torch, dev)
    if args.only_config >= 0:
        print(json.dumps({f"cfg{args.only_config}": measure_config(args.only_config, st, synth, torch, dev,
                                                                   not args.no_graph)}), flush=True)
        return

    wl = synth.config(2)
    B, N, H, P, S, G, W = wl.batch, wl.nnodes, wl.nheads, wl.headdim, wl.dstate, wl.ngroups, wl.conv_width
    Cc = wl.conv_channels

    def bf16(a):
        return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(dev)

    base = dict(parent=torch.from_numpy(wl.parent).to(dev), xbc_pre=bf16(wl.xbc_pre), conv_state=bf16(wl.conv_state),
                dt=torch.from_numpy(wl.dt).to(dev), h0=torch.from_numpy(wl.h0).to(dev),
                accepted=torch.from_numpy(wl.accepted).to(dev))
    conv_w, conv_b = bf16(wl.conv_w), bf16(wl.conv_b)
    A, D = torch.from_numpy(wl.A).to(dev), torch.from_numpy(wl.D).to(dev)

    # rotating sets: the same seeded sequences rolled along the batch (distinct memory)
    sets = []
    for r in range(N_SETS):
        s = {k: torch.roll(v, r, 0).contiguous() for k, v in base.items()}
        s["xbc"] = torch.empty((B, N, Cc), dtype=torch.bfloat16, device=dev)
        s["y"] = torch.empty((B, N, H, P), dtype=torch.bfloat16, device=dev)
        s["h_out"] = torch.empty((B, H, P, S), dtype=torch.float32, device=dev)
        s["cs_out"] = torch.empty_like(s["conv_state"])
        s["z"] = torch.randn((B, N, H, P), device=dev).to(torch.bfloat16)     # gate input (random: not part of the step)
        s["yn"] = torch.empty((B, N, H, P), dtype=torch.bfloat16, device=dev)
        s["x"] = s["xbc"][:, :, : H * P].unflatten(2, (H, P))
        s["Bm"] = s["xbc"][:, :, H * P: H * P + G * S].unflatten(2, (G, S))
        s["Cm"] = s["xbc"][:, :, H * P + G * S:].unflatten(2, (G, S))
        sets.append(s)

    def conv(s):
        st.stree_tree_conv(s["parent"], s["xbc_pre"], s["conv_state"], conv_w, conv_b, H, P, S, G, silu=True,
                           out=s["xbc"])

    def ssd(s):
        st.stree_tree_ssd(s["parent"], s["x"], s["dt"], A, s["Bm"], s["Cm"], D, s["h0"], out=s["y"])

    def commit(s):
        st.stree_commit_state(s["parent"], s["accepted"], s["x"], s["dt"], A, s["Bm"], s["h0"], h_out=s["h_out"],
                              xbc_pre=s["xbc_pre"], conv_state=s["conv_state"], conv_state_out=s["cs_out"])

    norm_w = torch.ones(H * P, dtype=torch.bfloat16, device=dev)

    def gate_norm(s):        # the block's output gate + grouped RMS norm behind the scan (timed on its own)
        st.stree_gate_norm(s["y"], s["z"], norm_w, G, 1e-5, out=s["yn"])

    def step(s):
        conv(s)
        ssd(s)
        commit(s)

    def conv_ssd(s):         # the verification pass without the commit
        conv(s)
        ssd(s)

    # fused sequence: the "previous tree" of a set is the tree of the set before it in the
    # rotation, with the activations that set's conv left in its buffer
    for r, s in enumerate(sets):
        s["prev"] = sets[r - 1]

    def conv_replay(s):
        q = s["prev"]
        st.stree_tree_conv_replay(q["parent"], q["accepted"], q["xbc_pre"], s["parent"], s["xbc_pre"],
                                  s["conv_state"], conv_w, conv_b, H, P, S, G, silu=True, out=s["xbc"],
                                  conv_state_out=s["cs_out"])

    def fused(s):
        q = s["prev"]
        st.stree_tree_ssd_replay(q["parent"], q["accepted"], q["x"], q["dt"], q["Bm"], s["parent"], s["x"], s["dt"],
                                 A, s["Bm"], s["Cm"], D, s["h0"], h_out=s["h_out"], out=s["y"])

    def step_fused(s):
        conv_replay(s)
        fused(s)

    # the variant with the state kept in bf16 (reported on its own, never as `value`)
    for s in sets:
        s["h0b"] = s["h0"].to(torch.bfloat16)
        s["h_outb"] = torch.empty_like(s["h0b"])

    def ssd_b(s):
        st.stree_tree_ssd(s["parent"], s["x"], s["dt"], A, s["Bm"], s["Cm"], D, s["h0b"], out=s["y"])

    def commit_b(s):
        st.stree_commit_state(s["parent"], s["accepted"], s["x"], s["dt"], A, s["Bm"], s["h0b"], h_out=s["h_outb"],
                              xbc_pre=s["xbc_pre"], conv_state=s["conv_state"], conv_state_out=s["cs_out"])

    def fused_b(s):
        q = s["prev"]
        st.stree_tree_ssd_replay(q["parent"], q["accepted"], q["x"], q["dt"], q["Bm"], s["parent"], s["x"], s["dt"],
                                 A, s["Bm"], s["Cm"], D, s["h0b"], h_out=s["h_outb"], out=s["y"])

    def step_fused_b(s):
        conv_replay(s)
        fused_b(s)

    for s in sets:           # first launches (also sets the kernel's LDS attribute) outside any capture
        step(s)
    for s in sets:
        step_fused(s)
    for s in sets:
        ssd_b(s)
        commit_b(s)
        step_fused_b(s)
    torch.cuda.synchronize()

    if args.only_ssd or args.only_fused or args.only_gate:
        for k in range(args.only_ssd):
            ssd(sets[k % N_SETS])
        for k in range(args.only_fused):
            fused(sets[k % N_SETS])
        for k in range(args.only_gate):
            gate_norm(sets[k % N_SETS])
        torch.cuda.synchronize()
        return

    use_graph = not args.no_graph

    def make_runner(fn, count=N_SETS):
        """fn on the first `count` buffer sets in turn, as one HIP graph (a replay's own launch cost
        is then shared by `count` kernels) or, without graphs, as direct launches."""
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for s in sets[:count]:
                    fn(s)
            torch.cuda.synchronize()
            return g.replay

        def run():
            for s in sets[:count]:
                fn(s)
        return run

    def timed(fn, k, warm):
        """Wall-clock and HIP-event time per launch of EXACTLY k launches of fn on the current stream:
        whole rotations of the buffer sets, then the remaining k % N_SETS launches."""
        run = make_runner(fn)
        rem = k % N_SETS
        run_rem = make_runner(fn, rem) if rem else None
        for _ in range(max(1, warm // N_SETS)):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = k // N_SETS
        t0 = time.perf_counter()
        e0.record()
        for _ in range(reps):
            run()
        if run_rem:
            run_rem()
        e1.record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        return (t1 - t0) * 1e3 / k, e0.elapsed_time(e1) / k

    K, Wm = max(1, args.steps), args.warmup
    try:
        ms_step, ms_step_ev = timed(step, K, Wm)
    except Exception as exc:  # pragma: no cover
        if not use_graph:
            raise
        log(f"[bench] HIP graph capture failed ({exc}); falling back to direct launches")
        use_graph = False
        ms_step, ms_step_ev = timed(step, K, Wm)
    # dominant kernel alone, same rotation (HBM-cold), HIP events on the launch stream
    _, ms_ssd = timed(ssd, K, Wm)
    _, ms_conv = timed(conv, K, Wm)
    _, ms_commit = timed(commit, K, Wm)
    ms_fstep, ms_fstep_ev = timed(step_fused, K, Wm)
    _, ms_fused = timed(fused, K, Wm)
    _, ms_tail = timed(conv_replay, K, Wm)
    ms_cs, _ = timed(conv_ssd, K, Wm)
    _, ms_gn = timed(gate_norm, K, Wm)
    _, ms_ssd_b = timed(ssd_b, K, Wm)
    _, ms_commit_b = timed(commit_b, K, Wm)
    _, ms_fused_b = timed(fused_b, K, Wm)
    ms_fstep_b, _ = timed(step_fused_b, K, Wm)
    # one buffer set only: inputs stay in the 256 MB Infinity Cache
    keep = sets
    sets = [keep[0]] * N_SETS
    _, ms_ssd_warm = timed(ssd, K, Wm)
    sets = keep

    nodes = B * N
    alg_bytes = algorithmic_bytes_tree_ssd(B, N, H, P, S, G)
    alg_flops = algorithmic_flops_tree_ssd(B, N, H, P, S, G)
    achieved = alg_bytes / (ms_ssd * 1e-3) / 1e9
    # nodes on the accepted paths (integer bookkeeping on the inputs, for the byte count only)
    depth = np.stack([synth.tree_depths(wl.parent[b]) for b in range(B)])
    path_nodes = int(sum(depth[b, wl.accepted[b]] + 1 for b in range(B) if wl.accepted[b] >= 0))
    alg_bytes_f = algorithmic_bytes_replay(B, N, N, H, P, S, G, path_nodes)
    achieved_f = alg_bytes_f / (ms_fused * 1e-3) / 1e9
    log(f"[bench] separate: step {ms_step*1e3:.1f} us wall ({ms_step_ev*1e3:.1f} us events)  graph={use_graph}")
    log(f"[bench]   tree_conv {ms_conv*1e3:.2f} us | tree_ssd {ms_ssd*1e3:.2f} us (warm {ms_ssd_warm*1e3:.2f} us) | "
        f"commit {ms_commit*1e3:.2f} us")
    log(f"[bench]   tree_ssd: {alg_bytes/1e6:.2f} MB algorithmic -> {achieved:.0f} GB/s "
        f"({achieved/HBM_PEAK_GBS*100:.1f}% of 8 TB/s); {alg_flops/ (ms_ssd*1e-3)/1e12:.1f} TFLOP/s bf16 MFMA "
        f"(dense-masked count); scan-only {nodes/(ms_ssd*1e-3)/1e6:.1f} M nodes/s")
    log(f"[bench]   gate + RMS norm behind the scan {ms_gn*1e3:.2f} us "
        f"({(3 * B * N * H * P * 2) / (ms_gn * 1e-3) / 1e9:.0f} GB/s)")
    log(f"[bench] fused:    step {ms_fstep*1e3:.1f} us wall ({ms_fstep_ev*1e3:.1f} us events)")
    log(f"[bench]   conv (tail folded in) {ms_tail*1e3:.2f} us | replay+scan {ms_fused*1e3:.2f} us")
    log(f"[bench]   replay+scan: {alg_bytes_f/1e6:.2f} MB algorithmic -> {achieved_f:.0f} GB/s "
        f"({achieved_f/HBM_PEAK_GBS*100:.1f}% of 8 TB/s)")

    ab_b = {"tree_ssd": algorithmic_bytes_tree_ssd(B, N, H, P, S, G, se=2),
            "tree_ssd_replay": algorithmic_bytes_replay(B, N, N, H, P, S, G, path_nodes, se=2),
            "commit_state": algorithmic_bytes_commit(B, N, H, P, S, G, W, path_nodes, se=2)}
    us_b = {"tree_ssd": ms_ssd_b * 1e3, "tree_ssd_replay": ms_fused_b * 1e3, "commit_state": ms_commit_b * 1e3}
    log(f"[bench] bf16 state (variant): tree_ssd {us_b['tree_ssd']:.2f} us | replay+scan {us_b['tree_ssd_replay']:.2f} us | "
        f"commit {us_b['commit_state']:.2f} us | fused step {ms_fstep_b*1e3:.1f} us")
    steps = {"separate": ms_step, "fused": ms_fstep}
    best = min(steps, key=steps.get)
    ms_best = steps[best]
    tr_scan, src_scan = read_traffic("tree_ssd_mfma_cfg2")
    tr_fused, src_fused = read_traffic("tree_ssd_replay_cfg2")
    roof_scan = {"bound": "hbm", "kernel": "tree_ssd_mfma64_kernel<64,128,4,false,false,float>", "achieved": achieved,
                 "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                 "traffic": tr_scan, "traffic_source": src_scan,
                 "algorithmic_bytes": alg_bytes, "avg_launch_us": ms_ssd * 1e3,
                 "cache_warm_us": ms_ssd_warm * 1e3,
                 "mfma_tflops": alg_flops / (ms_ssd * 1e-3) / 1e12}
    roof_fused = {"bound": "hbm", "kernel": "tree_ssd_mfma64_kernel<64,128,4,true,false,float>", "achieved": achieved_f,
                  "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved_f / HBM_PEAK_GBS,
                  "traffic": tr_fused, "traffic_source": src_fused,
                  "algorithmic_bytes": alg_bytes_f, "avg_launch_us": ms_fused * 1e3}
    what = {"separate": "tree_conv + tree_ssd + commit_state",
            "fused": "tree_conv_replay + tree_ssd_replay (the previous tree is committed inside both: conv tail "
                     "while the conv rows are staged, state while it is loaded for the scan)"}
    out = {
        "metric": "tree-nodes/sec per SSD layer at 1 MI355X; % of MFMA/HBM roofline",
        "value": nodes / (ms_best * 1e-3),
        "unit": "tree-nodes/s",
        "n_gpus": 1, "steps": K, "warmup": Wm, "ms_per_step": ms_best,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "cfg2: batch 16 x 64-node random trees (depth 4-8), 80 heads x headdim 64, "
                               "dstate 128, ngroups 1, conv width 4; step = " + what[best],
                   "sequence": best,
                   "batch": B, "nnodes": N, "hip_graph": use_graph, "buffer_sets": N_SETS},
        # the dominant kernel of the timed step
        "roofline": {"separate": roof_scan, "fused": roof_fused}[best],
        "roofline_tree_ssd_alone": roof_scan,
        "steps_us": {k: v * 1e3 for k, v in steps.items()},
        # tree-nodes/s of the scan alone, of conv + scan, and of the whole step (conv + scan + commit, best sequence)
        "nodes_per_s": {"tree_ssd": nodes / (ms_ssd * 1e-3), "conv+ssd": nodes / (ms_cs * 1e-3),
                        "conv+ssd+commit": nodes / (ms_best * 1e-3)},
        "kernels_us": {"tree_conv": ms_conv * 1e3, "tree_ssd": ms_ssd * 1e3, "commit_state": ms_commit * 1e3,
                       "tree_conv_replay": ms_tail * 1e3, "tree_ssd_replay": ms_fused * 1e3,
                       "gate_norm": ms_gn * 1e3},
        # the output gate + RMS norm behind the scan: y and z read, out written (not part of the timed step)
        # the same workload with the SSM state kept in bf16 (state_dtype): half the state traffic, one rounding
        # of the state per iteration; a variant, not the headline configuration (whose state is fp32)
        "state_bf16": {"kernels": {k: {"us": us_b[k], "algorithmic_bytes": ab_b[k],
                                       "GBps": ab_b[k] / (us_b[k] * 1e-6) / 1e9,
                                       "frac": ab_b[k] / (us_b[k] * 1e-6) / 1e9 / HBM_PEAK_GBS} for k in us_b},
                       "fused_step_us": ms_fstep_b * 1e3, "nodes_per_s": nodes / (ms_fstep_b * 1e-3)},
        "gate_norm": {"us": ms_gn * 1e3, "algorithmic_bytes": 3 * B * N * H * P * 2 + H * P * 2,
                      "GBps": (3 * B * N * H * P * 2 + H * P * 2) / (ms_gn * 1e-3) / 1e9},
    }
    del sets, keep
    torch.cuda.empty_cache()
    if not args.no_configs:
        out["configs"] = {f"cfg{c}": measure_config(c, st, synth, torch, dev, use_graph) for c in (0, 1, 3, 4)}
        out["configs"]["cfg2"] = {
            "workload": "the headline workload above", "tree_ssd": {
                "us_cold": ms_ssd * 1e3, "us_warm": ms_ssd_warm * 1e3, "algorithmic_bytes": alg_bytes,
                "GBps": achieved, "frac": achieved / HBM_PEAK_GBS, "nodes_per_s": nodes / (ms_ssd * 1e-3)},
            "tree_conv": {"us_cold": ms_conv * 1e3, "algorithmic_bytes": algorithmic_bytes_conv(B, N, H, P, S, G, W),
                          "GBps": algorithmic_bytes_conv(B, N, H, P, S, G, W) / (ms_conv * 1e-3) / 1e9},
            "commit_state": {"us_cold": ms_commit * 1e3,
                             "algorithmic_bytes": algorithmic_bytes_commit(B, N, H, P, S, G, W, path_nodes),
                             "GBps": algorithmic_bytes_commit(B, N, H, P, S, G, W, path_nodes) / (ms_commit * 1e-3) / 1e9}}

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl)
    print(json.dumps(out), flush=True)


def measure_config(cid, st, synth, torch, dev, use_graph):
    """One configuration kernel by kernel: tree scan (and conv / commit where the configuration has
    them), HBM-cold (rotating buffer sets of more than 256 MB in total) and cache-warm (one set),
    HIP events around graph replays on the launch stream.  The trees are the configuration's seeded
    ones; activations are random tensors drawn on the device (timing depends on shapes and trees)."""
    wl = synth.config(cid, {"prefix": 64} if cid == 4 else None)
    B, N, H, P, S, G, W = wl.batch, wl.nnodes, wl.nheads, wl.headdim, wl.dstate, wl.ngroups, wl.conv_width
    Cc = H * P + 2 * G * S
    io = torch.bfloat16 if wl.io_dtype == "bf16" else torch.float32
    e = 2 if wl.io_dtype == "bf16" else 4
    per_set = B * (2 * N * Cc * e + N * H * P * e + 2 * H * P * S * 4 + N * H * 4)
    n_sets = int(min(96, max(3, -(-320 * 2 ** 20 // per_set))))
    parent = torch.from_numpy(wl.parent).to(dev)
    rng = np.random.default_rng(cid)
    depth = np.stack([synth.tree_depths(wl.parent[b]) for b in range(B)])
    acc_np = wl.accepted if wl.accepted is not None else np.array(
        [int(rng.integers(0, N)) for _ in range(B)], dtype=np.int32)
    path_nodes = int(sum(depth[b, acc_np[b]] + 1 for b in range(B) if acc_np[b] >= 0))
    accepted = torch.from_numpy(np.asarray(acc_np, dtype=np.int32)).to(dev)
    A = -torch.rand(H, device=dev) - 0.5
    D = torch.randn(H, device=dev)
    conv_w = (torch.rand((Cc, max(W, 1)), device=dev) - 0.5).to(io)
    conv_b = (torch.rand(Cc, device=dev) - 0.5).to(io)
    sets = []
    for _ in range(n_sets):
        s = dict(xbc_pre=torch.randn((B, N, Cc), device=dev).to(io), xbc=torch.randn((B, N, Cc), device=dev).to(io),
                 dt=torch.rand((B, N, H), device=dev) * 0.1 + 0.01, h0=torch.randn((B, H, P, S), device=dev) * 0.1,
                 y=torch.empty((B, N, H, P), dtype=io, device=dev),
                 h_out=torch.empty((B, H, P, S), dtype=torch.float32, device=dev))
        if W:
            s["cs"] = torch.randn((B, W - 1, Cc), device=dev).to(io)
            s["cs_out"] = torch.empty_like(s["cs"])
        s["x"] = s["xbc"][:, :, : H * P].unflatten(2, (H, P))
        s["Bm"] = s["xbc"][:, :, H * P: H * P + G * S].unflatten(2, (G, S))
        s["Cm"] = s["xbc"][:, :, H * P + G * S:].unflatten(2, (G, S))
        sets.append(s)

    # a plain copy of known size (the fp32 state of one set, read and written once): the kernel
    # that scales the FETCH_SIZE / WRITE_SIZE counters when this function runs under a profiler
    torch.roll(sets[0]["h0"], 1, 0)

    def ssd(s):
        st.stree_tree_ssd(parent, s["x"], s["dt"], A, s["Bm"], s["Cm"], D, s["h0"], out=s["y"])

    def conv(s):
        st.stree_tree_conv(parent, s["xbc_pre"], s["cs"], conv_w, conv_b, H, P, S, G, silu=True, out=s["xbc"])

    def commit(s):
        st.stree_commit_state(parent, accepted, s["x"], s["dt"], A, s["Bm"], s["h0"], h_out=s["h_out"],
                              xbc_pre=s["xbc_pre"] if W else None, conv_state=s["cs"] if W else None,
                              conv_state_out=s["cs_out"] if W else None)

    def time_us(fn, use_sets, reps):
        for s in use_sets:
            fn(s)
        torch.cuda.synchronize()
        run = None
        if use_graph:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for s in use_sets:
                    fn(s)
            run = g.replay
        else:
            def run():
                for s in use_sets:
                    fn(s)
        run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(use_sets)) * 1e3

    reps = max(2, 240 // n_sets)
    row = {"workload": f"{wl.name}: batch {B} x {N}-node trees, {H} heads x {P}, dstate {S}, ngroups {G}, "
                       f"conv width {W}, {wl.io_dtype} io", "buffer_sets": n_sets}
    kernels = [("tree_ssd", ssd, algorithmic_bytes_tree_ssd(B, N, H, P, S, G) if e == 2 else
                algorithmic_bytes_tree_ssd(B, N, H, P, S, G) + B * (2 * N * H * P + 2 * N * G * S) * 2)]
    if W:
        kernels.append(("tree_conv", conv, algorithmic_bytes_conv(B, N, H, P, S, G, W, e)))
    if wl.accepted is not None:
        kernels.append(("commit_state", commit, algorithmic_bytes_commit(B, N, H, P, S, G, W, path_nodes, e)))
    for name, fn, nbytes in kernels:
        cold = time_us(fn, sets, reps)
        warm = time_us(fn, [sets[0]] * min(n_sets, 8), max(2, 240 // min(n_sets, 8)))
        row[name] = {"us_cold": cold, "us_warm": warm, "algorithmic_bytes": nbytes, "GBps": nbytes / cold / 1e3,
                     "frac": nbytes / cold / 1e3 / HBM_PEAK_GBS}
        if name == "tree_ssd":
            row[name]["nodes_per_s"] = B * N / (cold * 1e-6)
            if N > 64:
                row[name]["traffic"], row[name]["traffic_source"] = read_traffic(f"tree_ssd_blocks_cfg{cid}")
        log(f"[bench] {wl.name}: {name:12s} {cold:7.2f} us cold ({nbytes/cold/1e3:5.0f} GB/s = "
            f"{nbytes/cold/8e4:4.1f}% of 8 TB/s), {warm:7.2f} us warm; {nbytes/1e6:.2f} MB algorithmic")
    del sets
    torch.cuda.empty_cache()
    return row


def prefix(st, synth, torch, dev):
    """cfg4's prefix: B 8 x T 4096 tokens, 80 heads x 64, dstate 128.  Times stree_linear_ssd (y and
    state; state only) and the route it replaces: per 256 tokens a chain-tree scan plus a commit."""
    wl = synth.config(4)
    e = wl.extras
    B, H, P, S, G = wl.batch, wl.nheads, wl.headdim, wl.dstate, wl.ngroups
    T = e["prefix_x"].shape[1]

    def bf16(a):
        return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(dev)

    x, Bm, Cm = bf16(e["prefix_x"]), bf16(e["prefix_B"]), bf16(e["prefix_C"])
    dt, A = torch.from_numpy(e["prefix_dt"]).to(dev), torch.from_numpy(wl.A).to(dev)
    y = torch.empty((B, T, H, P), dtype=torch.bfloat16, device=dev)
    h = torch.empty((B, H, P, S), dtype=torch.float32, device=dev)

    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps * 1e3

    t_full = timed(lambda: st.stree_linear_ssd(x, dt, A, Bm, Cm, None, None, out=y, h_out=h), 20)
    t_state = timed(lambda: st.stree_linear_ssd(x, dt, A, Bm, None, None, None, want_y=False, h_out=h), 20)
    chunk = 256
    chain = torch.from_numpy(np.stack([synth.chain_tree(chunk)] * B)).to(dev)
    last = torch.full((B,), chunk - 1, dtype=torch.int32, device=dev)
    parts = [(x[:, c:c + chunk].contiguous(), dt[:, c:c + chunk].contiguous(), Bm[:, c:c + chunk].contiguous(),
              Cm[:, c:c + chunk].contiguous()) for c in range(0, T, chunk)]
    hh = torch.zeros_like(h)
    yc = torch.empty((B, chunk, H, P), dtype=torch.bfloat16, device=dev)

    def chains():
        hh.zero_()
        for i, (xc, dc, bc, cc) in enumerate(parts):
            st.stree_tree_ssd(chain, xc, dc, A, bc, cc, None, hh, out=yc)
            st.stree_commit_state(chain, last, xc, dc, A, bc, hh, h_out=hh)

    t_chain = timed(chains, 5)
    alg = B * T * (2 * H * P * 2 + 2 * G * S * 2 + H * 4) + 2 * B * H * P * S * 4
    flops = B * T * (G * 2 * 64 * S + H * (2 * 64 * P + 2 * S * P + 3 * 2 * S * P))   # per token, 64-token chunks
    log(f"[prefix] B {B} x T {T}: linear scan {t_full:.0f} us ({B*T/t_full:.1f} M tokens/s, {alg/t_full/1e3:.0f} GB/s "
        f"algorithmic, {flops/t_full/1e6:.1f} TFLOP/s bf16 MFMA), state only {t_state:.0f} us, "
        f"16 x (chain-tree scan + commit) {t_chain:.0f} us")
    print(json.dumps({"metric": "prefix tokens/s per SSD layer (linear scan kernel, y and state)", "unit": "tokens/s",
                      "value": B * T / (t_full * 1e-6), "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": f"cfg4 prefix: batch {B} x {T} tokens, 80 heads x 64, dstate 128"},
                      "us": {"linear_ssd": t_full, "linear_ssd_state_only": t_state, "chain_tree_route": t_chain},
                      "algorithmic_bytes": alg, "achieved_GBps": alg / t_full / 1e3}), flush=True)


def unroll_paths(parent):
    """Root-to-leaf node lists of one tree (integer bookkeeping on the input, no arithmetic)."""
    n = len(parent)
    has_child = np.zeros(n, dtype=bool)
    has_child[parent[parent >= 0]] = True
    paths = []
    for leaf in np.nonzero(~has_child)[0]:
        p, v = [], int(leaf)
        while v >= 0:
            p.append(v)
            v = int(parent[v])
        paths.append(p[::-1])
    return paths


def latency(st, synth, torch, dev):
    """Single-sequence decoding, the paper's setting: the fused step (conv + conv tail, replay + scan, one call)
    and the scan alone at batch 1, 2, 4 on full binary trees of 15 / 31 / 63 nodes and a 64-node random tree,
    80 heads x 64, dstate 128.  HIP graph of six buffer sets, HIP-event time per call."""
    H, P, S, G, W = 80, 64, 128, 1, 4
    Cc = H * P + 2 * G * S
    n_sets, reps = 6, 200
    rng = np.random.default_rng(3)
    A, D = -torch.rand(H, device=dev) - 0.5, torch.randn(H, device=dev)
    cw, cb = torch.randn((Cc, W), device=dev).to(torch.bfloat16), torch.randn(Cc, device=dev).to(torch.bfloat16)
    rows = []
    for B in (1, 2, 4):
        for N in (15, 31, 63, 64):
            one = synth.full_binary_tree({15: 4, 31: 5, 63: 6}[N]) if N < 64 else synth.gen_tree(N, 6, 4, rng)
            parent = torch.from_numpy(np.stack([one] * B).astype(np.int32)).to(dev)
            acc = torch.full((B,), N // 2, dtype=torch.int32, device=dev)
            sets = [dict(pre=torch.randn((B, N, Cc), device=dev).to(torch.bfloat16),
                         pout=torch.randn((B, N, Cc), device=dev).to(torch.bfloat16),
                         cs=torch.randn((B, W - 1, Cc), device=dev).to(torch.bfloat16),
                         dt=torch.rand((B, N, H), device=dev) * 0.1 + 0.01,
                         h0=torch.randn((B, H, P, S), device=dev) * 0.1, h1=torch.empty((B, H, P, S), device=dev),
                         xbc=torch.empty((B, N, Cc), dtype=torch.bfloat16, device=dev),
                         cso=torch.empty((B, W - 1, Cc), dtype=torch.bfloat16, device=dev),
                         y=torch.empty((B, N, H, P), dtype=torch.bfloat16, device=dev)) for _ in range(n_sets)]

            def step(s):
                st.stree_tree_step(parent, acc, s["pre"], s["pout"], s["dt"], parent, s["pre"], s["cs"], cw, cb, s["dt"],
                                   A, D, s["h0"], H, P, S, G, xbc_out=s["xbc"], conv_state_out=s["cso"], h_out=s["h1"],
                                   out=s["y"])

            def scan(s):
                xbc = s["xbc"]
                st.stree_tree_ssd(parent, xbc[:, :, :H * P].unflatten(2, (H, P)), s["dt"], A,
                                  xbc[:, :, H * P:H * P + G * S].unflatten(2, (G, S)),
                                  xbc[:, :, H * P + G * S:].unflatten(2, (G, S)), D, s["h0"], out=s["y"])

            us = []
            for fn in (step, scan):
                for s in sets:
                    fn(s)
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g):
                    for s in sets:
                        fn(s)
                for _ in range(3):
                    g.replay()
                torch.cuda.synchronize()
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for _ in range(reps):
                    g.replay()
                e1.record()
                torch.cuda.synchronize()
                us.append(e0.elapsed_time(e1) / (reps * n_sets) * 1e3)
            log(f"[latency] batch {B} x {N:2d} nodes: step {us[0]:6.2f} us   scan alone {us[1]:5.2f} us")
            rows.append({"batch": B, "nnodes": N, "step_us": us[0], "scan_us": us[1]})
    print(json.dumps({"latency": rows}), flush=True)


def batches(st, synth, torch, dev):
    """The 64-node / 80-head layer shape at batch 8 .. 128 (cfg2's tree and path-length recipe, random
    activations): scan alone and replay + scan, HBM-cold (4 rotating buffer sets), in HIP graphs."""
    N, H, P, S, G = 64, 80, 64, 128, 1
    Cc = H * P + 2 * G * S
    n_sets = 4
    rows = []
    for B in (8, 16, 32, 64, 128):
        rng = np.random.default_rng(B)
        parent = np.stack([synth.gen_tree(N, int(rng.integers(4, 9)), 4, rng) for _ in range(B)]).astype(np.int32)
        depth = np.stack([synth.tree_depths(parent[b]) for b in range(B)])
        acc = np.array([int(rng.choice(np.nonzero(depth[b] == min(int(rng.integers(0, 8)), depth[b].max()))[0]))
                        for b in range(B)], dtype=np.int32)
        sets = []
        for r in range(n_sets):
            s = dict(parent=torch.from_numpy(np.roll(parent, r, 0).copy()).to(dev),
                     acc=torch.from_numpy(np.roll(acc, r, 0).copy()).to(dev),
                     dt=torch.rand((B, N, H), device=dev) * 0.1 + 0.01, h0=torch.randn((B, H, P, S), device=dev) * 0.1,
                     xbc=torch.randn((B, N, Cc), device=dev).to(torch.bfloat16))
            s["y"] = torch.empty((B, N, H, P), dtype=torch.bfloat16, device=dev)
            s["h_out"] = torch.empty((B, H, P, S), dtype=torch.float32, device=dev)
            s["x"] = s["xbc"][:, :, : H * P].unflatten(2, (H, P))
            s["Bm"] = s["xbc"][:, :, H * P: H * P + G * S].unflatten(2, (G, S))
            s["Cm"] = s["xbc"][:, :, H * P + G * S:].unflatten(2, (G, S))
            sets.append(s)
        for r, s in enumerate(sets):
            s["prev"] = sets[r - 1]
        A, D = -torch.rand(H, device=dev) - 0.5, torch.randn(H, device=dev)

        def timeit(fn, reps=50):
            for s in sets:
                fn(s)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for s in sets:
                    fn(s)
            for _ in range(5):
                g.replay()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                g.replay()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (reps * n_sets) * 1e3

        def scan(s):
            st.stree_tree_ssd(s["parent"], s["x"], s["dt"], A, s["Bm"], s["Cm"], D, s["h0"], out=s["y"])

        def fused(s):
            q = s["prev"]
            st.stree_tree_ssd_replay(q["parent"], q["acc"], q["x"], q["dt"], q["Bm"], s["parent"], s["x"], s["dt"], A,
                                     s["Bm"], s["Cm"], D, s["h0"], h_out=s["h_out"], out=s["y"])

        t_scan, t_fused = timeit(scan), timeit(fused)
        pn = int(sum(depth[b, acc[b]] + 1 for b in range(B)))
        ab = algorithmic_bytes_tree_ssd(B, N, H, P, S, G)
        af = algorithmic_bytes_replay(B, N, N, H, P, S, G, pn)
        log(f"[batches] B {B:3d}: scan {t_scan:7.2f} us {ab / t_scan / 1e3:5.0f} GB/s ({ab / t_scan / 8e4:4.1f}% of 8 TB/s)   "
            f"replay+scan {t_fused:7.2f} us {af / t_fused / 1e3:5.0f} GB/s ({af / t_fused / 8e4:4.1f}%)")
        rows.append({"batch": B, "scan_us": t_scan, "scan_GBps": ab / t_scan / 1e3, "replay_scan_us": t_fused,
                     "replay_scan_GBps": af / t_fused / 1e3})
        del sets
        torch.cuda.empty_cache()
    print(json.dumps({"metric": "achieved algorithmic GB/s of the tree-scan kernels against batch", "unit": "GB/s",
                      "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "64-node trees, 80 heads x 64, dstate 128, batch 8..128"},
                      "rows": rows}), flush=True)


def sweep(st, synth, torch, dev):
    """Tree scan on the shapes the paper measures (Sec. 5 "Efficiency of STree against unrolled
    baseline": full binary trees of 15/31/63 tokens; beam trees M x N; static trees of 13-29 tokens),
    layer shape of the 2.7B model, batch 16: the packed tree in one call against the same kernel
    on the tree unrolled into one chain per leaf (one state per chain), plus a fit t = k N + C."""
    B, H, P, S, G = 16, 80, 64, 128, 1
    rng = np.random.default_rng(2025051499)
    A = torch.from_numpy((-np.exp(rng.uniform(0, 2, H))).astype(np.float32)).to(dev)
    D = torch.from_numpy(rng.standard_normal(H).astype(np.float32)).to(dev)
    NSETS = 4

    def bf16(a):
        return torch.from_numpy(synth.f32_to_bf16_bits(a).view(np.int16)).view(torch.bfloat16).to(dev)

    def time_graph(calls):
        for c in calls:
            c()
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in calls:
                c()
        for _ in range(5):
            g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        reps = 60
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(calls)) * 1e3

    shapes = [("binary-%d" % (2 ** l - 1), [synth.full_binary_tree(l)] * B) for l in (4, 5, 6)]
    shapes += [("static-%d" % (1 + w * d), [synth.static_tree(w, d)] * B) for w, d in ((3, 4), (3, 5), (4, 7))]
    shapes += [("beam-%dx%d" % (m, n), [synth.beam_tree(m, n, rng) for _ in range(B)])
               for m in (2, 3, 4, 5) for n in (4, 8, 16)]
    rows = []
    for name, trees in shapes:
        parent = np.stack(trees).astype(np.int32)
        N = parent.shape[1]
        x = rng.standard_normal((B, N, H, P)).astype(np.float32)
        Bm = rng.standard_normal((B, N, G, S)).astype(np.float32)
        Cm = rng.standard_normal((B, N, G, S)).astype(np.float32)
        dt = np.logaddexp(0, rng.standard_normal((B, N, H)) - 2).astype(np.float32)
        h0 = (0.1 * rng.standard_normal((B, H, P, S))).astype(np.float32)
        # unrolled: one chain per leaf, padded to the longest path with dt = 0 tokens (identity steps)
        paths = [unroll_paths(parent[b]) for b in range(B)]
        L = max(len(p) for ps in paths for p in ps)
        idx_b = np.array([b for b in range(B) for _ in paths[b]])
        idx_n = np.array([p + [p[-1]] * (L - len(p)) for ps in paths for p in ps])
        pad = np.array([[0] * len(p) + [1] * (L - len(p)) for ps in paths for p in ps], dtype=bool)
        ux, uB, uC = x[idx_b[:, None], idx_n], Bm[idx_b[:, None], idx_n], Cm[idx_b[:, None], idx_n]
        udt = dt[idx_b[:, None], idx_n].copy()
        udt[pad] = 0.0
        uh0 = h0[idx_b]
        chains = np.stack([synth.chain_tree(L)] * len(idx_b)).astype(np.int32)
        packed_calls, unrolled_calls = [], []
        for r in range(NSETS):
            t = dict(parent=torch.from_numpy(parent).to(dev), x=bf16(x), B=bf16(Bm), C=bf16(Cm),
                     dt=torch.from_numpy(dt).to(dev), h0=torch.from_numpy(h0).to(dev))
            t["y"] = torch.empty((B, N, H, P), dtype=torch.bfloat16, device=dev)
            u = dict(parent=torch.from_numpy(chains).to(dev), x=bf16(ux), B=bf16(uB), C=bf16(uC),
                     dt=torch.from_numpy(udt).to(dev), h0=torch.from_numpy(uh0).to(dev))
            u["y"] = torch.empty((len(idx_b), L, H, P), dtype=torch.bfloat16, device=dev)
            packed_calls.append(lambda t=t: st.stree_tree_ssd(t["parent"], t["x"], t["dt"], A, t["B"], t["C"], D,
                                                              t["h0"], out=t["y"]))
            unrolled_calls.append(lambda u=u: st.stree_tree_ssd(u["parent"], u["x"], u["dt"], A, u["B"], u["C"], D,
                                                                u["h0"], out=u["y"]))
        tp, tu = time_graph(packed_calls), time_graph(unrolled_calls)
        rows.append({"tree": name, "nodes": int(N), "states_unrolled": int(len(idx_b) // B),
                     "tokens_unrolled": int(sum(len(p) for p in paths[0])), "packed_us": tp, "unrolled_us": tu})
        log(f"[sweep] {name:12s} N={N:3d}  unrolled: {len(idx_b)//B:3d} states/seq, {rows[-1]['tokens_unrolled']:4d} tokens"
            f"   packed {tp:7.2f} us   unrolled {tu:7.2f} us   ratio {tu/tp:5.2f}")
        del packed_calls, unrolled_calls
        torch.cuda.empty_cache()
    n = np.array([r["nodes"] for r in rows if r["nodes"] <= 64], dtype=np.float64)
    t = np.array([r["packed_us"] for r in rows if r["nodes"] <= 64])
    k, c = np.polyfit(n, t, 1)
    log(f"[sweep] packed scan, trees of at most 64 nodes: t = {k:.3f} us * N + {c:.2f} us")
    print(json.dumps({"metric": "tree scan on the paper's tree shapes, packed vs unrolled (us per call, batch 16)",
                      "unit": "us", "n_gpus": 1, "dtype": "bf16", "data": "synthetic",
                      "config": {"workload": "full binary 15/31/63, static 13/16/29, beam MxN; 80 heads x 64, dstate 128"},
                      "fit_packed_us": {"per_node": k, "constant": c}, "rows": rows}), flush=True)


def cpu_baseline(wl):
    """The oracle as it stands (fp64 C, OpenMP over batch x head), timed on the host: full-size steps of
    the same workload (conv + scan + commit), repeated to about 12 s with the path-unrolled scan (the
    oracle's primary form) and to about 6 s more with its per-node-state scan (the faster formulation)."""
    from oracle import ref
    from paper_2505_14969_amd import synth
    H, P, S, G = wl.nheads, wl.headdim, wl.dstate, wl.ngroups
    f64 = lambda a: np.ascontiguousarray(a, dtype=np.float64)
    xbc_pre, cs, w, b, dt, A, D, h0 = map(f64, (wl.xbc_pre, wl.conv_state, wl.conv_w, wl.conv_b, wl.dt, wl.A, wl.D,
                                                wl.h0))

    def one(scan):
        conv = ref.tree_conv(wl.parent, xbc_pre, cs, w, b, True)
        xbc = synth.round_to_bf16(conv.astype(np.float32)).astype(np.float64)
        Bn, N, _ = xbc.shape
        x = np.ascontiguousarray(xbc[:, :, : H * P].reshape(Bn, N, H, P))
        Bm = np.ascontiguousarray(xbc[:, :, H * P: H * P + G * S].reshape(Bn, N, G, S))
        Cm = np.ascontiguousarray(xbc[:, :, H * P + G * S:].reshape(Bn, N, G, S))
        scan(wl.parent, x, dt, A, Bm, Cm, D, h0)
        ref.commit(wl.parent, wl.accepted, x, dt, A, Bm, h0, xbc_pre, cs)

    def run(scan, budget_s):
        one(scan)
        t0 = time.perf_counter()
        reps = 0
        while reps < 3 or (time.perf_counter() - t0 < budget_s and reps < 200):
            one(scan)
            reps += 1
        return reps, (time.perf_counter() - t0) / reps

    reps, dt_s = run(ref.ssd_paths, 12.0)
    reps2, dt2_s = run(ref.ssd_nodes, 6.0)
    nodes = wl.batch * wl.nnodes
    return {"value": nodes / dt_s, "unit": "tree-nodes/s", "cores": ref.num_threads(),
            "kind": "oracle", "sample": f"{reps} full-size steps of the same cfg2 batch (conv + path-unrolled "
                                       f"fp64 scan + commit), {dt_s*1e3:.0f} ms each",
            "per_node_state_scan": {"value": nodes / dt2_s, "unit": "tree-nodes/s",
                                    "sample": f"{reps2} full-size steps with the oracle's per-node-state scan "
                                              f"in place of the path-unrolled one, {dt2_s*1e3:.0f} ms each"}}


if __name__ == "__main__":
    main()
