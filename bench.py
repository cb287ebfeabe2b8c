#!/usr/bin/env python3
"""Benchmark of the MiCS per-GPU data path on one MI355X.

A step is one pass of the whole path as ONE rank of a partition group executes it for one
training iteration of one transformer layer (rank view, the real per-GPU shape):

    a1  hierarchical-gather reorder of the whole bf16 layer           (N elements)
    a2  s x  reduce-scatter-accumulate of the rank's gradient shard   (S elements, p inputs)
    a3  replica average over the r accumulator copies                 (S elements)
    a4  mixed-precision Adam on the shard                             (S elements)

Default workload: hidden size 8192 (805.4 M parameters per layer), p = 16 (2 nodes x k = 8),
r = 8, s = 12.  All inputs are synthetic, seeded, and resident in HBM before timing; every
micro-step has its own gradient buffers (19.3 GB), nothing is reused or cached.

Prints one JSON line.  `--view group` times the same kernels over all p shards at once
(p*S elements per call; the gradient buffers are then shared by the micro-steps because
s*p*N_pad bf16 would not fit).
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

PEAK_HBM_GBPS = 8000.0   # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="h8192")
    ap.add_argument("--view", choices=["rank", "group"], default="rank")
    ap.add_argument("--rank", type=int, default=5, help="which group rank's shard is simulated")
    ap.add_argument("--coalesced", action="store_true",
                    help="treat the layer as its 16 separately sharded tensors (coalesced gather / "
                         "reduce-scatter): a1 and a2 run through the *_coalesced entry points on "
                         "full-length rank gradient buffers (4 sets, cycled over the micro-steps)")
    ap.add_argument("--grad-dtype", choices=["bf16", "f16", "f32"], default="bf16",
                    help="storage format of the gradient buffers the reduce-scatter-accumulate reads "
                         "(rank view, flat layout)")
    ap.add_argument("--param-dtype", choices=["bf16", "f32"], default="bf16",
                    help="f32: plain float32 training -- the gathered parameter has 4-byte elements and "
                         "the Adam step writes no bf16 copy")
    ap.add_argument("--gathers-per-microstep", type=int, default=0,
                    help="run this many extra gather reorders before every reduce-scatter-accumulate, as "
                         "a training run does (parameters are gathered in the forward and in the backward "
                         "pass of every micro-step); the default step gathers once")
    ap.add_argument("--fused", action="store_true",
                    help="run the replica average and the Adam step as one fused call "
                         "(mics_replica_average_adam_shard): 4r+26 instead of 4r+34 bytes per element")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the steps, run one plain copy of known size (the reorder with "
                         "p = k = 1 over the whole layer: N bf16 read, N bf16 written) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE can be scaled against it")
    ap.add_argument("--cpu-sample", type=int, default=16 << 20,
                    help="shard elements the CPU oracle is timed on")
    return ap.parse_args()


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (cross-GPU transport is out of scope); "
              "use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import synth
    import paper_2205_00119_amd as mics

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    cfg = synth.CONFIGS[args.config]
    p, k, r, s, S, N, n_pad = cfg.p, cfg.k, cfg.r, cfg.s, cfg.S, cfg.N, cfg.N_pad
    if args.blocks_per_cu:
        mics.mics_set_blocks_per_cu(args.blocks_per_cu)
    group = args.view == "group"
    count = n_pad if group else S                 # elements per a2/a3/a4 call
    offset = 0 if group else args.rank * S
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    # ---- synthetic inputs, generated on the device ------------------------------------------
    tab_g = torch.from_numpy(synth.normal_table(cfg.sigma_grad, "bf16").view(np.int16)).to(dev)
    tab_go = None
    if cfg.outlier_frac:
        tab_go = torch.from_numpy(
            synth.normal_table(cfg.sigma_grad * cfg.outlier_scale, "bf16").view(np.int16)).to(dev)
    pf32 = args.param_dtype == "f32"
    pb, p_dt = (4, torch.float32) if pf32 else (2, torch.int16)      # parameter element bytes / dtype
    tab_p = (torch.from_numpy(synth.normal_table(cfg.sigma_master, "f32")).to(dev) if pf32 else
             torch.from_numpy(synth.normal_table(cfg.sigma_master, "bf16").view(np.int16)).to(dev))
    tab_w = torch.from_numpy(synth.normal_table(cfg.sigma_master, "f32")).to(dev)
    sigma_acc = cfg.sigma_grad * (p * s) ** 0.5
    tab_a = torch.from_numpy(synth.normal_table(sigma_acc, "f32")).to(dev)

    def fill(t, key, x0, table, elem_bytes, outl=None, frac=0.0):
        synth.fill_device(t.data_ptr(), key, x0, t.numel(), table.data_ptr(), elem_bytes,
                          outl.data_ptr() if outl is not None else 0, frac, sh)

    nodes = p // k
    F = torch.empty(N, dtype=p_dt, device=dev)
    if not args.coalesced:
        # a1: the gathered-but-unordered parameter W = [T_0 .. T_{k-1}], T_l = [C_l, C_{k+l}, ...]
        W = torch.empty(n_pad, dtype=p_dt, device=dev)
        for g in range(p):
            j, l = divmod(g, k)
            slot = (l * nodes + j) * S
            fill(W[slot:slot + S], synth.stream_key(cfg.seed, synth.ROLE_PARAM, 0, 0, g), 0, tab_p, pb)
        T_views = [W[l * nodes * S:(l + 1) * nodes * S] for l in range(k)]

        # a2: per micro-step, p gradient buffers covering the elements this call owns
        n_sets = 1 if group else s
        # Each rank buffer is its own 16-byte aligned allocation in a real run, and the rank reads
        # it from element offset g*S on: rows are padded so that every view below starts at the
        # same position inside a 16-byte line as that offset would (0 unless S is odd).
        lead = offset % 8
        row = -(-(lead + count) // 8) * 8
        if args.grad_dtype == "bf16":
            grads = torch.empty((n_sets, p, row), dtype=torch.int16, device=dev)
            g_tab, g_out, g_bytes = tab_g, tab_go, 2
        elif args.grad_dtype == "f16":
            grads = torch.empty((n_sets, p, row), dtype=torch.int16, device=dev)
            as_f16 = lambda sig: torch.from_numpy(
                synth.normal_table(sig, "f32").astype(np.float16).view(np.int16)).to(dev)
            g_tab = as_f16(cfg.sigma_grad * 1024)          # loss-scaled by 2^10
            g_out = as_f16(cfg.sigma_grad * 1024 * cfg.outlier_scale) if cfg.outlier_frac else None
            g_bytes = 2
        else:
            grads = torch.empty((n_sets, p, row), dtype=torch.float32, device=dev)
            g_tab = torch.from_numpy(synth.normal_table(cfg.sigma_grad, "f32")).to(dev)
            g_out = (torch.from_numpy(synth.normal_table(cfg.sigma_grad * cfg.outlier_scale, "f32")).to(dev)
                     if cfg.outlier_frac else None)
            g_bytes = 4
        for t in range(n_sets):
            for q in range(p):
                fill(grads[t, q, lead:lead + count], synth.stream_key(cfg.seed, synth.ROLE_GRAD, 0, t, q),
                     offset, g_tab, g_bytes, g_out, cfg.outlier_frac)
        grad_tables = [[grads[t % n_sets, q, lead:lead + count] for q in range(p)] for t in range(s)]
    else:
        if group or cfg.name == "tiny" or cfg.align != 8:
            print("--coalesced needs a transformer-layer configuration in rank view", file=sys.stderr)
            sys.exit(2)
        h = int(cfg.name[1:])
        lay = synth.coalesced_layout([n for _, n in synth.layer_tensors(h)], p, k, align=8)
        assert lay.shard_off[-1] == S and lay.flat_off[-1] == N
        # a1: k separate stage-1 buffers, tensor after tensor, each holding that tensor's p/k chunks
        T_views = [torch.empty(lay.stage1_off[-1], dtype=p_dt, device=dev) for _ in range(k)]
        for t, St in enumerate(lay.S):
            for g in range(p):
                j, l = divmod(g, k)
                at = lay.stage1_off[t] + j * St
                fill(T_views[l][at:at + St], synth.stream_key(cfg.seed, synth.ROLE_PARAM, t, 0, g), 0, tab_p, pb)
        reorder_segs = mics._segments(lay.reorder_segments())
        # a2: every rank's full gradient buffer (all tensors, p*S_t each); the rank reads its slices
        n_sets = min(s, 4)
        grads = torch.empty((n_sets, p, lay.grad_off[-1]), dtype=torch.int16, device=dev)
        for t in range(n_sets):
            for q in range(p):
                fill(grads[t, q], synth.stream_key(cfg.seed, synth.ROLE_GRAD, 0, t, q), 0, tab_g, 2,
                     tab_go, cfg.outlier_frac)
        grad_tables = [[grads[t % n_sets, q] for q in range(p)] for t in range(s)]
        reduce_segs = mics._segments(lay.reduce_segments(args.rank))

    # a3: this replica's accumulator plus the r-1 copies that arrive from the other replicas
    acc = torch.empty(count, dtype=torch.float32, device=dev)
    others = torch.empty((r - 1, count), dtype=torch.float32, device=dev)
    for c in range(1, r):
        fill(others[c - 1], synth.stream_key(cfg.seed, synth.ROLE_ACC, c), offset, tab_a, 4)
    copies = [acc] + [others[c] for c in range(r - 1)]
    avg = torch.empty(count, dtype=torch.float32, device=dev)
    scale = float(np.float32(1.0 / (r * p * s)))

    # a4: master weights, zero moments, bf16 parameter out
    master = torch.empty(count, dtype=torch.float32, device=dev)
    fill(master, synth.stream_key(cfg.seed, synth.ROLE_MASTER), offset, tab_w, 4)
    exp_avg = torch.zeros(count, dtype=torch.float32, device=dev)
    exp_avg_sq = torch.zeros(count, dtype=torch.float32, device=dev)
    param = None if pf32 else torch.empty(count, dtype=torch.int16, device=dev)
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)
    torch.cuda.synchronize()

    grad_code = {"bf16": mics.MICS_DTYPE_BF16, "f16": mics.MICS_DTYPE_F16, "f32": mics.MICS_DTYPE_F32}[args.grad_dtype]
    gb = 4 if args.grad_dtype == "f32" else 2
    if args.grad_dtype != "bf16" and args.coalesced:
        print("--grad-dtype other than bf16 is for the flat layout", file=sys.stderr)
        sys.exit(2)
    ev = {name: [] for name in ("a1", "a2", "a3", "a4")}
    all_marks = []

    def step(it, timed):
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(5)] if timed else None
        if timed:
            marks[0].record(stream)
        if args.coalesced:
            mics.mics_hier_gather_reorder_coalesced(F, T_views, reorder_segs, p, k, pb, stream=sh)
        else:
            mics.mics_hier_gather_reorder(F, T_views, N, S, p, k, pb, stream=sh)
        if timed:
            marks[1].record(stream)
        for t in range(s):
            for _ in range(args.gathers_per_microstep):
                if args.coalesced:
                    mics.mics_hier_gather_reorder_coalesced(F, T_views, reorder_segs, p, k, pb, stream=sh)
                else:
                    mics.mics_hier_gather_reorder(F, T_views, N, S, p, k, pb, stream=sh)
            if args.coalesced:
                mics.mics_reduce_scatter_accum_coalesced(acc, grad_tables[t], reduce_segs, t > 0, stream=sh)
            elif args.grad_dtype != "bf16":
                mics.mics_reduce_scatter_accum_typed(acc, grad_tables[t], 0, count, t > 0, grad_code, stream=sh)
            else:
                mics.mics_reduce_scatter_accum(acc, grad_tables[t], 0, count, t > 0, stream=sh)
        if timed:
            marks[2].record(stream)
        if args.fused:
            if timed:
                marks[3].record(stream)
            mics.mics_replica_average_adam_shard(master, exp_avg, exp_avg_sq, param, copies, count, scale,
                                                 step=it, stream=sh, **hp)
        else:
            mics.mics_replica_average(avg, copies, count, scale, stream=sh)
            if timed:
                marks[3].record(stream)
            mics.mics_adam_shard(master, exp_avg, exp_avg_sq, param, avg, count, step=it, stream=sh, **hp)
        if timed:
            marks[4].record(stream)
            all_marks.append(marks)

    if args.calibration_copy:
        if args.coalesced:
            print("--calibration-copy is for the flat layout", file=sys.stderr)
            sys.exit(2)
        mics.mics_hier_gather_reorder(F, [W], N, N, 1, 1, pb, stream=sh)
        torch.cuda.synchronize()
    for it in range(1, args.warmup + 1):
        step(it, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for it in range(args.warmup + 1, args.warmup + args.steps + 1):
        step(it, True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    # a plain copy of the layer (the reorder with p = k = 1) as this chip's practical ceiling for
    # a one-read-one-write stream; reported beside the nominal peak, outside the timed steps
    copy_gbps = None
    if not args.coalesced:
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        mics.mics_hier_gather_reorder(F, [W], N, N, 1, 1, pb, stream=sh)
        c0.record(stream)
        for _ in range(5):
            mics.mics_hier_gather_reorder(F, [W], N, N, 1, 1, pb, stream=sh)
        c1.record(stream)
        c1.synchronize()
        copy_gbps = 5 * 2 * pb * N / (c0.elapsed_time(c1) * 1e-3) / 1e9

    for marks in all_marks:
        for i, name in enumerate(("a1", "a2", "a3", "a4")):
            ev[name].append(marks[i].elapsed_time(marks[i + 1]))
    ms = {name: float(np.mean(ev[name])) for name in ("a1", "a2", "a3", "a4")}
    ms_step = wall * 1e3 / args.steps

    # ---- algorithmic bytes (what the method must move) ---------------------------------------
    b_a1 = 2 * pb * N
    b_a2_first, b_a2_next = count * (gb * p + 4), count * (gb * p + 8)
    b_a2 = b_a2_first + (s - 1) * b_a2_next
    b_a3 = 0 if args.fused else count * (4 * r + 4)
    out_a4 = 12 if pf32 else 14                      # master, m, v (+ bf16 parameter)
    b_a4 = count * (4 * r + 12 + out_a4) if args.fused else count * (16 + out_a4)
    extra_gathers = args.gathers_per_microstep * s
    b_step = b_a1 * (1 + extra_gathers) + b_a2 + b_a3 + b_a4
    gbps = b_step / (ms_step * 1e-3) / 1e9
    # with interleaved gathers the a2 bracket holds them too: bytes and launches of both
    a2_launch_ms = ms["a2"] / (s + extra_gathers)
    a2_gbps = ((b_a2 + extra_gathers * b_a1) / (s + extra_gathers)) / (a2_launch_ms * 1e-3) / 1e9

    result = {
        "metric": "effective HBM GB/s per shard step",
        "value": round(gbps, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": f"{args.grad_dtype} in / f32 accumulate" + (", f32 parameters" if pf32 else ""),
        "data": "synthetic",
        "pct_of_peak_hbm": round(100.0 * gbps / PEAK_HBM_GBPS, 2),
        "plain_copy_GBps": round(copy_gbps, 1) if copy_gbps else None,
        "pct_of_plain_copy": round(100.0 * gbps / copy_gbps, 2) if copy_gbps else None,
        "elements_per_s": round(count / (ms_step * 1e-3), 1),
        "config": {
            "workload": f"{cfg.name}: one transformer layer h={cfg.name[1:]} N={N}, p={p} "
                        f"({nodes} nodes x k={k}), r={r}, s={s}, {args.view} view "
                        f"({count} elements per reduce/average/Adam call)"
                        + (", coalesced: 16 separately sharded tensors" if args.coalesced else ""),
            "view": args.view, "coalesced": bool(args.coalesced), "fused_average_adam": bool(args.fused),
            "gathers_per_microstep": args.gathers_per_microstep, "N": N, "S": S, "p": p, "k": k, "r": r, "s": s,
            "algorithmic_bytes_per_step": b_step,
        },
        "kernels": {
            name: {"ms": round(ms[name], 4),
                   "GB/s": round(b / (ms[name] * 1e-3) / 1e9, 1)}
            for name, b in (("a1", b_a1), ("a2", b_a2 + extra_gathers * b_a1), ("a3", b_a3), ("a4", b_a4))
            if not (args.fused and name == "a3")
        },
        "roofline": {
            "kernel": (f"rsa_seg_kernel<{p}> (mics_reduce_scatter_accum_coalesced)" if args.coalesced
                       else f"rsa_vec_kernel<{p}> (mics_reduce_scatter_accum)" if args.grad_dtype == "bf16"
                       else f"rsa_typed_vec_kernel<{args.grad_dtype},{p}> (mics_reduce_scatter_accum_typed)"),
            "bound": "hbm",
            "achieved": round(a2_gbps, 1),
            "peak": PEAK_HBM_GBPS,
            "unit": "GB/s",
            "frac": round(a2_gbps / PEAK_HBM_GBPS, 4),
            "avg_launch_ms": round(a2_launch_ms, 5),
            "algorithmic_bytes_per_launch": b_a2 // s,
            "traffic": (None if args.coalesced or args.grad_dtype != "bf16"
                        else MEASURED_TRAFFIC.get((cfg.name, args.view))),
        },
    }
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(cfg, args)
    print(json.dumps(result))


# HBM bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# each scaled by what the same counter reads for a plain copy of known size (factors 1.9999 and
# 0.9983), averaged over a step's 11 accumulating + 1 overwriting launches
# (profiles/all_kernels_h8192_rank_view.md).  None = not measured for that workload.
MEASURED_TRAFFIC = {("h8192", "rank"): (11 * 2013200701 + 1811857686) // 12}


def cpu_baseline(cfg, args):
    """Time the CPU oracle (as it stands) on a bounded sample of the same workload: the first
    `m` elements of the rank's shard for a2/a3/a4 and the matching p*m elements for a1."""
    import numpy as np
    import oracle
    import synth

    p, k, r, s = cfg.p, cfg.k, cfg.r, cfg.s
    m = min(cfg.S, args.cpu_sample)
    offset = args.rank * cfg.S
    cores = min(16, os.cpu_count() or 1)
    gtab = synth.normal_table(cfg.sigma_grad, "bf16")
    gout = synth.normal_table(cfg.sigma_grad * cfg.outlier_scale, "bf16") if cfg.outlier_frac else None
    ptab = synth.normal_table(cfg.sigma_master, "bf16")
    shards = [synth.fill_host(synth.stream_key(cfg.seed, synth.ROLE_PARAM, 0, 0, g), 0, m, ptab)
              for g in range(p)]
    T = [np.concatenate([shards[j * k + l] for j in range(p // k)]) for l in range(k)]
    grads = [[synth.fill_host(synth.stream_key(cfg.seed, synth.ROLE_GRAD, 0, t, q), offset, m, gtab,
                              gout, cfg.outlier_frac) for q in range(p)] for t in range(s)]
    atab = synth.normal_table(cfg.sigma_grad * (p * s) ** 0.5, "f32")
    others = [synth.fill_host(synth.stream_key(cfg.seed, synth.ROLE_ACC, c), offset, m, atab)
              for c in range(1, r)]
    w = synth.fill_host(synth.stream_key(cfg.seed, synth.ROLE_MASTER), offset, m,
                        synth.normal_table(cfg.sigma_master, "f32"))
    mo, vo = np.zeros(m, np.float32), np.zeros(m, np.float32)
    acc = np.empty(m, np.float32)
    scale = float(np.float32(1.0 / (r * p * s)))
    hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)
    bytes_sample = 4 * p * m + m * ((2 * p + 4) + (s - 1) * (2 * p + 8)) + m * (4 * r + 4) + m * 30

    def one_pass(step):
        oracle.hier_gather_reorder(T, p * m, m, p)
        for t in range(s):
            oracle.reduce_scatter_accum(acc, grads[t], 0, t > 0)
        avg = oracle.replica_average([acc] + others, scale)
        oracle.adam_shard(w, mo, vo, avg, step=step, **hp)

    out = {}
    for label, threads in (("all", cores), ("one", 1)):
        oracle.set_threads(threads)
        t0 = time.perf_counter()
        one_pass(1 if label == "all" else 2)
        out[label] = time.perf_counter() - t0
    oracle.set_threads(1)
    return {
        "value": round(bytes_sample / out["all"] / 1e9, 2),
        "unit": "GB/s",
        "cores": cores,
        "kind": "oracle",
        "sample": f"first {m} of the rank's {cfg.S} shard elements (and the matching {p * m} of the "
                  f"layer for the reorder), one full step, {cores} threads",
        "seconds": round(out["all"], 3),
        "value_1_thread": round(bytes_sample / out["one"] / 1e9, 2),
        "seconds_1_thread": round(out["one"], 3),
        "elements_per_s": round(m / out["all"], 1),
    }


if __name__ == "__main__":
    main()
