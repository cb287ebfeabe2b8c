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

Prints one JSON line for the rank view.  Unless --no-group-view is given it then runs a few
steps of the whole-group view of the same configuration -- the same kernels over all p shards
at once (p*S elements per call, every accumulator and output far larger than the 256 MB
Infinity Cache; the gradient buffers are then shared by the micro-steps because s*p*N_pad bf16
would not fit) -- and reports it as the `group_view` object of the same line.  `--view group`
makes the whole-group view the main record instead.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBPS = 8000.0   # MI355X HBM3E, published
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic_per_launch.txt")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2205_00119_amd", "csrc", "kernels.hip")


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
                         "full-length rank gradient buffers (4 sets, cycled over the micro-steps); with "
                         "a configuration of shard alignment 1 every tensor gets 5 extra elements, so "
                         "that no shard, offset or chunk is 16-byte clean")
    ap.add_argument("--grad-dtype", choices=["bf16", "f16", "f32"], default="bf16",
                    help="storage format of the gradient buffers the reduce-scatter-accumulate reads")
    ap.add_argument("--param-dtype", choices=["bf16", "f16", "f32"], default="bf16",
                    help="f32: plain float32 training -- the gathered parameter has 4-byte elements and "
                         "the Adam step writes no 16-bit copy; f16: the Adam step writes IEEE binary16 "
                         "parameters (mixed precision without bf16), the gather moves the same 2-byte elements")
    ap.add_argument("--gathers-per-microstep", type=int, default=0,
                    help="run this many extra gather reorders before every reduce-scatter-accumulate, as "
                         "a training run does (parameters are gathered in the forward and in the backward "
                         "pass of every micro-step); the default step gathers once")
    ap.add_argument("--fused", action="store_true",
                    help="run the replica average and the Adam step as one fused call "
                         "(mics_replica_average_adam_shard): 4r+26 instead of 4r+34 bytes per element")
    ap.add_argument("--stage1-out", action="store_true",
                    help="the Adam step writes its bf16 shard straight into the stage-1 buffer of the next "
                         "parameter gather (at T_l + j*S) instead of a buffer of its own")
    ap.add_argument("--blocks-per-cu", type=int, default=0)
    ap.add_argument("--launch-shape", action="append", default=[], metavar="FAMILY:LANES:WAVES",
                    help="launch shape of a kernel family (reorder, reduce, average, adam, fused): lanes per "
                         "workgroup and wavefronts per compute unit, 0 = built-in choice (mics_set_launch_shape); "
                         "may be given several times")
    ap.add_argument("--stream-threshold-mb", type=int, default=0,
                    help="outputs larger than this are streamed past the caches; 0 = the library's default of "
                         "224 (mics_set_stream_threshold_bytes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-group-view", action="store_true",
                    help="skip the whole-group view that follows the rank-view steps")
    ap.add_argument("--group-steps", type=int, default=5, help="timed steps of the group_view record")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="before the steps, run one plain copy of known size (the reorder with "
                         "p = k = 1 over the whole layer: N bf16 read, N bf16 written) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE can be scaled against it")
    ap.add_argument("--cpu-sample", type=int, default=32 << 20,
                    help="shard elements the CPU oracle is timed on")
    return ap.parse_args()


def stats(samples):
    import numpy as np
    a = np.asarray(samples, dtype=np.float64)
    return {"mean": float(a.mean()), "median": float(np.median(a)), "min": float(a.min())}


def kernel_source_hash():
    with open(KERNEL_SOURCE, "rb") as f:
        return hashlib.sha256(f.read()).hexdigest()[:16]


def traffic_from_profile(workload, view, variant):
    """HBM bytes per launch of the dominant kernel as measured by rocprofv3 --pmc FETCH_SIZE /
    WRITE_SIZE runs of this workload (written by profile_summary.py into TRAFFIC_FILE together
    with the hash of the kernel source it was measured on).  None unless the file has a line for
    this workload, view and variant whose hash matches the current source."""
    try:
        lines = open(TRAFFIC_FILE).read().splitlines()
    except OSError:
        return None, None
    want = kernel_source_hash()
    for line in lines:
        f = line.split()
        if len(f) >= 5 and not line.startswith("#") and f[:3] == [workload, view, variant]:
            if f[3] == want:
                return int(f[4]), f"profiles/{os.path.basename(TRAFFIC_FILE)} (kernels.hip sha256 {want})"
            return None, f"stale: measured on kernels.hip sha256 {f[3]}, current {want}"
    return None, None


class Workload:
    """Buffers and the step of one view of one configuration."""

    def __init__(self, args, view, mics, synth, torch, np):
        self.args, self.view, self.mics, self.torch, self.np = args, view, mics, torch, np
        cfg = self.cfg = synth.CONFIGS[args.config]
        dev = torch.device("cuda:0")
        p, k, r, s, S = cfg.p, cfg.k, cfg.r, cfg.s, cfg.S
        self.group = group = view == "group"
        self.stream = torch.cuda.current_stream()
        sh = self.sh = self.stream.cuda_stream
        self.pf32 = pf32 = args.param_dtype == "f32"
        self.pb, p_dt = (4, torch.float32) if pf32 else (2, torch.int16)   # parameter element bytes / dtype
        pb = self.pb

        tab_g = torch.from_numpy(synth.normal_table(cfg.sigma_grad, "bf16").view(np.int16)).to(dev)
        tab_go = None
        if cfg.outlier_frac:
            tab_go = torch.from_numpy(
                synth.normal_table(cfg.sigma_grad * cfg.outlier_scale, "bf16").view(np.int16)).to(dev)
        tab_p = (torch.from_numpy(synth.normal_table(cfg.sigma_master, "f32")).to(dev) if pf32 else
                 torch.from_numpy(synth.normal_table(cfg.sigma_master, "bf16").view(np.int16)).to(dev))
        tab_w = torch.from_numpy(synth.normal_table(cfg.sigma_master, "f32")).to(dev)
        tab_a = torch.from_numpy(synth.normal_table(cfg.sigma_grad * (p * s) ** 0.5, "f32")).to(dev)

        def fill(t, key, x0, table, elem_bytes, outl=None, frac=0.0):
            synth.fill_device(t.data_ptr(), key, x0, t.numel(), table.data_ptr(), elem_bytes,
                              outl.data_ptr() if outl is not None else 0, frac, sh)

        nodes = p // k
        self.gb = 4 if args.grad_dtype == "f32" else 2
        self.grad_code = {"bf16": mics.MICS_DTYPE_BF16, "f16": mics.MICS_DTYPE_F16,
                          "f32": mics.MICS_DTYPE_F32}[args.grad_dtype]

        def grad_tables_for(fmt):
            """(torch dtype of a gradient buffer, value table, outlier table) for a storage format."""
            if fmt == "bf16":
                return torch.int16, tab_g, tab_go
            if fmt == "f16":
                as_f16 = lambda sig: torch.from_numpy(
                    synth.normal_table(sig, "f32").astype(np.float16).view(np.int16)).to(dev)
                return (torch.int16, as_f16(cfg.sigma_grad * 1024),                     # loss-scaled by 2^10
                        as_f16(cfg.sigma_grad * 1024 * cfg.outlier_scale) if cfg.outlier_frac else None)
            return (torch.float32, torch.from_numpy(synth.normal_table(cfg.sigma_grad, "f32")).to(dev),
                    torch.from_numpy(synth.normal_table(cfg.sigma_grad * cfg.outlier_scale, "f32")).to(dev)
                    if cfg.outlier_frac else None)

        g_dt, g_tab, g_out = grad_tables_for(args.grad_dtype)
        if not args.coalesced:
            self.N, self.S = N, S = cfg.N, cfg.S
            n_pad = cfg.N_pad
            self.count = count = n_pad if group else S          # elements per a2/a3/a4 call
            offset = 0 if group else args.rank * S
            self.F = torch.empty(N, dtype=p_dt, device=dev)
            # a1: the gathered-but-unordered parameter W = [T_0 .. T_{k-1}], T_l = [C_l, C_{k+l}, ...]
            self.W = W = torch.empty(n_pad, dtype=p_dt, device=dev)
            for g in range(p):
                j, l = divmod(g, k)
                slot = (l * nodes + j) * S
                fill(W[slot:slot + S], synth.stream_key(cfg.seed, synth.ROLE_PARAM, 0, 0, g), 0, tab_p, pb)
            self.T_views = [W[l * nodes * S:(l + 1) * nodes * S] for l in range(k)]

            # a2: per micro-step, p gradient buffers covering the elements this call owns.  Each rank
            # buffer is its own 16-byte aligned allocation in a real run, and the rank reads it from
            # element offset g*S on: rows are padded so that every view below starts at the same
            # position inside a 16-byte line as that offset would (0 unless S is odd).
            n_sets = 1 if group else s
            lead = offset % 8
            row = -(-(lead + count) // 8) * 8
            grads = torch.empty((n_sets, p, row), dtype=g_dt, device=dev)
            for t in range(n_sets):
                for q in range(p):
                    fill(grads[t, q, lead:lead + count], synth.stream_key(cfg.seed, synth.ROLE_GRAD, 0, t, q),
                         offset, g_tab, self.gb, g_out, cfg.outlier_frac)
            self.grads = grads
            self.grad_tables = [[grads[t % n_sets, q, lead:lead + count] for q in range(p)] for t in range(s)]
        else:
            if group or cfg.name == "tiny":
                raise SystemExit("--coalesced needs a transformer-layer configuration in rank view")
            h = int(cfg.name[1:].split("_")[0])
            numels = [n for _, n in synth.layer_tensors(h)]
            if cfg.align != 8:
                numels = [n + 5 for n in numels]        # every shard odd, nothing 16-byte clean
            lay = self.lay = synth.coalesced_layout(numels, p, k, align=cfg.align)
            self.N, self.S = N, S = lay.flat_off[-1], lay.shard_off[-1]
            self.count = count = S
            offset = args.rank * cfg.S
            self.F = torch.empty(N, dtype=p_dt, device=dev)
            # a1: k separate stage-1 buffers, tensor after tensor, each holding that tensor's p/k chunks
            self.T_views = [torch.empty(lay.stage1_off[-1], dtype=p_dt, device=dev) for _ in range(k)]
            for t, St in enumerate(lay.S):
                for g in range(p):
                    j, l = divmod(g, k)
                    at = lay.stage1_off[t] + j * St
                    fill(self.T_views[l][at:at + St], synth.stream_key(cfg.seed, synth.ROLE_PARAM, t, 0, g), 0,
                         tab_p, pb)
            self.reorder_segs = mics._segments(lay.reorder_segments())
            # a2: every rank's full gradient buffer (all tensors, p*S_t each); the rank reads its slices
            # distinct gradient data per micro-step as far as ~120 GB go (every set is far beyond any cache)
            n_sets = max(1, min(s, 4, int(120e9 // (self.gb * p * lay.grad_off[-1]))))
            grads = torch.empty((n_sets, p, -(-lay.grad_off[-1] // 8) * 8), dtype=g_dt, device=dev)
            for t in range(n_sets):
                for q in range(p):
                    fill(grads[t, q], synth.stream_key(cfg.seed, synth.ROLE_GRAD, 0, t, q), 0, g_tab, self.gb,
                         g_out, cfg.outlier_frac)
            self.grads = grads
            self.grad_tables = [[grads[t % n_sets, q] for q in range(p)] for t in range(s)]
            self.reduce_segs = mics._segments(lay.reduce_segments(args.rank))

        # a3: this replica's accumulator plus the r-1 copies that arrive from the other replicas,
        # each an allocation of its own as on a real rank
        self.acc = torch.empty(count, dtype=torch.float32, device=dev)
        others = [torch.empty(count, dtype=torch.float32, device=dev) for _ in range(r - 1)]
        for c in range(1, r):
            fill(others[c - 1], synth.stream_key(cfg.seed, synth.ROLE_ACC, c), offset, tab_a, 4)
        self.copies = [self.acc] + others
        self.avg = torch.empty(count, dtype=torch.float32, device=dev)
        self.scale = float(np.float32(1.0 / (r * p * s)))

        # a4: master weights, zero moments, bf16 parameter out
        self.master = torch.empty(count, dtype=torch.float32, device=dev)
        fill(self.master, synth.stream_key(cfg.seed, synth.ROLE_MASTER), offset, tab_w, 4)
        self.exp_avg = torch.zeros(count, dtype=torch.float32, device=dev)
        self.exp_avg_sq = torch.zeros(count, dtype=torch.float32, device=dev)
        if pf32:
            self.param = None
        elif args.stage1_out:
            if args.coalesced or group:
                raise SystemExit("--stage1-out is for the flat layout in rank view")
            j, l = divmod(args.rank, k)
            self.param = self.T_views[l][j * S:(j + 1) * S]     # T_l + j*S
        else:
            self.param = torch.empty(count, dtype=torch.int16, device=dev)
        self.hp = dict(lr=cfg.lr, beta1=cfg.beta1, beta2=cfg.beta2, eps=cfg.eps, weight_decay=cfg.weight_decay)
        torch.cuda.synchronize()
        self.marks = []

    def gather(self):
        a, cfg, m = self.args, self.cfg, self.mics
        if a.coalesced:
            m.mics_hier_gather_reorder_coalesced(self.F, self.T_views, self.reorder_segs, cfg.p, cfg.k, self.pb,
                                                 stream=self.sh)
        else:
            m.mics_hier_gather_reorder(self.F, self.T_views, self.N, self.S, cfg.p, cfg.k, self.pb, stream=self.sh)

    def step(self, it, timed):
        a, cfg, m, torch = self.args, self.cfg, self.mics, self.torch
        stream, sh, count = self.stream, self.sh, self.count
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(5)] if timed else None
        if timed:
            marks[0].record(stream)
        self.gather()
        if timed:
            marks[1].record(stream)
        for t in range(cfg.s):
            for _ in range(a.gathers_per_microstep):
                self.gather()
            if a.coalesced and a.grad_dtype != "bf16":
                m.mics_reduce_scatter_accum_coalesced_typed(self.acc, self.grad_tables[t], self.reduce_segs, t > 0,
                                                            self.grad_code, stream=sh)
            elif a.coalesced:
                m.mics_reduce_scatter_accum_coalesced(self.acc, self.grad_tables[t], self.reduce_segs, t > 0, stream=sh)
            elif a.grad_dtype != "bf16":
                m.mics_reduce_scatter_accum_typed(self.acc, self.grad_tables[t], 0, count, t > 0, self.grad_code,
                                                  stream=sh)
            else:
                m.mics_reduce_scatter_accum(self.acc, self.grad_tables[t], 0, count, t > 0, stream=sh)
        if timed:
            marks[2].record(stream)
        if a.fused:
            if timed:
                marks[3].record(stream)
            if a.param_dtype == "f16":
                m.mics_replica_average_adam_shard_typed(self.master, self.exp_avg, self.exp_avg_sq, self.param,
                                                        m.MICS_DTYPE_F16, self.copies, count, self.scale, step=it,
                                                        stream=sh, **self.hp)
            else:
                m.mics_replica_average_adam_shard(self.master, self.exp_avg, self.exp_avg_sq, self.param,
                                                  self.copies, count, self.scale, step=it, stream=sh, **self.hp)
        else:
            m.mics_replica_average(self.avg, self.copies, count, self.scale, stream=sh)
            if timed:
                marks[3].record(stream)
            if a.param_dtype == "f16":
                m.mics_adam_shard_typed(self.master, self.exp_avg, self.exp_avg_sq, self.param, m.MICS_DTYPE_F16,
                                        self.avg, count, step=it, stream=sh, **self.hp)
            else:
                m.mics_adam_shard(self.master, self.exp_avg, self.exp_avg_sq, self.param, self.avg, count, step=it,
                                  stream=sh, **self.hp)
        if timed:
            marks[4].record(stream)
            self.marks.append(marks)

    def plain_copy_gbps(self):
        """A plain copy of the layer (the reorder with p = k = 1) as this chip's practical ceiling
        for a one-read-one-write stream; outside the timed steps."""
        if self.args.coalesced:
            return None
        torch, m = self.torch, self.mics
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m.mics_hier_gather_reorder(self.F, [self.W], self.N, self.N, 1, 1, self.pb, stream=self.sh)
        c0.record(self.stream)
        for _ in range(5):
            m.mics_hier_gather_reorder(self.F, [self.W], self.N, self.N, 1, 1, self.pb, stream=self.sh)
        c1.record(self.stream)
        c1.synchronize()
        return 5 * 2 * self.pb * self.N / (c0.elapsed_time(c1) * 1e-3) / 1e9

    def run(self, steps, warmup):
        """`warmup` untimed steps, then exactly `steps` timed ones between two synchronisations."""
        torch = self.torch
        if self.args.calibration_copy and not self.args.coalesced:
            self.mics.mics_hier_gather_reorder(self.F, [self.W], self.N, self.N, 1, 1, self.pb, stream=self.sh)
            torch.cuda.synchronize()
        for it in range(1, warmup + 1):
            self.step(it, False)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for it in range(warmup + 1, warmup + steps + 1):
            self.step(it, True)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        # the same steps once more without the per-kernel event marks (each mark is a packet of its
        # own on the stream: about 4 us, which shows on the small configurations); reported beside
        # `value`, never instead of it
        t0 = time.perf_counter()
        for it in range(warmup + steps + 1, warmup + 2 * steps + 1):
            self.step(it, False)
        torch.cuda.synchronize()
        self.wall_unmarked = time.perf_counter() - t0
        return self.record(steps, warmup, wall)

    def record(self, steps, warmup, wall):
        a, cfg = self.args, self.cfg
        p, k, r, s, count, N, pb, gb = cfg.p, cfg.k, cfg.r, cfg.s, self.count, self.N, self.pb, self.gb
        names = ("a1", "a2", "a3", "a4")
        ev = {name: [] for name in names}
        step_ms = []
        for marks in self.marks:
            for i, name in enumerate(names):
                ev[name].append(marks[i].elapsed_time(marks[i + 1]))
            step_ms.append(marks[0].elapsed_time(marks[4]))
        st = {name: stats(ev[name]) for name in names}
        st_step = stats(step_ms)
        ms_step = wall * 1e3 / steps

        # ---- algorithmic bytes (what the method must move) ---------------------------------------
        b_a1 = 2 * pb * N
        b_a2_first, b_a2_next = count * (gb * p + 4), count * (gb * p + 8)
        b_a2 = b_a2_first + (s - 1) * b_a2_next
        b_a3 = 0 if a.fused else count * (4 * r + 4)
        out_a4 = 12 if self.pf32 else 14                      # master, m, v (+ bf16 parameter)
        b_a4 = count * (4 * r + 12 + out_a4) if a.fused else count * (16 + out_a4)
        extra_gathers = a.gathers_per_microstep * s
        b_step = b_a1 * (1 + extra_gathers) + b_a2 + b_a3 + b_a4
        gbps = b_step / (ms_step * 1e-3) / 1e9
        # with interleaved gathers the a2 bracket holds them too: bytes and launches of both
        launches = s + extra_gathers
        a2_bytes = b_a2 + extra_gathers * b_a1
        a2_launch = {key: st["a2"][key] / launches for key in ("mean", "median", "min")}
        a2_gbps = (a2_bytes / launches) / (a2_launch["mean"] * 1e-3) / 1e9
        variant = ("coalesced" if a.coalesced else "flat") + "-" + a.grad_dtype
        traffic, traffic_src = (None, None)
        if not extra_gathers and not self.pf32:
            traffic, traffic_src = traffic_from_profile(cfg.name, self.view, variant)
        kind = {"bf16": 0, "f16": 1, "f32": 2}[a.grad_dtype]
        bytes_of = {"a1": b_a1, "a2": a2_bytes, "a3": b_a3, "a4": b_a4}
        return {
            "metric": "effective HBM GB/s per shard step",
            "value": round(gbps, 1),
            "unit": "GB/s",
            "n_gpus": 1,
            "steps": steps,
            "warmup": warmup,
            "ms_per_step": round(ms_step, 4),
            "higher_is_better": True,
            "scaling": "weak",
            "vs_baseline": None,
            "dtype": f"{a.grad_dtype} in / f32 accumulate"
                     + (", f32 parameters" if self.pf32 else ", f16 parameters" if a.param_dtype == "f16" else ""),
            "data": "synthetic",
            "pct_of_peak_hbm": round(100.0 * gbps / PEAK_HBM_GBPS, 2),
            "ms_per_step_events": {key: round(val, 4) for key, val in st_step.items()},
            "without_kernel_event_marks": {
                "ms_per_step": round(self.wall_unmarked * 1e3 / steps, 4),
                "value": round(b_step / (self.wall_unmarked / steps) / 1e9, 1),
                "note": "the same number of steps after the timed region, no events between the kernels",
            },
            # shard elements updated per second: over the whole step, and by the Adam kernel alone
            "elements_per_s": round(count / (ms_step * 1e-3), 1),
            "elements_per_s_adam_kernel": round(count / (st["a4"]["mean"] * 1e-3), 1),
            "config": {
                "workload": f"{cfg.name}: "
                            + (f"one transformer layer h={cfg.name[1:].split('_')[0]} " if cfg.name != "tiny"
                               else "flat buffer ")
                            + f"N={N}, p={p} "
                            f"({p // k} nodes x k={k}), r={r}, s={s}, {self.view} view "
                            f"({count} elements per reduce/average/Adam call)"
                            + (", coalesced: 16 separately sharded tensors" if a.coalesced else ""),
                "view": self.view, "coalesced": bool(a.coalesced), "fused_average_adam": bool(a.fused),
                "adam_writes_stage1_buffer": bool(a.stage1_out), "launch_shape_overrides": list(a.launch_shape),
                "stream_threshold_mb_override": a.stream_threshold_mb,
                "gathers_per_microstep": a.gathers_per_microstep, "N": N, "S": self.S, "p": p, "k": k, "r": r, "s": s,
                "algorithmic_bytes_per_step": b_step,
                "accumulator_bytes": 4 * count,
                "accumulator_fits_infinity_cache": 4 * count <= 224 << 20,
            },
            "kernels": {
                name: {"ms": round(st[name]["mean"], 4), "ms_median": round(st[name]["median"], 4),
                       "ms_min": round(st[name]["min"], 4),
                       "GB/s": round(bytes_of[name] / (st[name]["mean"] * 1e-3) / 1e9, 1),
                       "GB/s_median": round(bytes_of[name] / (st[name]["median"] * 1e-3) / 1e9, 1)}
                for name in names if not (a.fused and name == "a3")
            },
            "roofline": {
                "kernel": (f"rsa_seg_kernel<{p}> (mics_reduce_scatter_accum_coalesced)" if a.coalesced
                           else f"rsa_kernel<{kind}, 4, {p if p in (1, 2, 4, 8, 16, 32) else 0}> "
                                f"({'mics_reduce_scatter_accum' if kind == 0 else 'mics_reduce_scatter_accum_typed'})"),
                "bound": "hbm",
                "achieved": round(a2_gbps, 1),
                "peak": PEAK_HBM_GBPS,
                "unit": "GB/s",
                "frac": round(a2_gbps / PEAK_HBM_GBPS, 4),
                "avg_launch_ms": round(a2_launch["mean"], 5),
                "median_launch_ms": round(a2_launch["median"], 5),
                "min_launch_ms": round(a2_launch["min"], 5),
                "algorithmic_bytes_per_launch": a2_bytes // launches,
                "traffic": traffic,
                "traffic_source": traffic_src,
                # in the rank view the accumulator fits the 256 MB Infinity Cache, so up to 8 of its
                # 2p+8 bytes per element may be served there instead of by HBM; the group view's cannot
                "accumulator_may_be_cache_resident": 4 * count <= 224 << 20,
            },
        }


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
    torch.cuda.set_device(torch.device("cuda:0"))
    if args.blocks_per_cu:
        mics.mics_set_blocks_per_cu(args.blocks_per_cu)
    if args.stream_threshold_mb:
        mics.mics_set_stream_threshold_bytes(args.stream_threshold_mb << 20)
    families = {"reorder": mics.MICS_KERNELS_REORDER, "reduce": mics.MICS_KERNELS_REDUCE,
                "average": mics.MICS_KERNELS_AVERAGE, "adam": mics.MICS_KERNELS_ADAM, "fused": mics.MICS_KERNELS_FUSED}
    for spec in args.launch_shape:
        fam, lanes, waves = spec.split(":")
        mics.mics_set_launch_shape(families[fam], int(lanes), int(waves))

    wl = Workload(args, args.view, mics, synth, torch, np)
    result = wl.run(args.steps, args.warmup)
    copy_gbps = wl.plain_copy_gbps()
    result["plain_copy_GBps"] = round(copy_gbps, 1) if copy_gbps else None
    result["pct_of_plain_copy"] = round(100.0 * result["value"] / copy_gbps, 2) if copy_gbps else None
    del wl
    torch.cuda.empty_cache()

    plain = not (args.coalesced or args.stage1_out or args.gathers_per_microstep or args.calibration_copy)
    if args.view == "rank" and plain and not args.no_group_view and args.config != "tiny":
        gv = Workload(args, "group", mics, synth, torch, np).run(args.group_steps, 1)
        result["group_view"] = {key: gv[key] for key in ("value", "unit", "pct_of_peak_hbm", "steps", "warmup",
                                                          "ms_per_step", "ms_per_step_events", "elements_per_s", "elements_per_s_adam_kernel",
                                                          "kernels", "roofline")}
        result["group_view"]["workload"] = gv["config"]["workload"]
        result["group_view"]["algorithmic_bytes_per_step"] = gv["config"]["algorithmic_bytes_per_step"]
        torch.cuda.empty_cache()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(synth.CONFIGS[args.config], args)
    print(json.dumps(result))


def cpu_baseline(cfg, args):
    """Time the CPU oracle (as it stands) on a bounded sample of the same workload: the first
    `m` elements of the rank's shard for a2/a3/a4 and the matching p*m elements for a1."""
    import numpy as np
    import oracle
    import synth

    p, k, r, s = cfg.p, cfg.k, cfg.r, cfg.s
    m = min(cfg.S, args.cpu_sample)
    offset = args.rank * cfg.S
    host_cores = os.cpu_count() or 1
    cores = min(16, host_cores)      # a one-GPU machine gives a job 16 of the host's cores
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
        "host_cores": host_cores,
        "kind": "oracle",
        "sample": f"first {m} of the rank's {cfg.S} shard elements (and the matching {p * m} of the "
                  f"layer for the reorder), one full step, {cores} threads (os.cpu_count() = {host_cores}; "
                  f"capped at the 16 cores a one-GPU job is given)",
        "seconds": round(out["all"], 3),
        "value_1_thread": round(bytes_sample / out["one"] / 1e9, 2),
        "seconds_1_thread": round(out["one"], 3),
        "elements_per_s": round(m / out["all"], 1),
    }


if __name__ == "__main__":
    main()
