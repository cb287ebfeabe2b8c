#!/usr/bin/env python3
"""Message-size sweep of the gather reorder and the reduce-scatter-accumulate on one MI355X.

The paper's collective micro-benchmark (Section 5.2) sweeps message sizes up to 256 MB, because a
single parameter fetch usually gathers less than that.  This script times the on-device halves of
those collectives over the same range, 1 MB .. 256 MB, for partition groups of 16, 32, 64 and 128
ranks (k = 8 devices per node): how the kernels behave on small messages and where the launch
latency floor lies.

  reorder : M = bytes of the gathered bf16 parameter (read M, write M)
  reduce  : M = bytes of one rank's bf16 gradient; the rank reduces its shard, M/(2p) elements,
            from p buffers (rank view, accumulate variant: 2p + 8 bytes per element)

Every measurement rotates through enough distinct buffers that the working set exceeds the
256 MB Infinity Cache, so the figures are HBM figures, not cache figures.  Prints a markdown table.
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--reps", type=int, default=30)
    ap.add_argument("--sizes-mb", default="1,2,4,8,16,32,64,128,256")
    ap.add_argument("--groups", default="16,32,64,128")
    ap.add_argument("--footprint-mb", type=int, default=1024,
                    help="rotate through at least this many MB of distinct buffers per measurement")
    args = ap.parse_args()

    import numpy as np
    import torch
    import synth
    import paper_2205_00119_amd as mics

    assert torch.cuda.is_available(), "needs a GPU"
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    tab = torch.from_numpy(synth.normal_table(1e-3, "bf16").view(np.int16)).to(dev)
    k = 8

    def timed(fn, n_variants):
        for i in range(3):
            fn(i % n_variants)
        torch.cuda.synchronize()
        # one event pair around a batch of back-to-back launches: per-launch time includes the
        # launch gap, which is what a caller of small messages pays
        batch = max(1, min(args.reps, 50))
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for i in range(batch):
            fn(i % n_variants)
        e1.record(stream)
        e1.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / batch

    rows = []
    for mb in [int(x) for x in args.sizes_mb.split(",")]:
        M = mb << 20
        n = M // 2                                    # bf16 elements of the message
        for p in [int(x) for x in args.groups.split(",")]:
            S = synth.shard_elems(n, p, 8)
            n_pad = S * p
            nodes = p // k
            # ---- reorder: rotate over several (source, destination) pairs
            nbuf = max(2, -(-args.footprint_mb // (2 * mb)))
            W = torch.empty((nbuf, n_pad), dtype=torch.int16, device=dev)
            synth.fill_device(W.data_ptr(), synth.stream_key(9, synth.ROLE_PARAM, mb, p), 0, W.numel(),
                              tab.data_ptr(), 2, stream=sh)
            F = torch.empty((nbuf, n), dtype=torch.int16, device=dev)
            # pointer tables are built once, as a C caller would hold them
            views = [mics._table([W[b, l * nodes * S:(l + 1) * nodes * S] for l in range(k)])
                     for b in range(nbuf)]
            dsts = [F[b].data_ptr() for b in range(nbuf)]

            def reorder(i):
                rc = mics.lib.mics_hier_gather_reorder(dsts[i], views[i], n, S, p, k, 2, sh)
                assert rc == 0, mics.mics_last_error()

            t_re = timed(reorder, nbuf)
            del W, F, views
            # ---- reduce (rank view): the rank's slice of each of the p rank buffers
            per_set = S * (2 * p + 4)
            nset = max(2, -(-(args.footprint_mb << 20) // per_set))
            G = torch.empty((nset, p, S), dtype=torch.int16, device=dev)
            synth.fill_device(G.data_ptr(), synth.stream_key(9, synth.ROLE_GRAD, mb, p), 0, G.numel(),
                              tab.data_ptr(), 2, stream=sh)
            acc = torch.zeros((nset, S), dtype=torch.float32, device=dev)
            tables = [mics._table([G[b, q] for q in range(p)]) for b in range(nset)]
            accs = [acc[b].data_ptr() for b in range(nset)]

            def reduce(i):
                rc = mics.lib.mics_reduce_scatter_accum(accs[i], tables[i], 0, S, p, 1, sh)
                assert rc == 0, mics.mics_last_error()

            t_rs = timed(reduce, nset)
            del G, acc, tables
            rows.append((mb, p, S, t_re, 2 * 2 * n / t_re / 1e9, t_rs, S * (2 * p + 8) / t_rs / 1e9))
            print(f"M={mb} MB p={p}: reorder {t_re * 1e6:8.1f} us {rows[-1][4]:7.0f} GB/s | "
                  f"reduce {t_rs * 1e6:8.1f} us {rows[-1][6]:7.0f} GB/s", file=sys.stderr, flush=True)

    print("| message M | p | shard elements | reorder us | reorder GB/s | reduce us | reduce GB/s |")
    print("|---|---|---|---|---|---|---|")
    for mb, p, S, t_re, g_re, t_rs, g_rs in rows:
        print(f"| {mb} MB | {p} | {S} | {t_re * 1e6:.1f} | {g_re:.0f} | {t_rs * 1e6:.1f} | {g_rs:.0f} |")


if __name__ == "__main__":
    main()
