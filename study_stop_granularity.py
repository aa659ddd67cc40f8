#!/usr/bin/env python3
"""Effect of the probe granularity on what the receiver accepts (Alg. "DBLP_RECV", the branch
that stops as soon as the loss-tolerance threshold is satisfied, even before the sender is done).

The graded path applies a batch completely and tests the threshold only at a probe, which keeps
the result independent of the arrival permutation.  Here the arrivals of one round are cut into
K equal sub-batches in arrival order, the threshold is tested after each, and the round stops at
the first probe that is satisfied: the remaining arrivals are never applied ("early stop").
K = 1 is the graded behaviour; large K approaches the paper's per-chunk test.  The outcome then
depends on the arrival order, which is why this lives outside the parity-graded path (a GPU test
drives the CPU checker through the same sub-batches).

Prints one JSON object.  GPU required.
"""
from __future__ import annotations

import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import numpy as np  # noqa: E402


def run_early_stop(rx, sc, bound_ppm: int, k_batches: int) -> dict:
    """Apply the round's arrivals in k sub-batches; stop at the first satisfied probe."""
    L = sc.L
    n = L.W * L.n_pkts
    b = sc.batches[0]
    order = np.arange(n, dtype=np.uint32) if b.order is None else b.order
    rx.begin_round(sc.rnd_id)
    edges = np.linspace(0, n, k_batches + 1).astype(np.int64)
    probes, applied = 0, 0
    met = False
    for i in range(k_batches):
        part = order[edges[i]:edges[i + 1]]
        rx.apply(0, n, b.mask, part, part.size)
        applied = int(edges[i + 1])
        missing, lst, count, met = rx.loss_account(bound_ppm)
        probes += 1
        if met:
            break
    out = rx.finalize()
    norm = rx.phase_signal()[0]
    c = rx.counters()
    return dict(k=k_batches, probes=probes, met=bool(met), arrivals_offered=applied, accepted=c["accepted"],
                accepted_fraction=c["accepted"] / n, norm=norm, out=out, bitmap=rx.bitmap(),
                left_for_retransmission=int(count))


def main():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--elems", type=int, default=25_600_000)
    ap.add_argument("--ks", default="1,8,64,256,1024")
    ap.add_argument("--bound-ppm", type=int, default=50_000)
    ap.add_argument("--per-layer", action="store_true",
                    help="keep the per-layer buckets (default: one accounting unit per worker, the paper's)")
    args = ap.parse_args()
    import workloads as wl
    from harness import GpuRx, build_scenario
    w = wl.workload("cfg2")
    if args.elems != w.layout.N:
        w = wl.scaled_down(w, args.elems)
    if not args.per_layer:
        import dataclasses
        L = w.layout
        w = dataclasses.replace(w, layout=wl.Layout(L.W, L.N, L.P, [0], [L.N]))
    sc = build_scenario(w)
    g = GpuRx(sc)
    g.packetize_all()
    rows = []
    for k in [int(x) for x in args.ks.split(",")]:
        got = run_early_stop(g, sc, args.bound_ppm, k)
        rows.append({kk: vv for kk, vv in got.items() if kk not in ("out", "bitmap")})
    print(json.dumps(dict(workload=w.name, N=w.layout.N, W=w.layout.W, bound_ppm=args.bound_ppm,
                          loss=w.loss, rows=rows)))


if __name__ == "__main__":
    main()
