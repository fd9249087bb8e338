#!/usr/bin/env python3
"""Per-iteration trace of the sparsifier's own metrics on a synthetic workload.

Runs the HIP library (never a CPU substitute) over a workload of
paper_2402_13781_amd.synthetic and prints one CSV line per iteration:
the actual density k'/n_g against the target d (Sec. 5.2's density plots), the
density error of Eq. 6, the traffic ratio f(t) of Eq. 5, the all-gather padding
C_t of Eq. 4, the threshold next to the error norm of Eq. 1 (the pair Sec. 5.3
compares), and the number of boundary moves Alg. 3 made.  A last line on stderr says at
which iteration k'/k first entered Alg. 5's band (1/beta, beta] and when it was last outside.  Two
switches turn the paper's ablations on:

  --static-partitions   blk_move = 0: coarse-grained, never rebalanced (Sec. 4.1)
  --fixed-threshold     gamma = 0: the hard-threshold sparsifier of Sec. 3

    python -m paper_2402_13781_amd.trace --config 5 --n-g 20000000 --steps 200
"""
from __future__ import annotations

import argparse
import sys


def run_trace(workload, steps, device="cuda:0", static_partitions=False, fixed_threshold=False,
              gamma=None, blk_move=None, out=None):
    """Returns a list of dicts, one per iteration; also writes CSV lines to `out` if given."""
    from . import binding, synthetic

    src = synthetic.GradientSource(workload, device)
    g = src.grad(0)
    thr = synthetic.initial_threshold(g, workload.density)
    kw = {}
    if static_partitions:
        kw["blk_move"] = 0
    elif blk_move is not None:
        kw["blk_move"] = blk_move
    if fixed_threshold:
        kw["gamma"] = 0.0
    elif gamma is not None:
        kw["gamma"] = gamma
    cfg = binding.default_config(n_g=workload.n_g, block_size=workload.block_size,
                                 n_parts=workload.n_parts, density=workload.density,
                                 threshold0=thr, want_err_norm=1, **kw)
    x = binding.ExDyna(cfg, device)
    rows = []
    cols = ("t", "k_actual", "density", "density_error", "traffic_ratio", "padding_overhead",
            "delta_used", "err_norm", "moves", "overflow")
    if out is not None:
        print(",".join(cols), file=out)
    for t in range(steps):
        if t:
            g = src.grad(t, out=g)
        x.step(g)
        s = x.get_stats()
        row = dict(t=t, k_actual=s.k_actual, density=s.k_actual / workload.n_g,
                   density_error=s.density_error, traffic_ratio=s.traffic_ratio,
                   padding_overhead=s.padding_overhead,
                   delta_used=s.delta_used, err_norm=s.err_norm, moves=s.moves, overflow=s.overflow)
        rows.append(row)
        if out is not None:
            print(",".join(f"{row[c]:.6g}" if isinstance(row[c], float) else str(row[c]) for c in cols),
                  file=out, flush=True)
    x.close()
    return rows


def band_entry(rows, k, beta):
    """Alg. 5 takes its fine step while 1/beta < k'/k <= beta.  Returns (first iteration inside
    that band, last iteration outside it), either None if there is none: how long the closed loop
    of Sec. 4.4 needs from the caller's first threshold to the target density, and whether it
    stays there."""
    inside = [1.0 / beta < r["k_actual"] / k <= beta for r in rows]
    first = next((r["t"] for r, ok in zip(rows, inside) if ok), None)
    last_out = next((r["t"] for r, ok in zip(reversed(rows), reversed(inside)) if not ok), None)
    return first, last_out


def caught_up(rows, k, beta):
    """First iteration after the first from which k'/k <= beta: the threshold has caught up with
    the residual build-up and Alg. 5 stops taking its coarse step up (k' may then swing across
    the band for a while without landing inside it).  None if it never does."""
    grown = False
    for r in rows:
        ratio = r["k_actual"] / k
        grown = grown or ratio > beta
        if grown and ratio <= beta:
            return r["t"]
    return None


def main(argv=None) -> int:
    from . import synthetic

    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--config", type=int, default=5, choices=sorted(synthetic.WORKLOADS))
    ap.add_argument("--n-g", type=int, default=0, help="scale the workload down to this many gradients")
    ap.add_argument("--block-size", type=int, default=0)
    ap.add_argument("--n-parts", type=int, default=0)
    ap.add_argument("--steps", type=int, default=0, help="default: the workload's own iteration count")
    ap.add_argument("--static-partitions", action="store_true")
    ap.add_argument("--fixed-threshold", action="store_true")
    ap.add_argument("--gamma", type=float, default=None)
    ap.add_argument("--blk-move", type=int, default=None)
    a = ap.parse_args(argv)
    w = synthetic.WORKLOADS[a.config]
    if a.n_g or a.block_size or a.n_parts:
        w = w.scaled(a.n_g or w.n_g, a.block_size or None, a.n_parts or None)
    rows = run_trace(w, a.steps or w.iters, static_partitions=a.static_partitions,
                     fixed_threshold=a.fixed_threshold, gamma=a.gamma, blk_move=a.blk_move, out=sys.stdout)
    from . import binding
    beta = binding.default_config().beta
    first, last_out = band_entry(rows, w.density * w.n_g, beta)
    print(f"# k'/k first within (1/{beta:g}, {beta:g}] at iteration {first}; last iteration outside: "
          f"{last_out} of {len(rows)}; back to k'/k <= {beta:g} after the build-up at iteration "
          f"{caught_up(rows, w.density * w.n_g, beta)}", file=sys.stderr)
    return 0


if __name__ == "__main__":
    sys.exit(main())
