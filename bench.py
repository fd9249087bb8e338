#!/usr/bin/env python3
"""Benchmark of the ExDyna gradient-selection hot path on one MI355X.

A step is one exdyna_step (the streaming accumulate + compare + stage pass, then
the finishing kernel: control + placement) over one synthetic gradient vector
that is already resident in HBM.  Prints ONE JSON line: whole-step throughput in G elements/s, the HBM
roofline of the dominant kernel measured with HIP events over the timed steps,
and the CPU oracle timed on a bounded sample of the same trajectory.

The headline numbers are those of the window the caller asks for (--warmup W, --steps K:
iterations W .. W+K-1 of the workload's trajectory from its first iteration on).  With the
default hyper-parameters the threshold needs about 50 iterations to catch up with the
residual build-up of workload 4, so a short warm-up times the transient, in which k' is far
above the output capacity.  Two more measurements ride along in the same JSON line, labelled
as such: `steady_state` (the same context carried on to iteration 60, then 40 more timed
steps) and `cfg5` (the 1.5 G-gradient workload, a few timed steps), so that one run shows
both windows and both configurations the target is stated for.
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

HBM_PEAK_GBS = 8000.0          # MI355X published HBM3E bandwidth
ALG_BYTES_PER_ELEM = 12.0      # read g (4) + read e (4) + write e' (4)
ALG_BYTES_PER_PAIR = 8.0       # u32 index + fp32 value per selected gradient
STEADY_FROM, STEADY_STEPS = 60, 40            # the second, settled window of the same context
CFG5_VECTORS, CFG5_WARMUP, CFG5_STEPS = 4, 5, 20   # the 1.5 G-gradient workload riding along
CFG5_BAND_LIMIT = 300                         # untimed search for the end of its threshold transient

# HBM bytes per k_stream launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised under profiles/ (each counter scaled by what it reads for a plain device copy of
# one gradient vector: FETCH_SIZE x2.000, WRITE_SIZE x1.000, KiB).  Counters cannot be read
# from inside this program, so the figure is the one of the committed summary for the same
# workload and kind of window, and `traffic_source` names it; None where nothing was measured.
MEASURED_TRAFFIC = {
    (4, "transient"): (int((543272.1 * 2.0 + 552501.6) * 1024),
                       "profiles/k_stream_cfg4_hbm_traffic.txt (rocprofv3 --pmc, --warmup 5 --steps 20 window)"),
    (4, "steady"): (int((543219.3 * 2.0 + 546323.1) * 1024),
                    "profiles/k_stream_cfg4_hbm_traffic.txt (rocprofv3 --pmc, --warmup 60 --steps 10 window)"),
}


def cpu_description():
    """Model string and logical core count of the host the oracle is timed on."""
    model = "unknown"
    try:
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.lower().startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
    except OSError:
        pass
    return model, os.cpu_count()


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=60)
    ap.add_argument("--config", type=int, default=4, help="workload 1..5 (default 4: n_g=138,357,544)")
    ap.add_argument("--cpu-steps", type=int, default=-1,
                    help="oracle steps for the CPU baseline (-1: sized for ~15 s, 0: skip)")
    ap.add_argument("--no-profile-events", action="store_true",
                    help="do not record per-kernel HIP events in the timed region")
    ap.add_argument("--event-every", type=int, default=4,
                    help="record the per-kernel HIP events on every N-th timed step (the event "
                         "markers cost a few microseconds per step they are recorded on)")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain device copy of one gradient vector before the timed "
                         "region (a known-size reference for rocprofv3 --pmc byte counters)")
    ap.add_argument("--grad-dtype", choices=("f32", "bf16", "f16"), default="f32",
                    help="f32 (default): exdyna_step on learning-rate-scaled fp32 gradients, the "
                         "headline configuration.  bf16 / f16: exdyna_step_scaled on 16-bit raw "
                         "gradients with the learning rate fused in (10 instead of 12 B/gradient)")
    ap.add_argument("--eta", type=float, default=1.0 / 1024.0,
                    help="learning rate of the --grad-dtype bf16/f16 variant")
    ap.add_argument("--worker-view", action="store_true",
                    help="time one worker's iteration instead (exdyna_worker_select + "
                         "exdyna_worker_exchange for rank 0).  All P workers are given the same "
                         "gradient, so the gathered lists are the partitions' lists of a whole-step "
                         "reference run, prepared before the clock starts; the worker's residual and "
                         "threshold must end bit-equal to the reference's")
    ap.add_argument("--block-size", type=int, default=0,
                    help="override the workload's block size b (any multiple of 32; multiples "
                         "of 256 take the faster kernel variant)")
    ap.add_argument("--density", type=float, default=0.0,
                    help="override the workload's target density d")
    ap.add_argument("--no-extras", dest="extras", action="store_false",
                    help="only the asked-for window: no steady_state and cfg5 measurements")
    ap.add_argument("--hbm-budget-gb", type=float, default=160.0,
                    help="HBM to spend on pre-generated gradient vectors")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the P partitions are index ranges on one "
              "device, no collectives); --gpus must be 1.", file=sys.stderr)
        return 2

    import numpy as np
    import torch

    from paper_2402_13781_amd import binding, synthetic

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    binding.load()   # fails loudly if the HIP library has not been built
    dev = torch.device("cuda:0")
    w = synthetic.WORKLOADS[args.config]
    if args.block_size:
        w = w.scaled(w.n_g, args.block_size)
    if args.density:
        import dataclasses
        w = dataclasses.replace(w, density=args.density, name=f"{w.name}/d={args.density:g}")
    K, W = args.steps, args.warmup
    src = synthetic.GradientSource(w, dev)

    # ---- gradients resident in HBM before the clock starts -------------------
    vec_gb = w.n_g * (4 if args.grad_dtype == "f32" else 2) / 1e9
    want_vec = W + K
    n_vec = int(max(2, min(want_vec, args.hbm_budget_gb // vec_gb)))
    scaled = args.grad_dtype != "f32"
    eta = float(np.float32(args.eta))
    if scaled:
        # raw gradients g / eta stored in 16 bits; eta * raw has the scale of the fp32 workload
        tdt = torch.bfloat16 if args.grad_dtype == "bf16" else torch.float16
        odt = 1 if args.grad_dtype == "bf16" else 2
        grads = [(src.grad(t) / eta).to(tdt) for t in range(n_vec)]
        thr = synthetic.initial_threshold(grads[0].float() * eta, w.density)
        alg_bytes_per_elem = ALG_BYTES_PER_ELEM - 2.0
    else:
        grads = [src.grad(t) for t in range(n_vec)]
        thr = synthetic.initial_threshold(grads[0], w.density)
        alg_bytes_per_elem = ALG_BYTES_PER_ELEM
    recycled = n_vec < want_vec

    def gpu_step(ctx, g):
        if scaled:
            ctx.step_scaled(g, eta)
        else:
            ctx.step(g)
    cfg = binding.default_config(n_g=w.n_g, block_size=w.block_size, n_parts=w.n_parts,
                                 density=w.density, threshold0=thr)

    # ---- CPU oracle on a bounded sample of the same trajectory, with parity --
    cpu = None
    cpu_steps = args.cpu_steps
    if cpu_steps < 0:
        cpu_steps = int(max(2, min(n_vec, 60, 15.0 / (w.n_g / 0.6e9))))   # oracle ~0.6 G elem/s: about 15 s
    if cpu_steps > 0:
        from oracle import oracle
        o = oracle.Oracle(w.n_g, w.block_size, w.n_parts, w.density, thr)
        xv = binding.ExDyna(cfg, dev)
        cpu_s = 0.0
        for t in range(cpu_steps):
            if scaled:
                h = grads[t % n_vec].view(torch.int16).cpu().numpy().view(np.uint16)
            else:
                h = grads[t % n_vec].cpu().numpy()
            t0 = time.perf_counter()
            if scaled:
                o.step_scaled(h, odt, eta)
            else:
                o.step(h)
            cpu_s += time.perf_counter() - t0
            gpu_step(xv, grads[t % n_vec])
            idx, val, off, ka, ke = xv.get_selected()
            ok = (ka == o.k_actual and ke == o.k_emitted
                  and np.array_equal(idx.cpu().numpy().view(np.uint32), o.out_idx())
                  and np.array_equal(val.cpu().numpy().view(np.uint32), o.out_val().view(np.uint32))
                  and np.float32(xv.get_stats().delta_next) == o.threshold)
            if not ok:
                print(f"bench.py: GPU/oracle mismatch at step {t}", file=sys.stderr)
                return 1
        res_ok = np.array_equal(xv.residual.cpu().numpy().view(np.uint32),
                                o.residual(copy=False).view(np.uint32))
        if not res_ok:
            print("bench.py: residual mismatch against the oracle", file=sys.stderr)
            return 1
        xv.close()
        del xv, o, h
        cpu_model, host_cores = cpu_description()
        cpu = {"value": round(w.n_g * cpu_steps / cpu_s / 1e9, 4), "unit": "G elem/s", "cores": 1,
               "kind": "oracle", "cpu_model": cpu_model, "host_cores_total": host_cores,
               "sample": f"first {cpu_steps} iterations of the same trajectory at full n_g, "
                         f"single thread, {cpu_s:.1f} s; GPU outputs bit-equal on these steps"}
        # (no empty_cache() here: the timed context takes over this one's blocks from torch's
        # allocator; memory handed back to the driver right before the clock starts costs the
        # streaming kernel about 1.5 % while the driver is still busy with it)

    if args.calibration_copy:
        ref = torch.empty_like(grads[0])
        ref.copy_(grads[0])        # reads 4*n_g bytes, writes 4*n_g bytes
        torch.cuda.synchronize()
        del ref

    # ---- worker view: what the AllGather would deliver, for every iteration ----
    gathered = None
    if args.worker_view:
        P = w.n_parts
        ref_cfg = binding.default_config(n_g=w.n_g, block_size=w.block_size, n_parts=P,
                                         density=w.density, threshold0=thr, max_selected=w.n_g)
        ref = binding.ExDyna(ref_cfg, dev)
        probe = binding.ExDyna(cfg, dev)
        worker_cap = probe.capacity
        probe.close()
        del probe
        gathered = []
        max_elems = 0
        for t in range(W + K):
            gpu_step(ref, grads[t % n_vec])
            idx, _, off, ka, ke = ref.get_selected()
            assert ka == ke
            offs = off.cpu().numpy()
            lens = np.diff(offs)
            if lens.max() > worker_cap:
                print("bench.py: a worker's list exceeds the capacity; the reference run cannot "
                      "stand in for the gather", file=sys.stderr)
                return 1
            stride = int(lens.max())
            idx_all = torch.zeros((P, stride), dtype=torch.int32, device=dev)
            counts = np.empty(P, np.int64)
            for r in range(P):
                p = (t % P + r) % P                      # Alg. 3 (cyclic allocation)
                idx_all[r, :lens[p]] = idx[offs[p]:offs[p + 1]]
                counts[r] = lens[p]
            gathered.append((idx_all, torch.from_numpy(counts).to(dev)))
            max_elems = max(max_elems, P * stride)
        val_buf = torch.empty(max(max_elems, 1), dtype=torch.float32, device=dev)
        ref_residual = ref.residual.clone()
        ref_delta = ref.get_stats().delta_next
        ref.close()
        del ref

        def gpu_step(ctx, g, _t=[0]):                    # noqa: F811 -- one worker's iteration
            idx_all, counts = gathered[_t[0]]
            _t[0] += 1
            if scaled:
                ctx.worker_select(g, 0, eta)
            else:
                ctx.worker_select(g, 0)
            n = idx_all.numel()
            ctx.worker_exchange(idx_all, counts, val_buf[:n].view(idx_all.shape))

    # ---- timed regions ---------------------------------------------------------
    prof = not args.no_profile_events
    every = max(1, args.event_every)

    def timed_window(ctx, step_fn, grad_at, t_first, n_steps, n_g, bytes_per_elem):
        """Times iterations t_first .. t_first + n_steps - 1 of `ctx` (already at t_first)."""
        torch.cuda.synchronize()
        if prof:
            ctx.set_profiling((n_steps + every - 1) // every, every)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(t_first, t_first + n_steps):
            step_fn(ctx, grad_at(t))
        torch.cuda.synchronize()
        elapsed = time.perf_counter() - t0
        st = ctx.get_stats()
        step_bytes = bytes_per_elem * n_g + ALG_BYTES_PER_PAIR * st.k_emitted
        res = {"first_iteration": t_first, "steps": n_steps,
               "ms_per_step": round(elapsed / n_steps * 1e3, 5),
               "value": round(n_g * n_steps / elapsed / 1e9, 3),
               "hbm_roofline_pct_per_step": round(100.0 * step_bytes / (elapsed / n_steps) / (HBM_PEAK_GBS * 1e9), 2),
               "step_alg_gb_per_s": round(step_bytes / (elapsed / n_steps) / 1e9, 1),
               "last_step": {"k_actual": st.k_actual, "k_emitted": st.k_emitted,
                             "k_target": ctx.cfg.density * n_g, "traffic_ratio": round(st.traffic_ratio, 4),
                             "delta_next": st.delta_next},
               "kernels": None, "roofline": None}
        if prof:
            ms = np.array([ctx.get_kernel_ms(t) for t in range(t_first, t_first + n_steps, every)],
                          dtype=np.float64)
            ctx.set_profiling(0)
            res["kernels"] = {
                "k_stream_ms": round(float(ms[:, 0].mean()), 5),
                "k_finish_ms": round(float(ms[:, 1].mean()), 5),
                "k_stream_ms_p10_p50_p90": [round(float(v), 5) for v in np.percentile(ms[:, 0], [10, 50, 90])],
                "k_finish_ms_p10_p50_p90": [round(float(v), 5) for v in np.percentile(ms[:, 1], [10, 50, 90])]}
            achieved = bytes_per_elem * n_g / (ms[:, 0].mean() * 1e-3) / 1e9
            res["roofline"] = {"bound": "hbm", "kernel": "k_stream", "achieved": round(achieved, 1),
                               "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                               "traffic": None, "traffic_source": None,
                               "alg_bytes_per_launch": bytes_per_elem * n_g,
                               "launches_timed": int(ms.shape[0])}
        return res, elapsed

    def in_band(k_actual, c):
        """Alg. 5 takes its fine step: 1/beta < k'/k <= beta."""
        return 1.0 / c.beta < k_actual / (c.density * c.n_g) <= c.beta

    def caught_up(k_actual, c):
        """The threshold has caught up: Alg. 5 no longer takes its coarse step up (k'/k <= beta)."""
        return k_actual / (c.density * c.n_g) <= c.beta

    def add_traffic(res, index, settled):
        """Counter-measured HBM bytes of one k_stream launch, from the committed summary for this
        workload and kind of window (transient: k' still far above the capacity)."""
        if res["roofline"] is None or scaled or args.worker_view or args.block_size or args.density:
            return
        hit = MEASURED_TRAFFIC.get((index, "steady" if settled else "transient"))
        if hit:
            res["roofline"]["traffic"], res["roofline"]["traffic_source"] = hit

    x = binding.ExDyna(cfg, dev)
    for t in range(W):
        gpu_step(x, grads[t % n_vec])
    head, elapsed = timed_window(x, gpu_step, lambda t: grads[t % n_vec], W, K, w.n_g, alg_bytes_per_elem)
    settled = head["last_step"]["k_actual"] <= x.capacity
    add_traffic(head, args.config, settled)

    if args.worker_view:
        same = (torch.equal(x.residual.view(torch.int32), ref_residual.view(torch.int32))
                and x.get_stats().delta_next == ref_delta)
        if not same:
            print("bench.py: the worker's trajectory left the reference's", file=sys.stderr)
            return 1

    # ---- the same context carried on past the threshold transient -------------
    steady = None
    extras = args.extras and not args.worker_view
    if extras and W + K < STEADY_FROM:
        def fresh(t, out):
            g = src.grad(t, out=out if not scaled else None)
            return (g / eta).to(tdt) if scaled else g
        # the vectors of the first window are done with: they are overwritten with the gradients
        # of the iterations in between, and a few more buffers make room for the second window
        band_at = caught_at = None
        for t in range(W + K, STEADY_FROM):
            grads[t % n_vec] = fresh(t, grads[t % n_vec])
            gpu_step(x, grads[t % n_vec])
            ka = x.get_stats().k_actual
            if caught_at is None and caught_up(ka, cfg):
                caught_at = t
            if band_at is None and in_band(ka, cfg):
                band_at = t
        n_vec2 = int(max(2, min(STEADY_STEPS, args.hbm_budget_gb // vec_gb)))
        while len(grads) < n_vec2:
            grads.append(torch.empty_like(grads[0]))
        for t in range(STEADY_FROM, STEADY_FROM + n_vec2):
            grads[t % n_vec2] = fresh(t, grads[t % n_vec2])
        steady, _ = timed_window(x, gpu_step, lambda t: grads[t % n_vec2], STEADY_FROM, STEADY_STEPS, w.n_g,
                                 alg_bytes_per_elem)
        add_traffic(steady, args.config, steady["last_step"]["k_actual"] <= x.capacity)
        steady["first_iteration_k_within_beta_k"] = caught_at      # the end of the threshold transient
        steady["first_iteration_in_band"] = band_at                # (k' may swing across the band without landing in it)
        steady["band_searched"] = [W + K, STEADY_FROM - 1]
        steady["note"] = (f"same context and trajectory carried on untimed to iteration {STEADY_FROM}, "
                          f"then {STEADY_STEPS} timed steps; gradient vectors "
                          f"{'recycled' if n_vec2 < STEADY_STEPS or recycled else 'fresh'}")
    x.close()
    del x, grads
    torch.cuda.empty_cache()

    # ---- the 1.5 G-gradient workload, a few steps ------------------------------
    cfg5 = None
    if extras and args.config == 4 and not scaled and not args.block_size and not args.density:
        w5 = synthetic.WORKLOADS[5]
        src5 = synthetic.GradientSource(w5, dev)
        g5 = [src5.grad(t) for t in range(CFG5_VECTORS)]
        thr5 = synthetic.initial_threshold(g5[0], w5.density)
        c5 = binding.default_config(n_g=w5.n_g, block_size=w5.block_size, n_parts=w5.n_parts,
                                    density=w5.density, threshold0=thr5)
        x5 = binding.ExDyna(c5, dev)
        for t in range(CFG5_WARMUP):
            x5.step(g5[t % CFG5_VECTORS])
        cfg5, _ = timed_window(x5, lambda c, g: c.step(g), lambda t: g5[t % CFG5_VECTORS], CFG5_WARMUP,
                               CFG5_STEPS, w5.n_g, ALG_BYTES_PER_ELEM)
        cfg5["config"] = {"workload": w5.name, "n_g": w5.n_g, "block_size": w5.block_size,
                          "n_parts": w5.n_parts, "density": w5.density, "threshold0": thr5,
                          "gradient_vectors_in_hbm": CFG5_VECTORS, "recycled": True}
        cfg5["note"] = (f"{CFG5_WARMUP} untimed iterations, then {CFG5_STEPS} timed; with gamma = 0.01 this "
                        "workload's threshold transient outlasts the window (first_iteration_k_within_beta_k, found by "
                        "carrying the same context on untimed over the recycled vectors), so k' is still "
                        "far above the capacity here; parity at this size is covered by the GPU tests")
        band5 = caught5 = None
        for t in range(CFG5_WARMUP + CFG5_STEPS, CFG5_BAND_LIMIT):      # untimed: how long the transient lasts
            x5.step(g5[t % CFG5_VECTORS])
            ka5 = x5.get_stats().k_actual
            if caught5 is None and caught_up(ka5, c5):
                caught5 = t
            if in_band(ka5, c5):
                band5 = t
                break
        cfg5["first_iteration_k_within_beta_k"] = caught5
        cfg5["first_iteration_in_band"] = band5
        cfg5["band_searched"] = [CFG5_WARMUP + CFG5_STEPS, CFG5_BAND_LIMIT - 1]
        x5.close()
        del x5, g5
        torch.cuda.empty_cache()

    out = {
        "metric": "gradient elements sparsified/sec",
        "value": head["value"],
        "unit": "G elem/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": head["ms_per_step"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "n_g": w.n_g, "block_size": w.block_size,
                   "n_parts": w.n_parts, "density": w.density, "threshold0": thr,
                   "gradient_vectors_in_hbm": n_vec, "recycled": recycled,
                   "cmp": ">=", "grad_dtype": args.grad_dtype, "eta_fused": eta if scaled else None,
                   "view": "worker rank 0: select + exchange" if args.worker_view else "whole step",
                   "window": ("threshold transient: k' above the output capacity" if not settled
                              else "threshold settled: k' within the output capacity"),
                   "parallelism": "1 GPU, P partitions as index ranges"},
        "hbm_roofline_pct_per_step": head["hbm_roofline_pct_per_step"],
        "step_alg_gb_per_s": head["step_alg_gb_per_s"],
        "last_step": head["last_step"],
        "kernels": head["kernels"],
        "roofline": head["roofline"],
        "cpu_baseline": cpu,
        "steady_state": steady,
        "cfg5": cfg5,
    }
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
