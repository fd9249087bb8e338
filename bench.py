#!/usr/bin/env python3
"""Benchmark of the ExDyna gradient-selection hot path on one MI355X.

A step is one exdyna_step (the streaming accumulate + compare + stage pass, then
the finishing kernel: control + compaction) over one synthetic gradient vector
that is already resident in HBM.  Prints ONE JSON line: whole-step throughput in G elements/s, the HBM
roofline of the dominant kernel measured with HIP events over the timed steps,
and the CPU oracle timed on a bounded sample of the same trajectory.
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

# HBM bytes per k_stream launch from the rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs
# summarised in profiles/k_stream_cfg4_hbm_traffic.txt (each counter scaled by what it reads for
# a plain device copy of one gradient vector: FETCH_SIZE x2.000, WRITE_SIZE x1.000, KiB), keyed
# by workload index; None for workloads that have not been measured.
MEASURED_TRAFFIC_BYTES = {4: int((542666.0 * 2.0 + 546328.1) * 1024)}


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
    n_vec = int(max(2, min(W + K, args.hbm_budget_gb // vec_gb)))
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
    recycled = n_vec < W + K

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
        cpu = {"value": round(w.n_g * cpu_steps / cpu_s / 1e9, 4), "unit": "G elem/s", "cores": 1,
               "kind": "oracle",
               "sample": f"first {cpu_steps} iterations of the same trajectory at full n_g, "
                         f"single thread, {cpu_s:.1f} s; GPU outputs bit-equal on these steps"}
        torch.cuda.empty_cache()

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
        torch.cuda.empty_cache()

        def gpu_step(ctx, g, _t=[0]):                    # noqa: F811 -- one worker's iteration
            idx_all, counts = gathered[_t[0]]
            _t[0] += 1
            if scaled:
                ctx.worker_select(g, 0, eta)
            else:
                ctx.worker_select(g, 0)
            n = idx_all.numel()
            ctx.worker_exchange(idx_all, counts, val_buf[:n].view(idx_all.shape))

    # ---- timed region ---------------------------------------------------------
    x = binding.ExDyna(cfg, dev)
    for t in range(W):
        gpu_step(x, grads[t % n_vec])
    torch.cuda.synchronize()
    prof = not args.no_profile_events
    every = max(1, args.event_every)
    if prof:
        x.set_profiling((K + every - 1) // every, every)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for t in range(W, W + K):
        gpu_step(x, grads[t % n_vec])
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    if args.worker_view:
        same = (torch.equal(x.residual.view(torch.int32), ref_residual.view(torch.int32))
                and x.get_stats().delta_next == ref_delta)
        if not same:
            print("bench.py: the worker's trajectory left the reference's", file=sys.stderr)
            return 1
    ms_events = None
    if prof:
        ms_events = np.array([x.get_kernel_ms(t) for t in range(W, W + K, every)], dtype=np.float64)
    st = x.get_stats()
    ms_per_step = elapsed / K * 1e3
    value = w.n_g * K / elapsed / 1e9
    step_bytes = alg_bytes_per_elem * w.n_g + ALG_BYTES_PER_PAIR * st.k_emitted
    kern = None
    roofline = None
    if prof:
        ms = ms_events
        kern = {"k_stream_ms": round(float(ms[:, 0].mean()), 5),
                "k_finish_ms": round(float(ms[:, 1].mean()), 5),
                "k_stream_ms_p10_p50_p90": [round(float(v), 5) for v in np.percentile(ms[:, 0], [10, 50, 90])],
                "k_finish_ms_p10_p50_p90": [round(float(v), 5) for v in np.percentile(ms[:, 1], [10, 50, 90])]}
        achieved = alg_bytes_per_elem * w.n_g / (ms[:, 0].mean() * 1e-3) / 1e9
        roofline = {"bound": "hbm", "kernel": "k_stream", "achieved": round(achieved, 1),
                    "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                    "traffic": None if (scaled or args.worker_view) else MEASURED_TRAFFIC_BYTES.get(args.config),
                    "alg_bytes_per_launch": alg_bytes_per_elem * w.n_g,
                    "launches_timed": int(ms.shape[0])}
    out = {
        "metric": "gradient elements sparsified/sec",
        "value": round(value, 3),
        "unit": "G elem/s",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": round(ms_per_step, 5),
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
                   "parallelism": "1 GPU, P partitions as index ranges"},
        "hbm_roofline_pct_per_step": round(100.0 * step_bytes / (elapsed / K) / (HBM_PEAK_GBS * 1e9), 2),
        "step_alg_gb_per_s": round(step_bytes / (elapsed / K) / 1e9, 1),
        "last_step": {"k_actual": st.k_actual, "k_emitted": st.k_emitted,
                      "k_target": w.density * w.n_g, "traffic_ratio": round(st.traffic_ratio, 4),
                      "delta_next": st.delta_next},
        "kernels": kern,
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    x.close()
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
