"""Offline choice of the refresh interval (Sec. 3.3 "Interval-based Expert Refresh", Eq. 4-7) from
measurements on this machine:

  python -m paper_2605_20179_amd.interval_search --config 1 --taus 1,2,4,8,16

For every candidate interval the block of the chosen workload is run on the GPU with a refresh every
tau steps; the run logs the experts migrated per refresh, the miss rate, the time of the refresh
copies (host link) and the time of the miss path: --miss-path host = the paper's CPU experts (host worker
threads, tide_moe_apply_misses_host), --miss-path device = the GPU reading the missed experts in place
across the host link (tide_moe_apply_misses).
From these the constants of the model are taken -- C_io = seconds per migrated expert, C_cpu = seconds
per unit of f, f(tau) = measured miss rate made monotone and interpolated, d = Eq. 4 on the logged
activation vectors and, beside it, the d that Eq. 5 needs to reproduce each measured migration count --
and tide_optimal_interval scans Eq. 7.  The model, the drift, the stability figures and the minimisation run in the
library; this file drives the runs and calibrates the constants (averages and a one-parameter least-squares fit)."""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np


def run_block(sess, tb, torch, wl, hidden, tau, miss_path):
    sess_layer = 0
    import tide_inputs as ti
    tb.tide_set_resident(sess.ctx, sess_layer, ti.initial_resident(wl))
    sess.stats(sess_layer, reset=True)
    migrated, refreshes, copy_ms, misses, miss_ms = 0, 0, 0.0, 0, 0.0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for t, h in enumerate(hidden):
        if t > 0 and t % tau == 0:
            _, plan = sess.refresh(sess_layer)
            migrated += len(plan)
            refreshes += 1
            if plan:
                copy_ms += tb.tide_refresh_copy_ms(sess.ctx, sess_layer)
        sess.step(sess_layer, h, want_topk=False)
        if miss_path == "host":
            sess.apply_misses_host(sess_layer, h)             # blocks this thread while the workers run
            torch.cuda.synchronize()
            miss_ms += tb.tide_host_miss_ms(sess.ctx)[2]
        else:
            ev0.record()
            sess.apply_misses(sess_layer, h)
            ev1.record()
            torch.cuda.synchronize()
            miss_ms += ev0.elapsed_time(ev1)
        misses += int(sess.n_miss.item())
    return dict(tau=tau, refreshes=refreshes, migrated=migrated, copy_ms=copy_ms, misses=misses, miss_ms=miss_ms)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--config", type=int, default=1)
    ap.add_argument("--layer", type=int, default=0)
    ap.add_argument("--taus", default="1,2,4,8,16")
    ap.add_argument("--miss-path", choices=("device", "host"), default="host")
    ap.add_argument("--host-threads", type=int, default=16)
    ap.add_argument("--refresh-source", choices=("raw", "packed12"), default="packed12")
    args = ap.parse_args()
    import torch
    import tide_inputs as ti
    from . import binding as tb
    from .session import TideSession

    wl = ti.CONFIGS[args.config]
    taus = sorted(int(v) for v in args.taus.split(","))
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode)
    t0 = time.time()
    sess.load_layer(0, lambda e: ti.expert_weights(wl, args.layer, e), ti.router_weights(wl, args.layer),
                    ti.router_bias(wl, args.layer), ti.initial_resident(wl), workers=16)
    if args.refresh_source == "packed12":
        sess.compress_layer(0, workers=16)
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, args.layer)]
    T, B, pairs = len(hidden), wl.C, wl.N * wl.k
    print("loaded %s layer %d in %.1f s: T=%d steps, budget %d, %d pairs per step" % (wl.name, args.layer, time.time() - t0, T, B, pairs),
          file=sys.stderr, flush=True)

    # activation vectors of the block -> stability figures and Eq. 4 on the device
    counts = []
    for h in hidden:
        sess.step(0, h, want_topk=False)
        counts.append(tb.tide_step_histogram(sess.ctx, wl.E, torch.cuda.current_stream()))
    cd = torch.from_numpy(np.array(counts, dtype=np.int32)).cuda()
    sim = torch.empty((T, T), dtype=torch.float64, device="cuda")
    uniq = torch.empty(T, dtype=torch.int32, device="cuda")
    drift = torch.empty(T, dtype=torch.float64, device="cuda")
    tb.tide_routing_stability(sess.ctx, cd, T, wl.E, B, sim, uniq, drift, torch.cuda.current_stream())
    torch.cuda.synchronize()
    sim_h, d_steps = sim.cpu().numpy(), drift.cpu().numpy()
    d_eq4 = float(d_steps[1:].mean())

    if args.miss_path == "host":
        sess.host_experts(args.host_threads)
    rows = [run_block(sess, tb, torch, wl, hidden, tau, args.miss_path) for tau in taus]
    for r in rows:
        r["miss_rate"] = r["misses"] / float(T * pairs)
        r["d_fit"] = tb.tide_fit_drift(float(r["migrated"]), B, T, r["tau"])
    moved = sum(r["migrated"] for r in rows)
    c_io = sum(r["copy_ms"] for r in rows) * 1e-3 / max(moved, 1)                 # seconds per migrated expert
    # f(tau): measured miss rates, non-decreasing in tau, linear between the measured intervals
    f_meas = np.maximum.accumulate([r["miss_rate"] for r in rows])
    f = np.interp(np.arange(1, T), taus, f_meas)
    # C_cpu * T * B * f(tau) = seconds of miss execution over the block: fit the one constant by least squares
    x = np.array([T * B * v for v in f_meas])
    y = np.array([r["miss_ms"] * 1e-3 for r in rows])
    c_cpu = float((x * y).sum() / max((x * x).sum(), 1e-300))
    d_model = float(np.mean([r["d_fit"] for r in rows]))
    tau_opt, cost = tb.tide_optimal_interval(B, T, d_model, c_io, c_cpu, f)
    io, cpu = tb.tide_interval_costs(B, T, d_model, c_io, c_cpu, f)
    for r in rows:
        r["model_io_ms"] = io[r["tau"] - 1] * 1e3
        r["model_cpu_ms"] = cpu[r["tau"] - 1] * 1e3
    for r in rows:
        r["measured_total_ms"] = r["copy_ms"] + r["miss_ms"]
    best = min(rows, key=lambda r: (r["measured_total_ms"], r["tau"]))
    out = dict(workload=wl.name, miss_path=args.miss_path, refresh_source=args.refresh_source, measured_best_tau=best["tau"],
               measured_best_ms=best["measured_total_ms"], steps=T, budget=B, adjacent_similarity=float(np.mean([sim_h[t, t + 1] for t in range(T - 1)])),
               similarity_5_apart=float(np.mean([sim_h[t, t + 5] for t in range(T - 5)])),
               distinct_experts=[int(uniq.min().item()), int(uniq.max().item())], drift_eq4=d_eq4, drift_model=d_model,
               c_io_s_per_expert=c_io, c_cpu=c_cpu, optimal_tau=tau_opt, optimal_cost_ms=cost * 1e3, sweep=rows)
    print(json.dumps(out))
    print("\n tau  refreshes  migrated  d(Eq.5 fit)  miss rate   copies ms (model)   miss pass ms (model)", file=sys.stderr)
    for r in rows:
        print("%4d %10d %9d %12.4f %10.4f %10.2f (%7.2f) %12.2f (%7.2f)" % (
            r["tau"], r["refreshes"], r["migrated"], r["d_fit"], r["miss_rate"], r["copy_ms"], r["model_io_ms"], r["miss_ms"],
            r["model_cpu_ms"]), file=sys.stderr)
    print("Eq. 4 mean drift %.4f; model drift %.4f; C_io %.3e s/expert; C_cpu %.3e; Eq. 7 optimum tau = %d (%.2f ms per block); "
          "smallest measured copies + miss time: tau = %d (%.2f ms per block)"
          % (d_eq4, d_model, c_io, c_cpu, tau_opt, cost * 1e3, best["tau"], best["measured_total_ms"]), file=sys.stderr)
    sess.close()


if __name__ == "__main__":
    main()
