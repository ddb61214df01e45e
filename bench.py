#!/usr/bin/env python3
"""Benchmark of the TIDE MoE-step hot path on one MI355X.

A "step" is one denoise step of one MoE layer: (every tau-th step) the refresh --
top-B selection, plan, pinned-host -> HBM expert copies (by default from the lossless 12-bit
form of the blobs; --refresh-source raw copies them as they are) -- followed by tide_moe_step
(router, top-k, hit counts, hit/miss split + miss list, grouped SwiGLU expert GEMMs
over the resident experts, weighted combine).  The workload is the LLaDA2.0-mini-shaped
single layer (block of 32 tokens, batch 1, 256 experts top-8 + shared, capacity 64,
refresh interval 4) on seeded synthetic weights and drifting hidden states; the 32
hidden-state tensors of the block are resident in HBM before timing starts and the
block is replayed cyclically.

Prints ONE JSON line.  `value` is tokens/s over the whole timed region (refreshes
included).  `roofline` is for the dominant kernel (grouped gate/up GEMM + SwiGLU):
algorithmic bytes per launch / its mean duration between the start and stop HIP events
that each launch stamps on its own stream inside the timed region.  `cpu_baseline` is the CPU oracle timed on a
bounded sample of the same workload on this host."""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MFMA_BF16_PEAK_TFLOPS = 2500.0
HBM_PEAK_GBS = 8000.0


def cpu_baseline(wl, ti, sample_steps=None):
    """The oracle as it stands, on `sample_steps` consecutive denoise steps (all tokens,
    cold-start placement) of the benchmark workload.  The default sample is 512 steps of the
    headline layer and as many steps of a larger one as cost about the same CPU time."""
    import numpy as np
    if sample_steps is None:
        sample_steps = max(2, min(512, int(512 * 32 * 2048 * 512 / (wl.N * wl.d * wl.I))))
    from oracle import tide_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = 1
    store = orc.ExpertStore(lambda e: ti.expert_weights(wl, 0, e), max_cached=wl.E + 1)
    shared = tuple(orc.bf16_to_f64(m) for m in ti.expert_weights(wl, 0, wl.E)) if wl.n_shared else None
    hidden = list(ti.hidden_stream(wl, 0, sample_steps))
    wr, b = ti.router_weights(wl, 0), ti.router_bias(wl, 0)
    t0 = time.perf_counter()
    orc.run_block(hidden, wr, b, wl.gating, wl.bias_mode, wl.k, wl.E, wl.C, wl.K, ti.initial_resident(wl),
                  weights=store, shared=shared)
    dt = time.perf_counter() - t0
    return {"value": wl.N * sample_steps / dt, "unit": "tokens/s", "cores": int(threads), "kind": "oracle",
            "sample": "%d denoise steps x %d tokens of the same layer, routing + resident and full outputs in fp64, "
                      "%.1f s (includes bf16->fp64 weight conversion on first use)" % (sample_steps, wl.N, dt)}


# --resident: the form the cache slots keep the blobs in (set per workload, read by every session made here).
# "auto": the 12-bit form where a step is bound by the weight bytes it streams (up to 768 tokens at d = 4096, up to 1024 at d = 2048: a
# slot sees a handful to a hundred rows), bf16 blobs where the large-item kernels do most of the work (the decode costs
# them more than the bytes it saves, and a 12-bit large item is capped at 192 rows).
RESIDENT_P12 = False


def resident_p12_for(args, wl):
    policy = getattr(args, "resident_policy", args.resident)
    # auto: the 12-bit form where it measured faster -- steps of up to 768 tokens, up to 1024 for layers whose steps
    # of that size still run as small work items only (weight rows shorter than 4096)
    return policy == "p12" or (policy == "auto" and wl.N <= (768 if wl.d >= 4096 else 1024))


def choose_resident(args, wl):
    global RESIDENT_P12
    RESIDENT_P12 = resident_p12_for(args, wl)
    return "p12" if RESIDENT_P12 else "bf16"


def bf16_reference(wl, args, ti, tb, TideSession, torch, packed, comp, hidden_bits):
    """The timed loop of the headline once more over bf16 slots, without event brackets: refresh copies from the raw blobs
    (Alg. 1's copies as they are) and from the 12-bit form.  Reference figures beside a run over 12-bit slots."""
    ref = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode)
    ref.load_layer(0, None, ti.router_weights(wl, 0), ti.router_bias(wl, 0), ti.initial_resident(wl), packed=packed)
    hidden = [ref.to_device_bf16(h) for h in hidden_bits]
    out = {}
    for source in ("raw", "packed12"):
        if source == "packed12":
            tb.tide_register_compressed(ref.ctx, 0, comp, tb.tide_compressed_blob_bytes(ref.cfg))
        tb.tide_set_resident(ref.ctx, 0, ti.initial_resident(wl))
        ref.stats(0, reset=True)
        for phase, n in (("warm", args.warmup), ("timed", args.steps)):
            torch.cuda.synchronize()
            r0 = time.perf_counter()
            for i in range(n):
                t = (i if phase == "warm" else args.warmup + i) % wl.S
                if t > 0 and t % wl.K == 0:
                    ref.refresh(0)
                ref.step(0, hidden[t], want_topk=False)
            torch.cuda.synchronize()
            rdt = time.perf_counter() - r0
        out[source] = {"tokens_per_s": wl.N * args.steps / rdt, "us_per_step": rdt / args.steps * 1e6}
    ref.close()
    return out


def run_stack(args, wl, ti, tb, TideSession, torch):
    """A stack of L independent MoE layers per denoise step (the stack workloads' metric: N / sum over the
    layers).  Detail measurement, not the headline: prints its own JSON line."""
    L = args.stack
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, n_layers=L, resident_p12=RESIDENT_P12)
    packed = sess.pack_layer(lambda e: ti.expert_weights(wl, 0, e), workers=16)
    hidden = []
    for l in range(L):                                 # the layers share layer 0's blobs, so one compressed copy serves all
        sess.load_layer(l, None, ti.router_weights(wl, l), ti.router_bias(wl, l), ti.initial_resident(wl), packed=packed,
                        workers=16, comp=sess.comp_blobs.get(0))
        hidden.append([sess.to_device_bf16(h) for h in ti.hidden_stream(wl, l)])
    if args.refresh_source == "packed12" and not RESIDENT_P12:
        sess.compress_layer(0, workers=16)
        for l in range(1, L):
            tb.tide_register_compressed(sess.ctx, l, sess.comp_blobs[0], tb.tide_compressed_blob_bytes(sess.cfg))
    torch.cuda.synchronize()
    state = {"t": 0, "copies": 0}

    def one_step():
        t = state["t"] % wl.S
        due = t > 0 and t % wl.K == 0
        if due and args.refresh_order == "all-first":
            for l in range(L):
                state["copies"] += len(sess.refresh(l)[1])
        if args.refresh_order == "per-layer":
            for l in range(L):
                if due:
                    state["copies"] += len(sess.refresh(l)[1])
                sess.step(l, hidden[l][t], want_topk=False)
        else:
            sess.stack_step([hidden[l][t] for l in range(L)])
        state["t"] += 1

    for _ in range(args.warmup):
        one_step()
    torch.cuda.synchronize()
    state["copies"] = 0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for i in range(args.steps):
        sess.stack_step([hidden[l][i % wl.S] for l in range(L)])
    torch.cuda.synchronize()
    frozen = (time.perf_counter() - s0) / args.steps
    print(json.dumps({
        "metric": "MoE-layer tokens/s per denoise step", "value": wl.N * args.steps / dt, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "d": wl.d, "experts": wl.E, "top_k": wl.k, "d_ff": wl.I, "shared_experts": wl.n_shared,
                   "tokens_per_step": wl.N, "capacity": wl.C, "refresh_interval": wl.K, "steps_per_block": wl.S, "layers": L,
                   "refresh_order": args.refresh_order, "refresh_source": args.refresh_source, "resident_format": args.resident, "note": "layers share layer 0's expert values; routers, streams, caches differ"},
        "detail": {"experts_copied": state["copies"], "blob_MiB": sess.blob_bytes / 2 ** 20,
                   "frozen_placement_us_per_step": frozen * 1e6, "frozen_placement_us_per_layer": frozen * 1e6 / L,
                   "us_per_layer": 1e6 * dt / args.steps / L}}))
    sess.close()


def layer_rooflines(wl, blob, active, rows, gate_up_s, down_s, step_s):
    """Fractions of the HBM and bf16-MFMA peaks for the two grouped GEMM passes and for the whole step, from the
    step's own counters: `active` cache slots with at least one token (shared expert included), `rows` (token,
    expert) rows evaluated.  Algorithmic bytes: every active slot's weights once, the hidden states once, the
    activations / outputs a pass writes once.  The step figure is given twice: the algorithmic bytes alone, and
    with the intermediates the implementation materialises (activations and per-row outputs, written once and
    read once each)."""
    def pass_(bytes_, flop, secs):
        if not secs:
            return None
        return {"us": secs * 1e6, "algorithmic_bytes": bytes_, "flop": flop,
                "hbm": {"achieved": bytes_ / secs / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": bytes_ / secs / 1e9 / HBM_PEAK_GBS},
                "mfma": {"achieved": flop / secs / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                         "frac": flop / secs / 1e12 / MFMA_BF16_PEAK_TFLOPS}}
    step_alg = active * blob + wl.E * wl.d * 4 + wl.N * wl.d * 2 + wl.N * wl.d * 4
    step_mat = step_alg + 2 * rows * wl.I * 2 + 2 * rows * wl.d * 4
    step_flop = rows * 6.0 * wl.d * wl.I + 2.0 * wl.N * wl.d * wl.E
    return {"gate_up": pass_(active * (2 * blob / 3) + wl.N * wl.d * 2 + rows * wl.I * 2, rows * 4.0 * wl.d * wl.I, gate_up_s),
            "down": pass_(active * (blob / 3) + rows * wl.I * 2 + rows * wl.d * 4, rows * 2.0 * wl.d * wl.I, down_s),
            "step": {"us": step_s * 1e6, "algorithmic_bytes": step_alg, "flop": step_flop,
                     "hbm_frac": step_alg / step_s / 1e9 / HBM_PEAK_GBS,
                     "bytes_with_activation_and_row_output_round_trips": step_mat,
                     "hbm_frac_with_round_trips": step_mat / step_s / 1e9 / HBM_PEAK_GBS,
                     "mfma_frac": step_flop / step_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}}


def pair_seconds(prof, small, big):
    """Mean duration of one pass of a step: its small-item and large-item launches start together on two streams,
    so the pass lasts as long as the longer of the two."""
    ms_s, n_s = prof.get(small, (0.0, 0))
    ms_b, n_b = prof.get(big, (0.0, 0))
    cand = [ms / n for ms, n in ((ms_s, n_s), (ms_b, n_b)) if n]
    return 1e-3 * max(cand) if cand else None


def measure_layer(wl, ti, tb, TideSession, torch, packed, steps, warmup, refresh_source, comp=None):
    """One layer of workload `wl` (any of the five configurations): tokens/s with the refresh every K steps (copies
    from `refresh_source`, and once more from the raw blobs), tokens/s with the placement frozen, per-kernel
    durations from event-stamped launches of a frozen pass, and the roofline fractions they give."""
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=RESIDENT_P12)
    sess.load_layer(0, None, ti.router_weights(wl, 0), ti.router_bias(wl, 0), ti.initial_resident(wl), packed=packed,
                    workers=16, comp=comp if RESIDENT_P12 else None)
    use_p12 = refresh_source == "packed12" and wl.C < wl.E and not RESIDENT_P12
    if RESIDENT_P12:
        comp = sess.comp_blobs[0]
    if use_p12:
        if comp is None:
            sess.compress_layer(0, workers=16)
            comp = sess.comp_blobs[0]
        else:
            tb.tide_register_compressed(sess.ctx, 0, comp, tb.tide_compressed_blob_bytes(sess.cfg))
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, 0)]
    torch.cuda.synchronize()

    def block_loop(n_steps, warm):
        tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
        sess.stats(0, reset=True)
        copies = 0
        for i in range(warm + n_steps):
            if i == warm:
                torch.cuda.synchronize()
                tb.tide_counters(sess.ctx, reset=True)
                copies = 0
                t0 = time.perf_counter()
            t = i % wl.S
            if t > 0 and t % wl.K == 0:
                copies += len(sess.refresh(0)[1])
            sess.step(0, hidden[t], want_topk=False)
        torch.cuda.synchronize()
        return time.perf_counter() - t0, copies, tb.tide_counters(sess.ctx)

    dt, copies, cnt = block_loop(steps, warmup)
    raw = None
    if use_p12:
        tb.tide_register_compressed(sess.ctx, 0, None, 0)
        raw_dt, _, _ = block_loop(steps, warmup)
        raw = wl.N * steps / raw_dt
    # placement as the loop left it, no refresh: every kernel stamped, then the same steps unstamped
    tb.tide_profile(sess.ctx, 1)
    tb.tide_counters(sess.ctx, reset=True)
    for i in range(steps):
        sess.step(0, hidden[i % wl.S], want_topk=False)
    prof = tb.tide_profile_read(sess.ctx)
    fcnt = tb.tide_counters(sess.ctx)
    tb.tide_profile(sess.ctx, False)
    torch.cuda.synchronize()
    f0 = time.perf_counter()
    for i in range(steps):
        sess.step(0, hidden[i % wl.S], want_topk=False)
    torch.cuda.synchronize()
    frozen_s = (time.perf_counter() - f0) / steps
    active, rows = fcnt["active_slots"] / fcnt["steps"], fcnt["rows"] / fcnt["steps"]
    res = {"workload": wl.name, "tokens_per_step": wl.N, "d": wl.d, "d_ff": wl.I, "capacity": wl.C, "layers_in_workload": wl.L,
           "layers_measured": 1, "steps": steps, "warmup": warmup,
           "tokens_per_s": wl.N * steps / dt, "ms_per_step": 1e3 * dt / steps, "refresh_source": refresh_source if use_p12 else "raw",
           "tokens_per_s_raw_refresh_copies": raw if raw is not None else (None if RESIDENT_P12 else wl.N * steps / dt),
           "experts_copied": copies, "hit_rate": 1.0 - cnt["misses"] / (wl.N * wl.k * cnt["steps"]),
           "frozen_placement": {"us_per_step": frozen_s * 1e6, "tokens_per_s": wl.N / frozen_s, "hit_rate": 1.0 - fcnt["misses"] / (wl.N * wl.k * fcnt["steps"]),
                                "active_slots_per_step": active, "rows_per_step": rows},
           "kernels_us": {name: 1e3 * ms / n for name, (ms, n) in prof.items() if n},
           "roofline": layer_rooflines(wl, sess.blob_bytes, active, rows, pair_seconds(prof, "gate_up_swiglu", "gate_up_swiglu_big"),
                                       pair_seconds(prof, "down", "down_big"), frozen_s)}
    rate, nbytes = tb.tide_hbm_stream_probe(sess.ctx, 0, 8)
    res["hbm_stream_probe"] = {"GB/s": rate, "bytes_per_launch": nbytes, "frac_of_peak": rate / HBM_PEAK_GBS,
                               "what": "a kernel that only reads this layer's cache slots once, in the GEMMs' weight-stream shape"}
    sess.close()
    return res, comp


def measure_stack(wl, L, ti, tb, TideSession, torch, packed, steps, comp=None, refresh=True):
    """The workload as the stack it is: L independent layers per denoise step in one context (own router, hidden
    stream, cache, counter, refresh per layer; the layers share layer 0's expert values).  tokens/s = N / sum of
    the layers' times, with the placement frozen and (refresh=True) with every layer refreshed every K steps, all
    layers first so that later layers' copies run under earlier layers' compute."""
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, n_layers=L, resident_p12=RESIDENT_P12)
    import concurrent.futures
    n_hidden = min(wl.S, 2 * wl.K) if (refresh and wl.C < wl.E) else 2
    with concurrent.futures.ThreadPoolExecutor(max_workers=16) as ex:
        streams = list(ex.map(lambda l: list(ti.hidden_stream(wl, l, n_hidden)), range(L)))
    hidden = []
    for l in range(L):
        sess.load_layer(l, None, ti.router_weights(wl, l), ti.router_bias(wl, l), ti.initial_resident(wl), packed=packed,
                        workers=16, comp=(comp if comp is not None else sess.comp_blobs.get(0)) if RESIDENT_P12 else None)
        if comp is not None and wl.C < wl.E and not RESIDENT_P12:
            tb.tide_register_compressed(sess.ctx, l, comp, tb.tide_compressed_blob_bytes(sess.cfg))
        hidden.append([sess.to_device_bf16(h) for h in streams[l]])
    del streams
    torch.cuda.synchronize()
    free_b, total_b = torch.cuda.mem_get_info()
    out = {"layers": L, "capacity": wl.C, "tokens_per_step": wl.N, "cache_slots_GiB": L * (wl.C + 1) * sess.blob_bytes / 2 ** 30,
           "device_memory_in_use_GiB": (total_b - free_b) / 2 ** 30,
           "note": "layers share layer 0's expert values in pinned host memory; routers, hidden streams, caches, counters and refreshes are per layer"}
    copies = 0
    if refresh and wl.C < wl.E:
        def one(i):                                    # the hidden states cycle; the refresh schedule keeps counting
            n = 0
            if i > 0 and i % wl.K == 0:
                for l in range(L):
                    n += len(sess.refresh(l)[1])
            sess.stack_step([hidden[l][i % n_hidden] for l in range(L)])
            return n
        for i in range(n_hidden):                     # one pass to leave the cold start behind
            one(i)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(n_hidden, n_hidden + steps):
            copies += one(i)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        out.update({"tokens_per_s": wl.N / dt, "ms_per_stack_step": dt * 1e3, "experts_copied": copies, "steps": steps})
    sess.stack_step([hidden[l][0] for l in range(L)])
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for i in range(steps):
        sess.stack_step([hidden[l][i % n_hidden] for l in range(L)])
    torch.cuda.synchronize()
    frozen = (time.perf_counter() - s0) / steps
    out["frozen_placement"] = {"ms_per_stack_step": frozen * 1e3, "us_per_layer": frozen * 1e6 / L, "tokens_per_s": wl.N / frozen}
    # the same steps as one tide_moe_step per layer, in turn on one stream (what the stack call overlaps)
    s0 = time.perf_counter()
    for i in range(steps):
        for l in range(L):
            sess.step(l, hidden[l][i % n_hidden], want_topk=False)
    torch.cuda.synchronize()
    serial = (time.perf_counter() - s0) / steps
    out["frozen_placement"]["ms_per_stack_step_layer_by_layer"] = serial * 1e3
    if "tokens_per_s" not in out:
        out.update({"tokens_per_s": wl.N / frozen, "ms_per_stack_step": frozen * 1e3, "steps": steps, "experts_copied": 0})
    sess.close()
    return out


def run_all_configs(args, ti, tb, TideSession, torch, cfg1_entry, packed_mini, comp_mini):
    """The other configurations in the same run, short: one layer of each (tokens/s with refresh and with the placement
    frozen, kernel durations, roofline fractions), and the two stack workloads at their depth (20 mini layers; 32 flash
    layers with 64 slots per layer and with every expert resident).  Keyed by configuration id."""
    out = {"1": cfg1_entry}
    mini, flash = ti.CONFIGS[2], ti.CONFIGS[3]
    t0 = time.perf_counter()
    wl0 = ti.CONFIGS[0]
    s0 = TideSession(wl0.d, wl0.E, wl0.k, wl0.I, wl0.n_shared, wl0.C, wl0.N, wl0.gating, wl0.bias_mode)      # packs only
    packed0 = s0.pack_layer(lambda e: ti.expert_weights(wl0, 0, e), workers=4)
    s0.close()
    def layer(wl, *a, **kw):                           # one layer in the form of slots this run uses for its size
        fmt = choose_resident(args, wl)
        res, comp = measure_layer(wl, ti, tb, TideSession, torch, *a, **kw)
        res["resident_format"] = fmt
        return res, comp

    def stack(wl, *a, **kw):
        fmt = choose_resident(args, wl)
        res = measure_stack(wl, wl.L, ti, tb, TideSession, torch, *a, **kw)
        res["resident_format"] = fmt
        return res

    out["0"], _ = layer(wl0, packed0, 64, 16, args.refresh_source)
    out["2"], comp_mini = layer(mini, packed_mini, 64, 8, args.refresh_source, comp=comp_mini)
    out["2"]["stack"] = stack(mini, packed_mini, 16, comp=comp_mini)
    probe = TideSession(flash.d, flash.E, flash.k, flash.I, flash.n_shared, 1, 1, flash.gating, flash.bias_mode)
    packed_flash = probe.pack_layer(lambda e: ti.expert_weights(flash, 0, e), workers=16)
    probe.close()
    out["3"], comp_flash = layer(flash, packed_flash, 64, 8, args.refresh_source)
    c4 = ti.CONFIGS[4]
    out["4"], _ = layer(c4, packed_flash, 64, 8, args.refresh_source, comp=comp_flash)
    out["4"]["all_experts_resident"], _ = layer(c4.replace(C=c4.E), packed_flash, 16, 4, "raw")
    # the same layer at batch 256 (8192 tokens per step): every large work item then holds 256 rows
    out["4"]["batch_256"], _ = layer(c4.replace(N=8192), packed_flash, 32, 32, args.refresh_source, comp=comp_flash)
    torch.cuda.empty_cache()
    out["4"]["stack"] = stack(c4, packed_flash, 8, comp=comp_flash)
    out["4"]["stack_all_experts_resident"] = stack(c4.replace(C=c4.E), packed_flash, 4, refresh=False)
    out["seconds_spent_on_this_table"] = time.perf_counter() - t0
    return out


TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "cfg1_mini_layer_hbm_traffic.md")


def read_traffic_summary():
    """HBM bytes per launch of the dominant kernel as measured by rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE
    (scaled by a plain copy of known size); the measurement is kept as text under profiles/ because
    a benchmark run cannot collect hardware counters on itself."""
    try:
        for line in open(TRAFFIC_SUMMARY):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":")[1]), os.path.relpath(TRAFFIC_SUMMARY, ROOT)
    except OSError:
        pass
    return None, None


def run_lossless(args, sess, wl, hidden, tb, ti, torch, mode, share):
    """The layer with its misses evaluated too (full MoE output at every step), refresh every K steps as in the timed
    region.  mode 'device': tide_moe_apply_misses; mode 'host': tide_moe_apply_misses_host, whose workers run while the
    GPU is on the step's hits (Sec. 3.3: layer time = the longer of the two)."""
    if mode == "host":
        sess.host_experts(args.host_threads)
        tb.tide_host_link_share(sess.ctx, share)
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    sess.stats(0, reset=True)
    tb.tide_counters(sess.ctx, reset=True)
    steps = min(args.steps, 4 * wl.S)
    acc = [0.0, 0.0, 0.0]

    def one(t, timed):
        if t > 0 and t % wl.K == 0:
            sess.refresh(0)
        sess.step(0, hidden[t], want_topk=False)
        if mode == "host":
            sess.apply_misses_host(0, hidden[t])
            if timed:
                for i, v in enumerate(tb.tide_host_miss_ms(sess.ctx)):
                    acc[i] += v
        else:
            sess.apply_misses(0, hidden[t])

    for i in range(wl.K * 2):
        one(i % wl.S, False)
    torch.cuda.synchronize()
    tb.tide_counters(sess.ctx, reset=True)
    t0 = time.perf_counter()
    for i in range(steps):
        one((wl.K * 2 + i) % wl.S, True)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    cnt = tb.tide_counters(sess.ctx)
    res = {"us_per_step": dt * 1e6, "tokens_per_s": wl.N / dt, "steps": steps,
           "missed_pairs_per_step": cnt["misses"] / max(cnt["steps"], 1)}
    if mode == "host":
        res.update({"host_threads": args.host_threads, "link_share_percent": share, "wait_for_list_us": acc[0] / steps * 1e3,
                    "host_experts_us": acc[1] / steps * 1e3, "call_us": acc[2] / steps * 1e3})
        sess.host_experts(0)
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=256)
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--config", type=int, default=1, help="workload id (1 = the headline layer; 3 = flash-shaped layer)")
    ap.add_argument("--refresh-mode", choices=("immediate", "deferred"), default="immediate",
                    help="immediate: Alg. 1 as written, the refresh step's GEMMs wait for the copies (default, the headline figure); "
                         "deferred: the refresh step runs on the old placement while the copies land, the new one serves from the next step")
    ap.add_argument("--refresh-call", choices=("sync", "async"), default="sync",
                    help="immediate refresh through tide_refresh (the host waits for the plan, then queues the copies) or "
                         "tide_refresh_async (everything queued at once; the plans are read after the timed region)")
    ap.add_argument("--copy-engine", choices=("kernel", "dma"), default="kernel",
                    help="who moves a refresh's blobs over the host link: the library's copy kernel on the side stream (reads the 12-bit "
                         "form when --refresh-source packed12), or one hipMemcpyAsync per entering expert (raw blobs, copy engines only)")
    ap.add_argument("--commit-after", type=int, default=1,
                    help="deferred mode: steps that still run on the old placement before the new one is committed (1..refresh interval)")
    ap.add_argument("--tokens", type=int, default=0, help="tokens per step (0 = the workload's own; e.g. 4096 = batch 128 of block 32)")
    ap.add_argument("--stack", type=int, default=0,
                    help="run L layers of the workload per denoise step (own router, hidden stream, cache, counter and refresh "
                         "per layer; the layers share layer 0's expert values) and report N / sum of the layers' times")
    ap.add_argument("--refresh-order", choices=("per-layer", "all-first"), default="all-first",
                    help="--stack: at a refresh step, refresh each layer right before its own step, or all layers first so "
                         "that later layers' copies overlap earlier layers' compute")
    ap.add_argument("--capacity", type=int, default=0, help="cache slots (0 = the workload's own budget); 256 = every expert resident")
    ap.add_argument("--resident", choices=("auto", "bf16", "p12"), default="auto",
                    help="the form a cache slot keeps its blob in: the bf16 blob, or its lossless 12-bit form decoded by the "
                         "expert GEMMs in registers (3/4 of the HBM bytes per step; refresh copies then move compressed blobs); "
                         "auto = 12-bit for steps of up to 768 tokens (1024 when d < 4096)")
    ap.add_argument("--refresh-source", choices=("raw", "packed12"), default="packed12",
                    help="what the refresh copies read over the host link: the raw blobs, or their lossless 12-bit form "
                         "(3/4 of the bytes; slots bit-identical)")
    ap.add_argument("--miss-mode", choices=("none", "device", "host", "both"), default="both",
                    help="detail only: also time the lossless layer (step + evaluation of its misses): 'device' = the GPU reads the "
                         "missed experts in place from pinned host memory; 'host' = host worker threads evaluate them while the GPU runs the hits")
    ap.add_argument("--host-threads", type=int, default=16)
    ap.add_argument("--link-share", default="0",
                    help="comma list of percents: share of a step's missed experts the GPU evaluates over the host link while the host "
                         "workers do the rest (0 = all on the host cores, the paper's design); one 'host' measurement per value")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--headline-only", action="store_true",
                    help="only the headline workload: skip the per-configuration table (configurations 0, 2, 3, 4 and the two stacks "
                         "at their depth) that the default run appends after it")
    ap.add_argument("--no-kernel-events", action="store_true", help="do not bracket kernels with HIP events")
    ap.add_argument("--events", choices=("all", "gemm", "gate-up"), default="gate-up",
                    help="which launches of the timed region carry start/stop events (an event-stamped launch costs the host ~15 us): "
                         "'gate-up' = the dominant kernel (grouped gate/up GEMM) and the kernel right before it, so that the interval "
                         "starts as it does under a profiler; 'gemm' = the expert GEMMs only (the cache maintenance between two kernels "
                         "then falls inside the gate/up interval, ~1 us); 'all' = every kernel of a step (what a profiler does).  "
                         "Kernels not bracketed in the timed region are measured in a pass of their own with the placement frozen")
    ap.add_argument("--gemm-calibration", action="store_true",
                    help="print what the vendor library's bf16 GEMM sustains on this GPU at comparable shapes and exit")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="only run 8 plain device copies of 1 GiB (what rocprofv3's FETCH_SIZE / WRITE_SIZE are scaled by) and exit")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (no collectives, no sharding)." % args.gpus,
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import tide_inputs as ti
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; there is no CPU path.", file=sys.stderr)
        sys.exit(2)
    if args.copy_calibration:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda:0")        # 1 GiB
        dst = torch.empty_like(src)
        for _ in range(8):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration": {"bytes_read": 1 << 30, "bytes_written": 1 << 30, "copies": 8}}))
        return
    if args.gemm_calibration:
        # what the vendor's bf16 GEMM (torch.matmul / torch.bmm -> hipBLASLt) sustains on this machine at comparable shapes:
        # a yardstick for the grouped expert GEMM's MFMA fraction, not part of the path
        def rate(fn, flop, n=20):
            for _ in range(3):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(n):
                fn()
            torch.cuda.synchronize()
            return flop / ((time.perf_counter() - t0) / n) / 1e12
        res = {}
        for m, k, n in ((16384, 4096, 2048), (8192, 8192, 8192)):
            a = torch.randn(m, k, device="cuda:0", dtype=torch.bfloat16)
            b = torch.randn(k, n, device="cuda:0", dtype=torch.bfloat16)
            res["mm_%dx%dx%d" % (m, k, n)] = rate(lambda: a @ b, 2.0 * m * k * n)
        for g, m, k, n in ((65, 208, 4096, 2048), (65, 1024, 4096, 2048)):      # 65 slots x rows per slot, gate+up of the flash shape
            a = torch.randn(g, m, k, device="cuda:0", dtype=torch.bfloat16)
            b = torch.randn(g, k, n, device="cuda:0", dtype=torch.bfloat16)
            res["bmm_%dx%dx%dx%d" % (g, m, k, n)] = rate(lambda: torch.bmm(a, b), 2.0 * g * m * k * n)
        print(json.dumps({"gemm_calibration_TFLOP/s": res, "peak": MFMA_BF16_PEAK_TFLOPS}))
        return
    wl = ti.CONFIGS[args.config]
    if args.capacity:
        wl = wl.replace(C=args.capacity)
    if args.tokens:
        wl = wl.replace(N=args.tokens)
    args.resident_policy = args.resident
    args.resident = choose_resident(args, wl)                  # what this run uses, as the JSON line reports it
    if RESIDENT_P12:
        args.refresh_source = "packed12"                       # 12-bit slots are filled with compressed blobs by every engine
    if args.stack:
        run_stack(args, wl, ti, tb, TideSession, torch)
        return
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=RESIDENT_P12)
    packed = sess.pack_layer(lambda e: ti.expert_weights(wl, 0, e), workers=16)
    sess.load_layer(0, None, ti.router_weights(wl, 0), ti.router_bias(wl, 0), ti.initial_resident(wl), packed=packed, workers=16)
    if args.refresh_source == "packed12" and not RESIDENT_P12:
        sess.compress_layer(0, workers=16)
    if args.copy_engine == "dma":
        tb.tide_refresh_engine(sess.ctx, tb.TIDE_COPY_DMA)
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, 0)]
    torch.cuda.synchronize()

    state = {"t": 0, "refresh_s": 0.0, "copies": 0, "copy_ms": 0.0, "refreshes": 0}

    def one_step(timed):
        t = state["t"] % wl.S
        if state.get("uncommitted") and state["t"] >= state["commit_at"]:
            sess.commit(0)
            state["uncommitted"] = False
        if t > 0 and t % wl.K == 0:
            r0 = time.perf_counter()
            if args.refresh_call == "async" and args.refresh_mode == "immediate":
                # the previous refresh's plan is read now, long after its selection ran: no wait
                plan = sess.refresh_result(0)[1] if state.get("result_due") else []
                sess.refresh_async(0)
                state["result_due"] = timed
            else:
                _, plan = sess.refresh(0, deferred=args.refresh_mode == "deferred")
            state["uncommitted"] = args.refresh_mode == "deferred"
            state["commit_at"] = state["t"] + args.commit_after
            if timed:
                state["refresh_s"] += time.perf_counter() - r0
                state["copies"] += len(plan)
                state["refreshes"] += 1
        sess.step(0, hidden[t], want_topk=False)
        state["t"] += 1

    for _ in range(args.warmup):
        one_step(False)
    torch.cuda.synchronize()
    tb.tide_counters(sess.ctx, reset=True)
    if not args.no_kernel_events:
        tb.tide_profile(sess.ctx, {"all": 1, "gemm": 2, "gate-up": 3}[args.events])

    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        one_step(True)
    if state.get("uncommitted"):                    # a deferred refresh of the last step still belongs to the timed work
        sess.commit(0)
        state["uncommitted"] = False
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    if state.get("result_due"):                     # the last asynchronous refresh's plan (outside the timed region)
        state["copies"] += len(sess.refresh_result(0)[1])
        state["result_due"] = False

    prof = tb.tide_profile_read(sess.ctx) if not args.no_kernel_events else {}
    tb.tide_profile(sess.ctx, False)
    cnt = tb.tide_counters(sess.ctx)
    assert cnt["steps"] == args.steps

    # detail only: every kernel of the step bracketed, over the same steps with the placement frozen
    frozen_cnt, from_frozen_pass = None, []
    if prof:
        tb.tide_profile(sess.ctx, 1)
        tb.tide_counters(sess.ctx, reset=True)
        for i in range(args.steps):
            sess.step(0, hidden[i % wl.S], want_topk=False)
        for name, v in tb.tide_profile_read(sess.ctx).items():
            if not prof.get(name, (0.0, 0))[1]:          # not bracketed in the timed region
                prof[name] = v
                if v[1]:
                    from_frozen_pass.append(name)
        frozen_cnt = tb.tide_counters(sess.ctx)
        tb.tide_profile(sess.ctx, False)

    # detail only: the same steps with the placement frozen (no refresh, no event brackets)
    torch.cuda.synchronize()
    s0 = time.perf_counter()
    for i in range(args.steps):
        sess.step(0, hidden[i % wl.S], want_topk=False)
    torch.cuda.synchronize()
    step_only_s = (time.perf_counter() - s0) / args.steps

    # detail only: the same frozen-placement step recorded once into a HIP graph and replayed
    graph_us = None
    try:
        static_in = hidden[0].clone()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            sess.step(0, static_in, want_topk=False)
        for _ in range(8):
            graph.replay()
        torch.cuda.synchronize()
        g0 = time.perf_counter()
        for i in range(args.steps):
            static_in.copy_(hidden[i % wl.S])         # the same inputs as the eager loop above (one small device copy more)
            graph.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - g0) / args.steps * 1e6
        del graph
    except Exception as e:                            # reported, never fatal: the figure is a detail
        print("bench.py: graph replay skipped: %s" % e, file=sys.stderr)

    # measured separately (outside the timed region): one more block with every refresh's copies timed by their own
    # events (this synchronises after each refresh, which the timed region must not do)
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    sess.stats(0, reset=True)
    copied, copy_ms, n_ref = 0, 0.0, 0
    for t in range(wl.S):
        if t > 0 and t % wl.K == 0:
            _, plan = sess.refresh(0)
            n_ref += 1
            if plan:
                copied += len(plan)
                copy_ms += tb.tide_refresh_copy_ms(sess.ctx, 0)
        sess.step(0, hidden[t], want_topk=False)
    torch.cuda.synchronize()
    link_bytes = tb.tide_compressed_blob_bytes(sess.cfg) if args.refresh_source == "packed12" else sess.blob_bytes
    refresh_stats = {"refreshes": n_ref, "experts_copied": copied, "copy_ms_total": copy_ms,
                     "copy_GB/s": (copied * sess.blob_bytes / copy_ms / 1e6) if copy_ms > 0 else None,       # expert bytes landed
                     "link_GB/s": (copied * link_bytes / copy_ms / 1e6) if copy_ms > 0 else None}             # bytes that crossed the link

    # pinned-host -> HBM rate of one refresh's copies when a whole budget of experts moves
    h2d = None
    probe = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode)
    probe.host_blobs[0] = sess.host_blobs[0]
    tb.tide_register_experts(probe.ctx, 0, sess.host_blobs[0], sess.blob_bytes)
    tb.tide_set_resident(probe.ctx, 0, list(range(wl.C)))
    counts = np.zeros(wl.E, dtype=np.int32)
    counts[wl.C:2 * wl.C] = 1                      # swaps in `capacity` new experts
    _, plan = probe.refresh(0, counts=counts)
    ms = tb.tide_refresh_copy_ms(probe.ctx, 0)
    if plan and ms > 0:
        h2d = {"GB/s": len(plan) * sess.blob_bytes / ms / 1e6, "copies": len(plan), "MiB_each": sess.blob_bytes / 2 ** 20}
    # detail only: the timed loop once more without event brackets, and (if the copies read the 12-bit form) once more
    # with the refresh copies reading the raw blobs (Alg. 1's copies as they are)
    def plain_pass():
        tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
        sess.stats(0, reset=True)
        state.update({"t": 0, "uncommitted": False})
        for _ in range(args.warmup):
            one_step(False)
        torch.cuda.synchronize()
        r0 = time.perf_counter()
        for _ in range(args.steps):
            one_step(False)
        if state.get("uncommitted"):
            sess.commit(0)
            state["uncommitted"] = False
        torch.cuda.synchronize()
        rdt = time.perf_counter() - r0
        return {"tokens_per_s": wl.N * args.steps / rdt, "us_per_step": rdt / args.steps * 1e6}

    no_events = plain_pass()
    raw_source = None
    if args.refresh_source == "packed12" and not RESIDENT_P12:     # bf16 slots can also be refreshed from the raw blobs
        tb.tide_register_compressed(sess.ctx, 0, None, 0)
        raw_source = plain_pass()
        tb.tide_register_compressed(sess.ctx, 0, sess.comp_blobs[0], tb.tide_compressed_blob_bytes(sess.cfg))
    bf16_ref = None
    if RESIDENT_P12 and not args.headline_only and args.refresh_mode == "immediate" and args.refresh_call == "sync" and args.copy_engine == "kernel":
        bf16_ref = bf16_reference(wl, args, ti, tb, TideSession, torch, packed, sess.comp_blobs[0], list(ti.hidden_stream(wl, 0)))
        raw_source = bf16_ref["raw"]
    h2d_p12 = None
    if args.refresh_source == "packed12":
        cbytes = tb.tide_compressed_blob_bytes(sess.cfg)
        tb.tide_register_compressed(probe.ctx, 0, sess.comp_blobs[0], cbytes)
        tb.tide_set_resident(probe.ctx, 0, list(range(wl.C)))
        _, plan = probe.refresh(0, counts=counts)
        ms = tb.tide_refresh_copy_ms(probe.ctx, 0)
        if plan and ms > 0:
            h2d_p12 = {"expert_GB/s": len(plan) * sess.blob_bytes / ms / 1e6, "link_GB/s": len(plan) * cbytes / ms / 1e6,
                       "copies": len(plan), "bytes_over_link_per_expert": cbytes}
    probe.close()

    lossless = None
    if args.miss_mode != "none":
        lossless = {}
        for m in (("device", "host") if args.miss_mode == "both" else (args.miss_mode,)):
            if m == "device":
                lossless[m] = run_lossless(args, sess, wl, hidden, tb, ti, torch, m, 0)
            else:
                for share in [int(v) for v in args.link_share.split(",")]:
                    lossless["host" if share == 0 else "host+link%d" % share] = run_lossless(args, sess, wl, hidden, tb, ti, torch, m, share)

    tokens = wl.N * args.steps
    value = tokens / dt
    blob = sess.blob_bytes
    roofline = None
    kernels = {}
    if prof:
        # avg_us: mean time between the start and stop events each launch stamps on its own stream
        for name, (ms_sum, n) in prof.items():
            if n:
                kernels[name] = {"avg_us": 1e3 * ms_sum / n, "launches": n}
        ms_sum, n = prof["gate_up_swiglu"]
        ms_big, n_big = prof.get("gate_up_swiglu_big", (0.0, 0))
        # slots with more than 32 rows run in a second launch of the same GEMM, on a second stream beside the
        # first: the two start together, so the pair's duration is taken as the longer of the two averages
        if n_big:
            ms_sum = max(ms_sum, ms_big * n / n_big)
        # algorithmic bytes of one gate/up launch: the gate and up matrices (2/3 of a blob) of every cache
        # slot that has a token this step (shared expert included), the step's hidden states once, and the
        # bf16 activations written
        active_per_launch = cnt["active_slots"] / cnt["steps"]
        rows_per_launch = cnt["rows"] / cnt["steps"]
        bytes_per_launch = active_per_launch * (2 * blob / 3) + wl.N * wl.d * 2 + rows_per_launch * wl.I * 2
        avg_s = 1e-3 * ms_sum / n
        achieved = bytes_per_launch / avg_s / 1e9
        roofline = {"bound": "hbm", "kernel": "expert_gemm_kernel<0>%s (grouped gate/up GEMM + SwiGLU)" % (" + expert_gemm_big_kernel<0>" if n_big else ""),
                    "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                    "traffic": None, "avg_kernel_us": avg_s * 1e6, "algorithmic_bytes_per_launch": bytes_per_launch,
                    "active_slots_per_launch": active_per_launch, "resident_format": args.resident}
        if RESIDENT_P12:
            # what the launch actually asks HBM for: the 12-bit form of the same matrices (768 + 16 bytes per 1 KiB
            # tile); `achieved` stays the method's own bytes (bf16 weights) over the launch time, as for bf16 slots
            streamed = active_per_launch * (2 * blob / 3) * 784.0 / 1024.0 + wl.N * wl.d * 2 + rows_per_launch * wl.I * 2
            roofline["bytes_streamed_per_launch"] = streamed
            roofline["streamed"] = {"achieved": streamed / avg_s / 1e9, "frac": streamed / avg_s / 1e9 / HBM_PEAK_GBS, "unit": "GB/s"}
        # the same launch against the matrix cores: 2 * rows * d * 2I flop (gate and up) on the bf16 MFMA peak
        roofline["mfma"] = {"achieved": rows_per_launch * 4.0 * wl.d * wl.I / avg_s / 1e12, "peak": MFMA_BF16_PEAK_TFLOPS,
                            "unit": "TFLOP/s", "frac": rows_per_launch * 4.0 * wl.d * wl.I / avg_s / 1e12 / MFMA_BF16_PEAK_TFLOPS}
        ms2, n2 = prof["down"]
        ms2b, n2b = prof.get("down_big", (0.0, 0))
        if n2b:
            ms2 = max(ms2, ms2b * n2 / n2b)
        if n2:
            # bytes from the counters of the pass the duration comes from
            c2 = frozen_cnt if "down" in from_frozen_pass else cnt
            a2, r2 = c2["active_slots"] / c2["steps"], c2["rows"] / c2["steps"]
            b2 = a2 * (blob / 3) + r2 * wl.I * 2 + r2 * wl.d * 4
            roofline["down_kernel"] = {"achieved": b2 / (1e-3 * ms2 / n2) / 1e9, "frac": b2 / (1e-3 * ms2 / n2) / 1e9 / HBM_PEAK_GBS,
                                       "avg_kernel_us": 1e3 * ms2 / n2,
                                       "measured_in": "frozen-placement pass" if "down" in from_frozen_pass else "timed region"}

    if roofline is not None:
        rate, nbytes = tb.tide_hbm_stream_probe(sess.ctx, 0, 8)
        roofline["hbm_stream_probe"] = {"GB/s": rate, "bytes_per_launch": nbytes, "frac_of_peak": rate / HBM_PEAK_GBS,
                                        "what": "a kernel that only reads this layer's cache slots once, in the GEMMs' weight-stream shape "
                                                "(slot sets under the chip's 256 MB memory-side cache read faster than HBM delivers)"}
    if roofline is not None and args.config == 1 and not (args.tokens or args.capacity):
        roofline["traffic"], src = read_traffic_summary()
        roofline["traffic_measured"] = ("offline, not by this run: rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this command, "
                                        "scaled by a plain copy of known size; summary in %s" % src)
    step_bytes = (cnt["active_slots"] / cnt["steps"]) * blob + wl.E * wl.d * 4 + wl.N * wl.d * 2 + wl.N * wl.d * 4
    configs = None
    if not args.headline_only and args.config == 1 and not (args.tokens or args.capacity):
        comp1 = sess.comp_blobs[0] if args.refresh_source == "packed12" else None
        sess.close()
        this = {"workload": wl.name, "tokens_per_step": wl.N, "d": wl.d, "d_ff": wl.I, "capacity": wl.C, "layers_in_workload": 1,
                "layers_measured": 1, "steps": args.steps, "warmup": args.warmup, "tokens_per_s": value, "ms_per_step": 1e3 * dt / args.steps,
                "refresh_source": args.refresh_source,
                "tokens_per_s_raw_refresh_copies": raw_source["tokens_per_s"] if raw_source else (None if RESIDENT_P12 else no_events["tokens_per_s"]),
                "frozen_placement": {"us_per_step": step_only_s * 1e6, "tokens_per_s": wl.N / step_only_s},
                "kernels_us": {k_: v_["avg_us"] for k_, v_ in kernels.items()},
                "roofline": None if frozen_cnt is None else layer_rooflines(
                    wl, blob, frozen_cnt["active_slots"] / frozen_cnt["steps"], frozen_cnt["rows"] / frozen_cnt["steps"],
                    1e-6 * kernels["gate_up_swiglu"]["avg_us"], 1e-6 * kernels["down"]["avg_us"], step_only_s)}
        this["resident_format"] = args.resident
        configs = run_all_configs(args, ti, tb, TideSession, torch, this, packed, comp1)
        choose_resident(args, wl)
        if roofline is not None and configs.get("4") and configs["4"].get("roofline"):
            c4 = configs["4"]
            roofline["cfg4"] = {"workload": c4["workload"], "tokens_per_step": c4["tokens_per_step"], "capacity": c4["capacity"],
                                "layers_measured": 1, "tokens_per_s": c4["tokens_per_s"],
                                "tokens_per_s_frozen_placement": c4["frozen_placement"]["tokens_per_s"],
                                "kernel": "expert_gemm_big_kernel<0> beside expert_gemm_kernel<0> (grouped gate/up GEMM + SwiGLU)",
                                "bound": "mfma", "mfma": c4["roofline"]["gate_up"]["mfma"], "hbm": c4["roofline"]["gate_up"]["hbm"],
                                "avg_kernel_us": c4["roofline"]["gate_up"]["us"], "down_kernel": c4["roofline"]["down"],
                                "step": c4["roofline"]["step"]}
            b256 = c4.get("batch_256")
            if b256 and b256.get("roofline"):
                roofline["cfg4"]["batch_256"] = {"tokens_per_step": b256["tokens_per_step"], "tokens_per_s": b256["tokens_per_s"],
                                                 "tokens_per_s_frozen_placement": b256["frozen_placement"]["tokens_per_s"],
                                                 "mfma": b256["roofline"]["gate_up"]["mfma"], "hbm": b256["roofline"]["gate_up"]["hbm"],
                                                 "avg_kernel_us": b256["roofline"]["gate_up"]["us"], "down_kernel": b256["roofline"]["down"]}
    out = {
        "metric": "MoE-layer tokens/s per denoise step", "value": value, "unit": "tokens/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps, "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "d": wl.d, "experts": wl.E, "top_k": wl.k, "d_ff": wl.I, "shared_experts": wl.n_shared,
                   "tokens_per_step": wl.N, "capacity": wl.C, "refresh_interval": wl.K, "steps_per_block": wl.S, "layers": 1,
                   "refresh_source": args.refresh_source if (args.copy_engine == "kernel" or RESIDENT_P12) else "raw", "refresh_call": args.refresh_call,
                   "copy_engine": args.copy_engine, "resident_format": args.resident,
                   "refresh_mode": args.refresh_mode if args.refresh_mode == "immediate" else "deferred by %d step(s)" % args.commit_after},
        "value_refresh_source": args.refresh_source + (" (lossless 12-bit form of the blobs read over the host link)" if args.refresh_source == "packed12" else " blobs"),
        "value_with_raw_refresh_copies": raw_source["tokens_per_s"] if raw_source else (None if RESIDENT_P12 else no_events["tokens_per_s"]),
        "value_resident_format": ("12-bit slots (the blobs' lossless 12-bit form, decoded in the expert GEMMs' registers)" if RESIDENT_P12 else "bf16 slots"),
        "value_with_bf16_slots": None if bf16_ref is None else bf16_ref["packed12"]["tokens_per_s"],
        "roofline": roofline,
        "configs": configs,
        "detail": {
            "kernels": kernels, "kernels_measured_in_frozen_placement_pass": from_frozen_pass,
            "step_hbm_roofline_us": step_bytes / (HBM_PEAK_GBS * 1e9) * 1e6,
            "hit_rate": 1.0 - cnt["misses"] / (tokens * wl.k),
            "refreshes": state["refreshes"], "experts_copied": state["copies"],
            "refresh_host_s": state["refresh_s"],
            "frozen_placement_us_per_step": step_only_s * 1e6,
            "frozen_placement_graph_replay_us_per_step": graph_us,
            "exposed_refresh_us_per_interval": (dt / args.steps - step_only_s) * 1e6 * wl.K,
            "refresh_copies": refresh_stats,
            "frozen_placement_tokens_per_s": wl.N / step_only_s,
            "h2d_probe": h2d,
            "h2d_probe_packed12": h2d_p12,
            "without_kernel_events": no_events,
            "without_kernel_events_raw_refresh_copies": raw_source,
            "lossless_layer": lossless,
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, ti)
    if sess.ctx:
        sess.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
