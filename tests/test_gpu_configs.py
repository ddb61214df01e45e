"""GPU parity at the shapes AND depths of workload configurations 2, 3 and 4 (the larger ones).

Routing, hit counters, miss lists, resident sets and copy plans are compared bit for bit for every
token of every step of every layer that runs -- the stacks at their full depth (20 and 32 layers,
the flash stack in both cache settings).  Expert outputs are compared on samples the fp64 oracle can
evaluate one (token, expert) pair at a time: every token of two steps at configuration 3, and at
every other checked step at least 64 tokens chosen AFTER the step has run, from the library's own
work-item list, so that every kind of grouped-GEMM work item of that step (small items of one and two
16-token tiles, large items of 1..16 tiles, the shared expert, the slots with the fewest rows) has
rows in the sample; a seeded random draw fills the rest.  Beside the error against the oracle's
default (SwiGLU activation stored in bf16, as the kernels store it) the error against the un-rounded
definition is computed and reported.  A step of every output-checked layer is run twice and must
repeat bit for bit.  Near-tie tokens (selection keys closer than 1e-5, where fp32 and fp64 may order
differently) and the errors are written to a JSON report (REPORT below; the un-rounded figure is a report, not
a bound: the bf16 store alone moves single outputs by up to about 1e-2 x RMS).

Stacks: layers are independent (own router, hidden stream, cache, counter, refresh).  To bound host
memory and set-up time only the layers whose outputs are checked carry their own seeded expert
values; the other layers of a stack reuse layer 0's packed blobs (their routers, bias permutations
and hidden streams are their own, so routing, counters, placements and plans differ per layer)."""
import concurrent.futures
import json
import os
import time

import numpy as np
import pytest
import torch

import tide_inputs as ti
from oracle import tide_oracle as orc
from test_gpu_parity import (_session, check_miss, check_out, check_routing, load, oracle_block, run_block_on_gpu,
                             say)

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
REPORT = os.path.join(ROOT, "gpurun_out", "parity_report.json")

_BITS = {}       # (d, I, E, seed, layer) -> list of E+1 (wg, wu, wd) bf16 bit triples
_PACKED = {}     # same key -> (pinned blobs, shared blob)
_COMP = {}       # same key -> pinned 12-bit form of the blobs (sessions with 12-bit slots)


def _key(wl, layer):
    return (wl.d, wl.I, wl.E, wl.seed, layer)


def layer_bits(wl, layer):
    """The layer's seeded expert matrices (E routed + the shared one), drawn once with 16 threads and kept:
    the packed blobs and the oracle's fp64 copies are both made from them."""
    key = _key(wl, layer)
    if key not in _BITS:
        say("drawing %d experts d=%d I=%d layer %d" % (wl.E + 1, wl.d, wl.I, layer))
        with concurrent.futures.ThreadPoolExecutor(max_workers=16) as ex:
            _BITS[key] = list(ex.map(lambda e: ti.expert_weights(wl, layer, e), range(wl.E + 1)))
    return _BITS[key]


def packed_layer(sess, wl, layer):
    """Pinned packed blobs of (shape, layer), built once per test session."""
    key = _key(wl, layer)
    if key not in _PACKED:
        bits = layer_bits(wl, layer)
        _PACKED[key] = sess.pack_layer(lambda e: bits[e], workers=16)
    return _PACKED[key]


def compressed_layer(sess, wl, layer):
    """Pinned 12-bit form of packed_layer's blobs, built once per test session."""
    from paper_2605_20179_amd import binding as tb
    key = _key(wl, layer)
    if key not in _COMP:
        raw = packed_layer(sess, wl, layer)[0].numpy()
        comp = torch.empty((wl.E, tb.tide_compressed_blob_bytes(sess.cfg)), dtype=torch.uint8, pin_memory=True)
        out = comp.numpy()
        with concurrent.futures.ThreadPoolExecutor(max_workers=16) as ex:
            list(ex.map(lambda e: tb.tide_compress_expert(sess.cfg, raw[e], out[e]), range(wl.E)))
        _COMP[key] = comp
    return _COMP[key]


def forget(wl, layer):
    _BITS.pop(_key(wl, layer), None)
    _PACKED.pop(_key(wl, layer), None)
    _COMP.pop(_key(wl, layer), None)


def load_packed(sess, wl, layer, sess_layer=None, resident=None, values_of=None):
    """Layer `layer`'s router, bias and placement into session layer `sess_layer`, with the expert values of
    workload layer `values_of` (default: its own)."""
    sess.load_layer(layer if sess_layer is None else sess_layer, None, ti.router_weights(wl, layer),
                    ti.router_bias(wl, layer), ti.initial_resident(wl) if resident is None else resident,
                    packed=packed_layer(sess, wl, layer if values_of is None else values_of),
                    comp=compressed_layer(sess, wl, layer if values_of is None else values_of) if sess.resident_p12 else None)


def report(section, payload):
    """Merges `payload` into the JSON report under `section`."""
    os.makedirs(os.path.dirname(REPORT), exist_ok=True)
    try:
        doc = json.load(open(REPORT))
    except (OSError, ValueError):
        doc = {}
    doc.setdefault(section, {}).update(payload)
    with open(REPORT, "w") as f:
        json.dump(doc, f, indent=1, sort_keys=True)
    say("%s: %s" % (section, json.dumps(payload, sort_keys=True)))


class LayerRun:
    """One layer of a run: its workload layer id, its index in the session, the oracle's routing / placement log,
    its hidden-state stream, and (for output-checked layers) the oracle's fp64 expert store."""

    def __init__(self, wl, layer, li, with_outputs=False, values_of=None):
        self.wl, self.layer, self.li = wl, layer, li
        self.hidden = list(ti.hidden_stream(wl, layer))
        self.log = orc.run_block(self.hidden, ti.router_weights(wl, layer), ti.router_bias(wl, layer), wl.gating,
                                 wl.bias_mode, wl.k, wl.E, wl.C, wl.K, ti.initial_resident(wl))
        self.values_of = layer if values_of is None else values_of
        self.store = self.shared = None
        if with_outputs:
            bits = layer_bits(wl, self.values_of)
            self.store = orc.ExpertStore(lambda e: bits[e], max_cached=wl.E + 1)
            self.shared = tuple(orc.bf16_to_f64(m) for m in bits[wl.E]) if wl.n_shared else None
        self.near = [int(r["ambiguous"].sum()) for r in self.log]
        self.flips = [0] * len(self.log)
        self.exact = True

    def drop_store(self):
        self.store = self.shared = None


def item_classes(items, capacity):
    """Kind of every work item: ('shared', tiles) for the shared expert's, else ('small' | 'large', tiles)."""
    out = []
    for it in items:
        tiles = (int(it["nrows"]) + 15) // 16
        if int(it["slot"]) == capacity:
            out.append(("shared-" + ("large" if it["kind"] else "small"), tiles))
        else:
            out.append(("large" if it["kind"] else "small", tiles))
    return out


def stratified_tokens(items, row_token, capacity, n_tokens, want, seed):
    """At least `want` tokens such that every class of work item of the step, and the three slots with the fewest
    rows, have rows in the sample: from the first and the last item of each class the tokens of its first and
    last row (the last row sits in the item's ragged tile); the rest drawn at random."""
    classes = item_classes(items, capacity)
    chosen = set()
    by_class = {}
    for i, c in enumerate(classes):
        by_class.setdefault(c, []).append(i)
    picks = [i for idx in by_class.values() for i in (idx[0], idx[-1])]
    rows_of_slot = {}
    for it in items:
        rows_of_slot[int(it["slot"])] = rows_of_slot.get(int(it["slot"]), 0) + int(it["nrows"])
    tail_slots = sorted(rows_of_slot, key=lambda s: (rows_of_slot[s], s))[:3]
    picks += [i for i, it in enumerate(items) if int(it["slot"]) in tail_slots]
    for i in picks:
        it = items[i]
        chosen.add(int(row_token[int(it["row0"])]))
        chosen.add(int(row_token[int(it["row0"]) + int(it["nrows"]) - 1]))
    rng = np.random.default_rng(seed)
    for n in rng.permutation(n_tokens).tolist():
        if len(chosen) >= want:
            break
        chosen.add(int(n))
    toks = sorted(chosen)
    # the claim, checked: every class (and every tail slot) has at least one row whose token is sampled
    in_sample = np.zeros(n_tokens, dtype=bool)
    in_sample[toks] = True
    covered, tails = set(), set()
    for it, c in zip(items, classes):
        if in_sample[row_token[int(it["row0"]):int(it["row0"]) + int(it["nrows"])]].any():
            covered.add(c)
            if int(it["slot"]) in tail_slots:
                tails.add(int(it["slot"]))
    assert covered == set(classes), "work-item classes without a sampled row: %s" % (set(classes) - covered)
    assert tails == set(tail_slots)
    return toks, sorted(set(classes))


def outputs_check(sess, tb, run, t, x, mode, stats):
    """After a forced-routing step of an output-checked layer: run-to-run identity, resident-partial output,
    the miss pass's completed output, both against the oracle, on every token ("all") or a stratified sample."""
    wl, rec, li = run.wl, run.log[t], run.li
    out1 = sess.out[:wl.N].cpu().numpy().copy()
    miss1 = sess.miss[:max(len(rec["miss"]), 1)].cpu().numpy().copy()
    items, row_token = tb.tide_read_work_items(sess.ctx, 4 * (wl.C + 1) + wl.N * (wl.k + 1) // 32 + 64, wl.N * (wl.k + 1))
    assert int(items["nrows"].sum()) == len(row_token) == wl.N * (wl.k + wl.n_shared) - len(rec["miss"])
    # the same step once more from the same counter: every output bit and every list entry repeats
    h_now = sess.stats(li)
    tb.tide_set_counts(sess.ctx, li, h_now - rec["hist"].astype(np.int32))
    sess.step_routed(li, x, torch.from_numpy(rec["idx"]).to(sess.device),
                     torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device))
    torch.cuda.synchronize()
    assert np.array_equal(sess.out[:wl.N].cpu().numpy(), out1), "layer %d step %d: output differs run to run" % (run.layer, t)
    assert np.array_equal(sess.miss[:max(len(rec["miss"]), 1)].cpu().numpy(), miss1)
    assert np.array_equal(sess.stats(li), h_now)
    if mode == "all":
        toks, classes = list(range(wl.N)), sorted(set(item_classes(items, wl.C)))
    else:
        toks, classes = stratified_tokens(items, row_token, wl.C, wl.N, mode, seed=1000 * run.layer + t)
    t0 = time.perf_counter()
    y_res, y_full, _ = orc.moe_outputs(run.hidden[t], rec["idx"], rec["w"], rec["slot_of"], run.store, run.shared, tokens=toks)
    err = check_out(out1, y_res, rows=toks)
    # the same tokens against the definition with the activation left un-rounded: reported, not asserted -- storing
    # the activation in bf16 is part of the computation (2^-9 relative per element ahead of a d_ff-term sum), and its
    # largest effect over thousands of outputs sits right at the 1e-2 x RMS bound
    few = toks[:: max(1, len(toks) // 16)]
    y_exact, _, _ = orc.moe_outputs(run.hidden[t], rec["idx"], rec["w"], rec["slot_of"], run.store, run.shared,
                                    act_bf16=False, tokens=few, want_full=False)
    err_exact = float(np.abs(out1[few] - y_exact).max() / np.sqrt(np.mean(y_exact ** 2)))
    stats["oracle_s"] += time.perf_counter() - t0
    # misses evaluated from the pinned host blobs complete the output: resident part + misses == full layer
    sess.apply_misses(li, x)
    torch.cuda.synchronize()
    err_full = check_out(sess.out[:wl.N].cpu().numpy(), y_full, rows=toks)
    assert np.array_equal(sess.stats(li), h_now), "the miss pass must not count"
    stats["worst"] = max(stats["worst"], err, err_full)
    stats["worst_vs_unrounded_activation"] = max(stats["worst_vs_unrounded_activation"], err_exact)
    stats["checked"].append({"layer": run.layer, "step": t, "tokens": len(toks),
                             "work_item_classes": ["%s x%d" % c for c in classes]})


def drive(sess, tb, runs, forced, out_checks=None):
    """All layers of `runs` through the block in stack order (per step: every layer in turn, its refresh right
    before its step), every step compared with the oracle's log.  out_checks: {(layer, t): "all" | n_tokens}."""
    out_checks = out_checks or {}
    stats = {"worst": 0.0, "worst_vs_unrounded_activation": 0.0, "checked": [], "oracle_s": 0.0}
    S = len(runs[0].log)
    dev = {}
    for t in range(S):
        for run in runs:
            wl, rec, li = run.wl, run.log[t], run.li
            if t > 0 and t % wl.K == 0:
                eis, plan = sess.refresh(li)
                if run.exact:
                    assert eis.tolist() == rec["expert_in_slot"].tolist(), "layer %d step %d: resident set" % (run.layer, t)
                    assert [(e, s) for e, s, _, _ in plan] == [tuple(p) for p in rec["plan"]], "layer %d step %d: plan" % (run.layer, t)
            x = sess.to_device_bf16(run.hidden[t])
            if forced:
                sess.step_routed(li, x, torch.from_numpy(rec["idx"]).to(sess.device),
                                 torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device))
                _, _, _, miss, n_miss = sess.results(wl.N)
            else:
                sess.step(li, x)
                _, idx, w, miss, n_miss = sess.results(wl.N)
                flips = check_routing(rec, idx, w, wl.k)
                run.flips[t] = len(flips)
                if flips:
                    run.exact = False
            if run.exact:
                check_miss(rec["miss"], miss, n_miss)
                assert np.array_equal(sess.stats(li), rec["hits"].astype(np.int32)), "layer %d step %d: hit counter" % (run.layer, t)
                assert np.array_equal(sess.table(li), rec["slot_of"]), "layer %d step %d: table" % (run.layer, t)
                if forced and (run.layer, t) in out_checks:
                    outputs_check(sess, tb, run, t, x, out_checks[(run.layer, t)], stats)
            else:
                start = (t // wl.K) * wl.K
                assert sess.stats(li).sum() == sum(int(r["hist"].sum()) for r in run.log[start:t + 1])
    return stats


def stack_rate(sess, runs, steps):
    """tokens/s of the stack with the placement as the run left it (no refresh): N / sum over the layers."""
    xs = [[sess.to_device_bf16(run.hidden[t]) for t in range(min(steps, len(run.hidden)))] for run in runs]
    assert [run.li for run in runs] == list(range(len(runs)))
    for _ in range(2):
        sess.stack_step([x[0] for x in xs])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(steps):
        sess.stack_step([x[i % len(x)] for x in xs])
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    return {"layers": len(runs), "us_per_stack_step_frozen_placement": dt * 1e6, "tokens_per_s": runs[0].wl.N / dt}


def near_tie_summary(runs):
    return {"near_tie_tokens_per_step": {str(r.layer): r.near for r in runs},
            "tokens_selected_differently_per_step": {str(r.layer): r.flips for r in runs if any(r.flips)},
            "near_tie_tokens_total": int(sum(sum(r.near) for r in runs)),
            "tokens_selected_differently_total": int(sum(sum(r.flips) for r in runs))}


def run_config(name, wl, layers, own_values, out_checks, sample_rate_steps=0, p12=False):
    """Context of len(layers) layers; forced-routing run (everything downstream of routing bit-exact, outputs),
    then a run with the library's own routing (selections, weights; downstream exact until a near-tie flips)."""
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    t0 = time.perf_counter()
    runs = [LayerRun(wl, layer, li, with_outputs=layer in own_values, values_of=layer if layer in own_values else layers[0])
            for li, layer in enumerate(layers)]
    say("%s: oracle routing of %d layers x %d steps in %.1f s" % (name, len(runs), wl.S, time.perf_counter() - t0))
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, n_layers=len(layers),
                       resident_p12=p12)
    summary = {"resident_format": "p12" if p12 else "bf16"}
    for forced in (True, False):
        for run in runs:
            load_packed(sess, wl, run.layer, sess_layer=run.li, values_of=run.values_of)
            sess.stats(run.li, reset=True)
            run.exact = True
        stats = drive(sess, tb, runs, forced, out_checks if forced else None)
        if forced:
            summary.update(stats)
            assert len(stats["checked"]) == len(out_checks)
        say("%s forced=%s done" % (name, forced))
    summary.update(near_tie_summary(runs))
    if sample_rate_steps:
        summary["stack_rate"] = stack_rate(sess, runs, sample_rate_steps)
    summary["hbm_GiB_of_cache_slots"] = len(layers) * (wl.C + 1) * sess.blob_bytes / 2 ** 30
    summary["layers_with_own_expert_values"] = sorted(own_values)
    sess.close()
    for run in runs:
        run.drop_store()
    report(name, summary)
    return summary


# ----------------------------------------------------------------------------- configuration 2
@pytest.mark.parametrize("p12", [False, True], ids=["bf16 slots", "12-bit slots"])
def test_config2_stack_at_depth(p12):
    """Mini-shaped stack at its depth: 20 layers x 256 tokens x the 32-step block, K = 4.  Outputs on layers 0, 7
    and 19 (own expert values) at a cold step, a refresh step, the step after it and the last one.  Once over bf16
    slots and once over 12-bit slots (the form bench.py times this configuration in)."""
    wl = ti.CONFIGS[2]
    checks = {(layer, t): 48 for layer in (0, 7, 19) for t in (0, 4, 5, 31)}
    s = run_config("cfg2-mini-stack L=20" + (" 12-bit slots" if p12 else ""), wl, list(range(wl.L)), {0, 7, 19}, checks,
                   sample_rate_steps=16, p12=p12)
    assert s["worst"] <= 1e-2


def test_config2_interval_sweep():
    """K in {1, 2, 8} on layer 0 (17 steps): routing, counters, refreshes, miss lists."""
    base = ti.CONFIGS[2]
    sess = _session(base)
    swaps = {}
    for K in (1, 2, 8):
        wl = base.replace(K=K, S=17)
        log, hidden = oracle_block(wl, 0, [])
        load_packed(sess, wl, 0)
        sess.stats(0, reset=True)
        run_block_on_gpu(wl, 0, sess, log, hidden, True, [])
        swaps[str(K)] = [len(r["plan"]) for r in log if r["plan"] is not None]
    report("cfg2 interval sweep", {"experts_copied_per_refresh": swaps})
    sess.close()


# ----------------------------------------------------------------------------- configuration 3
@pytest.mark.parametrize("p12", [False, True], ids=["bf16 slots", "12-bit slots"])
def test_config3_flash_layer(p12):
    """Flash-shaped layer, 512 tokens per step, the whole 32-step block.  Outputs on EVERY token at step 0 (cold
    placement, most misses) and step 4 (first refresh), on 64 stratified tokens at every other step.  Over bf16 slots
    and over 12-bit slots (the form bench.py times this configuration in; large work items of up to 192 rows)."""
    wl = ti.CONFIGS[3]
    checks = {(0, t): ("all" if t in (0, 4) else 64) for t in range(wl.S)}
    s = run_config("cfg3-flash-layer" + (" 12-bit slots" if p12 else ""), wl, [0], {0}, checks, p12=p12)
    assert s["worst"] <= 1e-2
    if p12:
        return
    # the host-core miss path at this size (over a thousand missed pairs over most of the 192 non-resident experts)
    log, hidden = oracle_block(wl.replace(S=1), 0, [])
    bits = layer_bits(wl, 0)
    store = orc.ExpertStore(lambda e: bits[e], max_cached=wl.E + 1)
    shared = tuple(orc.bf16_to_f64(m) for m in bits[wl.E])
    toks = sorted(np.random.default_rng(3).choice(wl.N, size=24, replace=False).tolist())
    _, y_full, _ = orc.moe_outputs(hidden[0], log[0]["idx"], log[0]["w"], log[0]["slot_of"], store, shared, tokens=toks)
    sess = _session(wl)
    load_packed(sess, wl, 0)
    sess.host_experts(16)
    x = sess.to_device_bf16(hidden[0])
    sess.step_routed(0, x, torch.from_numpy(log[0]["idx"]).to(sess.device),
                     torch.from_numpy(log[0]["w"].astype(np.float32)).to(sess.device))
    sess.apply_misses_host(0, x)
    torch.cuda.synchronize()
    err = check_out(sess.out[:wl.N].cpu().numpy(), y_full, rows=toks)
    say("cfg3 host miss path: %d misses, worst=%.2e" % (len(log[0]["miss"]), err))
    sess.close()


# ----------------------------------------------------------------------------- configuration 4
def test_config4_flash_stack_eight_layers():
    """Flash-shaped stack, capacity 64 per layer with the remainder in pinned host memory: an 8-layer context
    (layers 0, 5, 11, 17, 23, 29, 30, 31 of the 32) through the whole 32-step block at 2048 tokens per step.
    Outputs on layers 0 and 31 (own expert values) at the cold step, the first refresh step and the step after."""
    wl = ti.CONFIGS[4]
    layers = [0, 5, 11, 17, 23, 29, 30, 31]
    checks = {(layer, t): 64 for layer in (0, 31) for t in (0, 4, 5)}
    s = run_config("cfg4-flash-stack C=64, 8 of 32 layers, 32 steps", wl, layers, {0, 31}, checks)
    assert s["worst"] <= 1e-2
    big = {c for ch in s["checked"] for c in ch["work_item_classes"] if c.startswith("large")}
    assert any(int(c.split("x")[1]) <= 8 for c in big) and any(int(c.split("x")[1]) > 8 for c in big), \
        "both large-item forms (up to 8 and 9..16 token tiles) must have been checked: %s" % sorted(big)


@pytest.mark.parametrize("capacity", [64, 256])
def test_config4_flash_stack_full_depth(capacity):
    """The flash stack as the 32-layer stack it is, in both cache settings: capacity 64 per layer (48.8 GiB of
    slots, the other experts in pinned host memory) and every expert resident (192.8 GiB of slots).  Five steps
    with the refresh before step 4; every layer's routing, counters, miss lists, placement and plan; outputs on
    layers 0 and 31 at steps 0 and 4; the stack's step rate from the same context."""
    wl = ti.CONFIGS[4].replace(S=5, C=capacity)
    checks = {(layer, t): 64 for layer in (0, 31) for t in (0, 4)}
    s = run_config("cfg4-flash-stack C=%d, 32 layers, 5 steps" % capacity, wl, list(range(wl.L)), {0, 31}, checks,
                   sample_rate_steps=4)
    assert s["worst"] <= 1e-2
    assert abs(s["hbm_GiB_of_cache_slots"] - 32 * (capacity + 1) * 24 / 1024) < 1e-6
    if capacity == 256:
        forget(wl, 31)                       # last user of these 12 GiB of host memory


def test_maximum_tokens_per_step():
    """The largest step the library accepts (max_tokens = 65535, a ragged last tile everywhere) on small matrices:
    three steps with a refresh, every token's routing, the 160 000-entry miss lists, counters, tables and the copy
    plan compared; outputs (resident part, then completed by the miss pass) on 12 sampled tokens."""
    wl = ti.TideWorkload("max-tokens", d=64, E=32, k=4, I=64, n_shared=1, N=65535, S=3, K=2, C=8, L=1,
                         gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_LOGIT, seed=91)
    toks = sorted(np.random.default_rng(5).choice(wl.N, size=12, replace=False).tolist())
    out_steps = [0, 2]
    log, hidden = oracle_block(wl, 0, out_steps, tokens=toks)
    say("max-tokens oracle done; near-ties per step %s, misses per step %s" %
        ([int(r["ambiguous"].sum()) for r in log], [len(r["miss"]) for r in log]))
    sess = _session(wl)
    for forced in (True, False):
        load(sess, wl, 0)
        sess.stats(0, reset=True)
        flips, worst = run_block_on_gpu(wl, 0, sess, log, hidden, forced, out_steps, tokens=toks)
        say("max-tokens forced=%s flips=%d worst=%.2e" % (forced, flips, worst))
    from paper_2605_20179_amd import binding as tb
    with pytest.raises(tb.TideError) as ei:               # one token more is refused when the context is made
        _session(wl.replace(N=65536))
    assert ei.value.code == tb.TIDE_E_RANGE
    sess.close()
