"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the
same seeded inputs.

Bar: top-k indices, hit counts, resident sets, copy plans and miss lists bit-exact
(tokens whose selection scores are within 1e-5 of each other are near-ties: there
fp32 may order differently from fp64; they are counted and reported separately, and
the downstream bit-exact checks are then made on a second run that feeds the oracle's
routing to tide_moe_step_routed); routing weights within 1e-5; outputs within
max-abs 1e-2 x RMS of the oracle output."""
import sys

import numpy as np
import pytest
import torch

import tide_inputs as ti
from oracle import tide_oracle as orc

pytestmark = pytest.mark.gpu

OUT_TOL = 1e-2
W_TOL = 1e-5


def _session(wl, n_layers=1, max_tokens=None, capacity=None):
    from paper_2605_20179_amd.session import TideSession
    return TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C if capacity is None else capacity,
                       wl.N if max_tokens is None else max_tokens, wl.gating, wl.bias_mode, n_layers=n_layers)


def say(msg):
    print("[parity] " + msg, flush=True)
    sys.stdout.flush()


def check_routing(rec, idx, w, k):
    """Exact outside near-ties; inside them any selection that is valid within the band."""
    flips = []
    for n in range(idx.shape[0]):
        if np.array_equal(idx[n], rec["idx"][n]):
            continue
        assert rec["ambiguous"][n], "token %d: selection %s != oracle %s and it is not a near-tie" % (
            n, idx[n], rec["idx"][n])
        key = rec["key"][n]
        ranked = np.sort(key)[::-1]
        got = key[idx[n]]
        assert len(set(idx[n].tolist())) == k
        assert got.min() >= ranked[k - 1] - orc.TIE_EPS
        assert np.all(np.diff(got) <= orc.TIE_EPS)
        must = set(np.nonzero(key > ranked[k - 1] + orc.TIE_EPS)[0].tolist())
        assert must <= set(idx[n].tolist())
        flips.append(n)
    same = np.array([n for n in range(idx.shape[0]) if n not in flips], dtype=np.int64)
    if len(same):
        assert np.abs(w[same] - rec["w"][same]).max() < W_TOL
        assert np.abs(w[same].sum(axis=1) - 1).max() < 1e-5
    return flips


def check_miss(rec_miss, miss, n_miss):
    assert n_miss == len(rec_miss)
    assert [(m[0], m[1]) for m in miss] == [(m[0], m[1]) for m in rec_miss]
    if miss:
        assert max(abs(a[2] - b[2]) for a, b in zip(miss, rec_miss)) < W_TOL


def check_out(out, y_ref, rows=None):
    got = out if rows is None else out[rows]
    rms = float(np.sqrt(np.mean(y_ref ** 2)))
    err = float(np.abs(got - y_ref).max())
    assert rms > 0
    assert err <= OUT_TOL * rms, "max-abs error %.3e exceeds %.0e x RMS (%.3e)" % (err, OUT_TOL, rms)
    return err / rms


def run_block_on_gpu(wl, layer, sess, log, hidden, forced, out_steps, tokens=None):
    """Drive one block in the oracle's order and compare every step.  Returns (flips, worst rel err)."""
    total_flips, worst = 0, 0.0
    exact = True          # unforced run: downstream is bit-exact until the first near-tie flip
    for t, rec in enumerate(log):
        if t > 0 and t % wl.K == 0:
            eis, plan = sess.refresh(layer)
            if exact:
                assert eis.tolist() == rec["expert_in_slot"].tolist(), "step %d: resident set" % t
                assert [(e, s) for e, s, _, _ in plan] == [tuple(p) for p in rec["plan"]], "step %d: plan" % t
                assert all(b == sess.blob_bytes and off == e * sess.blob_bytes for e, s, off, b in plan)
        x = sess.to_device_bf16(hidden[t])
        if forced:
            idx_d = torch.from_numpy(rec["idx"]).to(sess.device)
            w_d = torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device)
            sess.step_routed(layer, x, idx_d, w_d)
            out, _, _, miss, n_miss = sess.results(wl.N)
        else:
            sess.step(layer, x)
            out, idx, w, miss, n_miss = sess.results(wl.N)
            flips = check_routing(rec, idx, w, wl.k)
            if flips:
                say("%s step %d: %d near-tie token(s) selected differently: %s" % (wl.name, t, len(flips), flips))
                total_flips += len(flips)
                exact = False
        if exact:
            check_miss(rec["miss"], miss, n_miss)
            assert np.array_equal(sess.stats(layer), rec["hits"].astype(np.int32)), "step %d: hit counter" % t
            assert np.array_equal(sess.table(layer), rec["slot_of"]), "step %d: table" % t
            if "y_res" in rec and t in out_steps:
                worst = max(worst, check_out(out, rec["y_res"], rows=tokens))
                # the miss pass (weights read in place from pinned host memory) completes the output:
                # resident part + misses == the full MoE layer, whatever the placement (lossless)
                sess.apply_misses(layer, x)
                torch.cuda.synchronize()
                full = sess.out[:wl.N].cpu().numpy()
                worst = max(worst, check_out(full, rec["y_full"], rows=tokens))
                assert np.array_equal(sess.stats(layer), rec["hits"].astype(np.int32)), "miss pass must not count"
        else:
            start = (t // wl.K) * wl.K          # first step of the interval in progress
            assert sess.stats(layer).sum() == sum(int(r["hist"].sum()) for r in log[start:t + 1])
    return total_flips, worst


def oracle_block(wl, layer, out_steps, tokens=None):
    # fp64 copies of the experts the sampled tokens touch, capped at about 4 GB of host memory
    store = orc.ExpertStore(lambda e: ti.expert_weights(wl, layer, e),
                            max_cached=min(wl.E + 1, max(8, int(4e9 // (wl.expert_elems * 8)))))
    shared = tuple(orc.bf16_to_f64(m) for m in ti.expert_weights(wl, layer, wl.E)) if wl.n_shared else None
    hidden = list(ti.hidden_stream(wl, layer))
    log = orc.run_block(hidden, ti.router_weights(wl, layer), ti.router_bias(wl, layer), wl.gating, wl.bias_mode,
                        wl.k, wl.E, wl.C, wl.K, ti.initial_resident(wl), weights=store, shared=shared,
                        output_steps=out_steps, output_tokens=tokens)
    return log, hidden


def load(sess, wl, layer):
    sess.load_layer(layer, lambda e: ti.expert_weights(wl, layer, e), ti.router_weights(wl, layer),
                    ti.router_bias(wl, layer), ti.initial_resident(wl))


# ----------------------------------------------------------------------------- configs 0 and 1
@pytest.mark.parametrize("cfg_id,out_steps", [(0, [0, 1, 2, 3]), (1, [0, 3, 4, 5, 16, 31])])
def test_block_parity(cfg_id, out_steps):
    wl = ti.CONFIGS[cfg_id]
    say("block parity %s" % wl.name)
    log, hidden = oracle_block(wl, 0, out_steps)
    say("oracle done; near-tie tokens per step: %s" % [int(r["ambiguous"].sum()) for r in log])
    for forced in (True, False):
        sess = _session(wl)
        load(sess, wl, 0)
        flips, worst = run_block_on_gpu(wl, 0, sess, log, hidden, forced, out_steps)
        say("%s forced=%s: flips=%d worst out err = %.2e x RMS" % (wl.name, forced, flips, worst))
        # slots hold exactly the host blobs of the experts the table names
        eis = log[-1]["expert_in_slot"]
        for s in (0, wl.C // 2, wl.C - 1):
            if forced or flips == 0:
                assert np.array_equal(sess.read_slot(0, s), sess.host_blobs[0][int(eis[s])].numpy()), "slot %d bytes" % s
        sess.close()


# ----------------------------------------------------------------------------- ragged shapes
RAGGED = [
    # d,  E,  k,  I,  sh, N,   C,  gating, bias_mode
    (128, 24, 3, 192, 1, 37, 5, ti.GATING_SIGMOID, ti.BIAS_LOGIT),
    (64, 7, 2, 64, 0, 1, 3, ti.GATING_SOFTMAX, ti.BIAS_NONE),
    (192, 12, 4, 128, 1, 150, 6, ti.GATING_SIGMOID, ti.BIAS_SELECT),
    (128, 9, 9, 64, 0, 70, 9, ti.GATING_SOFTMAX, ti.BIAS_LOGIT),
    (256, 300, 6, 128, 1, 33, 40, ti.GATING_SIGMOID, ti.BIAS_NONE),
    # steps of >= 256 tokens: the 64-expert x 128-token router kernel with a partial expert group (70 = 64 + 6) and a
    # partial gate/up group (12 column blocks = 8 + 4); its fallback when d is not a multiple of 128; slots with
    # hundreds of rows (large work items of 9..16 token tiles) and a partial down group (20 stripes = 16 + 4)
    (384, 70, 4, 192, 1, 257, 30, ti.GATING_SOFTMAX, ti.BIAS_LOGIT),
    (192, 100, 5, 320, 0, 300, 20, ti.GATING_SIGMOID, ti.BIAS_SELECT),
    (320, 8, 2, 192, 1, 700, 4, ti.GATING_SIGMOID, ti.BIAS_NONE),
    # the largest expert count and top-k the library takes, on the one-workgroup path and on the many-workgroup
    # path, the second with every expert resident
    (128, 512, 16, 64, 1, 20, 100, ti.GATING_SIGMOID, ti.BIAS_LOGIT),
    (128, 512, 16, 64, 0, 90, 512, ti.GATING_SOFTMAX, ti.BIAS_NONE),
]


@pytest.mark.parametrize("shape", RAGGED)
def test_ragged_shapes(shape):
    d, E, k, I, sh, N, C, gating, bias_mode = shape
    wl = ti.TideWorkload("ragged", d=d, E=E, k=k, I=I, n_shared=sh, N=N, S=5, K=2, C=C, L=1, gating=gating,
                         bias_mode=bias_mode, seed=77 + N)
    say("ragged %s" % (shape,))
    log, hidden = oracle_block(wl, 0, [0, 2, 4])
    for forced in (True, False):
        sess = _session(wl)
        load(sess, wl, 0)
        flips, worst = run_block_on_gpu(wl, 0, sess, log, hidden, forced, [0, 2, 4])
        say("ragged forced=%s flips=%d worst=%.2e" % (forced, flips, worst))
        sess.close()


# ----------------------------------------------------------------------------- edge cases
def test_edge_cases_and_errors():
    from paper_2605_20179_amd import binding as tb
    wl = ti.CONFIGS[0]
    say("edge cases")
    log, hidden = oracle_block(wl, 0, [0])
    sess = _session(wl, max_tokens=16)
    # calls before set-up are refused, not run
    with pytest.raises(tb.TideError) as ei:
        sess.step(0, sess.to_device_bf16(hidden[0]))
    assert ei.value.code == tb.TIDE_E_STATE
    load(sess, wl, 0)
    x = sess.to_device_bf16(hidden[0])
    # empty step
    sess.n_miss.fill_(7)
    sess.step(0, x[:0], n_tokens=0)
    torch.cuda.synchronize()
    assert int(sess.n_miss.item()) == 0
    assert sess.stats(0).sum() == 0
    # truncated miss list: count is the full count, entries are the first miss_cap
    sess.step(0, x)
    out, idx, w, miss_full, n_full = sess.results(wl.N)
    check_miss(log[0]["miss"], miss_full, n_full)
    assert n_full >= 2
    sess.miss.fill_(-1)
    sess.stats(0, reset=True)
    sess.step(0, x, miss_cap=1)
    torch.cuda.synchronize()
    assert int(sess.n_miss.item()) == n_full
    raw = sess.miss.cpu().numpy()
    assert raw[0, 0] == miss_full[0][0] and raw[0, 1] == miss_full[0][1] and (raw[1:] == -1).all()
    # run-to-run determinism (bitwise)
    sess.step(0, x)
    out2 = sess.results(wl.N)[0]
    assert np.array_equal(out, out2)
    # fewer tokens than max_tokens, and a one-token step
    sess.stats(0, reset=True)
    sess.step(0, x[:1].contiguous())
    o1 = sess.results(1)[0]
    assert np.array_equal(o1[0], out[0])
    # range / argument errors
    with pytest.raises(tb.TideError) as ei:
        sess.step(0, torch.zeros((17, wl.d), dtype=torch.int16, device=sess.device))
    assert ei.value.code == tb.TIDE_E_RANGE
    with pytest.raises(tb.TideError) as ei:
        sess.refresh(0, capacity=wl.C + 1)
    assert ei.value.code == tb.TIDE_E_RANGE
    with pytest.raises(tb.TideError) as ei:
        tb.tide_set_resident(sess.ctx, 0, [0, 0])
    assert ei.value.code == tb.TIDE_E_INVAL
    with pytest.raises(tb.TideError) as ei:
        tb.tide_set_resident(sess.ctx, 3, [0])
    assert ei.value.code == tb.TIDE_E_INVAL
    with pytest.raises(tb.TideError):
        tb.tide_create(tb.make_config(100, 16, 2, 128, 0, 1, 8, 8, 0, 0))      # d not a multiple of 64
    sess.close()


def test_all_resident_and_none_resident_and_lossless():
    """Capacity = all experts: no misses and out == full MoE output.  One resident expert:
    out + sum over the miss list of w * e(x) (oracle experts) == the same full output."""
    wl = ti.CONFIGS[0]
    say("lossless")
    hidden = list(ti.hidden_stream(wl, 0))
    wr = ti.router_weights(wl, 0)
    store = orc.ExpertStore(lambda e: ti.expert_weights(wl, 0, e))
    idx, w, amb, key = orc.route(hidden[0], wr, None, wl.gating, wl.bias_mode, wl.k)
    all_slots = np.arange(wl.E, dtype=np.int32)
    y_res, y_full, miss = orc.moe_outputs(hidden[0], idx, w, all_slots, store, None)
    sess = _session(wl, capacity=wl.E)
    sess.load_layer(0, lambda e: ti.expert_weights(wl, 0, e), wr, None, list(range(wl.E)))
    x = sess.to_device_bf16(hidden[0])
    sess.step(0, x)
    out, gidx, gw, gmiss, n_miss = sess.results(wl.N)
    assert n_miss == 0 and np.array_equal(gidx, idx)
    check_out(out, y_full)
    # refresh with capacity = E keeps everything resident whatever the counts
    eis, plan = sess.refresh(0)
    assert plan == [] and sorted(eis.tolist()) == list(range(wl.E))
    # shrink to one resident expert (the most hit one), everything else misses
    sess.step(0, x)
    eis, plan = sess.refresh(0, capacity=1)
    hist = orc.step_histogram(idx, wl.E)
    keep = int(np.argmax(hist))
    assert plan == [] and [e for e in eis.tolist() if e >= 0] == [keep]
    sess.step(0, x)
    out, gidx, gw, gmiss, n_miss = sess.results(wl.N)
    xf = orc.bf16_to_f64(hidden[0])
    rebuilt = out.astype(np.float64)
    for (n, e, wt) in gmiss:
        assert e != keep
        rebuilt[n] += wt * orc.expert_ffn(xf[n], *store(e))
    assert n_miss == wl.N * wl.k - hist[keep]
    check_out(rebuilt, y_full)
    sess.close()


def test_refresh_against_oracle_random_counts():
    """tide_refresh with caller-supplied counts, random placements, free slots and shrinking capacity."""
    say("refresh random")
    wl = ti.CONFIGS[0].replace(E=16, C=8)
    sess = _session(wl)
    load(sess, wl, 0)
    g = np.random.default_rng(5)
    eis = np.arange(wl.C, dtype=np.int32)
    for trial in range(40):
        counts = g.integers(0, 5, size=wl.E).astype(np.int32) * (0 if trial % 9 == 8 else 1)
        cap = int(g.integers(0, wl.C + 1)) if trial % 3 == 2 else wl.C
        want_eis, want_plan = orc.refresh(counts, eis, cap)
        got_eis, got_plan = sess.refresh(0, capacity=cap, counts=counts)
        assert got_eis.tolist() == want_eis.tolist(), "trial %d" % trial
        assert [(e, s) for e, s, _, _ in got_plan] == want_plan, "trial %d" % trial
        assert np.array_equal(sess.table(0), orc.slot_table(want_eis, wl.E))
        eis = want_eis
        from paper_2605_20179_amd import binding as tb
        tb.tide_wait_refresh(sess.ctx, 0)
        for s, e in enumerate(eis):
            if e >= 0 and trial % 10 == 0:
                assert np.array_equal(sess.read_slot(0, s), sess.host_blobs[0][int(e)].numpy())
    sess.close()


def test_two_layers_keep_separate_caches_and_counters():
    wl = ti.CONFIGS[0].replace(L=2)
    say("two layers")
    logs = [oracle_block(wl, l, [0, 2, 3]) for l in range(2)]
    sess = _session(wl, n_layers=2)
    for l in range(2):
        load(sess, wl, l)
    for t in range(wl.S):
        for l in range(2):
            log, hidden = logs[l]
            rec = log[t]
            if t > 0 and t % wl.K == 0:
                eis, plan = sess.refresh(l)
                assert eis.tolist() == rec["expert_in_slot"].tolist()
            sess.step(l, sess.to_device_bf16(hidden[t]))
            out, idx, w, miss, n_miss = sess.results(wl.N)
            assert not check_routing(rec, idx, w, wl.k)
            check_miss(rec["miss"], miss, n_miss)
            assert np.array_equal(sess.stats(l), rec["hits"].astype(np.int32))
            if "y_res" in rec:
                check_out(out, rec["y_res"])
    sess.close()


@pytest.mark.parametrize("n_tokens,d_ff", [(24, 128), (600, 1024)])
def test_routed_step_with_an_expert_repeated_inside_a_token(n_tokens, d_ff):
    """tide_moe_step_routed documents distinct expert ids per token; a caller that repeats one still gets every row
    evaluated and both weights applied (the sum the definition gives), hits counted per pair, nothing out of bounds --
    also when the repeats pile more rows onto one slot than the step has tokens (1200 rows of 600 tokens, large work items)."""
    wl = ti.TideWorkload("repeats", d=128, E=12, k=4, I=d_ff, n_shared=1, N=n_tokens, S=1, K=1, C=6, L=1,
                         gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_NONE, seed=808)
    hidden = next(iter(ti.hidden_stream(wl, 0)))
    rng = np.random.default_rng(9)
    idx = rng.integers(0, wl.E, size=(wl.N, wl.k)).astype(np.int32)
    idx[:, 1] = idx[:, 0]                                   # every token names its first expert twice
    idx[: wl.N // 2] = 3                                    # and half of the tokens name one resident expert four times
    w = rng.random((wl.N, wl.k)).astype(np.float32)
    w /= w.sum(axis=1, keepdims=True)
    store = orc.ExpertStore(lambda e: ti.expert_weights(wl, 0, e))
    shared = tuple(orc.bf16_to_f64(m) for m in ti.expert_weights(wl, 0, wl.E))
    slot_of = orc.slot_table(ti.initial_resident(wl), wl.E)
    y_res, y_full, miss = orc.moe_outputs(hidden, idx, w.astype(np.float64), slot_of, store, shared)
    sess = _session(wl)
    load(sess, wl, 0)
    x = sess.to_device_bf16(hidden)
    sess.step_routed(0, x, torch.from_numpy(idx).to(sess.device), torch.from_numpy(w).to(sess.device))
    out, _, _, gmiss, n_miss = sess.results(wl.N)
    check_miss(miss, gmiss, n_miss)
    check_out(out, y_res)
    assert np.array_equal(sess.stats(0), orc.step_histogram(idx, wl.E).astype(np.int32))
    sess.apply_misses(0, x)
    torch.cuda.synchronize()
    check_out(sess.out[:wl.N].cpu().numpy(), y_full)
    sess.close()


@pytest.mark.parametrize("n_tokens,n_experts,k,bias_mode", [(16, 64, 6, ti.BIAS_NONE), (32, 256, 8, ti.BIAS_LOGIT),
                                                             (200, 64, 6, ti.BIAS_SELECT), (90, 300, 16, ti.BIAS_NONE)])
def test_exactly_equal_scores_go_to_the_lower_expert_id(n_tokens, n_experts, k, bias_mode):
    """Experts with identical router rows (and biases) have bit-identical scores for every token: among them the
    selection must take the lower ids first, inside the top-k and at its boundary, and list them in id order --
    the oracle's convention for equal keys.  Covers the one-workgroup path (<= 32 tokens) and the general one,
    both register layouts (E <= 256, E > 256) and the three bias modes."""
    wl = ti.TideWorkload("ties", d=128, E=n_experts, k=k, I=64, n_shared=0, N=n_tokens, S=1, K=1, C=min(8, n_experts),
                         L=1, gating=ti.GATING_SIGMOID, bias_mode=bias_mode, seed=4242 + n_tokens)
    rng = np.random.default_rng(wl.seed)
    wr = ti.router_weights(wl, 0).copy()
    bias = ti.router_bias(wl, 0)
    bias = None if bias is None else bias.copy()
    # families of 2, 3 and 5 identical experts, spread over the id range (different lanes and registers)
    families = []
    free = rng.permutation(n_experts).tolist()
    for size in (2, 3, 5, 2, 3, 2):
        fam = sorted(free.pop() for _ in range(size))
        families.append(fam)
        for e in fam[1:]:
            wr[e] = wr[fam[0]]
            if bias is not None:
                bias[e] = bias[fam[0]]
    # make the families attractive so that they reach the top-k and its boundary often
    for fam in families:
        wr[fam] *= 3.0
    hidden = next(iter(ti.hidden_stream(wl, 0)))
    idx_ref, w_ref, amb, key = orc.route(hidden, wr, bias, wl.gating, wl.bias_mode, wl.k)
    sess = _session(wl)
    sess.load_layer(0, lambda e: ti.expert_weights(wl, 0, e), wr, bias, ti.initial_resident(wl))
    sess.step(0, sess.to_device_bf16(hidden))
    _, idx, w, _, _ = sess.results(wl.N)
    member = {e: f for f, fam in enumerate(families) for e in fam}
    hit_families = 0
    for n in range(wl.N):
        chosen = idx[n].tolist()
        assert len(set(chosen)) == wl.k
        for f, fam in enumerate(families):
            took = [e for e in fam if e in chosen]
            assert took == fam[:len(took)], "token %d: family %s, selected %s" % (n, fam, took)
            pos = [chosen.index(e) for e in took]
            assert pos == list(range(pos[0], pos[0] + len(pos))) if pos else True, "token %d: equal scores out of id order" % n
            hit_families += 0 < len(took) < len(fam)
    assert hit_families > 0, "no family straddles the top-k boundary: the case tests nothing"
    rec = {"idx": idx_ref, "w": w_ref, "ambiguous": amb, "key": key}
    flips = check_routing(rec, idx, w, wl.k)
    say("ties: %d tokens x top-%d of %d, %d family/token pairs cut by the boundary, %d near-tie flips elsewhere"
        % (wl.N, wl.k, wl.E, hit_families, len(flips)))
    sess.close()


@pytest.mark.parametrize("d,n_tokens,large", [(2048, 768, False), (2048, 1024, True), (4096, 512, True), (4096, 256, False)])
def test_where_large_work_items_start(d, n_tokens, large):
    """A step uses large work items from 48 rows per slot on average when the weight rows hold 4096 elements and from
    144 when they are shorter (32 slots here, shared expert included, and 5 rows per token: 40 rows per slot at 256
    tokens, 80 at 512, 120 at 768, 160 at 1024).  Every expert shares one blob: only the split is looked at."""
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    say("large work items at d=%d, %d tokens" % (d, n_tokens))
    E, C, k, I = 64, 31, 4, 512
    wl = ti.TideWorkload("split-%d" % d, d=d, E=E, k=k, I=I, n_shared=1, N=n_tokens, S=1, K=1, C=C, L=1,
                         gating=ti.GATING_SOFTMAX, bias_mode=ti.BIAS_NONE, seed=99)
    sess = TideSession(d, E, k, I, 1, C, n_tokens, wl.gating, wl.bias_mode)
    one = np.empty(sess.blob_bytes, dtype=np.uint8)
    tb.tide_pack_expert(sess.cfg, *ti.expert_weights(wl, 0, 0), one)
    blobs = torch.empty((E, sess.blob_bytes), dtype=torch.uint8, pin_memory=True)
    blobs[:] = torch.from_numpy(one)
    sess.load_layer(0, None, ti.router_weights(wl, 0), None, ti.initial_resident(wl), packed=(blobs, one))
    rng = np.random.default_rng(3)
    # every pair goes to a resident expert: 4 distinct ones per token
    idx = np.stack([rng.choice(C, size=k, replace=False) for _ in range(n_tokens)]).astype(np.int32)
    w = np.full((n_tokens, k), 1.0 / k, dtype=np.float32)
    x = sess.to_device_bf16(next(iter(ti.hidden_stream(wl, 0))))
    sess.step_routed(0, x, torch.from_numpy(idx).to(sess.device), torch.from_numpy(w).to(sess.device))
    items, _ = tb.tide_read_work_items(sess.ctx, 4096, 65536, torch.cuda.current_stream())
    kinds = {int(it["kind"]) for it in items}
    rows = sum(int(it["nrows"]) for it in items)
    assert rows == n_tokens * (k + 1)
    if large:
        assert 1 in kinds, "no large work items"
        assert all(int(it["nrows"]) > 32 for it in items if it["kind"] == 1)
    else:
        assert kinds == {0}, "large work items in a step with few rows per slot"
    sess.close()
