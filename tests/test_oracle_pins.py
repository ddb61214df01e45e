"""Pins for the CPU oracle: every check compares it with something that is not
the oracle itself -- hand-worked fixtures, closed forms, library routines used
differently, brute force, or invariants the paper states (lossless placement,
refresh = top-B by hits, skipped steps do nothing, hits = tokens per expert)."""
import itertools
import json
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

import tide_inputs as ti
from oracle import tide_oracle as orc

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "handworked.json")))


# ------------------------------------------------------------------ formats
def test_bf16_roundtrip_and_rounding_match_torch():
    g = np.random.default_rng(1)
    x32 = (g.standard_normal(200000) * np.exp(g.uniform(-20, 20, 200000))).astype(np.float32)
    want = torch.from_numpy(x32).to(torch.bfloat16).to(torch.float64).numpy()   # fp32 -> bf16 RNE by torch
    got = orc.round_to_bf16(x32.astype(np.float64))
    assert np.array_equal(want, got)
    # exact halfway cases go to even
    half_up = np.float64(1.0 + 2.0 ** -8)            # between 1.0 and 1+2^-7 -> even is 1.0
    assert orc.round_to_bf16(np.array([half_up]))[0] == 1.0
    half_up2 = np.float64(1.0 + 3 * 2.0 ** -8)       # between 1+2^-7 and 1+2^-6 -> even is 1+2^-6
    assert orc.round_to_bf16(np.array([half_up2]))[0] == 1.0 + 2.0 ** -6
    bits = ti.f32_to_bf16_bits(x32)
    assert np.array_equal(orc.bf16_to_f64(bits), want)
    assert np.array_equal(ti.bf16_bits_to_f32(bits).astype(np.float64), want)


# ------------------------------------------------------------------ routing
def test_handworked_softmax_and_sigmoid_routes():
    fx = GOLD["softmax_route"]
    z = np.log(np.array([fx["logit_exp"]], dtype=np.float64))
    sel, score, key = orc.gate(z, None, orc.GATING_SOFTMAX, orc.BIAS_NONE)
    idx, w, amb = orc.topk_route(sel, score, key, fx["k"])
    assert idx[0].tolist() == fx["idx"]
    assert np.allclose(w[0], fx["w"], rtol=0, atol=1e-15)
    fx = GOLD["sigmoid_route"]
    z = np.log(np.array([fx["odds"]], dtype=np.float64))
    sel, score, key = orc.gate(z, None, orc.GATING_SIGMOID, orc.BIAS_NONE)
    idx, w, amb = orc.topk_route(sel, score, key, fx["k"])
    assert idx[0].tolist() == fx["idx"]
    assert np.allclose(w[0], fx["w"], rtol=0, atol=1e-15)
    assert not amb[0]


def test_router_logits_are_a_plain_dot_product():
    g = np.random.default_rng(2)
    x = ti.f32_to_bf16_bits(g.standard_normal((5, 7)).astype(np.float32))
    wr = g.standard_normal((3, 7)).astype(np.float32)
    b = g.standard_normal(3).astype(np.float32)
    z = orc.router_logits(x, wr, b, orc.BIAS_LOGIT)
    xf = ti.bf16_bits_to_f32(x)
    for n in range(5):
        for e in range(3):
            ref = math.fsum(float(xf[n, j]) * float(wr[e, j]) for j in range(7)) + float(b[e])
            assert abs(z[n, e] - ref) < 1e-12
    # a transposed router or a missing bias must show
    z0 = orc.router_logits(x, wr, b, orc.BIAS_NONE)
    assert np.allclose(z - z0, b[None, :].astype(np.float64))


@pytest.mark.parametrize("gating", [orc.GATING_SOFTMAX, orc.GATING_SIGMOID])
@pytest.mark.parametrize("bias_mode", [orc.BIAS_NONE, orc.BIAS_LOGIT, orc.BIAS_SELECT])
def test_topk_brute_force_and_weight_closed_forms(gating, bias_mode):
    g = np.random.default_rng(3 + gating * 10 + bias_mode)
    for E, k in [(4, 1), (5, 2), (8, 3), (16, 2), (16, 16), (37, 8)]:
        z = g.standard_normal((40, E)) * 1.5
        b = g.standard_normal(E) * 0.5
        zz = z + b[None, :] if bias_mode == orc.BIAS_LOGIT else z
        sel, score, key = orc.gate(zz, b, gating, bias_mode)
        idx, w, amb = orc.topk_route(sel, score, key, k)
        for n in range(z.shape[0]):
            # brute force: a full stable sort of (-sel, index)
            order = sorted(range(E), key=lambda e: (-sel[n, e], e))[:k]
            assert idx[n].tolist() == order
            assert abs(w[n].sum() - 1.0) < 1e-12
            assert len(set(idx[n].tolist())) == k
        # closed forms for the weights, by library routines
        if gating == orc.GATING_SOFTMAX:
            # softmax over E renormalised over the k selected == softmax over the selected logits
            for n in range(z.shape[0]):
                ref = scipy.special.softmax(zz[n, idx[n]])
                assert np.allclose(w[n], ref, atol=1e-12)
            assert np.allclose(score, scipy.special.softmax(zz, axis=1), atol=1e-14)
        else:
            s = scipy.special.expit(zz)
            assert np.allclose(score, s, atol=1e-15)
            for n in range(z.shape[0]):
                ref = s[n, idx[n]] / s[n, idx[n]].sum()
                assert np.allclose(w[n], ref, atol=1e-12)
        if bias_mode == orc.BIAS_SELECT:
            assert np.allclose(sel, score + b[None, :])


def test_topk_exhaustive_small():
    # every ordering of 5 distinct scores and every k
    vals = np.array([0.1, 0.2, 0.3, 0.4, 0.5])
    for perm in itertools.permutations(range(5)):
        sel = vals[list(perm)][None, :]
        for k in range(1, 6):
            idx, w, amb = orc.topk_route(sel, sel, sel, k)
            want = sorted(range(5), key=lambda e: -sel[0, e])[:k]
            assert idx[0].tolist() == want


def test_topk_ties_prefer_lower_index_and_are_flagged():
    sel = np.array([[0.3, 0.7, 0.7, 0.1, 0.7]])
    idx, w, amb = orc.topk_route(sel, sel, sel, 2)
    assert idx[0].tolist() == [1, 2]
    assert amb[0]
    sel = np.array([[0.3, 0.7, 0.5, 0.1, 0.5 + 5e-6]])   # k-th and (k+1)-th closer than the tie band
    idx, w, amb = orc.topk_route(sel, sel, sel, 2)
    assert idx[0].tolist() == [1, 4] and amb[0]
    sel = np.array([[0.3, 0.7, 0.5, 0.1, 0.6]])
    idx, w, amb = orc.topk_route(sel, sel, sel, 2)
    assert idx[0].tolist() == [1, 4] and not amb[0]


# ------------------------------------------------------------------ counter
def test_histogram_is_bincount_and_sums_to_pairs():
    g = np.random.default_rng(5)
    idx = g.integers(0, 16, size=(33, 4)).astype(np.int32)
    h = orc.step_histogram(idx, 16)
    assert np.array_equal(h, np.bincount(idx.ravel(), minlength=16))
    assert h.sum() == idx.size


# ------------------------------------------------------------------ experts
def test_handworked_swiglu_expert():
    fx = GOLD["swiglu_expert"]
    L = math.log(3.0)
    y = orc.expert_ffn(np.array([L, -L]), np.array(fx["wg"], float), np.array(fx["wu"], float),
                       np.array(fx["wd"], float), act_bf16=False)
    assert np.allclose(y, np.array(fx["y_over_ln3_squared"]) * L * L, atol=1e-14)


def _tiny_layer(seed, d=24, I=12, E=6, N=7):
    g = np.random.default_rng(seed)
    bits = lambda a: ti.f32_to_bf16_bits(a.astype(np.float32))
    experts = [(bits(g.standard_normal((I, d)) * 0.3), bits(g.standard_normal((I, d)) * 0.3),
                bits(g.standard_normal((d, I)) * 0.3)) for _ in range(E + 1)]
    x = bits(g.standard_normal((N, d)))
    wr = (g.standard_normal((E, d)) * 0.3).astype(np.float32)
    b = (g.standard_normal(E) * 0.2).astype(np.float32)
    return experts, x, wr, b


def _torch_expert(X, wg, wu, wd, act_bf16):
    G = X @ wg.T
    U = X @ wu.T
    A = torch.nn.functional.silu(G) * U
    if act_bf16:
        A = A.to(torch.float32).to(torch.bfloat16).to(torch.float64)
    return A @ wd.T


@pytest.mark.parametrize("gating,bias_mode", [(orc.GATING_SOFTMAX, orc.BIAS_NONE), (orc.GATING_SIGMOID, orc.BIAS_LOGIT),
                                              (orc.GATING_SIGMOID, orc.BIAS_SELECT)])
def test_full_output_equals_dense_masked_sum_in_torch(gating, bias_mode):
    """y_full == sum over ALL experts of mask[n,e] * w[n,e] * e(x_n), written as a
    dense batched computation in torch fp64 (independent of the oracle's loops)."""
    E, k = 6, 3
    experts, x, wr, b = _tiny_layer(11)
    idx, w, amb, key = orc.route(x, wr, b, gating, bias_mode, k)
    store = orc.ExpertStore(lambda e: experts[e])
    slot_of = np.full(E, -1, dtype=np.int32)
    slot_of[[1, 4]] = [0, 1]
    shared = tuple(orc.bf16_to_f64(m) for m in experts[E])
    y_res, y_full, miss = orc.moe_outputs(x, idx, w, slot_of, store, shared, act_bf16=False)

    X = torch.from_numpy(ti.bf16_bits_to_f32(x)).double()
    tw = lambda e: [torch.from_numpy(ti.bf16_bits_to_f32(m)).double() for m in experts[e]]
    dense_w = torch.zeros(X.shape[0], E, dtype=torch.float64)
    dense_w.scatter_(1, torch.from_numpy(idx.astype(np.int64)), torch.from_numpy(w))
    full = _torch_expert(X, *tw(E), act_bf16=False)
    res = full.clone()
    for e in range(E):
        ye = _torch_expert(X, *tw(e), act_bf16=False)
        full += dense_w[:, e:e + 1] * ye
        if slot_of[e] >= 0:
            res += dense_w[:, e:e + 1] * ye
    assert np.allclose(y_full, full.numpy(), rtol=1e-12, atol=1e-12)
    assert np.allclose(y_res, res.numpy(), rtol=1e-12, atol=1e-12)


def test_bf16_activation_variant_matches_torch_rounding():
    E, k = 6, 2
    experts, x, wr, b = _tiny_layer(12)
    idx, w, amb, key = orc.route(x, wr, None, orc.GATING_SOFTMAX, orc.BIAS_NONE, k)
    store = orc.ExpertStore(lambda e: experts[e])
    slot_of = np.arange(E, dtype=np.int32)
    y_res, y_full, miss = orc.moe_outputs(x, idx, w, slot_of, store, None, act_bf16=True)
    X = torch.from_numpy(ti.bf16_bits_to_f32(x)).double()
    ref = torch.zeros_like(X)
    for e in range(E):
        wts = [torch.from_numpy(ti.bf16_bits_to_f32(m)).double() for m in experts[e]]
        ye = _torch_expert(X, *wts, act_bf16=True)
        for n in range(X.shape[0]):
            for i in range(k):
                if idx[n, i] == e:
                    ref[n] += w[n, i] * ye[n]
    # torch rounds via fp32 (double rounding can differ by one bf16 ulp on rare halfway cases)
    assert np.allclose(y_res, ref.numpy(), rtol=0, atol=2e-3 * np.abs(ref.numpy()).max())
    assert miss == []
    assert np.array_equal(y_res, y_full)


def test_lossless_for_every_resident_set():
    """Placement never changes the result: y_res + sum over misses of w*e(x) == y_full,
    for every resident set including none and all (Sec. 3.3 'Lossless Inference')."""
    E, k = 6, 3
    experts, x, wr, b = _tiny_layer(13)
    idx, w, amb, key = orc.route(x, wr, b, orc.GATING_SIGMOID, orc.BIAS_LOGIT, k)
    store = orc.ExpertStore(lambda e: experts[e])
    shared = tuple(orc.bf16_to_f64(m) for m in experts[E])
    xf = orc.bf16_to_f64(x)
    full_ref = None
    for r in range(E + 1):
        for res in itertools.combinations(range(E), r):
            slot_of = np.full(E, -1, dtype=np.int32)
            for s, e in enumerate(res):
                slot_of[e] = s
            y_res, y_full, miss = orc.moe_outputs(x, idx, w, slot_of, store, shared)
            rebuilt = y_res.copy()
            for (n, e, wt) in miss:
                rebuilt[n] += wt * orc.expert_ffn(xf[n], *store(e))
            assert np.allclose(rebuilt, y_full, rtol=1e-12, atol=1e-13)
            if full_ref is None:
                full_ref = y_full
            assert np.array_equal(full_ref, y_full)
            # miss list: partition of the pairs, canonical order
            n_hit = sum(1 for n in range(idx.shape[0]) for i in range(k) if slot_of[idx[n, i]] >= 0)
            assert n_hit + len(miss) == idx.size
            assert miss == sorted(miss, key=lambda m: (m[0], list(idx[m[0]]).index(m[1])))
            if r == E:
                assert miss == []
            if r == 0:
                assert len(miss) == idx.size


def test_all_experts_uniform_weights_is_the_mean_of_experts():
    E = 5
    experts, x, wr, b = _tiny_layer(14, E=E)
    store = orc.ExpertStore(lambda e: experts[e])
    idx = np.tile(np.arange(E, dtype=np.int32), (x.shape[0], 1))
    w = np.full(idx.shape, 1.0 / E)
    y_res, y_full, miss = orc.moe_outputs(x, idx, w, np.arange(E, dtype=np.int32), store, None)
    xf = orc.bf16_to_f64(x)
    mean = np.mean([[orc.expert_ffn(xf[n], *store(e)) for e in range(E)] for n in range(x.shape[0])], axis=1)
    assert np.allclose(y_res, mean, rtol=1e-12, atol=1e-14)


def test_sampled_tokens_equal_full_rows():
    E, k = 6, 2
    experts, x, wr, b = _tiny_layer(15)
    idx, w, amb, key = orc.route(x, wr, b, orc.GATING_SIGMOID, orc.BIAS_LOGIT, k)
    store = orc.ExpertStore(lambda e: experts[e])
    slot_of = np.array([0, -1, 1, -1, 2, -1], dtype=np.int32)
    a = orc.moe_outputs(x, idx, w, slot_of, store, None)
    b2 = orc.moe_outputs(x, idx, w, slot_of, store, None, tokens=[5, 2])
    assert np.array_equal(a[0][[5, 2]], b2[0]) and np.array_equal(a[1][[5, 2]], b2[1]) and a[2] == b2[2]


# ------------------------------------------------------------------ refresh
def test_handworked_refresh():
    for name in ("refresh", "refresh_two_swaps"):
        fx = GOLD[name]
        eis, plan = orc.refresh(np.array(fx["hits"]), np.array(fx["expert_in_slot"], dtype=np.int32), fx["capacity"])
        assert eis.tolist() == fx["new_expert_in_slot"], name
        assert [list(p) for p in plan] == fx["plan"], name


def _literal_swap_rule(hits, resident):
    """The refresh step as Alg. 1 words it: line up the most-hit CPU experts against
    the least-hit GPU experts and swap a pair while the CPU one has strictly more hits."""
    E = len(hits)
    cpu = sorted((e for e in range(E) if e not in resident), key=lambda e: (-hits[e], e))
    # equal-hit ties are this build's convention (lower index is kept); the paper is silent on them
    gpu = sorted(resident, key=lambda e: (hits[e], -e))
    res = set(resident)
    for c, gp in zip(cpu, gpu):
        if hits[c] > hits[gp]:
            res.remove(gp)
            res.add(c)
        else:
            break
    return res


def test_refresh_brute_force_properties():
    g = np.random.default_rng(21)
    for trial in range(300):
        E = int(g.integers(2, 24))
        C = int(g.integers(1, E + 1))
        hits = g.integers(0, 6, size=E) * int(g.integers(0, 2) if trial % 7 == 0 else 1)
        eis = g.permutation(E)[:C].astype(np.int32)
        new, plan = orc.refresh(hits, eis, C)
        old_set, new_set = set(eis.tolist()), set(new.tolist())
        assert len(new_set) == C and -1 not in new_set
        # a top-C set: the multiset of resident hit counts is the C largest
        assert sorted((int(hits[e]) for e in new_set), reverse=True) == sorted(map(int, hits), reverse=True)[:C]
        # same set as the literal pairwise swap rule
        assert new_set == _literal_swap_rule(hits, old_set)
        # minimal number of copies, one per newcomer, bijection onto freed slots
        assert len(plan) == len(new_set - old_set)
        assert {e for e, s in plan} == new_set - old_set
        freed = {s for s in range(C) if eis[s] not in new_set}
        assert {s for e, s in plan} == freed
        for s in range(C):
            if eis[s] in new_set:
                assert new[s] == eis[s]            # survivors never move
        for e, s in plan:
            assert new[s] == e
        # newcomers strictly out-hit everyone they displace
        if plan:
            assert min(int(hits[e]) for e, s in plan) > max(int(hits[eis[s]]) for e, s in plan)
        if not hits.any():
            assert plan == [] and np.array_equal(new, eis)
        # capacity == all experts -> everything resident whatever the counts
    hits = g.integers(0, 9, size=10)
    new, plan = orc.refresh(hits, np.arange(10, dtype=np.int32), 10)
    assert plan == [] and sorted(new.tolist()) == list(range(10))


def test_refresh_with_free_slots_and_smaller_capacity():
    hits = np.array([4, 0, 9, 1, 7, 3])
    eis = np.array([0, -1, 3, -1], dtype=np.int32)
    new, plan = orc.refresh(hits, eis, 4)           # top-4: e2, e4, e0, e5 ; e3 leaves slot 2
    assert set(new.tolist()) == {2, 4, 0, 5}
    assert plan == [(2, 2), (4, 1), (5, 3)]
    new2, plan2 = orc.refresh(hits, new, 2)         # shrink to 2: e2, e4 stay, others leave, no copies
    assert plan2 == [] and sorted(e for e in new2.tolist() if e >= 0) == [2, 4]
    assert (new2 == -1).sum() == 2


def test_run_block_schedule_invariants():
    wl = ti.CONFIGS[0]
    wr = ti.router_weights(wl, 0)
    log = orc.run_block(ti.hidden_stream(wl, 0), wr, None, wl.gating, wl.bias_mode, wl.k, wl.E, wl.C, wl.K,
                        ti.initial_resident(wl))
    assert len(log) == wl.S
    running = np.zeros(wl.E, dtype=np.int64)
    for r in log:
        t = r["t"]
        assert r["hist"].sum() == wl.N * wl.k
        if t > 0 and t % wl.K == 0:
            assert r["plan"] is not None
            assert np.array_equal(r["hits_at_refresh"], running)      # hits of the interval just ended
            running[:] = 0
        else:
            assert r["plan"] is None                                  # skipped steps migrate nothing
            if t > 0:
                assert np.array_equal(r["expert_in_slot"], log[t - 1]["expert_in_slot"])
        running += r["hist"]
        assert np.array_equal(r["hits"], running)
        assert np.allclose(r["w"].sum(axis=1), 1.0, atol=1e-12)
    # interval 1 with capacity = all experts: the resident set is all experts at every step
    log = orc.run_block(ti.hidden_stream(wl, 0), wr, None, wl.gating, wl.bias_mode, wl.k, wl.E, wl.E, 1,
                        np.arange(wl.E, dtype=np.int32))
    for r in log:
        assert sorted(r["expert_in_slot"].tolist()) == list(range(wl.E)) and r["miss"] == []
        assert r["plan"] in (None, [])
    # interval 1: placement at step t is a top-C set of step t-1's histogram
    log = orc.run_block(ti.hidden_stream(wl, 0), wr, None, wl.gating, wl.bias_mode, wl.k, wl.E, wl.C, 1,
                        ti.initial_resident(wl))
    for t in range(1, wl.S):
        prev = log[t - 1]["hist"]
        res = [e for e in log[t]["expert_in_slot"] if e >= 0]
        assert sorted((int(prev[e]) for e in res), reverse=True) == sorted(map(int, prev), reverse=True)[:wl.C]


def test_config0_end_to_end_outputs_and_lossless():
    wl = ti.CONFIGS[0]
    wr = ti.router_weights(wl, 0)
    store = orc.ExpertStore(lambda e: ti.expert_weights(wl, 0, e))
    log = orc.run_block(ti.hidden_stream(wl, 0), wr, None, wl.gating, wl.bias_mode, wl.k, wl.E, wl.C, wl.K,
                        ti.initial_resident(wl), weights=store, shared=None)
    hidden = list(ti.hidden_stream(wl, 0))
    for r in log:
        xf = orc.bf16_to_f64(hidden[r["t"]])
        rebuilt = r["y_res"].copy()
        for (n, e, wt) in r["miss"]:
            rebuilt[n] += wt * orc.expert_ffn(xf[n], *store(e))
        assert np.allclose(rebuilt, r["y_full"], rtol=1e-12, atol=1e-15)
        assert np.isfinite(r["y_full"]).all() and np.abs(r["y_full"]).max() > 0


# ------------------------------------------------------------------ inputs
def test_inputs_are_seeded_and_shaped():
    wl = ti.CONFIGS[1]
    a = ti.router_weights(wl, 0)
    assert a.shape == (256, 2048) and a.dtype == np.float32 and np.array_equal(a, ti.router_weights(wl, 0))
    assert abs(a.std() - 0.02) < 1e-3
    b = ti.router_bias(wl, 0)
    assert b.shape == (256,) and b.max() == 0.0 and np.isclose(b.min(), -0.25 * 1.1 * math.log(256), rtol=1e-6)
    wl0 = ti.CONFIGS[0]
    wg, wu, wd = ti.expert_weights(wl0, 0, 3)
    assert wg.shape == (128, 256) and wd.shape == (256, 128) and wg.dtype == np.uint16
    assert not np.array_equal(wg, wu)
    assert np.array_equal(wg, ti.expert_weights(wl0, 0, 3)[0])
    hs = list(ti.hidden_stream(wl0, 0))
    assert len(hs) == 4 and hs[0].shape == (8, 256)
    h0, h1 = ti.bf16_bits_to_f32(hs[0]), ti.bf16_bits_to_f32(hs[1])
    # drift keeps neighbouring steps close
    cos = (h0 * h1).sum() / np.linalg.norm(h0) / np.linalg.norm(h1)
    assert cos > 0.99


# ------------------------------------------------------------------ placement policies
def _policy_inputs(steps=12):
    wl = ti.CONFIGS[0].replace(S=steps)
    hidden = list(ti.hidden_stream(wl, 0))
    args = (hidden, ti.router_weights(wl, 0), ti.router_bias(wl, 0), wl.gating, wl.bias_mode, wl.k, wl.E, wl.C,
            ti.initial_resident(wl))
    return wl, hidden, args


def test_policy_interval_equals_alg1_driver_and_static_never_moves():
    wl, hidden, args = _policy_inputs()
    for K in (1, 2, 5):
        log, _, _ = orc.run_block_policy(*args, interval=K)
        ref = orc.run_block(hidden, *args[1:8], K, args[8])
        for a, b in zip(log, ref):
            assert a["expert_in_slot"].tolist() == b["expert_in_slot"].tolist() and a["plan"] == b["plan"]
            assert np.array_equal(a["hits"], b["hits"]) and a["miss"] == b["miss"]
    log, eis, hits = orc.run_block_policy(*args, interval=None)
    assert all(r["plan"] is None and r["expert_in_slot"].tolist() == list(args[8]) for r in log)
    assert np.array_equal(hits, sum(r["hist"] for r in log))


def test_policy_counters_follow_their_definitions():
    wl, hidden, args = _policy_inputs()
    hists = [orc.step_histogram(orc.route(h, *args[1:6])[0], wl.E) for h in hidden]
    K = 3
    log, _, _ = orc.run_block_policy(*args, interval=K, counter="cumulative")
    for t, r in enumerate(log):
        assert np.array_equal(r["hits"], sum(hists[:t + 1]))
        if t > 0 and t % K == 0:                      # placement = top-C of everything seen so far
            assert set(r["expert_in_slot"].tolist()) == set(orc.refresh(sum(hists[:t]), log[t - 1]["expert_in_slot"], wl.C)[0].tolist())
    log, _, _ = orc.run_block_policy(*args, interval=K, counter="decay", decay=(1, 2))
    h = np.zeros(wl.E, dtype=np.int64)
    for t, r in enumerate(log):
        if t > 0 and t % K == 0:
            h = h // 2
        h = h + hists[t]
        assert np.array_equal(r["hits"], h)
    with pytest.raises(ValueError):
        orc.run_block_policy(*args, interval=K, counter="nonsense")


def test_policy_warm_start_and_carry_over():
    wl, hidden, args = _policy_inputs()
    hist0 = orc.step_histogram(orc.route(hidden[0], *args[1:6])[0], wl.E)
    log, _, _ = orc.run_block_policy(*args, interval=4, warm_start=True)
    want, plan = orc.refresh(hist0, np.asarray(args[8]), wl.C)
    assert log[0]["expert_in_slot"].tolist() == want.tolist() and log[0]["plan"] == plan
    assert np.array_equal(log[0]["hits"], hist0)       # counted once into the interval that starts at step 0
    # the warm placement holds step 0's most-hit experts: no other set of C experts has fewer misses at step 0
    served = sum(int(hist0[e]) for e in want if e >= 0)
    assert served == int(np.sort(hist0)[::-1][:wl.C].sum())
    # two blocks with carry-over == one run over the concatenated steps when the first block's length is a
    # multiple of the interval (the second block's step 0 is then a refresh step of the long run)
    first, eis, hits = orc.run_block_policy(*args, interval=4, counter="cumulative")
    second, _, _ = orc.run_block_policy(hidden, *args[1:8], eis, interval=4, counter="cumulative", initial_hits=hits)
    long_log, _, _ = orc.run_block_policy(hidden + hidden, *args[1:], interval=4, counter="cumulative")
    for a, b in zip(second[1:], long_log[len(hidden) + 1:]):
        assert np.array_equal(a["hits"], b["hits"])
    assert np.array_equal(second[0]["hits"], long_log[len(hidden)]["hits"])


def test_policy_deferred_refresh_is_the_same_choice_one_step_late():
    wl, hidden, args = _policy_inputs()
    for K in (1, 2, 4):
        now, _, _ = orc.run_block_policy(*args, interval=K)
        late, _, _ = orc.run_block_policy(*args, interval=K, deferred=True)
        for t, (a, b) in enumerate(zip(now, late)):
            assert a["plan"] == b["plan"] and np.array_equal(a["hits"], b["hits"])
            if t > 0 and t % K == 0:
                assert b["expert_in_slot"].tolist() == now[t - 1]["expert_in_slot"].tolist()
                assert b["pending_expert_in_slot"].tolist() == a["expert_in_slot"].tolist()
            else:
                assert b["expert_in_slot"].tolist() == a["expert_in_slot"].tolist()
            # the miss list is the split against the placement in force, stated directly
            live = set(int(e) for e in b["expert_in_slot"] if e >= 0)
            assert b["miss"] == [(n, int(b["idx"][n, i]), float(b["w"][n, i])) for n in range(b["idx"].shape[0])
                                 for i in range(wl.k) if int(b["idx"][n, i]) not in live]
    # a longer delay: the same choices, each serving j steps late
    now, _, _ = orc.run_block_policy(*args, interval=4)
    late, _, _ = orc.run_block_policy(*args, interval=4, deferred=3)
    for t, (a, b) in enumerate(zip(now, late)):
        assert a["plan"] == b["plan"] and np.array_equal(a["hits"], b["hits"])
        src = t if (t < 4 or t % 4 == 3) else (t // 4) * 4 - 1       # steps 4k..4k+2 still run on the placement of step 4k-1
        assert b["expert_in_slot"].tolist() == now[src]["expert_in_slot"].tolist(), t
    with pytest.raises(ValueError):
        orc.run_block_policy(*args, interval=4, warm_start=True, deferred=True)
    with pytest.raises(ValueError):
        orc.run_block_policy(*args, interval=4, deferred=5)
