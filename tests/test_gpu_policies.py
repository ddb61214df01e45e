"""Placement policies driven through the same C ABI (Sec. 4's static and every-step baselines as policy
settings; counters that outlive an interval or a block; warm start; other budgets and block lengths),
each compared step by step with the oracle's policy driver: counter, placement table, copy plan and
miss list bit-exact.  Token routing is forced to the oracle's so that every comparison is exact (the
router itself is compared in test_gpu_parity / test_gpu_configs).  Expert outputs do not depend on the
policy beyond the placement, which test_all_resident_and_none_resident_and_lossless covers."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
from oracle import tide_oracle as orc
from paper_2605_20179_amd import binding as tb
from test_gpu_parity import _session, check_miss, load, say

pytestmark = pytest.mark.gpu


def drive(sess, wl, hidden, log, interval, counter, decay, warm_start, first_t0_refresh=False):
    """The policy in library calls; returns (misses, migrated experts)."""
    misses = migrated = 0

    def refresh_and_check(rec):
        eis, plan = sess.refresh(0, reset_counts=(counter == "interval"))
        if counter == "decay":
            tb.tide_scale_counts(sess.ctx, 0, decay[0], decay[1], torch.cuda.current_stream())
        assert eis.tolist() == rec["expert_in_slot"].tolist(), "step %d: resident set" % rec["t"]
        assert [(e, s) for e, s, _, _ in plan] == [tuple(p) for p in rec["plan"]], "step %d: plan" % rec["t"]
        return len(plan)

    for t, rec in enumerate(log):
        x = sess.to_device_bf16(hidden[t])
        idx_d = torch.from_numpy(rec["idx"]).to(sess.device)
        w_d = torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device)
        if t == 0 and warm_start:
            sess.step_routed(0, x, idx_d, w_d)            # counts step 0 on the cold placement
            migrated += refresh_and_check(rec)
        elif interval is not None and t > 0 and t % interval == 0:
            migrated += refresh_and_check(rec)
        sess.step_routed(0, x, idx_d, w_d)
        _, _, _, miss, n_miss = sess.results(wl.N)
        check_miss(rec["miss"], miss, n_miss)
        misses += n_miss
        assert np.array_equal(sess.table(0), rec["slot_of"]), "step %d: table" % t
        assert np.array_equal(sess.stats(0), rec["hits"].astype(np.int32)), "step %d: counter" % t
    return misses, migrated


POLICIES = [
    ("alg1 tau=4", dict(interval=4, counter="interval")),
    ("static (never refresh)", dict(interval=None, counter="interval")),
    ("every step (tau=1)", dict(interval=1, counter="interval")),
    ("cumulative counter tau=4", dict(interval=4, counter="cumulative")),
    ("decayed counter 1/2 tau=4", dict(interval=4, counter="decay", decay=(1, 2))),
    ("decayed counter 3/4 tau=2", dict(interval=2, counter="decay", decay=(3, 4))),
    ("warm start tau=4", dict(interval=4, counter="interval", warm_start=True)),
]


def test_policies_on_the_headline_layer():
    wl = ti.CONFIGS[1]
    hidden = list(ti.hidden_stream(wl, 0))
    args = (hidden, ti.router_weights(wl, 0), ti.router_bias(wl, 0), wl.gating, wl.bias_mode, wl.k, wl.E, wl.C,
            ti.initial_resident(wl))
    sess = _session(wl)
    load(sess, wl, 0)
    pairs = len(hidden) * wl.N * wl.k
    for name, pol in POLICIES:
        kw = dict(interval=pol["interval"], counter=pol["counter"], decay=pol.get("decay", (1, 2)),
                  warm_start=pol.get("warm_start", False))
        log, _, _ = orc.run_block_policy(*args, **kw)
        tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
        sess.stats(0, reset=True)
        misses, migrated = drive(sess, wl, hidden, log, **kw)
        assert misses == sum(len(r["miss"]) for r in log)
        say("policy %-28s miss rate %.4f, experts migrated %d" % (name, misses / pairs, migrated))
    # carry-over across blocks: the second block starts from the first one's placement and counter
    first, eis, hits = orc.run_block_policy(*args, interval=4, counter="cumulative")
    second, _, _ = orc.run_block_policy(hidden, *args[1:8], eis, interval=4, counter="cumulative", initial_hits=hits)
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    sess.stats(0, reset=True)
    drive(sess, wl, hidden, first, 4, "cumulative", (1, 2), False)
    m2, g2 = drive(sess, wl, hidden, second, 4, "cumulative", (1, 2), False)
    say("second block with carried-over counter: miss rate %.4f, experts migrated %d" % (m2 / pairs, g2))
    with pytest.raises(tb.TideError):
        tb.tide_scale_counts(sess.ctx, 0, 3, 2)
    with pytest.raises(tb.TideError):
        tb.tide_scale_counts(sess.ctx, 1, 1, 2)
    sess.close()


@pytest.mark.parametrize("budget,block", [(32, 32), (128, 32), (64, 64), (64, 128), (128, 128)])
def test_other_budgets_and_block_lengths(budget, block):
    """Table 2 / Fig. 5 vary the GPU expert budget (32, 64, 128) and the block length (32, 64, 128)."""
    wl = ti.CONFIGS[1].replace(C=budget, N=block, S=9)
    hidden = list(ti.hidden_stream(wl, 0))
    args = (hidden, ti.router_weights(wl, 0), ti.router_bias(wl, 0), wl.gating, wl.bias_mode, wl.k, wl.E, wl.C,
            ti.initial_resident(wl))
    log, _, _ = orc.run_block_policy(*args, interval=wl.K)
    sess = _session(wl)
    load(sess, wl, 0)
    misses, migrated = drive(sess, wl, hidden, log, wl.K, "interval", (1, 2), False)
    say("budget %d block %d: miss rate %.4f, experts migrated %d" % (budget, block, misses / (len(hidden) * wl.N * wl.k), migrated))
    sess.close()


@pytest.mark.parametrize("engine", [tb.TIDE_COPY_KERNEL, tb.TIDE_COPY_DMA], ids=["copy-kernel", "dma"])
def test_deferred_refresh_and_commit(engine):
    """Both copy engines (the side-stream copy kernel; one DMA transfer per entering expert).  The overlapped variant: the refresh before step t only stages its newcomers; step t runs on the old
    placement; tide_commit installs the new one before step t+1 (or, called later, before step t+j).  Counter, tables, plans, miss lists and the
    bytes of every cache slot are compared with the oracle's delayed placement."""
    wl = ti.CONFIGS[1].replace(S=14)
    hidden = list(ti.hidden_stream(wl, 0))
    args = (hidden, ti.router_weights(wl, 0), ti.router_bias(wl, 0), wl.gating, wl.bias_mode, wl.k, wl.E, wl.C,
            ti.initial_resident(wl))
    sess = _session(wl)
    load(sess, wl, 0)
    tb.tide_refresh_engine(sess.ctx, engine)
    with pytest.raises(tb.TideError) as err:
        tb.tide_refresh_engine(sess.ctx, 2)
    assert err.value.code == tb.TIDE_E_INVAL
    host = sess.host_blobs[0].numpy()
    with pytest.raises(tb.TideError) as err:
        sess.commit(0)
    assert err.value.code == tb.TIDE_E_STATE
    for K, delay in ((1, 1), (4, 1), (4, 3)):
        log, _, _ = orc.run_block_policy(*args, interval=K, deferred=delay)
        tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
        sess.stats(0, reset=True)
        pending, due = False, -1
        for t, rec in enumerate(log):
            if pending and t == due:
                sess.commit(0)
                pending = False
            if t > 0 and t % K == 0:
                eis, plan = sess.refresh(0, deferred=True)
                pending, due, chosen = True, t + delay, rec["pending_expert_in_slot"]
                assert eis.tolist() == rec["pending_expert_in_slot"].tolist(), "step %d: chosen set" % t
                assert [(e, s) for e, s, _, _ in plan] == [tuple(p) for p in rec["plan"]], "step %d: plan" % t
                for call in (lambda: sess.refresh(0), lambda: sess.refresh(0, deferred=True)):
                    with pytest.raises(tb.TideError) as err:
                        call()
                    assert err.value.code == tb.TIDE_E_STATE
            x = sess.to_device_bf16(hidden[t])
            sess.step_routed(0, x, torch.from_numpy(rec["idx"]).to(sess.device),
                             torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device))
            _, _, _, miss, n_miss = sess.results(wl.N)
            check_miss(rec["miss"], miss, n_miss)
            assert np.array_equal(sess.table(0), rec["slot_of"]), "step %d: table" % t
            assert np.array_equal(sess.stats(0), rec["hits"].astype(np.int32)), "step %d: counter" % t
        if pending:
            sess.commit(0)
        torch.cuda.synchronize()
        final = chosen                                  # the last refresh's choice is in force once committed
        assert np.array_equal(sess.table(0), orc.slot_table(final, wl.E))
        for s in (0, 1, wl.C // 2, wl.C - 1):                 # the slots hold their experts' bytes
            assert np.array_equal(sess.read_slot(0, s), host[final[s]]), "slot %d" % s
        say("deferred refresh K=%d, serving %d step(s) late: %d steps exact, miss rate %.4f"
            % (K, delay, len(log), sum(len(r["miss"]) for r in log) / (len(log) * wl.N * wl.k)))
    # the immediate refresh through the same engine: slots byte-equal to the host blobs of the experts the table names
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    counts = np.zeros(wl.E, dtype=np.int32)
    counts[wl.C:wl.C + 5] = 3
    eis, plan = sess.refresh(0, counts=counts)
    assert len(plan) == 5 and sorted(e for e, _, _, _ in plan) == list(range(wl.C, wl.C + 5))
    tb.tide_wait_refresh(sess.ctx, 0)
    for e, s_, off, nbytes in plan:
        assert np.array_equal(sess.read_slot(0, s_), host[e]), "slot %d after an immediate refresh" % s_
    # a placement set by hand cancels a pending refresh
    sess.refresh(0, deferred=True)
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    with pytest.raises(tb.TideError):
        sess.commit(0)
    sess.close()
