"""GPU parity of tide_refresh_async: the refresh queued without a host round trip must install the same placement,
plan and counter state as tide_refresh (compared with the oracle's block), with raw and with compressed copies, into
bf16 and into 12-bit slots."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
import test_gpu_parity as tp

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("cfg_id,compressed", [(0, False), (1, False), (1, True), (1, "12-bit slots")])
def test_async_refresh_matches_the_oracle(cfg_id, compressed):
    wl = ti.CONFIGS[cfg_id]
    out_steps = [0, 1, 2, 3] if cfg_id == 0 else [0, 4, 5, 9]
    tp.say("async refresh %s compressed=%s" % (wl.name, compressed))
    log, hidden = tp.oracle_block(wl, 0, out_steps)
    p12 = compressed == "12-bit slots"                # the slots keep the compressed blobs: copied as they are
    if p12:
        from paper_2605_20179_amd.session import TideSession
        sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=True)
    else:
        sess = tp._session(wl)
    tp.load(sess, wl, 0)
    if compressed and not p12:
        sess.compress_layer(0, workers=8)
    worst, pending = 0.0, None
    for t, rec in enumerate(log):
        if t > 0 and t % wl.K == 0:
            sess.refresh_async(0)                      # returns at once; the step below is queued behind it
            pending = rec
        x = sess.to_device_bf16(hidden[t])
        sess.step_routed(0, x, torch.from_numpy(rec["idx"]).to(sess.device),
                         torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device))
        if pending is not None:
            eis, plan = sess.refresh_result(0)
            assert eis.tolist() == pending["expert_in_slot"].tolist(), "step %d: resident set" % t
            assert [(e, s) for e, s, _, _ in plan] == [tuple(p) for p in pending["plan"]], "step %d: plan" % t
            pending = None
        out, _, _, miss, n_miss = sess.results(wl.N)
        tp.check_miss(rec["miss"], miss, n_miss)
        assert np.array_equal(sess.stats(0), rec["hits"].astype(np.int32)), "step %d: hit counter" % t
        assert np.array_equal(sess.table(0), rec["slot_of"]), "step %d: table" % t
        if t in out_steps:
            worst = max(worst, tp.check_out(out, rec["y_res"]))
    eis = log[-1]["expert_in_slot"]
    for s in (0, wl.C // 2, wl.C - 1):
        want = sess.host_blobs[0][int(eis[s])].numpy()
        if p12 and not sess.comp_blobs[0][int(eis[s])][:64].numpy().view(np.uint32)[2]:
            want = sess.comp_blobs[0][int(eis[s])].numpy()
        assert np.array_equal(sess.read_slot(0, s)[:len(want)], want), "slot %d bytes" % s
    # the result of a synchronous refresh can be read the same way; before any refresh the call is refused
    eis2, plan2 = sess.refresh(0)
    eis3, plan3 = sess.refresh_result(0)
    assert eis2.tolist() == eis3.tolist() and plan2 == plan3
    tp.say("async refresh worst out err %.2e x RMS" % worst)
    sess.close()
    from paper_2605_20179_amd import binding as tb
    fresh = tp._session(wl)
    tp.load(fresh, wl, 0)
    with pytest.raises(tb.TideError) as ei:
        fresh.refresh_result(0)
    assert ei.value.code == tb.TIDE_E_STATE
    fresh.close()
