"""The entry point that allocates nothing, tide_moe_step_noalloc, against tide_moe_step on the same context and
inputs: selections, weights, miss lists, hit counters and outputs must be identical bit for bit (the two calls run
the same kernels; only the workspace they are handed differs).  Each case makes two calls in a row, the second with
fewer tokens, so that whatever the first call left in the shared scratch array is there when the second runs."""
import numpy as np
import pytest
import torch

import tide_inputs as ti

pytestmark = pytest.mark.gpu

CASES = [
    # name, workload, token counts of the two calls
    ("mini layer, block 32", ti.CONFIGS[1], (32, 9)),
    ("mini layer, 8 blocks (many small work items per slot)", ti.CONFIGS[2].replace(L=1), (256, 100)),
    ("slots of hundreds of rows (large work items)",
     ti.TideWorkload("noalloc-big", d=256, E=32, k=4, I=1024, n_shared=1, N=1000, S=1, K=1, C=8, L=1,
                     gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_LOGIT, seed=311), (1000, 333)),
    ("tiny softmax layer without shared expert", ti.CONFIGS[0], (8, 1)),
]


def _run(sess, tb, fn, x, n):
    sess.stats(0, reset=True)
    sess.out.fill_(float("nan"))
    sess.miss.fill_(-1)
    sess.n_miss.fill_(-1)
    sess.topk_idx.fill_(-1)
    sess.topk_w.fill_(-1.0)
    fn(sess.ctx, 0, x, n, sess.router_w[0], sess.router_b[0], sess.out, sess.miss, n * sess.k, sess.n_miss,
       sess.topk_idx, sess.topk_w, torch.cuda.current_stream())
    out, idx, w, miss, n_miss = sess.results(n)
    raw_miss = sess.miss[:n_miss].cpu().numpy().copy()
    return out.copy(), idx.copy(), w.copy(), raw_miss, n_miss, sess.stats(0).copy(), tb.tide_step_histogram(sess.ctx, sess.E)


@pytest.mark.parametrize("p12", [False, True], ids=["bf16 slots", "12-bit slots"])
@pytest.mark.parametrize("name,wl,token_counts", CASES, ids=[c[0] for c in CASES])
def test_noalloc_step_equals_the_allocating_one(name, wl, token_counts, p12):
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    print("[noalloc] %s: %s, %s" % (name, token_counts, "12-bit slots" if p12 else "bf16 slots"), flush=True)
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=p12)
    sess.load_layer(0, lambda e: ti.expert_weights(wl, 0, e), ti.router_weights(wl, 0), ti.router_bias(wl, 0),
                    ti.initial_resident(wl), workers=16)
    hidden = sess.to_device_bf16(next(iter(ti.hidden_stream(wl, 0))))
    want = [_run(sess, tb, tb.tide_moe_step, hidden[:n].contiguous(), n) for n in token_counts]
    got = [_run(sess, tb, tb.tide_moe_step_noalloc, hidden[:n].contiguous(), n) for n in token_counts]   # back to back
    for n, a, b in zip(token_counts, want, got):
        assert a[4] == b[4], "%d tokens: miss count" % n
        for what, u, v in zip(("out", "idx", "w", "miss list", "n_miss", "H", "step histogram"), a, b):
            assert np.array_equal(u, v), "%d tokens: %s differs" % (n, what)
        assert np.isfinite(b[0]).all() and (b[1] >= 0).all()
    cnt = tb.tide_counters(sess.ctx, reset=True)
    assert cnt["steps"] == 2 * len(token_counts)
    sess.close()


def test_noalloc_refuses_a_step_that_does_not_fit_and_profiled_runs():
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    assert tb.tide_noalloc_scratch_bytes() == 32 << 20
    wl = ti.CONFIGS[3]                       # 512 tokens at d = 4096: 75 MB of per-row outputs alone
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, 2, wl.N, wl.gating, wl.bias_mode)
    blobs = torch.zeros((wl.E, sess.blob_bytes), dtype=torch.uint8, pin_memory=True)
    sess.load_layer(0, None, ti.router_weights(wl, 0), ti.router_bias(wl, 0), [0, 1],
                    packed=(blobs, np.zeros(sess.blob_bytes, dtype=np.uint8)))
    x = torch.zeros((wl.N, wl.d), dtype=torch.int16, device=sess.device)
    args = (sess.router_w[0], sess.router_b[0], sess.out, sess.miss, wl.N * wl.k, sess.n_miss, None, None,
            torch.cuda.current_stream())
    sess.n_miss.fill_(-5)
    with pytest.raises(tb.TideError) as ei:
        tb.tide_moe_step_noalloc(sess.ctx, 0, x, wl.N, *args)
    assert ei.value.code == tb.TIDE_E_RANGE and "static scratch" in str(ei.value)
    torch.cuda.synchronize()
    assert int(sess.n_miss.item()) == -5 and tb.tide_counters(sess.ctx)["steps"] == 0       # nothing was queued
    tb.tide_moe_step_noalloc(sess.ctx, 0, x[:64].contiguous(), 64, *args[:4], 64 * wl.k, *args[5:])   # 64 tokens fit
    tb.tide_profile(sess.ctx, 1)
    with pytest.raises(tb.TideError) as ei:
        tb.tide_moe_step_noalloc(sess.ctx, 0, x[:64].contiguous(), 64, *args[:4], 64 * wl.k, *args[5:])
    assert ei.value.code == tb.TIDE_E_STATE
    tb.tide_profile(sess.ctx, 0)
    torch.cuda.synchronize()
    assert tb.tide_counters(sess.ctx)["steps"] == 1
    sess.close()
