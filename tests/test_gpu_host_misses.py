"""GPU parity of the host-core miss path (Sec. 3.3: tokens whose expert is not resident run on CPU
experts while the GPU runs the hits): tide_moe_step + tide_moe_apply_misses_host must give the
oracle's full MoE output, whatever the placement, and must agree with the device miss pass."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
import test_gpu_parity as tp

pytestmark = pytest.mark.gpu

CASES = [
    # workload, steps whose outputs are compared, host threads, percent of the missed experts the GPU takes over the link
    ("cfg0", [0, 1, 2, 3], 3, 0),
    ("cfg1", [0, 4, 5], 16, 0),
    ("cfg1", [0, 4], 16, 25),
    ("cfg0", [0, 1, 2, 3], 2, 50),
    ("cfg0", [1, 2], 2, 100),
    # partial gate/up group (12 column blocks) and partial down group (20 stripes); hundreds of misses per expert
    ((320, 8, 2, 192, 1, 700, 4, ti.GATING_SIGMOID, ti.BIAS_NONE), [0, 2], 4, 0),
    ((384, 70, 4, 192, 1, 257, 30, ti.GATING_SOFTMAX, ti.BIAS_LOGIT), [0, 3], 1, 0),
    ((384, 70, 4, 192, 1, 257, 30, ti.GATING_SOFTMAX, ti.BIAS_LOGIT), [0, 3], 4, 30),
    # more missed experts than 4 x threads: one work item per expert
    ((128, 300, 6, 128, 1, 33, 40, ti.GATING_SIGMOID, ti.BIAS_NONE), [1], 2, 0),
]


def _workload(spec):
    if spec == "cfg0":
        return ti.CONFIGS[0]
    if spec == "cfg1":
        return ti.CONFIGS[1]
    d, E, k, I, sh, N, C, gating, bias_mode = spec
    return ti.TideWorkload("ragged", d=d, E=E, k=k, I=I, n_shared=sh, N=N, S=5, K=2, C=C, L=1, gating=gating,
                           bias_mode=bias_mode, seed=177 + N)


@pytest.mark.parametrize("spec,out_steps,threads,share", CASES)
def test_host_miss_path_completes_the_output(spec, out_steps, threads, share):
    from paper_2605_20179_amd import binding as tb
    wl = _workload(spec)
    tp.say("host miss path %s, %d threads, link share %d" % (wl.name if isinstance(spec, str) else spec, threads, share))
    log, hidden = tp.oracle_block(wl, 0, out_steps)
    sess = tp._session(wl)
    tp.load(sess, wl, 0)
    with pytest.raises(tb.TideError) as ei:                      # no workers yet
        sess.apply_misses_host(0, sess.to_device_bf16(hidden[0]))
    assert ei.value.code == tb.TIDE_E_STATE
    sess.host_experts(threads)
    tb.tide_host_link_share(sess.ctx, share)
    worst = 0.0
    for t, rec in enumerate(log):
        if t > 0 and t % wl.K == 0:
            sess.refresh(0)
        x = sess.to_device_bf16(hidden[t])
        idx_d = torch.from_numpy(rec["idx"]).to(sess.device)
        w_d = torch.from_numpy(rec["w"].astype(np.float32)).to(sess.device)
        torch.cuda.synchronize()
        sess.step_routed(0, x, idx_d, w_d)
        if t not in out_steps:
            continue
        # no synchronisation in between: the host workers start from the step's split while the GPU is still
        # in the step's GEMMs, and the rows are added after the step's own combine
        sess.apply_misses_host(0, x)
        torch.cuda.synchronize()
        full = sess.out[:wl.N].cpu().numpy()
        worst = max(worst, tp.check_out(full, rec["y_full"]))
        assert np.array_equal(sess.stats(0), rec["hits"].astype(np.int32)), "the miss path must not count"
        assert np.array_equal(sess.table(0), rec["slot_of"]), "the miss path must not move experts"
        # the same list handed over in other buffers (no shortcut through the step's split event), added to zeros:
        # the misses' own sum = full - resident part
        miss2, n2, zeros = sess.miss.clone(), sess.n_miss.clone(), torch.zeros_like(sess.out)
        tb.tide_moe_apply_misses_host(sess.ctx, 0, x.clone(), wl.N, miss2, wl.N * wl.k, n2, zeros, torch.cuda.current_stream())
        torch.cuda.synchronize()
        want = rec["y_full"] - rec["y_res"]
        rms = float(np.sqrt(np.mean(rec["y_full"] ** 2)))
        assert np.abs(zeros[:wl.N].cpu().numpy() - want).max() <= tp.OUT_TOL * rms
        ms = tb.tide_host_miss_ms(sess.ctx)
        assert ms[2] >= ms[1] >= 0.0
    tp.say("host miss path worst err %.2e x RMS" % worst)
    sess.host_experts(0)                                         # workers stopped: the call is refused again
    with pytest.raises(tb.TideError):
        sess.apply_misses_host(0, sess.to_device_bf16(hidden[0]))
    sess.close()


def test_host_miss_path_is_deterministic_and_thread_count_changes_only_rounding():
    """Same thread count: bit-identical rows (fixed work decomposition, fixed summation order).  Another thread
    count may cut experts into column groups differently: the sums differ by fp32 rounding only."""
    from paper_2605_20179_amd import binding as tb
    wl = ti.CONFIGS[1]
    sess = tp._session(wl)
    tp.load(sess, wl, 0)
    x = sess.to_device_bf16(next(iter(ti.hidden_stream(wl, 0))))
    outs = []
    for threads in (16, 16, 1):
        sess.host_experts(threads)
        sess.stats(0, reset=True)
        sess.step(0, x)
        sess.apply_misses_host(0, x)
        torch.cuda.synchronize()
        outs.append(sess.out[:wl.N].cpu().numpy().copy())
    assert int(sess.n_miss.item()) > 0
    assert np.array_equal(outs[0], outs[1])
    rms = float(np.sqrt(np.mean(outs[0] ** 2)))
    assert np.abs(outs[0] - outs[2]).max() <= 1e-5 * rms
    sess.close()


def test_host_miss_path_after_a_graph_replay():
    """A step recorded into a HIP graph while host workers exist (its list hand-over is part of the graph), replayed,
    then completed by the host path: the same full output as the eager pair of calls, replay after replay."""
    wl = ti.CONFIGS[1].replace(S=4)
    sess = tp._session(wl)
    tp.load(sess, wl, 0)
    sess.host_experts(4)
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, 0, 4)]
    eager = []
    for h in hidden:
        sess.step(0, h)
        sess.apply_misses_host(0, h)
        torch.cuda.synchronize()
        eager.append(sess.out[:wl.N].clone())
    assert int(sess.n_miss.item()) > 0
    static_in = hidden[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sess.step(0, static_in)                       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sess.step(0, static_in)
    for rep in range(2):
        for i, h in enumerate(hidden):
            static_in.copy_(h)
            graph.replay()
            sess.apply_misses_host(0, static_in)
            torch.cuda.synchronize()
            assert torch.equal(sess.out[:wl.N], eager[i]), "replay %d step %d" % (rep, i)
        sess.step(0, hidden[rep])                     # eager work between the rounds
        sess.apply_misses_host(0, hidden[rep])
        torch.cuda.synchronize()
        assert torch.equal(sess.out[:wl.N], eager[rep])
    sess.close()


def test_host_miss_path_rejects_a_bad_list():
    from paper_2605_20179_amd import binding as tb
    wl = ti.CONFIGS[0]
    sess = tp._session(wl)
    tp.load(sess, wl, 0)
    sess.host_experts(2)
    x = sess.to_device_bf16(next(iter(ti.hidden_stream(wl, 0))))
    out = torch.zeros_like(sess.out)
    for token, expert in ((wl.N, 0), (-1, 0), (0, wl.E), (0, -1)):
        bad = np.zeros(wl.N * wl.k, dtype=tb.MISS_DTYPE)
        bad[0] = (token, expert, 1.0)
        miss = torch.from_numpy(bad.view(np.int32).reshape(-1, 3)).to(sess.device)
        n = torch.ones(1, dtype=torch.int32, device=sess.device)
        with pytest.raises(tb.TideError) as ei:
            tb.tide_moe_apply_misses_host(sess.ctx, 0, x, wl.N, miss, wl.N * wl.k, n, out, torch.cuda.current_stream())
        assert ei.value.code == tb.TIDE_E_INVAL
        # the device miss pass skips such an entry (its kernels check the ranges themselves)
        tb.tide_moe_apply_misses(sess.ctx, 0, x, wl.N, miss, wl.N * wl.k, n, out, torch.cuda.current_stream())
    torch.cuda.synchronize()
    assert float(out.abs().max()) == 0.0
    sess.close()
