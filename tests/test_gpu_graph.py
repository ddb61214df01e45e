"""A step (placement frozen) recorded into a HIP graph and replayed: every replay must give what the eager
call gives -- outputs, routing, miss count and the counter -- with eager work and synchronisations between
the replays.  Covers both the five-launch small step and a large step whose GEMMs fork onto the library's
second stream and join back (the fork/join events are captured with the graph).  The library clears its
counters and flags with fill kernels, never with memset nodes."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
from test_gpu_parity import _session, load, say

pytestmark = pytest.mark.gpu

LARGE = ti.TideWorkload("graph-large", d=320, E=8, k=2, I=192, n_shared=1, N=700, S=4, K=2, C=4, L=1,
                        gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_NONE, seed=5)


def _make(wl, p12):
    from paper_2605_20179_amd.session import TideSession
    if not p12:
        return _session(wl)
    return TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=True)


@pytest.mark.parametrize("p12", [False, True], ids=["bf16 slots", "12-bit slots"])
@pytest.mark.parametrize("wl", [ti.CONFIGS[1].replace(S=4), LARGE], ids=["small-step", "large-step"])
def test_step_replayed_from_a_graph(wl, p12):
    sess = _make(wl, p12)
    load(sess, wl, 0)
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, 0, 4)]
    eager = []
    for h in hidden:
        sess.step(0, h)
        torch.cuda.synchronize()
        eager.append((sess.out[:wl.N].clone(), sess.topk_idx[:wl.N].clone(), sess.topk_w[:wl.N].clone(),
                      sess.miss[:int(sess.n_miss.item())].clone(), int(sess.n_miss.item())))
    per_block = sess.stats(0, reset=True).copy()
    static_in = hidden[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sess.step(0, static_in)                       # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    sess.stats(0, reset=True)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sess.step(0, static_in)
    for rep in range(3):
        for i, h in enumerate(hidden):
            static_in.copy_(h)
            graph.replay()
            torch.cuda.synchronize()
            out, idx, w, miss, n_miss = eager[i]
            assert int(sess.n_miss.item()) == n_miss, "replay %d step %d: miss count" % (rep, i)
            assert torch.equal(sess.topk_idx[:wl.N], idx) and torch.equal(sess.topk_w[:wl.N], w)
            assert torch.equal(sess.miss[:n_miss], miss)
            assert torch.equal(sess.out[:wl.N], out), "replay %d step %d: output" % (rep, i)
        # eager work between the rounds of replays
        sess.step(0, hidden[rep % 4])
        torch.cuda.synchronize()
        assert torch.equal(sess.out[:wl.N], eager[rep % 4][0])
    # every replay and every eager call counted its step: 3 rounds x 4 steps, plus steps 0, 1, 2 once more
    fresh = _make(wl, p12)
    load(fresh, wl, 0)
    for i in range(3):
        fresh.step(0, hidden[i])
    want = 3 * per_block.astype(np.int64) + fresh.stats(0).astype(np.int64)
    assert np.array_equal(sess.stats(0).astype(np.int64), want)
    fresh.close()
    say("%s: 12 graph replays identical to the eager calls" % wl.name)
    sess.close()


def test_replay_after_a_refresh_needs_the_queued_wait():
    """A captured step holds no wait for refresh copies (the wait is decided when a step is issued).  After a
    refresh, tide_queue_refresh_wait on the replay's stream orders the replay behind the copies: the replay then
    equals the eager step on the new placement."""
    from paper_2605_20179_amd import binding as tb
    wl = ti.CONFIGS[1].replace(S=4)
    sess = _session(wl)
    load(sess, wl, 0)
    hidden = [sess.to_device_bf16(h) for h in ti.hidden_stream(wl, 0, 2)]
    static_in = hidden[0].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sess.step(0, static_in)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sess.step(0, static_in)
    # a refresh that replaces the whole budget: 64 blobs are in flight on the side stream when the replay is queued
    counts = np.zeros(wl.E, dtype=np.int32)
    counts[wl.C:2 * wl.C] = 1
    eis, plan = sess.refresh(0, counts=counts)
    assert len(plan) == wl.C
    tb.tide_queue_refresh_wait(sess.ctx, 0, torch.cuda.current_stream())
    static_in.copy_(hidden[1])
    graph.replay()
    torch.cuda.synchronize()
    got = (sess.out[:wl.N].clone(), sess.miss[:int(sess.n_miss.item())].clone(), int(sess.n_miss.item()))
    sess.step(0, hidden[1])                                # eager, on the settled new placement
    torch.cuda.synchronize()
    assert int(sess.n_miss.item()) == got[2] and torch.equal(sess.miss[:got[2]], got[1])
    assert torch.equal(sess.out[:wl.N], got[0])
    assert sorted(np.nonzero(sess.table(0) >= 0)[0].tolist()) == list(range(wl.C, 2 * wl.C))
    sess.close()


def test_stack_step_replayed_from_a_graph():
    """tide_moe_stack_step forks onto the library's lane streams and joins back by events: all of it is captured with
    the caller's stream, and every replay equals the eager stack step."""
    wl = ti.CONFIGS[2].replace(N=96, S=3, L=4, C=16)
    from paper_2605_20179_amd.session import TideSession
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, n_layers=wl.L)
    packed = sess.pack_layer(lambda e: ti.expert_weights(wl, 0, e), workers=16)
    for l in range(wl.L):
        sess.load_layer(l, None, ti.router_weights(wl, l), ti.router_bias(wl, l), ti.initial_resident(wl), packed=packed)
    hidden = [[sess.to_device_bf16(h) for h in ti.hidden_stream(wl, l)] for l in range(wl.L)]
    eager = []
    for t in range(wl.S):
        sess.stack_step([hidden[l][t] for l in range(wl.L)])
        torch.cuda.synchronize()
        eager.append([(sess.stack_out[l][:wl.N].clone(), int(sess.stack_n_miss[l].item())) for l in range(wl.L)])
    static_in = [hidden[l][0].clone() for l in range(wl.L)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        sess.stack_step(static_in)                     # warm-up outside the capture (the lanes exist already)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sess.stack_step(static_in)
    for rep in range(2):
        for t in range(wl.S):
            for l in range(wl.L):
                static_in[l].copy_(hidden[l][t])
            graph.replay()
            torch.cuda.synchronize()
            for l in range(wl.L):
                assert int(sess.stack_n_miss[l].item()) == eager[t][l][1]
                assert torch.equal(sess.stack_out[l][:wl.N], eager[t][l][0]), "replay %d step %d layer %d" % (rep, t, l)
        sess.step(0, hidden[0][rep], want_topk=False)      # eager work between the rounds of replays
        torch.cuda.synchronize()
    sess.close()
