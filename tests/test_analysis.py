"""The refresh-interval analysis of the library against its oracle (oracle/tide_analysis.py).

Host part (no GPU): the cost model Eq. 5-6 and the optimal interval Eq. 7 through the C ABI.
GPU part: activation vectors logged step by step from the routing kernels, and the similarity /
distinct-expert / drift kernels (Sec. 3.2, Eq. 4), element by element."""
import numpy as np
import pytest

from oracle import tide_analysis as ana


def test_interval_cost_model_through_the_c_abi():
    from paper_2605_20179_amd import binding as tb
    rng = np.random.default_rng(21)
    for _ in range(50):
        B, T = int(rng.integers(1, 257)), int(rng.integers(2, 129))
        d, cio, ccpu = float(rng.random()), float(rng.random() * 1e-3), float(rng.random() * 1e-4)
        f = np.cumsum(rng.random(T - 1)) / T
        io, cpu = tb.tide_interval_costs(B, T, d, cio, ccpu, f)
        for tau in range(1, T):
            assert abs(io[tau - 1] - ana.lat_io(cio, B, T, tau, d)) <= 1e-12 * max(1e-30, abs(io[tau - 1]))
            assert abs(cpu[tau - 1] - ana.lat_cpu(ccpu, B, T, f[tau - 1])) <= 1e-12 * max(1e-30, abs(cpu[tau - 1]))
        tau, cost = tb.tide_optimal_interval(B, T, d, cio, ccpu, f)
        want_tau, want_cost = ana.optimal_interval(B, T, d, cio, ccpu, f)
        assert tau == want_tau and abs(cost - want_cost) <= 1e-12 * max(1e-30, abs(want_cost))
        assert abs(tb.tide_fit_drift(float(io[2 % (T - 1)] / max(cio, 1e-300)), B, T, 2 % (T - 1) + 1) - ana.fit_drift(float(io[2 % (T - 1)] / max(cio, 1e-300)), B, T, 2 % (T - 1) + 1)) <= 1e-12
    assert tb.tide_fit_drift(1e9, 4, 8, 2) == 1.0 and tb.tide_fit_drift(-3.0, 4, 8, 2) == 0.0
    # edge cases: d = 0 (nothing ever moves), d = 1 (everything moves), ties resolved to the smaller tau, T = 2
    assert tb.tide_interval_costs(64, 32, 0.0, 1.0, 0.0, np.zeros(31))[0].tolist() == [0.0] * 31
    assert np.allclose(tb.tide_interval_costs(64, 32, 1.0, 1.0, 0.0, np.zeros(31))[0], 64 * 32 / np.arange(1, 32))
    assert tb.tide_optimal_interval(4, 6, 0.0, 1.0, 1.0, [0.5] * 5)[0] == 1
    assert tb.tide_optimal_interval(8, 2, 0.3, 1.0, 1.0, [0.2]) == (1, pytest.approx(8 * 2 * 0.3 + 2 * 8 * 0.2))
    # bad arguments are refused with the documented codes
    for args in ((0, 8, 0.1), (4, 1, 0.1), (4, 8, -0.1), (4, 8, 1.5)):
        with pytest.raises(tb.TideError) as e:
            tb.tide_optimal_interval(args[0], args[1], args[2], 1.0, 1.0, np.zeros(max(args[1] - 1, 1)))
        assert e.value.code == tb.TIDE_E_RANGE


@pytest.mark.gpu
def test_stability_kernels_on_random_and_edge_counts():
    import torch
    from paper_2605_20179_amd import binding as tb
    rng = np.random.default_rng(22)
    cases = []
    for S, E, B, lam in ((32, 256, 64, 1.0), (7, 512, 512, 0.2), (1, 16, 4, 2.0), (40, 1, 1, 3.0), (33, 100, 17, 0.05)):
        c = rng.poisson(lam, size=(S, E)).astype(np.int32)
        if S > 3:
            c[2] = 0                          # a step without activations
            c[3] = c[1]                       # identical neighbours two apart
        cases.append((c, B))
    big = np.full((4, 64), 2 ** 20, dtype=np.int32)      # squares near 2^40: exact only in 64-bit sums
    big[1, ::2] = 0
    cases.append((big, 8))
    for c, B in cases:
        S, E = c.shape
        print("stability case S=%d E=%d B=%d" % (S, E, B), flush=True)
        cd = torch.from_numpy(c).cuda()
        sim = torch.empty((S, S), dtype=torch.float64, device="cuda")
        uniq = torch.empty(S, dtype=torch.int32, device="cuda")
        drift = torch.empty(S, dtype=torch.float64, device="cuda")
        tb.tide_routing_stability(None, cd, S, E, B, sim, uniq, drift, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert np.abs(sim.cpu().numpy() - ana.cosine_similarity_matrix(c)).max() <= 1e-12
        assert uniq.cpu().numpy().tolist() == ana.unique_experts(c).tolist()
        assert drift.cpu().numpy().tolist() == ana.drift_rates(c, B).tolist()
        # outputs are optional
        tb.tide_routing_stability(None, cd, S, E, B, None, uniq, None, torch.cuda.current_stream())
        tb.tide_routing_stability(None, cd, S, E, B, None, None, drift, torch.cuda.current_stream())
        torch.cuda.synchronize()
        assert uniq.cpu().numpy().tolist() == ana.unique_experts(c).tolist()
    with pytest.raises(tb.TideError):
        tb.tide_routing_stability(None, cd, 4, 513, 8, None, uniq, None, torch.cuda.current_stream())
    with pytest.raises(tb.TideError):
        tb.tide_routing_stability(None, cd, 4, 64, 65, None, None, drift, torch.cuda.current_stream())


@pytest.mark.gpu
def test_logged_activation_vectors_and_interval_choice_on_a_block():
    """cfg 1: the activation vector of every step of a block, logged from the routing kernels, equals the
    oracle's step histograms; stability figures and the chosen interval computed from them agree."""
    import torch
    import tide_inputs as ti
    from oracle import tide_oracle as orc
    from paper_2605_20179_amd import binding as tb
    from test_gpu_parity import _session, load, say
    wl = ti.CONFIGS[1]
    sess = _session(wl)
    load(sess, wl, 0)
    w_r, bias = ti.router_weights(wl, 0), ti.router_bias(wl, 0)
    want, got, amb = [], [], 0
    for t, h in enumerate(ti.hidden_stream(wl, 0)):
        idx, _, ambiguous = orc.route(h, w_r, bias, wl.gating, wl.bias_mode, wl.k)[:3]
        amb += int(np.sum(ambiguous))
        want.append(orc.step_histogram(idx, wl.E))
        sess.step(0, sess.to_device_bf16(h))
        got.append(tb.tide_step_histogram(sess.ctx, wl.E, torch.cuda.current_stream()))
    want, got = np.array(want), np.array(got)
    say("near-tie tokens in the block: %d" % amb)
    if amb == 0:
        assert np.array_equal(want, got)
    else:
        assert np.abs(want - got).sum() <= 2 * amb
    cd = torch.from_numpy(got.astype(np.int32)).cuda()
    S = got.shape[0]
    sim = torch.empty((S, S), dtype=torch.float64, device="cuda")
    uniq = torch.empty(S, dtype=torch.int32, device="cuda")
    drift = torch.empty(S, dtype=torch.float64, device="cuda")
    tb.tide_routing_stability(sess.ctx, cd, S, wl.E, wl.C, sim, uniq, drift, torch.cuda.current_stream())
    torch.cuda.synchronize()
    sim_h = sim.cpu().numpy()
    assert np.abs(sim_h - ana.cosine_similarity_matrix(got)).max() <= 1e-12
    assert uniq.cpu().numpy().tolist() == ana.unique_experts(got).tolist()
    d = drift.cpu().numpy()
    assert d.tolist() == ana.drift_rates(got, wl.C).tolist()
    adjacent = float(np.mean([sim_h[t, t + 1] for t in range(S - 1)]))
    say("adjacent-step similarity %.4f, 5 apart %.4f, mean drift %.4f, distinct experts %d..%d"
        % (adjacent, float(np.mean([sim_h[t, t + 5] for t in range(S - 5)])), float(d[1:].mean()), uniq.min().item(), uniq.max().item()))
    assert adjacent > 0.9                     # the synthetic stream is built to be stable across adjacent steps (Sec. 3.2)
    # interval choice from measured-like constants: same answer from the library and the oracle
    f = np.maximum.accumulate(1.0 - np.array([sim_h[0, min(tau, S - 1)] for tau in range(1, S)]))
    tau, cost = tb.tide_optimal_interval(wl.C, S, float(d[1:].mean()), 1.1e-4, 2.0e-6, f)
    assert (tau, cost) == (ana.optimal_interval(wl.C, S, float(d[1:].mean()), 1.1e-4, 2.0e-6, f)[0], pytest.approx(ana.optimal_interval(wl.C, S, float(d[1:].mean()), 1.1e-4, 2.0e-6, f)[1], rel=1e-12))
    sess.close()
