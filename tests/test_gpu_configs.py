"""GPU parity at the shapes of workload configurations 2, 3 and 4 (the larger ones).

Routing, hit counters, miss lists, resident sets and copy plans are compared for every
token of every step run; expert outputs are compared on a stated sample of tokens and
steps (the fp64 oracle evaluates one (token, expert) pair at a time).  Stacks are run on
a subset of their layers -- layers are independent (own weights, stream, cache, counter)
-- and on a shortened block where noted."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
from oracle import tide_oracle as orc
from test_gpu_parity import (_session, check_miss, check_out, check_routing, load, oracle_block, run_block_on_gpu,
                             say)

pytestmark = pytest.mark.gpu

_PACKED = {}


def packed_layer(sess, wl, layer):
    """Pinned packed blobs of (shape, layer), built once per test session."""
    key = (wl.d, wl.I, wl.E, wl.seed, layer)
    if key not in _PACKED:
        say("packing %d experts d=%d I=%d layer %d" % (wl.E, wl.d, wl.I, layer))
        _PACKED[key] = sess.pack_layer(lambda e: ti.expert_weights(wl, layer, e), workers=16)
    return _PACKED[key]


def load_packed(sess, wl, layer, sess_layer=None, resident=None):
    sess.load_layer(layer if sess_layer is None else sess_layer, None, ti.router_weights(wl, layer),
                    ti.router_bias(wl, layer), ti.initial_resident(wl) if resident is None else resident,
                    packed=packed_layer(sess, wl, layer))


def sample_tokens(wl, n, seed):
    return sorted(np.random.default_rng(seed).choice(wl.N, size=n, replace=False).tolist())


def test_config2_stack_layers_and_interval_sweep():
    """Mini-shaped stack: 3 of the 20 layers, 256 tokens per step, full 32-step block at K = 4;
    then K in {1, 2, 8} on layer 0 for routing / counters / refresh / miss lists."""
    base = ti.CONFIGS[2]
    layers = [0, 7, 19]
    toks = sample_tokens(base, 12, 2)
    out_steps = [0, 4, 5, 31]
    from paper_2605_20179_amd.session import TideSession
    sess = TideSession(base.d, base.E, base.k, base.I, base.n_shared, base.C, base.N, base.gating, base.bias_mode,
                       n_layers=len(layers))
    for li, layer in enumerate(layers):
        say("cfg2 layer %d" % layer)
        log, hidden = oracle_block(base, layer, out_steps, tokens=toks)
        say("near-tie tokens per step: %s" % [int(r["ambiguous"].sum()) for r in log])
        for forced in (True, False):
            load_packed(sess, base, layer, sess_layer=li)
            sess.stats(li, reset=True)
            flips, worst = run_block_on_gpu(base, li, sess, log, hidden, forced, out_steps, tokens=toks)
            say("cfg2 layer %d forced=%s flips=%d worst=%.2e" % (layer, forced, flips, worst))
    for K in (1, 2, 8):
        wl = base.replace(K=K, S=17)
        log, hidden = oracle_block(wl, 0, [])
        load_packed(sess, wl, 0, sess_layer=0)
        sess.stats(0, reset=True)
        flips, _ = run_block_on_gpu(wl, 0, sess, log, hidden, True, [])
        swaps = [len(r["plan"]) for r in log if r["plan"] is not None]
        say("cfg2 K=%d: experts copied per refresh %s" % (K, swaps))
    sess.close()


def test_config3_flash_layer():
    """Flash-shaped layer, 512 tokens per step; 9 steps (refreshes at 4 and 8); outputs on 10 sampled tokens."""
    wl = ti.CONFIGS[3].replace(S=9)
    toks = sample_tokens(wl, 10, 3)
    out_steps = [0, 4, 5]
    log, hidden = oracle_block(wl, 0, out_steps, tokens=toks)
    say("cfg3 oracle done; near-ties per step %s" % [int(r["ambiguous"].sum()) for r in log])
    sess = _session(wl)
    for forced in (True, False):
        load_packed(sess, wl, 0)
        sess.stats(0, reset=True)
        flips, worst = run_block_on_gpu(wl, 0, sess, log, hidden, forced, out_steps, tokens=toks)
        say("cfg3 forced=%s flips=%d worst=%.2e" % (forced, flips, worst))
    # the host-core miss path at this size (hundreds of missed pairs over most of the 192 non-resident experts):
    # step 0 from the initial placement, with the oracle's routing
    load_packed(sess, wl, 0)
    sess.stats(0, reset=True)
    sess.host_experts(16)
    x = sess.to_device_bf16(hidden[0])
    sess.step_routed(0, x, torch.from_numpy(log[0]["idx"]).to(sess.device),
                     torch.from_numpy(log[0]["w"].astype(np.float32)).to(sess.device))
    sess.apply_misses_host(0, x)
    torch.cuda.synchronize()
    err = check_out(sess.out[:wl.N].cpu().numpy(), log[0]["y_full"], rows=toks)
    say("cfg3 host miss path: %d misses, worst=%.2e" % (len(log[0]["miss"]), err))
    sess.close()


@pytest.mark.parametrize("capacity", [64, 256])
def test_config4_flash_stack_layer(capacity):
    """Flash-shaped stack at 2048 tokens per step, one of its 32 layers, 6 steps (refresh at 4),
    in both cache settings: capacity 64 with the remainder in pinned host memory, and all 256
    experts resident (no misses, no copies)."""
    wl = ti.CONFIGS[4].replace(S=6, C=capacity)
    toks = sample_tokens(wl, 8, 4)
    out_steps = [0, 4]
    log, hidden = oracle_block(wl, 0, out_steps, tokens=toks)
    say("cfg4 C=%d oracle done; near-ties per step %s" % (capacity, [int(r["ambiguous"].sum()) for r in log]))
    sess = _session(wl)
    for forced in (True, False):
        load_packed(sess, wl, 0)
        sess.stats(0, reset=True)
        flips, worst = run_block_on_gpu(wl, 0, sess, log, hidden, forced, out_steps, tokens=toks)
        say("cfg4 C=%d forced=%s flips=%d worst=%.2e" % (capacity, forced, flips, worst))
    if capacity == 256:
        assert all(r["miss"] == [] for r in log) and all(not r["plan"] for r in log)
    sess.close()


def test_maximum_tokens_per_step():
    """The largest step the library accepts (max_tokens = 65535, a ragged last tile everywhere) on small matrices:
    three steps with a refresh, every token's routing, the 160 000-entry miss lists, counters, tables and the copy
    plan compared; outputs (resident part, then completed by the miss pass) on 12 sampled tokens."""
    wl = ti.TideWorkload("max-tokens", d=64, E=32, k=4, I=64, n_shared=1, N=65535, S=3, K=2, C=8, L=1,
                         gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_LOGIT, seed=91)
    toks = sample_tokens(wl, 12, 5)
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
