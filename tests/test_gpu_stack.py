"""tide_moe_stack_step (the independent layers of a stack overlapped on the library's own streams and workspaces)
against tide_moe_step called layer by layer: outputs, miss lists, counters and tables must be identical bit for bit,
across refreshes, also when a stack step is followed by ordinary calls and when it covers only part of the layers."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
from test_gpu_parity import say

pytestmark = pytest.mark.gpu

CASES = [
    ("mini-shaped, 5 layers, small work items", ti.CONFIGS[2].replace(N=96, S=6, K=2, L=5, C=16)),
    ("slots of hundreds of rows on the second stream, 3 layers",
     ti.TideWorkload("stack-big", d=256, E=24, k=4, I=1024, n_shared=1, N=900, S=5, K=2, C=8, L=3,
                     gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_LOGIT, seed=77)),
    ("block of 32 tokens, 4 layers (one-workgroup routing)", ti.CONFIGS[1].replace(S=5, K=2, L=4, C=12, E=48, d=512, I=256)),
]


@pytest.mark.parametrize("p12", [False, True], ids=["bf16 slots", "12-bit slots"])
@pytest.mark.parametrize("name,wl", CASES, ids=[c[0] for c in CASES])
def test_stack_step_equals_layer_by_layer(name, wl, p12):
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    say("stack: %s, %s" % (name, "12-bit slots" if p12 else "bf16 slots"))

    def make():
        sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, n_layers=wl.L, resident_p12=p12)
        packed = sess.pack_layer(lambda e: ti.expert_weights(wl, 0, e), workers=16)
        for l in range(wl.L):                             # the layers share layer 0's blobs, compressed once
            sess.load_layer(l, None, ti.router_weights(wl, l), ti.router_bias(wl, l), ti.initial_resident(wl), packed=packed,
                            comp=sess.comp_blobs.get(0))
        return sess

    ref, stk = make(), make()
    hidden = [[ref.to_device_bf16(h) for h in ti.hidden_stream(wl, l)] for l in range(wl.L)]
    for t in range(wl.S):
        if t > 0 and t % wl.K == 0:
            for l in range(wl.L):
                a, b = ref.refresh(l), stk.refresh(l)
                assert a[0].tolist() == b[0].tolist() and a[1] == b[1]
        want = []
        for l in range(wl.L):
            ref.step(l, hidden[l][t], want_topk=False)
            torch.cuda.synchronize()
            n = int(ref.n_miss.item())
            want.append((ref.out[:wl.N].clone(), ref.miss[:n].clone(), n))
        if t == 3:                                        # a stack step over layers 1.. only, layer 0 by the ordinary call
            stk.step(0, hidden[0][t], want_topk=False)
            torch.cuda.synchronize()
            assert torch.equal(stk.out[:wl.N], want[0][0])
            stk.stack_step([hidden[l][t] for l in range(1, wl.L)], first_layer=1)
            check_from = 1
        else:
            stk.stack_step([hidden[l][t] for l in range(wl.L)])
            check_from = 0
        torch.cuda.synchronize()
        for l in range(check_from, wl.L):
            out, miss, n = want[l]
            assert int(stk.stack_n_miss[l].item()) == n, "step %d layer %d: miss count" % (t, l)
            assert torch.equal(stk.stack_miss[l][:n], miss), "step %d layer %d: miss list" % (t, l)
            assert torch.equal(stk.stack_out[l][:wl.N], out), "step %d layer %d: output" % (t, l)
        for l in range(wl.L):
            assert np.array_equal(ref.stats(l), stk.stats(l)), "step %d layer %d: hit counter" % (t, l)
            assert np.array_equal(ref.table(l), stk.table(l))
    assert tb.tide_counters(ref.ctx) == tb.tide_counters(stk.ctx)
    # argument checks
    with pytest.raises(tb.TideError) as ei:                 # two layers starting at the last one
        tb.tide_moe_stack_step(stk.ctx, wl.L - 1, [hidden[0][0]] * 2, wl.N, stk.router_w[:2], stk.router_b[:2], stk.stack_out[:2],
                               stk.stack_miss[:2], wl.N * wl.k, stk.stack_n_miss[:2], torch.cuda.current_stream())
    assert ei.value.code == tb.TIDE_E_INVAL
    stk.host_experts(2)
    with pytest.raises(tb.TideError) as ei:
        stk.stack_step([hidden[l][0] for l in range(wl.L)])
    assert ei.value.code == tb.TIDE_E_STATE
    stk.host_experts(0)
    ref.close()
    stk.close()
