"""GPU checks of cache slots kept in the 12-bit form of the blobs (tide_config.resident_format = TIDE_RESIDENT_P12):
the expert GEMMs decode the weights in registers, so every output must be bit-identical to the same step over bf16
slots -- and within the usual bound of the oracle; the slots hold the compressed blobs byte for byte (the bf16 blob
for an expert that cannot be encoded); refreshes, immediate, deferred and through the copy engines, move compressed
blobs; a large work item holds at most 192 rows."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
import test_gpu_parity as tp
from oracle import tide_oracle as orc

pytestmark = pytest.mark.gpu


def _sessions(wl, expert_bits=None, max_tokens=None):
    """A session over bf16 slots and one over 12-bit slots, same blobs, same placement."""
    from paper_2605_20179_amd.session import TideSession
    bits = expert_bits or (lambda e: ti.expert_weights(wl, 0, e))
    pair = []
    packed = None
    for p12 in (False, True):
        sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, max_tokens or wl.N, wl.gating, wl.bias_mode, resident_p12=p12)
        if packed is None:
            packed = sess.pack_layer(bits, workers=8)
        sess.load_layer(0, None, ti.router_weights(wl, 0), ti.router_bias(wl, 0), ti.initial_resident(wl), packed=packed)
        sess.shared_blob = packed[1]
        pair.append(sess)
    return pair


def _check_slots(sess, eis):
    """Every occupied slot holds what the library says a 12-bit slot holds: the expert's compressed blob, or its bf16
    blob when the compressed one is marked raw."""
    from paper_2605_20179_amd import binding as tb
    comp_bytes = tb.tide_compressed_blob_bytes(sess.cfg)
    comp, raw = sess.comp_blobs[0].numpy(), sess.host_blobs[0].numpy()
    raw_experts = []
    for s, e in enumerate(eis):
        if e < 0:
            continue
        got = sess.read_slot(0, s)
        if comp[e][:64].view(np.uint32)[2]:
            assert np.array_equal(got, raw[e]), "slot %d: expert %d is marked raw" % (s, e)
            raw_experts.append(e)
        else:
            assert np.array_equal(got[:comp_bytes], comp[e]), "slot %d: compressed blob of expert %d" % (s, e)
    if sess.n_shared:
        # the shared expert's slot: the 12-bit form in a context of at most 64 tokens per step, else the bf16 blob
        got = sess.read_slot(0, sess.C)
        if sess.max_tokens <= 64:
            want = np.empty(comp_bytes, dtype=np.uint8)
            tb.tide_compress_expert(sess.cfg, sess.shared_blob, want)
            assert not want[:64].view(np.uint32)[2]
            assert np.array_equal(got[:comp_bytes], want), "shared expert's slot: its compressed blob"
        else:
            assert np.array_equal(got, sess.shared_blob), "shared expert's slot: its bf16 blob"
    return raw_experts


@pytest.mark.parametrize("cfg_id,out_steps", [(0, [0, 1, 2, 3]), (1, [0, 3, 4, 5, 16, 31])])
def test_block_over_12bit_slots(cfg_id, out_steps):
    """The block of configurations 0 and 1 over 12-bit slots: everything the plain parity test checks against the
    oracle (routing, counters, tables, plans, miss lists, outputs, the lossless sum with the miss pass), with the
    library's own routing and with the oracle's forced in."""
    wl = ti.CONFIGS[cfg_id]
    tp.say("block over 12-bit slots %s" % wl.name)
    log, hidden = tp.oracle_block(wl, 0, out_steps)
    for forced in (True, False):
        bf16, p12 = _sessions(wl)
        bf16.close()
        flips, worst = tp.run_block_on_gpu(wl, 0, p12, log, hidden, forced, out_steps)
        tp.say("%s 12-bit slots forced=%s: %d near-tie flips, worst out err %.2e x RMS" % (wl.name, forced, flips, worst))
        if forced:
            _check_slots(p12, log[-1]["expert_in_slot"].tolist())
        p12.close()


@pytest.mark.parametrize("engine,deferred", [("kernel", False), ("kernel", True), ("dma", False), ("dma", True)])
def test_steps_and_refreshes_are_bit_identical_to_bf16_slots(engine, deferred):
    """Configuration 1's first 12 steps on both kinds of slots, refreshes through both copy engines, immediate and
    deferred: identical plans and tables, and outputs equal bit for bit at every step."""
    from paper_2605_20179_amd import binding as tb
    wl = ti.CONFIGS[1]
    tp.say("12-bit vs bf16 slots, engine=%s deferred=%s" % (engine, deferred))
    hidden = list(ti.hidden_stream(wl, 0, 12))
    bf16, p12 = _sessions(wl)
    for s in (bf16, p12):
        if engine == "dma":
            tb.tide_refresh_engine(s.ctx, tb.TIDE_COPY_DMA)
    eis = None
    for t, h in enumerate(hidden):
        if t > 0 and t % wl.K == 0:
            res = [s.refresh(0, deferred=deferred) for s in (bf16, p12)]
            assert res[0][0].tolist() == res[1][0].tolist() and res[0][1] == res[1][1], "step %d: refresh" % t
            eis = res[1][0].tolist()
            if deferred:
                for s in (bf16, p12):
                    s.commit(0)
        outs = []
        for s in (bf16, p12):
            x = s.to_device_bf16(h)
            s.step(0, x)
            torch.cuda.synchronize()
            outs.append((s.out[:wl.N].clone(), s.topk_idx[:wl.N].clone(), int(s.n_miss.item())))
        assert torch.equal(outs[0][1], outs[1][1]) and outs[0][2] == outs[1][2], "step %d: routing" % t
        assert torch.equal(outs[0][0], outs[1][0]), "step %d: outputs differ between bf16 and 12-bit slots" % t
        assert np.array_equal(bf16.table(0), p12.table(0))
    _check_slots(p12, eis)
    bf16.close()
    p12.close()


def _forced_routing(wl, rows_of_expert, rng):
    """Routing with exactly rows_of_expert[e] tokens on expert e (distinct experts per token): the listed experts are
    dealt to the tokens that have the fewest picks so far, the remaining picks go to the other experts."""
    picks = [[] for _ in range(wl.N)]
    for e, r in sorted(rows_of_expert.items(), key=lambda kv: -kv[1]):
        order = sorted(range(wl.N), key=lambda n: (len(picks[n]), rng.random()))
        assert r <= wl.N and len(picks[order[r - 1]]) < wl.k
        for n in order[:r]:
            picks[n].append(e)
    others = [e for e in range(wl.E) if e not in rows_of_expert]
    idx = np.zeros((wl.N, wl.k), dtype=np.int32)
    for n in range(wl.N):
        fill = [int(e) for e in rng.permutation(others)[: wl.k - len(picks[n])]]
        idx[n] = picks[n] + fill
    return idx


def test_large_work_items_over_12bit_slots():
    """Every size class of the large-item kernels over 12-bit slots: forced routing gives the resident experts 33 to
    640 rows (1 to 12 token tiles per work item, slots cut into several items, the shared expert's 640), one resident
    expert is stored raw.  Outputs: equal to the bf16-slot session bit for bit, and within the bound of the oracle
    (resident part and the full layer).  Work items hold at most 192 rows."""
    from paper_2605_20179_amd import binding as tb
    wl = ti.TideWorkload("p12-large", d=1024, E=32, k=4, I=1024, n_shared=1, N=640, S=1, K=1, C=16, L=1,
                         gating=ti.GATING_SIGMOID, bias_mode=ti.BIAS_NONE, seed=4242)
    rng = np.random.default_rng(77)
    resident = [int(e) for e in ti.initial_resident(wl)]
    want = [33, 40, 48, 64, 70, 80, 96, 100, 112, 128, 140, 160, 176, 192, 200, 400]
    rows_of_expert = dict(zip(resident, want))
    idx = _forced_routing(wl, rows_of_expert, rng)
    w = rng.random((wl.N, wl.k)).astype(np.float32)
    w /= w.sum(axis=1, keepdims=True)
    raw_expert = resident[3]

    def expert_bits(e):
        wg, wu, wd = ti.expert_weights(wl, 0, e)
        if e == raw_expert:                          # 17 distinct high bytes (tiny values) in one tile: cannot be encoded
            wd = wd.copy()
            wd[0, :17] = (np.arange(17, dtype=np.uint16) + 0x20) << 8
        return wg, wu, wd

    hidden = next(iter(ti.hidden_stream(wl, 0)))
    store = orc.ExpertStore(expert_bits)
    shared = tuple(orc.bf16_to_f64(m) for m in expert_bits(wl.E))
    slot_of = orc.slot_table(ti.initial_resident(wl), wl.E)
    y_res, y_full, miss = orc.moe_outputs(hidden, idx, w.astype(np.float64), slot_of, store, shared)

    bf16, p12 = _sessions(wl, expert_bits)
    assert raw_expert in _check_slots(p12, resident)
    outs = []
    for s in (bf16, p12):
        x = s.to_device_bf16(hidden)
        s.step_routed(0, x, torch.from_numpy(idx).to(s.device), torch.from_numpy(w).to(s.device))
        out, _, _, gmiss, n_miss = s.results(wl.N)
        tp.check_miss(miss, gmiss, n_miss)
        tp.check_out(out, y_res)
        items, row_token = tb.tide_read_work_items(s.ctx, 4096, 65536, torch.cuda.current_stream())
        s.apply_misses(0, x)
        torch.cuda.synchronize()
        full = s.out[:wl.N].cpu().numpy()
        tp.check_out(full, y_full)
        outs.append((out, full, items))
    assert np.array_equal(outs[0][0], outs[1][0]), "resident part differs between bf16 and 12-bit slots"
    assert np.array_equal(outs[0][1], outs[1][1])
    big = [it for it in outs[1][2] if it["kind"] == 1]
    tiles = sorted({(int(it["nrows"]) + 15) // 16 for it in big})
    tp.say("12-bit large items: %d, token tiles per item %s" % (len(big), tiles))
    assert big and max(int(it["nrows"]) for it in big) <= 192
    assert set(tiles) >= {3, 4, 5, 6, 7, 8, 9, 10, 11, 12}, tiles
    assert max(int(it["nrows"]) for it in outs[0][2] if it["kind"] == 1) > 192      # bf16 slots keep the 256-row limit
    bf16.close()
    p12.close()


def test_12bit_slots_need_the_compressed_blobs():
    """Error paths: no placement and no unregistering without the compressed blobs; registering them again withdraws
    the placement until tide_set_resident is called again."""
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    wl = ti.CONFIGS[0]
    sess = TideSession(wl.d, wl.E, wl.k, wl.I, wl.n_shared, wl.C, wl.N, wl.gating, wl.bias_mode, resident_p12=True)
    packed = sess.pack_layer(lambda e: ti.expert_weights(wl, 0, e), workers=4)
    sess.host_blobs[0] = packed[0]
    tb.tide_register_experts(sess.ctx, 0, packed[0], sess.blob_bytes)
    with pytest.raises(tb.TideError) as ei:
        tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    assert ei.value.code == tb.TIDE_E_STATE
    sess.compress_layer(0, workers=4)
    with pytest.raises(tb.TideError) as ei:
        tb.tide_register_compressed(sess.ctx, 0, None, 0)
    assert ei.value.code == tb.TIDE_E_STATE
    if wl.n_shared:
        tb.tide_set_shared(sess.ctx, 0, packed[1])
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    sess.router_w[0] = torch.from_numpy(np.ascontiguousarray(ti.router_weights(wl, 0), dtype=np.float32)).to(sess.device)
    bias = ti.router_bias(wl, 0)
    sess.router_b[0] = None if bias is None else torch.from_numpy(np.ascontiguousarray(bias, dtype=np.float32)).to(sess.device)
    x = sess.to_device_bf16(next(iter(ti.hidden_stream(wl, 0))))
    sess.step(0, x)
    want = sess.results(wl.N)[0].copy()
    # registering compressed blobs again withdraws the placement: the slots were filled from the earlier ones
    sess.compress_layer(0, workers=4)
    with pytest.raises(tb.TideError) as ei:
        sess.step(0, x)
    assert ei.value.code == tb.TIDE_E_STATE
    with pytest.raises(tb.TideError) as ei:
        sess.refresh(0)
    assert ei.value.code == tb.TIDE_E_STATE
    tb.tide_set_resident(sess.ctx, 0, ti.initial_resident(wl))
    sess.stats(0, reset=True)
    sess.step(0, x)
    assert np.array_equal(sess.results(wl.N)[0], want)
    sess.close()
