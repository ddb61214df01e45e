"""GPU check of the 12-bit refresh source: a refresh whose copies read the compressed form of the expert blobs
must leave every cache slot bit-identical to the raw blob of the expert the table names (immediate and deferred
refresh; Gaussian experts, experts with zeros / denormals / outliers, an expert stored raw), and nothing else
about the refresh (resident set, plan, counters) may change."""
import numpy as np
import pytest
import torch

import tide_inputs as ti
import test_gpu_parity as tp

pytestmark = pytest.mark.gpu


def _bits(rng, shape, scale):
    return (np.ascontiguousarray(rng.normal(0, scale, size=shape), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)


@pytest.mark.parametrize("deferred", [False, True])
def test_slots_are_bit_identical_after_a_compressed_refresh(deferred):
    from paper_2605_20179_amd import binding as tb
    from paper_2605_20179_amd.session import TideSession
    d, I, E, C, N, k = 256, 192, 24, 8, 8, 2
    tp.say("compressed refresh, deferred=%s" % deferred)
    rng = np.random.default_rng(5)
    specials = np.array([0x0000, 0x8000, 0x0001, 0x807f, 0x0080, 0x7f7f, 0xff80, 0x7fc1, 0x1234, 0x3f80], dtype=np.uint16)

    def expert_bits(e):
        wg, wu, wd = _bits(rng, (I, d), 0.02), _bits(rng, (I, d), 0.02), _bits(rng, (d, I), 0.02)
        if e % 3 == 1:                                   # a few zeros, denormals, infinities, NaNs
            for m in (wg, wu, wd):
                at = rng.choice(m.size, size=7, replace=False)
                m.reshape(-1)[at] = specials[:7]
        if e == 20:                                      # exponents everywhere: stored raw
            wd = rng.integers(0, 2 ** 16, size=(d, I), dtype=np.uint16)
        return wg, wu, wd

    sess = TideSession(d, E, k, I, 0, C, N, ti.GATING_SOFTMAX, ti.BIAS_NONE)
    sess.load_layer(0, expert_bits, _bits(rng, (E, d), 0.02).astype(np.float32), None, np.arange(C), workers=1)
    sess.compress_layer(0, workers=2)
    comp = sess.comp_blobs[0].numpy()
    raw_flags = [int(comp[e][:64].view(np.uint32)[2]) for e in range(E)]
    assert raw_flags[20] == 1 and sum(raw_flags) == 1
    raw = sess.host_blobs[0].numpy()
    # three refreshes from caller-supplied counts: bring in experts 8..15, then 16..23, then a mix
    for wanted in (range(8, 16), range(16, 24), (1, 4, 20, 7, 13, 22, 10, 19)):
        counts = np.zeros(E, dtype=np.int32)
        counts[list(wanted)] = 5
        eis, plan = sess.refresh(0, counts=counts, deferred=deferred)
        assert sorted(eis.tolist()) == sorted(wanted)
        assert all(b == sess.blob_bytes and off == e * sess.blob_bytes for e, s, off, b in plan)
        if deferred:
            sess.commit(0)
        torch.cuda.synchronize()
        table = sess.table(0)
        for s in range(C):
            e = int(eis[s])
            assert table[e] == s
            assert np.array_equal(sess.read_slot(0, s), raw[e]), "slot %d (expert %d) differs from the raw blob" % (s, e)
    # back to raw copies: same result
    tb.tide_register_compressed(sess.ctx, 0, None, 0)
    counts = np.zeros(E, dtype=np.int32)
    counts[:C] = 3
    eis, _ = sess.refresh(0, counts=counts)
    for s in range(C):
        assert np.array_equal(sess.read_slot(0, s), raw[int(eis[s])])
    sess.close()


def test_block_with_compressed_refresh_matches_the_oracle():
    """The cfg 1 block, refresh copies from the compressed blobs: routing, counters, plans, miss lists and outputs as
    in the plain run (the same comparison against the oracle)."""
    wl = ti.CONFIGS[1]
    out_steps = [0, 4, 5]
    log, hidden = tp.oracle_block(wl, 0, out_steps)
    sess = tp._session(wl)
    tp.load(sess, wl, 0)
    sess.compress_layer(0, workers=8)
    flips, worst = tp.run_block_on_gpu(wl, 0, sess, log, hidden, True, out_steps)
    tp.say("cfg1 with compressed refresh: worst out err %.2e x RMS" % worst)
    eis = log[-1]["expert_in_slot"]
    for s in (0, wl.C // 2, wl.C - 1):
        assert np.array_equal(sess.read_slot(0, s), sess.host_blobs[0][int(eis[s])].numpy())
    sess.close()
