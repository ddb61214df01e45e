"""Host-side checks of libtide that need no GPU: the library loads, exports every
symbol include/tide.h declares, validates configurations, packs expert weights into
the documented tile order, and refuses to create a context without a device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def tb():
    from paper_2605_20179_amd import binding
    return binding


def test_every_declared_symbol_is_exported(tb):
    header = open(os.path.join(ROOT, "include", "tide.h")).read()
    declared = set(re.findall(r"\b(tide_[a-z_0-9]+)\s*\(", header))
    declared -= {"tide_ctx"}
    assert declared, "no declarations found"
    lib = ctypes.CDLL(tb.LIB_PATH)
    for name in sorted(declared):
        assert hasattr(lib, name), "libtide.so does not export %s" % name
    assert declared == set(tb.EXPORTS)


def test_struct_layouts_match_the_header(tb):
    assert ctypes.sizeof(tb.tide_miss) == 12
    assert ctypes.sizeof(tb.tide_copy) == 24
    assert ctypes.sizeof(tb.tide_config) == 44
    assert tb.MISS_DTYPE.itemsize == 12


def test_pack_layout(tb):
    """A tile of 16 rows x 32 columns is 512 contiguous elements; lane l holds row stripe*16 + l%16,
    columns kc*32 + (l/16)*8 .. +7.  Stripes are stored in groups, K chunk slow inside a group:
    gate/up groups hold 8 SwiGLU column blocks (their gate stripes, then their up stripes), down
    groups 16 stripes; a last partial group holds fewer.  The down matrix follows gate/up."""
    d, I = 320, 192          # 10 K chunks; 12 column blocks (8 + 4); 20 down stripes (16 + 4)
    cfg = tb.make_config(d, 8, 2, I, 0, 1, 4, 8, 0, 0)
    rng = np.random.default_rng(3)
    wg, wu = (rng.integers(0, 2 ** 16, size=(I, d), dtype=np.uint16) for _ in range(2))
    wd = rng.integers(0, 2 ** 16, size=(d, I), dtype=np.uint16)
    blob = np.zeros(tb.tide_expert_blob_bytes(cfg), dtype=np.uint8)
    assert blob.size == 3 * d * I * 2
    tb.tide_pack_expert(cfg, wg, wu, wd, blob)
    b = blob.view(np.uint16)

    def check_tile(at, mat, stripe, kc):
        tile = b[at * 512:(at + 1) * 512].reshape(64, 8)
        for l in (0, 1, 15, 16, 37, 63):
            want = mat[stripe * 16 + l % 16, kc * 32 + (l // 16) * 8: kc * 32 + (l // 16) * 8 + 8]
            assert np.array_equal(tile[l], want), (at, stripe, kc, l)

    kch, blocks = d // 32, I // 16
    for g in range((blocks + 7) // 8):
        ng = min(8, blocks - 8 * g)
        for kc in range(kch):
            for j in range(ng):
                check_tile(g * 16 * kch + kc * 2 * ng + j, wg, 8 * g + j, kc)
                check_tile(g * 16 * kch + kc * 2 * ng + ng + j, wu, 8 * g + j, kc)
    kch, stripes, base = I // 32, d // 16, 2 * d * I // 512
    for g in range((stripes + 15) // 16):
        ng = min(16, stripes - 16 * g)
        for kc in range(kch):
            for j in range(ng):
                check_tile(base + g * 16 * kch + kc * ng + j, wd, 16 * g + j, kc)
    # a permutation: nothing lost, nothing duplicated
    assert np.array_equal(np.sort(b), np.sort(np.concatenate([wg.ravel(), wu.ravel(), wd.ravel()])))


@pytest.mark.parametrize("d,d_ff,m", [(256, 128, 1), (320, 192, 3), (320, 192, 6), (512, 256, 9)])
def test_host_expert_matches_the_oracle(tb, d, d_ff, m):
    """The host cores' expert path (Sec. 3.3: misses run on CPU experts) reads the packed blob in place;
    checked here against the oracle's e(x), full and ragged stripe groups, one to three token blocks."""
    import sys
    sys.path.insert(0, ROOT)
    from oracle import tide_oracle as orc
    cfg = tb.make_config(d, 8, 2, d_ff, 0, 1, 4, 16, 0, 0)
    rng = np.random.default_rng(d + m)
    def bits(shape, scale):          # any bf16 bit patterns will do: fp32 draws cut to their upper halves
        return (np.ascontiguousarray(rng.normal(0, scale, size=shape), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    wg, wu, wd, x = bits((d_ff, d), 0.05), bits((d_ff, d), 0.05), bits((d, d_ff), 0.05), bits((m, d), 1.0)
    blob = np.zeros(tb.tide_expert_blob_bytes(cfg), dtype=np.uint8)
    tb.tide_pack_expert(cfg, wg, wu, wd, blob)
    got = tb.tide_host_expert(cfg, blob, x)
    W = [orc.bf16_to_f64(w) for w in (wg, wu, wd)]
    want = np.stack([orc.expert_ffn(orc.bf16_to_f64(x[t]), *W) for t in range(m)])
    rms = float(np.sqrt(np.mean(want ** 2)))
    assert rms > 0
    assert np.max(np.abs(got - want)) <= 2e-3 * rms, np.max(np.abs(got - want)) / rms


@pytest.mark.parametrize("n_tokens,n_experts,k,threads,shuffle", [(5, 6, 2, 1, False), (40, 6, 3, 3, False), (9, 40, 4, 2, True)])
def test_host_miss_path_matches_the_oracle(tb, n_tokens, n_experts, k, threads, shuffle):
    """The host workers' grouping, threading and per-token summation against the definition: out[token] +=
    w * e(x_token) for every listed (token, expert, w).  Few experts per thread (each expert cut into its column
    groups) and many (one work item per expert); list in token order and shuffled; the result lands on top of
    what out already holds."""
    import sys
    sys.path.insert(0, ROOT)
    from oracle import tide_oracle as orc
    d, d_ff = 192, 192
    cfg = tb.make_config(d, n_experts, k, d_ff, 0, 1, 1, 64, 0, 0)
    rng = np.random.default_rng(n_tokens * 100 + n_experts)
    def bits(shape, scale):
        return (np.ascontiguousarray(rng.normal(0, scale, size=shape), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    W = [(bits((d_ff, d), 0.08), bits((d_ff, d), 0.08), bits((d, d_ff), 0.08)) for _ in range(n_experts)]
    blobs = np.zeros((n_experts, tb.tide_expert_blob_bytes(cfg)), dtype=np.uint8)
    for e, (wg, wu, wd) in enumerate(W):
        tb.tide_pack_expert(cfg, wg, wu, wd, blobs[e])
    x = bits((n_tokens, d), 1.0)
    entries = []
    for t in range(n_tokens):
        if t % 4 == 3:
            continue                                             # a token without misses keeps its row
        for e in rng.choice(n_experts, size=int(rng.integers(1, k + 1)), replace=False):
            entries.append((t, int(e), float(rng.uniform(0.05, 0.6))))
    if shuffle:
        rng.shuffle(entries)
    miss = np.array(entries, dtype=tb.MISS_DTYPE)
    base = rng.normal(0, 1, size=(n_tokens, d)).astype(np.float32)
    got = base.copy()
    tb.tide_host_misses(cfg, blobs, x, miss, threads, got)
    want = base.astype(np.float64)
    Wf = [tuple(orc.bf16_to_f64(m) for m in w) for w in W]
    for t, e, w in entries:
        want[t] += np.float32(w).astype(np.float64) * orc.expert_ffn(orc.bf16_to_f64(x[t]), *Wf[e])
    rms = float(np.sqrt(np.mean((want - base) ** 2)))
    assert np.max(np.abs(got - want)) <= 2e-3 * rms
    untouched = [t for t in range(n_tokens) if t % 4 == 3]
    assert np.array_equal(got[untouched], base[untouched])
    # a bad entry: refused, nothing added
    bad = miss.copy()
    bad[len(bad) // 2]["expert"] = n_experts
    again = base.copy()
    with pytest.raises(tb.TideError) as ei:
        tb.tide_host_misses(cfg, blobs, x, bad, threads, again)
    assert ei.value.code == tb.TIDE_E_INVAL and np.array_equal(again, base)


def _p12_table_slots(d: int, I: int) -> np.ndarray:
    """Table slot of every payload tile: payloads are ordered K chunk first inside a stripe group of the packed layout
    (8 SwiGLU column blocks = up to 16 gate / up stripes; 16 down stripes), tables stripe first."""
    slots = []
    at = 0
    for stripes_total, per_group, chunks in ((2 * (I // 16), 16, d // 32), (d // 16, 16, I // 32)):
        done = 0
        while done < stripes_total:
            w = min(per_group, stripes_total - done)
            for c in range(chunks):
                for j in range(w):
                    slots.append(at + j * chunks + c)
            at += w * chunks
            done += w
    return np.asarray(slots, dtype=np.int64)


def _p12_decode(comp: np.ndarray, n_tiles: int, d: int, I: int) -> np.ndarray:
    """Decoder written from the format's description in include/tide.h and csrc/packed12.h, independent of the
    library: a 128-byte header; per tile 64 lanes x 3 dwords (the low bytes of the lane's elements 0..3 and 4..7, then one byte
    per element pair j, 4+j holding their two 4-bit table indices); per tile a table of 16 high bytes, stored stripe first."""
    hdr = comp[:64].view(np.uint32)
    assert hdr[0] == 0x32315054 and hdr[1] == n_tiles and hdr[2] == 0
    off_table = 128 + n_tiles * 768
    words = comp[128:off_table].view(np.uint32).reshape(n_tiles, 64, 3).astype(np.int64)
    slots = _p12_table_slots(d, I)
    assert len(slots) == n_tiles and len(set(slots.tolist())) == n_tiles
    table = comp[off_table:off_table + 16 * n_tiles].reshape(n_tiles, 16).astype(np.int64)[slots]
    vals = np.zeros((n_tiles, 64, 8), dtype=np.int64)
    for j in range(8):
        low = (words[:, :, j // 4] >> (8 * (j % 4))) & 0xff
        code = (words[:, :, 2] >> (8 * (j % 4) + (0 if j < 4 else 4))) & 0xf
        vals[:, :, j] = low | (np.take_along_axis(table, code, axis=1) << 8)
    return vals.astype(np.uint16).reshape(-1)


def test_compressed_blob_round_trip(tb):
    """The 12-bit form is lossless: decoding it (here by hand, and with the library's own inverse) gives back the
    packed blob bit for bit -- for Gaussian weights, for weights with zeros / denormals / infinities / NaNs sprinkled
    in, for a tile that uses all 16 table entries -- and a blob with a tile of 17 distinct high bytes is marked raw."""
    d, I = 320, 192          # partial gate/up and down groups (12 column blocks, 20 down stripes)
    cfg = tb.make_config(d, 8, 2, I, 0, 1, 4, 8, 0, 0)
    n_tiles = 3 * d * I // 512
    cbytes = tb.tide_compressed_blob_bytes(cfg)
    assert cbytes % 64 == 0 and cbytes == 128 + n_tiles * (768 + 16) and cbytes < 0.77 * tb.tide_expert_blob_bytes(cfg)
    rng = np.random.default_rng(12)
    def bits(shape, scale):
        return (np.ascontiguousarray(rng.normal(0, scale, size=shape), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    blob = np.zeros(tb.tide_expert_blob_bytes(cfg), dtype=np.uint8)
    comp = np.zeros(cbytes, dtype=np.uint8)
    back = np.zeros_like(blob)

    def round_trip(src_u16):
        tb.tide_compress_expert(cfg, src_u16.view(np.uint8), comp)
        assert np.array_equal(_p12_decode(comp, n_tiles, d, I), src_u16)
        back[:] = 0xAA
        tb.tide_decompress_expert(cfg, comp, back)
        assert np.array_equal(back.view(np.uint16), src_u16)

    # Gaussian weights
    tb.tide_pack_expert(cfg, bits((I, d), 0.02), bits((I, d), 0.02), bits((d, I), 0.02), blob)
    round_trip(blob.view(np.uint16))
    # zeros, negative zeros, denormals, tiny and huge values, infinities and NaNs sprinkled in
    raw = blob.view(np.uint16).copy()
    at = rng.choice(raw.size, size=60, replace=False)
    raw[at] = np.resize(np.array([0x0000, 0x8000, 0x0001, 0x807f, 0x0080, 0x7f7f, 0xff80, 0x7fc1, 0x1234, 0x3f80], dtype=np.uint16), 60)
    round_trip(raw)
    # a tile whose elements use exactly 16 distinct high bytes still encodes ...
    full = blob.view(np.uint16).copy()
    full[512 * 5:512 * 6] = (np.resize(np.arange(16, dtype=np.uint16) * 9 + 3, 512) << 8) | rng.integers(0, 256, 512, dtype=np.uint16)
    round_trip(full)
    # ... a 17th does not: the blob is marked raw, and the inverse refuses it
    full[512 * 5 + 100] = 0xF1 << 8
    tb.tide_compress_expert(cfg, full.view(np.uint8), comp)
    assert comp[:64].view(np.uint32)[2] == 1
    with pytest.raises(tb.TideError) as ei:
        tb.tide_decompress_expert(cfg, comp, back)
    assert ei.value.code == tb.TIDE_E_INVAL
    # exponents all over the range: raw as well
    wild = rng.integers(0, 2 ** 16, size=raw.size, dtype=np.uint16)
    tb.tide_compress_expert(cfg, wild.view(np.uint8), comp)
    assert comp[:64].view(np.uint32)[2] == 1


@pytest.mark.parametrize("d,I", [(64, 64), (128, 192), (192, 448), (512, 320), (1024, 128)])
def test_compressed_blob_table_order_on_other_shapes(tb, d, I):
    """Whole and partial stripe groups in both matrices: the tables' stripe-first order is a permutation of the tiles
    and the hand decoder, which applies it, gives back the blob."""
    cfg = tb.make_config(d, 4, 2, I, 0, 1, 2, 8, 0, 0)
    n_tiles = 3 * d * I // 512
    slots = _p12_table_slots(d, I)
    assert sorted(slots.tolist()) == list(range(n_tiles))
    rng = np.random.default_rng(d * 7 + I)
    blob = (np.ascontiguousarray(rng.normal(0, 0.05, size=3 * d * I), dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    comp = np.zeros(tb.tide_compressed_blob_bytes(cfg), dtype=np.uint8)
    tb.tide_compress_expert(cfg, blob.view(np.uint8), comp)
    if comp[:64].view(np.uint32)[2]:
        pytest.skip("this draw has a tile with more than 16 distinct high bytes")
    assert np.array_equal(_p12_decode(comp, n_tiles, d, I), blob)
    back = np.zeros(blob.size * 2, dtype=np.uint8)
    tb.tide_decompress_expert(cfg, comp, back)
    assert np.array_equal(back.view(np.uint16), blob)


def test_config_validation_and_no_device(tb):
    ok = dict(d=256, n_experts=16, top_k=2, d_ff=128, n_shared=0, n_layers=1, capacity=8, max_tokens=8, gating=0, bias_mode=0)
    blob = np.zeros(3 * 256 * 128 * 2, dtype=np.uint8)
    w = np.zeros((128, 256), dtype=np.uint16)
    for bad, code in ((dict(d=100), tb.TIDE_E_INVAL), (dict(d_ff=96), tb.TIDE_E_INVAL), (dict(n_experts=0), tb.TIDE_E_INVAL),
                      (dict(n_experts=513), tb.TIDE_E_INVAL), (dict(top_k=17), tb.TIDE_E_INVAL), (dict(top_k=0), tb.TIDE_E_INVAL),
                      (dict(capacity=17), tb.TIDE_E_RANGE), (dict(capacity=0), tb.TIDE_E_RANGE), (dict(n_shared=2), tb.TIDE_E_INVAL),
                      (dict(gating=5), tb.TIDE_E_INVAL), (dict(bias_mode=3), tb.TIDE_E_INVAL), (dict(max_tokens=0), tb.TIDE_E_RANGE)):
        cfg = tb.make_config(**{**ok, **bad})
        rc = tb.lib.tide_pack_expert(ctypes.byref(cfg), w.ctypes.data, w.ctypes.data, w.ctypes.data, blob.ctypes.data)
        assert rc == code, (bad, rc)
        assert tb.lib.tide_last_error(None)
    import torch
    if not torch.cuda.is_available():
        with pytest.raises(tb.TideError) as ei:
            tb.tide_create(tb.make_config(**ok))
        assert ei.value.code == tb.TIDE_E_HIP        # no silent CPU path
        from paper_2605_20179_amd.session import TideSession
        with pytest.raises(RuntimeError):
            TideSession(256, 16, 2, 128, 0, 8, 8, 0, 0)
