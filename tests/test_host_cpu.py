"""CPU-only tests of the native library's host side: exported symbols, the offline weight
transform (bit-exact against the oracle's format writer and the paper's worked example),
the test-mask generator (bit-exact against the seeded generator module) and every error
path of the C ABI that needs no GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2407_19644_amd as ubp
from synthetic import CONFIGS, make_weights, select_blocks

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "ubp.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(ubp_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(ubp.EXPORTS)
    lib = ctypes.CDLL(ubp.library_path())
    for name in declared:
        assert getattr(lib, name) is not None


def test_status_strings():
    seen = {ubp.status_string(c) for c in range(8)}
    assert len(seen) == 8 and "ok" in seen


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_select_reference_matches_seeded_generator(cfg):
    mode = 1 if cfg.mask_mode == "zipf" else 0
    got = ubp.select_reference(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed, mode, cfg.zipf_s)
    want = select_blocks(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed, cfg.mask_mode, cfg.zipf_s)
    assert np.array_equal(got, want)
    assert len(got) == ubp.target_block_count(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density)
    assert oracle.validate(cfg.M, cfg.K, cfg.bh, cfg.bw, got) == len(got) * cfg.bh * cfg.bw
    again = ubp.select_reference(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed, mode, cfg.zipf_s)
    assert np.array_equal(got, again)
    other = ubp.select_reference(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed + 1, mode, cfg.zipf_s)
    assert not np.array_equal(got, other)


def test_block_counts_of_the_five_layers():
    assert [ubp.target_block_count(c.M, c.K, c.bh, c.bw, c.density) for c in CONFIGS] == [128, 2880, 819, 9216, 6553]


def test_zipf_stripe_counts_are_skewed_and_capped():
    c = CONFIGS[4]
    b = ubp.select_reference(c.M, c.K, c.bh, c.bw, c.density, c.mask_seed, 1, c.zipf_s)
    per = np.bincount(b[:, 0] // c.bh, minlength=256)
    cap = int(0.375 * c.K / c.bw)
    assert per.max() == cap and (per == cap).sum() == 21 and per.min() == 6 and per.sum() == 6553


def test_select_reference_errors():
    L = ubp.load_library()
    nb = ctypes.c_int64(0)
    buf = np.zeros((4, 2), np.int32)
    # capacity too small: reports the needed count
    rc = L.ubp_select_reference(64, 64, 4, 4, 0.5, 1, 0, 0.0, buf.ctypes.data, 4, ctypes.byref(nb))
    assert rc == 1 and nb.value == 128
    assert L.ubp_select_reference(64, 64, 4, 4, 0.5, 1, 7, 0.0, buf.ctypes.data, 4, ctypes.byref(nb)) == 1
    assert L.ubp_select_reference(64, 64, 0, 4, 0.5, 1, 0, 0.0, buf.ctypes.data, 4, ctypes.byref(nb)) == 1
    assert L.ubp_select_reference(64, 64, 4, 4, 1.5, 1, 0, 0.0, buf.ctypes.data, 4, ctypes.byref(nb)) == 1
    assert L.ubp_select_reference(64, 64, 4, 4, 0.5, 1, 0, 0.0, buf.ctypes.data, 4, None) == 1
    # density above the jamming limit of random sequential placement cannot be reached
    big = np.zeros((256, 2), np.int32)
    rc = L.ubp_select_reference(64, 64, 4, 4, 0.98, 1, 0, 0.0, big.ctypes.data, 256, ctypes.byref(nb))
    assert rc == 5
    # zipf: more blocks than the capped stripes can hold
    rc = L.ubp_select_reference(64, 64, 4, 4, 0.9, 1, 1, 1.1, big.ctypes.data, 256, ctypes.byref(nb))
    assert rc == 5


def test_pack_worked_example(worked_example):
    g, val = worked_example
    M, K, bh, bw = (int(g[k][0][0]) for k in ("M", "K", "bh", "bw"))
    W = np.zeros((M, K), np.float32)
    blocks = []
    for r, c, *letters in g["block"]:
        blocks.append((int(r), int(c)))
        for d, L in enumerate(letters):
            W[int(r) + d, int(c)] = val[L]
    for order in ([0, 1, 2, 3], [3, 2, 1, 0], [2, 0, 3, 1]):
        p = ubp.pack(W, "f32", bh, bw, [blocks[t] for t in order])
        assert p.indptr.tolist() == [int(t) for t in g["indptr"][0]]
        assert p.indices.tolist() == [int(t) for t in g["indices"][0]]
        assert p.values.tolist() == [val[L] for L in g["values"][0]]
        p.free()


@pytest.mark.parametrize("cfg", CONFIGS, ids=lambda c: c.name)
def test_pack_bit_exact_on_the_five_layers(cfg):
    blocks = select_blocks(cfg.M, cfg.K, cfg.bh, cfg.bw, cfg.density, cfg.mask_seed, cfg.mask_mode, cfg.zipf_s)
    W = make_weights(cfg.M, cfg.K, cfg.w_seed, cfg.dtype)
    shuffled = blocks[np.random.default_rng(1).permutation(len(blocks))]
    p = ubp.pack(W, cfg.dtype, cfg.bh, cfg.bw, shuffled)
    indptr, indices, values = oracle.pack(W, cfg.bh, cfg.bw, blocks)
    assert len(p.indptr) == cfg.M - cfg.bh + 2
    assert np.array_equal(p.indptr, indptr) and np.array_equal(p.indices, indices)
    assert np.array_equal(p.values.view(np.uint8), values.view(np.uint8))
    assert p.info(4) == len(blocks) and p.info(6) == -1
    p.free()


@pytest.mark.parametrize("bh,bw,dtype", [(3, 1, "f32"), (1, 1, "f16"), (5, 7, "bf16"), (16, 2, "f16"), (20, 3, "bf16")])
def test_pack_odd_shapes_and_pitch(bh, bw, dtype):
    rng = np.random.default_rng(bh * 100 + bw)
    M, K, ld = 61, 53, 64
    blocks = select_blocks(M, K, bh, bw, 0.3, seed=5)
    raw = rng.integers(1, 30000, size=(M, ld))
    Wbig = raw.astype({"f32": np.float32, "f16": np.float16, "bf16": np.uint16}[dtype])
    W = Wbig[:, :K]                      # leading dimension 64 > K
    p = ubp.pack(W, dtype, bh, bw, blocks)
    indptr, indices, values = oracle.pack(np.ascontiguousarray(W), bh, bw, blocks)
    assert np.array_equal(p.indptr, indptr) and np.array_equal(p.indices, indices)
    assert np.array_equal(p.values.view(np.uint8), values.view(np.uint8))
    p.free()


def test_pack_rejects_invalid_block_lists():
    W = np.ones((8, 8), np.float32)
    for bad, code in [([(0, 0), (3, 3)], 3), ([(0, 0), (0, 0)], 3), ([(5, 0)], 2), ([(0, 5)], 2),
                      ([(-1, 0)], 2), ([(0, -1)], 2)]:
        with pytest.raises(ubp.UBPError) as e:
            ubp.pack(W, "f32", 4, 4, bad)
        assert e.value.code == code
    L = ubp.load_library()
    out = ctypes.c_void_p(None)
    blk = np.zeros((1, 2), np.int32)
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 8, 4, 4, blk.ctypes.data, 1, -1, None) == 1
    assert L.ubp_pack(W.ctypes.data, 9, 8, 8, 8, 4, 4, blk.ctypes.data, 1, -1, ctypes.byref(out)) == 1
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 4, 4, 4, blk.ctypes.data, 1, -1, ctypes.byref(out)) == 1   # ldw < K
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 8, 0, 4, blk.ctypes.data, 1, -1, ctypes.byref(out)) == 1
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 8, 4, 4, None, 1, -1, ctypes.byref(out)) == 1
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 8, 4, 4, blk.ctypes.data, -1, -1, ctypes.byref(out)) == 1
    assert L.ubp_pack(W.ctypes.data, 0, 8, 8, 8, 4, 4, blk.ctypes.data, 1, -2, ctypes.byref(out)) == 1
    assert out.value is None


def test_empty_block_list_packs():
    p = ubp.pack(np.ones((8, 8), np.float16), "f16", 4, 4, np.zeros((0, 2), np.int32))
    assert p.indptr.tolist() == [0] * 6 and len(p.indices) == 0 and len(p.values) == 0
    p.free()


def test_spmm_argument_errors_need_no_gpu():
    L = ubp.load_library()
    p = ubp.pack(np.ones((8, 8), np.float32), "f32", 4, 4, [(0, 0)])
    h = p.handle
    assert L.ubp_spmm(None, 1, 8, 8, 1, 8, 0, None) == 1
    assert L.ubp_spmm(h, 16, 8, 8, 32, 8, 0, None) == 1      # host-only handle
    assert L.ubp_spmm(h, 16, 8, -1, 32, 8, 0, None) == 1
    assert L.ubp_packed_info(h, 99) == -1 and L.ubp_packed_info(None, 0) == -1
    L.ubp_packed_free(None)
    p.free()
