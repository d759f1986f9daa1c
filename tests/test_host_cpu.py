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


# ---------------------------------------------------------------- private MFMA layouts
def _ring_swizzle(CT, r):
    return ((r >> 2) & 1) if CT == 2 else ((r >> 1) & 3) if CT == 4 else (r & 7)


def _decode_layout(packed, G, CT, M, K):
    """Replays what the gather kernel does with a layout's step records, on the host and for the
    weights only: which X row every gathered entry is (ring address -> row, through the
    chunks the control words say are held) and which output rows every operand value feeds.
    Returns the dense matrix the records stand for (16-bit patterns) and the MFMA count."""
    rg_ptr, rg_order, stream = packed.layout(G, CT, 1)
    nrg = len(rg_order)
    assert sorted(rg_order.tolist()) == list(range(nrg))
    rec_dw = 128 + 256 * G
    PITCH, RR = 32 * CT, 131072 // (32 * CT)
    R = RR // 64
    nch = -(-K // 64)
    assert len(stream) == (rg_ptr[-1] + 4) * rec_dw          # four spare records at the end
    lanes = np.arange(64)
    g, t = lanes // 16, lanes % 16
    e_in, sub = t // 4, (t % 4) * 8
    idx_lo, idx_hi = 4 * g + e_in, 16 + 4 * g + e_in         # entry of the lane's two reads
    Wd = np.zeros((nrg * 16 * G, K), dtype=np.uint16)
    mfma = 0
    for rg in range(nrg):
        assert (rg_ptr[rg + 1] - rg_ptr[rg]) % 4 == 0
        prev_rel = 0
        for s in range(rg_ptr[rg], rg_ptr[rg + 1]):
            rec = stream[s * rec_dw:(s + 1) * rec_dw]
            d0, d1 = rec[0:128:2], rec[1:128:2]
            mask = int(d0[0] >> 28)
            assert np.all(d0 >> 28 == mask)
            ctl = int(d1[0])
            assert np.all(d1 == ctl)
            need, rel = ctl & 0xffff, ctl >> 16
            assert prev_rel <= rel <= nch                    # chunks are handed back in order
            prev_rel = rel
            if mask == 0:
                assert not rec[128:].any()                   # an empty step carries no weights
                continue
            assert rel <= need < nch and need - rel <= R - 2  # held chunks leave two ring slots free
            mfma += bin(mask).count("1")
            ks = np.zeros((2, 64), dtype=np.int64)
            for h, addr in enumerate(((d0 & 0x3fff).astype(np.int64) << 3, ((d0 >> 14) & 0x3fff).astype(np.int64) << 3)):
                r = addr // PITCH
                assert np.all(r < min(RR, nch * 64))
                sw = np.array([_ring_swizzle(CT, int(x)) for x in r])
                assert np.array_equal(addr % PITCH, (sw << 5) + sub)      # unit 0 of the row, swizzled, lane's 8 bytes
                k = r + RR * ((rel * 64 - r + RR - 1) // RR)              # first row >= rel*64 congruent to r
                assert np.all(k >= rel * 64) and np.all(k < (need + 1) * 64) and np.all(k < K)
                ks[h] = k
            # the four lanes of a quad read the same row; entry -> row
            krow = np.zeros(32, dtype=np.int64)
            krow[idx_lo], krow[idx_hi] = ks[0], ks[1]
            assert np.array_equal(krow[idx_lo], ks[0]) and np.array_equal(krow[idx_hi], ks[1])
            frag = rec[128:].view(np.uint16).reshape(G, 64, 8)
            ent = np.concatenate([(4 * g)[:, None] + np.arange(4), (16 + 4 * g)[:, None] + np.arange(4)], axis=1)  # [64, 8]
            for j in range(G):
                if not (mask >> j) & 1:
                    assert not frag[j].any()
                    continue
                vals = frag[j]
                rows = (rg * G + j) * 16 + t                                  # [64]
                rr = np.repeat(rows[:, None], 8, axis=1)
                kk = krow[ent]
                nz = vals != 0
                assert not Wd[rr[nz], kk[nz]].any()            # no weight is delivered twice
                Wd[rr[nz], kk[nz]] = vals[nz]
    assert not Wd[M:].any()
    return Wd[:M], mfma


def _decode_block_layout(packed, G, M, K):
    """The same for the block kernel's layout: the window rows a lane reads (entry i of a half =
    the window row congruent to i modulo 16), the stripe a row-slot's weight goes to (rows
    n >= o: the stripe the block starts in, rows n < o: the next one), the chunks a step needs
    against the chunks handed back.  Returns the dense matrix (16-bit patterns) and the MFMA count."""
    rg_ptr, rg_order, recs, meta = packed.layout(G, 0, 2)
    nrg = len(rg_ptr) - 1
    rg_order, first = rg_order[:nrg], rg_order[nrg:]                # order, then the first stripe of every row group
    assert sorted(rg_order.tolist()) == list(range(nrg))
    nstripes = -(-M // 16)
    assert len(first) == nrg + 1 and first[0] == 0 and first[-1] == nstripes
    assert (np.diff(first) >= 1).all() and (np.diff(first) <= G).all()  # consecutive runs of 1 .. G stripes
    assert nrg == min(nstripes, -(-(-(-nstripes // G)) // 14) * 14)     # fewest runs, rounded up to whole workgroup rows
    nsteps = int(rg_ptr[-1])
    assert recs.shape == (nsteps + 4, 256) and meta.shape == (nsteps + 128, 2)
    assert not recs[nsteps:].any() and not meta[nsteps:].any()
    R, nch = 16, -(-K // 64)
    lanes = np.arange(64)
    g, n = lanes // 16, lanes % 16
    Wd = np.zeros((nstripes * 16, K), dtype=np.uint16)
    mfma = 0
    for rg in range(nrg):
        cnt = int(first[rg + 1] - first[rg])
        assert (rg_ptr[rg + 1] - rg_ptr[rg]) % 4 == 0
        prev_rel = 0
        for s in range(rg_ptr[rg], rg_ptr[rg + 1]):
            m0, m1 = int(meta[s, 0]), int(meta[s, 1])
            a = (m0 & 0xffff, m0 >> 16)
            o = (m1 & 15, (m1 >> 4) & 15)
            jj, do_lo, do_hi, rel = (m1 >> 8) & 15, (m1 >> 12) & 1, (m1 >> 13) & 1, m1 >> 22
            assert (m1 >> 14) & 0xff == 0
            # rel is handed back after this step's reads: no later step may read below it, and
            # what the wavefront still holds while it waits for this step's chunks fits the ring
            assert prev_rel <= rel <= nch
            held_from, prev_rel = prev_rel, rel
            if s == rg_ptr[rg + 1] - 1:
                assert rel == nch
            frag = recs[s].view(np.uint16).reshape(64, 8)
            if jj == 15:
                assert m0 == 0 and not frag.any() and not do_lo and not do_hi
                continue
            assert jj <= cnt and do_lo == (jj >= 1) and (do_lo or do_hi)
            need = (max(a) + 15) >> 6
            assert held_from <= min(a) >> 6 and need < nch and need - held_from <= R - 2
            assert max(a) + 16 <= K
            mfma += do_lo + do_hi
            for e in range(8):
                h = e // 4
                i = 4 * g + (e & 3)
                rho = a[h] + ((i - a[h]) % 16)                       # row of X per lane
                v = frag[:, e]
                lower = n >= o[h]                                      # rows that stay in stripe jj - 1
                for part, stripe, on in ((lower, jj - 1, do_lo), (~lower, jj, do_hi)):
                    sel = part & (v != 0)
                    if not on:
                        assert not sel.any() or not 0 <= stripe < cnt     # (weights of a part that is off belong to a neighbour)
                        continue
                    assert 0 <= stripe < cnt
                    rows = (int(first[rg]) + stripe) * 16 + n[sel]
                    assert not Wd[rows, rho[sel]].any()                # no weight is delivered twice
                    Wd[rows, rho[sel]] = v[sel]
    assert not Wd[M:].any()
    return Wd[:M], mfma


LAYOUT_SHAPES = [(64, 64, 4, 4, 0.5), (100, 300, 8, 8, 0.2), (130, 600, 16, 16, 0.15), (33, 40, 5, 3, 0.3),
                 (40, 2100, 4, 4, 0.02), (96, 2304, 4, 8, 0.1), (257, 31, 1, 1, 0.3), (90, 64, 20, 3, 0.25),
                 (70, 4200, 16, 32, 0.08), (150, 1300, 16, 40, 0.2), (64, 15, 8, 8, 0.2), (200, 3000, 12, 16, 0.1)]


@pytest.mark.parametrize("shape", LAYOUT_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_private_layouts_decode_to_the_dense_matrix(shape, dtype):
    M, K, bh, bw, d = shape
    blocks = select_blocks(M, K, bh, bw, d, 77 + M, "uniform", 1.1)
    W = make_weights(M, K, 5, dtype)
    dense_bits = W.view(np.uint16).copy()
    keep = oracle.densify(np.ones((M, K)), bh, bw, blocks) != 0
    dense_bits[~keep] = 0
    p = ubp.pack(W, dtype, bh, bw, blocks, device=ubp.HOST_ONLY)
    for G in (1, 2, 4):
        for CT in (2, 4, 8):
            Wd, mfma = _decode_layout(p, G, CT, M, K)
            assert np.array_equal(Wd, dense_bits), (G, CT)
            assert mfma == p.info(100 + ubp.layout_slot(G, CT))
    for gi, G in enumerate((2, 4, 5)):
        if bh <= 16 and K >= 16:
            Wn, mfma_n = _decode_block_layout(p, G, M, K)
            assert np.array_equal(Wn, dense_bits), ("block", G)
            assert mfma_n == p.info(300 + gi)
            assert p.info(309 + gi) <= p.info(306 + gi)
        else:
            with pytest.raises(ubp.UBPError):
                p.layout(G, 0, 2)
    p.free()


def _decode_tiles(p, M, K):
    """Dense W (16-bit patterns) back from the operand tiles of the dense-tile kernels, from the
    lane order the header documents: lane 16 g + n of a tile = row n of the stripe, columns
    4 g .. 4 g + 3 and 16 + 4 g .. of the tile's 32."""
    _, _, T, occ = p.layout(0, 0, 3)
    nstripes, kt_pad = T.shape[:2]
    bits = (occ[:, np.arange(kt_pad) // 32] >> (np.arange(kt_pad) % 32).astype(np.uint32)) & 1
    assert np.array_equal(bits.astype(bool), T.reshape(nstripes, kt_pad, -1).any(axis=2))   # one bit per tile that keeps a weight
    assert int(bits.sum()) == p.info(10)
    assert nstripes == (M + 15) // 16 and kt_pad * 32 >= K
    Wd = np.zeros((nstripes * 16, kt_pad * 32), dtype=np.uint16)
    for g in range(4):
        for e in range(8):
            col = 4 * g + e if e < 4 else 16 + 4 * g + (e - 4)
            # T[:, :, 16 g : 16 g + 16, e] is [stripe][tile][n]
            Wd.reshape(nstripes, 16, kt_pad, 32)[:, :, :, col] = T[:, :, 16 * g:16 * g + 16, e].transpose(0, 2, 1)
    assert not Wd[M:].any() and not Wd[:, K:].any()     # the padding is zero
    return Wd[:M, :K], kt_pad


TILE_LAYOUT_SHAPES = [(64, 64, 4, 4, 0.5), (100, 200, 8, 8, 0.2), (130, 256, 16, 16, 0.15), (33, 40, 5, 3, 0.3),
                      (257, 31, 1, 1, 0.3), (90, 300, 20, 3, 0.25), (250, 1000, 8, 8, 0.2), (40, 2100, 4, 4, 0.02)]


@pytest.mark.parametrize("shape", TILE_LAYOUT_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_operand_tiles_decode_to_the_dense_matrix(shape, dtype):
    M, K, bh, bw, d = shape
    blocks = select_blocks(M, K, bh, bw, d, 78 + M, "uniform", 1.1)
    W = make_weights(M, K, 6, dtype)
    dense_bits = W.view(np.uint16).copy()
    dense_bits[oracle.densify(np.ones((M, K)), bh, bw, blocks) == 0] = 0
    p = ubp.pack(W, dtype, bh, bw, blocks, device=ubp.HOST_ONLY)
    Wd, kt_pad = _decode_tiles(p, M, K)
    assert np.array_equal(Wd, dense_bits)
    # tiles per stripe: 2, 4, 6 or 8 up to K = 256, whole chunks of 8 beyond
    assert kt_pad == (max(2, 2 * ((K + 63) // 64)) if K <= 256 else 8 * ((K + 255) // 256))
    p.free()


def test_operand_tiles_are_not_built_for_large_matrices_or_fp32():
    blocks = select_blocks(4096, 2048, 16, 16, 0.01, 5, "uniform", 1.1)       # 256 stripes x 64 tiles = 16 MB
    p = ubp.pack(make_weights(4096, 2048, 7, "bf16"), "bf16", 16, 16, blocks, device=ubp.HOST_ONLY)
    with pytest.raises(ubp.UBPError):
        p.layout(0, 0, 3)
    p.free()
    blocks = select_blocks(64, 64, 4, 4, 0.3, 5, "uniform", 1.1)
    p = ubp.pack(make_weights(64, 64, 7, "f32"), "f32", 4, 4, blocks, device=ubp.HOST_ONLY)
    with pytest.raises(ubp.UBPError):
        p.layout(0, 0, 3)
    p.free()


@pytest.mark.parametrize("cfg", [c for c in CONFIGS if c.dtype != "f32"], ids=lambda c: c.name)
def test_benchmark_layer_layouts_decode_to_the_dense_matrix(cfg):
    """The layouts the benchmark layers actually run with (and the block layout for all of them)."""
    from synthetic import make_layer
    blocks, W, _ = make_layer(cfg, N=16)
    dense_bits = W.view(np.uint16).copy()
    dense_bits[oracle.densify(np.ones((cfg.M, cfg.K)), cfg.bh, cfg.bw, blocks) == 0] = 0
    p = ubp.pack(W, cfg.dtype, cfg.bh, cfg.bw, blocks, device=ubp.HOST_ONLY)
    G = 4 if cfg.bh >= 16 else 2 if cfg.bh >= 8 else 1
    for g, ct in [(G, 8), (G, 2)]:
        Wd, _ = _decode_layout(p, g, ct, cfg.M, cfg.K)
        assert np.array_equal(Wd, dense_bits), (g, ct)
    for G in (4, 5):
        Wd, _ = _decode_block_layout(p, G, cfg.M, cfg.K)
        assert np.array_equal(Wd, dense_bits)
    if cfg.name != "c4":                                 # (c4's zero-filled matrix would be 32 MB: not built)
        assert np.array_equal(_decode_tiles(p, cfg.M, cfg.K)[0], dense_bits)
    p.free()


def test_benchmark_refuses_more_than_one_gpu():
    """The product path runs on exactly one GPU: asking the benchmark for more ends with a message
    and a non-zero status before anything touches a device."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], stdout=subprocess.PIPE,
                         stderr=subprocess.PIPE, text=True, timeout=120)
    assert res.returncode != 0 and "one GPU" in res.stderr and res.stdout.strip() == ""
