"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle, element by
element on the same seeded inputs."""
import itertools
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")

import oracle                                    # noqa: E402
import paper_2407_19644_amd as ubp               # noqa: E402
from synthetic import (CONFIGS, decode_f64, encode, get_config, make_activations, make_layer,   # noqa: E402
                       make_weights, select_blocks)
from gpu_util import check, run_spmm, to_device  # noqa: E402

pytestmark = pytest.mark.gpu


def _plan(**kw):
    p = ubp.Plan()
    for k, v in kw.items():
        setattr(p, k, v)
    return p


def _layer(M, K, N, bh, bw, density, dtype, seed, x_dist="normal", mode="uniform"):
    blocks = select_blocks(M, K, bh, bw, density, seed, mode, 1.1)
    W = make_weights(M, K, seed + 1, dtype)
    X = make_activations(K, N, seed + 2, dtype, x_dist)
    return blocks, W, X


def _oracle(W, dtype, bh, bw, blocks, X, rows=None):
    return oracle.spmm(decode_f64(W, dtype), bh, bw, blocks, decode_f64(X, dtype), rows=rows, want_abs=True)


# ------------------------------------------------------------------ small shapes, every kernel
SMALL = [  # M, K, N, bh, bw, density: several tiles, ragged tails, odd pitches
    (64, 64, 196, 4, 4, 0.5),
    (70, 45, 67, 3, 1, 0.4),
    (100, 300, 333, 8, 8, 0.2),
    (130, 600, 1000, 16, 16, 0.15),
    (33, 40, 129, 5, 3, 0.3),
    (48, 520, 72, 2, 6, 0.35),
    (96, 700, 256, 4, 4, 0.25),
    (40, 2100, 64, 4, 4, 0.02),
    (16, 16, 16, 16, 16, 1.0),
    (257, 31, 40, 1, 1, 0.3),
]


@pytest.mark.parametrize("shape", SMALL, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_wros_kernel_small(shape, dtype):
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for y_dtype in {dtype, "f32"}:
        for rpr in (0, bh, 3 * bh):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=1, rows_per_range=rpr))
            check(Y, Yref, Yabs, dtype, y_dtype)
            # the dataflow without weight rotation (Section 3.3): same additions in the same order
            Yn = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=3, rows_per_range=rpr))
            assert np.array_equal(Yn, Y)


@pytest.mark.parametrize("shape", SMALL + [(90, 64, 50, 20, 3, 0.25)], ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_stripe_kernel_small(shape, dtype):
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 1)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for G, CT in itertools.product((1, 2, 4), (2, 4, 8)):
        for y_dtype in (dtype, "f32"):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=2, sub_stripes=G, col_tiles=CT))
            check(Y, Yref, Yabs, dtype, y_dtype)
    for G, CT, waves in [(1, 4, 2), (2, 2, 5), (4, 8, 4), (4, 4, 8), (2, 4, 16), (1, 2, 3)]:
        Y = run_spmm(W, dtype, bh, bw, blocks, X, dtype, _plan(kernel=2, sub_stripes=G, col_tiles=CT, waves=waves))
        check(Y, Yref, Yabs, dtype)
    # several wavefronts staging X (each takes every n-th kilobyte of a chunk), and several
    # workgroups sharing a column tile whose consumers walk more than one row group each
    for G, CT, waves, producers, wg_rows in [(1, 2, 6, 4, 0), (1, 4, 3, 2, 0), (2, 8, 8, 4, 0), (4, 4, 5, 2, 0),
                                             (2, 2, 0, 2, 0), (1, 8, 0, 4, 0), (1, 2, 2, 1, 1), (1, 4, 3, 1, 2),
                                             (2, 2, 4, 2, 1), (1, 2, 5, 1, 3)]:
        plan = _plan(kernel=2, sub_stripes=G, col_tiles=CT, waves=waves, producers=producers, wg_rows=wg_rows)
        if wg_rows and -(-K // 64) > 64 // CT:
            continue  # the staged tile does not hold all of K: the number of workgroup rows is not free
        Y = run_spmm(W, dtype, bh, bw, blocks, X, dtype, plan)
        check(Y, Yref, Yabs, dtype)

TILE_SHAPES = [(64, 64, 200, 4, 4, 0.5), (100, 200, 336, 8, 8, 0.2), (130, 256, 1000, 16, 16, 0.15), (33, 40, 136, 5, 3, 0.3),
               (257, 31, 40, 1, 1, 0.3), (90, 64, 56, 20, 3, 0.25), (16, 16, 16, 16, 16, 1.0), (1040, 160, 520, 4, 4, 0.3),
               (48, 250, 72, 2, 6, 0.05)]


@pytest.mark.parametrize("shape", TILE_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_x_stationary_kernel_small_k(shape, dtype):
    """The small-K kernel (X of a pixel block held in registers as operands, stripes of
    W streamed past it, 16 finished rows stored at a time) in both tile widths, every
    workgroup size and several slice counts: more wavefronts than stripes, an odd number of
    stripes per wavefront, a pixel block that hangs over the right edge, a last stripe that
    hangs over the bottom."""
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 4)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for CT, waves, slices in [(4, 0, 0), (2, 0, 0), (4, 1, 1), (2, 8, 3), (4, 8, 1), (2, 3, 100), (4, 5, 2), (2, 1, 2),
                              (4, 7, 1), (2, 2, 1)]:
        for y_dtype in (dtype, "f32"):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=4, col_tiles=CT, waves=waves, wg_rows=slices))
            check(Y, Yref, Yabs, dtype, y_dtype)


CHUNK_SHAPES = [(64, 300, 200, 4, 4, 0.3), (250, 1000, 136, 8, 8, 0.2), (40, 257, 72, 5, 3, 0.3), (530, 600, 64, 16, 16, 0.15),
                (16, 512, 16, 16, 16, 0.4), (100, 256, 40, 4, 4, 0.3), (256, 2304, 192, 4, 4, 0.25),
                (1000, 1500, 1000, 8, 8, 0.25)]


@pytest.mark.parametrize("shape", CHUNK_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_chunked_x_stationary_kernel(shape, dtype):
    """The dense-tile kernel for K beyond 256 (X passes through the registers in chunks of 256
    rows, accumulators stay): K a multiple of the chunk and not, one chunk only, more stripes
    than a workgroup holds (slices), a last slice with fewer stripes than wavefronts, a pixel
    block that hangs over the right edge, more slices than needed."""
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 5)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for CT, slices, SW in [(4, 0, 0), (2, 0, 0), (4, 5, 4), (2, 100, 4), (4, 0, 2), (2, 3, 2)]:
        for y_dtype in (dtype, "f32"):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype,
                         _plan(kernel=5, col_tiles=CT, wg_rows=slices, sub_stripes=SW))
            check(Y, Yref, Yabs, dtype, y_dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_dense_tile_kernels_with_padded_pitches(dtype):
    """Kernels 4 and 5 on X and Y whose rows are longer than N (pitches that keep the rows 16-byte
    aligned, as these kernels require): nothing may be read as data or written beyond column N,
    and a ragged last pixel block must not spill into the padding."""
    for M, K, N, bh, bw, d, kernels in [(100, 200, 200, 8, 8, 0.25, (4,)), (70, 256, 72, 4, 4, 0.3, (4, 5)),
                                        (150, 700, 136, 4, 4, 0.25, (5,))]:
        blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 6)
        Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
        for kernel in kernels:
            for ldx, ldy in [(N + 8, N + 24), (N + 64, N), (N, N + 8)]:
                for y_dtype in (dtype, "f32"):
                    Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=kernel), ldx=ldx, ldy=ldy)
                    check(Y, Yref, Yabs, dtype, y_dtype)
        # pitches that break the alignment are refused by these kernels and served by the others
        with pytest.raises(ubp.UBPError):
            run_spmm(W, dtype, bh, bw, blocks, X, dtype, _plan(kernel=kernels[-1]), ldx=N + 4, ldy=N)
        check(run_spmm(W, dtype, bh, bw, blocks, X, dtype, None, ldx=N + 4, ldy=N + 2), Yref, Yabs, dtype)


def test_automatic_kernel_choice():
    """What ubp_spmm picks by itself must be the documented kernel's result bit for bit: dense
    tiles (LDS-staged, small-K or chunked kernel) while at least half the 16 x 32 tiles of W keep a weight,
    gathered rows otherwise, and whole blocks as operands for 16-row blocks on a K beyond the ring."""
    M, K, N, bh, bw = 160, 1100, 256, 4, 4
    blocks, W, X = _layer(M, K, N, bh, bw, 0.25, "bf16", seed=91)         # every tile keeps a weight, few pixels
    Ya = run_spmm(W, "bf16", bh, bw, blocks, X, "f32")
    assert np.array_equal(Ya, run_spmm(W, "bf16", bh, bw, blocks, X, "f32", _plan(kernel=7)))
    blocks8, W8, X8 = _layer(M, K, 4608, bh, bw, 0.25, "bf16", seed=97)  # many pixels: the chunked kernel
    p = ubp.pack(W8, "bf16", bh, bw, blocks8, device=0)
    Xd = torch.zeros((K, 4608), dtype=torch.bfloat16, device="cuda")
    Yd = torch.zeros((M, 4608), dtype=torch.bfloat16, device="cuda")
    assert ubp.spmm_prepare(p, Xd.data_ptr(), 4608, 4608, Yd.data_ptr(), 4608, "bf16").kernel == 5
    p.free()
    blocks, W, X = _layer(M, K, N, bh, bw, 0.01, "bf16", seed=92)         # most tiles empty: gathered rows
    Ya = run_spmm(W, "bf16", bh, bw, blocks, X, "f32")
    assert np.array_equal(Ya, run_spmm(W, "bf16", bh, bw, blocks, X, "f32", _plan(kernel=2)))
    blocks, W, X = _layer(M, 160, N, bh, bw, 0.3, "f16", seed=94)          # every tile keeps a weight: both operands through LDS
    Ya = run_spmm(W, "f16", bh, bw, blocks, X, "f32")
    assert np.array_equal(Ya, run_spmm(W, "f16", bh, bw, blocks, X, "f32", _plan(kernel=7)))
    blocks, W, X = _layer(M, 160, N, 8, 8, 0.12, "f16", seed=96)           # some tiles empty, most not: the small-K kernel
    Ya = run_spmm(W, "f16", 8, 8, blocks, X, "f32")
    assert np.array_equal(Ya, run_spmm(W, "f16", 8, 8, blocks, X, "f32", _plan(kernel=4)))
    blocks, W, X = _layer(M, 160, N, bh, bw, 0.01, "f16", seed=95)
    Ya = run_spmm(W, "f16", bh, bw, blocks, X, "f32")
    assert np.array_equal(Ya, run_spmm(W, "f16", bh, bw, blocks, X, "f32", _plan(kernel=2)))
    M, K, N, bh, bw = 256, 4608, 2048, 16, 16                             # 72 chunks of X against a ring of 16
    blocks, W, X = _layer(M, K, N, bh, bw, 0.1, "bf16", seed=93)
    Yref, Yabs = _oracle(W, "bf16", bh, bw, blocks, X)
    Ya = run_spmm(W, "bf16", bh, bw, blocks, X, "f32")
    check(Ya, Yref, Yabs, "bf16", "f32")
    Yn = run_spmm(W, "bf16", bh, bw, blocks, X, "f32", _plan(kernel=6))
    assert np.array_equal(Ya, Yn)
    check(run_spmm(W, "bf16", bh, bw, blocks, X, "bf16"), Yref, Yabs, "bf16")   # 16-bit tiles leave through LDS rows


BLOCK_SHAPES = [(130, 600, 1000, 16, 16, 0.15), (100, 300, 328, 8, 8, 0.2), (96, 700, 256, 4, 4, 0.25), (33, 40, 136, 5, 3, 0.3),
                (70, 45, 72, 3, 1, 0.4), (16, 16, 64, 16, 16, 1.0), (257, 31, 104, 1, 1, 0.3), (300, 2500, 192, 16, 32, 0.1),
                (150, 1300, 136, 16, 40, 0.2), (200, 3000, 64, 12, 16, 0.1), (64, 16, 200, 16, 16, 0.25),
                (160, 4096, 64, 16, 16, 0.004), (400, 6000, 128, 16, 16, 0.002), (64, 8192, 64, 16, 16, 0.0005)]   # row groups whose first block lies beyond the ring


@pytest.mark.parametrize("shape", BLOCK_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_block_kernel(shape, dtype):
    """Whole blocks as operands (kernel 6): blocks of 16 rows and fewer, widths below, at and
    above 16 and not a multiple of it, K below and beyond the ring, a ragged last column tile
    (which the gather kernel serves), one or several producers, few and many consumers."""
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 7)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for G in (2, 4, 5):
        for y_dtype in (dtype, "f32"):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=6, sub_stripes=G))
            check(Y, Yref, Yabs, dtype, y_dtype)
    for G, waves, NP in [(4, 3, 1), (2, 16, 4), (5, 5, 2), (2, 2, 1), (4, 16, 1), (5, 16, 2)]:
        Y = run_spmm(W, dtype, bh, bw, blocks, X, dtype, _plan(kernel=6, sub_stripes=G, waves=waves, producers=NP))
        check(Y, Yref, Yabs, dtype)


GEMM_SHAPES = [(100, 200, 328, 4, 4, 0.5), (270, 700, 520, 4, 4, 0.45), (64, 64, 200, 4, 4, 0.6), (530, 96, 1000, 4, 4, 0.5),
               (16, 32, 16, 16, 16, 1.0), (300, 257, 72, 2, 1, 0.4), (1040, 160, 264, 4, 4, 0.4), (250, 1000, 136, 8, 8, 0.1)]


@pytest.mark.parametrize("shape", GEMM_SHAPES, ids=lambda s: "x".join(map(str, s)))
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_lds_staged_dense_tile_kernel(shape, dtype):
    """Kernel 7 (both operands staged in LDS, a workgroup owns up to 256 rows x 256 pixels) in every
    tile shape: row and pixel blocks that hang over the edges, K not a multiple of 32, fewer
    stages than LDS slots, more than one row block per pixel block; a matrix with tiles that keep
    nothing is refused."""
    M, K, N, bh, bw, d = shape
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=M + K + 8)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    p = ubp.pack(W, dtype, bh, bw, blocks, device=0)
    full = p.info(10) == p.info(11)           # every 16 x 32 tile keeps a weight
    p.free()
    assert full == (d >= 0.4)
    for G, CT in [(0, 0), (16, 16), (8, 16), (8, 8), (16, 4), (4, 8), (4, 4)]:
        for y_dtype in (dtype, "f32"):
            plan = _plan(kernel=7, sub_stripes=G, col_tiles=CT)
            if not full:                                  # the kernel multiplies every tile: refused
                with pytest.raises(ubp.UBPError):
                    run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, plan)
                continue
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, plan)
            check(Y, Yref, Yabs, dtype, y_dtype)


def test_block_kernel_refuses_what_it_cannot_do():
    blocks, W, X = _layer(90, 64, 128, 20, 3, 0.25, "bf16", seed=5)      # blocks taller than a stripe
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 20, 3, blocks, X, "bf16", _plan(kernel=6))
    blocks, W, X = _layer(64, 12, 128, 4, 4, 0.3, "bf16", seed=6)        # K below one window
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=6))
    blocks, W, X = _layer(64, 64, 48, 4, 4, 0.3, "bf16", seed=7)         # not one full column tile
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=6))
    blocks, W, X = _layer(64, 64, 128, 4, 4, 0.3, "bf16", seed=8)
    for bad in (dict(col_tiles=8), dict(sub_stripes=1), dict(sub_stripes=3), dict(waves=17), dict(producers=3)):
        with pytest.raises(ubp.UBPError):
            run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=6, **bad))
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=6), ldx=132, ldy=128)   # rows not 16-byte aligned
    blocks, W, X = _layer(64, 64, 128, 4, 4, 0.3, "f32", seed=9)
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "f32", 4, 4, blocks, X, "f32", _plan(kernel=6))
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "f32", 4, 4, blocks, X, "f32", _plan(kernel=8))       # there is no kernel 8


def test_chunked_kernel_refuses_what_it_cannot_do():
    blocks, W, X = _layer(64, 160, 64, 4, 4, 0.3, "bf16", seed=5)        # 5 tiles per stripe: not whole chunks
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=5))
    blocks, W, X = _layer(64, 512, 66, 4, 4, 0.3, "bf16", seed=6)        # N not a multiple of 8
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=5))
    blocks, W, X = _layer(64, 512, 64, 4, 4, 0.3, "bf16", seed=7)
    for bad in (dict(col_tiles=8), dict(waves=4), dict(sub_stripes=1)):
        with pytest.raises(ubp.UBPError):
            run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=5, **bad))
    blocks, W, X = _layer(64, 512, 64, 4, 4, 0.3, "f32", seed=8)
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "f32", 4, 4, blocks, X, "f32", _plan(kernel=5))


@pytest.mark.parametrize("kernel", [4])
def test_small_k_kernel_refuses_what_it_cannot_do(kernel):
    blocks, W, X = _layer(64, 300, 64, 4, 4, 0.3, "bf16", seed=5)       # K too large
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=kernel))
    blocks, W, X = _layer(64, 64, 66, 4, 4, 0.3, "bf16", seed=6)        # N not a multiple of 8
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=kernel))
    Yref, Yabs = _oracle(W, "bf16", 4, 4, blocks, X)
    check(run_spmm(W, "bf16", 4, 4, blocks, X, "bf16"), Yref, Yabs, "bf16")  # falls back to the gather kernel
    blocks, W, X = _layer(64, 64, 64, 4, 4, 0.3, "f32", seed=7)
    with pytest.raises(ubp.UBPError):
        run_spmm(W, "f32", 4, 4, blocks, X, "f32", _plan(kernel=kernel))
    blocks, W, X = _layer(64, 64, 64, 4, 4, 0.3, "bf16", seed=8)
    for bad in (dict(col_tiles=8), dict(waves=9), dict(col_tiles=3)):
        with pytest.raises(ubp.UBPError):
            run_spmm(W, "bf16", 4, 4, blocks, X, "bf16", _plan(kernel=kernel, **bad))


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_unaligned_pitches_and_pointers(dtype):
    """Leading dimensions that are not multiples of the vector width take the element-wise
    path; nothing may be written beyond column N."""
    M, K, N, bh, bw = 50, 70, 101, 4, 4
    blocks, W, X = _layer(M, K, N, bh, bw, 0.3, dtype, seed=9)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for ldx, ldy in [(N, N), (N + 3, N + 5), (104, 112)]:
        Y = run_spmm(W, dtype, bh, bw, blocks, X, dtype, None, ldx=ldx, ldy=ldy)
        check(Y, Yref, Yabs, dtype)
        Y = run_spmm(W, dtype, bh, bw, blocks, X, dtype, _plan(kernel=1), ldx=ldx, ldy=ldy)
        check(Y, Yref, Yabs, dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_uneven_row_groups_share_the_lds_ring(dtype):
    """K is many times the LDS ring; one row group is dense over all of K, others touch only a
    few far-apart columns, so wavefronts of one workgroup run through the ring at very different
    paces (a slot must not be refilled while the slow one still needs it)."""
    M, K, N, bh, bw = 112, 3000, 200, 8, 8
    blocks = [(0, c) for c in range(0, K - bw, 12)] + [(9, c) for c in range(3, K - bw, 40)]
    blocks += [(40, 0), (40, 2900), (70, 1500), (100, 7), (100, 1000), (100, 2990)]
    W = make_weights(M, K, 31, dtype)
    X = make_activations(K, N, 32, dtype, "normal")
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    for G, CT in itertools.product((1, 2, 4), (2, 4, 8)):
        for rep in range(2):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, "f32", _plan(kernel=2, sub_stripes=G, col_tiles=CT))
            check(Y, Yref, Yabs, dtype, "f32")


# ------------------------------------------------------------------ exact special cases
@pytest.mark.parametrize("dtype,kernel,K,bh,bw", [("f32", 1, 128, 4, 4), ("f16", 1, 128, 4, 4), ("bf16", 1, 128, 4, 4),
                                                 ("f16", 2, 128, 4, 4), ("bf16", 2, 128, 4, 4), ("bf16", 2, 1280, 16, 16),
                                                 ("f16", 4, 128, 4, 4), ("bf16", 4, 256, 8, 8),
                                                 ("f16", 5, 512, 4, 4), ("bf16", 5, 512, 8, 8),
                                                 ("f16", 6, 128, 4, 4), ("bf16", 6, 1280, 16, 16), ("bf16", 6, 512, 16, 32),
                                                 ("f16", 7, 128, 4, 4), ("bf16", 7, 512, 4, 4),
                                                 ("bf16", 0, 1280, 16, 16), ("f16", 0, 128, 4, 4), ("bf16", 0, 512, 4, 4)])
def test_identity_x_returns_densified_w_bit_exactly(dtype, kernel, K, bh, bw):
    """X = I: every output is one kept weight times one, plus zeros - no rounding anywhere, so Y
    must be the densified W bit for bit, through every kernel (0 = the automatic choice)."""
    M = 90
    blocks = select_blocks(M, K, bh, bw, 0.3 if bh < 16 else 0.15, seed=3)
    W = make_weights(M, K, 4, dtype)
    X = encode(np.eye(K, dtype=np.float32), dtype)
    Wd = oracle.densify(decode_f64(W, dtype), bh, bw, blocks)
    for y_dtype in {dtype, "f32"}:
        Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, _plan(kernel=kernel))
        assert np.array_equal(Y, Wd)


@pytest.mark.parametrize("kernel", [1, 2, 4, 5, 6])
def test_non_finite_x_reaches_only_what_the_header_says(kernel):
    """An Inf and a NaN in two rows of X that no kept weight multiplies.  The vector kernel
    multiplies kept weights only: Y is unaffected.  The MFMA kernels multiply zero-filled
    operands: exactly the outputs the header names become NaN (in the two poisoned pixel
    columns), all others are unaffected."""
    M, K, N, bh, bw, dtype = 96, 256, 128, 16, 16, "bf16"
    blocks = [(3, 40), (20, 200), (50, 130), (70, 232), (35, 80)]
    W = make_weights(M, K, 11, dtype)
    X = make_activations(K, N, 12, dtype, "normal")
    Yclean, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    Xp = X.copy()
    k_inf, k_nan, px_inf, px_nan = 100, 150, 5, 77       # row 100: inside no block's columns; row 150: nor that one
    Xp[k_inf, px_inf] = encode(np.array([np.inf], np.float32), dtype)[0]
    Xp[k_nan, px_nan] = encode(np.array([np.nan], np.float32), dtype)[0]
    Y = run_spmm(W, dtype, bh, bw, blocks, Xp, "f32", _plan(kernel=kernel), prefill=7.0)
    bad = np.zeros((M, N), bool)
    rows_of = lambda r0: np.arange(16 * (r0 // 16), 16 * (r0 // 16) + 16)          # noqa: E731
    if kernel in (4, 5):
        # rows of every stripe that keeps a weight within the aligned 32 rows of X around the poisoned row
        for k, px in ((k_inf, px_inf), (k_nan, px_nan)):
            for r, c in blocks:
                if c < 32 * (k // 32) + 32 and c + bw > 32 * (k // 32):
                    for rr in (r, r + bh - 1):
                        bad[rows_of(rr)[rows_of(rr) < M], px] = True
    elif kernel == 2:
        pass        # no kept weight in those columns: the rows are never gathered
    elif kernel == 6:
        pass        # rows 100 and 150 lie in no block's 16-row window
    assert np.isnan(Y[bad]).all() and np.isfinite(Y[~bad]).all()
    assert np.abs(Y[~bad] - Yclean[~bad]).max() <= 2e-3 * np.abs(Yclean).max()
    # poison INSIDE a window of the block kernel / a gathered row: the whole stripes that block reaches into
    if kernel in (2, 6):
        Xq = X.copy()
        Xq[130 + 3, px_inf] = encode(np.array([np.inf], np.float32), dtype)[0]       # a column of block (50, 130)
        Y = run_spmm(W, dtype, bh, bw, blocks, Xq, "f32", _plan(kernel=kernel), prefill=7.0)
        rows = np.arange(50, 66)
        assert not np.isfinite(Y[rows, px_inf]).all()                               # the exact sum holds it there
        others = np.ones((M, N), bool)
        others[:, px_inf] = False
        assert np.isfinite(Y[others]).all()


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_empty_block_list_and_untouched_rows_are_zero(dtype):
    M, K, N = 40, 32, 70
    X = make_activations(K, N, 1, dtype, "normal")
    W = make_weights(M, K, 2, dtype)
    Y = run_spmm(W, dtype, 4, 4, np.zeros((0, 2), np.int32), X)
    assert np.array_equal(Y, np.zeros((M, N))) and not np.signbit(Y).any()
    Y = run_spmm(W, dtype, 4, 4, [(17, 5)], X)          # rows 0..16 and 21..39 have no block
    Yref, Yabs = _oracle(W, dtype, 4, 4, [(17, 5)], X)
    check(Y, Yref, Yabs, dtype)
    assert (Y[:17] == 0).all() and (Y[21:] == 0).all()


def test_aligned_origins_match_oracle():
    """Aligned block pruning is the special case with origins on multiples of the block size."""
    M, K, N, bh, bw = 64, 96, 200, 8, 8
    rng = np.random.default_rng(0)
    cells = [(i * bh, j * bw) for i in range(M // bh) for j in range(K // bw)]
    blocks = [cells[t] for t in rng.permutation(len(cells))[:30]]
    for dtype in ("f32", "f16"):
        W = make_weights(M, K, 5, dtype)
        X = make_activations(K, N, 6, dtype, "normal")
        Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
        check(run_spmm(W, dtype, bh, bw, blocks, X), Yref, Yabs, dtype)


def test_all_blocks_kept_is_dense_gemm():
    M, K, N, bh, bw = 64, 64, 150, 16, 16
    blocks = [(r, c) for r in range(0, M, bh) for c in range(0, K, bw)]
    for dtype in ("f32", "bf16"):
        W = make_weights(M, K, 7, dtype)
        X = make_activations(K, N, 8, dtype, "normal")
        Yref = decode_f64(W, dtype) @ decode_f64(X, dtype)
        check(run_spmm(W, dtype, bh, bw, blocks, X, "f32"), Yref, None, dtype, "f32")


def test_two_runs_are_bit_identical_and_columns_commute():
    cfg = get_config("c1")
    blocks, W, X = make_layer(cfg, N=400)
    Y1 = run_spmm(W, cfg.dtype, cfg.bh, cfg.bw, blocks, X)
    Y2 = run_spmm(W, cfg.dtype, cfg.bh, cfg.bw, blocks, X)
    assert np.array_equal(Y1, Y2)
    perm = np.random.default_rng(0).permutation(400)
    Y3 = run_spmm(W, cfg.dtype, cfg.bh, cfg.bw, blocks, np.ascontiguousarray(X[:, perm]))
    assert np.array_equal(Y3, Y1[:, perm])


@pytest.mark.parametrize("kernel", [2, 4, 5, 6, 7])
def test_every_mfma_kernel_is_deterministic_and_column_order_free(kernel):
    """No kernel uses atomics on Y and every output element has one fixed summation order, whatever
    the pace of the wavefronts that hand data to each other: repeated runs agree bit for bit, and
    permuting the columns of X permutes the columns of Y."""
    M, K, N, bh, bw = 144, 512, 384, 8, 8
    blocks, W, X = _layer(M, K, N, bh, bw, 0.25, "bf16", seed=17)
    if kernel == 4:
        K = 256
        blocks, W, X = _layer(M, K, N, bh, bw, 0.25, "bf16", seed=18)
    if kernel == 7:                                    # (it wants every 16 x 32 tile to keep a weight)
        bh = bw = 4
        blocks, W, X = _layer(M, K, N, bh, bw, 0.45, "bf16", seed=19)
    plan = _plan(kernel=kernel)
    Y1 = run_spmm(W, "bf16", bh, bw, blocks, X, "f32", plan)
    for _ in range(3):
        assert np.array_equal(run_spmm(W, "bf16", bh, bw, blocks, X, "f32", plan), Y1)
    perm = np.random.default_rng(1).permutation(N)
    Yp = run_spmm(W, "bf16", bh, bw, blocks, np.ascontiguousarray(X[:, perm]), "f32", plan)
    assert np.array_equal(Yp, Y1[:, perm])


def test_device_errors_and_noop():
    cfg = get_config("c0")
    blocks, W, X = make_layer(cfg)
    p = ubp.pack(W, "f32", cfg.bh, cfg.bw, blocks, device=0)
    L = ubp.load_library()
    Xd = torch.zeros(64, 196, device="cuda")
    Yd = torch.full((64, 196), 7.0, device="cuda")
    h = p.handle
    assert L.ubp_spmm(h, Xd.data_ptr(), 196, 0, Yd.data_ptr(), 196, 0, None) == 0       # N = 0: no-op
    assert L.ubp_spmm(h, Xd.data_ptr(), 100, 196, Yd.data_ptr(), 196, 0, None) == 1     # ldx < N
    assert L.ubp_spmm(h, Xd.data_ptr(), 196, 196, Yd.data_ptr(), 196, 1, None) == 1     # y dtype mismatch
    assert L.ubp_spmm(h, None, 196, 196, Yd.data_ptr(), 196, 0, None) == 1
    assert L.ubp_spmm_plan(h, Xd.data_ptr(), 196, 196, Yd.data_ptr(), 196, 0, None, _plan(kernel=2)) == 4
    torch.cuda.synchronize()
    assert (Yd == 7.0).all()                                                           # nothing written on error
    assert p.info(6) == 0 and p.info(8) > 0
    p.free()
    with pytest.raises(ubp.UBPError) as e:
        ubp.pack(W, "f32", cfg.bh, cfg.bw, blocks, device=99)
    assert e.value.code == 7


# ------------------------------------------------------------------ the five layers at full size
_FULL = {}


def _full_reference(name):
    """The oracle over the whole layer (all rows, all columns), computed once per session.  The
    oracle itself is one plain thread; the test hands it disjoint row ranges from several threads
    (the C call releases the interpreter lock), which changes no value."""
    if name not in _FULL:
        from concurrent.futures import ThreadPoolExecutor
        cfg = get_config(name)
        blocks, W, X = make_layer(cfg)
        W64, X64 = decode_f64(W, cfg.dtype), decode_f64(X, cfg.dtype)
        want_abs = cfg.dtype == "f32"                      # the componentwise bound is the fp32 layer's
        step = max(1, min(128, cfg.M // 16))
        ranges = [np.arange(r, min(r + step, cfg.M)) for r in range(0, cfg.M, step)]
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as ex:
            parts = list(ex.map(lambda rows: oracle.spmm(W64, cfg.bh, cfg.bw, blocks, X64, rows=rows, want_abs=want_abs), ranges))
        if want_abs:
            Yref, Yabs = np.concatenate([p[0] for p in parts]), np.concatenate([p[1] for p in parts])
        else:
            Yref, Yabs = np.concatenate(parts), None
        _FULL[name] = (cfg, blocks, W, X, Yref, Yabs)
    return _FULL[name]


@pytest.mark.parametrize("name", ["c0", "c1", "c2", "c3", "c4"])
def test_layer_full_oracle(name):
    """Every element of Y of the five layers at full size against the oracle, through what
    ubp_spmm picks by itself (the launch shape the benchmark times), in both output types."""
    cfg, blocks, W, X, Yref, Yabs = _full_reference(name)
    for y_dtype in sorted({cfg.dtype, "f32"}):
        Y = run_spmm(W, cfg.dtype, cfg.bh, cfg.bw, blocks, X, y_dtype)
        check(Y, Yref, Yabs, cfg.dtype, y_dtype)


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_layer_full_size_other_kernels(name):
    """The kernels ubp_spmm does not pick for a layer, at full size, against the same full oracle."""
    cfg, blocks, W, X, Yref, Yabs = _full_reference(name)
    plans = [_plan(kernel=1), _plan(kernel=2)]
    if name == "c4":
        plans += [_plan(kernel=2, sub_stripes=4, col_tiles=8), _plan(kernel=6, sub_stripes=2), _plan(kernel=6, waves=10, producers=4)]
    elif name == "c3":
        plans += [_plan(kernel=2, sub_stripes=1, col_tiles=8), _plan(kernel=6)]
    else:
        plans += [_plan(kernel=6), _plan(kernel=4, col_tiles=2)]
    for plan in plans:
        Y = run_spmm(W, cfg.dtype, cfg.bh, cfg.bw, blocks, X, "f32", plan)
        check(Y, Yref, Yabs, cfg.dtype, "f32")


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "c4"])
def test_handle_holds_only_the_layout_that_runs(name):
    """Device memory of a handle after the automatic call: the canonical arrays plus the one
    layout that call used.  For the block-sparse layer that is at most three times the canonical
    arrays; for the layers served from dense tiles it is the densified matrix (padded to whole
    tiles) beside the canonical arrays' index part."""
    cfg = get_config(name)
    blocks, W, X = make_layer(cfg)
    p = ubp.pack(W, cfg.dtype, cfg.bh, cfg.bw, blocks, device=torch.cuda.current_device())
    canonical = p.info(7)
    before = p.info(8)
    assert before <= canonical                                  # nothing but indptr / indices before the first call
    Xd = to_device(X, cfg.dtype)
    Yd = torch.empty((cfg.M, cfg.N), dtype=torch.float32, device="cuda")
    ubp.spmm(p, Xd.data_ptr(), cfg.N, cfg.N, Yd.data_ptr(), cfg.N, "f32", torch.cuda.current_stream().cuda_stream, None)
    torch.cuda.synchronize()
    after = p.info(8)
    if name == "c4":
        assert after <= 3 * canonical, (after, canonical)
    else:
        dense = (-(-cfg.M // 16) * 16) * (-(-cfg.K // 256) * 256) * 2   # tiles padded to whole chunks of 256 columns
        assert after <= before + dense + 64 * 1024, (after, before, dense)
    # a second call allocates nothing more
    ubp.spmm(p, Xd.data_ptr(), cfg.N, cfg.N, Yd.data_ptr(), cfg.N, "f32", torch.cuda.current_stream().cuda_stream, None)
    torch.cuda.synchronize()
    assert p.info(8) == after
    p.free()


@pytest.mark.parametrize("method", ["greedy", "bed", "optimal"])
def test_selected_blocks_through_the_product(method):
    """Block lists chosen from the weights themselves (Sections 3.2 and 4.1) instead of sampled
    origins: magnitude-driven masks cluster differently from uniform ones, and the product must
    not care."""
    rng = np.random.default_rng(31)
    for M, K, N, bh, bw, dtype, density in ((192, 256, 200, 4, 1, "f16", 0.3), (256, 2048, 128, 16, 16, "bf16", 0.1),
                                            (96, 160, 72, 8, 2, "f32", 0.25)):
        W64 = rng.standard_normal((M, K)) * np.exp(rng.standard_normal((M, 1)))     # some rows matter more
        W = encode(W64, dtype)
        blocks = ubp.select_blocks(W, dtype, bh, bw, density, method)
        assert len(blocks) == ubp.target_block_count(M, K, bh, bw, density)
        X = make_activations(K, N, 5, dtype, "relu_normal")
        Yref, Yabs = oracle.spmm(decode_f64(W, dtype), bh, bw, blocks, decode_f64(X, dtype), want_abs=True)
        for y_dtype in sorted({dtype, "f32"}):
            Y = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype)
            check(Y, Yref, Yabs, dtype, y_dtype)


# ------------------------------------------------------------------ fused epilogue (bias, ReLU / clamp)
def _run_fused(W, dtype, bh, bw, blocks, X, y_dtype, bias, activation, lo, hi, plan):
    M = W.shape[0]
    K, N = X.shape
    p = ubp.pack(W, dtype, bh, bw, blocks, device=torch.cuda.current_device())
    Xd = to_device(X, dtype)
    tdt = {"f32": torch.float32, "f16": torch.float16, "bf16": torch.bfloat16}[y_dtype]
    Yd = torch.full((M, N), float("nan"), dtype=tdt, device="cuda")
    bd = None if bias is None else torch.from_numpy(bias.astype(np.float32)).cuda()
    ubp.spmm_fused(p, Xd.data_ptr(), N, N, Yd.data_ptr(), N, y_dtype, None if bd is None else bd.data_ptr(), activation, lo, hi,
                   torch.cuda.current_stream().cuda_stream, plan)
    torch.cuda.synchronize()
    assert p.device_error() == 0
    p.free()
    t = Yd.cpu()
    return decode_f64(t.view(torch.uint16).numpy(), "bf16") if y_dtype == "bf16" else t.numpy().astype(np.float64)


FUSED_CASES = [  # kernel, (M, K, N, bh, bw, density), dtype
    (1, (70, 45, 67, 3, 1, 0.4), "f32"), (1, (96, 300, 256, 4, 4, 0.25), "f16"), (3, (100, 300, 333, 8, 8, 0.2), "bf16"),
    (2, (130, 600, 1000, 16, 16, 0.15), "bf16"), (2, (33, 40, 129, 5, 3, 0.3), "f16"),
    (4, (200, 256, 328, 8, 8, 0.2), "f16"), (5, (160, 1024, 264, 4, 4, 0.25), "bf16"),
    (6, (300, 2500, 192, 16, 32, 0.1), "bf16"), (6, (130, 600, 1000, 16, 16, 0.15), "f16"),
    (7, (160, 320, 520, 4, 4, 0.45), "f16"), (0, (256, 2048, 128, 16, 16, 0.1), "bf16"), (0, (64, 64, 196, 4, 4, 0.5), "f32"),
]


@pytest.mark.parametrize("case", FUSED_CASES, ids=lambda c: "k%d-%s-%s" % (c[0], "x".join(map(str, c[1])), c[2]))
def test_fused_epilogue(case):
    """ubp_spmm_fused through every kernel: bias per output row, ReLU, clamp, bias alone, and the
    empty epilogue (= the plain product, bit for bit), in both output types."""
    kernel, (M, K, N, bh, bw, d), dtype = case
    blocks, W, X = _layer(M, K, N, bh, bw, d, dtype, seed=3 * M + K)
    Yref, Yabs = _oracle(W, dtype, bh, bw, blocks, X)
    rng = np.random.default_rng(M + N)
    scale = np.abs(Yref).max()
    bias = (rng.standard_normal(M) * 0.5 * scale).astype(np.float32)      # fp32: what the library is given
    plan = _plan(kernel=kernel) if kernel else None
    for y_dtype in sorted({dtype, "f32"}):
        plain = run_spmm(W, dtype, bh, bw, blocks, X, y_dtype, plan)
        for b, act, lo, hi in ((bias, "relu", 0, 0), (bias, "clamp", -0.4 * scale, 0.7 * scale), (bias, None, 0, 0),
                               (None, "relu", 0, 0), (None, None, 0, 0)):
            Y = _run_fused(W, dtype, bh, bw, blocks, X, y_dtype, b, act, lo, hi, plan)
            want = oracle.fused(Yref, None if b is None else b.astype(np.float64), act, lo, hi)
            if b is None and act is None:
                assert np.array_equal(Y, plain)
                continue
            # the bias is added to the fp32 accumulator: one more rounding of size |v| 2^-24
            check(Y, want, None if Yabs is None else Yabs + np.abs(want) + (0 if b is None else np.abs(b)[:, None]), dtype, y_dtype)
            if act == "relu":
                assert (Y >= 0).all()
            if act == "clamp" and y_dtype == "f32":                        # (a 16-bit Y rounds the bound itself)
                assert (Y >= np.float32(lo)).all() and (Y <= np.float32(hi)).all()


def test_fused_epilogue_arguments():
    blocks, W, X = _layer(64, 64, 128, 4, 4, 0.3, "f16", seed=2)
    with pytest.raises(ubp.UBPError) as e:
        _run_fused(W, "f16", 4, 4, blocks, X, "f16", None, "clamp", 1.0, -1.0, None)     # lo > hi
    assert e.value.code == 1
    with pytest.raises(ubp.UBPError) as e:
        _run_fused(W, "f16", 4, 4, blocks, X, "f16", None, "clamp", float("nan"), 1.0, None)
    assert e.value.code == 1
    # a NaN in the accumulator becomes the lower bound (IEEE maxNum), as the header says
    Xn = decode_f64(X, "f16")
    Xn[5, 7] = np.nan
    Y = _run_fused(W, "f16", 4, 4, blocks, encode(Xn, "f16"), "f32", None, "relu", 0, 0, _plan(kernel=1))
    assert np.isfinite(Y).all() and (Y >= 0).all()


def test_fused_epilogue_full_layer():
    """c4 at full size with bias + ReLU through the automatic choice, every element."""
    cfg, blocks, W, X, Yref, Yabs = _full_reference("c4")
    rng = np.random.default_rng(8)
    bias = (rng.standard_normal(cfg.M) * 0.3 * np.abs(Yref).max()).astype(np.float32)
    Y = _run_fused(W, cfg.dtype, cfg.bh, cfg.bw, blocks, X, cfg.dtype, bias, "relu", 0, 0, None)
    check(Y, oracle.fused(Yref, bias.astype(np.float64), "relu"), None, cfg.dtype, cfg.dtype)
