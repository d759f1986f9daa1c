"""Pins for the CPU oracle: it is checked here against things other than itself.

 * the paper's N = 3 worked example (Section 3.3 sum for O_23, Section 4.2 rotation);
 * brute force that walks the block list and never densifies (tiny inputs, pure Python);
 * an all-blocks-kept W reproduces dense GEMM (numpy matmul in float64);
 * aligned origins are ordinary BSR (Section 3.1: ABP is the aligned special case);
 * a single block has a closed form; X = identity returns the densified W;
 * the validator rejects overlap / out-of-bounds, and planted mistakes are caught.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp

import oracle
from synthetic import select_blocks


# ----------------------------------------------------------------------------- worked example
def _example_arrays(g, val):
    M, K = int(g["M"][0][0]), int(g["K"][0][0])
    bh, bw = int(g["bh"][0][0]), int(g["bw"][0][0])
    W = np.zeros((M, K))
    blocks = []
    for r, c, *letters in g["block"]:
        r, c = int(r), int(c)
        blocks.append((r, c))
        for d, L in enumerate(letters):
            W[r + d, c] = val[L]
    return M, K, bh, bw, W, blocks


def test_worked_example_format(worked_example):
    g, val = worked_example
    M, K, bh, bw, W, blocks = _example_arrays(g, val)
    # present the blocks in a scrambled order: the packed arrays must not depend on it
    for perm in itertools.permutations(range(len(blocks))):
        indptr, indices, values = oracle.pack(W, bh, bw, [blocks[p] for p in perm])
        assert indptr.tolist() == [int(t) for t in g["indptr"][0]]
        assert indices.tolist() == [int(t) for t in g["indices"][0]]
        assert values.tolist() == [val[L] for L in g["values"][0]]


def test_worked_example_o23(worked_example):
    g, val = worked_example
    M, K, bh, bw, W, blocks = _example_arrays(g, val)
    rng = np.random.default_rng(7)
    X = rng.integers(1, 50, size=(K, 6)).astype(np.float64)
    # make the densify step matter: junk outside the blocks must be pruned
    Wjunk = W + (W == 0) * 1000.0
    Y = oracle.spmm(Wjunk, bh, bw, blocks, X)
    terms = g["o23"][0]
    expect = sum(val[terms[t]] * X[int(terms[t + 1]), 3] for t in range(0, len(terms), 2))
    assert Y[2, 3] == expect
    # D sits in slot 1 of its block (the paper's remark on R_1)
    _, _, values = oracle.pack(W, bh, bw, blocks)
    assert values[1 * bh + 1] == val["D"]


# ----------------------------------------------------------------------------- brute force
def brute_force(W, bh, bw, blocks, X):
    """Walk the block list term by term; never builds a dense W."""
    M, K = W.shape
    N = X.shape[1]
    Y = [[0.0] * N for _ in range(M)]
    for (r, c) in blocks:
        for di in range(bh):
            for dj in range(bw):
                w = float(W[r + di, c + dj])
                for j in range(N):
                    Y[r + di][j] += w * float(X[c + dj, j])
    return np.array(Y)


def random_mask(rng, M, K, bh, bw, tries=40):
    occ = np.zeros((M, K), bool)
    out = []
    for _ in range(tries):
        r = int(rng.integers(0, M - bh + 1))
        c = int(rng.integers(0, K - bw + 1))
        if not occ[r:r + bh, c:c + bw].any():
            occ[r:r + bh, c:c + bw] = True
            out.append((r, c))
    return out


@pytest.mark.parametrize("bh,bw", list(itertools.product([1, 2, 3, 4], [1, 2, 3, 4])))
def test_brute_force_tiny(bh, bw):
    rng = np.random.default_rng(100 * bh + bw)
    for M, K, N in [(8, 8, 3), (7, 5, 2), (bh, bw, 1), (bh + 1, bw + 2, 4)]:
        if bh > M or bw > K:
            continue
        # small integers: every partial sum is exact, so any summation order agrees exactly
        W = rng.integers(-9, 10, size=(M, K)).astype(np.float64)
        X = rng.integers(-9, 10, size=(K, N)).astype(np.float64)
        blocks = random_mask(rng, M, K, bh, bw)
        Y, Ya = oracle.spmm(W, bh, bw, blocks, X, want_abs=True)
        assert np.array_equal(Y, brute_force(W, bh, bw, blocks, X))
        assert np.array_equal(Ya, brute_force(np.abs(W), bh, bw, blocks, np.abs(X)))


def test_brute_force_real_valued():
    rng = np.random.default_rng(5)
    W = rng.standard_normal((12, 10))
    X = rng.standard_normal((10, 5))
    blocks = random_mask(rng, 12, 10, 3, 2)
    Y = oracle.spmm(W, 3, 2, blocks, X)
    np.testing.assert_allclose(Y, brute_force(W, 3, 2, blocks, X), rtol=1e-13, atol=1e-13)


def test_row_subset_matches_full():
    rng = np.random.default_rng(6)
    W = rng.standard_normal((20, 16))
    X = rng.standard_normal((16, 7))
    blocks = random_mask(rng, 20, 16, 4, 4)
    Y = oracle.spmm(W, 4, 4, blocks, X)
    rows = [19, 0, 7, 7, 3]
    assert np.array_equal(oracle.spmm(W, 4, 4, blocks, X, rows=rows), Y[rows])


# ----------------------------------------------------------------------------- library special cases
def test_all_blocks_kept_is_dense_gemm():
    rng = np.random.default_rng(1)
    M, K, N, bh, bw = 24, 20, 9, 4, 5
    W = rng.standard_normal((M, K))
    X = rng.standard_normal((K, N))
    blocks = [(r, c) for r in range(0, M, bh) for c in range(0, K, bw)]
    assert oracle.validate(M, K, bh, bw, blocks) == M * K
    Y = oracle.spmm(W, bh, bw, blocks, X)
    np.testing.assert_allclose(Y, W @ X, rtol=1e-12, atol=1e-12)


def test_aligned_origins_are_bsr():
    rng = np.random.default_rng(2)
    M, K, N, bh, bw = 32, 24, 5, 4, 2
    W = rng.standard_normal((M, K))
    X = rng.standard_normal((K, N))
    cells = [(i, j) for i in range(M // bh) for j in range(K // bw)]
    keep = [cells[t] for t in rng.permutation(len(cells))[:30]]
    blocks = [(i * bh, j * bw) for i, j in keep]
    data = np.stack([W[r:r + bh, c:c + bw] for r, c in blocks])
    order = sorted(range(len(keep)), key=lambda t: keep[t])
    indptr = np.zeros(M // bh + 1, dtype=np.int64)
    for i, _ in keep:
        indptr[i + 1] += 1
    indptr = np.cumsum(indptr)
    bsr = sp.bsr_matrix((data[order], np.array([keep[t][1] for t in order]), indptr), shape=(M, K))
    Y = oracle.spmm(W, bh, bw, blocks, X)
    np.testing.assert_allclose(Y, bsr @ X, rtol=1e-12, atol=1e-12)


def test_single_block_closed_form():
    rng = np.random.default_rng(3)
    M, K, N, bh, bw, r, c = 11, 13, 4, 3, 5, 7, 6
    W = rng.standard_normal((M, K))
    X = rng.standard_normal((K, N))
    Y = oracle.spmm(W, bh, bw, [(r, c)], X)
    expect = np.zeros((M, N))
    expect[r:r + bh] = W[r:r + bh, c:c + bw] @ X[c:c + bw]
    np.testing.assert_allclose(Y, expect, rtol=1e-13, atol=1e-13)
    assert np.all(Y[:r] == 0) and np.all(Y[r + bh:] == 0)


def test_identity_x_returns_densified_w():
    rng = np.random.default_rng(4)
    M, K, bh, bw = 17, 15, 4, 3
    W = rng.standard_normal((M, K))
    blocks = random_mask(rng, M, K, bh, bw)
    Wd = np.zeros_like(W)
    for r, c in blocks:
        Wd[r:r + bh, c:c + bw] = W[r:r + bh, c:c + bw]
    assert np.array_equal(oracle.densify(W, bh, bw, blocks), Wd)
    assert np.array_equal(oracle.spmm(W, bh, bw, blocks, np.eye(K)), Wd)


def test_empty_block_list_gives_zero():
    Y = oracle.spmm(np.ones((5, 4)), 2, 2, np.zeros((0, 2), np.int32), np.ones((4, 3)))
    assert np.array_equal(Y, np.zeros((5, 3)))


# ----------------------------------------------------------------------------- format, independent re-derivation
def numpy_pack(W, bh, bw, blocks):
    """The format written again from its definition, with numpy indexing only."""
    M, K = W.shape
    blk = sorted((int(r), int(c)) for r, c in blocks)
    starts = np.array([r for r, _ in blk], dtype=np.int64)
    indptr = np.array([(starts < i).sum() for i in range(M - bh + 2)], dtype=np.int32)
    indices = np.array([c for _, c in blk], dtype=np.int32)
    values = np.zeros((len(blk), bw, bh), dtype=W.dtype)
    for b, (r, c) in enumerate(blk):
        rot = np.roll(W[r:r + bh, c:c + bw], r % bh, axis=0)   # row r lands in slot r mod bh
        values[b] = rot.T
    return indptr, indices, values.reshape(-1)


@pytest.mark.parametrize("bh,bw,dtype", [(3, 1, np.float32), (4, 4, np.float16), (8, 8, np.uint16),
                                          (16, 16, np.uint16), (5, 3, np.float64), (1, 1, np.float32)])
def test_pack_matches_definition(bh, bw, dtype):
    rng = np.random.default_rng(bh * 31 + bw)
    M, K = 45, 50
    W = rng.integers(1, 60000, size=(M, K)).astype(dtype)
    blocks = random_mask(rng, M, K, bh, bw, tries=60)
    got = oracle.pack(W, bh, bw, [blocks[t] for t in rng.permutation(len(blocks))])
    want = numpy_pack(W, bh, bw, blocks)
    for a, b in zip(got, want):
        assert a.dtype == b.dtype and np.array_equal(a, b)


# ----------------------------------------------------------------------------- validator and invariants
def test_validator_rejects_bad_lists():
    with pytest.raises(oracle.OracleError) as e:
        oracle.validate(8, 8, 4, 4, [(0, 0), (3, 3)])
    assert e.value.code == oracle.ORC_OVERLAP
    with pytest.raises(oracle.OracleError) as e:
        oracle.validate(8, 8, 4, 4, [(0, 0), (0, 0)])
    assert e.value.code == oracle.ORC_OVERLAP
    for bad in [(5, 0), (0, 5), (-1, 0), (0, -1)]:
        with pytest.raises(oracle.OracleError) as e:
            oracle.validate(8, 8, 4, 4, [bad])
        assert e.value.code == oracle.ORC_OUT_OF_BOUNDS
    assert oracle.validate(8, 8, 4, 4, [(0, 0), (4, 4), (0, 4), (4, 0)]) == 64
    assert oracle.validate(8, 8, 4, 4, [(1, 1)]) == 16


def test_generated_masks_satisfy_invariants():
    for (M, K, bh, bw, d, mode) in [(64, 64, 4, 4, 0.5, "uniform"), (96, 80, 8, 8, 0.2, "uniform"),
                                    (256, 256, 16, 16, 0.1, "zipf"), (60, 50, 3, 1, 0.3, "uniform")]:
        b = select_blocks(M, K, bh, bw, d, seed=11, mode=mode, zipf_s=1.1)
        nb = int(np.floor(M * K * d / (bh * bw) + 1e-9))
        assert len(b) == nb
        assert oracle.validate(M, K, bh, bw, b) == nb * bh * bw      # in bounds, disjoint, count


# ----------------------------------------------------------------------------- planted mistakes are caught
def test_planted_mistakes_fail_the_pins(worked_example):
    """Plausible wrong formats / sums differ from what the pins fix."""
    g, val = worked_example
    M, K, bh, bw, W, blocks = _example_arrays(g, val)
    want_vals = [val[L] for L in g["values"][0]]
    _, _, values = oracle.pack(W, bh, bw, blocks)
    unrotated = [W[r + d, c] for r, c in sorted(blocks) for d in range(bh)]
    wrong_dir = [W[r + (s + r) % bh, c] if r + (s + r) % bh < M else None
                 for r, c in sorted(blocks) for s in range(bh)]
    assert values.tolist() == want_vals
    assert unrotated != want_vals and wrong_dir != want_vals
    # transposed operand: W^T X differs from the pinned O_23
    X = np.arange(1.0, 1 + K * 4).reshape(K, 4)
    Y = oracle.spmm(W, bh, bw, blocks, X)
    assert not np.array_equal(Y, W.T[:M, :K] @ X)


def test_fused_epilogue_of_the_oracle():
    """The epilogue function against hand values: bias goes by output ROW (a transposed bias, a
    missing bias, relu before bias, swapped clamp bounds would all show), NaN becomes the lower
    bound."""
    Y = np.array([[1.0, -2.0, 0.5], [-1.0, 3.0, np.nan]])
    b = np.array([0.25, -0.5])
    assert np.array_equal(oracle.fused(Y), Y, equal_nan=True)
    assert oracle.fused(Y, b)[:, :2].tolist() == [[1.25, -1.75], [-1.5, 2.5]]
    assert oracle.fused(Y, b, "relu").tolist() == [[1.25, 0.0, 0.75], [0.0, 2.5, 0.0]]
    assert oracle.fused(Y, b, "clamp", -1.0, 2.0).tolist() == [[1.25, -1.0, 0.75], [-1.0, 2.0, -1.0]]
    assert oracle.fused(Y, None, "relu").tolist() == [[1.0, 0.0, 0.5], [0.0, 3.0, 0.0]]
    assert oracle.fused(Y[1:], b, "relu", rows=[1]).tolist() == [[0.0, 2.5, 0.0]]
    with pytest.raises(ValueError):
        oracle.fused(Y, b, "clamp", 1.0, 0.0)
