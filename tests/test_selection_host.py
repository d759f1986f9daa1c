"""The library's block selectors (host functions of the C ABI) against the selection oracle, index
by index on the same seeded scores, and on layer-sized inputs through properties that hold at any
size."""
import time

import numpy as np
import pytest

import paper_2407_19644_amd as ubp
from oracle import selection as sel
from synthetic import decode_f64, encode

NEG = -np.inf


def _weights(rng, c_out, K, dtype="f32", integer=False):
    W = rng.integers(-9, 10, size=(c_out, K)).astype(np.float64) if integer else rng.standard_normal((c_out, K))
    enc = encode(W, dtype)
    return enc, decode_f64(enc, dtype)


def _valid(I, S, N):
    I = np.sort(np.asarray(I))
    assert len(np.unique(I)) == len(I)
    assert (S[I] > NEG).all()
    assert (np.diff(I) >= N).all()


# ------------------------------------------------------------------ Eq. 1
@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
@pytest.mark.parametrize("shape", [(8, 6, 2, 1), (33, 20, 4, 3), (16, 16, 16, 16), (40, 27, 5, 9), (7, 5, 7, 2)])
def test_scores_match_oracle(dtype, shape):
    c_out, K, N, bw = shape
    rng = np.random.default_rng(c_out * 131 + K)
    enc, W = _weights(rng, c_out, K, dtype)
    for aligned in (False, True):
        S = ubp.block_scores(enc, dtype, N, bw, aligned)
        want = sel.block_scores(W, N, bw, aligned)
        assert S.shape == want.shape
        assert ((S == NEG) == (want == NEG)).all()
        fin = want > NEG
        np.testing.assert_allclose(S[fin], want[fin], rtol=1e-13, atol=0)


def test_scores_with_a_pitch_and_bad_arguments():
    rng = np.random.default_rng(1)
    big = rng.standard_normal((10, 12)).astype(np.float32)
    view = big[:, :9]
    S = ubp.block_scores(view, "f32", 3, 2)
    want = sel.block_scores(view.astype(np.float64), 3, 2)
    np.testing.assert_allclose(S[want > NEG], want[want > NEG], rtol=1e-13)
    with pytest.raises(ubp.UBPError) as e:
        ubp.block_scores(view, "f32", 11, 2)                             # block taller than the matrix
    assert e.value.code == 1


# ------------------------------------------------------------------ the three selectors, index by index
@pytest.mark.parametrize("seed", range(60))
def test_selectors_match_oracle(seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(1, 9))
    c_in = int(rng.integers(1, 7))
    c_out = int(rng.integers(N, 70))
    _, W = _weights(rng, c_out, c_in, integer=bool(seed % 3 == 0))     # integer scores: many ties
    S = sel.block_scores(W, N, aligned=bool(seed % 7 == 3))
    if seed % 5 == 4:                                                    # forbid some candidates outright
        S[rng.integers(0, len(S), size=len(S) // 4)] = NEG
    cap = c_in * (c_out // N)
    for m in sorted({0, 1, cap // 4, cap // 2, cap, cap + 3}):
        assert ubp.select_greedy(S, N, m).tolist() == sel.select_greedy(S, N, m)
        assert ubp.select_bed(S, N, m).tolist() == sel.select_bed(S, N, m)
        want = sel.select_optimal(S, N, m)
        if want is None:
            with pytest.raises(ubp.UBPError) as e:
                ubp.select_optimal(S, N, m)
            assert e.value.code == 5
        else:
            assert ubp.select_optimal(S, N, m).tolist() == want


def test_the_two_examples_of_the_text():
    e = np.array([4., 9., 8., 5., 2., 7., 6., 1.])                      # Section 3.2: N = 2, three blocks
    S = sel.block_scores(e.reshape(-1, 1), 2)
    assert ubp.select_greedy(S, 2, 3).tolist() == [1, 5, 3]
    assert ubp.select_optimal(S, 2, 3).tolist() == [0, 2, 5]
    assert ubp.select_bed(S, 2, 3).tolist() == [0, 2, 5]
    e = np.array([5., 9., 9., 4., 1., 0.5])                              # Section 4.1: w0 and w3 join (w1, w2)
    S = sel.block_scores(e.reshape(-1, 1), 2)
    assert ubp.select_bed(S, 2, 2).tolist() == [0, 2]
    assert ubp.select_greedy(S, 2, 2).tolist() == [1, 3]


def test_scores_that_are_not_ordered_are_refused():
    for bad in (np.nan, np.inf):
        S = np.array([1., bad, 2., NEG])
        for f in (ubp.select_greedy, ubp.select_bed, ubp.select_optimal):
            with pytest.raises(ubp.UBPError) as e:
                f(S, 2, 1)
            assert e.value.code == 1
    assert ubp.select_greedy(np.zeros(0), 2, 3).size == 0
    assert ubp.select_bed(np.zeros(0), 2, 3).size == 0
    with pytest.raises(ubp.UBPError):
        ubp.select_greedy(np.ones(4), 0, 1)                              # N < 1


# ------------------------------------------------------------------ layer-sized inputs
def test_layer_sized_selection_properties():
    """256 x 256 layer, N = 4, 30 % density: sizes the oracle's expansion still finishes (it is
    compared index by index), the optimum checked through what must hold: valid, exactly m blocks,
    total >= expansion+division >= ... and >= greedy; aligned pruning <= all of them."""
    rng = np.random.default_rng(77)
    c_out = c_in = 256
    N = 4
    enc, W = _weights(rng, c_out, c_in, "f16")
    S = ubp.block_scores(enc, "f16", N, 1)
    Sa = ubp.block_scores(enc, "f16", N, 1, aligned=True)
    m = ubp.target_block_count(c_out, c_in, N, 1, 0.3)
    t0 = time.perf_counter()
    g = ubp.select_greedy(S, N, m)
    t1 = time.perf_counter()
    b = ubp.select_bed(S, N, m)
    t2 = time.perf_counter()
    o = ubp.select_optimal(S, N, m)
    t3 = time.perf_counter()
    a = ubp.select_greedy(Sa, N, m)
    print("greedy %.1f ms, expansion+division %.1f ms, optimal %.1f ms" % ((t1 - t0) * 1e3, (t2 - t1) * 1e3, (t3 - t2) * 1e3))
    for I in (g, b, o, a):
        assert len(I) == m
        _valid(I, S, N)
    assert (a % c_out % N == 0).all()
    tot = {k: float(S[v].sum()) for k, v in dict(g=g, b=b, o=o, a=a).items()}
    assert tot["o"] >= tot["b"] - 1e-9 and tot["o"] >= tot["g"] - 1e-9
    assert tot["b"] > tot["g"] > tot["a"]
    assert b.tolist() == sel.select_bed(S, N, m)
    assert g.tolist() == sel.select_greedy(S, N, m)
    # Eq. 5 through the library and through the oracle
    blocks = {k: ubp.selection_to_blocks(v, c_out, 1) for k, v in dict(g=g, b=b, o=o, a=a).items()}
    eff = {}
    for k in "gbo":
        eff[k], l1 = ubp.selection_efficacy(enc, "f16", N, 1, blocks[k], blocks["a"])
        want = sel.efficacy(W, N, v := dict(g=g, b=b, o=o)[k].tolist(), a.tolist())
        assert eff[k] == pytest.approx(want, rel=1e-12)
        assert l1[0] == pytest.approx(sel.kept_l1(W, v, N), rel=1e-12)
        assert l1[0] == pytest.approx(tot[k], rel=1e-12)
    assert 0.0 < eff["g"] < eff["b"] <= eff["o"] < 1.0
    assert eff["o"] - eff["b"] < 0.25 * (eff["o"] - eff["g"])           # expansion+division closes most of greedy's gap


def test_select_blocks_feeds_pack():
    rng = np.random.default_rng(9)
    enc, W = _weights(rng, 64, 96, "bf16")
    for method in ("greedy", "bed", "optimal"):
        for bh, bw, aligned in ((4, 1, False), (8, 3, False), (4, 4, True), (16, 16, False)):
            blocks = ubp.select_blocks(enc, "bf16", bh, bw, 0.25, method, aligned)
            S = sel.block_scores(W, bh, bw, aligned)
            m = ubp.target_block_count(64, 96, bh, bw, 0.25)
            want = dict(greedy=sel.select_greedy, bed=sel.select_bed, optimal=sel.select_optimal)[method](S, bh, m)
            assert blocks.tolist() == sel.indices_to_blocks(want, 64, bw).tolist()
            if aligned:
                assert (blocks[:, 0] % bh == 0).all()
            assert (blocks[:, 1] % bw == 0).all()
            p = ubp.pack(enc, "bf16", bh, bw, blocks)                   # host-only handle: the list is a valid one
            assert p.info(4) == len(blocks)
            p.free()
    with pytest.raises(ubp.UBPError):
        ubp.select_blocks(enc, "bf16", 4, 1, 1.5)


def test_expansion_is_fast_on_the_largest_layer_shape():
    """2048 x 512 candidates (the size of a ResNet-50 stage-4 1x1 layer), N = 2, half of the weights
    kept: the case the text times at tens of seconds (Section 5.1)."""
    rng = np.random.default_rng(2)
    c_out, c_in, N = 2048, 512, 2
    W = np.abs(rng.standard_normal((c_out, c_in))).astype(np.float32)
    S = ubp.block_scores(W, "f32", N, 1)
    m = ubp.target_block_count(c_out, c_in, N, 1, 0.5)
    t0 = time.perf_counter()
    b = ubp.select_bed(S, N, m)
    t1 = time.perf_counter()
    g = ubp.select_greedy(S, N, m)
    t2 = time.perf_counter()
    print("b = %d, m = %d: expansion+division %.2f s, greedy %.2f s" % (len(S), m, t1 - t0, t2 - t1))
    assert len(b) == m
    _valid(b, S, N)
    _valid(g, S, N)
    assert S[b].sum() > S[g].sum()
    assert t1 - t0 < 20.0
    with pytest.raises(ubp.UBPError) as e:                               # the optimum's table would not fit
        ubp.select_optimal(S, N, m)
    assert e.value.code == 4
