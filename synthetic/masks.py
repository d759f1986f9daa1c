"""Seeded generator of valid unaligned block lists (test masks).

A block list is a set of non-overlapping bh x bw rectangles inside an M x K matrix,
each given by its top-left origin (r, c); origins are arbitrary (not multiples of the
block size).  Non-overlap and the block count follow the constraints of Eq. 2 and the
count rule m = floor(b (1 - p) / N) of Section 3.1, generalised from 1-D runs to
rectangles.

The recipe is fixed so that an independent implementation of it reproduces the same
lists bit for bit:

* RNG: SplitMix64 seeded with `seed`; `bounded(n)` draws 64-bit words until one is
  below floor(2^64 / n) * n and returns it modulo n (unbiased).
* count: nb = floor(M * K * density / (bh * bw) + 1e-9), evaluated in IEEE double in
  exactly that order.
* "uniform": repeat { r = bounded(M - bh + 1); c = bounded(K - bw + 1) }, accept the
  candidate iff all its cells are free, until nb are accepted.
* "zipf": stripes of bh origin rows, S = ceil((M - bh + 1) / bh) of them.  Stripe
  targets by water-filling t = min(cap, lambda * rank^-s), cap = floor(0.375 * K / bw),
  sum t = nb, rounded by largest remainder (ties to the lower rank); ranks are mapped to
  stripes by a Fisher-Yates shuffle driven by the same RNG (before any sampling); then
  stripe by stripe, r = bh * stripe + bounded(rows in stripe), c = bounded(K - bw + 1),
  accept iff free.
* "col_aligned": as "uniform" with c = bw * bounded(K // bw): the paper's convolution block
  (N, 1, h, w), which in the lowered matrix is N x (h w) with a column origin that is a multiple
  of h w (Section 3.1); rows stay unaligned.
* "aligned": r = bh * bounded(M // bh), c = bw * bounded(K // bw): aligned block pruning, the
  special case the paper compares against (Section 3.1, Section 5.4).
* the result is sorted by (r, c).
"""
import math
import numpy as np

_M64 = (1 << 64) - 1


class SplitMix64:
    def __init__(self, seed: int):
        self.s = seed & _M64

    def next(self) -> int:
        self.s = (self.s + 0x9E3779B97F4A7C15) & _M64
        z = self.s
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _M64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _M64
        return z ^ (z >> 31)

    def bounded(self, n: int) -> int:
        limit = ((1 << 64) // n) * n
        while True:
            x = self.next()
            if x < limit:
                return x % n


def target_block_count(M, K, bh, bw, density) -> int:
    return int(math.floor((float(M) * float(K) * float(density)) / float(bh * bw) + 1e-9))


def zipf_stripe_targets(nb, S, cap, s):
    """Integer per-rank targets: water-filled min(cap, lambda * rank^-s), sum == nb."""
    if nb > S * cap:
        raise ValueError("infeasible: nb exceeds the capped capacity")
    w = [math.pow(float(j + 1), -float(s)) for j in range(S)]
    capped = [False] * S
    remaining = float(nb)
    lam = 0.0
    while True:
        wsum = 0.0
        for j in range(S):
            if not capped[j]:
                wsum += w[j]
        if wsum <= 0.0:
            break
        lam = remaining / wsum
        changed = False
        for j in range(S):
            if not capped[j] and lam * w[j] > float(cap):
                capped[j] = True
                remaining -= float(cap)
                changed = True
        if not changed:
            break
    real = [float(cap) if capped[j] else lam * w[j] for j in range(S)]
    t = [int(math.floor(x)) for x in real]
    left = nb - sum(t)
    frac = [real[j] - float(t[j]) for j in range(S)]
    order = sorted(range(S), key=lambda j: (-frac[j], j))
    i = 0
    while left > 0:
        j = order[i % S]
        if t[j] < cap:
            t[j] += 1
            left -= 1
        i += 1
    return t


def select_blocks(M, K, bh, bw, density, seed, mode="uniform", zipf_s=0.0):
    """Return an int32 array [nb, 2] of (r, c) origins, sorted by (r, c)."""
    if bh < 1 or bw < 1 or bh > M or bw > K or not (0.0 <= density <= 1.0):
        raise ValueError("bad arguments")
    nb = target_block_count(M, K, bh, bw, density)
    rng = SplitMix64(seed)
    occ = np.zeros((M, K), dtype=bool)
    out = []
    nr, nc = M - bh + 1, K - bw + 1
    max_attempts = 2000 * nb + 100000

    def fill(count, r_base, r_span, r_unit=1, c_unit=1):
        attempts = 0
        got = 0
        while got < count:
            attempts += 1
            if attempts > max_attempts:
                raise RuntimeError("infeasible: rejection sampling did not terminate")
            r = r_base + r_unit * rng.bounded(r_span)
            c = c_unit * rng.bounded(nc if c_unit == 1 else K // bw)
            cell = occ[r:r + bh, c:c + bw]
            if cell.any():
                continue
            cell[...] = True
            out.append((r, c))
            got += 1

    if mode == "uniform":
        fill(nb, 0, nr)
    elif mode == "col_aligned":
        fill(nb, 0, nr, 1, bw)
    elif mode == "aligned":
        if nb > (M // bh) * (K // bw):
            raise ValueError("infeasible: more blocks than aligned positions")
        fill(nb, 0, M // bh, bh, bw)
    elif mode == "zipf":
        S = (nr + bh - 1) // bh
        cap = int(math.floor(0.375 * float(K) / float(bw)))
        t_rank = zipf_stripe_targets(nb, S, cap, zipf_s)
        perm = list(range(S))
        for i in range(S - 1, 0, -1):
            j = rng.bounded(i + 1)
            perm[i], perm[j] = perm[j], perm[i]
        t_stripe = [0] * S
        for rank in range(S):
            t_stripe[perm[rank]] = t_rank[rank]
        for st in range(S):
            rows = min(bh, nr - bh * st)
            fill(t_stripe[st], bh * st, rows)
    else:
        raise ValueError("unknown mode")
    out.sort()
    return np.asarray(out, dtype=np.int32).reshape(-1, 2)
