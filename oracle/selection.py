"""CPU oracle for block selection: which m of the b candidate 1xN blocks of a layer are kept.

TEST INFRASTRUCTURE ONLY: imported by tests/, never by the product package.  Plain numpy and
Python loops, float64, no blocking and no cleverness: every function takes the steps of the
passage it cites, in that passage's order and notation.  Sizes of a few thousand candidates
finish in seconds; nothing here is meant to be fast.

Notation (Section 3.1).  A layer has c_out output channels and c_in input channels.  Candidate
block k = i + c_out * j starts at output channel i of input channel j and covers output channels
i .. i+N-1, so the candidates of one input channel are consecutive in k and a block that would
run past channel c_out-1 has score -inf (Eq. 1).  b = c_out * c_in, and m = floor(b (1-p) / N)
blocks are kept at pruning rate p.  No two kept blocks may share a weight, which in k means that
any N consecutive candidates hold at most one kept block (Eq. 2).

Readings taken where the text leaves a choice (they are listed with the design notes too):
  * arg max returns the lowest index among equal scores;
  * a selector stops early, returning fewer than m indices, once no candidate with a score above
    -inf is left (greedy, expansion) or when no m non-overlapping candidates exist (optimal: it
    returns None);
  * Algorithm 1 indexes the *shrinking* score list: after a removal, positions k-n and k-n+N are
    positions in the list as it stands, which is what makes line 8 the score of the block formed
    by the n elements left of the removed block and the N-n elements right of it;
  * in Algorithm 1 a position k-n below 0 is skipped, and a position k-n+N past the end of the
    list reads as -inf (the joined block would run past the last weight);
  * Eq. 4's T[k, n] is read over prefixes: T[k, n] is the best total of n blocks chosen among the
    first k candidates (candidates 0 .. k-1); choosing candidate k-1 leaves the first k-N
    candidates for the other n-1; T[k, 0] = 0, and T[k, n] = -inf for k <= 0 < n.

Parity pins (tests/test_selection_oracle.py): exhaustive enumeration of every valid selection for
b <= 16 (the optimal selector equals the best one; greedy and expansion+division are valid and
never better), the two examples the text walks through (Section 3.2's greedy example and
Section 4.1's expansion example, with scores chosen to produce the described order since the
figures' numbers are not in the text), closed forms (N = 1: all three are the top-m; two blocks
that tile the layer), and the invariant that the scores recorded by Algorithm 1 add up to the l1
norm kept by the divided blocks.
"""
import numpy as np

NEG = -np.inf


def block_scores(W, N, bw=1, aligned=False):
    """Eq. 1 with F = l1 norm.  W: (c_out, K) float64 array whose K columns are c_in = K // bw
    groups of bw consecutive columns (one input channel's h*w kernel weights each).  Returns
    S of length b = c_out * c_in with S[i + c_out*j] = sum |W[i:i+N, j*bw:(j+1)*bw]|, and -inf
    where i+N-1 >= c_out.  aligned=True additionally sets -inf where i is not a multiple of N,
    which turns every selector below into aligned block-wise pruning (remark after Eq. 2)."""
    W = np.asarray(W, dtype=np.float64)
    c_out, K = W.shape
    c_in = K // bw
    S = np.full(c_out * c_in, NEG)
    for j in range(c_in):
        for i in range(c_out):
            if i + N - 1 < c_out and not (aligned and i % N):
                S[i + c_out * j] = np.abs(W[i:i + N, j * bw:(j + 1) * bw]).sum()
    return S


def select_greedy(S, N, m):
    """Greedy selection (Section 3.2, Eq. 3): take the best remaining candidate m times; when k
    is taken, S[k+n] = -inf for every -N < n < N."""
    S = np.array(S, dtype=np.float64)
    b = len(S)
    I = []
    for _ in range(m):
        if b == 0:
            break
        k = int(np.argmax(S))
        if S[k] == NEG:
            break
        I.append(k)
        for n in range(-N + 1, N):
            if 0 <= k + n < b:
                S[k + n] = NEG
    return I


def select_optimal(S, N, m):
    """Optimal selection by dynamic programming (Section 3.2, Eq. 4): tables T[k, n] and index
    sets I[k, n] filled for k = 1..b, n = 1..m; the answer is I[b, m] (sorted), or None when no m
    candidates with finite scores fit."""
    S = np.asarray(S, dtype=np.float64)
    b = len(S)
    if m == 0:
        return []

    def T_at(T, k, n):
        if n == 0:
            return 0.0
        return T[k][n] if k > 0 else NEG

    def I_at(I, k, n):
        return I[k][n] if (k > 0 and n > 0) else ()

    T = [[NEG] * (m + 1) for _ in range(b + 1)]
    I = [[()] * (m + 1) for _ in range(b + 1)]
    for k in range(1, b + 1):
        for n in range(1, m + 1):
            take = T_at(T, k - N, n - 1) + S[k - 1]
            skip = T_at(T, k - 1, n)
            T[k][n] = max(take, skip)
            if T[k][n] > skip:
                I[k][n] = I_at(I, k - N, n - 1) + (k - 1,)
            else:
                I[k][n] = I_at(I, k - 1, n)
    if T[b][m] == NEG:
        return None
    return list(I[b][m])


def block_expansion(S, N, m):
    """Algorithm 1.  Returns (I_bar, picked): the index set of the expanded blocks, in the order
    they were chosen, and the score each had when it was chosen."""
    S = [float(v) for v in S]
    R = list(range(len(S)))
    I_bar, picked = [], []
    for _ in range(m):
        if not S:
            break
        k = int(np.argmax(S))
        if S[k] == NEG:
            break
        for n in range(1, N):
            if k - n < 0:
                continue
            right = S[k - n + N] if k - n + N < len(S) else NEG
            S[k - n] = S[k - n] + right - S[k]
        picked.append(S[k])
        I_bar.append(R[k])
        del S[k:k + N]
        del R[k:k + N]
    return I_bar, picked


def block_division(I_bar, N):
    """Algorithm 2: the expanded index set, sorted, re-cut into blocks of N."""
    I = []
    next_idx = 0
    for k in sorted(I_bar):
        if next_idx > k:
            I.append(next_idx)
            next_idx = next_idx + N
        else:
            I.append(k)
            next_idx = k + N
    return I


def select_bed(S, N, m):
    """Block expansion and division (Section 4.1): Algorithm 1, then Algorithm 2."""
    return block_division(block_expansion(S, N, m)[0], N)


def indices_to_blocks(I, c_out, bw=1):
    """k = i + c_out * j  ->  block origin (row i, column j*bw) of the (c_out, K) weight matrix."""
    return np.array([(k % c_out, (k // c_out) * bw) for k in I], dtype=np.int32).reshape(-1, 2)


def kept_l1(W, I, N, bw=1):
    """l1 norm of the weights the blocks I keep (each weight once)."""
    W = np.asarray(W, dtype=np.float64)
    c_out = W.shape[0]
    keep = np.zeros(W.shape, dtype=bool)
    for k in I:
        i, j = k % c_out, k // c_out
        keep[i:i + N, j * bw:(j + 1) * bw] = True
    return float(np.abs(W[keep]).sum())


def efficacy(W, N, I_ubp, I_abp, bw=1):
    """Eq. 5: (|W_UBP| - |W_ABP|) / (|W_EP| - |W_ABP|), all l1 norms of what is kept; element-wise
    pruning keeps the |I_ubp| * N * bw largest magnitudes."""
    W = np.asarray(W, dtype=np.float64)
    n_keep = len(I_ubp) * N * bw
    mags = np.sort(np.abs(W).ravel())[::-1]
    ep = float(mags[:n_keep].sum())
    ubp, abp = kept_l1(W, I_ubp, N, bw), kept_l1(W, I_abp, N, bw)
    return (ubp - abp) / (ep - abp)
