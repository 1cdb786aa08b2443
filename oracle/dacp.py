"""DACP scheduling heuristic -- TEST INFRASTRUCTURE ONLY (plain Python, exact rationals).

What it follows: the heuristic of Sec. 4.3.2 (Alg. 1) with the bookkeeping
functions UpdateLocal / UpdateAll / RollBack of App. A.1 (Alg. 3), the cost
function FLOPs(S) of App. B.2, and the constraints Eq. 7 (every sequence is
either distributed or local to exactly one rank) and Eq. 8 (per-rank token
budget C) of Sec. 4.1.  The steps are taken in the paper's order and notation
(S, C, N, RB, L, ret); S/N is kept as an exact fraction, as the paper uses it.

Readings (the listing is silent or inconsistent there):
  * ret values are ranks 0..N-1 (the text says ws-1) or -1 for "distributed";
    ret is returned in the caller's sequence order (the listing indexes the
    sorted array).  The sort is stable (equal lengths keep their order).
  * argmin / argmax take the lowest rank among equals.
  * FLOPs(S, N), which the listing never defines, is FLOPs(S) / N (Eq. 4).
  * "i <- i-1; continue" retries the same sequence after a roll-back.
  * RollBack prints RB[rank] <- RB[rank] - S + S/N, the pattern of its load update; RB
    is the REMAINING capacity, UpdateLocal took S off it, so undoing that and charging
    the slice is RB[rank] + S - S/N (with the printed sign a roll-back would shrink the
    bucket it is meant to relieve).
  * RollBack as printed only credits the rank it is called for; turning a local
    sequence into a distributed one also puts S/N tokens and FLOPs(S)/N of
    load on every OTHER rank (Eq. 4, Eq. 8), so those are charged too.
  * The text promises that the result respects Eq. 8; a run that ends with a
    negative remaining bucket anywhere is therefore reported as the
    scheduling error the text describes (None), like a failed roll-back.

Nothing here is imported by the product; the library's C++ implementation is
written separately (scaled integers instead of fractions).
"""
from __future__ import annotations

from fractions import Fraction


def flops(S: int, h: int, h_kv: int, b: int = 1) -> int:
    """FLOPs(S_k) = 20 b h^2 S + 4 b h h_kv S + 4 b h S^2  (App. B.2)."""
    return 20 * b * h * h * S + 4 * b * h * h_kv * S + 4 * b * h * S * S


def dacp_schedule(S_in, C: int, N: int, h: int, h_kv: int, b: int = 1):
    """Alg. 1.  Returns ret (list, caller's order: -1 = distributed, else the rank
    that holds the sequence whole) or None for a scheduling error."""
    K = len(S_in)
    order = sorted(range(K), key=lambda k: (S_in[k], k))  # Sort(SeqLens, ascending)
    S = [S_in[k] for k in order]
    RB = [Fraction(C) for _ in range(N)]  # remaining bucket (tokens)
    L = [Fraction(0) for _ in range(N)]   # load (FLOPs)
    ret = [None] * K                      # indexed like the sorted S

    def FLOPs(s, n=1):
        return Fraction(flops(s, h, h_kv, b), n)

    def UpdateLocal(idx, rank):
        RB[rank] -= S[idx]
        L[rank] += FLOPs(S[idx])

    def UpdateAll(idx):
        for i in range(N):
            RB[i] -= Fraction(S[idx], N)
            L[i] += FLOPs(S[idx], N)

    def RollBack(rank):
        for i in range(K):
            if ret[i] == rank:
                ret[i] = -1
                RB[rank] = RB[rank] + S[i] - Fraction(S[i], N)  # see "Readings" (sign)
                L[rank] = L[rank] - FLOPs(S[i]) + FLOPs(S[i], N)
                for other in range(N):  # see "Readings": the other ranks get their slices
                    if other != rank:
                        RB[other] -= Fraction(S[i], N)
                        L[other] += FLOPs(S[i], N)
                return True
        return False

    def argmin(a):
        return min(range(N), key=lambda j: (a[j], j))

    def argmax(a):
        return min(range(N), key=lambda j: (-a[j], j))

    i = 0
    while i < K:
        t = argmin(L)
        if RB[t] >= S[i]:
            ret[i] = t
            UpdateLocal(i, t)
        else:
            t = argmax(RB)
            if RB[t] >= S[i]:
                ret[i] = t
                UpdateLocal(i, t)
            else:
                t = argmin(RB)
                if RB[t] >= Fraction(S[i], N):
                    ret[i] = -1
                    UpdateAll(i)
                else:
                    if not RollBack(t):
                        return None
                    continue  # retry the same sequence
        i += 1
    if min(RB) < 0:
        return None
    out = [None] * K
    for pos, k in enumerate(order):
        out[k] = ret[pos]
    return out


def rank_batch(S, ret, N: int, j: int):
    """The micro-batch of CP rank j: its local sequences whole (degree 1) and slice j
    of every distributed one (degree N), in the caller's order.  Returns
    (seq_len, shard_degree, shard_index, source_index)."""
    seq, deg, idx, src = [], [], [], []
    for k, (s, r) in enumerate(zip(S, ret)):
        if r == -1:
            seq.append(s); deg.append(N); idx.append(j); src.append(k)
        elif r == j:
            seq.append(s); deg.append(1); idx.append(0); src.append(k)
    return seq, deg, idx, src
