"""GDS scheduling heuristic -- TEST INFRASTRUCTURE ONLY (plain Python, exact integers).

What it follows: the global data scheduling heuristic of Sec. 4.3.2 (Alg. 2): bin-pack
the global batch over the DP ranks by FLOPs(S) (App. B.2), take this rank's subset,
sort it ascending, cut it into `init` micro-batches by stride (Subset[j::init], which
pairs long sequences with short ones), and take one micro-batch more whenever a
micro-batch exceeds the C*N tokens of Eq. "sum_k B_kij S_k <= C*N" (Sec. 4.2, joint
formulation) or DACP (Alg. 1) cannot schedule it.

Readings (the listing is garbled or silent there):
  * Binpack is not named.  Reading: longest-processing-time greedy -- sequences by
    descending FLOPs (stable: equal costs keep the caller's order), each to the bin
    with the least load so far (lowest rank among equals).
    The paper fixes no values for it (parity unpinned as far as the choice of algorithm
    goes); the tests pin what any such greedy must satisfy: Graham's bound
    (4/3 - 1/(3 ws)) against the brute-force optimum, and its special cases.
  * "init <- ceil(Sum(Subset)/C x N) - 1" is ceil(Sum / (C*N)) - 1: the loop adds one
    before its first use, so the first attempt is the smallest number of micro-batches
    the token constraint allows (at least 1).
  * "for j <- 0 to init" builds exactly init micro-batches, j = 0 .. init-1 (a stride
    of init has that many residues).  Empty ones (init > |Subset|) are left out.
  * The overflow test prints ">= C x N"; the constraint it enforces allows equality, and
    so does this reading (a micro-batch is rejected if its tokens EXCEED C*N).
  * "Continue" inside the for loop means: give this init up and try init + 1.
  * The while bound "init <= K+1" never ends a successful run early; the run fails
    (None) when even one sequence per micro-batch is rejected, i.e. init > |Subset|.
  * A DP rank whose bin is empty gets no micro-batches.
  * The sort of Subset is stable on (length, caller's position).

Nothing here is imported by the product.
"""
from __future__ import annotations

from .dacp import dacp_schedule, flops


def binpack(S, ws: int, h: int, h_kv: int, b: int = 1):
    """bin[k] = DP rank of sequence k (Alg. 2 line 1)."""
    cost = [flops(s, h, h_kv, b) for s in S]
    order = sorted(range(len(S)), key=lambda k: (-cost[k], k))
    load = [0] * ws
    out = [None] * len(S)
    for k in order:
        i = min(range(ws), key=lambda r: (load[r], r))
        out[k] = i
        load[i] += cost[k]
    return out


def gds_schedule(S, C: int, N: int, ws: int, dp_rank: int, h: int, h_kv: int, b: int = 1):
    """Alg. 2 for DP rank `dp_rank`.  Returns (bin, mbs) where bin[k] is the DP rank of
    every sequence and mbs is this rank's list of micro-batches, each a list of
    (k, ret_k) in ascending-length order with ret_k the DACP decision; None if some
    sequence cannot be scheduled at all."""
    bins = binpack(S, ws, h, h_kv, b)
    Subset = sorted((k for k in range(len(S)) if bins[k] == dp_rank), key=lambda k: (S[k], k))
    if not Subset:
        return bins, []
    Sum = sum(S[k] for k in Subset)
    init = -(-Sum // (C * N)) - 1
    while init < len(Subset):
        init += 1
        mbs, ok = [], True
        for j in range(init):
            mb = Subset[j::init]
            if not mb:
                continue
            if sum(S[k] for k in mb) > C * N:
                ok = False
                break
            ret = dacp_schedule([S[k] for k in mb], C, N, h, h_kv, b)
            if ret is None:
                ok = False
                break
            mbs.append(list(zip(mb, ret)))
        if ok:
            return bins, mbs
    return None
