"""Oracle of the automatic stage partitioning (paper Sec. 4.4).

TEST INFRASTRUCTURE ONLY (see the package docstring).

Model (Sec. 3.2, asymmetric stage splitting; Sec. 3.3, bubble analysis): forward stages F_1..F_Sf cover the front
layers, backward stages B_1..B_Sb cover all layers from the back, B_1 (the last layers) is fused -- its forward is the
recomputation -- so sum F + B_1 = sum B = L.  GPU time of the pipeline = (M S + N (N - 1)) t_max with S = Sf + Sb and
t_max the longest stage; no stage may exceed the memory limit.

`brute_force` is the definition: every pair of partitions is tried.  `partition` follows the paper's algorithm: the
candidates for t_max are the sums of contiguous runs of forward and of backward times; for each, stages are packed
greedily, the fused stage first and as full as possible; the cheapest candidate wins.  The paper does not say how a
layer's time inside the fused stage relates to its backward time (taken equal: forward + backward proper is what a
recomputing backward stage executes), nor how ties are broken (fewer stages, then the earlier candidate).
"""
import itertools


def compositions(n):
    """All ordered ways to write n as a sum of positive integers."""
    if n == 0:
        yield ()
        return
    for cuts in itertools.product((0, 1), repeat=n - 1):
        parts, run = [], 1
        for c in cuts:
            if c:
                parts.append(run)
                run = 1
            else:
                run += 1
        parts.append(run)
        yield tuple(parts)


def evaluate(fwd, bwd, tf, tb, mf, mb, mem, n_gpus, n_micro):
    """Cost of a given pair of partitions, or None if a stage exceeds the memory limit.  bwd[0] is the fused stage."""
    L = len(tf)
    assert sum(bwd) == L and sum(fwd) + bwd[0] == L
    t_max = 0.0
    hi = L
    for n in bwd:
        t_max = max(t_max, sum(tb[hi - n:hi]))
        if sum(mb[hi - n:hi]) > mem:
            return None
        hi -= n
    lo = 0
    for n in fwd:
        t_max = max(t_max, sum(tf[lo:lo + n]))
        if sum(mf[lo:lo + n]) > mem:
            return None
        lo += n
    return (n_micro * (len(fwd) + len(bwd)) + n_gpus * (n_gpus - 1)) * t_max


def brute_force(tf, tb, mf, mb, mem, n_gpus, n_micro):
    """Smallest cost over every pair of partitions (small L only), or None when nothing is feasible."""
    L = len(tf)
    best = None
    for bwd in compositions(L):
        for fwd in compositions(L - bwd[0]):
            c = evaluate(fwd, bwd, tf, tb, mf, mb, mem, n_gpus, n_micro)
            if c is not None and (best is None or c < best):
                best = c
    return best


def pack(tf, tb, mf, mb, mem, t):
    """Greedy packing under the bound t.  Returns (fwd, bwd, t_max) or None."""
    L = len(tf)
    bwd, t_max = [], 0.0
    hi = L
    while hi > 0:
        st, sm, n = 0.0, 0.0, 0
        while hi - n > 0 and st + tb[hi - n - 1] <= t and sm + mb[hi - n - 1] <= mem:
            st += tb[hi - n - 1]
            sm += mb[hi - n - 1]
            n += 1
        if n == 0:
            return None
        bwd.append(n)
        t_max = max(t_max, st)
        hi -= n
    fwd, lo, lf = [], 0, L - bwd[0]
    while lo < lf:
        st, sm, n = 0.0, 0.0, 0
        while lo + n < lf and st + tf[lo + n] <= t and sm + mf[lo + n] <= mem:
            st += tf[lo + n]
            sm += mf[lo + n]
            n += 1
        if n == 0:
            return None
        fwd.append(n)
        t_max = max(t_max, st)
        lo += n
    return fwd, bwd, t_max


def partition(tf, tb, mf, mb, mem, n_gpus, n_micro):
    """The paper's O(L^3) algorithm.  Returns (fwd, bwd, t_max, cost) or None."""
    L = len(tf)
    best = None
    for tt in (tf, tb):
        for i in range(L):
            s = 0.0
            for j in range(i, L):
                s += tt[j]
                got = pack(tf, tb, mf, mb, mem, s)
                if got is None:
                    continue
                fwd, bwd, t_max = got
                cost = (n_micro * (len(fwd) + len(bwd)) + n_gpus * (n_gpus - 1)) * t_max
                if best is None or cost < best[3] or (cost == best[3] and len(fwd) + len(bwd) < len(best[0]) + len(best[1])):
                    best = (fwd, bwd, t_max, cost)
    return best
