"""Stage split oracle -- TEST INFRASTRUCTURE ONLY.

The paper cuts a DNN into sequential stages along its logical structure (Sec. III-B1) and gives no rule for an
arbitrary stage count k.  Reading taken: a cut after layer l is legal when every later layer reads only l's
output or later tensors (exactly one tensor crosses the boundary); among all choices of k-1 legal cuts take the
one minimising the largest per-stage multiply-accumulate count, ties to the lexicographically smallest cut
tuple.  This file is the plain definition: enumerate every combination.
"""
from itertools import combinations


def legal_cuts(layers):
    n = len(layers)
    out = []
    for l in range(n - 1):
        ok = True
        for q in range(l + 1, n):
            L = layers[q]
            if L.in_from < l or (0 <= L.res_from < l):
                ok = False
                break
        if ok:
            out.append(l)
    return out


def split(macs, legal, k):
    """First layer of each stage, or None if k-1 exceeds the number of legal cuts."""
    n = len(macs)
    if k - 1 > len(legal):
        return None
    best, best_cost = None, None
    for cuts in combinations(legal, k - 1):          # lexicographic order
        bounds = [0] + [c + 1 for c in cuts] + [n]
        cost = max(sum(macs[a:b]) for a, b in zip(bounds, bounds[1:]))
        if best_cost is None or cost < best_cost:    # strict: first (smallest) tuple wins ties
            best, best_cost = cuts, cost
    return [0] + [c + 1 for c in best]
