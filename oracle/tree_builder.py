"""Oracle of the drafting-tree construction (Section 4 of the paper), from the property that defines the tree.

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: plain Python, vertices are index tuples (j_1, .., j_l).  R is the
0-th order acceptance function of the paper's experiments (Section 5): R(j_1 .. j_l) = r[j_1] * ... * r[j_l] with
r non-increasing (a later arrival is accepted less often).

Section 4: a vertex is accepted only if its parent is, so the expected number of accepted tokens of a tree is the sum
of R over its vertices, and the optimal tree of k vertices consists of the k vertices with the largest R.  That is
what this module computes, by enumeration: every vertex whose R reaches a threshold is listed (R does not grow along a
path or from a sibling to the next, which bounds the search), the list is sorted, the first k are the tree.  Equal
values are ordered by depth, then by index tuple, which keeps parents before children and siblings in order.
"""

MAX_LISTED = 2_000_000  # vertices this oracle is willing to list (equal values in great number exceed it)


def acceptance(r, idx):
    """R(idx) under the 0-th order model: the product along the path, from the root down."""
    value = 1.0
    for j in idx:
        value = value * r[j]
    return value


def _vertices_reaching(r, threshold, max_depth):
    """All vertices of depth <= max_depth with R >= threshold, as (R, index tuple)."""
    found = []
    stack = [((), 1.0)]
    while stack:
        idx, value = stack.pop()
        if len(idx) == max_depth:
            continue
        for j in range(len(r)):
            v = value * r[j]
            if v < threshold:
                break              # r does not increase: later siblings and all their descendants are below too
            found.append((v, idx + (j,)))
            if len(found) > MAX_LISTED:
                raise ValueError("too many vertices of equal or near-equal acceptance for this oracle")
            stack.append((idx + (j,), v))
    return found


def optimal_tree(r, k):
    """-> list of the k vertices (index tuples) with the largest R: decreasing R, then depth, then index tuple."""
    r = tuple(float(x) for x in r)
    assert all(0.0 <= x <= 1.0 for x in r) and all(a >= b for a, b in zip(r, r[1:])), "r must be non-increasing in [0, 1]"
    threshold = 1.0
    while True:
        found = _vertices_reaching(r, threshold, k)   # a tree of k vertices is at most k deep
        if len(found) >= k or threshold == 0.0:
            break
        threshold = threshold / 2 if threshold > 1e-300 else 0.0
    found.sort(key=lambda t: (-t[0], len(t[1]), t[1]))
    assert len(found) >= k, "fewer than k vertices exist (k deeper than the chain allows?)"
    return [idx for _, idx in found[:k]]


def flat(vertices):
    """Index tuples (in an order where parents come first) -> (parent, rank) lists, -1 = the root."""
    number = {(): -1}
    parent, rank = [], []
    for n, idx in enumerate(vertices):
        parent.append(number[idx[:-1]])
        rank.append(idx[-1])
        number[idx] = n
    return parent, rank


def specinfer_tree(k, shared=2, branches=3):
    """`branches` sequences sharing their first `shared` drafted tokens (Section 5's fixed comparison tree),
    grown in turn until k vertices are placed -> list of index tuples."""
    out = []
    prefix = ()
    while len(out) < k and len(prefix) < shared:
        prefix = prefix + (0,)
        out.append(prefix)
    tips = [None] * branches
    b = 0
    while len(out) < k:
        tips[b] = prefix + (b,) if tips[b] is None else tips[b] + (0,)
        out.append(tips[b])
        b = (b + 1) % branches
    return out
