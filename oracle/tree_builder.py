"""Oracle of the drafting-tree construction (Algorithm 3 of the paper), in the paper's own terms.

TEST INFRASTRUCTURE ONLY, like the rest of oracle/: plain Python, vertices are index tuples (j_1, .., j_l), the
priority queue is a list searched for its maximum.  R is the 0-th order acceptance function of the paper's
experiments (Section 5): R(j_1 .. j_l) = r[j_1] * ... * r[j_l].
"""


def acceptance(r, idx):
    """R(idx) under the 0-th order model: the product along the path, from the root down."""
    value = 1.0
    for j in idx:
        value = value * r[j]
    return value


def optimal_tree(r, k):
    """Algorithm 3: -> list of the k vertices (index tuples) in the order they join the tree.

    The queue starts with the root's first child (0).  Each step takes the vertex with the largest R out of the
    queue (equal values: the one that entered first), adds it to the tree and offers its first child and, if
    there is one, its next sibling.
    """
    tree = [()]
    queue = [(acceptance(r, (0,)), 0, (0,))]  # (R, entry number, vertex)
    entered = 1
    for _ in range(k):
        best = 0
        for q in range(1, len(queue)):
            if queue[q][0] > queue[best][0] or (queue[q][0] == queue[best][0] and queue[q][1] < queue[best][1]):
                best = q
        _, _, idx = queue.pop(best)
        tree.append(idx)
        child = idx + (0,)
        queue.append((acceptance(r, child), entered, child))
        entered += 1
        if idx[-1] + 1 < len(r):
            sibling = idx[:-1] + (idx[-1] + 1,)
            queue.append((acceptance(r, sibling), entered, sibling))
            entered += 1
    return tree[1:]


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
