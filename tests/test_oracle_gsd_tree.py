"""The oracle of GSD on a draft tree (Algorithm 4's verification: recursive rejection over the children of a context)
pinned by: the sequence oracle on chains, a literal restatement with lists of probabilities, the target law of the
emitted token (the property the procedure exists for), and special cases.  No GPU."""
import numpy as np
import pytest
from scipy import stats

import mini_oracle


def softmax(z):
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def literal(draft, target, parent, rank, tokens, T, seed, oracle_mod, max_rank=8):
    """Algorithm 4's verification written with Python lists, exponentials from the pure-Python generator."""
    B, C, V = draft.shape
    N = C - 1
    rounds = oracle_mod.get_rounds()
    valid, _ = oracle_mod.arrival_tree_shape(parent, rank, max_rank)
    res = []
    for b in range(B):
        ctx, y, node = 0, [], -1
        while True:
            P = list(softmax(draft[b, ctx] * 0 + target[b, ctx].astype(np.float64) / float(np.float32(T))))
            Q = list(softmax(draft[b, ctx].astype(np.float64) / float(np.float32(T))))
            kids = sorted((rank[n], n) for n in range(N) if valid[n] and parent[n] + 1 == ctx)
            took = None
            for r, n in kids:
                x = int(tokens[b, n])
                if x < 0:
                    continue
                w = mini_oracle.philox4x32((r, ctx, b, 2), (seed & 0xFFFFFFFF, seed >> 32), rounds)[0]
                if P[x] / Q[x] > (w + 0.5) / 4294967296.0:
                    took = n
                    break
                P = [max(p - q, 0.0) for p, q in zip(P, Q)]
                sp = sum(P)
                if sp > 0:
                    P = [p / sp for p in P]
                Q[x] = 0.0
                sq = sum(Q)
                if sq > 0:
                    Q = [q / sq for q in Q]
            if took is not None:
                y.append(int(tokens[b, took]))
                node, ctx = took, took + 1
                continue
            e = mini_oracle.exponentials(V, seed, ctx, b, 1, rounds)
            arrival = [e[i] / P[i] if P[i] > 0 else np.inf for i in range(V)]
            tok = int(np.argmin(arrival)) if np.isfinite(min(arrival)) else 0
            res.append((len(y), node, y + [tok]))
            break
    return res


def random_tree(rng, N, max_children=3):
    parent = np.full(N, -1, dtype=np.int32)
    rank = np.zeros(N, dtype=np.int32)
    count = {}
    for n in range(N):
        while True:
            p = int(rng.integers(-1, n)) if n else -1
            if count.get(p, 0) < max_children:
                break
        parent[n], rank[n] = p, count.get(p, 0)
        count[p] = count.get(p, 0) + 1
    return parent, rank


def test_chain_equals_the_sequence_oracle(oracle_mod):
    rng = np.random.default_rng(3)
    B, k, V = 6, 4, 300
    target = (2.0 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    draft = (target + 0.8 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    tok = oracle_mod.race_sample(draft[:, None, :k].copy(), 0, 0.9, 17)[:, 0]
    seq = oracle_mod.gsd_verify(draft[:, :k].copy(), target, tok, 0.9, 17)
    parent = np.arange(-1, k - 1, dtype=np.int32)
    rank = np.zeros(k, dtype=np.int32)
    tree = oracle_mod.gsd_verify_tree(draft, target, parent, rank, tok, 0.9, 17)
    assert np.array_equal(tree["accept_len"], seq["accept_len"])
    assert 0 < seq["accept_len"].mean() < k
    for b in range(B):
        a = int(seq["accept_len"][b])
        assert tree["emitted"][b, :a].tolist() == tok[b, :a].tolist()
        assert tree["emitted"][b, a] == seq["next_token"][b] and (tree["emitted"][b, a + 1:] == -1).all()
        assert tree["accept_node"][b] == a - 1


@pytest.mark.parametrize("trial", range(4))
def test_literal_restatement_token_for_token(oracle_mod, trial):
    rng = np.random.default_rng(100 + trial)
    B, N, V = 5, 7, 9
    target = (1.5 * rng.standard_normal((B, N + 1, V))).astype(np.float32)
    draft = (target + rng.standard_normal((B, N + 1, V))).astype(np.float32)
    parent, rank = random_tree(rng, N)
    if trial == 3:
        parent[4], rank[5] = 6, 9      # malformed nodes draft nothing and are never tested
    arr = oracle_mod.race_verify_arrival_tree(draft, target, parent, rank, 1.1, 40 + trial)
    tok = arr["draft_tokens"]
    o = oracle_mod.gsd_verify_tree(draft, target, parent, rank, tok, 1.1, 40 + trial)
    ref = literal(draft, target, parent, rank, tok, 1.1, 40 + trial, oracle_mod)
    for b, (n_acc, node, y) in enumerate(ref):
        assert o["accept_len"][b] == n_acc and o["accept_node"][b] == node
        assert o["emitted"][b, : len(y)].tolist() == y and (o["emitted"][b, len(y):] == -1).all()


def test_emitted_token_follows_the_target_law(oracle_mod):
    """Three alternatives at the root drawn from Q without replacement (the first arrivals of a race under Q), verified
    by recursive rejection: the first emitted token is distributed as P, whatever Q is (Algorithm 4's purpose)."""
    rng = np.random.default_rng(8)
    B, V, N = 30000, 6, 3
    lp, lq = rng.standard_normal(V) * 1.2, rng.standard_normal(V) * 1.2
    target = np.tile(lp.astype(np.float32), (B, N + 1, 1))
    draft = np.tile(lq.astype(np.float32), (B, N + 1, 1))
    parent = np.full(N, -1, dtype=np.int32)
    rank = np.arange(N, dtype=np.int32)
    tok = oracle_mod.race_verify_arrival_tree(draft, target, parent, rank, 1.0, 77)["draft_tokens"]
    o = oracle_mod.gsd_verify_tree(draft, target, parent, rank, tok, 1.0, 77)
    first = o["emitted"][:, 0]
    counts = np.bincount(first, minlength=V)
    p = softmax(lp.astype(np.float32).astype(np.float64))
    chi2, pval = stats.chisquare(counts, p * B)
    assert pval > 1e-3, (chi2, pval)
    # and more alternatives are accepted more often than one
    q = softmax(lq.astype(np.float32).astype(np.float64))
    single = 1.0 - 0.5 * np.abs(p - q).sum()       # acceptance probability of one alternative: 1 - D_TV (Section 3)
    rate = (o["accept_len"] >= 1).mean()
    assert rate > single + 0.02


def test_identical_models_accept_the_first_child_and_no_children_draws_from_the_target(oracle_mod):
    rng = np.random.default_rng(9)
    B, N, V = 8, 5, 50
    x = rng.standard_normal((B, N + 1, V)).astype(np.float32)
    parent = np.array([-1, -1, 0, 0, 2], dtype=np.int32)
    rank = np.array([0, 1, 0, 1, 0], dtype=np.int32)
    tok = oracle_mod.race_verify_arrival_tree(x, x, parent, rank, 1.0, 5)["draft_tokens"]
    o = oracle_mod.gsd_verify_tree(x, x, parent, rank, tok, 1.0, 5)
    assert (o["accept_len"] == 3).all() and (o["accept_node"] == 4).all()      # 0 -> 2 -> 4: always the first child
    # a missing arrival (-1) is passed over: with every token -1 nothing can be accepted
    none = oracle_mod.gsd_verify_tree(x, x, parent, rank, np.full_like(tok, -1), 1.0, 5)
    assert (none["accept_len"] == 0).all() and (none["accept_node"] == -1).all() and (none["emitted"][:, 1:] == -1).all()
    # that draw follows the target law: chi-square over many prompts with the same logits
    B2, V2 = 20000, 5
    l = rng.standard_normal(V2).astype(np.float32)
    t = np.tile(l, (B2, 2, 1))
    drawn = oracle_mod.gsd_verify_tree(t, t, np.array([-1], np.int32), np.array([0], np.int32),
                                       np.full((B2, 1), -1, np.int32), 0.8, 11)["emitted"][:, 0]
    p = softmax(l.astype(np.float64) / float(np.float32(0.8)))
    assert stats.chisquare(np.bincount(drawn, minlength=V2), p * B2)[1] > 1e-3
    with pytest.raises(ValueError):
        oracle_mod.gsd_verify_tree(x, x, parent, rank, np.full_like(tok, V), 1.0, 5)
