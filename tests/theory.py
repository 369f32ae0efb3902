"""Closed forms and brute-force estimates that the paper and elementary probability fix.

Written independently of oracle/ and of the GPU library (numpy only); used to pin the oracle.
"""
import numpy as np


def softmax(logits, T=1.0):
    z = np.asarray(logits, dtype=np.float64) / T
    z = z - z.max()
    e = np.exp(z)
    return e / e.sum()


def total_variation(p, q):
    """D_TV of Section 3."""
    return 0.5 * np.abs(np.asarray(p) - np.asarray(q)).sum()


def harmonic_mean_distance(p, q):
    """D_HM of Lemma 3.1: sum_i p_i q_i / (p_i + q_i)."""
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    return float((p * q / (p + q)).sum())


def coupling_probability(p, q):
    """Pr{ argmin e_i/p_i == argmin e_i/q_i } for iid e_i ~ Exp(1).

    Both races are won by i iff e_j >= e_i * max(p_j/p_i, q_j/q_i) for all j != i; with independent
    exponentials Pr = integral of exp(-e_i * sum_j max(...)) de_i = 1 / sum_j max(p_j/p_i, q_j/q_i)
    (the j = i term contributes 1).  Direct O(V^2) evaluation.
    """
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    total = 0.0
    for i in range(len(p)):
        total += 1.0 / np.maximum(p / p[i], q / q[i]).sum()
    return float(total)


def coupling_probability_sorted(p, q):
    """Same quantity in O(V log V): sort by r_j = p_j/q_j; for winner i the tokens with r_j >= r_i
    contribute p_j/p_i and the others q_j/q_i."""
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    order = np.argsort(p / q, kind="stable")
    ps, qs = p[order], q[order]
    r = ps / qs
    # for position a in sorted order: sum_{r_j >= r_a} p_j  and  sum_{r_j < r_a} q_j (ties go to the p side,
    # where p_j/p_i == q_j/q_i anyway)
    p_suffix = np.cumsum(ps[::-1])[::-1]
    q_prefix = np.concatenate(([0.0], np.cumsum(qs)[:-1]))
    first_ge = np.searchsorted(r, r, side="left")
    psum = p_suffix[first_ge]
    qsum = q_prefix[first_ge]
    return float((1.0 / (psum / ps + qsum / qs)).sum())


def coupling_monte_carlo(p, q, n, seed):
    """Brute force with numpy's own generator (unrelated to Philox): fraction of races with equal winners."""
    rng = np.random.default_rng(seed)
    p, q = np.asarray(p, dtype=np.float64), np.asarray(q, dtype=np.float64)
    same = 0
    done = 0
    while done < n:
        c = min(200000, n - done)
        e = rng.exponential(size=(c, len(p)))
        same += int((np.argmin(e / p, axis=1) == np.argmin(e / q, axis=1)).sum())
        done += c
    return same / n
