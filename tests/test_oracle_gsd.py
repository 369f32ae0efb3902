"""Pins for the oracle of the comparison method (GSD, Section 2 / Algorithm 1 per position); no GPU."""
import numpy as np
import pytest
from scipy import stats
from scipy.special import logsumexp

import mini_oracle
import theory


def _draft_tokens(oracle_mod, draft, T, seed):
    """The drafting stage: a draw from Q per position (here by the one-model race, a Gumbel-max draw)."""
    return oracle_mod.race_sample(draft[:, None], 0, T, seed)[:, 0]


def test_normaliser_against_library_routine(oracle_mod):
    rng = np.random.default_rng(1)
    for T in (1.0, 0.6, 2.5):
        row = (5 * rng.standard_normal(777)).astype(np.float32)
        row[::50] = -np.inf
        assert oracle_mod.logsumexp(row, T) == pytest.approx(logsumexp(row.astype(np.float64) / np.float32(T)), rel=1e-13)
    assert oracle_mod.logsumexp(np.full(5, -np.inf, dtype=np.float32), 1.0) == -np.inf
    bf = (np.array([1.5, -2.0, 0.25], dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)
    assert oracle_mod.logsumexp(bf, 1.0) == pytest.approx(logsumexp([1.5, -2.0, 0.25]), rel=1e-14)


def test_acceptance_uniform_is_the_stated_counter_word(oracle_mod):
    for seed, j, b in ((0, 0, 0), (12345678901234, 3, 7)):
        w = mini_oracle.philox4x32((0, j, b, 2), (seed & 0xFFFFFFFF, seed >> 32), oracle_mod.get_rounds())[0]
        assert oracle_mod.gsd_uniform(seed, j, b) == (w + 0.5) / 2**32


def test_single_position_against_a_literal_restatement(oracle_mod):
    # Algorithm 1 in probabilities: accept iff P(x)/Q(x) > U, else draw from max(P - Q, 0) normalised, here by
    # the literal arrival times e_i / weight_i
    rng = np.random.default_rng(4)
    B, V, T = 200, 11, 0.8
    target = (1.5 * rng.standard_normal((B, 2, V))).astype(np.float32)
    draft = (target[:, :1] + rng.standard_normal((B, 1, V))).astype(np.float32)
    seed = 99
    tok = _draft_tokens(oracle_mod, draft, T, seed)
    o = oracle_mod.gsd_verify(draft, target, tok, T, seed)
    rounds = oracle_mod.get_rounds()
    n_rej = 0
    for b in range(B):
        p = theory.softmax(target[b, 0].astype(np.float64), np.float32(T))
        q = theory.softmax(draft[b, 0].astype(np.float64), np.float32(T))
        x = tok[b, 0]
        U = oracle_mod.gsd_uniform(seed, 0, b)
        if p[x] / q[x] > U:
            assert o["accept_len"][b] == 1
            e = mini_oracle.exponentials(V, seed, 1, b, 1, rounds)
            assert o["next_token"][b] == int(np.argmin(e / theory.softmax(target[b, 1].astype(np.float64), np.float32(T))))
        else:
            n_rej += 1
            assert o["accept_len"][b] == 0
            w = np.maximum(p - q, 0)
            e = mini_oracle.exponentials(V, seed, 0, b, 1, rounds)
            with np.errstate(divide="ignore"):
                assert o["next_token"][b] == int(np.argmin(np.where(w > 0, e / w, np.inf)))
    assert 20 < n_rej < 180


def test_acceptance_rate_is_one_minus_total_variation_and_output_follows_the_target(oracle_mod):
    # Section 3: GSD accepts the first drafted token with probability 1 - D_TV; Section 2: the emitted token
    # (the drafted one if accepted, the residual draw if not) is distributed as P
    V, B, T = 6, 60000, 1.0
    rng = np.random.default_rng(8)
    lp = (1.2 * rng.standard_normal(V)).astype(np.float32)
    lq = (lp + 0.9 * rng.standard_normal(V)).astype(np.float32)
    p, q = theory.softmax(lp.astype(np.float64)), theory.softmax(lq.astype(np.float64))
    target = np.broadcast_to(lp, (B, 2, V)).copy()
    draft = np.broadcast_to(lq, (B, 1, V)).copy()
    tok = _draft_tokens(oracle_mod, draft, T, 2718)
    o = oracle_mod.gsd_verify(draft, target, tok, T, 2718)
    acc = o["accept_len"] == 1
    a = 1 - theory.total_variation(p, q)
    assert abs(acc.mean() - a) < 5 * np.sqrt(a * (1 - a) / B)
    first = np.where(acc, tok[:, 0], o["next_token"])
    obs = np.bincount(first, minlength=V)
    assert float(((obs - B * p) ** 2 / (B * p)).sum()) < stats.chi2.ppf(1 - 1e-4, V - 1)
    # given a rejection, the draw follows the normalised residual
    res = np.maximum(p - q, 0)
    res = res / res.sum()
    rej = o["next_token"][~acc]
    obs = np.bincount(rej, minlength=V)
    keep = res > 0
    assert obs[~keep].sum() == 0
    n = len(rej)
    assert float(((obs[keep] - n * res[keep]) ** 2 / (n * res[keep])).sum()) < stats.chi2.ppf(1 - 1e-4, keep.sum() - 1)
    # after an acceptance the bonus token follows P at the next position
    obs = np.bincount(o["next_token"][acc], minlength=V)
    n = int(acc.sum())
    assert float(((obs - n * p) ** 2 / (n * p)).sum()) < stats.chi2.ppf(1 - 1e-4, V - 1)


def test_sequence_stops_at_the_first_rejection(oracle_mod):
    rng = np.random.default_rng(15)
    B, k, V, T = 300, 4, 20, 1.0
    target = (2 * rng.standard_normal((B, k + 1, V))).astype(np.float32)
    draft = (target[:, :k] + 0.8 * rng.standard_normal((B, k, V))).astype(np.float32)
    tok = _draft_tokens(oracle_mod, draft, T, 5)
    o = oracle_mod.gsd_verify(draft, target, tok, T, 5)
    for b in range(B):
        a = 0
        while a < k:
            p = theory.softmax(target[b, a].astype(np.float64))
            q = theory.softmax(draft[b, a].astype(np.float64))
            if not p[tok[b, a]] / q[tok[b, a]] > oracle_mod.gsd_uniform(5, a, b):
                break
            a += 1
        assert o["accept_len"][b] == a
    assert set(o["accept_len"].tolist()) == set(range(k + 1))
    # identical models accept every drafted token
    o2 = oracle_mod.gsd_verify(target[:, :k].copy(), target, tok, T, 5)
    assert np.all(o2["accept_len"] == k)
    # later positions do not matter once a token is rejected
    target2 = target.copy()
    for b in range(B):
        target2[b, o["accept_len"][b] + 1:] = 0
    o3 = oracle_mod.gsd_verify(draft, target2, tok, T, 5)
    assert np.array_equal(o3["accept_len"], o["accept_len"]) and np.array_equal(o3["next_token"], o["next_token"])


def test_sensitivity_flags(oracle_mod):
    # a residual with one clear winner has no rivals; two tokens with the same weight and nearly the same word do
    V = 8
    target = np.zeros((1, 2, V), dtype=np.float32)
    draft = np.zeros((1, 1, V), dtype=np.float32)
    target[0, 0, 3] = 6.0
    draft[0, 0, 5] = 3.0
    o = oracle_mod.gsd_verify(draft, target, np.array([[5]], dtype=np.int32), 1.0, 1, want_info=True)
    assert o["accept_len"][0] == 0 and o["next_token"][0] == 3 and o["info"]["rivals"][0] == 0
    assert o["info"]["lse_p"][0] == pytest.approx(np.log(7 + np.exp(6.0)), rel=1e-14)
    with pytest.raises(ValueError):
        oracle_mod.gsd_verify(draft, target, np.array([[V]], dtype=np.int32), 1.0, 1)
    # the report follows the tolerances it is given and the results never do: P(5)/Q(5) against its uniform
    gap = o["info"]["min_accept_gap"][0]
    assert 0 < gap < 1
    for tol, flag in ((0.0, 0), (gap * 0.99, 0), (gap * 1.01, 1), (1.0, 1)):
        o2 = oracle_mod.gsd_verify(draft, target, np.array([[5]], dtype=np.int32), 1.0, 1, want_info=True,
                                   accept_rel_tol=tol, weight_rel_tol=tol)
        assert o2["info"]["near_accept"][0] == flag
        assert o2["accept_len"][0] == o["accept_len"][0] and o2["next_token"][0] == o["next_token"][0]
    # with weights allowed to move by their own size every other token with positive mass is a rival
    o3 = oracle_mod.gsd_verify(draft, target, np.array([[5]], dtype=np.int32), 1.0, 1, want_info=True,
                               weight_rel_tol=1.0)
    assert o3["info"]["rivals"][0] >= 1
