"""Invariants and special cases of the oracle (no GPU): what must hold for any inputs."""
import numpy as np
import pytest

import mini_oracle


def _seq(rng, B, k, V, noise=0.6, scale=3.0):
    target = rng.normal(0, scale, size=(B, k + 1, V)).astype(np.float32)
    draft = (target[:, :k] + rng.normal(0, noise, size=(B, k, V))).astype(np.float32)
    return draft, target


def test_target_tokens_do_not_depend_on_draft_logits(oracle_mod):
    """Section 1: the output law is that of sampling from P alone -- the target winners are a target-only race."""
    rng = np.random.default_rng(0)
    draft, target = _seq(rng, 3, 5, 300)
    a = oracle_mod.race_verify(draft, target, 0.8, 5)
    other = rng.normal(0, 5, size=draft.shape).astype(np.float32)
    b = oracle_mod.race_verify(other, target, 0.8, 5)
    assert np.array_equal(a["target_tokens"], b["target_tokens"])
    # and each target token equals a one-sided race on that row
    for bi in range(3):
        for j in range(6):
            info = oracle_mod.race_rows(None, target[bi, j], 0.8, 5, c1=j, c2=bi, c3=0)
            assert info[1]["token"] == a["target_tokens"][bi, j]


def test_accept_len_is_the_run_of_leading_agreements(oracle_mod):
    rng = np.random.default_rng(1)
    draft, target = _seq(rng, 40, 6, 64, noise=0.4)
    o = oracle_mod.race_verify(draft, target, 1.0, 8)
    d, t, a = o["draft_tokens"], o["target_tokens"], o["accept_len"]
    assert ((0 <= a) & (a <= 6)).all()
    assert len(set(a.tolist())) > 2          # the case mix really has early and late rejections
    for b in range(40):
        assert (d[b, : a[b]] == t[b, : a[b]]).all()
        if a[b] < 6:
            assert d[b, a[b]] != t[b, a[b]]


def test_identical_models_accept_everything(oracle_mod):
    rng = np.random.default_rng(2)
    _, target = _seq(rng, 4, 7, 500)
    o = oracle_mod.race_verify(target[:, :7].copy(), target, 1.0, 3)
    assert (o["accept_len"] == 7).all()
    assert np.array_equal(o["draft_tokens"], o["target_tokens"][:, :7])


def test_single_token_vocabulary_and_masked_rows(oracle_mod):
    one = np.zeros((2, 3, 1), dtype=np.float32)
    o = oracle_mod.race_verify(one[:, :2].copy(), one, 1.0, 0)
    assert (o["target_tokens"] == 0).all() and (o["accept_len"] == 2).all()
    ninf = np.full((1, 3, 37), -np.inf, dtype=np.float32)
    o = oracle_mod.race_verify(ninf[:, :2].copy(), ninf, 1.0, 0, want_info=True)
    assert (o["target_tokens"] == 0).all() and (o["draft_tokens"] == 0).all()
    assert (o["target_info"]["exact_tie"] == 1).all()
    # a masked token never wins
    rng = np.random.default_rng(3)
    draft, target = _seq(rng, 2, 3, 50)
    masked = rng.random(50) < 0.7
    masked[7] = False
    target[..., masked] = -np.inf
    draft[..., masked] = -np.inf
    o = oracle_mod.race_verify(draft, target, 1.0, 4)
    assert not masked[o["target_tokens"]].any() and not masked[o["draft_tokens"]].any()


def test_exact_ties_go_to_the_lowest_index(oracle_mod):
    # -inf everywhere except two equal +huge logits at positions whose exponentials differ: no tie;
    # a genuine exact tie needs equal (logit, word): all -inf rows are the reachable case, covered above.
    # Here: the winner must be the first index attaining the maximum score reported in s1.
    rng = np.random.default_rng(4)
    draft, target = _seq(rng, 1, 1, 200)
    info = oracle_mod.race_rows(draft[0, 0], target[0, 0], 1.0, 9, 0, 0, 0)
    for s, row in ((0, draft[0, 0]), (1, target[0, 0])):
        e = mini_oracle.exponentials(200, 9, 0, 0, 0, rounds=oracle_mod.get_rounds())
        scores = row.astype(np.float64) - np.log(e)
        assert info[s]["token"] == int(np.argmax(scores))
        assert info[s]["s1"] == pytest.approx(scores.max(), rel=1e-14)
        second = np.partition(scores, -2)[-2]
        assert info[s]["s2"] == pytest.approx(second, rel=1e-14)
        assert info[s]["runner_up"] == int(np.argsort(-scores, kind="stable")[1])


def test_shift_and_power_of_two_scaling_leave_tokens_unchanged(oracle_mod):
    rng = np.random.default_rng(5)
    draft, target = _seq(rng, 3, 4, 400)
    base = oracle_mod.race_verify(draft, target, 1.0, 6, want_info=True)
    assert base["target_info"]["near_tie"].sum() == 0 and base["draft_info"]["near_tie"].sum() == 0
    # softmax is shift invariant (the race needs no normaliser): add a constant per row
    shifted = oracle_mod.race_verify(draft + np.float32(2.0), target + np.float32(-4.0), 1.0, 6)
    # (l, T) -> (2l, 2T) is exact in binary floating point
    scaled = oracle_mod.race_verify(draft * np.float32(2), target * np.float32(2), 2.0, 6)
    for other in (shifted, scaled):
        for key in ("draft_tokens", "target_tokens", "accept_len"):
            assert np.array_equal(base[key], other[key])


def test_temperature_changes_the_law_not_the_noise(oracle_mod):
    rng = np.random.default_rng(6)
    _, target = _seq(rng, 1, 1, 64)
    cold = oracle_mod.race_rows(None, target[0, 0], 1e-3, 1)[1]["token"]
    assert cold == int(np.argmax(target[0, 0]))      # T -> 0 approaches greedy


def test_multi_with_one_draft_equals_sequence_and_best_draft_rule(oracle_mod):
    rng = np.random.default_rng(7)
    draft, target = _seq(rng, 3, 4, 128)
    seq = oracle_mod.race_verify(draft, target, 1.0, 21)
    mul = oracle_mod.race_verify_multi(draft[:, None].copy(), target[:, None].copy(), 1.0, 21)
    assert np.array_equal(mul["draft_tokens"][:, 0], seq["draft_tokens"])
    assert np.array_equal(mul["target_tokens"][:, 0], seq["target_tokens"])
    assert np.array_equal(mul["accept_len"][:, 0], seq["accept_len"])
    assert np.array_equal(mul["best_len"], seq["accept_len"]) and (mul["best_draft"] == 0).all()
    # m drafts: each (b, d) is an independent race keyed by the draft index; draft 0 is the sequence result
    B, m, k, V = 5, 6, 3, 40
    t = rng.normal(0, 2, size=(B, m, k + 1, V)).astype(np.float32)
    d = (t[:, :, :k] + rng.normal(0, 0.5, size=(B, m, k, V))).astype(np.float32)
    o = oracle_mod.race_verify_multi(d, t, 1.0, 33)
    first = oracle_mod.race_verify(d[:, 0].copy(), t[:, 0].copy(), 1.0, 33)
    assert np.array_equal(o["accept_len"][:, 0], first["accept_len"])
    for b in range(B):
        assert o["best_len"][b] == o["accept_len"][b].max()
        assert o["best_draft"][b] == int(np.argmax(o["accept_len"][b]))       # lowest draft index on ties
    # identical logits in two drafts still race with different exponentials
    t2 = np.repeat(t[:, :1], 2, axis=1).copy()
    d2 = np.repeat(d[:, :1], 2, axis=1).copy()
    o2 = oracle_mod.race_verify_multi(d2, t2, 1.0, 33)
    assert not np.array_equal(o2["target_tokens"][:, 0], o2["target_tokens"][:, 1])


def test_chain_tree_equals_sequence_without_bonus(oracle_mod):
    rng = np.random.default_rng(8)
    B, N, V = 6, 5, 90
    target = rng.normal(0, 2.5, size=(B, N, V)).astype(np.float32)
    draft = (target + rng.normal(0, 0.4, size=(B, N, V))).astype(np.float32)
    parent = np.arange(-1, N - 1, dtype=np.int32)
    tree = oracle_mod.race_verify_tree(draft, target, parent, 1.0, 17)
    bonus = rng.normal(size=(B, 1, V)).astype(np.float32)
    seq = oracle_mod.race_verify(draft, np.concatenate([target, bonus], axis=1), 1.0, 17)
    assert np.array_equal(tree["draft_tokens"], seq["draft_tokens"])
    assert np.array_equal(tree["target_tokens"], seq["target_tokens"][:, :N])
    assert np.array_equal(tree["accept_len"], seq["accept_len"])
    assert np.array_equal(tree["accept_node"], seq["accept_len"] - 1)


def test_tree_walk_against_path_enumeration(oracle_mod):
    rng = np.random.default_rng(9)
    B, N, V = 30, 14, 12          # tiny vocabulary with close models: many agreements
    for trial in range(5):
        parent = np.array([-1 if n < 2 else int(rng.integers(-1 if n < 4 else 0, n)) for n in range(N)],
                          dtype=np.int32)
        target = rng.normal(0, 3.0, size=(B, N, V)).astype(np.float32)
        draft = (target + rng.normal(0, 1.5, size=(B, N, V))).astype(np.float32)
        o = oracle_mod.race_verify_tree(draft, target, parent, 1.0, 100 + trial)
        lens = []
        for b in range(B):
            L, node = mini_oracle.tree_accept(o["draft_tokens"][b], o["target_tokens"][b], parent)
            assert (o["accept_len"][b], o["accept_node"][b]) == (L, node)
            lens.append(L)
            # ancestor-closed: every ancestor of the accepted node agrees (Section 4)
            cur = o["accept_node"][b]
            while cur != -1:
                assert o["draft_tokens"][b, cur] == o["target_tokens"][b, cur]
                cur = parent[cur]
        assert max(lens) >= 2 and min(lens) < max(lens)
    # per-node races use the node index as counter word: node n of sequence b == sequence position n
    info = oracle_mod.race_rows(draft[3, 5], target[3, 5], 1.0, 100 + trial, c1=5, c2=3, c3=0)
    assert info[0]["token"] == o["draft_tokens"][3, 5] and info[1]["token"] == o["target_tokens"][3, 5]


def test_malformed_parent_entries_reject_the_node(oracle_mod):
    rng = np.random.default_rng(10)
    B, N, V = 4, 4, 6
    target = rng.normal(0, 3, size=(B, N, V)).astype(np.float32)
    parent = np.array([-1, 0, 5, 2], dtype=np.int32)      # node 2 points forward: nodes 2 and 3 can never be accepted
    o = oracle_mod.race_verify_tree(target.copy(), target, parent, 1.0, 1)
    assert (o["accept_len"] == 2).all() and (o["accept_node"] == 1).all()
    parent = np.array([-7, -1, 1, 2], dtype=np.int32)
    o = oracle_mod.race_verify_tree(target.copy(), target, parent, 1.0, 1)
    assert (o["accept_len"] == 3).all() and (o["accept_node"] == 3).all()


def test_near_tie_flags_and_candidate_sets(oracle_mod):
    V = 64
    row = np.zeros(V, dtype=np.float32)
    e = mini_oracle.exponentials(V, 55, 0, 0, 0, rounds=oracle_mod.get_rounds())
    g = -np.log(e)
    order = np.argsort(-g)
    a, b = int(order[0]), int(order[1])
    # raise the runner-up's logit so that it lands within 1e-7 (relative) of the winner, in fp32 steps
    gap = g[a] - g[b]
    row[b] = np.float32(gap)
    info = oracle_mod.race_rows(None, row, 1.0, 55)[1]
    resid = abs((row[b] + g[b]) - g[a])
    if resid <= 1e-6 * max(1.0, abs(g[a])) and resid > 0:
        assert info["near_tie"] == 1 and info["exact_tie"] == 0
        cand, n = oracle_mod.row_candidates(row, 1.0, 55)
        assert n == 2 and sorted(cand.tolist()) == sorted([a, b])
    row[b] = 0.0
    info = oracle_mod.race_rows(None, row, 1.0, 55)[1]
    assert info["near_tie"] == 0 and info["token"] == a and info["runner_up"] == b
    cand, n = oracle_mod.row_candidates(row, 1.0, 55)
    assert n == 1 and cand[0] == a


def test_invalid_arguments_are_rejected(oracle_mod):
    d = np.zeros((1, 2, 8), dtype=np.float32)
    t = np.zeros((1, 3, 8), dtype=np.float32)
    for T in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(ValueError):
            oracle_mod.race_verify(d, t, T, 0)


def test_seed_and_counter_words_select_independent_races(oracle_mod):
    rng = np.random.default_rng(12)
    row = rng.normal(0, 1, size=256).astype(np.float32)
    toks = {(s, c1, c2, c3): int(oracle_mod.race_rows(None, row, 1.0, s, c1, c2, c3)[1]["token"])
            for s in (0, 1, 2**32, 2**63 + 5) for c1 in (0, 1) for c2 in (0, 1) for c3 in (0, 1)}
    assert len(set(toks.values())) > 20           # 32 contexts, nearly all distinct winners on a flat-ish row
    # high and low seed words both matter
    assert toks[(0, 0, 0, 0)] != toks[(2**32, 0, 0, 0)] or toks[(0, 1, 0, 0)] != toks[(2**32, 1, 0, 0)]


def test_one_model_races_reproduce_the_two_model_race(oracle_mod):
    """Algorithm 2 runs the draft race before the target model is evaluated and the target race after it, on the
    same exponentials: racing each model's rows separately must give the fused result, also position by position."""
    rng = np.random.default_rng(13)
    B, m, k, V = 3, 2, 4, 200
    t = rng.normal(0, 2.5, size=(B, m, k + 1, V)).astype(np.float32)
    d = (t[:, :, :k] + rng.normal(0, 0.6, size=(B, m, k, V))).astype(np.float32)
    fused = oracle_mod.race_verify_multi(d, t, 0.9, 31)
    assert np.array_equal(oracle_mod.race_sample(d, 0, 0.9, 31), fused["draft_tokens"])
    assert np.array_equal(oracle_mod.race_sample(t, 0, 0.9, 31), fused["target_tokens"])
    for j in range(k):      # a drafting loop: one position per call
        step = oracle_mod.race_sample(np.ascontiguousarray(d[:, :, j:j + 1]), j, 0.9, 31)
        assert np.array_equal(step[:, :, 0], fused["draft_tokens"][:, :, j])
    # and against the independent pure-Python statement
    e = mini_oracle.exponentials(V, 31, 2, 1, 1, rounds=oracle_mod.get_rounds())
    assert fused["target_tokens"][1, 1, 2] == mini_oracle.race_winner(t[1, 1, 2].astype(np.float64), 0.9, e)
    with pytest.raises(ValueError):
        oracle_mod.race_sample(d, -1, 0.9, 31)
