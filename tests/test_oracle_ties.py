"""The lowest-index rule at finite exact ties (reading R6 of the race definition: exactly equal scores go to the
lowest token index).  Two tokens of one race whose generator words coincide and whose logits are equal have equal
scores; such pairs exist in every large vocabulary (tests/ties.py finds them)."""
import numpy as np
import pytest
import torch

import ties

V = 256000


@pytest.fixture(scope="module")
def tied(oracle_mod):
    rounds = oracle_mod.get_rounds()
    seed, pairs, words = ties.find_context_with_pairs(V, rounds, min_pairs=2)
    # the search's own generator against the oracle's, at the tokens that matter and a few others
    for i in [0, 1, 2, 3, V - 1] + [t for p in pairs for t in p]:
        got = oracle_mod.philox4x32((i >> 2, 0, 0, 0), (seed & 0xFFFFFFFF, seed >> 32), rounds)[i & 3]
        assert int(got) == int(words[i])
    return seed, pairs


def _row(pair, dtype, rng, top=30.0):
    row = rng.standard_normal(V).astype(np.float32)
    row[list(pair)] = top          # 30 is exact in bf16 and dominates every other score of the row
    t = torch.from_numpy(row)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_equal_words_and_logits_tie_exactly_and_the_lower_index_wins(oracle_mod, tied, dtype):
    seed, pairs = tied
    rng = np.random.default_rng(1)
    for lo, hi in pairs[:4]:
        assert lo < hi
        row = _row((lo, hi), dtype, rng)
        info = oracle_mod.race_rows(row, row, 1.0, seed, 0, 0, 0)
        for side in (0, 1):
            assert info[side]["token"] == lo and info[side]["runner_up"] == hi
            assert info[side]["exact_tie"] == 1
            assert info[side]["s1"] == info[side]["s2"] and np.isfinite(info[side]["s1"])
        cand, n = oracle_mod.row_candidates(row, 1.0, seed, 0, 0, 0)
        assert n == 2 and sorted(cand.tolist()) == [lo, hi]


def test_the_tie_is_broken_by_one_ulp_of_logit_in_either_direction(oracle_mod, tied):
    seed, pairs = tied
    lo, hi = pairs[0]
    rng = np.random.default_rng(2)
    base = _row((lo, hi), "f32", rng).numpy()
    up = np.nextafter(np.float32(30.0), np.float32(31.0))
    for winner, other in ((lo, hi), (hi, lo)):
        row = base.copy()
        row[winner] = up
        info = oracle_mod.race_rows(None, row, 1.0, seed, 0, 0, 0)[1]
        assert info["token"] == winner and info["runner_up"] == other and info["exact_tie"] == 0
        assert info["s1"] > info["s2"]


def test_a_tie_on_one_side_only_decides_acceptance(oracle_mod, tied):
    """Draft row tied, target row with the higher token alone on top (and the other way round): the race is shared,
    the rows are not, and the accept length follows from the tokens."""
    seed, pairs = tied
    lo, hi = pairs[1]
    rng = np.random.default_rng(3)
    tie_row = _row((lo, hi), "f32", rng)
    hi_row = tie_row.clone()
    hi_row[lo] = 0.0
    bonus = torch.from_numpy(rng.standard_normal(V).astype(np.float32))
    for draft_row, target_row, want in ((tie_row, hi_row, (lo, hi, 0)), (hi_row, tie_row, (hi, lo, 0)),
                                        (tie_row, tie_row, (lo, lo, 1))):
        o = oracle_mod.race_verify(draft_row[None, None], torch.stack([target_row, bonus])[None], 1.0, seed)
        assert (int(o["draft_tokens"][0, 0]), int(o["target_tokens"][0, 0]), int(o["accept_len"][0])) == want


def test_tied_tokens_are_consecutive_arrivals_in_index_order(oracle_mod, tied):
    """Algorithm 5: children are the first arrivals under the draft model; tokens with equal scores arrive in index
    order, wherever in the order the pair stands."""
    seed, pairs = tied
    lo, hi = pairs[2]
    rng = np.random.default_rng(4)
    third = 777 if 777 not in (lo, hi) else 778
    draft0 = _row((lo, hi), "f32", rng)
    draft0[third] = 45.0                              # arrives first; the pair are arrivals 1 and 2
    rows = [draft0] + [torch.from_numpy(rng.standard_normal(V).astype(np.float32)) for _ in range(3)]
    draft = torch.stack(rows)[None]                   # contexts 0..3
    target = torch.stack([torch.from_numpy(rng.standard_normal(V).astype(np.float32)) for _ in range(4)])[None]
    parent = np.array([-1, -1, -1], dtype=np.int32)
    rank = np.array([2, 0, 1], dtype=np.int32)        # node 0 drafts arrival 2, node 1 arrival 0, node 2 arrival 1
    o = oracle_mod.race_verify_arrival_tree(draft, target, parent, rank, 1.0, seed, want_info=True)
    assert o["draft_tokens"][0].tolist() == [hi, third, lo]
