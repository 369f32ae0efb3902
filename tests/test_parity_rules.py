"""The comparison rules of tests/parity.py themselves, on the CPU: "GPU" results are the oracle's own with planted
deviations.  A near-tied row is built from two tokens with the same generator word whose logits differ by one unit
in the last place: their scores differ by 2e-6 in 50, inside the near-tie tolerance and not exactly equal."""
import numpy as np
import pytest
import torch

import parity
import ties

V = 256000


@pytest.fixture(scope="module")
def case(oracle_mod):
    rounds = oracle_mod.get_rounds()
    seed, pairs, _ = ties.find_context_with_pairs(V, rounds, min_pairs=1)    # race (0, 0, 0): sequence 0, position 0
    lo, hi = pairs[0]
    rng = np.random.default_rng(21)
    B, k = 2, 2
    target = rng.standard_normal((B, k + 1, V)).astype(np.float32)
    draft = (target[:, :k] + 0.3 * rng.standard_normal((B, k, V))).astype(np.float32)
    up = np.nextafter(np.float32(30.0), np.float32(31.0))
    target[0, 0, lo], target[0, 0, hi] = 30.0, up          # near-tied: hi wins by one ulp of logit
    draft[0, 0, lo], draft[0, 0, hi] = 10.0, 31.0          # the draft race picks hi clearly
    draft, target = torch.from_numpy(draft), torch.from_numpy(target)
    ora = oracle_mod.race_verify(draft, target, 1.0, seed, want_info=True)
    assert ora["target_info"]["near_tie"][0, 0] == 1 and ora["target_info"]["exact_tie"][0, 0] == 0
    assert ora["target_tokens"][0, 0] == hi and ora["draft_tokens"][0, 0] == hi and ora["accept_len"][0] >= 1
    assert ora["target_info"]["near_tie"].sum() == 1 and ora["draft_info"]["near_tie"].sum() == 0
    return seed, lo, hi, draft, target, ora


def _gpu_like(ora):
    return [ora["draft_tokens"].copy(), ora["target_tokens"].copy(), ora["accept_len"].copy()]


def test_identical_results_pass_with_no_exemption(oracle_mod, case):
    seed, lo, hi, draft, target, ora = case
    assert parity.check_sequence(_gpu_like(ora), ora, oracle_mod, draft, target, 1.0, seed) == 0


def test_other_candidate_of_a_near_tied_row_is_accepted_and_only_that_sequence_is_exempt(oracle_mod, case):
    seed, lo, hi, draft, target, ora = case
    gpu = _gpu_like(ora)
    gpu[1][0, 0] = lo                 # the other near-tied candidate
    gpu[2][0] = 0                     # and the accept length that follows from it
    assert parity.check_sequence(gpu, ora, oracle_mod, draft, target, 1.0, seed) == 1
    gpu[2][1] += 1                    # a wrong accept length in ANOTHER sequence is not covered by that exemption
    with pytest.raises(AssertionError):
        parity.check_sequence(gpu, ora, oracle_mod, draft, target, 1.0, seed)


def test_deviation_at_a_row_that_is_not_near_tied_fails(oracle_mod, case):
    seed, lo, hi, draft, target, ora = case
    gpu = _gpu_like(ora)
    gpu[1][1, 1] = (gpu[1][1, 1] + 1) % V
    with pytest.raises(AssertionError):
        parity.check_sequence(gpu, ora, oracle_mod, draft, target, 1.0, seed)


def test_token_outside_the_candidate_set_of_a_near_tied_row_fails(oracle_mod, case):
    seed, lo, hi, draft, target, ora = case
    gpu = _gpu_like(ora)
    gpu[1][0, 0] = 12345 if 12345 not in (lo, hi) else 12346
    gpu[2][0] = 0
    with pytest.raises(AssertionError):
        parity.check_sequence(gpu, ora, oracle_mod, draft, target, 1.0, seed)


def test_accept_length_must_follow_from_the_tokens(oracle_mod, case):
    seed, lo, hi, draft, target, ora = case
    gpu = _gpu_like(ora)
    gpu[2][1] = (gpu[2][1] + 1) % 3
    with pytest.raises(AssertionError):
        parity.check_sequence(gpu, ora, oracle_mod, draft, target, 1.0, seed)
