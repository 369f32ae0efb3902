"""GPU parity at finite exact ties: two tokens of one race with the same generator word and the same dominant
logit.  Every level of the library's reduction is made to decide such a tie: inside one row segment (the
candidate list and its hand-over), across two segments of a row (the finishing kernel's merge), on the draft and
on the target side, with the streaming filter and with the exhaustive scoring path, and as consecutive arrivals of
an arrival tree."""
import numpy as np
import pytest
import torch

import parity
import ties

pytestmark = pytest.mark.gpu

V = 256000


@pytest.fixture(scope="module")
def race():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2504_15475_amd import race as r
    r.lib()
    return r


@pytest.fixture(autouse=True)
def clean_hooks():
    parity.hooks.reset()
    yield
    parity.hooks.reset()


@pytest.fixture(scope="module")
def tied(oracle_mod, race):
    assert race.philox_rounds() == oracle_mod.get_rounds()
    seed, pairs, _ = ties.find_context_with_pairs(V, race.philox_rounds(), min_pairs=3)
    return seed, pairs


def _rows(n, pair, dtype, rng, top=30.0):
    """n rows of small noise [n, V]; row 0 holds the tied pair on top."""
    x = torch.from_numpy(rng.standard_normal((n, V)).astype(np.float32))
    if pair is not None:
        x[0, list(pair)] = top
    return x.to(dtype)


def _block_of(race, token, blocks, code):
    """Share that holds token `token` of row 0 when a B=1, k=1 job of this vocabulary is cut for `blocks` workgroups."""
    d = race.plan_describe(race.VARIANT_SEQUENCE, 1, 1, 1, V, blocks, code)
    return int(np.searchsorted(d["block_start"].astype(np.int64), token // 8, side="right") - 1)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("side", ["draft", "target", "both"])
@pytest.mark.parametrize("kernel", ["filtered", "exhaustive"])
def test_tied_pair_in_one_segment_and_in_two(race, oracle_mod, tied, dtype, side, kernel):
    seed, pairs = tied
    code = race.ERSD_F32 if dtype == torch.float32 else race.ERSD_BF16
    rng = np.random.default_rng(11)
    for lo, hi in pairs[:3]:
        # a split that keeps the pair in one share, and one that separates it
        together = [g for g in (1, 2, 3) if _block_of(race, lo, g, code) == _block_of(race, hi, g, code)]
        apart = [g for g in range(2, 40) if _block_of(race, lo, g, code) != _block_of(race, hi, g, code)]
        assert together and apart
        draft = _rows(1, (lo, hi) if side in ("draft", "both") else None, dtype, rng)[None].cuda()
        target = _rows(2, (lo, hi) if side in ("target", "both") else None, dtype, rng)[None].cuda()
        ora = oracle_mod.race_verify(draft.cpu(), target.cpu(), 1.0, seed, want_info=True)
        if side in ("draft", "both"):
            assert ora["draft_info"]["exact_tie"][0, 0] == 1 and ora["draft_tokens"][0, 0] == lo
        if side in ("target", "both"):
            assert ora["target_info"]["exact_tie"][0, 0] == 1 and ora["target_tokens"][0, 0] == lo
        for split in (together[0], apart[0], apart[-1]):
            print(f"[case] pair ({lo},{hi}) {side} {kernel} split={split}", flush=True)
            parity.hooks.set(force_blocks=split, exhaustive=kernel == "exhaustive")
            gpu = race.race_verify(draft, target, 1.0, seed)
            torch.cuda.synchronize()
            # exact ties are not near-ties to be exempted: everything must be equal
            for got, key in zip(gpu, ("draft_tokens", "target_tokens", "accept_len")):
                assert np.array_equal(got.cpu().numpy(), ora[key]), (key, split)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
def test_tied_pair_in_the_one_model_race(race, oracle_mod, tied, dtype):
    seed, pairs = tied
    rng = np.random.default_rng(12)
    lo, hi = pairs[0]
    x = _rows(3, (lo, hi), dtype, rng)[None, None].cuda()       # [1, 1, 3, V]
    want = oracle_mod.race_sample(x.cpu(), 0, 1.0, seed)
    assert want[0, 0, 0] == lo
    for split in (1, 7, 23):
        parity.hooks.set(force_blocks=split)
        got = race.race_sample(x, 0, 1.0, seed)
        assert np.array_equal(got.cpu().numpy(), want), split


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16], ids=["f32", "bf16"])
@pytest.mark.parametrize("kernel", ["filtered", "exhaustive"])
def test_tied_pair_as_consecutive_arrivals(race, oracle_mod, tied, dtype, kernel):
    """Algorithm 5: the pair as arrivals r and r + 1 of the root context's race, r = 0 and r = 1."""
    seed, pairs = tied
    rng = np.random.default_rng(13)
    lo, hi = pairs[1]
    third = 4242
    for lead in (False, True):            # without / with a token that arrives before the pair
        d0 = _rows(4, (lo, hi), dtype, rng)
        if lead:
            d0[0, third] = 45.0
        draft = d0[None].cuda()
        target = _rows(4, None, dtype, rng)[None].cuda()
        parent = torch.tensor([-1, -1, -1], dtype=torch.int32, device="cuda")
        rank = torch.tensor([2, 0, 1], dtype=torch.int32, device="cuda")
        ora = oracle_mod.race_verify_arrival_tree(draft.cpu(), target.cpu(), parent.cpu().numpy(), rank.cpu().numpy(),
                                                  1.0, seed, max_rank=race.max_rank(), want_info=True)
        if lead:
            assert ora["draft_tokens"][0].tolist() == [hi, third, lo]
        else:
            assert ora["draft_tokens"][0].tolist()[1:] == [lo, hi]
        for split in (1, 5, 31):
            parity.hooks.set(force_blocks=split, exhaustive=kernel == "exhaustive")
            gpu = race.race_verify_arrival_tree(draft, target, parent, rank, 1.0, seed)
            torch.cuda.synchronize()
            for got, key in zip(gpu, ("draft_tokens", "target_tokens", "accept_len", "accept_node", "emitted")):
                assert np.array_equal(got.cpu().numpy(), ora[key]), (key, split, lead)
