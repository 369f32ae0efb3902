"""GPU parity of the comparison method (GSD) against its CPU oracle, through the C ABI."""
import numpy as np
import pytest
import torch

from paper_2504_15475_amd import workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def race():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2504_15475_amd import race as r
    r.lib()
    return r


# What the library's single-precision normalisers can move, stated here and handed to the oracle's sensitivity
# report (the oracle itself decides in double precision with no tolerance).  A normaliser is a sum of V terms
# 2^(z - max) kept per lane in fp32 and merged: with V = 131072 and 256 lanes a lane adds 512 terms, each addition
# rounding by at most 2^-24 relative, so a normaliser is off by at most 512 * 6e-8 = 3e-5 and typically by
# sqrt(512) * 6e-8 = 1.4e-6.  The acceptance ratio divides two of them; a weight p - q inherits the error of each
# scaled by p + q.
ACCEPT_REL_TOL = 1e-5     # |P(x)/Q(x) - U| relative: closer than this the accept decision is not compared
WEIGHT_REL_TOL = 4e-6     # weights moved by this times (p + q): a token another could overtake is not compared


def check(race, oracle_mod, draft, target, T, seed, note=""):
    """Bit-exact accept lengths and next tokens, except where the oracle's sensitivity report says normalisers off
    by the tolerances above can decide differently: an acceptance ratio that close to its uniform (the sequence is
    skipped), or rivals within reach of the final race's winner (the token is not compared)."""
    B, k, V = draft.shape
    print(f"[case] gsd B={B} k={k} V={V} {draft.dtype} T={T} seed={seed} {note}", flush=True)
    tok = race.race_sample(draft.unsqueeze(1).contiguous(), 0, T, seed)[:, 0].contiguous()  # the drafting stage
    acc, nxt = race.gsd_verify(draft, target, tok, T, seed)
    torch.cuda.synchronize()
    o = oracle_mod.gsd_verify(draft.cpu(), target.cpu(), tok.cpu().numpy(), T, seed, want_info=True,
                              accept_rel_tol=ACCEPT_REL_TOL, weight_rel_tol=WEIGHT_REL_TOL)
    acc, nxt = acc.cpu().numpy(), nxt.cpu().numpy()
    skipped = loose = 0
    for b in range(B):
        if o["info"]["near_accept"][b]:
            skipped += 1
            continue
        assert acc[b] == o["accept_len"][b], f"sequence {b}: accept_len {acc[b]} != {o['accept_len'][b]}"
        if o["info"]["rivals"][b] > 0:
            loose += 1
            continue
        assert nxt[b] == o["next_token"][b], f"sequence {b}: next_token {nxt[b]} != {o['next_token'][b]}"
    print(f"[case] ok: skipped {skipped}, tokens with rivals {loose}, mean accepted {o['accept_len'].mean():.2f}",
          flush=True)
    assert skipped + loose <= max(1, B // 50)      # (none is flagged in the committed cases)
    return o


def inputs(B, k, V, dtype, seed, noise=0.6):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    target = 3.0 * torch.randn((B, k + 1, V), generator=g, device="cuda")
    draft = target[:, :k] + noise * torch.randn((B, k, V), generator=g, device="cuda")
    return draft.to(dtype).contiguous(), target.to(dtype).contiguous()


@pytest.mark.parametrize("shape", [(5, 3, 1000, torch.float32), (4, 2, 4099, torch.bfloat16), (3, 4, 40960, torch.bfloat16),
                                   (2, 1, 70001, torch.float32), (70, 2, 8, torch.float32), (1, 6, 131072, torch.bfloat16)],
                         ids=lambda s: f"B{s[0]}-k{s[1]}-V{s[2]}-{str(s[3])[6:]}")
@pytest.mark.parametrize("T", [1.0, 0.7])
def test_small_shapes_match_oracle(race, oracle_mod, shape, T):
    B, k, V, dtype = shape
    draft, target = inputs(B, k, V, dtype, 31)
    o = check(race, oracle_mod, draft, target, T, 77)
    if B >= 4 and V >= 1000:
        assert o["accept_len"].min() < k or o["accept_len"].max() > 0


def test_identical_models_masked_tokens_and_invalid_drafts(race, oracle_mod):
    B, k, V = 6, 3, 4096
    draft, target = inputs(B, k, V, torch.float32, 9, noise=0.0)
    o = check(race, oracle_mod, draft, target, 1.0, 3, note="identical models")
    assert np.all(o["accept_len"] == k)
    draft, target = inputs(B, k, V, torch.float32, 10, noise=1.0)
    draft[:, :, ::3] = -float("inf")
    target[:, :, 1::5] = -float("inf")
    check(race, oracle_mod, draft, target, 1.0, 4, note="masked tokens")
    tok = torch.full((B, k), -1, dtype=torch.int32, device="cuda")
    tok[:, 0] = 5
    tok[0, 0] = V  # out of range at the first position
    acc, nxt = race.gsd_verify(draft, target, tok, 1.0, 4)
    torch.cuda.synchronize()
    assert acc[0].item() == 0 and int(acc.max()) <= 1 and int(nxt.min()) >= 0 and int(nxt.max()) < V


def test_peaked_rows_where_the_residual_cancels(race, oracle_mod):
    # nearly equal models: p - q is a small difference of large terms almost everywhere
    B, k, V = 16, 2, 32768
    draft, target = inputs(B, k, V, torch.float32, 12, noise=0.01)
    check(race, oracle_mod, draft, target, 1.0, 8, note="nearly equal models")


@pytest.mark.parametrize("idx", [1, 2])
def test_full_size_sequence_workloads(race, oracle_mod, idx):
    w = wl.WORKLOADS[idx]
    if idx == 2:
        w = wl.shrink(w, B=64)  # the oracle's two passes per row in double precision: keep the CPU side to seconds
    x = wl.make_inputs(w, "cuda")
    check(race, oracle_mod, x["draft"], x["target"], w.temperature, w.seed, note=w.name)
