"""GPU, no oracle involved: the library's own outputs obey what Section 3 proves.  The winner of a race under a model
follows that model's softmax (chi-square), the drafted and the target token coincide with the closed-form coupling
probability (which lies between the bounds of Lemma 3.1), and Algorithm 5's emitted token follows the target law
whatever the draft model is.  Many tiny rows in one call, which is also the shape with the most rows per workgroup."""
import numpy as np
import pytest
import torch
from scipy import stats

import theory

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def race():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2504_15475_amd import race as r
    r.lib()
    return r


@pytest.mark.parametrize("V,T,dtype", [(5, 1.0, torch.float32), (12, 0.6, torch.float32), (16, 1.3, torch.bfloat16)])
def test_winner_law_and_coupling_probability(race, V, T, dtype):
    rng = np.random.default_rng(100 + V)
    lt = torch.from_numpy((1.5 * rng.standard_normal(V)).astype(np.float32)).to(dtype)
    ld = (lt.float() + torch.from_numpy((0.8 * rng.standard_normal(V)).astype(np.float32))).to(dtype)
    p, q = theory.softmax(lt.float().numpy(), T), theory.softmax(ld.float().numpy(), T)
    B, k = 60000, 2
    draft = ld.cuda().expand(B, k, V).contiguous()
    target = lt.cuda().expand(B, k + 1, V).contiguous()
    print(f"[case] law V={V} T={T} {dtype} B={B}", flush=True)
    dtok, ttok, acc = race.race_verify(draft, target, T, 777)
    torch.cuda.synchronize()
    dtok, ttok, acc = dtok.cpu().numpy(), ttok.cpu().numpy(), acc.cpu().numpy()
    n = B * (k + 1)
    chi_p = stats.chisquare(np.bincount(ttok.ravel(), minlength=V), p * n)
    chi_q = stats.chisquare(np.bincount(dtok.ravel(), minlength=V), q * B * k)
    print(f"  chi-square p-values: target {chi_p.pvalue:.3f} draft {chi_q.pvalue:.3f}", flush=True)
    assert chi_p.pvalue > 1e-4 and chi_q.pvalue > 1e-4
    c = theory.coupling_probability(p, q)
    match = (dtok == ttok[:, :k]).mean()
    sd = np.sqrt(c * (1 - c) / (B * k))
    print(f"  match rate {match:.4f} against closed form {c:.4f} (sd {sd:.4f})", flush=True)
    assert abs(match - c) < 5 * sd
    assert theory.harmonic_mean_distance(p, q) - 1e-12 <= c <= 1 - theory.total_variation(p, q) + 1e-12
    # accept length: geometric in the per-position match probability, capped at k
    expect = sum(c ** j for j in range(1, k + 1))
    assert abs(acc.mean() - expect) < 5 * np.sqrt(k * k / B)


def test_algorithm5_emits_the_target_law(race):
    """Three alternatives at the root (the batch strategy): the first emitted token follows P exactly, although the
    alternatives come from a different model, and a drafted token is accepted more often than with one alternative."""
    V, T, B = 10, 1.0, 80000
    rng = np.random.default_rng(5)
    lt = torch.from_numpy((1.2 * rng.standard_normal(V)).astype(np.float32))
    ld = lt + torch.from_numpy((1.0 * rng.standard_normal(V)).astype(np.float32))
    p, q = theory.softmax(lt.numpy(), T), theory.softmax(ld.numpy(), T)
    parent = torch.tensor([-1, -1, -1], dtype=torch.int32).cuda()
    rank = torch.tensor([0, 1, 2], dtype=torch.int32).cuda()
    draft = ld.cuda().expand(B, 4, V).contiguous()
    target = lt.cuda().expand(B, 4, V).contiguous()
    print(f"[case] Algorithm 5 law V={V} B={B}", flush=True)
    dtok, ttok, acc, node, emitted = race.race_verify_arrival_tree(draft, target, parent, rank, T, 4242)
    torch.cuda.synchronize()
    first = emitted[:, 0].cpu().numpy()
    chi = stats.chisquare(np.bincount(first, minlength=V), p * B)
    print(f"  first emitted token: chi-square p-value {chi.pvalue:.3f}", flush=True)
    assert chi.pvalue > 1e-4
    d = dtok.cpu().numpy()
    assert (d[:, 0] != d[:, 1]).all() and (d[:, 1] != d[:, 2]).all() and (d[:, 0] != d[:, 2]).all()  # distinct arrivals
    chi_d = stats.chisquare(np.bincount(d[:, 0], minlength=V), q * B)
    assert chi_d.pvalue > 1e-4                                   # the first arrival follows Q
    rate3 = (acc.cpu().numpy() > 0).mean()
    c1 = theory.coupling_probability(p, q)
    print(f"  accepted with three alternatives {rate3:.4f}, closed form with one {c1:.4f}", flush=True)
    assert rate3 > c1 + 0.02
