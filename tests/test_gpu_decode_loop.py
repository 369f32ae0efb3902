"""GPU, end to end: a speculative decoding loop built from the library's calls alone (Algorithm 2 extended to k drafted
tokens, Section 3) emits sequences that follow the TARGET model's law exactly, although every token but the last of a
round is proposed by a different draft model.  Both models are first-order Markov chains over a small vocabulary, so the
law of the first tokens is known in closed form.  The drafting step uses the one-model race (one position per call, as
a real drafting loop would), the verification the one-model race on the target rows plus the acceptance step; the
fused call must give the same tokens."""
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


def test_decoding_loop_keeps_the_target_chain(race):
    V, T, B, L, k = 5, 0.9, 60000, 3, 3
    rng = np.random.default_rng(2024)
    LP = torch.from_numpy((1.3 * rng.standard_normal((V, V))).astype(np.float32)).cuda()   # row = previous token
    LQ = LP + torch.from_numpy((0.9 * rng.standard_normal((V, V))).astype(np.float32)).cuda()
    last = torch.zeros(B, dtype=torch.long, device="cuda")          # every sequence starts after token 0
    out = torch.full((B, L + k + 1), -1, dtype=torch.long, device="cuda")
    n_out = torch.zeros(B, dtype=torch.long, device="cuda")
    rows = torch.arange(B, device="cuda")
    accepted_total, rounds = 0, 0
    print(f"[case] decoding loop V={V} B={B} k={k}", flush=True)
    while int(n_out.min()) < L:
        seed = 5000 + rounds                                        # a fresh set of races for every round
        # drafting: one position at a time, each from the draft model's row for the token before it
        prev, drafted = last, []
        for j in range(k):
            tok = race.race_sample(LQ[prev].reshape(B, 1, 1, V).contiguous(), j, T, seed)
            prev = tok.reshape(B).long()
            drafted.append(prev)
        d = torch.stack(drafted, dim=1)                             # [B, k]
        # verification: the target model's rows at the k drafted positions and the one after them
        ctx = torch.cat([last[:, None], d], dim=1)                  # token before each of the k + 1 positions
        target_logits = LP[ctx].contiguous()                        # [B, k + 1, V]
        t = race.race_sample(target_logits.reshape(B, 1, k + 1, V), 0, T, seed).reshape(B, k + 1)
        acc = race.accept_lengths(race.VARIANT_SEQUENCE, d.int().contiguous(), t.contiguous())
        fused = race.race_verify(LQ[ctx[:, :k]].contiguous(), target_logits, T, seed)
        assert torch.equal(fused[0].long(), d) and torch.equal(fused[1], t) and torch.equal(fused[2], acc)
        # emit the accepted drafted tokens and the target's token at the first disagreement (or the bonus token)
        a = acc.long()
        for j in range(k + 1):
            take = j <= a
            pos = n_out + j
            ok = take & (pos < out.shape[1])
            out[rows[ok], pos[ok]] = t[ok, j].long()
        n_out = n_out + a + 1
        last = t[rows, a].long()
        accepted_total += int(a.sum())
        rounds += 1
        assert rounds <= L
    torch.cuda.synchronize()
    seqs = out[:, :L].cpu().numpy()
    assert (seqs >= 0).all()
    # closed-form law of the first L tokens of the target chain started after token 0
    P = np.stack([theory.softmax(LP[v].cpu().numpy(), T) for v in range(V)])
    expect = np.zeros((V,) * L)
    for idx in np.ndindex(*expect.shape):
        p, prev = 1.0, 0
        for x in idx:
            p *= P[prev, x]
            prev = x
        expect[idx] = p * B
    counts = np.zeros((V,) * L)
    np.add.at(counts, tuple(seqs[:, i] for i in range(L)), 1)
    e, c = expect.ravel(), counts.ravel()
    order = np.argsort(e)
    e, c = e[order], c[order]
    small = np.cumsum(e) < 10.0                                      # merge the rarest cells into one
    if small.any():
        e = np.concatenate(([e[small].sum()], e[~small]))
        c = np.concatenate(([c[small].sum()], c[~small]))
    chi = stats.chisquare(c, e)
    per_round = accepted_total / (B * rounds)
    print(f"  {len(e)} cells, chi-square p-value {chi.pvalue:.3f}; accepted drafted tokens per round {per_round:.2f}", flush=True)
    assert chi.pvalue > 1e-4
    assert per_round > 0.5
