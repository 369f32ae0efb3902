"""GPU parity on seeded random shapes, value distributions, temperatures, seeds, splits and row strides: every case is
checked against the CPU oracle to the same bar as the fixed cases (bit-exact outside oracle-flagged near-ties)."""
import os

import numpy as np
import pytest
import torch

import parity

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def race():
    assert torch.cuda.is_available(), "GPU tests need the MI355X"
    from paper_2504_15475_amd import race as r
    r.lib()
    return r


@pytest.fixture(autouse=True)
def clean_env():
    parity.hooks.reset()
    yield
    parity.hooks.reset()


def logits(rng, shape, dtype, kind):
    """Host fp32 logits of a few characters: broad, narrow, peaked, coarse (many equal logits), heavily masked."""
    x = rng.standard_normal(shape).astype(np.float32)
    if kind == "broad":
        x *= 6.0
    elif kind == "narrow":
        x *= 0.05
    elif kind == "peaked":
        x *= 1.5
        hot = rng.random(shape) < 3.0 / shape[-1]
        x[hot] += 12.0
    elif kind == "coarse":
        x = np.round(x * 2.0) / 2.0 * 3.0
    elif kind == "masked":
        x *= 3.0
        x[rng.random(shape) < 0.97] = -np.inf
    elif kind == "shifted":
        x = x * 2.0 + 500.0
    t = torch.from_numpy(x)
    return t.to(dtype)


def widen(x, pad):
    if pad == 0:
        return x
    wide = torch.full(x.shape[:-1] + (x.shape[-1] + pad,), 3.0e4, dtype=x.dtype, device=x.device)
    wide[..., : x.shape[-1]] = x
    return wide[..., : x.shape[-1]]


KINDS = ["broad", "narrow", "peaked", "coarse", "masked", "shifted"]


def random_case(i):
    rng = np.random.default_rng(9000 + i)
    c = dict(i=i, rng=rng)
    c["variant"] = ["sequence", "multi", "tree", "arrival"][i % 4]
    c["dtype"] = [torch.bfloat16, torch.float32][int(rng.integers(2))]
    c["V"] = int(rng.choice([rng.integers(1, 64), rng.integers(64, 5000), rng.integers(5000, 40000)]))
    c["B"] = int(rng.integers(1, 5))
    c["k"] = int(rng.integers(1, 6))
    c["m"] = int(rng.integers(1, 4))
    c["T"] = float(rng.choice([0.3, 0.7, 1.0, 1.7]))
    c["seed"] = int(rng.integers(0, 2 ** 63))
    c["split"] = int(rng.choice([0, 0, 1, 2, 5, 37]))
    c["kernel"] = None if rng.random() < 0.8 else "exhaustive"
    c["kind"] = KINDS[int(rng.integers(len(KINDS)))]
    c["pads"] = (int(rng.choice([0, 0, 1, 8, 56])), int(rng.choice([0, 0, 3, 16])))
    return c


@pytest.mark.parametrize("i", range(int(os.environ.get("ERSD_RANDOM_CASES", "64"))))  # more for a soak run
def test_random_case(race, oracle_mod, i):
    c = random_case(i)
    rng, V, B, k, m, T, seed, dt = c["rng"], c["V"], c["B"], c["k"], c["m"], c["T"], c["seed"], c["dtype"]
    print("[case] random", {a: b for a, b in c.items() if a != "rng"}, flush=True)
    if c["split"]:
        parity.hooks.set(force_blocks=c["split"])
    if c["kernel"]:
        parity.hooks.set(exhaustive=c["kernel"] == "exhaustive")
    if c["variant"] == "sequence":
        t_host = logits(rng, (B, k + 1, V), dt, c["kind"])
        d_host = (t_host[:, :k].float() + torch.from_numpy(0.5 * rng.standard_normal((B, k, V)).astype(np.float32))).to(dt)
        gpu = race.race_verify(widen(d_host.cuda(), c["pads"][0]), widen(t_host.cuda(), c["pads"][1]), T, seed)
        torch.cuda.synchronize()
        ora = oracle_mod.race_verify(d_host, t_host, T, seed, want_info=True)
        parity.check_sequence(gpu, ora, oracle_mod, d_host, t_host, T, seed)
    elif c["variant"] == "multi":
        t_host = logits(rng, (B, m, k + 1, V), dt, c["kind"])
        d_host = (t_host[:, :, :k].float() + torch.from_numpy(0.5 * rng.standard_normal((B, m, k, V)).astype(np.float32))).to(dt)
        gpu = race.race_verify_multi(widen(d_host.cuda(), c["pads"][0]), widen(t_host.cuda(), c["pads"][1]), T, seed)
        torch.cuda.synchronize()
        ora = oracle_mod.race_verify_multi(d_host, t_host, T, seed, want_info=True)
        parity.check_sequence(gpu, ora, oracle_mod, d_host, t_host, T, seed, multi=True)
    else:
        N = int(rng.integers(1, 14))
        parent = np.array([int(rng.integers(-1, n)) for n in range(N)], dtype=np.int32)
        if c["variant"] == "tree":
            t_host = logits(rng, (B, N, V), dt, c["kind"])
            d_host = (t_host.float() + torch.from_numpy(0.5 * rng.standard_normal((B, N, V)).astype(np.float32))).to(dt)
            gpu = race.race_verify_tree(widen(d_host.cuda(), c["pads"][0]), widen(t_host.cuda(), c["pads"][1]),
                                        torch.from_numpy(parent).cuda(), T, seed)
            torch.cuda.synchronize()
            ora = oracle_mod.race_verify_tree(d_host, t_host, parent, T, seed, want_info=True)
            parity.check_tree(gpu, ora, oracle_mod, d_host, t_host, parent, T, seed)
        else:
            # ranks: siblings count up from 0 in node order (a few skipped, which leaves those arrivals unused)
            rank = np.zeros(N, dtype=np.int32)
            seen = {}
            for n in range(N):
                r = seen.get(int(parent[n]), 0)
                rank[n] = r if r < race.max_rank() else race.max_rank() - 1   # a duplicate rank: the node is invalid
                seen[int(parent[n])] = r + 1 + int(rng.random() < 0.15)
            t_host = logits(rng, (B, N + 1, V), dt, c["kind"])
            d_host = (t_host.float() + torch.from_numpy(0.5 * rng.standard_normal((B, N + 1, V)).astype(np.float32))).to(dt)
            gpu = race.race_verify_arrival_tree(widen(d_host.cuda(), c["pads"][0]), widen(t_host.cuda(), c["pads"][1]),
                                                torch.from_numpy(parent).cuda(), torch.from_numpy(rank).cuda(), T, seed)
            torch.cuda.synchronize()
            ora = oracle_mod.race_verify_arrival_tree(d_host, t_host, parent, rank, T, seed, max_rank=race.max_rank(),
                                                      want_info=True)
            parity.check_arrival_tree(gpu, ora, oracle_mod, t_host, parent, rank, T, seed, race.max_rank())
