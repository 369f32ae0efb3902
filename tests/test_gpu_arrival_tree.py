"""GPU parity of the Algorithm 5 tree form (children = first arrivals of one race) against the CPU oracle."""
import os

import numpy as np
import pytest
import torch

import parity
from paper_2504_15475_amd import workloads as wl

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


def run(race, oracle_mod, draft, target, parent, rank, T, seed, split=0, kernel=None, note=""):
    print(f"[case] arrival tree B={draft.shape[0]} N={len(parent)} V={draft.shape[2]} {draft.dtype} T={T} seed={seed} "
          f"split={split} kernel={kernel} {note}", flush=True)
    if split:
        parity.hooks.set(force_blocks=split)
    if kernel:
        parity.hooks.set(exhaustive=kernel == "exhaustive")
    par_d = torch.as_tensor(np.asarray(parent, dtype=np.int32)).cuda()
    rk_d = torch.as_tensor(np.asarray(rank, dtype=np.int32)).cuda()
    gpu = race.race_verify_arrival_tree(draft, target, par_d, rk_d, T, seed)
    # the same through a tree shape prepared ahead of time: identical outputs
    plan = race.arrival_tree_prepare(par_d, rk_d)
    again = race.race_verify_arrival_tree(draft, target, par_d, rk_d, T, seed, plan=plan)
    torch.cuda.synchronize()
    for a, b in zip(gpu, again):
        assert torch.equal(a, b)
    parity.hooks.set(force_blocks=0)
    parity.hooks.set(exhaustive=False)
    d_host, t_host = draft.cpu(), target.cpu()
    ora = oracle_mod.race_verify_arrival_tree(d_host, t_host, parent, rank, T, seed, max_rank=race.max_rank(),
                                              want_info=True)
    ex = parity.check_arrival_tree(gpu, ora, oracle_mod, t_host, parent, rank, T, seed, race.max_rank())
    print(f"[case] ok: near-tied contexts {int(ora['arrival_near_tie'].sum())}, exempted {ex}, "
          f"mean accepted {float(ora['accept_len'].mean()):.2f}", flush=True)
    return gpu, ora, ex


def small_inputs(B, N, V, dtype, seed, noise=0.6):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    target = 3.0 * torch.randn((B, N + 1, V), generator=g, device="cuda")
    draft = target + noise * torch.randn((B, N + 1, V), generator=g, device="cuda")
    return draft.to(dtype).contiguous(), target.to(dtype).contiguous()


TREES = {
    "chain": ([-1, 0, 1, 2], [0, 0, 0, 0]),
    "batch8": ([-1] * 8, list(range(8))),
    "mixed": ([-1, -1, -1, 0, 0, 1, 3, 3, 3, 6], [0, 1, 2, 0, 1, 0, 0, 1, 2, 0]),
    "gaps": ([-1, -1, 0, 0, 2], [0, 3, 7, 2, 1]),
}


@pytest.mark.parametrize("tree", list(TREES), ids=list(TREES))
@pytest.mark.parametrize("shape", [(3, 1000, torch.float32), (2, 4099, torch.bfloat16), (2, 40960, torch.bfloat16),
                                   (1, 70001, torch.float32)], ids=lambda s: f"B{s[0]}-V{s[1]}-{str(s[2])[6:]}")
@pytest.mark.parametrize("kernel", ["exhaustive", None], ids=["exhaustive", "filtered"])
@pytest.mark.parametrize("split", [0, 2, 37])
def test_small_trees_match_oracle(race, oracle_mod, tree, shape, kernel, split):
    parent, rank = TREES[tree]
    B, V, dtype = shape
    draft, target = small_inputs(B, len(parent), V, dtype, 17)
    run(race, oracle_mod, draft, target, parent, rank, 0.9, 123, split, kernel)


def test_chain_equals_the_sequence_call(race):
    k, B, V = 5, 4, 30000
    draft, target = small_inputs(B, k, V, torch.bfloat16, 3)
    par = torch.arange(-1, k - 1, dtype=torch.int32, device="cuda")
    rk = torch.zeros(k, dtype=torch.int32, device="cuda")
    a = race.race_verify_arrival_tree(draft, target, par, rk, 1.1, 9)
    s = race.race_verify(draft[:, :k].contiguous(), target, 1.1, 9)
    torch.cuda.synchronize()
    assert torch.equal(a[0], s[0]) and torch.equal(a[1], s[1]) and torch.equal(a[2], s[2])


def test_malformed_nodes_masked_rows_and_missing_arrivals(race, oracle_mod):
    parent = [-1, -1, -1, -1, 6, 3, 0, 0]
    rank = [0, 0, 1, 8, 0, 0, 0, 2]
    B, V = 3, 2048
    draft, target = small_inputs(B, len(parent), V, torch.float32, 5, noise=0.2)
    draft[:, 1, 2:] = -float("inf")     # context of node 0: two tokens in the support, three arrivals asked for
    draft[1, 0, :] = -float("inf")      # a draft row without support: no arrivals at all
    target[2, 3, :] = -float("inf")     # a target row without support: token 0 by convention
    for split in (0, 5):
        gpu, ora, ex = run(race, oracle_mod, draft, target, parent, rank, 1.0, 77, split)
        d = gpu[0].cpu().numpy()
        assert np.all(d[:, [1, 3, 4, 5]] == -1) and np.all(d[:, 7] == -1) and np.all(d[1, [0, 2]] == -1)
    assert not race.arrival_tree_validate_host(parent, rank)
    assert race.arrival_tree_validate_host([-1, 0, 0], [0, 0, 1])


def test_many_close_scores_overflow_the_lists_and_stay_exact(race, oracle_mod):
    # scores rising along the row make every token a new arrival candidate: lists overflow, the exact path decides
    B, V = 2, 16384
    parent, rank = [-1, -1, -1, 0], [0, 1, 2, 0]
    ramp = torch.arange(V, device="cuda", dtype=torch.float32) * 0.01
    target = ramp.repeat(B, len(parent) + 1, 1).contiguous()
    draft = (ramp + 0.001 * torch.randn(V, device="cuda")).repeat(B, len(parent) + 1, 1).contiguous()
    for split in (0, 3):
        run(race, oracle_mod, draft, target, parent, rank, 1.0, 5, split)


def test_results_do_not_depend_on_the_partition(race):
    parent, rank = TREES["mixed"]
    draft, target = small_inputs(4, len(parent), 50000, torch.bfloat16, 23)
    par = torch.tensor(parent, dtype=torch.int32, device="cuda")
    rk = torch.tensor(rank, dtype=torch.int32, device="cuda")
    ref = None
    for split in (0, 1, 7, 200):
        if split:
            parity.hooks.set(force_blocks=split)
        out = race.race_verify_arrival_tree(draft, target, par, rk, 1.0, 1)
        torch.cuda.synchronize()
        parity.hooks.set(force_blocks=0)
        if ref is None:
            ref = out
        else:
            assert all(torch.equal(a, b) for a, b in zip(out, ref))


def test_full_size_arrival_tree_matches_oracle(race, oracle_mod):
    w = wl.ARRIVAL_TREE
    inp = wl.make_inputs(w, "cuda")
    run(race, oracle_mod, inp["draft"], inp["target"], inp["parent"].cpu().numpy(), inp["rank"].cpu().numpy(),
        w.temperature, w.seed, note="full size")


def test_trees_from_the_builders_verify_like_the_oracle(race, oracle_mod):
    opt_parent, opt_rank, _, _ = race.tree_build_optimal([0.6, 0.2, 0.1, 0.05, 0.02], 40)
    si_parent, si_rank = race.tree_build_specinfer(20)
    for parent, rank in ((opt_parent, opt_rank), (si_parent, si_rank)):
        draft, target = small_inputs(3, len(parent), 32768, torch.bfloat16, 41, noise=0.4)
        run(race, oracle_mod, draft, target, parent, rank, 1.0, 8, note="builder tree")


@pytest.mark.parametrize("N,shape", [(2048, "bushy"), (2049, "bushy"), (8192, "bushy"), (3000, "chain")])
def test_largest_trees(race, oracle_mod, N, shape):
    """The node limit (8192), both sides of the size up to which the tree is staged in LDS (2048), and a walk that
    is thousands of contexts long."""
    rng = np.random.default_rng(N)
    if shape == "chain":
        parent = np.arange(-1, N - 1, dtype=np.int32)
        rank = np.zeros(N, dtype=np.int32)
    else:
        parent = np.array([int(rng.integers(max(-1, n - 40), n)) for n in range(N)], dtype=np.int32)
        rank = np.zeros(N, dtype=np.int32)
        seen = {}
        for n in range(N):
            r = seen.get(int(parent[n]), 0)
            rank[n] = min(r, race.max_rank() - 1)        # a ninth sibling repeats rank 7 and is thereby invalid
            seen[int(parent[n])] = r + 1
    B, V = 2, 40
    g = torch.Generator(device="cuda")
    g.manual_seed(N)
    target = 2.0 * torch.randn((B, N + 1, V), generator=g, device="cuda")
    noise = 0.05 if shape == "chain" else 0.6                 # close models: the chain is followed far down
    draft = target + noise * torch.randn((B, N + 1, V), generator=g, device="cuda")
    gpu, ora, ex = run(race, oracle_mod, draft.contiguous(), target.contiguous(), parent, rank, 1.0, 11, note=f"{shape} N={N}")
    if shape == "chain":
        assert int(ora["accept_len"].max()) > 5
