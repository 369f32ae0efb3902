"""GPU parity: the HIP library (called through its C ABI) against the CPU oracle on the same seeded inputs."""
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
    r.lib()  # raises if libersd.so was not built
    return r


@pytest.fixture(autouse=True)
def clean_env():
    parity.hooks.reset()
    yield
    parity.hooks.reset()


def run_case(race, oracle_mod, w, split=0, kernel=None, note=""):
    print(f"[case] {wl.describe(w)} split={split} kernel={kernel} {note}", flush=True)
    if split:
        parity.hooks.set(force_blocks=split)
    if kernel:
        parity.hooks.set(exhaustive=kernel == "exhaustive")
    inp = wl.make_inputs(w, "cuda")
    T, seed = w.temperature, w.seed
    d_host, t_host = inp["draft"].cpu(), inp["target"].cpu()
    if w.variant == "sequence":
        gpu = race.race_verify(inp["draft"], inp["target"], T, seed)
        torch.cuda.synchronize()
        ora = oracle_mod.race_verify(d_host, t_host, T, seed, want_info=True)
        ex = parity.check_sequence(gpu, ora, oracle_mod, d_host, t_host, T, seed)
    elif w.variant == "multi":
        gpu = race.race_verify_multi(inp["draft"], inp["target"], T, seed)
        torch.cuda.synchronize()
        ora = oracle_mod.race_verify_multi(d_host, t_host, T, seed, want_info=True)
        ex = parity.check_sequence(gpu, ora, oracle_mod, d_host, t_host, T, seed, multi=True)
    else:
        gpu = race.race_verify_tree(inp["draft"], inp["target"], inp["parent"], T, seed)
        torch.cuda.synchronize()
        par = inp["parent"].cpu().numpy()
        ora = oracle_mod.race_verify_tree(d_host, t_host, par, T, seed, want_info=True)
        ex = parity.check_tree(gpu, ora, oracle_mod, d_host, t_host, par, T, seed)
    flagged = int(ora["draft_info"]["near_tie"].sum() + ora["target_info"]["near_tie"].sum())
    print(f"[case] ok: oracle near-tie rows {flagged}, exempted rows {ex}", flush=True)
    parity.hooks.set(force_blocks=0)
    parity.hooks.set(exhaustive=False)
    return gpu, ora, ex


def test_filter_bounds_hold_for_every_generator_word(race):
    """The streaming filter is exact only if its two fp32 bounds hold (the device checks all 2^32 words) and if the
    packed half-precision maximum orders bf16 bit patterns (checked for every pair of in-domain patterns)."""
    r = race.selftest_bounds()
    print(r, flush=True)
    assert r["bad_upper"] == 0 and r["bad_refine"] == 0 and r["bad_pkmax"] == 0
    assert r["max_refine_err"] <= 2.0 ** -9


SMALL = [
    # several tiles plus a ragged tail, both dtypes, vocabulary sizes that are multiples of 8 and not (rows then start
    # at every alignment and end in a group of fewer than 8 tokens)
    wl.shrink(wl.WORKLOADS[0], B=2, k=3, V=5000),
    wl.shrink(wl.WORKLOADS[0], B=2, k=2, V=4999),
    wl.shrink(wl.WORKLOADS[1], B=3, k=4, V=20008),
    wl.shrink(wl.WORKLOADS[1], B=2, k=2, V=12345),
    wl.shrink(wl.WORKLOADS[2], B=4, k=3, V=9000),
    wl.shrink(wl.WORKLOADS[3], B=2, m=3, k=2, V=6152),
    wl.shrink(wl.WORKLOADS[4], B=3, N=12, V=7000),
    wl.shrink(wl.WORKLOADS[4], B=2, N=9, V=4101),
]


@pytest.mark.parametrize("w", SMALL, ids=lambda w: f"{w.name}-V{w.V}")
@pytest.mark.parametrize("kernel", ["exhaustive", None], ids=["exhaustive", "filtered"])
@pytest.mark.parametrize("split", [0, 1, 3, 50])
def test_small_shapes_match_oracle(race, oracle_mod, w, kernel, split):
    run_case(race, oracle_mod, w, split=split, kernel=kernel)


def test_results_do_not_depend_on_split_or_kernel_and_are_deterministic(race):
    w = wl.shrink(wl.WORKLOADS[1], B=4, k=4, V=40000)
    inp = wl.make_inputs(w, "cuda")
    ref = None
    for split in (0, 1, 2, 5, 19, 300):
        for kernel in (None, "exhaustive"):
            parity.hooks.set(force_blocks=split)
            if kernel:
                parity.hooks.set(exhaustive=kernel == "exhaustive")
            else:
                parity.hooks.set(exhaustive=False)
            for rep in range(2):
                out = [x.cpu() for x in race.race_verify(inp["draft"], inp["target"], 1.0, 77)]
                if ref is None:
                    ref = out
                for a, b in zip(ref, out):
                    assert torch.equal(a, b), (split, kernel, rep)


def test_degenerate_rows(race, oracle_mod):
    dev = "cuda"
    # V = 1, all -inf rows, heavily masked rows, identical models
    one = torch.zeros(2, 3, 1, device=dev)
    d, t, a = race.race_verify(one[:, :2].contiguous(), one, 1.0, 0)
    assert (t == 0).all() and (a == 2).all()
    ninf = torch.full((2, 3, 4104), float("-inf"), device=dev)
    for split in (1, 2, 6):
        parity.hooks.set(force_blocks=split)
        d, t, a = race.race_verify(ninf[:, :2].contiguous(), ninf, 1.0, 0)
        assert (t == 0).all() and (d == 0).all() and (a == 2).all()
    parity.hooks.set(force_blocks=0)
    g = torch.Generator(device=dev).manual_seed(5)
    V = 30000
    target = 3 * torch.randn(2, 4, V, generator=g, device=dev)
    draft = target[:, :3] + 0.5 * torch.randn(2, 3, V, generator=g, device=dev)
    keep = torch.randperm(V, generator=g, device=dev)[:40]          # top-k style mask: 40 live tokens
    mask = torch.ones(V, dtype=torch.bool, device=dev)
    mask[keep] = False
    target[..., mask] = float("-inf")
    draft[..., mask] = float("-inf")
    for dt in (torch.float32, torch.bfloat16):
        dd, tt = draft.to(dt).contiguous(), target.to(dt).contiguous()
        gpu = race.race_verify(dd, tt, 0.8, 9)
        torch.cuda.synchronize()
        ora = oracle_mod.race_verify(dd.cpu(), tt.cpu(), 0.8, 9, want_info=True)
        parity.check_sequence(gpu, ora, oracle_mod, dd.cpu(), tt.cpu(), 0.8, 9)
        assert not mask[gpu[1].long()].any()
    # identical logits: everything accepted, bit-exactly
    same = (3 * torch.randn(3, 5, 8192, generator=g, device=dev)).to(torch.bfloat16)
    d, t, a = race.race_verify(same[:, :4].contiguous(), same, 1.0, 3)
    assert (a == 4).all() and torch.equal(d, t[:, :4])


def test_adversarial_rows_overflow_the_candidate_list_and_stay_exact(race, oracle_mod):
    """Scores that keep rising with the token index make every token a new record: the candidate list overflows
    and the workgroup falls back to scoring its whole split exactly."""
    V = 16384
    ramp = torch.arange(V, device="cuda", dtype=torch.float32) * 0.5
    target = ramp.repeat(1, 3, 1).contiguous()
    draft = (ramp.repeat(1, 2, 1) * 1.01).contiguous()
    gpu = race.race_verify(draft, target, 1.0, 4)
    torch.cuda.synchronize()
    ora = oracle_mod.race_verify(draft.cpu(), target.cpu(), 1.0, 4, want_info=True)
    parity.check_sequence(gpu, ora, oracle_mod, draft.cpu(), target.cpu(), 1.0, 4)


def test_two_equal_dominant_logits_are_decided_by_their_own_words(race, oracle_mod):
    """Two equal huge logits dominate every exponential, so the race is between those two tokens and is decided by
    their own generator words; the GPU must agree with the oracle also when they sit in different row segments.
    (Finite EXACT ties, equal logits with equal words, are the subject of tests/test_gpu_ties.py.)"""
    V = 40960
    row = torch.full((V,), -50.0)
    row[100] = 40.0
    row[40000] = 40.0
    target = row.repeat(1, 2, 1).contiguous().cuda()
    draft = row.repeat(1, 1, 1).contiguous().cuda()
    for split in (1, 9):
        parity.hooks.set(force_blocks=split)
        for seed in range(6):
            gpu = race.race_verify(draft, target, 1.0, seed)
            ora = oracle_mod.race_verify(draft.cpu(), target.cpu(), 1.0, seed, want_info=True)
            parity.check_sequence(gpu, ora, oracle_mod, draft.cpu(), target.cpu(), 1.0, seed)
            assert int(gpu[1][0, 0]) in (100, 40000)


def test_tree_contract_on_device(race, oracle_mod):
    w = wl.shrink(wl.WORKLOADS[4], B=4, N=10, V=2048)
    inp = wl.make_inputs(w, "cuda")
    # chain-shaped tree equals the sequence variant
    chain = torch.arange(-1, 9, dtype=torch.int32, device="cuda")
    td, tt, ta, tn = race.race_verify_tree(inp["draft"], inp["target"], chain, 1.0, 5)
    bonus = torch.zeros(4, 1, 2048, dtype=inp["target"].dtype, device="cuda")
    sd, st, sa = race.race_verify(inp["draft"], torch.cat([inp["target"], bonus], 1).contiguous(), 1.0, 5)
    assert torch.equal(td, sd) and torch.equal(tt, st[:, :10]) and torch.equal(ta, sa) and torch.equal(tn, sa - 1)
    # malformed parents are rejected per node, identical logits make every well-formed node agree
    bad = torch.tensor([-1, 0, 7, 2, -1, 4, 5, -3, 7, 6], dtype=torch.int32, device="cuda")
    same = inp["target"]
    gd, gt, ga, gn = race.race_verify_tree(same, same, bad, 1.0, 5)
    ora = oracle_mod.race_verify_tree(same.cpu(), same.cpu(), bad.cpu().numpy(), 1.0, 5)
    assert np.array_equal(ga.cpu().numpy(), ora["accept_len"]) and np.array_equal(gn.cpu().numpy(), ora["accept_node"])
    assert (ga == 4).all() and (gn == 9).all()      # path 4 -> 5 -> 6 -> 9


def test_runs_on_a_side_stream_and_with_caller_workspace(race, oracle_mod):
    w = wl.shrink(wl.WORKLOADS[1], B=2, k=3, V=16384)
    inp = wl.make_inputs(w, "cuda")
    need = race.workspace_bytes(race.VARIANT_SEQUENCE, 2, 1, 3, 16384, race.ERSD_BF16)
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    ref = [x.cpu() for x in race.race_verify(inp["draft"], inp["target"], 1.0, 1)]
    s = torch.cuda.Stream()
    s.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(s):
        out = race.race_verify(inp["draft"], inp["target"], 1.0, 1, workspace=ws)
    s.synchronize()
    for a, b in zip(ref, out):
        assert torch.equal(a, b.cpu())
    with pytest.raises(race.ErsdError):
        race.race_verify(inp["draft"], inp["target"], 1.0, 1, workspace=ws[:16])


@pytest.mark.parametrize("idx", [0, 1, 2, 3, 4])
def test_full_size_workloads_match_oracle(race, oracle_mod, idx):
    """The five benchmark workloads at full size, in the launch configuration the benchmark times, against the
    oracle on every row."""
    w = wl.WORKLOADS[idx]
    gpu, ora, ex = run_case(race, oracle_mod, w, note="(full size)")
    acc = gpu[2].cpu().numpy()
    print(f"[full] {w.name}: mean accept_len {acc.mean():.3f}, exempted rows {ex}", flush=True)


def test_one_model_races_and_acceptance_step_equal_the_fused_calls(race, oracle_mod):
    """Drafting position by position with the draft model, racing the target rows afterwards and running the
    acceptance step on the tokens gives exactly what the fused verify calls give (and what the oracle gives)."""
    # sequence / multi
    w = wl.shrink(wl.WORKLOADS[3], B=3, m=2, k=3, V=10240)
    x = wl.make_inputs(w, "cuda")
    T, seed = w.temperature, w.seed
    fused = [v.cpu() for v in race.race_verify_multi(x["draft"], x["target"], T, seed)]
    steps = [race.race_sample(x["draft"][:, :, j:j + 1].contiguous(), j, T, seed) for j in range(w.k)]
    dtok = torch.cat(steps, dim=2).contiguous()
    ttok = race.race_sample(x["target"], 0, T, seed)
    acc, bd, bl = race.accept_lengths(race.VARIANT_MULTI, dtok, ttok)
    for got, ref in zip((dtok, ttok, acc, bd, bl), fused):
        assert torch.equal(got.cpu(), ref)
    o_d = oracle_mod.race_sample(x["draft"].cpu(), 0, T, seed)
    o_t = oracle_mod.race_sample(x["target"].cpu(), 0, T, seed)
    assert np.array_equal(dtok.cpu().numpy(), o_d) and np.array_equal(ttok.cpu().numpy(), o_t)
    # whole draft tensor in one call, fp32 and an odd vocabulary (element loads)
    w2 = wl.shrink(wl.WORKLOADS[0], B=2, k=3, V=4999)
    y = wl.make_inputs(w2, "cuda")
    fd, ft, fa = race.race_verify(y["draft"], y["target"], 1.0, 5)
    sd = race.race_sample(y["draft"].unsqueeze(1).contiguous(), 0, 1.0, 5)[:, 0]
    st = race.race_sample(y["target"].unsqueeze(1).contiguous(), 0, 1.0, 5)[:, 0]
    assert torch.equal(sd, fd) and torch.equal(st, ft)
    assert torch.equal(race.accept_lengths(race.VARIANT_SEQUENCE, sd.contiguous(), st.contiguous()), fa)
    # tree: positions are node indices
    w3 = wl.shrink(wl.WORKLOADS[4], B=2, N=12, V=8192)
    z = wl.make_inputs(w3, "cuda")
    td, tt, ta, tn = race.race_verify_tree(z["draft"], z["target"], z["parent"], 1.0, 9)
    sd = race.race_sample(z["draft"].unsqueeze(1).contiguous(), 0, 1.0, 9)[:, 0].contiguous()
    st = race.race_sample(z["target"].unsqueeze(1).contiguous(), 0, 1.0, 9)[:, 0].contiguous()
    assert torch.equal(sd, td) and torch.equal(st, tt)
    a2, n2 = race.accept_lengths(race.VARIANT_TREE, sd, st, z["parent"])
    assert torch.equal(a2, ta) and torch.equal(n2, tn)


def test_one_model_race_full_size_target_rows(race, oracle_mod):
    """Target-only races at the headline shape (B=64, 9 positions, V=128256, bf16) against the oracle."""
    w = wl.WORKLOADS[1]
    x = wl.make_inputs(w, "cuda")
    tok = race.race_sample(x["target"].unsqueeze(1).contiguous(), 0, w.temperature, w.seed)
    torch.cuda.synchronize()
    ref, info = oracle_mod.race_sample(x["target"].unsqueeze(1).contiguous().cpu(), 0, w.temperature, w.seed, want_info=True)
    assert info["near_tie"].sum() == 0
    assert np.array_equal(tok.cpu().numpy(), ref)


def test_verify_call_can_be_captured_in_a_graph_and_replayed(race):
    # the entry points allocate nothing, never synchronise and clear nothing with memsets: a captured call replays
    # to the same outputs, also after other work on the device
    w = wl.shrink(wl.WORKLOADS[1], B=8, k=4, V=65536)
    x = wl.make_inputs(w, "cuda")
    call = race.PreparedVerify(race.VARIANT_SEQUENCE, x["draft"], x["target"], w.temperature, w.seed)
    call.run()
    torch.cuda.synchronize()
    ref = tuple(o.clone() for o in call.outputs())
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            call.run()
    torch.cuda.synchronize()
    for rep in range(3):
        for o in call.outputs():
            o.fill_(-7)
        call.workspace.random_(0, 255)            # replays must not depend on what the workspace held
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(call.outputs(), ref)), f"replay {rep}"
        y = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between replays
        assert y == y


@pytest.mark.parametrize("tail", [1, 2, 3, 4, 5, 6, 7])
@pytest.mark.parametrize("idx", [1, 2], ids=["bf16", "f32"])
def test_every_ragged_row_end_and_row_alignment(race, oracle_mod, idx, tail):
    # V = 8 n + tail: rows begin at all element alignments and end in a group of `tail` tokens
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[idx], B=3, k=3, V=16384 + tail), split=0)
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[idx], B=2, k=2, V=8 + tail), split=5, note="barely more than a group")


def test_vocabulary_smaller_than_a_group_and_gpt2_size(race, oracle_mod):
    for V in (1, 2, 5, 7):
        run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[0], B=4, k=2, V=V), note="no whole group")
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[1], B=8, k=4, V=50257), note="odd vocabulary at full row length")


def test_long_sequences_many_drafts_and_big_trees(race, oracle_mod):
    """Shapes far from the benchmark's: thousands of positions, hundreds of drafts, thousands of tree nodes, each
    with a small vocabulary (many rows per workgroup, and the two-launch finishing path)."""
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[0], B=2, k=3000, V=24), note="k = 3000")
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[3], B=2, m=300, k=3, V=40), note="m = 300")
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[4], B=2, N=5000, V=16), note="N = 5000")
    run_case(race, oracle_mod, wl.shrink(wl.WORKLOADS[1], B=3000, k=1, V=8), note="B = 3000")


def test_read_probe_runs_and_leaves_its_inputs_alone(race):
    x = torch.randn(3, 5, 4096, device="cuda")
    y = torch.randn(7, 4096, device="cuda").to(torch.bfloat16)
    x0, y0 = x.clone(), y.clone()
    sink = race.read_probe(x, y)
    race.read_probe(y)
    torch.cuda.synchronize()
    assert torch.equal(x, x0) and torch.equal(y, y0) and int(sink.item()) in (0, 1)
