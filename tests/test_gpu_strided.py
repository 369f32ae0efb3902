"""GPU: logits whose rows are strided (a padded vocabulary, a slice of a wider tensor) give exactly the results of
the same rows laid back to back, and match the CPU oracle.  The padding holds values that would win every race if
they were read."""
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


def padded(x, pad):
    """x [..., V] -> a view [..., V] of a tensor [..., V + pad] whose extra columns hold a huge logit."""
    wide = torch.full(x.shape[:-1] + (x.shape[-1] + pad,), 3.0e4, dtype=x.dtype, device=x.device)
    wide[..., : x.shape[-1]] = x
    view = wide[..., : x.shape[-1]]
    assert not view.is_contiguous() or pad == 0
    return view


def same(a, b):
    for x, y in zip(a, b):
        assert torch.equal(x, y)


@pytest.mark.parametrize("kernel", [None, "exhaustive"], ids=["filtered", "exhaustive"])
@pytest.mark.parametrize("split", [0, 7])
@pytest.mark.parametrize("pads", [(1, 0), (3, 8), (24, 5), (4096, 4096)])
@pytest.mark.parametrize("idx", [1, 2], ids=["bf16", "f32"])
def test_sequence_rows_with_padding(race, oracle_mod, idx, pads, split, kernel):
    w = wl.shrink(wl.WORKLOADS[idx], B=3, k=3, V=9001 if pads[0] % 2 else 9000)
    print(f"[case] strided {wl.describe(w)} pads={pads} split={split} kernel={kernel}", flush=True)
    inp = wl.make_inputs(w, "cuda")
    if split:
        parity.hooks.set(force_blocks=split)
    if kernel:
        parity.hooks.set(exhaustive=kernel == "exhaustive")
    ref = race.race_verify(inp["draft"], inp["target"], w.temperature, w.seed)
    out = race.race_verify(padded(inp["draft"], pads[0]), padded(inp["target"], pads[1]), w.temperature, w.seed)
    torch.cuda.synchronize()
    same(ref, out)
    d_host, t_host = inp["draft"].cpu(), inp["target"].cpu()
    ora = oracle_mod.race_verify(d_host, t_host, w.temperature, w.seed, want_info=True)
    parity.check_sequence(out, ora, oracle_mod, d_host, t_host, w.temperature, w.seed)


def test_multi_tree_sample_and_arrival_tree_with_padding(race, oracle_mod):
    w = wl.shrink(wl.WORKLOADS[3], B=2, m=3, k=2, V=6152)
    inp = wl.make_inputs(w, "cuda")
    print(f"[case] strided {wl.describe(w)}", flush=True)
    same(race.race_verify_multi(inp["draft"], inp["target"], w.temperature, w.seed),
         race.race_verify_multi(padded(inp["draft"], 7), padded(inp["target"], 40), w.temperature, w.seed))
    same([race.race_sample(inp["target"], 0, w.temperature, w.seed)],
         [race.race_sample(padded(inp["target"], 11), 0, w.temperature, w.seed)])

    w = wl.shrink(wl.WORKLOADS[4], B=3, N=12, V=7001)
    inp = wl.make_inputs(w, "cuda")
    print(f"[case] strided {wl.describe(w)}", flush=True)
    ref = race.race_verify_tree(inp["draft"], inp["target"], inp["parent"], w.temperature, w.seed)
    out = race.race_verify_tree(padded(inp["draft"], 3), padded(inp["target"], 3), inp["parent"], w.temperature, w.seed)
    same(ref, out)
    par = inp["parent"].cpu().numpy()
    d_host, t_host = inp["draft"].cpu(), inp["target"].cpu()
    ora = oracle_mod.race_verify_tree(d_host, t_host, par, w.temperature, w.seed, want_info=True)
    parity.check_tree(out, ora, oracle_mod, d_host, t_host, par, w.temperature, w.seed)

    w = wl.shrink(wl.ARRIVAL_TREE, B=2, N=10, V=5003)
    inp = wl.make_inputs(w, "cuda")
    print(f"[case] strided {wl.describe(w)}", flush=True)
    for split in (0, 5):
        if split:
            parity.hooks.set(force_blocks=split)
        ref = race.race_verify_arrival_tree(inp["draft"], inp["target"], inp["parent"], inp["rank"], w.temperature, w.seed)
        out = race.race_verify_arrival_tree(padded(inp["draft"], 13), padded(inp["target"], 2), inp["parent"],
                                            inp["rank"], w.temperature, w.seed)
        torch.cuda.synchronize()
        same(ref, out)


def test_strided_call_at_the_headline_shape(race, oracle_mod):
    """Full size, the launch configuration the benchmark times, vocabulary padded to the next multiple of 128:
    equal to the dense call, which the other tests tie to the oracle."""
    w = wl.WORKLOADS[1]
    inp = wl.make_inputs(w, "cuda")
    pad = (-w.V) % 128 or 128
    ref = race.race_verify(inp["draft"], inp["target"], w.temperature, w.seed)
    out = race.race_verify(padded(inp["draft"], pad), padded(inp["target"], pad), w.temperature, w.seed)
    torch.cuda.synchronize()
    same(ref, out)
