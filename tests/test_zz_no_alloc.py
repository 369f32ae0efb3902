"""ersd_race_verify_noalloc (the entry point for callers that cannot allocate) against ersd_race_verify: same
tokens and accept lengths, on two calls in a row, the second with a smaller input (the library's scratch array
keeps what the first call left there)."""
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
    r.set_test_hooks()
    return r


def _outs(B, k):
    i32 = dict(dtype=torch.int32, device="cuda")
    return (torch.full((B, k), -7, **i32), torch.full((B, k + 1), -7, **i32), torch.full((B,), -7, **i32))


@pytest.mark.parametrize("dtype_workload", [1, 2], ids=["bf16", "f32"])
def test_noalloc_equals_verify_on_two_calls_in_a_row(race, oracle_mod, dtype_workload):
    race.noalloc_prepare()
    shapes = [dict(B=6, k=5, V=50008), dict(B=2, k=3, V=12345)]      # the second call is the smaller one
    for n, shp in enumerate(shapes):
        w = wl.shrink(wl.WORKLOADS[dtype_workload], **shp)
        x = wl.make_inputs(w, "cuda")
        print(f"[case] noalloc call {n}: {wl.describe(w)}", flush=True)
        want = race.race_verify(x["draft"], x["target"], w.temperature, w.seed)
        out = _outs(w.B, w.k)
        torch.cuda.synchronize()
        before = torch.cuda.memory_allocated()
        got = race.race_verify_noalloc(x["draft"], x["target"], w.temperature, w.seed, out)
        torch.cuda.synchronize()
        assert torch.cuda.memory_allocated() == before
        for a, b in zip(got, want):
            assert torch.equal(a, b)
        ora = oracle_mod.race_verify(x["draft"].cpu(), x["target"].cpu(), w.temperature, w.seed, want_info=True)
        assert ora["draft_info"]["near_tie"].sum() + ora["target_info"]["near_tie"].sum() == 0
        for a, key in zip(got, ("draft_tokens", "target_tokens", "accept_len")):
            assert np.array_equal(a.cpu().numpy(), ora[key]), key
        del got, out, want, x      # nothing of this call is freed inside the next call's allocation check


def test_noalloc_refuses_a_job_beyond_its_scratch(race):
    B, k, V = 4096, 16, 152064
    assert race.workspace_bytes(race.VARIANT_SEQUENCE, B, 1, k, V, race.ERSD_F32) > (8 << 20)
    d = torch.zeros(1, 1, 8, device="cuda")      # never read: the sizes are refused on the host
    L = race.lib()
    rc = L.ersd_race_verify_noalloc(d.data_ptr(), d.data_ptr(), race.ERSD_F32, B, k, V, 1.0, 0, d.data_ptr(),
                                    d.data_ptr(), d.data_ptr(), None)
    assert rc == -7


def test_noalloc_call_can_be_captured_in_a_graph_and_replayed(race):
    """What the entry point is for: no allocation and no memset inside the call, so a captured call replays to the
    same outputs, also after other work on the device and after another call has used the library's scratch array."""
    race.noalloc_prepare()      # the address and occupancy queries happen here, before the capture
    w = wl.shrink(wl.WORKLOADS[1], B=8, k=4, V=65536)
    x = wl.make_inputs(w, "cuda")
    ref = race.race_verify(x["draft"], x["target"], w.temperature, w.seed)
    out = _outs(w.B, w.k)
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.stream(s):
        with torch.cuda.graph(g, stream=s):
            race.race_verify_noalloc(x["draft"], x["target"], w.temperature, w.seed, out)
    torch.cuda.synchronize()
    other = wl.make_inputs(wl.shrink(wl.WORKLOADS[2], B=3, k=2, V=30000), "cuda")
    for rep in range(3):
        for o in out:
            o.fill_(-7)
        race.race_verify_noalloc(other["draft"], other["target"], 0.7, 5, _outs(3, 2))   # overwrites the scratch array
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert all(torch.equal(a, b) for a, b in zip(out, ref)), f"replay {rep}"
        y = torch.randn(1 << 20, device="cuda").sum().item()   # eager work between replays
        assert y == y
