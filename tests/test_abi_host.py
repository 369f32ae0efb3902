"""Host-side checks of the C ABI that need no GPU: the library loads, exports what include/ersd.h declares,
and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    from paper_2504_15475_amd import race
    return race.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ersd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ersd_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(L):
    names = declared_functions()
    assert {"ersd_race_verify", "ersd_race_verify_multi", "ersd_race_verify_tree", "ersd_race_workspace_bytes",
            "ersd_status_string", "ersd_version", "ersd_tree_validate_host", "ersd_selftest_bounds",
            "ersd_race_stage_races", "ersd_race_stage_accept", "ersd_plan_describe_host", "ersd_philox_rounds", "ersd_race_sample",
            "ersd_race_sample_workspace_bytes", "ersd_accept_lengths", "ersd_race_verify_noalloc", "ersd_noalloc_prepare",
            "ersd_test_hooks_set"} <= set(names)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings(L):
    assert L.ersd_version() >= 300
    import oracle
    assert L.ersd_philox_rounds() == oracle.get_rounds() and L.ersd_philox_rounds() in (7, 10)   # same generator on both sides
    seen = set()
    for s in range(0, -8, -1):
        txt = L.ersd_status_string(s)
        assert txt and txt not in seen
        seen.add(txt)
    assert L.ersd_status_string(-99) == b"unknown status"


FAKE = 0x10000  # non-null, 16-byte aligned; never dereferenced because every call below fails validation first


def seq_call(L, d=FAKE, t=FAKE, dt=0, B=1, k=2, V=64, T=1.0, seed=0, o1=FAKE, o2=FAKE, o3=FAKE, ws=FAKE, wsb=1 << 30):
    return L.ersd_race_verify(d, t, dt, B, k, V, T, seed, o1, o2, o3, ws, wsb, None)


def test_sequence_argument_errors(L):
    assert seq_call(L, d=None) == -1 and seq_call(L, t=None) == -1
    assert seq_call(L, o1=None) == -1 and seq_call(L, o2=None) == -1 and seq_call(L, o3=None) == -1
    assert seq_call(L, ws=None) == -1
    assert seq_call(L, dt=2) == -3 and seq_call(L, dt=-1) == -3
    for T in (0.0, -1.0, float("nan"), float("inf")):
        assert seq_call(L, T=T) == -2
    assert seq_call(L, B=0) == -2 and seq_call(L, k=0) == -2 and seq_call(L, V=0) == -2 and seq_call(L, B=-3) == -2
    assert seq_call(L, k=2**31 - 1) == -2                     # k + 1 would overflow
    assert seq_call(L, B=2**30, k=2**12, V=2**20) == -2       # job too large for the 64-bit work partition
    assert seq_call(L, d=FAKE + 4) == -4 and seq_call(L, t=FAKE + 8) == -4 and seq_call(L, ws=FAKE + 2) == -4
    assert seq_call(L, wsb=8) == -5


def test_multi_and_tree_argument_errors(L):
    def multi(**kw):
        a = dict(d=FAKE, t=FAKE, dt=1, B=2, m=3, k=2, V=64, T=1.0, seed=0, o=[FAKE] * 5, ws=FAKE, wsb=1 << 30)
        a.update(kw)
        return L.ersd_race_verify_multi(a["d"], a["t"], a["dt"], a["B"], a["m"], a["k"], a["V"], a["T"], a["seed"],
                                        *a["o"], a["ws"], a["wsb"], None)
    assert multi(m=0) == -2 and multi(T=0.0) == -2 and multi(d=None) == -1 and multi(wsb=0) == -5
    for i in range(5):
        o = [FAKE] * 5
        o[i] = None
        assert multi(o=o) == -1

    def tree(**kw):
        a = dict(d=FAKE, t=FAKE, dt=1, B=2, N=5, V=64, parent=FAKE, T=1.0, seed=0, o=[FAKE] * 4, ws=FAKE, wsb=1 << 30)
        a.update(kw)
        return L.ersd_race_verify_tree(a["d"], a["t"], a["dt"], a["B"], a["N"], a["V"], a["parent"], a["T"],
                                       a["seed"], *a["o"], a["ws"], a["wsb"], None)
    assert tree(parent=None) == -1 and tree(N=0) == -2 and tree(T=-2.0) == -2 and tree(wsb=1) == -5
    assert tree(o=[FAKE, FAKE, None, FAKE]) == -1
    assert L.ersd_selftest_bounds(None, None) == -1
    # the two stages validate like the verify calls
    assert L.ersd_race_stage_races(0, None, FAKE, 0, 1, 1, 2, 64, 1.0, 0, FAKE, 1 << 30, None) == -1
    assert L.ersd_race_stage_races(0, FAKE, FAKE, 0, 1, 1, 2, 64, 0.0, 0, FAKE, 1 << 30, None) == -2
    assert L.ersd_race_stage_races(7, FAKE, FAKE, 0, 1, 1, 2, 64, 1.0, 0, FAKE, 1 << 30, None) == -2
    assert L.ersd_race_stage_races(0, FAKE, FAKE, 0, 1, 1, 2, 64, 1.0, 0, FAKE, 8, None) == -5
    assert L.ersd_race_stage_accept(0, 0, 1, 1, 2, 64, 1.0, None, FAKE, FAKE, FAKE, None, None, None, FAKE, 8, None) == -5
    assert L.ersd_race_stage_accept(0, 0, 1, 1, 2, 64, 1.0, None, None, FAKE, FAKE, None, None, None, FAKE, 1 << 30, None) == -1
    assert L.ersd_race_stage_accept(2, 0, 1, 1, 2, 64, 1.0, None, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 30, None) == -1
    assert L.ersd_race_stage_accept(1, 0, 1, 1, 2, 64, 1.0, None, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 30, None) == -1
    assert L.ersd_race_stage_accept(0, 9, 1, 1, 2, 64, 1.0, None, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 30, None) == -3
    assert L.ersd_race_stage_accept(0, 0, 1, 1, 2, 64, 0.0, None, FAKE, FAKE, FAKE, None, None, None, FAKE, 1 << 30, None) == -2


def test_sample_and_accept_argument_errors(L):
    def sample(**kw):
        a = dict(x=FAKE, dt=1, B=2, m=1, npos=3, V=64, pos0=0, T=1.0, seed=0, tok=FAKE, ws=FAKE, wsb=1 << 30)
        a.update(kw)
        return L.ersd_race_sample(a["x"], a["dt"], a["B"], a["m"], a["npos"], a["V"], a["pos0"], a["T"], a["seed"],
                                  a["tok"], a["ws"], a["wsb"], None)
    assert sample(x=None) == -1 and sample(tok=None) == -1 and sample(ws=None) == -1
    assert sample(dt=7) == -3 and sample(T=0.0) == -2 and sample(npos=0) == -2 and sample(pos0=-1) == -2
    assert sample(pos0=2**31 - 2) == -2 and sample(x=FAKE + 2) == -4 and sample(wsb=4) == -5
    assert L.ersd_race_sample_workspace_bytes(2, 1, 3, 64, 1) > 0
    assert L.ersd_race_sample_workspace_bytes(0, 1, 3, 64, 1) == 0 and L.ersd_race_sample_workspace_bytes(2, 1, 3, 64, 4) == 0
    acc = L.ersd_accept_lengths
    assert acc(0, 2, 1, 3, None, None, FAKE, FAKE, None, None, None, None) == -1
    assert acc(0, 2, 1, 3, None, FAKE, FAKE, None, None, None, None, None) == -1
    assert acc(2, 2, 1, 3, None, FAKE, FAKE, FAKE, None, None, None, None) == -1      # tree without parent
    assert acc(1, 2, 2, 3, None, FAKE, FAKE, FAKE, None, None, None, None) == -1      # multi without best outputs
    assert acc(0, 0, 1, 3, None, FAKE, FAKE, FAKE, None, None, None, None) == -2 and acc(5, 2, 1, 3, None, FAKE, FAKE, FAKE, None, None, None, None) == -2


def test_workspace_bytes(L):
    wb = L.ersd_race_workspace_bytes
    assert wb(0, 1, 1, 4, 32000, 0) > 0
    assert wb(0, 0, 1, 4, 32000, 0) == 0 and wb(3, 1, 1, 4, 32000, 0) == 0 and wb(0, 1, 1, 4, 32000, 5) == 0
    # enough for one 16-byte partial per (row, side); more rows never need less
    assert wb(0, 64, 1, 8, 128256, 1) >= 64 * 9 * 2 * 16
    assert wb(1, 32, 8, 8, 128256, 1) >= 32 * 8 * 9 * 2 * 16
    assert wb(2, 16, 1, 64, 256000, 1) >= 16 * 64 * 2 * 16
    # the documented size is sufficient and one byte less is rejected (checked before any device work)
    need = wb(0, 2, 1, 3, 4096, 0)
    assert seq_call(L, B=2, k=3, V=4096, wsb=need - 1) == -5


def test_tree_validate_host():
    from paper_2504_15475_amd import race
    assert race.tree_validate_host(np.array([-1, 0, 0, 1, -1], dtype=np.int32))
    assert not race.tree_validate_host(np.array([-1, 1], dtype=np.int32))       # self / forward reference
    assert not race.tree_validate_host(np.array([-2, 0], dtype=np.int32))
    assert not race.tree_validate_host(np.array([0], dtype=np.int32))


def test_binding_refuses_cpu_tensors():
    import torch
    from paper_2504_15475_amd import race
    d = torch.zeros(1, 2, 8)
    t = torch.zeros(1, 3, 8)
    with pytest.raises(ValueError):
        race.race_verify(d, t, 1.0, 0)


def test_workload_generators_are_seeded_and_shaped():
    import torch
    from paper_2504_15475_amd import workloads as wl
    assert [w.race_elements for w in wl.WORKLOADS] == [288000, 139542528, 1284636672, 558170112, 524288000]
    small = wl.shrink(wl.WORKLOADS[1], B=2, k=3, V=1024)
    a, b = wl.make_inputs(small), wl.make_inputs(small)
    assert a["draft"].dtype == torch.bfloat16 and tuple(a["target"].shape) == (2, 4, 1024)
    assert torch.equal(a["target"], b["target"]) and torch.equal(a["draft"], b["draft"])
    t = wl.shrink(wl.WORKLOADS[4], B=2, N=64, V=256, level_sizes=(4, 8, 12, 14, 14, 12))
    p = wl.tree_parents(t)
    from paper_2504_15475_amd import race
    assert race.tree_validate_host(p) and (p[:4] == -1).all() and p.max() < 63
    m = wl.make_inputs(wl.shrink(wl.WORKLOADS[3], B=2, m=3, k=2, V=512))
    assert tuple(m["draft"].shape) == (2, 3, 2, 512) and tuple(m["target"].shape) == (2, 3, 3, 512)
    c2 = wl.make_inputs(wl.shrink(wl.WORKLOADS[2], B=2, k=2, V=4096))
    assert c2["target"].dtype == torch.float32 and float(c2["target"].max()) > 12.0     # boosted tokens present


def test_arrival_tree_and_gsd_argument_errors(L):
    def arr(**kw):
        a = dict(d=FAKE, t=FAKE, dt=1, B=2, N=5, V=64, par=FAKE, rk=FAKE, T=1.0, seed=0, o=[FAKE] * 5, ws=FAKE,
                 wsb=1 << 30)
        a.update(kw)
        return L.ersd_race_verify_arrival_tree(a["d"], a["t"], a["dt"], a["B"], a["N"], a["V"], a["par"], a["rk"],
                                               a["T"], a["seed"], *a["o"], a["ws"], a["wsb"], None)
    assert arr(d=None) == -1 and arr(t=None) == -1 and arr(par=None) == -1 and arr(rk=None) == -1 and arr(ws=None) == -1
    for i in range(5):
        o = [FAKE] * 5
        o[i] = None
        assert arr(o=o) == -1
    assert arr(dt=7) == -3 and arr(T=0.0) == -2 and arr(T=float("nan")) == -2
    assert arr(B=0) == -2 and arr(N=0) == -2 and arr(V=0) == -2 and arr(N=8193) == -2   # ERSD_MAX_ARRIVAL_TREE_NODES
    assert arr(d=FAKE + 8) == -4 and arr(ws=FAKE + 4) == -4
    assert arr(wsb=16) == -5
    need = L.ersd_race_arrival_tree_workspace_bytes(2, 5, 64, 1)
    assert need > 0 and arr(wsb=need - 1) == -5
    assert L.ersd_race_arrival_tree_workspace_bytes(0, 5, 64, 1) == 0
    assert L.ersd_race_arrival_tree_workspace_bytes(2, 5, 64, 9) == 0
    assert L.ersd_max_rank() == 8

    def gsd(**kw):
        a = dict(d=FAKE, t=FAKE, dt=0, B=2, k=3, V=64, tok=FAKE, T=1.0, seed=0, o1=FAKE, o2=FAKE, ws=FAKE, wsb=1 << 30)
        a.update(kw)
        return L.ersd_gsd_verify(a["d"], a["t"], a["dt"], a["B"], a["k"], a["V"], a["tok"], a["T"], a["seed"], a["o1"],
                                 a["o2"], a["ws"], a["wsb"], None)
    assert gsd(d=None) == -1 and gsd(t=None) == -1 and gsd(tok=None) == -1 and gsd(o1=None) == -1 and gsd(o2=None) == -1
    assert gsd(ws=None) == -1 and gsd(dt=3) == -3 and gsd(T=-2.0) == -2 and gsd(T=float("inf")) == -2
    assert gsd(B=0) == -2 and gsd(k=0) == -2 and gsd(V=0) == -2 and gsd(B=2**30, k=2**10) == -2
    assert gsd(t=FAKE + 2) == -4 and gsd(wsb=0) == -5
    need = L.ersd_gsd_workspace_bytes(2, 3, 64, 0)
    assert need > 0 and gsd(wsb=need - 1) == -5 and L.ersd_gsd_workspace_bytes(2, 0, 64, 0) == 0


def test_tree_builders_argument_errors(L):
    r = (ctypes.c_double * 2)(0.5, 0.2)
    par = (ctypes.c_int32 * 4)()
    rk = (ctypes.c_int32 * 4)()
    assert L.ersd_tree_build_optimal_host(None, 2, 4, par, rk, None, None) == -1
    assert L.ersd_tree_build_optimal_host(r, 2, 4, None, rk, None, None) == -1
    assert L.ersd_tree_build_optimal_host(r, 0, 4, par, rk, None, None) == -2
    assert L.ersd_tree_build_optimal_host(r, 2, 0, par, rk, None, None) == -2
    assert L.ersd_tree_build_optimal_host(r, 2, 4, par, rk, None, None) == 0
    assert list(par) == [-1, 0, -1, 1] and list(rk) == [0, 0, 1, 0]     # R: .5, .25, .2, .125
    assert L.ersd_tree_build_specinfer_host(4, 2, 3, None, rk) == -1
    assert L.ersd_tree_build_specinfer_host(0, 2, 3, par, rk) == -2
    assert L.ersd_tree_build_specinfer_host(4, -1, 3, par, rk) == -2
    assert L.ersd_tree_build_specinfer_host(4, 2, 0, par, rk) == -2


def test_strided_argument_errors(L):
    """Row strides are checked on the host: rows must not overlap and the tensors must stay addressable."""
    def seq(ds=64, ts=64, V=64, **kw):
        a = dict(d=FAKE, t=FAKE, dt=0, B=1, k=2, T=1.0, seed=0, o1=FAKE, o2=FAKE, o3=FAKE, ws=FAKE, wsb=1 << 30)
        a.update(kw)
        return L.ersd_race_verify_strided(a["d"], ds, a["t"], ts, a["dt"], a["B"], a["k"], V, a["T"], a["seed"],
                                          a["o1"], a["o2"], a["o3"], a["ws"], a["wsb"], None)
    assert seq(ds=63) == -2 and seq(ts=63) == -2 and seq(ds=0) == -2 and seq(ts=-64) == -2
    assert seq(ds=1 << 41) == -2                      # beyond what the row offsets are sized for
    assert seq(d=None) == -1 and seq(o3=None) == -1 and seq(dt=5) == -3 and seq(T=0.0) == -2
    assert seq(ds=72, ts=64, wsb=16) == -5            # valid strides reach the workspace check
    assert L.ersd_race_verify_multi_strided(FAKE, 63, FAKE, 64, 0, 1, 2, 2, 64, 1.0, 0, FAKE, FAKE, FAKE, FAKE, FAKE,
                                            FAKE, 1 << 30, None) == -2
    assert L.ersd_race_verify_multi_strided(FAKE, 64, FAKE, 64, 0, 1, 2, 2, 64, 1.0, 0, FAKE, FAKE, FAKE, None, FAKE,
                                            FAKE, 1 << 30, None) == -1
    assert L.ersd_race_verify_tree_strided(FAKE, 64, FAKE, 32, 0, 1, 3, 64, FAKE, 1.0, 0, FAKE, FAKE, FAKE, FAKE,
                                           FAKE, 1 << 30, None) == -2
    assert L.ersd_race_verify_tree_strided(FAKE, 64, FAKE, 64, 0, 1, 3, 64, None, 1.0, 0, FAKE, FAKE, FAKE, FAKE,
                                           FAKE, 1 << 30, None) == -1
    assert L.ersd_race_sample_strided(FAKE, 10, 0, 1, 1, 2, 64, 0, 1.0, 0, FAKE, FAKE, 1 << 30, None) == -2
    assert L.ersd_race_sample_strided(FAKE, 64, 0, 1, 1, 2, 64, 0, 1.0, 0, None, FAKE, 1 << 30, None) == -1
    assert L.ersd_race_verify_arrival_tree_strided(FAKE, 64, FAKE, 63, 0, 1, 3, 64, FAKE, FAKE, 1.0, 0, FAKE, FAKE,
                                                   FAKE, FAKE, FAKE, FAKE, 1 << 30, None) == -2


def test_binding_row_stride_of_views():
    """The binding derives the row stride from a tensor's shape and strides alone."""
    import torch
    from paper_2504_15475_amd import race

    class View:  # shape and strides of a tensor, flagged as device memory
        def __init__(self, t):
            self.shape, self._s, self.is_cuda = t.shape, t.stride(), True

        def stride(self, i=None):
            return self._s if i is None else self._s[i]

    x = torch.zeros(3, 4, 40, device="meta")
    assert race._rows(View(x), "x") == 40
    assert race._rows(View(x[..., :33]), "x") == 40          # padded vocabulary
    assert race._rows(View(x[:1, :3, :33]), "x") == 40       # a single leading block keeps rows evenly spaced
    with pytest.raises(ValueError):
        race._rows(View(x[:, :3, :33]), "x")                 # a cut middle axis does not
    with pytest.raises(ValueError):
        race._rows(View(x[..., ::2]), "x")                   # vocabulary axis not dense
    y = torch.zeros(5, 64, device="meta").unsqueeze(0)
    assert race._rows(View(y[..., :50]), "y") == 64


def test_noalloc_entry_point_checks_its_arguments_on_the_host(L):
    import ctypes
    vp, i32 = ctypes.c_void_p, ctypes.c_int32
    L.ersd_race_verify_noalloc.argtypes = [vp, vp, ctypes.c_int, i32, i32, i32, ctypes.c_float, ctypes.c_uint64, vp, vp,
                                           vp, vp]

    def call(d=FAKE, t=FAKE, dt=0, B=1, k=2, V=64, T=1.0, o1=FAKE, o2=FAKE, o3=FAKE):
        return L.ersd_race_verify_noalloc(d, t, dt, B, k, V, T, 0, o1, o2, o3, None)

    assert call(d=None) == -1 and call(o2=None) == -1 and call(dt=5) == -3 and call(T=0.0) == -2 and call(B=0) == -2
    assert call(d=FAKE + 4) == -4
    # more scratch than the library holds: refused before any GPU call, with its own status
    big = dict(dt=0, B=4096, k=16, V=152064)
    assert L.ersd_race_workspace_bytes(0, big["B"], 1, big["k"], big["V"], 0) > (8 << 20)
    assert call(**big) == -7
    assert b"scratch" in L.ersd_status_string(-7)


def test_prepared_arrival_tree_entry_points_check_their_arguments_on_the_host(L):
    import ctypes
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    L.ersd_arrival_tree_plan_bytes.argtypes = [i32]
    L.ersd_arrival_tree_plan_bytes.restype = sz
    assert L.ersd_arrival_tree_plan_bytes(0) == 0 and L.ersd_arrival_tree_plan_bytes(8193) == 0
    need = L.ersd_arrival_tree_plan_bytes(64)
    assert need >= 4 * (64 + 65 + 66) and need % 16 == 0
    L.ersd_arrival_tree_prepare.argtypes = [vp, vp, i32, vp, sz, vp]
    assert L.ersd_arrival_tree_prepare(None, FAKE, 64, FAKE, need, None) == -1
    assert L.ersd_arrival_tree_prepare(FAKE, FAKE, 64, None, need, None) == -1
    assert L.ersd_arrival_tree_prepare(FAKE, FAKE, 0, FAKE, need, None) == -2
    assert L.ersd_arrival_tree_prepare(FAKE, FAKE, 64, FAKE + 8, need, None) == -4
    assert L.ersd_arrival_tree_prepare(FAKE, FAKE, 64, FAKE, need - 1, None) == -5
    L.ersd_race_verify_arrival_tree_prepared.argtypes = [vp, i64, vp, i64, ctypes.c_int, i32, i32, i32, vp, vp, vp, sz,
                                                         ctypes.c_float, ctypes.c_uint64, vp, vp, vp, vp, vp, vp, sz, vp]

    def call(d=FAKE, plan=FAKE, pb=need, B=2, N=64, V=1000, stride=1000, T=1.0, ws=FAKE, wsb=1 << 30):
        return L.ersd_race_verify_arrival_tree_prepared(d, stride, FAKE, stride, 0, B, N, V, FAKE, FAKE, plan, pb, T, 0,
                                                        FAKE, FAKE, FAKE, FAKE, FAKE, ws, wsb, None)

    assert call(d=None) == -1 and call(plan=None) == -1 and call(plan=FAKE + 4) == -4 and call(T=-1.0) == -2
    assert call(N=0) == -2 and call(stride=999) == -2 and call(pb=need - 16) == -5 and call(wsb=64) == -5


def test_gsd_tree_entry_point_checks_its_arguments_on_the_host(L):
    import ctypes
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    L.ersd_arrival_tree_plan_bytes.argtypes = [i32]
    L.ersd_arrival_tree_plan_bytes.restype = sz
    need = L.ersd_arrival_tree_plan_bytes(10)
    L.ersd_gsd_verify_tree.argtypes = [vp, vp, ctypes.c_int, i32, i32, i32, vp, vp, vp, sz, vp, ctypes.c_float,
                                       ctypes.c_uint64, vp, vp, vp, vp]

    def call(d=FAKE, dt=0, B=2, N=10, V=1000, plan=FAKE, pb=need, tok=FAKE, T=1.0, o=FAKE):
        return L.ersd_gsd_verify_tree(d, FAKE, dt, B, N, V, FAKE, FAKE, plan, pb, tok, T, 0, o, FAKE, FAKE, None)

    assert call(d=None) == -1 and call(plan=None) == -1 and call(tok=None) == -1 and call(o=None) == -1
    assert call(dt=4) == -3 and call(T=float("inf")) == -2 and call(B=0) == -2 and call(N=0) == -2 and call(N=8193) == -2
    assert call(d=FAKE + 2) == -4 and call(plan=FAKE + 8) == -4 and call(pb=need - 16) == -5
