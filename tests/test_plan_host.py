"""The balanced work partition, checked on the host by brute force: shares tile the job exactly, every row's
writers are exactly the shares that overlap it, the slot bound the workspace is sized for holds, and the shares
cost the same under the stated model (10 per group of a row pair, 5 per group of a target-only row, a fixed
charge per row start)."""
import numpy as np
import pytest

from paper_2504_15475_amd import race

SEQ, MULTI, TREE = race.VARIANT_SEQUENCE, race.VARIANT_MULTI, race.VARIANT_TREE

CASES = [
    (SEQ, 1, 1, 4, 32000), (SEQ, 64, 1, 8, 128256), (SEQ, 256, 1, 16, 152064), (MULTI, 32, 8, 8, 128256),
    (TREE, 16, 1, 64, 256000), (SEQ, 3, 1, 2, 4999), (SEQ, 2, 1, 1, 7), (TREE, 5, 1, 3, 100001), (MULTI, 2, 3, 2, 6152),
    (SEQ, 1, 1, 1, 1), (SEQ, 7, 1, 5, 81920),
]


@pytest.mark.parametrize("variant,B,m,k,V", CASES)
@pytest.mark.parametrize("blocks", [1, 2, 7, 300, 768, 1792, 2048, 4096])
@pytest.mark.parametrize("dt", [race.ERSD_F32, race.ERSD_BF16])
def test_partition_invariants(variant, B, m, k, V, blocks, dt):
    d = race.plan_describe(variant, B, m, k, V, blocks, dt)
    G, nslot, S, start = d["G"], d["nslot"], d["seg_cost"], d["block_start"].astype(np.int64)
    kt = k if variant == TREE else k + 1
    mm = m if variant == MULTI else 1
    rows = B * mm * kt
    V8 = (V + 7) // 8
    assert 1 <= G <= blocks and len(start) == G + 1
    assert start[0] == 0 and start[-1] == rows * V8
    assert (np.diff(start) > 0).all()                      # no empty share
    # brute force: which shares overlap each row
    first_bf = np.searchsorted(start, np.arange(rows) * V8, side="right") - 1
    last_bf = np.searchsorted(start, (np.arange(rows) + 1) * V8 - 1, side="right") - 1
    assert np.array_equal(first_bf, d["row_first"].astype(np.int64))
    assert np.array_equal(last_bf, d["row_last"].astype(np.int64))
    assert (last_bf - first_bf + 1).max() <= nslot
    # balance: shares differ by at most one group's worth of cost and two row-start charges (a share boundary may
    # fall inside a charge, which this count gives whole to the share that holds the row's first group)
    assert S <= (32000 if dt == race.ERSD_BF16 else 16000)
    if G > 1:
        kd = k
        def cost(lo, hi):      # cost of global groups [lo, hi)
            c = 0
            pos = lo
            while pos < hi:
                row = pos // V8
                nxt = min(hi, (row + 1) * V8)
                c += (nxt - pos) * (10 if (row % kt) < kd else 5) + (S if pos == row * V8 else 0)
                pos = nxt
            return c
        costs = [cost(int(start[b]), int(start[b + 1])) for b in range(0, G, max(1, G // 50))]
        assert max(costs) - min(costs) <= 22 + 2 * S
        assert S * 2 <= min(costs) + S
    # the workspace covers the slots of any workgroup count the library may choose
    need = race.workspace_bytes(variant, B, m, k, V, race.ERSD_BF16)
    assert need >= rows * 2 * nslot * 80


def test_plan_rejects_bad_arguments():
    L = race.lib()
    import ctypes
    G, ns = ctypes.c_uint32(), ctypes.c_uint32()
    assert L.ersd_plan_describe_host(0, 1, 1, 4, 32000, 0, 0, ctypes.byref(G), ctypes.byref(ns), None, None, None, None) == -2
    assert L.ersd_plan_describe_host(0, 1, 1, 4, 32000, 0, 5000, ctypes.byref(G), ctypes.byref(ns), None, None, None, None) == -2
    assert L.ersd_plan_describe_host(0, 0, 1, 4, 32000, 0, 8, ctypes.byref(G), ctypes.byref(ns), None, None, None, None) == -2
    assert L.ersd_plan_describe_host(0, 1, 1, 4, 32000, 0, 8, None, ctypes.byref(ns), None, None, None, None) == -1
    assert L.ersd_plan_describe_host(0, 1, 1, 4, 32000, 0, 8, ctypes.byref(G), ctypes.byref(ns), None, None, None, None) == 0
    assert G.value >= 1


def _random_tree(rng, N, branching):
    """(parent, rank) with up to `branching` children per context, some nodes malformed on purpose."""
    parent = np.full(N, -1, dtype=np.int32)
    rank = np.zeros(N, dtype=np.int32)
    used = {}
    for n in range(N):
        p = int(rng.integers(-1, n)) if n else -1
        r = used.get(p, 0)
        used[p] = r + 1
        parent[n], rank[n] = p, min(r, 7) if r < branching else int(rng.integers(0, 8))
    for n in rng.integers(0, N, size=max(1, N // 10)):      # malformed entries: parent >= node, rank out of range
        if rng.random() < 0.5:
            parent[n] = int(rng.integers(n, N + 3))
        else:
            rank[n] = int(rng.integers(8, 12))
    return parent, rank


@pytest.mark.parametrize("B,N,V", [(16, 64, 256000), (3, 12, 1000), (1, 1, 8), (2, 700, 4999), (5, 3, 100001),
                                   (4, 2500, 32000)])
@pytest.mark.parametrize("blocks", [1, 2, 7, 300, 768, 4096])
def test_arrival_tree_partition_stays_inside_the_job(oracle_mod, B, N, V, blocks):
    """The arrival tree's partition is evaluated on the device from a weight table that only exists there; here the
    same functions run on the host over a table built from the oracle's reading of the tree (which contexts have
    children), and every share, every row's writers and the slot bound are checked by brute force."""
    rng = np.random.default_rng(N * 131 + B)
    for trial in range(3):
        parent, rank = _random_tree(rng, N, branching=int(rng.integers(1, 5)))
        _, need = oracle_mod.arrival_tree_shape(parent, rank, 8)
        d = race.arrival_plan_describe(B, N, V, need, blocks, race.ERSD_BF16 if trial % 2 else race.ERSD_F32)
        G, nslot, start = d["G"], d["nslot"], d["block_start"].astype(np.int64)
        rows, V8 = B * (N + 1), (V + 7) // 8
        assert 1 <= G <= blocks and len(start) == G + 1
        assert start[0] == 0 and start[-1] == rows * V8 and (np.diff(start) > 0).all()
        first_bf = np.searchsorted(start, np.arange(rows) * V8, side="right") - 1
        last_bf = np.searchsorted(start, (np.arange(rows) + 1) * V8 - 1, side="right") - 1
        assert np.array_equal(first_bf, d["row_first"].astype(np.int64))
        assert np.array_equal(last_bf, d["row_last"].astype(np.int64))
        assert (last_bf - first_bf + 1).max() <= nslot
        # shares cost the same: 10 per group of a context with a draft row, 5 otherwise
        w = np.where(np.tile(need, B) > 0, 10, 5).astype(np.int64)
        cum = np.concatenate([[0], np.cumsum(w * V8)])
        def units(g):           # cost units before global group g
            r = np.minimum(g // V8, rows - 1)
            return np.where(g >= rows * V8, cum[-1], cum[r] + (g - r * V8) * w[r])
        costs = np.diff(units(start))
        assert costs.max() - costs.min() <= 22 + 2 * 8 * 10      # share starts are aligned to 8 (bf16) or 4 groups
        # the workspace covers these slots
        for code in (race.ERSD_F32, race.ERSD_BF16):
            assert race.arrival_tree_workspace_bytes(B, N, V, code) >= rows * (2 * 80 + 272) * nslot
