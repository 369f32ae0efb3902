"""ctypes front end of the fp64 CPU oracle (oracle/ersd_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
CPU-baseline leg of bench.py.  The GPU library never imports or links this.

Logit arrays are host arrays: numpy float32, numpy uint16 holding bfloat16 bit
patterns, or CPU torch tensors of dtype float32 / bfloat16.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

F32, BF16 = 0, 1


class RowInfo(ctypes.Structure):
    _fields_ = [
        ("token", ctypes.c_int32),
        ("runner_up", ctypes.c_int32),
        ("s1", ctypes.c_double),
        ("s2", ctypes.c_double),
        ("near_tie", ctypes.c_int32),
        ("exact_tie", ctypes.c_int32),
    ]


ROW_INFO_DTYPE = np.dtype(
    [("token", "<i4"), ("runner_up", "<i4"), ("s1", "<f8"), ("s2", "<f8"), ("near_tie", "<i4"), ("exact_tie", "<i4")],
    align=True,
)
assert ROW_INFO_DTYPE.itemsize == ctypes.sizeof(RowInfo)


def lib():
    global _LIB
    if _LIB is None:
        path = _build.LIB
        if not os.path.exists(path):
            path = _build.build()
        L = ctypes.CDLL(path)
        vp, i32, i64, u32, u64, f32 = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_uint32,
                                       ctypes.c_uint64, ctypes.c_float)
        L.oracle_philox4x32.argtypes = [ctypes.c_int, vp, vp, vp]
        L.oracle_philox4x32.restype = None
        L.oracle_set_rounds.argtypes = [ctypes.c_int]
        L.oracle_get_rounds.restype = ctypes.c_int
        L.oracle_exponential.argtypes = [u32]
        L.oracle_exponential.restype = ctypes.c_double
        L.oracle_gumbel.argtypes = [u32]
        L.oracle_gumbel.restype = ctypes.c_double
        L.oracle_race_rows.argtypes = [vp, ctypes.c_int, i64, f32, u64, u32, u32, u32, vp]
        L.oracle_race_rows.restype = None
        L.oracle_row_candidates.argtypes = [vp, ctypes.c_int, i64, f32, u64, u32, u32, u32, ctypes.c_double, vp, i64]
        L.oracle_row_candidates.restype = i64
        L.oracle_race_sample.argtypes = [vp, ctypes.c_int, i32, i32, i32, i64, i32, f32, u64, vp, vp]
        L.oracle_race_sample.restype = ctypes.c_int
        L.oracle_race_verify.argtypes = [vp, vp, ctypes.c_int, i32, i32, i64, f32, u64, vp, vp, vp, vp, vp]
        L.oracle_race_verify.restype = ctypes.c_int
        L.oracle_race_verify_multi.argtypes = [vp, vp, ctypes.c_int, i32, i32, i32, i64, f32, u64,
                                               vp, vp, vp, vp, vp, vp, vp]
        L.oracle_race_verify_multi.restype = ctypes.c_int
        L.oracle_race_verify_tree.argtypes = [vp, vp, ctypes.c_int, i32, i32, i64, vp, f32, u64,
                                              vp, vp, vp, vp, vp, vp]
        L.oracle_race_verify_tree.restype = ctypes.c_int
        L.oracle_race_verify_arrival_tree.argtypes = [vp, vp, ctypes.c_int, i32, i32, i64, vp, vp, i32, f32, u64,
                                                      vp, vp, vp, vp, vp, vp, vp, vp]
        L.oracle_race_verify_arrival_tree.restype = ctypes.c_int
        L.oracle_arrival_tree_shape.argtypes = [vp, vp, i32, i32, vp, vp]
        L.oracle_arrival_tree_shape.restype = None
        L.oracle_gsd_verify.argtypes = [vp, vp, ctypes.c_int, i32, i32, i64, vp, f32, u64, vp, vp, vp, ctypes.c_double,
                                        ctypes.c_double]
        L.oracle_gsd_verify.restype = ctypes.c_int
        L.oracle_gsd_verify_tree.argtypes = [vp, vp, ctypes.c_int, i32, i32, i64, vp, vp, i32, vp, f32, u64, vp, vp, vp,
                                             vp, ctypes.c_double, ctypes.c_double]
        L.oracle_gsd_verify_tree.restype = ctypes.c_int
        L.oracle_gsd_uniform_ctr.argtypes = [u64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32]
        L.oracle_gsd_uniform_ctr.restype = ctypes.c_double
        L.oracle_logsumexp.argtypes = [vp, ctypes.c_int, i64, f32]
        L.oracle_logsumexp.restype = ctypes.c_double
        L.oracle_gsd_uniform.argtypes = [u64, u32, u32]
        L.oracle_gsd_uniform.restype = ctypes.c_double
        L.oracle_num_threads.restype = ctypes.c_int
        L.oracle_set_num_threads.argtypes = [ctypes.c_int]
        _LIB = L
    return _LIB


def _host(a):
    """-> (contiguous numpy array kept alive, dtype code)."""
    try:
        import torch
        if isinstance(a, torch.Tensor):
            assert a.device.type == "cpu", "the oracle takes host tensors"
            a = a.contiguous()
            if a.dtype == torch.bfloat16:
                return a.view(torch.int16).numpy().view(np.uint16), BF16
            if a.dtype == torch.float32:
                return a.numpy(), F32
            raise TypeError(f"unsupported dtype {a.dtype}")
    except ImportError:
        pass
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    raise TypeError(f"unsupported dtype {a.dtype}")


def _ptr(a):
    return ctypes.c_void_p(a.ctypes.data)


def philox4x32(ctr, key, rounds=10):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().oracle_philox4x32(rounds, _ptr(c), _ptr(k), _ptr(out))
    return out


def set_rounds(r):
    lib().oracle_set_rounds(int(r))


def get_rounds():
    return lib().oracle_get_rounds()


def exponential(x):
    return lib().oracle_exponential(int(x))


def gumbel(x):
    return lib().oracle_gumbel(int(x))


def num_threads():
    return lib().oracle_num_threads()


def set_num_threads(n):
    lib().oracle_set_num_threads(int(n))


def race_rows(draft_row, target_row, temperature, seed, c1=0, c2=0, c3=0):
    """One race shared by an optional draft row and an optional target row -> info records (numpy struct [2])."""
    rows = (ctypes.c_void_p * 2)()
    keep = []
    dt = None
    V = None
    for s, r in enumerate((draft_row, target_row)):
        if r is None:
            rows[s] = None
            continue
        a, d = _host(r)
        assert a.ndim == 1
        assert dt in (None, d) and V in (None, a.shape[0])
        dt, V = d, a.shape[0]
        keep.append(a)
        rows[s] = a.ctypes.data
    info = np.zeros(2, dtype=ROW_INFO_DTYPE)
    lib().oracle_race_rows(rows, dt, V, float(temperature), int(seed), int(c1), int(c2), int(c3), _ptr(info))
    return info


def row_candidates(row, temperature, seed, c1=0, c2=0, c3=0, tol_rel=1e-6, cap=4096):
    a, d = _host(row)
    out = np.zeros(cap, dtype=np.int32)
    n = lib().oracle_row_candidates(_ptr(a), d, a.shape[0], float(temperature), int(seed), int(c1), int(c2), int(c3),
                                    float(tol_rel), _ptr(out), cap)
    return out[: min(n, cap)], n


def race_sample(logits, pos0, temperature, seed, want_info=False):
    """One model's races.  logits [B,m,npos,V] -> tokens [B,m,npos] (and the row records)."""
    a, dt = _host(logits)
    B, m, npos, V = a.shape
    tok = np.zeros((B, m, npos), dtype=np.int32)
    info = np.zeros((B, m, npos), dtype=ROW_INFO_DTYPE) if want_info else None
    rc = lib().oracle_race_sample(_ptr(a), dt, B, m, npos, V, int(pos0), float(temperature), int(seed), _ptr(tok),
                                  _ptr(info) if want_info else None)
    if rc != 0:
        raise ValueError("oracle_race_sample: invalid arguments")
    return (tok, info) if want_info else tok


def race_verify(draft, target, temperature, seed, want_info=False):
    """draft [B,k,V], target [B,k+1,V] -> dict(draft_tokens, target_tokens, accept_len[, draft_info, target_info])."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, k, V = d.shape
    assert t.shape == (B, k + 1, V)
    dtok = np.zeros((B, k), dtype=np.int32)
    ttok = np.zeros((B, k + 1), dtype=np.int32)
    acc = np.zeros(B, dtype=np.int32)
    di = np.zeros((B, k), dtype=ROW_INFO_DTYPE) if want_info else None
    ti = np.zeros((B, k + 1), dtype=ROW_INFO_DTYPE) if want_info else None
    rc = lib().oracle_race_verify(_ptr(d), _ptr(t), dt, B, k, V, float(temperature), int(seed), _ptr(dtok), _ptr(ttok),
                                  _ptr(acc), _ptr(di) if want_info else None, _ptr(ti) if want_info else None)
    if rc != 0:
        raise ValueError("oracle_race_verify: invalid arguments")
    out = dict(draft_tokens=dtok, target_tokens=ttok, accept_len=acc)
    if want_info:
        out.update(draft_info=di, target_info=ti)
    return out


def race_verify_multi(draft, target, temperature, seed, want_info=False):
    """draft [B,m,k,V], target [B,m,k+1,V]."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, m, k, V = d.shape
    assert t.shape == (B, m, k + 1, V)
    dtok = np.zeros((B, m, k), dtype=np.int32)
    ttok = np.zeros((B, m, k + 1), dtype=np.int32)
    acc = np.zeros((B, m), dtype=np.int32)
    bd = np.zeros(B, dtype=np.int32)
    bl = np.zeros(B, dtype=np.int32)
    di = np.zeros((B, m, k), dtype=ROW_INFO_DTYPE) if want_info else None
    ti = np.zeros((B, m, k + 1), dtype=ROW_INFO_DTYPE) if want_info else None
    rc = lib().oracle_race_verify_multi(_ptr(d), _ptr(t), dt, B, m, k, V, float(temperature), int(seed), _ptr(dtok),
                                        _ptr(ttok), _ptr(acc), _ptr(bd), _ptr(bl),
                                        _ptr(di) if want_info else None, _ptr(ti) if want_info else None)
    if rc != 0:
        raise ValueError("oracle_race_verify_multi: invalid arguments")
    out = dict(draft_tokens=dtok, target_tokens=ttok, accept_len=acc, best_draft=bd, best_len=bl)
    if want_info:
        out.update(draft_info=di, target_info=ti)
    return out


def race_verify_tree(draft, target, parent, temperature, seed, want_info=False):
    """draft, target [B,N,V]; parent int32 [N]."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, N, V = d.shape
    assert t.shape == (B, N, V)
    par = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    assert par.shape == (N,)
    dtok = np.zeros((B, N), dtype=np.int32)
    ttok = np.zeros((B, N), dtype=np.int32)
    acc = np.zeros(B, dtype=np.int32)
    node = np.zeros(B, dtype=np.int32)
    di = np.zeros((B, N), dtype=ROW_INFO_DTYPE) if want_info else None
    ti = np.zeros((B, N), dtype=ROW_INFO_DTYPE) if want_info else None
    rc = lib().oracle_race_verify_tree(_ptr(d), _ptr(t), dt, B, N, V, _ptr(par), float(temperature), int(seed),
                                       _ptr(dtok), _ptr(ttok), _ptr(acc), _ptr(node),
                                       _ptr(di) if want_info else None, _ptr(ti) if want_info else None)
    if rc != 0:
        raise ValueError("oracle_race_verify_tree: invalid arguments")
    out = dict(draft_tokens=dtok, target_tokens=ttok, accept_len=acc, accept_node=node)
    if want_info:
        out.update(draft_info=di, target_info=ti)
    return out


def arrival_tree_shape(parent, rank, max_rank=8):
    """-> (valid [N], need [N+1]) of a (parent, rank) tree."""
    par = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    rk = np.ascontiguousarray(np.asarray(rank, dtype=np.int32))
    N = par.shape[0]
    valid = np.zeros(N, dtype=np.int32)
    need = np.zeros(N + 1, dtype=np.int32)
    lib().oracle_arrival_tree_shape(_ptr(par), _ptr(rk), N, int(max_rank), _ptr(valid), _ptr(need))
    return valid, need


def race_verify_arrival_tree(draft, target, parent, rank, temperature, seed, max_rank=8, want_info=False):
    """Algorithm 5: draft, target [B,N+1,V] (one row per context); parent, rank int32 [N]."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, C, V = d.shape
    N = C - 1
    assert t.shape == (B, C, V)
    par = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    rk = np.ascontiguousarray(np.asarray(rank, dtype=np.int32))
    assert par.shape == (N,) and rk.shape == (N,)
    arr = np.zeros((B, C, max_rank), dtype=np.int32)
    dtok = np.zeros((B, N), dtype=np.int32)
    ttok = np.zeros((B, C), dtype=np.int32)
    acc = np.zeros(B, dtype=np.int32)
    node = np.zeros(B, dtype=np.int32)
    emitted = np.zeros((B, C), dtype=np.int32)
    near = np.zeros((B, C), dtype=np.int32) if want_info else None
    ti = np.zeros((B, C), dtype=ROW_INFO_DTYPE) if want_info else None
    rc = lib().oracle_race_verify_arrival_tree(_ptr(d), _ptr(t), dt, B, N, V, _ptr(par), _ptr(rk), int(max_rank),
                                               float(temperature), int(seed), _ptr(arr), _ptr(dtok), _ptr(ttok),
                                               _ptr(acc), _ptr(node), _ptr(emitted),
                                               _ptr(near) if want_info else None, _ptr(ti) if want_info else None)
    if rc != 0:
        raise ValueError("oracle_race_verify_arrival_tree: invalid arguments")
    out = dict(arrivals=arr, draft_tokens=dtok, target_tokens=ttok, accept_len=acc, accept_node=node, emitted=emitted)
    if want_info:
        out.update(arrival_near_tie=near, target_info=ti)
    return out


GSD_INFO_DTYPE = np.dtype([("near_accept", "<i4"), ("rivals", "<i4"), ("lse_p", "<f8"), ("lse_q", "<f8"),
                           ("score", "<f8"), ("min_accept_gap", "<f8")], align=True)


def logsumexp(row, temperature):
    a, d = _host(row)
    return lib().oracle_logsumexp(_ptr(a), d, a.shape[0], float(temperature))


def gsd_uniform(seed, j, b):
    return lib().oracle_gsd_uniform(int(seed), int(j), int(b))


def gsd_verify(draft, target, draft_tokens, temperature, seed, want_info=False, accept_rel_tol=0.0,
               weight_rel_tol=0.0):
    """GSD sequence verification: draft [B,k,V], target [B,k+1,V], draft_tokens [B,k] -> dict(accept_len, next_token).
    The two tolerances only shape the sensitivity report in `info` (near_accept, rivals), never the results."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, k, V = d.shape
    assert t.shape == (B, k + 1, V)
    tok = np.ascontiguousarray(np.asarray(draft_tokens, dtype=np.int32))
    assert tok.shape == (B, k)
    acc = np.zeros(B, dtype=np.int32)
    nxt = np.zeros(B, dtype=np.int32)
    info = np.zeros(B, dtype=GSD_INFO_DTYPE) if want_info else None
    rc = lib().oracle_gsd_verify(_ptr(d), _ptr(t), dt, B, k, V, _ptr(tok), float(temperature), int(seed), _ptr(acc),
                                 _ptr(nxt), _ptr(info) if want_info else None, float(accept_rel_tol),
                                 float(weight_rel_tol))
    if rc != 0:
        raise ValueError("oracle_gsd_verify: invalid arguments")
    out = dict(accept_len=acc, next_token=nxt)
    if want_info:
        out["info"] = info
    return out


def gsd_uniform_ctr(seed, r, j, b):
    return lib().oracle_gsd_uniform_ctr(int(seed), int(r), int(j), int(b))


def gsd_verify_tree(draft, target, parent, rank, draft_tokens, temperature, seed, max_rank=8, want_info=False,
                    accept_rel_tol=0.0, weight_rel_tol=0.0):
    """GSD on a draft tree (Algorithm 4's verification): draft, target [B,N+1,V]; parent, rank int32 [N];
    draft_tokens [B,N] -> dict(accept_len, accept_node, emitted [B,N+1])."""
    d, dt = _host(draft)
    t, dt2 = _host(target)
    assert dt == dt2
    B, C, V = d.shape
    N = C - 1
    assert t.shape == (B, C, V)
    par = np.ascontiguousarray(np.asarray(parent, dtype=np.int32))
    rk = np.ascontiguousarray(np.asarray(rank, dtype=np.int32))
    tok = np.ascontiguousarray(np.asarray(draft_tokens, dtype=np.int32))
    assert par.shape == (N,) and rk.shape == (N,) and tok.shape == (B, N)
    acc = np.zeros(B, dtype=np.int32)
    node = np.zeros(B, dtype=np.int32)
    emitted = np.zeros((B, C), dtype=np.int32)
    info = np.zeros(B, dtype=GSD_INFO_DTYPE) if want_info else None
    rc = lib().oracle_gsd_verify_tree(_ptr(d), _ptr(t), dt, B, N, V, _ptr(par), _ptr(rk), int(max_rank), _ptr(tok),
                                      float(temperature), int(seed), _ptr(acc), _ptr(node), _ptr(emitted),
                                      _ptr(info) if want_info else None, float(accept_rel_tol), float(weight_rel_tol))
    if rc != 0:
        raise ValueError("oracle_gsd_verify_tree: invalid arguments")
    out = dict(accept_len=acc, accept_node=node, emitted=emitted)
    if want_info:
        out["info"] = info
    return out
