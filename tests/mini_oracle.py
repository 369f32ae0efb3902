"""Tiny brute-force re-statement of the race in pure Python, for small V only.

Independent of oracle/ (different language, the paper's literal argmin e_i / p_i form with normalised
probabilities instead of the log form) and of the GPU library.  Used to pin the C oracle token by token.
"""
import math

import numpy as np

M0, M1 = 0xD2511F53, 0xCD9E8D57
W0, W1 = 0x9E3779B9, 0xBB67AE85
MASK = 0xFFFFFFFF


def philox4x32(ctr, key, rounds=10):
    c = [int(x) & MASK for x in ctr]
    k = [int(x) & MASK for x in key]
    for r in range(rounds):
        if r:
            k = [(k[0] + W0) & MASK, (k[1] + W1) & MASK]
        a, b = M0 * c[0], M1 * c[2]
        c = [(b >> 32) ^ c[1] ^ k[0], b & MASK, (a >> 32) ^ c[3] ^ k[1], a & MASK]
    return c


def exponentials(V, seed, c1, c2, c3, rounds=7):
    key = (seed & MASK, (seed >> 32) & MASK)
    e = np.empty(V, dtype=np.float64)
    for i in range(V):
        x = philox4x32((i >> 2, c1, c2, c3), key, rounds)[i & 3]
        v = (x + 0.5) / 4294967296.0
        e[i] = -math.log1p(-v)
    return e


def bf16_to_f64(bits_u16):
    return (np.asarray(bits_u16, dtype=np.uint32) << 16).view(np.float32).astype(np.float64)


def race_winner(logits_f64, T, e):
    """argmin_i e_i / p_i with p = softmax(logits / T); first index on ties."""
    z = np.asarray(logits_f64, dtype=np.float64) / float(np.float32(T))
    if np.all(np.isneginf(z)):
        return 0
    p = np.exp(z - z.max())
    p = p / p.sum()
    with np.errstate(divide="ignore"):
        arrival = np.where(p > 0, e / p, np.inf)
    return int(np.argmin(arrival))


def race_verify(draft, target, T, seed, rounds=7):
    """draft [B,k,V], target [B,k+1,V] float64 -> (draft_tokens, target_tokens, accept_len)."""
    B, k, V = draft.shape
    dt = np.zeros((B, k), dtype=np.int32)
    tt = np.zeros((B, k + 1), dtype=np.int32)
    acc = np.zeros(B, dtype=np.int32)
    for b in range(B):
        for j in range(k + 1):
            e = exponentials(V, seed, j, b, 0, rounds)
            if j < k:
                dt[b, j] = race_winner(draft[b, j], T, e)
            tt[b, j] = race_winner(target[b, j], T, e)
        a = 0
        while a < k and dt[b, a] == tt[b, a]:
            a += 1
        acc[b] = a
    return dt, tt, acc


def tree_accept(dtok, ttok, parent):
    """Longest agreeing root path by explicit enumeration of every node's ancestor chain."""
    N = len(parent)
    best_len, best_node = 0, -1
    for n in range(N):
        path, cur, ok = [], n, True
        while cur != -1:
            if not (0 <= cur < N) or (path and cur >= path[-1]):
                ok = False
                break
            path.append(cur)
            cur = parent[cur]
            if cur < -1:
                ok = False
                break
        if ok and all(dtok[x] == ttok[x] for x in path) and len(path) > best_len:
            best_len, best_node = len(path), n
    return best_len, best_node


def arrival_tree(draft, target, parent, rank, T, seed, max_rank=8, rounds=7):
    """Algorithm 5 in its literal form: arrival times e_i / q_i, children = first arrivals under Q.

    draft, target [B,N+1,V] float64 (row c = context c: 0 the partial output, n+1 the path ending at node n).
    -> (draft_tokens [B,N], target_tokens [B,N+1], accept_len [B], accept_node [B], emitted list of lists)
    """
    B, C, V = draft.shape
    N = C - 1
    valid = [False] * N
    for n in range(N):
        p, r = parent[n], rank[n]
        ok = -1 <= p < n and 0 <= r < max_rank and (p == -1 or valid[p])
        ok = ok and not any(valid[o] and parent[o] == p and rank[o] == r for o in range(n))
        valid[n] = ok
    dtok = -np.ones((B, N), dtype=np.int32)
    ttok = np.zeros((B, C), dtype=np.int32)
    acc = np.zeros(B, dtype=np.int32)
    node = -np.ones(B, dtype=np.int32)
    emitted = []
    Tf = float(np.float32(T))
    for b in range(B):
        order = []
        for c in range(C):
            e = exponentials(V, seed, c, b, 0, rounds)
            ttok[b, c] = race_winner(target[b, c], T, e)
            z = np.asarray(draft[b, c], dtype=np.float64) / Tf
            if np.all(np.isneginf(z)):
                order.append([])
                continue
            q = np.exp(z - z.max())
            q = q / q.sum()
            with np.errstate(divide="ignore"):
                t = np.where(q > 0, e / q, np.inf)
            idx = np.argsort(t, kind="stable")
            order.append([int(i) for i in idx if np.isfinite(t[i])])
        for n in range(N):
            if valid[n]:
                o = order[parent[n] + 1]
                dtok[b, n] = o[rank[n]] if rank[n] < len(o) else -1
        ctx, y, last = 0, [], -1
        while True:
            t = int(ttok[b, ctx])
            y.append(t)
            nxt = [n for n in range(N) if valid[n] and parent[n] + 1 == ctx and dtok[b, n] == t]
            if not nxt:
                break
            last = nxt[0]
            ctx = last + 1
        emitted.append(y)
        acc[b] = len(y) - 1
        node[b] = last
    return dtok, ttok, acc, node, emitted
