"""Brute-force references used to pin the oracle (numpy / pure Python only).

These are written independently of ``oracle/``: attention goes through one
explicit boolean visibility matrix over the whole token sequence
(prefix, then every rollout's block), the unmask rule through Python loops.
"""
import math

import numpy as np


def visibility_matrix(N, B, L, causal_block=False):
    """vis[i, j] = may token i attend to token j.

    Token order: L prefix tokens, then rollout 0's block, rollout 1's, ...
    Prefix tokens are causal among themselves (irrelevant to block rows but
    kept so B=1 is the textbook causal matrix).  A block token sees the
    whole prefix and every token of its own rollout's block; nothing else.
    """
    T = L + N * B
    vis = np.zeros((T, T), dtype=bool)
    for i in range(L):
        vis[i, : i + 1] = True
    for n in range(N):
        lo, hi = L + n * B, L + (n + 1) * B
        vis[lo:hi, :L] = True
        vis[lo:hi, lo:hi] = np.tril(np.ones((B, B), dtype=bool)) if causal_block else True
    return vis


def attention_explicit_mask(q, pk, pv, bk, bv, scale, causal_block=False):
    """Dense masked attention over the concatenated sequence, float64."""
    N, B, Hq, D = q.shape
    L, Hkv, _ = pk.shape
    G = Hq // Hkv
    vis = visibility_matrix(N, B, L, causal_block)[L:, :]       # block rows only
    out = np.zeros((N, B, Hq, D))
    for h in range(Hq):
        kh = h // G
        K = np.concatenate([pk[:, kh, :], bk[:, :, kh, :].reshape(N * B, D)], axis=0)
        Vv = np.concatenate([pv[:, kh, :], bv[:, :, kh, :].reshape(N * B, D)], axis=0)
        Q = q[:, :, h, :].reshape(N * B, D)
        S = scale * (Q @ K.T)
        S = np.where(vis, S, -np.inf)
        S = S - S.max(axis=1, keepdims=True)
        P = np.exp(S)
        P = P / P.sum(axis=1, keepdims=True)
        out[:, :, h, :] = (P @ Vv).reshape(N, B, D)
    return out


def unmask_python(logits, mask, scaffold, tokens, tau):
    """The commit rule in plain Python floats (double precision)."""
    N, B, V = logits.shape
    tokens = [list(map(int, row)) for row in tokens]
    mask = [list(map(int, row)) for row in mask]
    conf = [[-math.inf] * B for _ in range(N)]
    nun = [0] * N
    for n in range(N):
        cand = {}
        for b in range(B):
            if mask[n][b] != 1 or scaffold[n][b]:
                continue
            row = [float(x) for x in logits[n, b]]
            mx = max(row)
            arg = row.index(mx)
            z = math.fsum(math.exp(x - mx) for x in row)
            conf[n][b] = 1.0 / z
            cand[b] = arg
        chosen = [b for b in cand if conf[n][b] >= tau]
        if not chosen and cand:
            best = max(conf[n][b] for b in cand)
            chosen = [min(b for b in cand if conf[n][b] == best)]
        for b in chosen:
            tokens[n][b] = cand[b]
            mask[n][b] = 0
        nun[n] = len(chosen)
    return np.array(tokens, dtype=np.int32), np.array(mask, dtype=np.uint8), np.array(conf), np.array(nun, dtype=np.int32)


def verify_python(ar_logits, mask, scaffold, draft, tokens):
    """Accept scan of scaffold speculative decoding in plain Python."""
    N, B, V = ar_logits.shape
    tokens = [list(map(int, r)) for r in tokens]
    mask = [list(map(int, r)) for r in mask]
    nacc = [0] * N
    for n in range(N):
        alive = True
        for b in range(B):
            if mask[n][b] != 1 or scaffold[n][b]:
                continue                     # scaffold / already visible: auto-accepted, not verified
            if not alive:
                continue                     # discarded draft stays masked
            row = [float(x) for x in ar_logits[n, b]]
            ar = row.index(max(row))
            if ar == int(draft[n][b]):
                tokens[n][b] = int(draft[n][b])
            else:
                tokens[n][b] = ar
                alive = False
            mask[n][b] = 0
            nacc[n] += 1
    return np.array(tokens, dtype=np.int32), np.array(mask, dtype=np.uint8), np.array(nacc, dtype=np.int32)
