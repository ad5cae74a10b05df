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


def accept_scan_python(ar_tokens, mask, scaffold, draft, tokens):
    """The accept rule given the verifier's token at every position."""
    N, B = np.asarray(mask).shape
    tokens = np.array(tokens, dtype=np.int32, copy=True)
    mask = np.array(mask, dtype=np.uint8, copy=True)
    accepted = np.zeros((N, B), dtype=np.uint8)
    nacc = np.zeros(N, dtype=np.int32)
    for n in range(N):
        alive = True
        for b in range(B):
            if mask[n, b] != 1 or scaffold[n, b] or not alive:
                continue
            if int(ar_tokens[n, b]) == int(draft[n, b]):
                tokens[n, b] = draft[n, b]
                accepted[n, b] = 1
            else:
                tokens[n, b] = ar_tokens[n, b]
                accepted[n, b] = 2
                alive = False
            mask[n, b] = 0
            nacc[n] += 1
    return dict(tokens=tokens, mask=mask, n_accepted=nacc, accepted=accepted)


# ---- sampled verifier: an independent statement of the sampler in Python -------

def philox4x32_10_python(counter, key):
    """Philox-4x32-10 with Python integers (Salmon et al., SC'11)."""
    c = [int(x) & 0xFFFFFFFF for x in counter]
    k = [int(x) & 0xFFFFFFFF for x in key]
    for _ in range(10):
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [((p1 >> 32) ^ c[1] ^ k[0]) & 0xFFFFFFFF, p1 & 0xFFFFFFFF,
             ((p0 >> 32) ^ c[3] ^ k[1]) & 0xFFFFFFFF, p0 & 0xFFFFFFFF]
        k = [(k[0] + 0x9E3779B9) & 0xFFFFFFFF, (k[1] + 0xBB67AE85) & 0xFFFFFFFF]
    return c


def _fma32(a, b, c):
    # a*b is exact in binary64 for binary32 inputs; the sum is rounded to binary64
    # and then to binary32 (agrees with a fused operation except in rare double roundings)
    return np.float32(np.float64(a) * np.float64(b) + np.float64(c))


_LOG2_POLY = [0.12614846229553223, -0.20742103457450867, 0.21566985547542572, -0.23892034590244293,
              0.2879183292388916, -0.36070483922958374, 0.48091059923171997, -0.7213473320007324,
              1.4426950216293335]


def flog2_python(x):
    x = np.float32(x)
    bits = int(np.frombuffer(np.float32(x).tobytes(), dtype=np.uint32)[0])
    e = ((bits >> 23) & 255) - 127
    m = np.frombuffer(np.uint32((bits & 0x7FFFFF) | 0x3F800000).tobytes(), dtype=np.float32)[0]
    if m > np.float32(1.41421354):
        m = np.float32(m * np.float32(0.5))
        e += 1
    f = np.float32(m - np.float32(1.0))
    p = np.float32(_LOG2_POLY[0])
    for c in _LOG2_POLY[1:]:
        p = _fma32(p, f, np.float32(c))
    return _fma32(f, p, np.float32(e))


def sample_key_python(x, temperature, seed, row, v):
    c = np.float32(1.4426950408889634 / float(np.float32(temperature)))
    r = philox4x32_10_python([v >> 2, row, 0, 0], [seed & 0xFFFFFFFF, seed >> 32])[v & 3]
    u = np.float32((np.float32(r >> 9) + np.float32(0.5)) * np.float32(2.0 ** -23))
    a = np.float32(-flog2_python(u))
    g = np.float32(-flog2_python(a))
    return _fma32(np.float32(x), c, g)
