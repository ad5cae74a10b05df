"""Pins for the oracle's three-run attention (shared prefix, per-rollout
extension, live block) and for the block commit (CPU only).

What fixes the expected values: "a block attends ... causally to the prompt
and all earlier blocks" (paper, "Block-Causal Diffusion"), and "fork the KV
cache N times" and continue the trajectory section N times (paper, "Shared
prefix"): after the fork, the blocks a rollout finishes are its own.
"""
import numpy as np
import pytest
import torch

from tests import brute


def rand(rng, N, B, L, E, Ecap, Hq, Hkv, D):
    f = lambda *s: rng.standard_normal(s)
    return dict(q=f(N, B, Hq, D), pk=f(L, Hkv, D), pv=f(L, Hkv, D), ek=f(N, Ecap, Hkv, D), ev=f(N, Ecap, Hkv, D),
                bk=f(N, B, Hkv, D), bv=f(N, B, Hkv, D))


CASES = [(1, 4, 7, 3, 5, 2, 1, 8), (3, 5, 11, 10, 10, 6, 2, 16), (2, 1, 0, 6, 9, 4, 4, 8), (4, 3, 5, 1, 4, 3, 1, 4)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("N,B,L,E,Ecap,Hq,Hkv,D", CASES)
def test_extension_is_a_private_continuation_of_the_prefix(oracle, N, B, L, E, Ecap, Hq, Hkv, D, causal):
    # rollout n alone, with [prefix ; its extension] as an ordinary prefix, must give the same rows
    rng = np.random.default_rng(N * 1000 + B * 10 + E)
    d = rand(rng, N, B, L, E, Ecap, Hq, Hkv, D)
    d["ek"][:, E:] = np.nan           # rows beyond E do not exist
    d["ev"][:, E:] = np.nan
    got = oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"], scale=0.41, causal_block=causal,
                            ext_k=d["ek"], ext_v=d["ev"], E=E)
    for n in range(N):
        pk = np.concatenate([d["pk"], d["ek"][n, :E]], axis=0)
        pv = np.concatenate([d["pv"], d["ev"][n, :E]], axis=0)
        want = oracle.block_attn(d["q"][n:n + 1], pk, pv, d["bk"][n:n + 1], d["bv"][n:n + 1], scale=0.41, causal_block=causal)
        np.testing.assert_allclose(got[n:n + 1], want, rtol=0, atol=1e-12)


def test_matches_explicit_mask_over_the_whole_sequence(oracle):
    # one dense masked attention over [prefix ; every extension ; every block], mask built here
    rng = np.random.default_rng(5)
    N, B, L, E, Ecap, Hq, Hkv, D = 3, 4, 6, 5, 7, 4, 2, 8
    d = rand(rng, N, B, L, E, Ecap, Hq, Hkv, D)
    scale = 0.3
    got = oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"], scale=scale, ext_k=d["ek"], ext_v=d["ev"], E=E)
    T = L + N * E + N * B
    vis = np.zeros((N * B, T), dtype=bool)
    for n in range(N):
        rows = slice(n * B, (n + 1) * B)
        vis[rows, :L] = True
        vis[rows, L + n * E: L + (n + 1) * E] = True
        vis[rows, L + N * E + n * B: L + N * E + (n + 1) * B] = True
    G = Hq // Hkv
    for h in range(Hq):
        kh = h // G
        K = np.concatenate([d["pk"][:, kh], d["ek"][:, :E, kh].reshape(N * E, D), d["bk"][:, :, kh].reshape(N * B, D)])
        V = np.concatenate([d["pv"][:, kh], d["ev"][:, :E, kh].reshape(N * E, D), d["bv"][:, :, kh].reshape(N * B, D)])
        Q = torch.from_numpy(d["q"][:, :, h].reshape(1, 1, N * B, D))
        want = torch.nn.functional.scaled_dot_product_attention(
            Q, torch.from_numpy(K)[None, None], torch.from_numpy(V)[None, None],
            attn_mask=torch.from_numpy(vis)[None, None], scale=scale)[0, 0].numpy()
        np.testing.assert_allclose(got[:, :, h].reshape(N * B, D), want, rtol=0, atol=1e-12)


def test_three_chained_blocks_are_block_causal_attention(oracle):
    # Decode three blocks per rollout after the fork, committing each.  The rows of the third
    # block must equal block-causal attention over [prefix, block 1, block 2, block 3] of that
    # rollout, written as textbook masked attention with the block-causal mask of the sequence.
    rng = np.random.default_rng(9)
    N, B, L, Hq, Hkv, D = 2, 3, 5, 2, 1, 8
    f = lambda *s: rng.standard_normal(s)
    pk, pv = f(L, Hkv, D), f(L, Hkv, D)
    blocks_k = [f(N, B, Hkv, D) for _ in range(3)]
    blocks_v = [f(N, B, Hkv, D) for _ in range(3)]
    q3 = f(N, B, Hq, D)
    ek, ev = np.full((N, 2 * B, Hkv, D), np.nan), np.full((N, 2 * B, Hkv, D), np.nan)
    ek, ev = oracle.block_commit(blocks_k[0], blocks_v[0], ek, ev, 0)
    ek, ev = oracle.block_commit(blocks_k[1], blocks_v[1], ek, ev, B)
    got = oracle.block_attn(q3, pk, pv, blocks_k[2], blocks_v[2], scale=0.5, ext_k=ek, ext_v=ev, E=2 * B)
    T = L + 3 * B
    blk = np.concatenate([np.zeros(L, dtype=int), 1 + np.repeat(np.arange(3), B)])     # block id of each token; prefix = 0
    causal = np.tril(np.ones((T, T), dtype=bool))
    vis = causal | (blk[:, None] == blk[None, :]) & (blk[:, None] > 0)                  # bidirectional inside a block
    for n in range(N):
        K = np.concatenate([pk[:, 0]] + [bk[n, :, 0] for bk in blocks_k])
        V = np.concatenate([pv[:, 0]] + [bv[n, :, 0] for bv in blocks_v])
        for h in range(Hq):
            S = 0.5 * (q3[n, :, h] @ K.T)
            S = np.where(vis[L + 2 * B:], S, -np.inf)
            P = np.exp(S - S.max(1, keepdims=True))
            P /= P.sum(1, keepdims=True)
            np.testing.assert_allclose(got[n, :, h], P @ V, rtol=0, atol=1e-12)


def test_other_rollouts_extensions_are_invisible_and_e0_ignores_them(oracle):
    rng = np.random.default_rng(2)
    N, B, L, E, Ecap, Hq, Hkv, D = 3, 4, 6, 4, 4, 2, 2, 8
    d = rand(rng, N, B, L, E, Ecap, Hq, Hkv, D)
    base = oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"], ext_k=d["ek"], ext_v=d["ev"], E=E)
    ek2, ev2 = d["ek"].copy(), d["ev"].copy()
    ek2[1] += 3.0
    ev2[1] -= 2.0
    moved = oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"], ext_k=ek2, ext_v=ev2, E=E)
    assert np.array_equal(base[0], moved[0]) and np.array_equal(base[2], moved[2])
    assert not np.allclose(base[1], moved[1])
    plain = oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"])
    assert np.array_equal(plain, oracle.block_attn(d["q"], d["pk"], d["pv"], d["bk"], d["bv"], ext_k=d["ek"], ext_v=d["ev"], E=0))
    assert not np.allclose(plain, base)


def test_block_commit_is_a_copy_into_rows_e_to_e_plus_b(oracle):
    rng = np.random.default_rng(4)
    N, B, Ecap, Hkv, D = 3, 4, 11, 2, 8
    for dtype in (np.float64, np.float32, np.uint16):
        bk = (rng.standard_normal((N, B, Hkv, D)) * 100).astype(dtype)
        bv = (rng.standard_normal((N, B, Hkv, D)) * 100).astype(dtype)
        ek = (rng.standard_normal((N, Ecap, Hkv, D)) * 100).astype(dtype)
        ev = (rng.standard_normal((N, Ecap, Hkv, D)) * 100).astype(dtype)
        for E in (0, 3, 7):
            k2, v2 = oracle.block_commit(bk, bv, ek, ev, E)
            wk, wv = ek.copy(), ev.copy()
            wk[:, E:E + B] = bk
            wv[:, E:E + B] = bv
            assert np.array_equal(k2, wk) and np.array_equal(v2, wv)
    with pytest.raises(ValueError):
        oracle.block_commit(bk, bv, ek, ev, 8)      # 8 + 4 > 11
