"""Pins for the fp64 attention oracle (CPU only).

Each test checks the oracle against something fixed by the paper's attention
rule (Preliminaries, "Block-Causal Diffusion"; "Shared prefix" paragraph) or
by mathematics, through code that does not live in ``oracle/``.
"""
import numpy as np
import pytest
import torch

from tests import brute


def rand_inputs(rng, N, B, L, Hq, Hkv, D, std=1.0):
    f = lambda *s: rng.standard_normal(s) * std
    return f(N, B, Hq, D), f(L, Hkv, D), f(L, Hkv, D), f(N, B, Hkv, D), f(N, B, Hkv, D)


@pytest.mark.parametrize("N,B,L,Hq,Hkv,D", [(1, 4, 7, 2, 1, 8), (3, 5, 11, 6, 2, 16), (2, 1, 9, 4, 4, 8),
                                            (4, 3, 0, 3, 1, 4), (2, 8, 33, 7, 1, 32)])
def test_matches_explicit_mask_brute_force(oracle, N, B, L, Hq, Hkv, D):
    rng = np.random.default_rng(N * 100 + B)
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, L, Hq, Hkv, D)
    scale = 0.37
    got = oracle.block_attn(q, pk, pv, bk, bv, scale=scale)
    want = brute.attention_explicit_mask(q, pk, pv, bk, bv, scale)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)


def test_visibility_matrix_is_block_causal():
    # the brute force's own mask: own block bidirectional, prefix visible,
    # other rollouts' blocks and nothing "later" visible
    vis = brute.visibility_matrix(N=2, B=3, L=2)
    r0 = vis[2]          # first token of rollout 0
    assert r0.tolist() == [True, True, True, True, True, False, False, False]
    r1 = vis[7]          # last token of rollout 1
    assert r1.tolist() == [True, True, False, False, False, True, True, True]


def test_b1_is_ordinary_causal_attention(oracle):
    # B=1: the block row is the last row of textbook causal attention over
    # the (L+1)-token sequence [prefix ; block]
    rng = np.random.default_rng(1)
    L, H, D = 13, 2, 8
    q, pk, pv, bk, bv = rand_inputs(rng, 1, 1, L, H, H, D)
    got = oracle.block_attn(q, pk, pv, bk, bv)
    K = torch.from_numpy(np.concatenate([pk, bk[0]], 0)).permute(1, 0, 2)      # [H, L+1, D]
    V = torch.from_numpy(np.concatenate([pv, bv[0]], 0)).permute(1, 0, 2)
    # queries for the earlier positions are arbitrary; only the last row is compared
    Q = torch.from_numpy(np.concatenate([rng.standard_normal((L, H, D)), q[0]], 0)).permute(1, 0, 2)
    ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
    np.testing.assert_allclose(got[0, 0], ref[:, -1, :].numpy(), atol=1e-12)


def test_matches_library_attention_with_explicit_mask(oracle):
    # shared prefix == per-rollout copied prefix, via a library routine:
    # each rollout alone is full attention over its own copy of [prefix ; block]
    rng = np.random.default_rng(2)
    N, B, L, Hq, Hkv, D = 3, 4, 10, 4, 2, 16
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, L, Hq, Hkv, D)
    got = oracle.block_attn(q, pk, pv, bk, bv)
    G = Hq // Hkv
    for n in range(N):
        K = torch.from_numpy(np.concatenate([pk.copy(), bk[n]], 0)).permute(1, 0, 2).repeat_interleave(G, 0)
        V = torch.from_numpy(np.concatenate([pv.copy(), bv[n]], 0)).permute(1, 0, 2).repeat_interleave(G, 0)
        Q = torch.from_numpy(q[n]).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V)       # no mask: all L+B visible
        np.testing.assert_allclose(got[n], ref.permute(1, 0, 2).numpy(), atol=1e-12)


def test_shared_prefix_equals_single_rollout_calls(oracle):
    rng = np.random.default_rng(3)
    q, pk, pv, bk, bv = rand_inputs(rng, 4, 3, 6, 4, 2, 8)
    got = oracle.block_attn(q, pk, pv, bk, bv)
    for n in range(4):
        one = oracle.block_attn(q[n:n + 1], pk, pv, bk[n:n + 1], bv[n:n + 1])
        np.testing.assert_array_equal(got[n], one[0])


def test_identical_forked_rollouts_give_identical_outputs(oracle):
    rng = np.random.default_rng(4)
    q, pk, pv, bk, bv = rand_inputs(rng, 1, 5, 9, 4, 2, 8)
    N = 4
    rep = lambda a: np.repeat(a, N, axis=0)
    got = oracle.block_attn(rep(q), pk, pv, rep(bk), rep(bv))
    for n in range(1, N):
        np.testing.assert_array_equal(got[n], got[0])


def test_permuting_rollouts_permutes_outputs(oracle):
    rng = np.random.default_rng(5)
    q, pk, pv, bk, bv = rand_inputs(rng, 4, 3, 6, 2, 1, 8)
    perm = np.array([2, 0, 3, 1])
    a = oracle.block_attn(q, pk, pv, bk, bv)
    b = oracle.block_attn(q[perm], pk, pv, bk[perm], bv[perm])
    np.testing.assert_array_equal(a[perm], b)


def test_other_rollouts_blocks_are_invisible(oracle):
    rng = np.random.default_rng(6)
    q, pk, pv, bk, bv = rand_inputs(rng, 3, 4, 5, 2, 2, 8)
    a = oracle.block_attn(q, pk, pv, bk, bv)
    bk2, bv2 = bk.copy(), bv.copy()
    bk2[1] += 5.0
    bv2[1] -= 3.0
    b = oracle.block_attn(q, pk, pv, bk2, bv2)
    np.testing.assert_array_equal(a[[0, 2]], b[[0, 2]])
    assert np.abs(a[1] - b[1]).max() > 1e-3


def test_no_prefix_is_bidirectional_block_attention(oracle):
    rng = np.random.default_rng(7)
    N, B, H, D = 2, 6, 2, 8
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, 0, H, H, D)
    got = oracle.block_attn(q, pk, pv, bk, bv)
    for n in range(N):
        Q, K, V = (torch.from_numpy(x[n]).permute(1, 0, 2) for x in (q, bk, bv))
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V)
        np.testing.assert_allclose(got[n], ref.permute(1, 0, 2).numpy(), atol=1e-12)
    # B=1, L=0: softmax over one key is 1, so out = v exactly
    one = oracle.block_attn(q[:, :1], pk, pv, bk[:, :1], bv[:, :1])
    np.testing.assert_allclose(one, bv[:, :1], atol=1e-15)


def test_closed_forms(oracle):
    rng = np.random.default_rng(8)
    N, B, L, H, D = 2, 3, 7, 2, 4
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, L, H, H, D)
    # all keys equal -> uniform weights -> mean of the L+B visible value rows
    pk1 = np.broadcast_to(pk[:1], pk.shape).copy()
    bk1 = np.broadcast_to(pk[:1][None], bk.shape).copy()
    got = oracle.block_attn(q, pk1, pv, bk1, bv)
    for n in range(N):
        mean = (pv.sum(0) + bv[n].sum(0)) / (L + B)                    # [H, D]
        np.testing.assert_allclose(got[n], np.broadcast_to(mean, (B, H, D)), atol=1e-13)
    # V constant -> out constant
    got = oracle.block_attn(q, pk, np.full_like(pv, 2.5), bk, np.full_like(bv, 2.5))
    np.testing.assert_allclose(got, 2.5, atol=1e-13)
    # one prefix key with a huge score takes all the weight
    pk2 = pk.copy()
    qq = np.ones_like(q)
    pk2[:] = 0.0
    pk2[3] = 50.0
    got = oracle.block_attn(qq, pk2, pv, np.zeros_like(bk), bv, scale=1.0)
    np.testing.assert_allclose(got, np.broadcast_to(pv[3], got.shape), atol=1e-13)
    # scaling q by c with scale/c leaves the result unchanged; a key transposed
    # with a value (wrong operand) would not
    a = oracle.block_attn(q, pk, pv, bk, bv, scale=0.5)
    b = oracle.block_attn(q * 4.0, pk, pv, bk, bv, scale=0.125)
    np.testing.assert_allclose(a, b, atol=1e-13)


def test_default_scale_is_inverse_sqrt_d(oracle):
    rng = np.random.default_rng(9)
    q, pk, pv, bk, bv = rand_inputs(rng, 1, 2, 5, 2, 1, 16)
    np.testing.assert_array_equal(oracle.block_attn(q, pk, pv, bk, bv),
                                  oracle.block_attn(q, pk, pv, bk, bv, scale=0.25))


def test_gqa_head_mapping(oracle):
    # query head h uses KV head h // (Hq/Hkv): changing KV head 1 only
    # changes query heads G..2G-1
    rng = np.random.default_rng(10)
    q, pk, pv, bk, bv = rand_inputs(rng, 1, 2, 5, 6, 3, 8)
    a = oracle.block_attn(q, pk, pv, bk, bv)
    pv2 = pv.copy()
    pv2[:, 1] += 1.0
    b = oracle.block_attn(q, pk, pv2, bk, bv)
    changed = [h for h in range(6) if np.abs(a[:, :, h] - b[:, :, h]).max() > 0]
    assert changed == [2, 3]


def test_row_subset_and_storage_types(oracle):
    import fdd_workloads as W
    rng = np.random.default_rng(11)
    q, pk, pv, bk, bv = (x.astype(np.float32) for x in rand_inputs(rng, 2, 3, 6, 4, 2, 8))
    full = oracle.block_attn(*(x.astype(np.float64) for x in (q, pk, pv, bk, bv)))
    np.testing.assert_array_equal(full, oracle.block_attn(q, pk, pv, bk, bv))      # f32 widened exactly
    rows = np.array([[1, 2, 3], [0, 0, 0], [1, 0, 2]])
    sub = oracle.block_attn(q, pk, pv, bk, bv, rows=rows)
    for i, (n, b, h) in enumerate(rows):
        np.testing.assert_array_equal(sub[i], full[n, b, h])
    bits = [W.f32_to_bf16_bits(x) for x in (q, pk, pv, bk, bv)]
    wide = [W.bf16_bits_to_f32(x).astype(np.float64) for x in bits]
    np.testing.assert_array_equal(oracle.block_attn(*bits), oracle.block_attn(*wide))


def test_split_merge_identity_in_fp64():
    # log-sum-exp merge of per-chunk (m, l, o) equals the unsplit softmax:
    # the identity any split-K scheme rests on, checked on plain numpy
    rng = np.random.default_rng(12)
    s = rng.standard_normal(50) * 3
    v = rng.standard_normal((50, 4))
    p = np.exp(s - s.max())
    want = (p[:, None] * v).sum(0) / p.sum()
    parts = []
    for lo, hi in [(0, 7), (7, 31), (31, 50)]:
        m = s[lo:hi].max()
        e = np.exp(s[lo:hi] - m)
        parts.append((m, e.sum(), (e[:, None] * v[lo:hi]).sum(0)))
    M = max(m for m, _, _ in parts)
    l = sum(l_ * np.exp(m - M) for m, l_, _ in parts)
    o = sum(o_ * np.exp(m - M) for m, _, o_ in parts)
    np.testing.assert_allclose(o / l, want, atol=1e-14)
