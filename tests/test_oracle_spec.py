"""Pins for the oracle's scaffold-speculative-decoding pieces (CPU only):
the causal in-block attention of the verify pass and the accept scan
(paper, "Scaffold Speculative Decoding (SS)", steps 1-3)."""
import numpy as np
import pytest
import torch

from tests import brute
from tests.test_oracle_attn import rand_inputs


@pytest.mark.parametrize("N,B,L,Hq,Hkv,D", [(1, 4, 7, 2, 1, 8), (3, 5, 11, 6, 2, 16), (2, 6, 0, 3, 1, 4)])
def test_causal_block_matches_explicit_mask(oracle, N, B, L, Hq, Hkv, D):
    rng = np.random.default_rng(N + 10 * B)
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, L, Hq, Hkv, D)
    got = oracle.block_attn(q, pk, pv, bk, bv, scale=0.41, causal_block=True)
    want = brute.attention_explicit_mask(q, pk, pv, bk, bv, 0.41, causal_block=True)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-12)
    vis = brute.visibility_matrix(2, 3, 2, causal_block=True)
    assert vis[2].tolist() == [True, True, True, False, False, False, False, False]
    assert vis[6].tolist() == [True, True, False, False, False, True, True, False]


def test_causal_block_is_textbook_causal_attention_over_prefix_plus_block(oracle):
    # one rollout: rows L..L+B-1 of ordinary causal attention over [prefix ; block]
    rng = np.random.default_rng(3)
    N, B, L, H, D = 3, 6, 9, 2, 8
    q, pk, pv, bk, bv = rand_inputs(rng, N, B, L, H, H, D)
    got = oracle.block_attn(q, pk, pv, bk, bv, causal_block=True)
    for n in range(N):
        K = torch.from_numpy(np.concatenate([pk, bk[n]], 0)).permute(1, 0, 2)
        V = torch.from_numpy(np.concatenate([pv, bv[n]], 0)).permute(1, 0, 2)
        Q = torch.from_numpy(np.concatenate([rng.standard_normal((L, H, D)), q[n]], 0)).permute(1, 0, 2)
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
        np.testing.assert_allclose(got[n], ref[:, L:, :].permute(1, 0, 2).numpy(), atol=1e-12)


def test_causal_and_bidirectional_agree_where_they_must(oracle):
    rng = np.random.default_rng(4)
    q, pk, pv, bk, bv = rand_inputs(rng, 2, 5, 6, 4, 2, 8)
    bi = oracle.block_attn(q, pk, pv, bk, bv)
    ca = oracle.block_attn(q, pk, pv, bk, bv, causal_block=True)
    np.testing.assert_array_equal(bi[:, -1], ca[:, -1])            # the last position sees the whole block either way
    assert np.abs(bi[:, 0] - ca[:, 0]).max() > 1e-3
    # the first position sees prefix + itself: a one-token block
    one = oracle.block_attn(q[:, :1], pk, pv, bk[:, :1], bv[:, :1])
    np.testing.assert_allclose(ca[:, :1], one, atol=1e-15)
    # later block keys do not influence earlier positions
    bk2, bv2 = bk.copy(), bv.copy()
    bk2[:, 3:] += 2.0
    bv2[:, 3:] -= 1.0
    ca2 = oracle.block_attn(q, pk, pv, bk2, bv2, causal_block=True)
    np.testing.assert_array_equal(ca[:, :3], ca2[:, :3])


def spec_case(rng, N, B, V, agree=0.7):
    logits = rng.standard_normal((N, B, V))
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    mask = ((rng.random((N, B)) < 0.8) & (scaffold == 0)).astype(np.uint8)
    ar = logits.argmax(-1)
    draft = np.where(rng.random((N, B)) < agree, ar, (ar + 1 + rng.integers(0, V - 1, (N, B))) % V).astype(np.int32)
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    return logits, mask, scaffold, draft, tokens


@pytest.mark.parametrize("seed,agree", [(0, 0.7), (1, 1.0), (2, 0.0), (3, 0.9)])
def test_verify_matches_python_brute_force(oracle, seed, agree):
    rng = np.random.default_rng(seed)
    logits, mask, scaffold, draft, tokens = spec_case(rng, 5, 9, 31, agree)
    r = oracle.verify_step(logits, mask, scaffold, draft, tokens)
    t, m, n = brute.verify_python(logits, mask, scaffold, draft, tokens)
    np.testing.assert_array_equal(r["tokens"], t)
    np.testing.assert_array_equal(r["mask"], m)
    np.testing.assert_array_equal(r["n_accepted"], n)


def test_verify_rule_properties(oracle):
    rng = np.random.default_rng(7)
    N, B, V = 6, 10, 17
    logits, mask, scaffold, draft, tokens = spec_case(rng, N, B, V, agree=0.8)
    r = oracle.verify_step(logits, mask, scaffold, draft, tokens)
    is_draft = (mask == 1) & (scaffold == 0)
    ar = logits.argmax(-1)
    for n in range(N):
        pos = np.flatnonzero(is_draft[n])
        wrong = [p for p in pos if ar[n, p] != draft[n, p]]
        k = pos.tolist().index(wrong[0]) if wrong else len(pos)       # drafts accepted before the first mismatch
        assert r["n_accepted"][n] == (k + 1 if wrong else k)            # plus the one bonus token
        assert np.all(r["accepted"][n, pos[:k]] == 1)
        assert np.all(r["tokens"][n, pos[:k]] == draft[n, pos[:k]])
        if wrong:
            assert r["accepted"][n, pos[k]] == 2 and r["tokens"][n, pos[k]] == ar[n, pos[k]]
            rest = pos[k + 1:]
            assert np.all(r["mask"][n, rest] == 1) and np.all(r["tokens"][n, rest] == tokens[n, rest])
        if len(pos):
            assert r["n_accepted"][n] >= 1
    untouched = ~is_draft
    np.testing.assert_array_equal(r["tokens"][untouched], tokens[untouched])     # scaffold / visible never rewritten
    np.testing.assert_array_equal(r["mask"][untouched], mask[untouched])
    np.testing.assert_array_equal(r["ar_tokens"][is_draft], ar[is_draft])
    assert np.all(r["ar_tokens"][untouched] == -1)
    # a draft equal to the AR arg max everywhere is accepted whole; ties in the AR row go to the lowest id
    logits2 = logits.copy()
    logits2[0, :, 5] = logits2[0].max(-1)          # id 5 ties with the maximum
    ar2 = np.array([min(int(a), 5) if logits2[0, b, 5] >= logits2[0, b].max() else int(a)
                    for b, a in enumerate(logits2[0].argmax(-1))])
    r2 = oracle.verify_step(logits2, mask, scaffold, np.broadcast_to(ar2, (N, B)).copy(), tokens)
    assert r2["n_accepted"][0] == is_draft[0].sum() and np.all(r2["mask"][0][is_draft[0]] == 0)
