"""Pins for the fp64 unmask oracle, the KV refresh and the fork copy (CPU only).

The commit rule is the task's reading of "iteratively unmasks value
positions" (paper, "Section Diffusion (SD)") with frozen scaffold positions
(paper, Eq. 2): confidence = largest softmax probability, commit at
confidence >= tau, lowest index on ties, at least one commit per block that
still has an eligible position.
"""
import numpy as np
import pytest
from scipy.special import logsumexp

from tests import brute


def case(rng, N, B, V, scaffold_frac=0.3, masked_frac=0.7, spike=0.0):
    logits = rng.standard_normal((N, B, V))
    if spike:
        hit = rng.random((N, B)) < 0.5
        ids = rng.integers(0, V, size=(N, B))
        n, b = np.nonzero(hit)
        logits[n, b, ids[n, b]] += spike
    scaffold = (rng.random((N, B)) < scaffold_frac).astype(np.uint8)
    mask = ((rng.random((N, B)) < masked_frac) & (scaffold == 0)).astype(np.uint8)
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    tokens[mask == 1] = -1
    return logits, mask, scaffold, tokens


@pytest.mark.parametrize("seed,spike,tau", [(0, 0.0, 0.9), (1, 8.0, 0.9), (2, 8.0, 0.5), (3, 5.0, 0.2)])
def test_matches_python_brute_force(oracle, seed, spike, tau):
    rng = np.random.default_rng(seed)
    logits, mask, scaffold, tokens = case(rng, 4, 6, 37, spike=spike)
    r = oracle.unmask_step(logits, mask, scaffold, tokens, tau)
    t, m, c, nu = brute.unmask_python(logits, mask, scaffold, tokens, tau)
    np.testing.assert_array_equal(r["tokens"], t)
    np.testing.assert_array_equal(r["mask"], m)
    np.testing.assert_array_equal(r["n_unmasked"], nu)
    np.testing.assert_allclose(r["confidences"], c, rtol=1e-13)


def test_confidence_is_exp_of_max_minus_logsumexp(oracle):
    rng = np.random.default_rng(5)
    logits, mask, scaffold, tokens = case(rng, 3, 5, 101, spike=4.0)
    r = oracle.unmask_step(logits, mask, scaffold, tokens, 0.9)
    el = (mask == 1) & (scaffold == 0)
    want = np.exp(logits.max(-1) - logsumexp(logits, axis=-1))
    np.testing.assert_allclose(r["confidences"][el], want[el], rtol=1e-12)
    assert np.all(np.isneginf(r["confidences"][~el]))
    np.testing.assert_array_equal(r["candidates"][el], logits.argmax(-1)[el])
    assert np.all(r["candidates"][~el] == -1)


def test_row_closed_forms(oracle):
    V = 64
    logits = np.zeros((1, 4, V))
    logits[0, 1, 17] = 40.0                    # near one-hot
    logits[0, 2, [9, 30]] = 3.0                # two equal maxima -> lower id
    logits[0, 3, :] = -7.25                    # shifted constant row
    mask = np.ones((1, 4), np.uint8)
    sc = np.zeros((1, 4), np.uint8)
    r = oracle.unmask_step(logits, mask, sc, np.full((1, 4), -1, np.int32), tau=2.0)
    c = r["confidences"][0]
    assert c[0] == pytest.approx(1.0 / V, rel=1e-14) and r["candidates"][0, 0] == 0
    assert c[1] == pytest.approx(1.0, abs=1e-15) and r["candidates"][0, 1] == 17
    assert r["candidates"][0, 2] == 9
    assert c[2] == pytest.approx(1.0 / (2.0 + (V - 2) * np.exp(-3.0)), rel=1e-14)
    assert c[3] == pytest.approx(1.0 / V, rel=1e-14)
    # tau > 1: exactly one commit, the most confident position
    assert r["n_unmasked"][0] == 1 and r["committed"][0].tolist() == [0, 1, 0, 0]


def test_forced_commit_tie_takes_lowest_position(oracle):
    V = 16
    row = np.random.default_rng(0).standard_normal(V)
    logits = np.tile(row, (1, 5, 1))           # identical rows -> identical confidences
    mask = np.array([[0, 1, 1, 0, 1]], np.uint8)
    sc = np.zeros((1, 5), np.uint8)
    r = oracle.unmask_step(logits, mask, sc, np.full((1, 5), 7, np.int32), tau=0.99)
    assert r["committed"][0].tolist() == [0, 1, 0, 0, 0]


def test_threshold_is_inclusive(oracle):
    # two-way tie of the maximum in a row of otherwise -inf-like logits: conf = 0.5 exactly
    logits = np.full((1, 2, 8), -1e4)
    logits[0, :, [2, 5]] = 1.0
    r = oracle.unmask_step(logits, np.ones((1, 2), np.uint8), None, np.full((1, 2), -1, np.int32), tau=0.5)
    assert r["confidences"][0].tolist() == [0.5, 0.5]
    assert r["n_unmasked"][0] == 2 and r["tokens"][0].tolist() == [2, 2]


def test_minus_infinity_logits_are_entries_of_probability_zero(oracle):
    # a vocabulary entry at -inf (a banned token) has softmax probability exactly 0: the row's confidence
    # and arg max are those of the row with these entries removed (library log-sum-exp as the second opinion)
    from scipy.special import logsumexp
    rng = np.random.default_rng(31)
    V = 97
    x = rng.standard_normal((1, 6, V)) * 2
    holes = [np.arange(0, 9), np.arange(V - 11, V), np.arange(8, 24), np.array([0, 5, 50, 96]),
             np.setdiff1d(np.arange(V), [13]), np.setdiff1d(np.arange(V), [3, 77])]
    x[0, 5, 77] = x[0, 5, 3]            # two finite entries, equal: lowest id, confidence 1/2
    for b, h in enumerate(holes):
        x[0, b, h] = -np.inf
    r = oracle.unmask_step(x, np.ones((1, 6), np.uint8), None, np.full((1, 6), -1, np.int32), tau=2.0)
    for b, h in enumerate(holes):
        keep = np.setdiff1d(np.arange(V), h)
        assert r["candidates"][0, b] == keep[np.argmax(x[0, b, keep])]
        assert r["confidences"][0, b] == pytest.approx(np.exp(x[0, b, keep].max() - logsumexp(x[0, b, keep])), rel=1e-13)
    assert r["confidences"][0, 4] == 1.0 and r["candidates"][0, 4] == 13
    assert r["confidences"][0, 5] == 0.5 and r["candidates"][0, 5] == 3


@pytest.mark.parametrize("seed", range(5))
def test_block_invariants(oracle, seed):
    rng = np.random.default_rng(100 + seed)
    logits, mask, scaffold, tokens = case(rng, 5, 9, 53, spike=6.0)
    # a mask bit set on a scaffold position must be ignored: scaffold wins
    mask[0, 0], scaffold[0, 0] = 1, 1
    tau = 0.6
    r = oracle.unmask_step(logits, mask, scaffold, tokens, tau)
    el = (mask == 1) & (scaffold == 0)
    com = r["committed"] == 1
    assert np.all(el[com])                                        # commits only on eligible
    np.testing.assert_array_equal(r["tokens"][~com], tokens[~com])  # everything else untouched
    np.testing.assert_array_equal(r["mask"][~com], mask[~com])
    np.testing.assert_array_equal(r["tokens"][scaffold == 1], tokens[scaffold == 1])
    assert np.all(r["mask"][com] == 0)
    np.testing.assert_array_equal(r["n_unmasked"], com.sum(1))
    has = el.any(1)
    assert np.all(r["n_unmasked"][has] >= 1) and np.all(r["n_unmasked"][~has] == 0)
    over = el & (r["confidences"] >= tau)
    for n in range(5):
        if over[n].any():
            np.testing.assert_array_equal(com[n], over[n])
        elif el[n].any():
            assert com[n].sum() == 1
            assert r["confidences"][n][com[n]][0] == r["confidences"][n][el[n]].max()
    # tau = 0: every eligible position commits; tau > 1: exactly one per block with any eligible
    r0 = oracle.unmask_step(logits, mask, scaffold, tokens, 0.0)
    np.testing.assert_array_equal(r0["committed"] == 1, el)
    r2 = oracle.unmask_step(logits, mask, scaffold, tokens, 1.5)
    np.testing.assert_array_equal(r2["n_unmasked"], has.astype(np.int32))


def test_repeated_steps_terminate_and_are_idempotent(oracle):
    rng = np.random.default_rng(9)
    logits, mask, scaffold, tokens = case(rng, 3, 7, 29, masked_frac=1.0)
    el0 = ((mask == 1) & (scaffold == 0)).sum(1)
    steps = 0
    while ((mask == 1) & (scaffold == 0)).any():
        r = oracle.unmask_step(rng.standard_normal(logits.shape), mask, scaffold, tokens, 0.9)
        mask, tokens = r["mask"], r["tokens"]
        steps += 1
        assert steps <= el0.max()
    r = oracle.unmask_step(logits, mask, scaffold, tokens, 0.0)
    np.testing.assert_array_equal(r["tokens"], tokens)
    np.testing.assert_array_equal(r["mask"], mask)
    assert r["n_unmasked"].sum() == 0


def test_bf16_and_f32_storage_are_widened_exactly(oracle):
    import fdd_workloads as W
    rng = np.random.default_rng(10)
    logits, mask, scaffold, tokens = case(rng, 2, 4, 300, spike=6.0)
    bits = W.f32_to_bf16_bits(logits.astype(np.float32))
    wide = W.bf16_bits_to_f32(bits).astype(np.float64)
    a = oracle.unmask_step(bits, mask, scaffold, tokens, 0.5)
    b = oracle.unmask_step(wide, mask, scaffold, tokens, 0.5)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    # bf16 rows have real ties for the maximum; the lowest id must win
    el = (mask == 1) & (scaffold == 0)
    np.testing.assert_array_equal(a["candidates"][el], wide.argmax(-1)[el])


def test_kv_update_is_a_row_gather(oracle):
    rng = np.random.default_rng(11)
    N, B, Hkv, D, T = 3, 4, 2, 8, 10
    tk, tv = rng.standard_normal((T, Hkv, D)), rng.standard_normal((T, Hkv, D))
    bk, bv = rng.standard_normal((N, B, Hkv, D)), rng.standard_normal((N, B, Hkv, D))
    tokens = rng.integers(0, 1000, size=(N, B)).astype(np.int32)
    com = (rng.random((N, B)) < 0.4).astype(np.uint8)
    k2, v2 = oracle.block_kv_update(tokens, com, tk, tv, bk, bv)
    wk, wv = bk.copy(), bv.copy()
    wk[com == 1] = tk[tokens[com == 1] % T]
    wv[com == 1] = tv[tokens[com == 1] % T]
    np.testing.assert_array_equal(k2, wk)
    np.testing.assert_array_equal(v2, wv)


def test_fork_replicates_private_state(oracle):
    src = np.arange(24, dtype=np.float32).reshape(2, 3, 4)
    dst = oracle.fork_block(src, 5)
    assert dst.shape == (5, 2, 3, 4)
    np.testing.assert_array_equal(dst, np.broadcast_to(src, dst.shape))
