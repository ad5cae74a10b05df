"""Pins of the oracle's sampled verifier (paper, "Trajectory-only stochasticity":
the verifier samples from the softmax in the trajectory section).

The sampler is Gumbel-max over a Philox-4x32-10 stream.  It is pinned by the
generator's published known-answer vectors, by the accuracy of its log2 against
the library's, by the frequencies of its samples against softmax(x / T) (what
the sampler must reproduce, whatever its construction), by its limits in T and
by the accept rule's own properties.
"""
import os

import numpy as np
import pytest

import oracle
from tests import brute

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "philox4x32_10_kat.txt")


def _kat():
    rows = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        w = [int(t, 16) for t in line.split()]
        rows.append((w[0:4], w[4:6], w[6:10]))
    return rows


def test_philox_known_answers():
    rows = _kat()
    assert len(rows) == 3
    for ctr, key, out in rows:
        assert oracle.philox4x32_10(ctr, key) == out
        assert brute.philox4x32_10_python(ctr, key) == out


def test_flog2_against_library():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        np.exp2(rng.uniform(-24.5, 5.0, 20000)),
        1.0 + np.linspace(-1e-3, 1e-3, 2001),
        np.array([2.0 ** -24, 1 - 2.0 ** -24, 1.0, 1.41421354, 1.4142137, 2.0, 24.0]),
    ]).astype(np.float32)
    got = oracle.flog2(x).astype(np.float64)
    ref = np.log2(x.astype(np.float64))
    # one rounding of the result to binary32 plus the polynomial's 1e-7
    tol = np.spacing(np.abs(ref).astype(np.float32)).astype(np.float64) + 1.5e-7
    assert np.all(np.abs(got - ref) <= tol)
    # exact at powers of two, and monotone
    p2 = np.exp2(np.arange(-24, 6)).astype(np.float32)
    assert np.array_equal(oracle.flog2(p2), np.arange(-24, 6).astype(np.float32))
    xs = np.sort(x)
    assert np.all(np.diff(oracle.flog2(xs)) >= 0)


def _samples(logits_row, rows, temperature, seed, shape=None):
    V = len(logits_row)
    N, B = shape if shape else (rows, 1)
    logits = np.tile(np.asarray(logits_row, dtype=np.float32), (N, B, 1))
    mask = np.ones((N, B), dtype=np.uint8)
    draft = np.full((N, B), -1, dtype=np.int32)
    tokens = np.zeros((N, B), dtype=np.int32)
    out = oracle.verify_step(logits, mask, None, draft, tokens, temperature=temperature, seed=seed)
    return out["ar_tokens"].reshape(-1)


@pytest.mark.parametrize("temperature", [0.7, 1.0, 2.5])
def test_sample_frequencies_follow_softmax(temperature):
    x = np.array([1.5, -0.25, 0.75, 3.0, 2.0, -2.0, 0.0], dtype=np.float32)
    n = 60000
    tok = _samples(x, n, temperature, seed=1234)
    p = np.exp(x.astype(np.float64) / temperature)
    p /= p.sum()
    freq = np.bincount(tok, minlength=len(x)) / n
    sigma = np.sqrt(p * (1 - p) / n)
    assert np.all(np.abs(freq - p) < 5 * sigma), (freq, p)
    # chi-square with V-1 = 6 degrees of freedom: 0.9999 quantile is 27.9
    chi2 = float((n * (freq - p) ** 2 / p).sum())
    assert chi2 < 27.9


def test_temperature_limits():
    x = np.array([0.5, 2.0, 1.0, 2.0, -1.0], dtype=np.float32)
    cold = _samples(x, 2000, 1e-3, seed=5)
    assert set(cold.tolist()) <= {1, 3}           # the two maxima, and only them
    assert 0.4 < np.mean(cold == 1) < 0.6         # exactly tied logits are equally likely
    hot = _samples(x, 50000, 1e4, seed=5)
    freq = np.bincount(hot, minlength=5) / 50000
    assert np.all(np.abs(freq - 0.2) < 0.01)


def test_stream_is_keyed_by_seed_and_row():
    x = np.array([0.1, 0.2, 0.3, 0.25, 0.15, 0.05], dtype=np.float32)
    a = _samples(x, 0, 1.0, seed=77, shape=(6, 50))
    b = _samples(x, 0, 1.0, seed=77, shape=(6, 50))
    c = _samples(x, 0, 1.0, seed=78, shape=(6, 50))
    assert np.array_equal(a, b)
    assert not np.array_equal(a, c)
    # the row counter is n B + b: the same rows laid out differently sample the same tokens
    d = _samples(x, 0, 1.0, seed=77, shape=(300, 1))
    e = _samples(x, 0, 1.0, seed=77, shape=(1, 300))
    assert np.array_equal(a, d) and np.array_equal(a, e)
    # rows with identical logits do not repeat each other
    assert len(set(a.tolist())) > 1


def test_key_matches_independent_python_statement():
    rng = np.random.default_rng(3)
    for _ in range(300):
        x = np.float32(rng.normal(0, 2))
        t = float(np.float32(rng.uniform(0.3, 3.0)))
        seed = int(rng.integers(0, 2 ** 63))
        row = int(rng.integers(0, 2 ** 20))
        v = int(rng.integers(0, 200000))
        got = np.float32(oracle.sample_key(x, t, seed, row, v))
        ref = brute.sample_key_python(x, t, seed, row, v)
        assert got.tobytes() == np.float32(ref).tobytes(), (x, t, seed, row, v, got, ref)


def test_noise_is_standard_gumbel():
    # key - x c = -log2(-log2 u); times ln 2, minus ln ln 2, it is -ln(-ln u): mean = Euler's constant, variance pi^2/6
    g = np.array([oracle.sample_key(0.0, 1.0, 99, row, v) for row in range(40) for v in range(500)], dtype=np.float64)
    g = g * np.log(2.0) - np.log(np.log(2.0))
    n = g.size
    assert abs(g.mean() - 0.5772156649) < 5 * np.sqrt((np.pi ** 2 / 6) / n)
    assert abs(g.var() - np.pi ** 2 / 6) < 0.1


def test_accept_rule_with_a_sampled_verifier():
    rng = np.random.default_rng(11)
    N, B, V = 5, 12, 40
    logits = rng.normal(0, 1.5, (N, B, V)).astype(np.float32)
    mask = np.ones((N, B), dtype=np.uint8)
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    tokens = rng.integers(0, V, (N, B)).astype(np.int32)
    none = np.full((N, B), -1, dtype=np.int32)
    sampled = oracle.verify_step(logits, mask, scaffold, none, tokens, temperature=0.9, seed=42)["ar_tokens"]
    # drafts equal to the sampled tokens up to a chosen point, wrong from there on
    draft = sampled.copy()
    cut = rng.integers(0, B, N)
    for n in range(N):
        draft[n, cut[n]:] = (sampled[n, cut[n]:] + 1) % V
    out = oracle.verify_step(logits, mask, scaffold, draft, tokens, temperature=0.9, seed=42)
    ref = brute.accept_scan_python(sampled, mask, scaffold, draft, tokens)
    assert np.array_equal(out["tokens"], ref["tokens"])
    assert np.array_equal(out["mask"], ref["mask"])
    assert np.array_equal(out["n_accepted"], ref["n_accepted"])
    assert np.array_equal(out["accepted"], ref["accepted"])
    # greedy is what temperature 0 means
    greedy = oracle.verify_step(logits, mask, scaffold, none, tokens)["ar_tokens"]
    elig = (mask == 1) & (scaffold == 0)
    assert np.array_equal(greedy[elig], logits.argmax(-1)[elig])


def test_equal_keys_resolve_to_the_lowest_id():
    # at a very low temperature x c is so large that the noise is quantised coarsely
    # and exactly equal keys become common; the lowest id must win them
    x = np.array([2.0, 2.0, 2.0, 2.0, -1.0, 2.0], dtype=np.float32)
    t, seed, rows = 1e-6, 2024, 1500
    tok = _samples(x, rows, t, seed=seed)
    ties = 0
    for row in range(rows):
        keys = [np.float32(oracle.sample_key(float(x[v]), t, seed, row, v)) for v in range(len(x))]
        top = max(keys)
        winners = [v for v, k in enumerate(keys) if k == top]
        assert tok[row] == winners[0]
        ties += len(winners) > 1
    assert ties > 20      # the case is exercised
