"""GPU parity of fdd_unmask_step, fdd_block_kv_update and fdd_fork_block
against the fp64 oracle (through the C ABI).

Token ids, commit decisions and masks must be bit-exact.  Positions whose
fp64 confidence lies within 1e-3 of tau are exempt from the decision check
and reported; when nothing reaches tau and the two best fp64 confidences of
a block are closer than 1e-6 relative, either is a valid forced commit.
"""
import numpy as np
import pytest
import torch

import fdd_workloads as W
from tests.gpu_util import print_case, to_dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def F():
    import paper_2605_23163_amd as F
    F.load_library()
    assert torch.cuda.is_available()
    return F


def tau32(tau):
    return float(np.float32(tau))


def run_both(F, oracle, logits, mask, scaffold, tokens, tau):
    tau = tau32(tau)
    ref = oracle.unmask_step(logits, mask, scaffold, tokens, tau)
    lg = to_dev(logits)
    m = torch.from_numpy(mask.copy()).cuda()
    t = torch.from_numpy(tokens.copy()).cuda()
    sc = None if scaffold is None else torch.from_numpy(scaffold).cuda()
    _, conf, nun, com = F.fdd_unmask_step(lg, m, sc, tau, t)
    torch.cuda.synchronize()
    got = dict(tokens=t.cpu().numpy(), mask=m.cpu().numpy(), confidences=conf.cpu().numpy(),
               n_unmasked=nun.cpu().numpy(), committed=com.cpu().numpy())
    return ref, got, tau


def compare(ref, got, mask, scaffold, tokens, tau):
    """Returns (#near-tau positions, #near-tie forced blocks)."""
    N, B = mask.shape
    sc = np.zeros_like(mask) if scaffold is None else scaffold
    el = (mask == 1) & (sc == 0)
    c64 = ref["confidences"]
    # confidences: fp32 result of an fp32 sum
    np.testing.assert_allclose(got["confidences"][el], c64[el], rtol=2e-5)
    assert np.all(np.isneginf(got["confidences"][~el]))
    near_tau = el & (np.abs(c64 - tau) < 1e-3)
    near_tie_blocks = 0
    for n in range(N):
        strict = el[n] & ~near_tau[n]
        forced_ref = el[n].any() and not (c64[n][el[n]] >= tau).any()
        if forced_ref and not near_tau[n].any():
            srt = np.sort(c64[n][el[n]])[::-1]
            tie = len(srt) > 1 and (srt[0] - srt[1]) <= 1e-6 * srt[0]
            if tie:
                near_tie_blocks += 1
                b = int(np.flatnonzero(got["committed"][n])[0])
                assert got["committed"][n].sum() == 1 and el[n, b] and c64[n, b] >= srt[0] * (1 - 1e-6)
                assert got["tokens"][n, b] == ref["candidates"][n, b]
                continue
        if near_tau[n].any():
            # decisions at the exempt positions may differ; everything else may not,
            # except that a forced commit depends on them
            if forced_ref or (got["committed"][n] != ref["committed"][n])[near_tau[n]].any():
                ok = strict & (c64[n] >= tau)
                assert np.all(got["committed"][n][ok] == 1)
                continue
        np.testing.assert_array_equal(got["committed"][n], ref["committed"][n])
        np.testing.assert_array_equal(got["tokens"][n], ref["tokens"][n])
        np.testing.assert_array_equal(got["mask"][n], ref["mask"][n])
        assert got["n_unmasked"][n] == ref["n_unmasked"][n]
    # committed tokens are always the oracle's arg max; untouched positions keep their bits
    com = got["committed"] == 1
    np.testing.assert_array_equal(got["tokens"][com], ref["candidates"][com])
    np.testing.assert_array_equal(got["tokens"][~com], tokens[~com])
    np.testing.assert_array_equal(got["mask"][~com], mask[~com])
    assert np.all(el[com]) and np.all(got["mask"][com] == 0)
    np.testing.assert_array_equal(got["n_unmasked"], com.sum(1))
    return int(near_tau.sum()), near_tie_blocks


def synth(rng, N, B, V, dtype, std, spike, spike_frac, scaffold_frac, masked_frac=1.0):
    x = (rng.standard_normal((N, B, V)) * std).astype(np.float32)
    scaffold = (rng.random((N, B)) < scaffold_frac).astype(np.uint8)
    mask = ((rng.random((N, B)) < masked_frac) & (scaffold == 0)).astype(np.uint8)
    hit = (rng.random((N, B)) < spike_frac)
    ids = rng.integers(0, V, size=(N, B))
    n, b = np.nonzero(hit)
    x[n, b, ids[n, b]] += spike
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    tokens[mask == 1] = -1
    return W.to_storage(x, dtype), mask, scaffold, tokens


CASES = [
    # N, B,  V,      dtype,  std, spike, spike_frac, scaffold_frac, masked_frac, tau
    (1, 8, 512, W.F32, 1.0, 6.0, 0.5, 0.25, 1.0, 0.9),
    (3, 7, 1000, W.F32, 1.0, 10.0, 0.8, 0.3, 0.7, 0.9),       # most spiked rows pass tau
    (4, 9, 999, W.BF16, 1.0, 10.0, 0.8, 0.3, 0.7, 0.9),        # odd V: rows start off a 16-byte boundary
    (2, 5, 37, W.BF16, 1.0, 4.0, 0.5, 0.2, 1.0, 0.5),          # V smaller than one workgroup pass
    (2, 33, 20011, W.BF16, 2.0, 14.0, 0.5, 0.4, 0.8, 0.9),     # several pieces per row, ragged
    (5, 4, 152064, W.BF16, 2.0, 20.0, 0.5, 0.5, 1.0, 0.9),     # full vocabulary, peaked rows pass tau
    (2, 6, 70001, W.F32, 2.0, 18.0, 0.5, 0.0, 1.0, 0.9),
]


@pytest.mark.parametrize("case", CASES)
def test_matches_oracle(F, oracle, case):
    N, B, V, dtype, std, spike, sf, scf, mf, tau = case
    print_case(test="unmask_parity", case=case)
    rng = np.random.default_rng(hash(case[:3]) % 2**32)
    logits, mask, scaffold, tokens = synth(rng, N, B, V, dtype, std, spike, sf, scf, mf)
    ref, got, tau = run_both(F, oracle, logits, mask, scaffold, tokens, tau)
    near, ties = compare(ref, got, mask, scaffold, tokens, tau)
    print(f"near-tau positions: {near}, near-tie forced blocks: {ties}, commits: {int(got['n_unmasked'].sum())}")


def test_bf16_ties_take_the_lowest_id(F, oracle):
    print_case(test="unmask_ties")
    # coarse bf16 values: the row maximum is attained many times
    rng = np.random.default_rng(3)
    N, B, V = 2, 16, 50000
    x = np.round(rng.standard_normal((N, B, V)).astype(np.float32) * 2) / 2
    logits = W.to_storage(np.clip(x, -3, 3), W.BF16)
    mask = np.ones((N, B), np.uint8)
    tokens = np.full((N, B), -1, np.int32)
    ref, got, tau = run_both(F, oracle, logits, mask, None, tokens, 0.0)      # tau = 0: everything commits
    np.testing.assert_array_equal(got["tokens"], ref["tokens"])
    wide = W.widen(logits, W.BF16)
    np.testing.assert_array_equal(got["tokens"], wide.argmax(-1))
    assert (wide == wide.max(-1, keepdims=True)).sum(-1).min() > 1


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_minus_infinity_entries(F, oracle, dtype):
    # -inf logits (banned tokens) have probability 0; runs of them at the head of a row, over whole 16-byte
    # vectors, across a piece boundary and at the tail must not disturb the row's sum or its arg max
    print_case(test="unmask_minus_inf", dtype=dtype)
    rng = np.random.default_rng(17)
    N, B, V = 2, 8, 70001
    x = (rng.standard_normal((N, B, V)) * 2).astype(np.float32)
    ninf = np.float32(-np.inf)
    x[0, 0, :1] = ninf                      # head element
    x[0, 1, :4099] = ninf                   # every thread of the first pass meets only -inf first
    x[0, 2, 8:8 + 8 * 700] = ninf           # aligned runs of whole vectors
    x[0, 3, V - 5:] = ninf                  # tail
    x[0, 4, 30000:41000] = ninf             # across a piece boundary
    x[0, 5, :] = ninf
    x[0, 5, 12345] = 1.5                    # a single finite entry: confidence 1
    x[0, 6, 1::2] = ninf                    # every other entry
    x[0, 7, :] = ninf
    x[0, 7, [7, 69999]] = -3.0              # two equal finite entries far apart: lowest id, confidence 1/2
    x[1, :, rng.integers(0, V, 3000)] = ninf
    logits = W.to_storage(x, dtype)
    mask = np.ones((N, B), np.uint8)
    tokens = np.full((N, B), -1, np.int32)
    for tau in (0.0, 0.9):
        ref, got, t32 = run_both(F, oracle, logits, mask, None, tokens, tau)
        assert np.isfinite(got["confidences"]).all()
        compare(ref, got, mask, None, tokens, t32)
    assert abs(got["confidences"][0, 5] - 1.0) <= 2e-5 and abs(got["confidences"][0, 7] - 0.5) <= 1e-5
    assert ref["candidates"][0, 5] == 12345 and ref["candidates"][0, 7] == 7


def test_near_tau_rows_are_reported_not_failed(F, oracle):
    print_case(test="unmask_near_tau")
    # rows built so that conf = 1/(1 + (V-1) e^-s) sits within 1e-3 of tau
    V, tau = 4096, 0.9
    s0 = np.log((V - 1) * tau / (1 - tau))
    offs = np.linspace(-0.01, 0.01, 24)
    x = np.zeros((1, 24, V), np.float32)
    x[0, np.arange(24), 7] = (s0 + offs).astype(np.float32)
    mask = np.ones((1, 24), np.uint8)
    ref, got, tau = run_both(F, oracle, x, mask, None, np.full((1, 24), -1, np.int32), tau)
    near, _ = compare(ref, got, mask, None, np.full((1, 24), -1, np.int32), tau)
    assert near >= 1
    c = ref["confidences"][0]
    far = np.abs(c - tau) >= 1e-3
    np.testing.assert_array_equal(got["committed"][0][far], (c[far] >= tau).astype(np.uint8))


def test_block_rule_edge_cases(F, oracle):
    print_case(test="unmask_edges")
    rng = np.random.default_rng(4)
    N, B, V = 6, 8, 300
    logits = W.to_storage(rng.standard_normal((N, B, V)).astype(np.float32), W.F32)
    mask = np.ones((N, B), np.uint8)
    scaffold = np.zeros((N, B), np.uint8)
    mask[0] = 0                     # nothing masked: no-op block
    scaffold[1] = 1                 # all scaffold (mask bits set are ignored)
    mask[2] = 0
    mask[2, 5] = 1                  # exactly one eligible position
    logits[3, 1:] = logits[3, 0]    # identical rows: forced commit ties -> lowest position
    scaffold[4, ::2] = 1
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    for tau in (0.9, 0.0, 1.5):
        ref, got, t32 = run_both(F, oracle, logits, mask, scaffold, tokens, tau)
        compare(ref, got, mask, scaffold, tokens, t32)
        assert got["n_unmasked"][0] == 0 and got["n_unmasked"][1] == 0
        np.testing.assert_array_equal(got["tokens"][:2], tokens[:2])
    ref, got, _ = run_both(F, oracle, logits, mask, scaffold, tokens, 0.9)
    assert got["committed"][2].tolist() == [0, 0, 0, 0, 0, 1, 0, 0]
    assert got["committed"][3].tolist() == [1, 0, 0, 0, 0, 0, 0, 0]


def test_config4_full_step(F, oracle):
    w = W.CONFIGS["cfg4"]
    print_case(test="unmask_cfg4")
    rng = np.random.default_rng(w.seed)
    scaffold = W.scaffold_positions(w, rng)
    tokens, mask = W.initial_state(w, scaffold, rng)
    logits = W.step_logits(w, mask, rng)
    ref, got, tau = run_both(F, oracle, logits, mask, scaffold, tokens, w.tau)
    near, ties = compare(ref, got, mask, scaffold, tokens, tau)
    # at these logit statistics nothing reaches tau: every block makes its forced commit
    assert np.all(got["n_unmasked"] == 1)
    print(f"cfg4: near-tau {near}, near-tie {ties}, max conf {ref['confidences'].max():.3f}")


def test_repeated_steps_drain_the_block(F, oracle):
    print_case(test="unmask_multi_step")
    rng = np.random.default_rng(6)
    N, B, V = 3, 12, 2048
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    mask = (1 - scaffold).astype(np.uint8)
    tokens = np.where(scaffold == 1, 5, -1).astype(np.int32)
    m_o, t_o = mask.copy(), tokens.copy()
    m_g, t_g = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    sc_g = torch.from_numpy(scaffold).cuda()
    for step in range(B + 1):
        if not m_o.any():
            break
        x = (rng.standard_normal((N, B, V)) * 2).astype(np.float32)
        hit = rng.random((N, B)) < 0.4
        n, b = np.nonzero(hit)
        x[n, b, rng.integers(0, V, len(n))] += 16.0
        logits = W.to_storage(x, W.BF16)
        r = oracle.unmask_step(logits, m_o, scaffold, t_o, tau32(0.9))
        m_o, t_o = r["mask"], r["tokens"]
        F.fdd_unmask_step(to_dev(logits), m_g, sc_g, tau32(0.9), t_g)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(m_g.cpu().numpy(), m_o)
        np.testing.assert_array_equal(t_g.cpu().numpy(), t_o)
    assert not m_o.any() and step <= B


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_kv_update_and_fork(F, oracle, dtype):
    print_case(test="bookkeeping", dtype=dtype)
    rng = np.random.default_rng(7)
    N, B, Hkv, D, T = 5, 9, 4, 128, 64
    f = lambda *s: W.to_storage(rng.standard_normal(s).astype(np.float32), dtype)
    tk, tv, bk, bv = f(T, Hkv, D), f(T, Hkv, D), f(N, B, Hkv, D), f(N, B, Hkv, D)
    tokens = rng.integers(0, 100000, size=(N, B)).astype(np.int32)
    com = (rng.random((N, B)) < 0.4).astype(np.uint8)
    rk, rv = oracle.block_kv_update(tokens, com, tk, tv, bk, bv)
    gk, gv = to_dev(bk), to_dev(bv)
    F.fdd_block_kv_update(torch.from_numpy(tokens).cuda(), torch.from_numpy(com).cuda(), to_dev(tk), to_dev(tv), gk, gv)
    torch.cuda.synchronize()
    assert torch.equal(gk, to_dev(rk)) and torch.equal(gv, to_dev(rv))
    # fork: one rollout's block state replicated N times, any byte count that is a multiple of 4
    for src in (bk[0], tokens[0], np.arange(7, dtype=np.int32)):
        want = oracle.fork_block(src, 6)
        got = F.fdd_fork_block(to_dev(src), 6)
        torch.cuda.synchronize()
        assert torch.equal(got, to_dev(want))


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("tau", [0.0, 0.6, 1.5])
def test_refresh_inside_the_unmask_call_equals_the_separate_update(F, oracle, dtype, tau):
    # many commits per block (tau = 0), some (tau = 0.6) and the forced single commit (tau > 1); B > 64 so that a
    # wavefront walks more than one chunk of positions
    print_case(test="unmask_fused_refresh", dtype=dtype, tau=tau)
    rng = np.random.default_rng(41)
    N, B, V, Hkv, D, T = 3, 70, 777, 2, 64, 50
    logits, mask, scaffold, tokens = synth(rng, N, B, V, dtype, 1.0, 9.0, 0.5, 0.3, 0.8)
    f = lambda *s: W.to_storage(rng.standard_normal(s).astype(np.float32), dtype)
    tk, tv, bk, bv = f(T, Hkv, D), f(T, Hkv, D), f(N, B, Hkv, D), f(N, B, Hkv, D)
    t32 = tau32(tau)
    ref = oracle.unmask_step(logits, mask, scaffold, tokens, t32)
    assert not (((mask == 1) & (scaffold == 0)) & (np.abs(ref["confidences"] - t32) < 1e-3)).any()
    rk, rv = oracle.block_kv_update(ref["tokens"], ref["committed"], tk, tv, bk, bv)
    m, t = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    gk, gv = to_dev(bk), to_dev(bv)
    _, conf, nun, com = F.fdd_unmask_step(to_dev(logits), m, torch.from_numpy(scaffold).cuda(), t32, t,
                                          refresh=(to_dev(tk), to_dev(tv), gk, gv))
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), ref["tokens"])
    np.testing.assert_array_equal(com.cpu().numpy(), ref["committed"])
    assert torch.equal(gk, to_dev(rk)) and torch.equal(gv, to_dev(rv))
    assert int(ref["committed"].sum()) >= N
