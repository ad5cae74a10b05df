"""GPU parity of the scaffold-speculative-decoding pieces against the oracle:
causal in-block attention (verify pass), the accept scan, and the sampled
verifier of the trajectory section."""
import numpy as np
import pytest
import torch

import fdd_workloads as W
from tests.gpu_util import print_case, rand_attn, to_dev, to_f64

pytestmark = pytest.mark.gpu

TOL = {W.BF16: 2e-2, W.F32: 1e-4}


@pytest.fixture(scope="module")
def F():
    import paper_2605_23163_amd as F
    F.load_library()
    return F


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("shape", [(1, 8, 256, 4, 1, 64), (3, 20, 333, 14, 2, 128), (2, 70, 64, 8, 8, 64),
                                   (4, 16, 0, 4, 2, 128), (5, 32, 1000, 28, 4, 128), (9, 3, 200, 3, 1, 64)])
def test_causal_block_attention_matches_oracle(F, oracle, shape, dtype):
    N, B, L, Hq, Hkv, D = shape
    print_case(test="spec_causal_attn", shape=shape, dtype=dtype)
    rng = np.random.default_rng(hash(shape) % 2**32 + 1)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    t = {k: to_dev(v) for k, v in d.items()}
    out = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], causal_block=True)
    bi = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"])
    torch.cuda.synchronize()
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], causal_block=True)
    err = np.abs(to_f64(out) - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err}"
    # the last block position sees the same keys in both forms
    assert np.abs(to_f64(out[:, -1]) - to_f64(bi[:, -1])).max() <= (2e-3 if dtype == W.BF16 else 1e-5)
    if B > 1:
        assert not torch.equal(out[:, 0], bi[:, 0])


def synth(rng, N, B, V, dtype, agree):
    x = (rng.standard_normal((N, B, V)) * 2).astype(np.float32)
    logits = W.to_storage(x, dtype)
    wide = W.widen(logits, dtype)
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    mask = ((rng.random((N, B)) < 0.85) & (scaffold == 0)).astype(np.uint8)
    ar = wide.argmax(-1)
    draft = np.where(rng.random((N, B)) < agree, ar, (ar + 1 + rng.integers(0, V - 1, (N, B))) % V).astype(np.int32)
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    return logits, mask, scaffold, draft, tokens


@pytest.mark.parametrize("case", [(3, 9, 999, W.BF16, 0.8), (2, 33, 20011, W.BF16, 0.95), (4, 8, 152064, W.BF16, 0.9),
                                  (2, 70, 5000, W.F32, 0.97), (5, 6, 37, W.F32, 0.0), (3, 12, 4096, W.BF16, 1.0)])
def test_verify_step_is_bit_exact(F, oracle, case):
    N, B, V, dtype, agree = case
    print_case(test="spec_verify", case=case)
    rng = np.random.default_rng(hash(case[:3]) % 2**32)
    logits, mask, scaffold, draft, tokens = synth(rng, N, B, V, dtype, agree)
    ref = oracle.verify_step(logits, mask, scaffold, draft, tokens)
    m, t = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    _, nacc, acc = F.fdd_verify_step(to_dev(logits), m, torch.from_numpy(scaffold).cuda(), torch.from_numpy(draft).cuda(), t)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), ref["tokens"])
    np.testing.assert_array_equal(m.cpu().numpy(), ref["mask"])
    np.testing.assert_array_equal(nacc.cpu().numpy(), ref["n_accepted"])
    np.testing.assert_array_equal(acc.cpu().numpy(), ref["accepted"])
    print(f"accepted per block: {ref['n_accepted'].tolist()}")


def test_draft_then_verify_block(F, oracle):
    # one block of scaffold speculative decoding on synthetic logits: draft every value position from the
    # bidirectional pass (tau = 0 commits all), verify against AR logits, compare with the oracle end to end
    print_case(test="spec_draft_verify")
    rng = np.random.default_rng(5)
    N, B, V = 4, 32, 8192
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    mask0 = (1 - scaffold).astype(np.uint8)
    tokens0 = np.where(scaffold == 1, 7, -1).astype(np.int32)
    mdm = W.to_storage((rng.standard_normal((N, B, V)) * 2).astype(np.float32), W.BF16)
    ar = W.bf16_bits_to_f32(mdm).copy()
    flip = rng.random((N, B)) < 0.1                       # the AR head disagrees on ~10 % of positions
    n_, b_ = np.nonzero(flip)
    ar[n_, b_, rng.integers(0, V, len(n_))] += 30.0
    ar = W.to_storage(ar, W.BF16)
    # oracle
    d = oracle.unmask_step(mdm, mask0, scaffold, tokens0, 0.0)
    draft = d["tokens"]
    v = oracle.verify_step(ar, mask0, scaffold, draft, tokens0)
    # GPU: the draft pass works on a scratch copy of the state, the verify pass on the real one
    sc = torch.from_numpy(scaffold).cuda()
    dm, dt = torch.from_numpy(mask0.copy()).cuda(), torch.from_numpy(tokens0.copy()).cuda()
    F.fdd_unmask_step(to_dev(mdm), dm, sc, 0.0, dt)
    m, t = torch.from_numpy(mask0.copy()).cuda(), torch.from_numpy(tokens0.copy()).cuda()
    _, nacc, _ = F.fdd_verify_step(to_dev(ar), m, sc, dt, t)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(dt.cpu().numpy(), draft)
    np.testing.assert_array_equal(t.cpu().numpy(), v["tokens"])
    np.testing.assert_array_equal(m.cpu().numpy(), v["mask"])
    np.testing.assert_array_equal(nacc.cpu().numpy(), v["n_accepted"])
    assert np.all(t.cpu().numpy()[scaffold == 1] == 7)


@pytest.mark.parametrize("case", [(3, 9, 999, W.BF16, 0.9, 1), (2, 33, 20011, W.BF16, 1.3, 2 ** 40 + 7), (4, 8, 152064, W.BF16, 0.7, 3),
                                  (2, 70, 5000, W.F32, 1.0, 4), (5, 6, 37, W.F32, 2.0, 5), (3, 12, 4096, W.BF16, 0.25, 2 ** 63 + 11),
                                  (2, 5, 1003, W.F32, 1.0, 6), (2, 5, 1001, W.BF16, 1e-6, 7)])
def test_sampled_verifier_is_bit_exact(F, oracle, case):
    # the sampler is defined in binary32 arithmetic on both sides: the sampled tokens,
    # and with them every accept decision, must agree exactly
    N, B, V, dtype, temperature, seed = case
    print_case(test="spec_sampled_verify", case=case)
    rng = np.random.default_rng(hash(case[:3]) % 2**32 + 9)
    logits, mask, scaffold, _, tokens = synth(rng, N, B, V, dtype, 0.0)
    none = np.full((N, B), -1, dtype=np.int32)
    sampled = oracle.verify_step(logits, mask, scaffold, none, tokens, temperature=temperature, seed=seed)["ar_tokens"]
    # drafts that agree with the sampled tokens on most positions
    draft = np.where(rng.random((N, B)) < 0.85, sampled, (sampled + 1) % V).astype(np.int32)
    ref = oracle.verify_step(logits, mask, scaffold, draft, tokens, temperature=temperature, seed=seed)
    m, t = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    _, nacc, acc = F.fdd_verify_step(to_dev(logits), m, torch.from_numpy(scaffold).cuda(), torch.from_numpy(draft).cuda(), t,
                                     temperature=temperature, seed=seed)
    # all sampled tokens, not only those the scan reaches: verify against drafts that never match
    m2, t2 = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    first = np.zeros((N, B), dtype=bool)
    elig = (mask == 1) & (scaffold == 0)
    for n in range(N):
        idx = np.nonzero(elig[n])[0]
        if len(idx):
            first[n, idx[0]] = True
    F.fdd_verify_step(to_dev(logits), m2, torch.from_numpy(scaffold).cuda(), torch.from_numpy(none).cuda(), t2,
                      temperature=temperature, seed=seed)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), ref["tokens"])
    np.testing.assert_array_equal(m.cpu().numpy(), ref["mask"])
    np.testing.assert_array_equal(nacc.cpu().numpy(), ref["n_accepted"])
    np.testing.assert_array_equal(acc.cpu().numpy(), ref["accepted"])
    np.testing.assert_array_equal(t2.cpu().numpy()[first], sampled[first])
    # sampling is not the arg max (except at the near-zero temperature case)
    greedy = W.widen(logits, dtype).argmax(-1)
    if temperature > 0.1:
        assert np.mean(sampled[elig] == greedy[elig]) < 0.9
    print(f"accepted per block: {ref['n_accepted'].tolist()}")


def test_sampled_tokens_of_every_row_match_oracle(F, oracle):
    # one draft position per block, so that the scan exposes the sampled token of every row
    print_case(test="spec_sampled_rows")
    rng = np.random.default_rng(21)
    N, B, V = 64, 4, 3000
    logits = W.to_storage((rng.standard_normal((N, B, V)) * 2).astype(np.float32), W.BF16)
    mask = np.zeros((N, B), dtype=np.uint8)
    mask[np.arange(N), rng.integers(0, B, N)] = 1
    none = np.full((N, B), -1, dtype=np.int32)
    tokens = np.zeros((N, B), dtype=np.int32)
    ref = oracle.verify_step(logits, mask, None, none, tokens, temperature=0.8, seed=99)
    m, t = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    F.fdd_verify_step(to_dev(logits), m, None, torch.from_numpy(none).cuda(), t, temperature=0.8, seed=99)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(t.cpu().numpy(), ref["tokens"])
    assert len(set(ref["tokens"][mask == 1].tolist())) > 30
