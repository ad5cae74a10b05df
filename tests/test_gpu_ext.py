"""GPU parity of the per-rollout extension (blocks committed since the fork) and
of fdd_block_commit against the oracle."""
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


def rand_ext(rng, N, Ecap, Hkv, D, dtype):
    return (W.to_storage(rng.standard_normal((N, Ecap, Hkv, D)).astype(np.float32), dtype),
            W.to_storage(rng.standard_normal((N, Ecap, Hkv, D)).astype(np.float32), dtype))


# (N, B, L, Hq, Hkv, D, E, Ecap)
SHAPES = [(1, 8, 256, 4, 1, 64, 8, 8), (3, 20, 333, 14, 2, 128, 37, 40), (2, 32, 64, 8, 8, 64, 64, 96),
          (4, 16, 0, 4, 2, 128, 100, 128), (9, 32, 1000, 28, 4, 128, 64, 64), (5, 70, 200, 7, 1, 128, 130, 140),
          (16, 32, 4096, 28, 4, 128, 32, 64)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("shape", SHAPES)
def test_extension_matches_oracle(F, oracle, shape, dtype, causal):
    N, B, L, Hq, Hkv, D, E, Ecap = shape
    if dtype == W.F32 and N * B * Hq * (L + E + B) > 3e7:
        pytest.skip("fp32 path is for small exactness checks")
    print_case(test="ext_attn", shape=shape, dtype=dtype, causal=causal)
    rng = np.random.default_rng(hash(shape) % 2**32 + 3)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    ek, ev = rand_ext(rng, N, Ecap, Hkv, D, dtype)
    t = {k: to_dev(v) for k, v in d.items()}
    tek, tev = to_dev(ek), to_dev(ev)
    if Ecap > E:      # rows beyond E must not be read into the result
        junk = torch.full_like(tek[:, E:], float("nan"))
        tek[:, E:] = junk
        tev[:, E:] = junk
    out = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], causal_block=causal,
                           ext_k=tek, ext_v=tev, E=E)
    torch.cuda.synchronize()
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], causal_block=causal,
                            ext_k=ek, ext_v=ev, E=E)
    err = np.abs(to_f64(out) - ref).max()
    assert err <= TOL[dtype], f"max-abs error {err}"
    # E = 0 with the same pointers is the plain two-run form
    plain = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], causal_block=causal)
    e0 = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], causal_block=causal,
                          ext_k=tek, ext_v=tev, E=0)
    assert torch.equal(plain, e0) and not torch.equal(plain, out)


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_block_commit_is_bit_exact(F, oracle, dtype):
    print_case(test="block_commit", dtype=dtype)
    rng = np.random.default_rng(8)
    N, B, Hkv, D, Ecap = 5, 32, 4, 128, 100
    bk, bv = rand_ext(rng, N, B, Hkv, D, dtype)
    ek, ev = rand_ext(rng, N, Ecap, Hkv, D, dtype)
    for E in (0, 32, 68):
        tek, tev = to_dev(ek), to_dev(ev)
        assert F.fdd_block_commit(to_dev(bk), to_dev(bv), tek, tev, E) == E + B
        torch.cuda.synchronize()
        rk, rv = oracle.block_commit(bk, bv, ek, ev, E)
        view = (lambda x: x.view(torch.int16).cpu().numpy().view(np.uint16)) if dtype == W.BF16 else (lambda x: x.cpu().numpy())
        assert np.array_equal(view(tek), rk) and np.array_equal(view(tev), rv)
    with pytest.raises(F.FddError):
        F.fdd_block_commit(to_dev(bk), to_dev(bv), to_dev(ek), to_dev(ev), 69)


def test_three_block_lifecycle_after_a_fork(F, oracle):
    # fork, then three blocks per rollout: attend, commit, attend with a longer extension.
    # Every block's output must match the oracle given the same extension, and the extension
    # built on the GPU must equal the one the oracle builds.
    print_case(test="ext_lifecycle")
    rng = np.random.default_rng(12)
    N, B, L, Hq, Hkv, D = 6, 32, 2048, 28, 4, 128
    pre = rand_attn(rng, N, B, L, Hq, Hkv, D, W.BF16)
    pk, pv = to_dev(pre["prefix_k"]), to_dev(pre["prefix_v"])
    packed = F.fdd_prefix_pack(pv)
    ek_h = np.zeros((N, 2 * B, Hkv, D), dtype=np.uint16)
    ev_h = np.zeros((N, 2 * B, Hkv, D), dtype=np.uint16)
    ek, ev = to_dev(ek_h), to_dev(ev_h)
    E = 0
    for blk in range(3):
        d = rand_attn(rng, N, B, L, Hq, Hkv, D, W.BF16)
        q, bk, bv = to_dev(d["q"]), to_dev(d["block_k"]), to_dev(d["block_v"])
        out = F.fdd_block_attn(q, pk, pv, bk, bv, prefix_v_packed=packed, ext_k=ek, ext_v=ev, E=E)
        torch.cuda.synchronize()
        ref = oracle.block_attn(d["q"], pre["prefix_k"], pre["prefix_v"], d["block_k"], d["block_v"],
                                ext_k=ek_h, ext_v=ev_h, E=E)
        err = np.abs(to_f64(out) - ref).max()
        assert err <= 2e-2, f"block {blk}: max-abs error {err}"
        if blk < 2:
            ek_h, ev_h = oracle.block_commit(d["block_k"], d["block_v"], ek_h, ev_h, E)
            E = F.fdd_block_commit(bk, bv, ek, ev, E)
            torch.cuda.synchronize()
            assert np.array_equal(ek.view(torch.int16).cpu().numpy().view(np.uint16), ek_h)
    assert E == 2 * B


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("shape", [(3, 1, 32, 2048, 28, 4, 128, 0), (5, 2, 8, 333, 4, 1, 64, 8), (28, 1, 32, 256, 28, 4, 128, 0),
                                   (2, 9, 32, 1000, 28, 4, 128, 32)])
def test_batch_of_independent_problems(F, oracle, shape, dtype):
    # P problems of one shape in one launch: each must match the oracle on its own arrays, with and
    # without a prefix V laid out beforehand, and nothing may leak between problems
    P, N, B, L, Hq, Hkv, D, E = shape
    if dtype == W.F32 and P * N * B * Hq * (L + B) > 2e7:
        pytest.skip("fp32 path is for small exactness checks")
    print_case(test="batched_attn", shape=shape, dtype=dtype)
    rng = np.random.default_rng(hash(shape) % 2**32 + 17)
    probs = [rand_attn(rng, N, B, L, Hq, Hkv, D, dtype) for _ in range(P)]
    exts = [rand_ext(rng, N, max(E, 1), Hkv, D, dtype) for _ in range(P)]
    stack = lambda k: to_dev(np.stack([pr[k] for pr in probs]))
    q, pk, pv, bk, bv = (stack(k) for k in ("q", "prefix_k", "prefix_v", "block_k", "block_v"))
    ek, ev = to_dev(np.stack([e[0] for e in exts])), to_dev(np.stack([e[1] for e in exts]))
    kw = dict(ext_k=ek, ext_v=ev, E=E) if E else {}
    out = F.fdd_block_attn_batched(q, pk, pv, bk, bv, **kw)
    outs = [out]
    if dtype == W.BF16 and L >= 64:
        packed = torch.stack([F.fdd_prefix_pack(pv[i]) for i in range(P)])
        outs.append(F.fdd_block_attn_batched(q, pk, pv, bk, bv, prefix_v_packed=packed, **kw))
    torch.cuda.synchronize()
    for o in outs:
        for i in range(P):
            okw = dict(ext_k=exts[i][0], ext_v=exts[i][1], E=E) if E else {}
            ref = oracle.block_attn(probs[i]["q"], probs[i]["prefix_k"], probs[i]["prefix_v"], probs[i]["block_k"],
                                    probs[i]["block_v"], **okw)
            err = np.abs(to_f64(o[i]) - ref).max()
            assert err <= TOL[dtype], f"problem {i}: max-abs error {err}"
    # a change in one problem's prefix moves that problem's output only
    pk2 = pk.clone()
    pk2[P - 1] = pk2[P - 1] * 0.5
    out2 = F.fdd_block_attn_batched(q, pk2, pv, bk, bv, **kw)
    assert torch.equal(out2[: P - 1], out[: P - 1]) and not torch.equal(out2[P - 1], out[P - 1])


def test_seeded_random_shapes_and_options(F, oracle):
    # a sweep of small seeded shapes over every option of the attention call at once
    # (storage type, head size, GQA ratio, ragged L, B across tile borders, extension, causal, split count)
    rng = np.random.default_rng(2024)
    worst = 0.0
    for case in range(48):
        dtype = W.BF16 if case % 3 else W.F32
        D = int(rng.choice([64, 128]))
        Hkv = int(rng.choice([1, 2, 4]))
        G = int(rng.choice([1, 3, 7]))
        N = int(rng.integers(1, 12))
        B = int(rng.choice([1, 5, 16, 32, 40, 64, 65, 100]))
        L = int(rng.choice([0, 1, 63, 64, 65, 200, 777, 1024, 1500]))
        E = int(rng.choice([0, 0, 7, 64, 90]))
        Ecap = E + int(rng.integers(0, 9))
        causal = bool(rng.integers(0, 2))
        splits = int(rng.choice([0, 0, 1, 2, 5]))
        if dtype == W.F32 and N * B * Hkv * G * (L + E + B) > 2e6:
            N, L = min(N, 3), min(L, 200)
        print_case(test="random_shape", case=case, dtype=dtype, N=N, B=B, L=L, Hq=Hkv * G, Hkv=Hkv, D=D, E=E, causal=causal,
                   splits=splits)
        d = rand_attn(rng, N, B, L, Hkv * G, Hkv, D, dtype)
        ek, ev = rand_ext(rng, N, max(Ecap, 1), Hkv, D, dtype)
        t = {k: to_dev(v) for k, v in d.items()}
        kw = dict(ext_k=to_dev(ek), ext_v=to_dev(ev), E=E) if E else {}
        out = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], causal_block=causal,
                               splits=splits, **kw)
        torch.cuda.synchronize()
        okw = dict(ext_k=ek, ext_v=ev, E=E) if E else {}
        ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], causal_block=causal, **okw)
        err = np.abs(to_f64(out) - ref).max()
        assert err <= TOL[dtype], f"case {case}: max-abs error {err}"
        worst = max(worst, err / TOL[dtype])
    print(f"worst error / tolerance: {worst:.3f}")
