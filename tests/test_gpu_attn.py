"""GPU parity of fdd_block_attn against the fp64 oracle (through the C ABI).

Tolerances are the task's: max-abs 2e-2 for bf16 storage, 1e-4 for fp32.
"""
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
    assert torch.cuda.is_available()
    return F


def run_gpu(F, d, **kw):
    t = {k: to_dev(v) for k, v in d.items() if k in ("q", "prefix_k", "prefix_v", "block_k", "block_v")}
    out = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], **kw)
    torch.cuda.synchronize()
    return out


def check(F, oracle, d, dtype, scale=None, **kw):
    out = to_f64(run_gpu(F, d, scale=scale, **kw))
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], scale=scale)
    err = np.abs(out - ref).max()
    assert np.isfinite(out).all()
    assert err <= TOL[dtype], f"max-abs error {err}"
    return out, err


# shapes that span several M-tiles and key tiles, with ragged ends on every axis
SHAPES = [
    # N, B,  L,   Hq, Hkv, D
    (1, 8, 256, 4, 1, 64),        # the tiny configuration
    (1, 1, 77, 4, 2, 64),         # B = 1: causal decode step
    (2, 5, 130, 6, 2, 128),       # nothing a multiple of a tile
    (3, 20, 333, 14, 2, 128),     # 420 stacked rows: 2 M-tiles, rollouts straddle wavefronts
    (5, 32, 1000, 28, 4, 128),    # G = 7, 1120 rows per KV head
    (2, 70, 64, 8, 8, 64),        # B > key tile: two tail tiles; G = 1
    (4, 16, 0, 4, 2, 128),        # no prefix at all
    (9, 3, 200, 3, 1, 64),        # many tiny rollouts inside one wavefront tile
]


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("shape", SHAPES)
def test_matches_oracle(F, oracle, shape, dtype):
    N, B, L, Hq, Hkv, D = shape
    print_case(test="attn_parity", shape=shape, dtype=dtype)
    rng = np.random.default_rng(hash(shape) % 2**32)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    check(F, oracle, d, dtype)


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("splits", [1, 2, 3, 7, 16])
def test_result_does_not_depend_on_split_count(F, oracle, dtype, splits):
    print_case(test="attn_splits", splits=splits, dtype=dtype)
    rng = np.random.default_rng(5)
    d = rand_attn(rng, 2, 12, 700, 8, 2, 128, dtype)
    check(F, oracle, d, dtype, splits=splits)


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_task_configurations_full(F, oracle, name):
    w = W.CONFIGS[name]
    print_case(test="attn_cfg", cfg=name)
    d = W.attention_inputs(w)
    _, err = check(F, oracle, d, w.dtype)
    print(f"{name}: max-abs err {err:.3e}")


def test_custom_scale_and_large_scores(F, oracle):
    print_case(test="attn_scale")
    rng = np.random.default_rng(11)
    d = rand_attn(rng, 2, 8, 300, 4, 2, 128, W.BF16, std=3.0)     # scores of magnitude ~100: sharp softmax
    unit = rand_attn(rng, 2, 8, 300, 4, 2, 128, W.BF16)           # values stay N(0,1): the tolerance is absolute
    d["prefix_v"], d["block_v"] = unit["prefix_v"], unit["block_v"]
    check(F, oracle, d, W.BF16, scale=0.11)


def test_b1_single_rollout_is_causal_decode(F, oracle):
    print_case(test="attn_b1")
    rng = np.random.default_rng(12)
    d = rand_attn(rng, 1, 1, 513, 28, 4, 128, W.BF16)
    out, _ = check(F, oracle, d, W.BF16)
    # textbook causal attention, last row, via torch on the CPU in fp64
    G = 7
    K = torch.from_numpy(np.concatenate([W.widen(d["prefix_k"], W.BF16), W.widen(d["block_k"], W.BF16)[0]], 0))
    V = torch.from_numpy(np.concatenate([W.widen(d["prefix_v"], W.BF16), W.widen(d["block_v"], W.BF16)[0]], 0))
    Q = torch.from_numpy(W.widen(d["q"], W.BF16))[0]                      # [1, Hq, D]
    ref = torch.nn.functional.scaled_dot_product_attention(
        Q.permute(1, 0, 2), K.permute(1, 0, 2).repeat_interleave(G, 0), V.permute(1, 0, 2).repeat_interleave(G, 0))
    assert np.abs(out[0, 0] - ref[:, 0, :].numpy()).max() <= 2e-2


def test_identical_forked_rollouts_give_identical_outputs(F):
    print_case(test="attn_fork_identical")
    w = W.Workload("fork", N=6, B=32, L=1500, Hq=28, Hkv=4, D=128, dtype=W.BF16, seed=21)
    d = W.attention_inputs(w, identical_blocks=True)
    # with a fixed number of pieces per M-tile every row sees the same tiles in
    # the same order, so forked rollouts agree bit for bit
    out = run_gpu(F, d, splits=3)
    for n in range(1, w.N):
        assert torch.equal(out[n], out[0])
    # the automatic (equal work per compute unit) schedule may cut the key range
    # of different M-tiles at different places; probabilities are then rounded to
    # bf16 against different reference maxima, so forked rollouts agree to that
    # rounding noise (far inside the 2e-2 parity tolerance), not bit for bit
    out = run_gpu(F, d).to(torch.float32)
    for n in range(1, w.N):
        assert float((out[n] - out[0]).abs().max()) <= 2e-3


def test_shared_prefix_equals_per_rollout_calls(F):
    print_case(test="attn_shared_vs_copied")
    rng = np.random.default_rng(13)
    N = 4
    d = rand_attn(rng, N, 32, 900, 28, 4, 128, W.BF16)
    t = {k: to_dev(v) for k, v in d.items()}
    shared = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], splits=4)
    for n in range(N):
        pk, pv = t["prefix_k"].clone(), t["prefix_v"].clone()            # a private copy of the prefix
        one = F.fdd_block_attn(t["q"][n:n + 1].contiguous(), pk, pv, t["block_k"][n:n + 1].contiguous(),
                               t["block_v"][n:n + 1].contiguous(), splits=4)
        torch.cuda.synchronize()
        # same tiles, same order, same split points: identical bits
        assert torch.equal(one[0], shared[n])


def test_other_rollouts_blocks_are_invisible_and_scaffold_mask_is_inert(F):
    print_case(test="attn_isolation")
    rng = np.random.default_rng(14)
    d = rand_attn(rng, 3, 10, 100, 4, 2, 64, W.BF16)
    a = run_gpu(F, d)
    d2 = dict(d)
    bk = W.bf16_bits_to_f32(d["block_k"]).copy()
    bk[1] += 4.0
    d2["block_k"] = W.to_storage(bk, W.BF16)
    b = run_gpu(F, d2)
    assert torch.equal(a[0], b[0]) and torch.equal(a[2], b[2]) and not torch.equal(a[1], b[1])
    sc = torch.from_numpy((rng.random((3, 10)) < 0.5).astype(np.uint8)).cuda()
    c = run_gpu(F, d, scaffold_mask=sc)
    assert torch.equal(a, c)


def test_prepacked_prefix_v_gives_the_same_bits(F, oracle):
    print_case(test="attn_prefix_pack")
    rng = np.random.default_rng(15)
    for shape in [(4, 32, 1000, 28, 4, 128), (1, 16, 300, 4, 2, 64), (3, 40, 64, 8, 2, 128), (2, 8, 63, 4, 1, 64)]:
        N, B, L, Hq, Hkv, D = shape
        d = rand_attn(rng, N, B, L, Hq, Hkv, D, W.BF16)
        t = {k: to_dev(v) for k, v in d.items()}
        packed = F.fdd_prefix_pack(t["prefix_v"])
        assert (packed is None) == (L < 64)
        plain = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"])
        pre = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], prefix_v_packed=packed)
        torch.cuda.synchronize()
        ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"])
        assert np.abs(to_f64(pre) - ref).max() <= 2e-2
        # the kernel that reads V as it lies and the one that reads it repacked see the same values in the
        # same order: same bits
        assert torch.equal(plain, pre)
        # the call repacks V itself only for very large problems; then the workspace shrinks by the packed
        # copy when the caller brings it
        a = F.fdd_block_attn_workspace(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"])
        b = F.fdd_block_attn_workspace(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"],
                                       prefix_v_packed=packed) if packed is not None else a
        assert a - b in (0, F.fdd_prefix_pack_bytes(t["prefix_v"]))
    big = dict(N=16, B=64, L=32768, Hq=28, Hkv=4, D=128)        # host arithmetic only: sizes of a problem that is repacked in the call
    from paper_2605_23163_amd import binding as bd
    import ctypes as C
    p = bd.AttnParams()
    for k, v in big.items():
        setattr(p, k, v)
    p.dtype = bd.FDD_BF16
    lib = F.load_library()
    with_pack = lib.fdd_block_attn_workspace(C.byref(p))
    p.prefix_v_packed = 256
    assert with_pack - lib.fdd_block_attn_workspace(C.byref(p)) == lib.fdd_prefix_pack_bytes(32768, 4, 128, bd.FDD_BF16)


def test_repeated_calls_are_bitwise_reproducible(F):
    print_case(test="attn_repro")
    d = W.attention_inputs(W.CONFIGS["cfg2"])
    a = run_gpu(F, d)
    for _ in range(3):
        assert torch.equal(a, run_gpu(F, d))


@pytest.mark.parametrize("name", ["cfg3", "cfg5"])
def test_full_size_every_row(F, oracle, name):
    # at the sizes the benchmark times: EVERY output row against the oracle, for the plain call (the call
    # lays V out itself) and for the call the benchmark makes (prefix V laid out beforehand by the caller)
    w = W.CONFIGS[name]
    print_case(test="attn_full_size", cfg=name)
    d = W.attention_inputs(w)
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"])
    t = {k: to_dev(v) for k, v in d.items()}
    plain = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"])
    packed = F.fdd_prefix_pack(t["prefix_v"])
    pre = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], prefix_v_packed=packed)
    torch.cuda.synchronize()
    for label, out in (("plain", plain), ("prefix_v_packed", pre)):
        o = to_f64(out)
        assert o.shape == ref.shape and np.isfinite(o).all()
        err = np.abs(o - ref).max()
        print(f"{name} {label}: max-abs err over all {ref.shape[0] * ref.shape[1] * ref.shape[2]} rows {err:.3e}")
        assert err <= 2e-2, f"{name} {label}: max-abs error {err}"


# Shapes whose M-tiles are cut into S = 2, 3, 4, 5, 7, 9, 10 equal pieces of 32 tiles or more, which is where
# the share of a piece is weighted by the XCD it runs on, and two with many short pieces; every row is compared.
@pytest.mark.parametrize("shape", [(16, 64, 4096), (10, 64, 8192), (8, 64, 8192), (6, 64, 12288), (5, 64, 16384),
                                   (4, 64, 20480), (3, 64, 20480), (2, 64, 8192), (4, 64, 4096)])
def test_weighted_equal_pieces_every_row(F, oracle, shape):
    N, B, L = shape
    print_case(test="attn_weighted_pieces", shape=shape)
    rng = np.random.default_rng(1000 + N * 131 + L)
    d = rand_attn(rng, N, B, L, 28, 4, 128, W.BF16)
    t = {k: to_dev(v) for k, v in d.items()}
    packed = F.fdd_prefix_pack(t["prefix_v"])
    out = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], prefix_v_packed=packed)
    torch.cuda.synchronize()
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"])
    o = to_f64(out)
    err = np.abs(o - ref).max()
    print(f"N={N} B={B} L={L}: max-abs err over all rows {err:.3e}")
    assert np.isfinite(o).all() and err <= 2e-2
