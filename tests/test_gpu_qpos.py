"""GPU parity of attention over a list of query positions (only the listed block
positions get output rows; the scaffold's rows are skipped where only logits of
non-scaffold positions are read).  The listed rows must equal the oracle's rows
of the full problem, the other rows of `out` must stay as they were."""
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


def sentinel_like(t):
    return torch.full_like(t, 7.0)


def check(F, oracle, d, t, pos, dtype, causal=False, ext=None, E=0, **kw):
    """Run with the list `pos` and compare listed rows with the oracle, the rest with the sentinel."""
    N, B, Hq, D = d["q"].shape
    out = sentinel_like(t["q"])
    extk = {}
    if ext is not None:
        extk = dict(ext_k=to_dev(ext[0]), ext_v=to_dev(ext[1]), E=E)
    F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], out=out, causal_block=causal,
                     q_positions=torch.from_numpy(pos.astype(np.int32)).cuda(), **extk, **kw)
    torch.cuda.synchronize()
    got = to_f64(out).reshape(N * B, Hq, D)
    listed = np.zeros(N * B, dtype=bool)
    listed[pos] = True
    assert np.all(got[~listed] == 7.0), "rows outside the list were written"
    rows = np.stack([np.repeat(pos // B, Hq), np.repeat(pos % B, Hq), np.tile(np.arange(Hq), len(pos))], 1).astype(np.int32)
    okw = {}
    if ext is not None:
        okw = dict(ext_k=ext[0], ext_v=ext[1], E=E)
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], causal_block=causal,
                            rows=rows, **okw)
    g = got[rows[:, 0] * B + rows[:, 1], rows[:, 2]]
    err = np.abs(g - ref).max()
    assert err <= TOL[dtype], err
    return out


# (N, B, L, Hq, Hkv, D)
SHAPES = [(1, 8, 256, 4, 1, 64), (3, 20, 333, 14, 2, 128), (1, 32, 2048, 28, 4, 128), (9, 32, 1000, 28, 4, 128),
          (16, 64, 4096, 28, 4, 128), (5, 70, 0, 7, 1, 128)]


@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
@pytest.mark.parametrize("shape", SHAPES)
def test_listed_positions_match_oracle(F, oracle, shape, dtype, causal):
    N, B, L, Hq, Hkv, D = shape
    if dtype == W.F32 and N * B * Hq * (L + B) > 3e7:
        pytest.skip("fp32 path is for small exactness checks")
    print_case(test="qpos", shape=shape, dtype=dtype, causal=causal)
    rng = np.random.default_rng(hash(shape) % 2**32 + 11)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    t = {k: to_dev(v) for k, v in d.items()}
    # the non-scaffold positions of a 40 % scaffold, the same schema in every rollout
    scaffold = rng.random(B) < 0.4
    scaffold[rng.integers(B)] = False
    pos = np.flatnonzero(np.tile(~scaffold, N))
    check(F, oracle, d, t, pos, dtype, causal)


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_degenerate_lists(F, oracle, dtype):
    N, B, L, Hq, Hkv, D = 4, 16, 200, 8, 2, 64
    rng = np.random.default_rng(5)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    t = {k: to_dev(v) for k, v in d.items()}
    full = F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"])
    torch.cuda.synchronize()
    for name, pos in [("one position", np.array([37])), ("first and last", np.array([0, N * B - 1])),
                      ("one rollout only", np.arange(2 * B, 3 * B)), ("ragged", np.array([1, 2, 17, 18, 19, 40, 63]))]:
        print_case(test="qpos_degenerate", case=name, dtype=dtype)
        check(F, oracle, d, t, pos, dtype)
    # the list of all positions is the call without a list, bit for bit
    out = check(F, oracle, d, t, np.arange(N * B), dtype)
    assert torch.equal(out, full)


@pytest.mark.parametrize("dtype", [W.BF16, W.F32])
def test_list_with_extension_and_causal_block(F, oracle, dtype):
    N, B, L, Hq, Hkv, D, E, Ecap = 6, 24, 300, 14, 2, 128, 40, 48
    print_case(test="qpos_ext", dtype=dtype)
    rng = np.random.default_rng(9)
    d = rand_attn(rng, N, B, L, Hq, Hkv, D, dtype)
    t = {k: to_dev(v) for k, v in d.items()}
    ext = (W.to_storage(rng.standard_normal((N, Ecap, Hkv, D)).astype(np.float32), dtype),
           W.to_storage(rng.standard_normal((N, Ecap, Hkv, D)).astype(np.float32), dtype))
    pos = np.flatnonzero(rng.random(N * B) < 0.6)
    check(F, oracle, d, t, pos, dtype, causal=True, ext=ext, E=E)
    check(F, oracle, d, t, pos, dtype, causal=False, ext=ext, E=E)


def test_bench_configuration_with_list(F, oracle):
    """Config 5's shape (N=16, B=64, L=16384) with its 30 % scaffold skipped: every listed row against the oracle."""
    w = W.CONFIGS["cfg5"]
    print_case(test="qpos_cfg5")
    d = W.attention_inputs(w)
    t = {k: to_dev(v) for k, v in d.items()}
    rng = np.random.default_rng(w.seed)
    scaffold = W.scaffold_positions(w, rng)
    pos = np.flatnonzero(scaffold.reshape(-1) == 0)
    N, B, Hq, D = d["q"].shape
    out = sentinel_like(t["q"])
    F.fdd_block_attn(t["q"], t["prefix_k"], t["prefix_v"], t["block_k"], t["block_v"], out=out,
                     q_positions=torch.from_numpy(pos.astype(np.int32)).cuda())
    torch.cuda.synchronize()
    got = to_f64(out).reshape(N * B, Hq, D)
    listed = np.zeros(N * B, dtype=bool)
    listed[pos] = True
    assert np.all(got[~listed] == 7.0)
    # every listed row (all heads of every listed position) against the oracle
    rows = np.stack([np.repeat(pos // B, Hq), np.repeat(pos % B, Hq), np.tile(np.arange(Hq), len(pos))], 1).astype(np.int32)
    ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"], rows=rows)
    err = np.abs(got[rows[:, 0] * B + rows[:, 1], rows[:, 2]] - ref).max()
    print(f"cfg5 with list: max-abs err over all {len(rows)} listed rows {err:.3e}")
    assert err <= TOL[W.BF16], err


def test_batch_with_list(F, oracle):
    P, N, B, L, Hq, Hkv, D = 3, 2, 16, 128, 8, 2, 64
    print_case(test="qpos_batch")
    rng = np.random.default_rng(21)
    ds = [rand_attn(rng, N, B, L, Hq, Hkv, D, W.BF16) for _ in range(P)]
    stack = {k: torch.stack([to_dev(x[k]) for x in ds]) for k in ds[0]}
    pos = np.array([0, 3, 4, 15, 16, 30])
    lib = F.load_library()
    from paper_2605_23163_amd import binding as bd
    import ctypes as C
    out = torch.full_like(stack["q"], 7.0)
    p = bd._batched_params(stack["q"], stack["prefix_k"], stack["prefix_v"], stack["block_k"], stack["block_v"], out,
                           None, 0, None, False, None, None, 0)
    qp = torch.from_numpy(pos.astype(np.int32)).cuda()
    p.q_positions, p.n_q_positions = qp.data_ptr(), len(pos)
    need = lib.fdd_block_attn_workspace(C.byref(p))
    ws = torch.empty(max(need, 256), dtype=torch.uint8, device="cuda")
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel()
    assert lib.fdd_block_attn(C.byref(p)) == 0, lib.fdd_last_error()
    torch.cuda.synchronize()
    for i, d in enumerate(ds):
        got = to_f64(out[i]).reshape(N * B, Hq, D)
        ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], d["block_k"], d["block_v"]).reshape(N * B, Hq, D)
        listed = np.zeros(N * B, dtype=bool)
        listed[pos] = True
        assert np.all(got[~listed] == 7.0)
        assert np.abs(got[listed] - ref[listed]).max() <= TOL[W.BF16]
