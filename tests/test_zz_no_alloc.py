"""fdd_unmask_step_static (the entry point that allocates nothing and takes no
workspace) against fdd_unmask_step, through the C ABI: two calls in a row, the
second on a smaller input, every output bit for bit; then against the oracle.
"""
import ctypes as C

import numpy as np
import pytest
import torch

import fdd_workloads as W
from tests.gpu_util import print_case, to_dev

pytestmark = pytest.mark.gpu


def _state(rng, N, B, V, dtype):
    x = (rng.standard_normal((N, B, V)) * 2).astype(np.float32)
    hit = rng.random((N, B)) < 0.4
    ids = rng.integers(0, V, size=(N, B))
    n, b = np.nonzero(hit)
    x[n, b, ids[n, b]] += 14.0
    scaffold = (rng.random((N, B)) < 0.3).astype(np.uint8)
    mask = ((rng.random((N, B)) < 0.8) & (scaffold == 0)).astype(np.uint8)
    tokens = rng.integers(0, V, size=(N, B)).astype(np.int32)
    tokens[mask == 1] = -1
    return W.to_storage(x, dtype), mask, scaffold, tokens


def _call(lib, bd, entry, logits, mask, scaffold, tokens, tau, workspace):
    """One raw C-ABI call on private copies of the in/out state; returns the outputs as host arrays."""
    N, B, V = logits.shape
    m, t = torch.from_numpy(mask.copy()).cuda(), torch.from_numpy(tokens.copy()).cuda()
    sc = torch.from_numpy(scaffold).cuda()
    conf = torch.full((N, B), 123.0, dtype=torch.float32, device="cuda")
    nun = torch.full((N,), -7, dtype=torch.int32, device="cuda")
    com = torch.full((N, B), 9, dtype=torch.uint8, device="cuda")
    p = bd._unmask_params(logits, m, sc, t, tau, conf, nun, com)
    p.stream = bd._stream_ptr(None)
    if workspace is not None:
        p.workspace, p.workspace_bytes = workspace.data_ptr(), workspace.numel()
    else:
        p.workspace, p.workspace_bytes = None, 0
    rc = getattr(lib, entry)(C.byref(p))
    assert rc == 0, lib.fdd_last_error()
    torch.cuda.synchronize()
    return dict(tokens=t.cpu().numpy(), mask=m.cpu().numpy(), confidences=conf.cpu().numpy(),
                n_unmasked=nun.cpu().numpy(), committed=com.cpu().numpy())


def test_static_scratch_entry_point_matches_the_workspace_one(oracle):
    import paper_2605_23163_amd as F
    from paper_2605_23163_amd import binding as bd
    lib = F.load_library()
    rng = np.random.default_rng(2024)
    tau = float(np.float32(0.9))
    # two calls in a row on the same device array: a large shape with several pieces per row, then a smaller one
    for shape, dtype in (((6, 24, 152064), W.BF16), ((3, 7, 20011), W.BF16), ((2, 5, 999), W.F32)):
        N, B, V = shape
        print_case(test="no_alloc", shape=shape, dtype=dtype)
        logits_h, mask, scaffold, tokens = _state(rng, N, B, V, dtype)
        logits = to_dev(logits_h)
        p = bd._unmask_params(logits, torch.from_numpy(mask).cuda(), None, torch.from_numpy(tokens).cuda(), tau,
                              torch.empty((N, B), device="cuda"), None, None)
        ws = torch.empty(max(256, lib.fdd_unmask_workspace(C.byref(p))), dtype=torch.uint8, device="cuda")
        ref = _call(lib, bd, "fdd_unmask_step", logits, mask, scaffold, tokens, tau, ws)
        before = torch.cuda.memory_allocated()
        got = _call(lib, bd, "fdd_unmask_step_static", logits, mask, scaffold, tokens, tau, None)
        for k in ref:
            np.testing.assert_array_equal(got[k], ref[k], err_msg=k)
        assert torch.cuda.memory_allocated() == before
        o = oracle.unmask_step(logits_h, mask, scaffold, tokens, tau)
        el = (mask == 1) & (scaffold == 0)
        assert not (el & (np.abs(o["confidences"] - tau) < 1e-3)).any()
        np.testing.assert_array_equal(got["tokens"], o["tokens"])
        np.testing.assert_array_equal(got["mask"], o["mask"])
        np.testing.assert_array_equal(got["n_unmasked"], o["n_unmasked"])


def test_static_scratch_entry_point_rejects_what_does_not_fit():
    import paper_2605_23163_amd as F
    from paper_2605_23163_amd import binding as bd
    lib = F.load_library()
    print_case(test="no_alloc_limit")
    # 70000 positions x 1 piece x 16 bytes > 1 MiB: host-side refusal, nothing is launched (logits are never read)
    N, B, V = 700, 100, 64
    logits = torch.zeros((N, B, V), dtype=torch.float32, device="cuda")
    mask = torch.ones((N, B), dtype=torch.uint8, device="cuda")
    tokens = torch.full((N, B), -1, dtype=torch.int32, device="cuda")
    conf = torch.full((N, B), 5.0, dtype=torch.float32, device="cuda")
    p = bd._unmask_params(logits, mask, None, tokens, 0.5, conf, None, None)
    assert lib.fdd_unmask_workspace(C.byref(p)) > (1 << 20)
    assert lib.fdd_unmask_step_static(C.byref(p)) == 5          # FDD_ERR_WORKSPACE
    assert b"scratch" in lib.fdd_last_error()
    torch.cuda.synchronize()
    assert bool((conf == 5.0).all()) and bool((tokens == -1).all())
