"""The denoise step recorded into a HIP graph and replayed: every replay must
reproduce the eager result.  The library allocates nothing and records no
memset, so the whole step (fork, prefix layout, attention with its split
merge, unmask, K/V refresh, verify, commit, trajectory mean) is capturable.
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
    return F


def test_traj_mean_matches_oracle(F, oracle):
    print_case(test="traj_mean")
    rng = np.random.default_rng(3)
    for N, shape in [(1, (20, 2)), (4, (20, 2)), (16, (20, 3)), (64, (1000,))]:
        t = (rng.standard_normal((N,) + shape) * 30).astype(np.float32)
        got = F.fdd_traj_mean(torch.from_numpy(t).cuda()).cpu().numpy().astype(np.float64)
        ref = oracle.traj_mean(t)
        tol = N * 2.0 ** -24 * np.abs(t).astype(np.float64).mean(0) + 1e-30      # fp32 running sum of N terms
        assert np.all(np.abs(got - ref) <= 2 * tol + 2.0 ** -24 * np.abs(ref))


def test_step_replays_from_a_hip_graph(F):
    print_case(test="graph_replay")
    w = W.Workload("graph", N=4, B=32, L=1024, Hq=28, Hkv=4, D=128, dtype=W.BF16, V=8192, scaffold_frac=0.4, tau=0.9,
                   spike=8.0, spike_frac=0.3, logit_std=2.0, seed=31)
    d = W.full_step_inputs(w, n_logit_steps=1)
    rng = np.random.default_rng(5)
    g = {k: to_dev(d[k]) for k in ("q", "prefix_k", "prefix_v", "table_k", "table_v")}
    logits = to_dev(d["logits"])
    scaffold = torch.from_numpy(d["scaffold_mask"]).cuda()
    parent = {k: to_dev(d[k][0]) if d[k].dtype == np.uint16 else torch.from_numpy(d[k][0]).cuda()
              for k in ("block_k", "block_v", "tokens", "mask")}
    st = {k: torch.empty((w.N,) + tuple(v.shape), dtype=v.dtype, device="cuda") for k, v in parent.items()}
    draft = torch.from_numpy(rng.integers(0, w.V, (w.N, w.B)).astype(np.int32)).cuda()
    ext_k = torch.zeros((w.N, w.B, w.Hkv, w.D), dtype=torch.bfloat16, device="cuda")   # filled completely by the commit
    ext_v = torch.zeros_like(ext_k)
    traj = torch.from_numpy(rng.standard_normal((w.N, 20, 2)).astype(np.float32)).cuda()
    out = torch.empty_like(g["q"])
    out2 = torch.empty_like(g["q"])
    conf = torch.empty((w.N, w.B), dtype=torch.float32, device="cuda")
    nun = torch.empty((w.N,), dtype=torch.int32, device="cuda")
    com = torch.empty((w.N, w.B), dtype=torch.uint8, device="cuda")
    nacc = torch.empty((w.N,), dtype=torch.int32, device="cuda")
    acc = torch.empty((w.N, w.B), dtype=torch.uint8, device="cuda")
    tmean = torch.empty((20, 2), dtype=torch.float32, device="cuda")
    packed = torch.empty(F.fdd_prefix_pack_bytes(g["prefix_v"]), dtype=torch.uint8, device="cuda")
    ws_a = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                           splits=4, prefix_v_packed=packed, ext_k=ext_k, ext_v=ext_v, E=w.B)),
                       dtype=torch.uint8, device="cuda")
    ws_u = torch.empty(max(256, F.fdd_unmask_workspace(logits)), dtype=torch.uint8, device="cuda")

    def step():
        for k in parent:
            F.fdd_fork_block(parent[k], w.N, dst=st[k])
        F.fdd_prefix_pack(g["prefix_v"], packed=packed)
        F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], scaffold, out=out,
                         workspace=ws_a, splits=4, prefix_v_packed=packed)
        F.fdd_unmask_step(logits, st["mask"], scaffold, 0.9, st["tokens"], conf, nun, com, workspace=ws_u)
        F.fdd_block_kv_update(st["tokens"], com, g["table_k"], g["table_v"], st["block_k"], st["block_v"])
        F.fdd_verify_step(logits, st["mask"], scaffold, draft, st["tokens"], nacc, acc, workspace=ws_u,
                          temperature=0.8, seed=7)
        F.fdd_block_commit(st["block_k"], st["block_v"], ext_k, ext_v, 0)
        F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], scaffold, out=out2,
                         workspace=ws_a, splits=4, prefix_v_packed=packed, causal_block=True, ext_k=ext_k, ext_v=ext_v, E=w.B)
        F.fdd_traj_mean(traj, out=tmean)

    results = (out, out2, conf, nun, com, nacc, acc, tmean, ext_k, ext_v, st["tokens"], st["mask"], st["block_k"])

    def scrub():
        # eager work between replays: every output is overwritten, so a replay that did nothing would be seen
        for t in results:
            t.fill_(3) if t.dtype in (torch.uint8, torch.int32) else t.fill_(float("nan"))
        torch.cuda.synchronize()

    step()
    torch.cuda.synchronize()
    eager = [t.clone() for t in results]

    scrub()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                              # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step()
    for replay in range(3):
        scrub()
        graph.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(results, eager)):
            same = torch.equal(a.view(torch.uint8) if a.dtype != torch.bool else a, b.view(torch.uint8))
            assert same, f"replay {replay}: result {i} differs from the eager run"
