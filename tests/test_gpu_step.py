"""The whole denoise step chained on the GPU vs the oracle: attention,
unmask, K/V refresh, over several consecutive steps on one shared prefix
(the shape of the long multi-camera configuration, reduced so that the
oracle finishes in seconds)."""
import numpy as np
import pytest
import torch

import fdd_workloads as W
from tests.gpu_util import print_case, to_dev, to_f64

pytestmark = pytest.mark.gpu


def test_multi_step_denoise_matches_oracle(oracle):
    import paper_2605_23163_amd as F
    w = W.Workload("mini5", N=4, B=64, L=1200, Hq=28, Hkv=4, D=128, dtype=W.BF16, V=8192, logit_std=2.0,
                   spike=12.0, spike_frac=0.3, scaffold_frac=0.30, tau=0.9, steps=4, table_rows=512, seed=55)
    print_case(test="multi_step", workload=w.name)
    d = W.full_step_inputs(w)
    tau = float(np.float32(w.tau))
    # oracle state
    o = {k: d[k].copy() for k in ("block_k", "block_v", "tokens", "mask")}
    # device state; the N rollouts start as forks of rollout 0's block state
    g = {k: to_dev(d[k]) for k in ("q", "prefix_k", "prefix_v", "table_k", "table_v")}
    g["scaffold"] = torch.from_numpy(d["scaffold_mask"]).cuda()
    for k in ("block_k", "block_v", "tokens", "mask"):
        o[k][:] = o[k][:1]
        g[k] = F.fdd_fork_block(to_dev(d[k][0]), w.N)
    prefix_ptr = g["prefix_k"].data_ptr()
    total_commits = 0
    for step in range(w.steps):
        logits = W.step_logits(w, o["mask"], d["logit_rngs"][step])
        ref_out = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], o["block_k"], o["block_v"])
        r = oracle.unmask_step(logits, o["mask"], d["scaffold_mask"], o["tokens"], tau)
        o["tokens"], o["mask"] = r["tokens"], r["mask"]
        o["block_k"], o["block_v"] = oracle.block_kv_update(o["tokens"], r["committed"], d["table_k"], d["table_v"],
                                                            o["block_k"], o["block_v"])
        out = F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], g["block_k"], g["block_v"], g["scaffold"])
        if step % 2 == 0:
            _, conf, nun, com = F.fdd_unmask_step(to_dev(logits), g["mask"], g["scaffold"], tau, g["tokens"])
            F.fdd_block_kv_update(g["tokens"], com, g["table_k"], g["table_v"], g["block_k"], g["block_v"])
        else:       # the same refresh done by the unmask call itself
            _, conf, nun, com = F.fdd_unmask_step(to_dev(logits), g["mask"], g["scaffold"], tau, g["tokens"],
                                                  refresh=(g["table_k"], g["table_v"], g["block_k"], g["block_v"]))
        torch.cuda.synchronize()
        err = np.abs(to_f64(out) - ref_out).max()
        assert err <= 2e-2, f"step {step}: attention max-abs {err}"
        near = np.abs(r["confidences"] - tau) < 1e-3
        assert not near.any(), "seed produced a near-tau confidence; pick another"
        np.testing.assert_array_equal(g["tokens"].cpu().numpy(), o["tokens"])
        np.testing.assert_array_equal(g["mask"].cpu().numpy(), o["mask"])
        np.testing.assert_array_equal(nun.cpu().numpy(), r["n_unmasked"])
        assert torch.equal(g["block_k"], to_dev(o["block_k"])) and torch.equal(g["block_v"], to_dev(o["block_v"]))
        total_commits += int(r["n_unmasked"].sum())
    assert g["prefix_k"].data_ptr() == prefix_ptr        # the prefix was never copied or replaced
    assert total_commits >= w.steps * w.N                # at least one commit per block per step
    sc = d["scaffold_mask"] == 1
    forked_tokens = np.broadcast_to(d["tokens"][:1], d["tokens"].shape)
    np.testing.assert_array_equal(g["tokens"].cpu().numpy()[sc], forked_tokens[sc])   # scaffold never rewritten


def test_config5_two_steps_in_the_bench_configuration(oracle):
    # The long multi-camera configuration at full size, launched as bench.py launches it (prefix V laid
    # out once, caller-owned workspaces, outputs reused): attention on sampled rows, the unmask decisions
    # of every position, the refreshed K/V rows, over two consecutive steps.
    import paper_2605_23163_amd as F
    w = W.CONFIGS["cfg5"]
    print_case(test="cfg5_bench_configuration")
    d = W.full_step_inputs(w, n_logit_steps=2)
    tau = float(np.float32(w.tau))
    g = {k: to_dev(d[k]) for k in ("q", "prefix_k", "prefix_v", "table_k", "table_v")}
    scaffold = torch.from_numpy(d["scaffold_mask"]).cuda()
    o = {k: np.broadcast_to(d[k][:1], d[k].shape).copy() for k in ("block_k", "block_v", "tokens", "mask")}
    st = {k: F.fdd_fork_block(to_dev(d[k][0]) if d[k].dtype == np.uint16 else torch.from_numpy(d[k][0]).cuda(), w.N)
          for k in ("block_k", "block_v", "tokens", "mask")}
    packed = F.fdd_prefix_pack(g["prefix_v"])
    out = torch.empty_like(g["q"])
    ws_a = torch.empty(max(256, F.fdd_block_attn_workspace(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"],
                                                           prefix_v_packed=packed)), dtype=torch.uint8, device="cuda")
    conf = torch.empty((w.N, w.B), dtype=torch.float32, device="cuda")
    nun = torch.empty((w.N,), dtype=torch.int32, device="cuda")
    com = torch.empty((w.N, w.B), dtype=torch.uint8, device="cuda")
    ws_u = None
    for step in range(2):
        logits = W.step_logits(w, o["mask"], d["logit_rngs"][step])
        tl = to_dev(logits)
        if ws_u is None:
            ws_u = torch.empty(max(256, F.fdd_unmask_workspace(tl)), dtype=torch.uint8, device="cuda")
        F.fdd_block_attn(g["q"], g["prefix_k"], g["prefix_v"], st["block_k"], st["block_v"], scaffold, out=out,
                         workspace=ws_a, prefix_v_packed=packed)
        # (the K/V refresh of the committed positions rides on the unmask call, as in bench.py)
        F.fdd_unmask_step(tl, st["mask"], scaffold, tau, st["tokens"], conf, nun, com, workspace=ws_u,
                          refresh=(g["table_k"], g["table_v"], st["block_k"], st["block_v"]))
        torch.cuda.synchronize()
        # every output row of the step against the oracle
        ref = oracle.block_attn(d["q"], d["prefix_k"], d["prefix_v"], o["block_k"], o["block_v"])
        err = np.abs(to_f64(out) - ref).max()
        print(f"step {step}: attention max-abs err over all rows {err:.3e}", flush=True)
        assert err <= 2e-2, f"step {step}: attention max-abs {err}"
        r = oracle.unmask_step(logits, o["mask"], d["scaffold_mask"], o["tokens"], tau)
        elig = (o["mask"] == 1) & (d["scaffold_mask"] == 0)
        near = elig & (np.abs(r["confidences"] - tau) < 1e-3)
        assert not near.any()
        # A forced single commit compares confidences across positions (fp32 sums on the GPU, fp64 in the
        # oracle): when the two best fp64 confidences of a block are within 1e-6 relative, either position is a
        # valid commit.  The oracle's state then follows the GPU's choice, so that the chain stays comparable.
        got_tok, got_mask, got_com = st["tokens"].cpu().numpy(), st["mask"].cpu().numpy(), com.cpu().numpy()
        for n in range(w.N):
            if np.array_equal(got_tok[n], r["tokens"][n]) and np.array_equal(got_mask[n], r["mask"][n]):
                continue
            c = np.sort(r["confidences"][n][elig[n]])[::-1]
            forced = not (r["confidences"][n][elig[n]] >= tau).any()
            assert forced and len(c) > 1 and (c[0] - c[1]) <= 1e-6 * c[0], f"step {step}, block {n}: decisions differ"
            b = np.flatnonzero(got_com[n])
            assert len(b) == 1 and elig[n, b[0]] and r["confidences"][n, b[0]] >= c[0] * (1 - 1e-6)
            assert got_tok[n, b[0]] == r["candidates"][n, b[0]]
            untouched = np.ones(w.B, dtype=bool)
            untouched[b[0]] = False
            np.testing.assert_array_equal(got_tok[n][untouched], o["tokens"][n][untouched])
            np.testing.assert_array_equal(got_mask[n][untouched], o["mask"][n][untouched])
            print(f"step {step}, block {n}: forced-commit near-tie, the GPU's candidate accepted", flush=True)
            r["tokens"][n], r["mask"][n], r["committed"][n] = got_tok[n], got_mask[n], got_com[n]
        np.testing.assert_array_equal(nun.cpu().numpy(), r["n_unmasked"])
        np.testing.assert_allclose(conf.cpu().numpy()[elig], r["confidences"][elig], rtol=2e-5)
        o["tokens"], o["mask"] = r["tokens"], r["mask"]
        o["block_k"], o["block_v"] = oracle.block_kv_update(o["tokens"], r["committed"], d["table_k"], d["table_v"],
                                                            o["block_k"], o["block_v"])
        assert torch.equal(st["block_k"], to_dev(o["block_k"])) and torch.equal(st["block_v"], to_dev(o["block_v"]))
        del tl
