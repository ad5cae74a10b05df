"""The trajectory section decoded end to end with every piece of the library, against the oracle:
shared prefix, N forked rollouts, three chained blocks, each block finished by rounds of
draft (bidirectional attention + unmask with tau = 0) and verify (causal attention + sampled
verifier + accept scan), K/V refresh of accepted positions, block commit into the rollout's
extension, and the mean of the rollouts' trajectories at the end.

There is no model here: logits are seeded and synthetic, and the attention outputs do not feed
them.  What is checked is the bookkeeping across calls (tokens, masks, accepted counts, refreshed
and committed K/V: bit-exact) and the attention of every pass on the evolving state (tolerance).
"""
import numpy as np
import pytest
import torch

import fdd_workloads as W
from tests.gpu_util import print_case, to_dev, to_f64

pytestmark = pytest.mark.gpu


def test_trajectory_section_with_forked_rollouts(oracle):
    import paper_2605_23163_amd as F
    print_case(test="trajectory_section_flow")
    rng = np.random.default_rng(314)
    N, B, L, Hq, Hkv, D, V, T = 4, 32, 700, 28, 4, 128, 4096, 256
    n_blocks, temperature = 3, 0.7
    bf = lambda *s: W.to_storage(rng.standard_normal(s).astype(np.float32), W.BF16)
    pk, pv = bf(L, Hkv, D), bf(L, Hkv, D)
    table_k, table_v = bf(T, Hkv, D), bf(T, Hkv, D)
    g_pk, g_pv, g_tk, g_tv = to_dev(pk), to_dev(pv), to_dev(table_k), to_dev(table_v)
    packed = F.fdd_prefix_pack(g_pv)
    ext_k = np.zeros((N, (n_blocks - 1) * B, Hkv, D), dtype=np.uint16)
    ext_v = np.zeros_like(ext_k)
    g_ek, g_ev = to_dev(ext_k), to_dev(ext_v)
    E = 0
    all_tokens = []
    rounds_total = 0
    for blk in range(n_blocks):
        # the schema fixes the scaffold of a block for every rollout; one parent state is forked N times
        scaffold1 = (rng.random(B) < 0.3).astype(np.uint8)
        scaffold = np.broadcast_to(scaffold1, (N, B)).copy()
        tokens1 = np.where(scaffold1 == 1, rng.integers(0, V, B), -1).astype(np.int32)
        mask1 = (1 - scaffold1).astype(np.uint8)
        bk1, bv1 = bf(B, Hkv, D), bf(B, Hkv, D)
        o = dict(tokens=oracle.fork_block(tokens1, N), mask=oracle.fork_block(mask1, N),
                 block_k=oracle.fork_block(bk1, N), block_v=oracle.fork_block(bv1, N))
        g = dict(tokens=F.fdd_fork_block(torch.from_numpy(tokens1).cuda(), N), mask=F.fdd_fork_block(torch.from_numpy(mask1).cuda(), N),
                 block_k=F.fdd_fork_block(to_dev(bk1), N), block_v=F.fdd_fork_block(to_dev(bv1), N))
        g_sc = torch.from_numpy(scaffold).cuda()
        for rnd in range(B + 1):
            if not o["mask"].any():
                break
            rounds_total += 1
            q = bf(N, B, Hq, D)
            g_q = to_dev(q)
            ekw = dict(ext_k=ext_k, ext_v=ext_v, E=E) if E else {}
            gkw = dict(ext_k=g_ek, ext_v=g_ev, E=E) if E else {}
            # draft: bidirectional pass, every masked value position drafted at once (tau = 0) on a scratch copy
            out_d = F.fdd_block_attn(g_q, g_pk, g_pv, g["block_k"], g["block_v"], g_sc, prefix_v_packed=packed, **gkw)
            mdm = W.to_storage((rng.standard_normal((N, B, V)) * 2).astype(np.float32), W.BF16)
            od = oracle.unmask_step(mdm, o["mask"], scaffold, o["tokens"], 0.0)
            gd_tok, gd_mask = g["tokens"].clone(), g["mask"].clone()
            F.fdd_unmask_step(to_dev(mdm), gd_mask, g_sc, 0.0, gd_tok)
            # verify: causal pass, sampled verifier; the AR head agrees with most drafts by construction
            out_v = F.fdd_block_attn(g_q, g_pk, g_pv, g["block_k"], g["block_v"], g_sc, prefix_v_packed=packed,
                                     causal_block=True, **gkw)
            ar = (rng.standard_normal((N, B, V)) * 1.0).astype(np.float32)
            agree = rng.random((N, B)) < 0.8
            nn, bb = np.nonzero(agree & (o["mask"] == 1))
            ar[nn, bb, od["tokens"][nn, bb]] += 25.0
            ar = W.to_storage(ar, W.BF16)
            seed = 1000 * blk + rnd
            ov = oracle.verify_step(ar, o["mask"], scaffold, od["tokens"], o["tokens"], temperature=temperature, seed=seed)
            _, g_nacc, g_acc = F.fdd_verify_step(to_dev(ar), g["mask"], g_sc, gd_tok, g["tokens"], temperature=temperature,
                                                 seed=seed)
            F.fdd_block_kv_update(g["tokens"], g_acc, g_tk, g_tv, g["block_k"], g["block_v"])
            torch.cuda.synchronize()
            # attention of both passes on the state before this round's commits
            for out, causal in ((out_d, False), (out_v, True)):
                ref = oracle.block_attn(q, pk, pv, o["block_k"], o["block_v"], causal_block=causal, **ekw)
                err = np.abs(to_f64(out) - ref).max()
                assert err <= 2e-2, f"block {blk} round {rnd} causal={causal}: max-abs {err}"
            np.testing.assert_array_equal(gd_tok.cpu().numpy(), od["tokens"])
            o["tokens"], o["mask"] = ov["tokens"], ov["mask"]
            o["block_k"], o["block_v"] = oracle.block_kv_update(o["tokens"], (ov["accepted"] > 0).astype(np.uint8), table_k,
                                                                table_v, o["block_k"], o["block_v"])
            np.testing.assert_array_equal(g["tokens"].cpu().numpy(), o["tokens"])
            np.testing.assert_array_equal(g["mask"].cpu().numpy(), o["mask"])
            np.testing.assert_array_equal(g_nacc.cpu().numpy(), ov["n_accepted"])
            np.testing.assert_array_equal(g_acc.cpu().numpy(), ov["accepted"])
            assert torch.equal(g["block_k"], to_dev(o["block_k"])) and torch.equal(g["block_v"], to_dev(o["block_v"]))
            assert (ov["n_accepted"][o["mask"].any(axis=1) | (ov["n_accepted"] > 0)] >= 1).all()
        assert not o["mask"].any(), "every block finishes"
        assert np.array_equal(o["tokens"][:, scaffold1 == 1], np.broadcast_to(tokens1[scaffold1 == 1], (N, int(scaffold1.sum()))))
        all_tokens.append(o["tokens"].copy())
        if blk < n_blocks - 1:
            ext_k, ext_v = oracle.block_commit(o["block_k"], o["block_v"], ext_k, ext_v, E)
            E = F.fdd_block_commit(g["block_k"], g["block_v"], g_ek, g_ev, E)
            torch.cuda.synchronize()
            assert torch.equal(g_ek, to_dev(ext_k)) and torch.equal(g_ev, to_dev(ext_v))
    # rollouts sampled differently in at least one block, and took fewer rounds than one position at a time would
    toks = np.concatenate(all_tokens, axis=1)
    assert len({tuple(r) for r in toks.tolist()}) > 1
    assert rounds_total < n_blocks * 22
    # a synthetic decoding of the trajectory tokens into 20 waypoints per rollout, then the mean over rollouts
    way = (toks[:, :40].astype(np.float32) % 97).reshape(N, 20, 2) * 0.25
    got = F.fdd_traj_mean(torch.from_numpy(way).cuda()).cpu().numpy()
    ref = oracle.traj_mean(way)
    assert np.abs(got - ref).max() <= 1e-5 * np.abs(ref).max()
