"""Host-side checks of the seeded input generators (CPU only)."""
import os

import numpy as np

import fdd_workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table1_sections.txt")


def read_table1():
    rows = {}
    with open(GOLDEN) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, v, s, b = line.split()
            rows[name] = (int(v), int(s), int(b))
    return rows


def test_section_layout_reproduces_table1_block_counts():
    # Table 1 of the paper: 1/6/1/3 blocks, 280 value + 124 scaffold tokens.
    # ceil(value/d) gives those block counts for d = 32 value tokens per block.
    t = read_table1()
    blocks = W.table1_block_layout(32)
    assert len(blocks) == t["total"][2] == 11
    for name, v, s in W.TABLE1_SECTIONS:
        mine = [m for n, m in blocks if n == name]
        assert (v, s, len(mine)) == t[name]
        assert sum(int((m == 0).sum()) for m in mine) == v
        assert sum(int(m.sum()) for m in mine) == s
        assert all((m == 0).sum() <= 32 for m in mine)
    tot_v = sum(int((m == 0).sum()) for _, m in blocks)
    tot_s = sum(int(m.sum()) for _, m in blocks)
    assert (tot_v, tot_s) == t["total"][:2]
    assert abs(tot_s / (tot_v + tot_s) - 0.30) < 0.02          # "~30 %" scaffold share
    # other block sizes do not reproduce the printed block counts
    assert len(W.table1_block_layout(16)) != 11 and len(W.table1_block_layout(64)) != 11


def test_bf16_rounding_is_nearest_even_and_exact_roundtrip():
    import torch
    x = np.random.default_rng(0).standard_normal(10000).astype(np.float32) * 37.0
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    np.testing.assert_array_equal(bits, ref)
    np.testing.assert_array_equal(W.f32_to_bf16_bits(W.bf16_bits_to_f32(bits)), bits)


def test_generators_are_seeded_and_shaped():
    w = W.CONFIGS["cfg1"]
    a, b = W.full_step_inputs(w), W.full_step_inputs(w)
    for k in a:
        np.testing.assert_array_equal(a[k], b[k])
    assert a["q"].shape == (1, 8, 4, 64) and a["q"].dtype == np.float32
    assert a["prefix_k"].shape == (256, 1, 64) and a["logits"].shape == (1, 8, 512)
    assert a["scaffold_mask"].sum() == 2                      # 25 % of 8
    assert np.all(a["mask"] == 1 - a["scaffold_mask"])
    w2 = W.CONFIGS["cfg2"]
    d = W.attention_inputs(w2)
    assert d["q"].dtype == np.uint16 and d["prefix_k"].shape == (2048, 4, 128)
    # per-channel scale on prefix K: channel stds spread over about [0.5, 2]
    std = W.bf16_bits_to_f32(d["prefix_k"]).std(axis=0)
    assert std.min() < 0.7 and std.max() > 1.6
    for name, w in W.CONFIGS.items():
        assert w.Hq % w.Hkv == 0 and w.D in (64, 128)
