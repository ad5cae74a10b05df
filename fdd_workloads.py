"""Seeded synthetic inputs for the block-diffusion denoise step.

This module only draws random numbers and rounds them to their storage type.
It holds none of the method's arithmetic (no attention, no softmax, no
unmask rule), so that the CPU oracle and the HIP path can both be fed the
same bytes without sharing any computation.

The paper evaluates on driving datasets with a trained 3B backbone; neither
is available, so the workloads below stand in for them: the shapes of a
decoder step of that model class (GQA heads, an image+prompt prefix, a 32 or
64 token section block) with a scaffold share that brackets the ~30 % the
paper's Table 1 reports.

Draw order for one workload (all from ``numpy.random.default_rng(seed)``):
q, prefix_k (then its per-channel scale), prefix_v, block_k, block_v,
scaffold positions, then -- per step -- logits, spike rows, spike ids, and
last the K/V refresh tables.  Arrays are rounded to the storage type before
anybody sees them; bf16 arrays are returned as uint16 bit patterns.
"""
from __future__ import annotations

import dataclasses
import numpy as np

BF16 = "bf16"
F32 = "f32"


@dataclasses.dataclass(frozen=True)
class Workload:
    name: str
    N: int
    B: int
    L: int
    Hq: int
    Hkv: int
    D: int
    dtype: str
    V: int = 0                 # 0: no unmask in this workload
    logit_std: float = 1.0
    spike: float = 0.0
    spike_frac: float = 0.0
    scaffold_frac: float = 0.0
    tau: float = 0.9
    steps: int = 1
    qkv_std: float = 1.0
    k_channel_scale: bool = False
    table_rows: int = 4096     # rows of the synthetic K/V refresh tables
    seed: int = 0


# The five configurations of the benchmark spec, in its order.
CONFIGS = {
    "cfg1": Workload("cfg1", N=1, B=8, L=256, Hq=4, Hkv=1, D=64, dtype=F32, V=512,
                     logit_std=1.0, spike=6.0, spike_frac=0.5, scaffold_frac=0.25,
                     tau=0.9, qkv_std=1.0 / 8.0, seed=0),
    "cfg2": Workload("cfg2", N=1, B=32, L=2048, Hq=28, Hkv=4, D=128, dtype=BF16,
                     scaffold_frac=0.40, k_channel_scale=True, seed=2),
    "cfg3": Workload("cfg3", N=8, B=32, L=4096, Hq=28, Hkv=4, D=128, dtype=BF16, seed=3),
    "cfg4": Workload("cfg4", N=8, B=32, L=4096, Hq=28, Hkv=4, D=128, dtype=BF16, V=152064,
                     logit_std=2.0, spike=8.0, spike_frac=0.30, scaffold_frac=0.50,
                     tau=0.9, seed=4),
    "cfg5": Workload("cfg5", N=16, B=64, L=16384, Hq=28, Hkv=4, D=128, dtype=BF16, V=152064,
                     logit_std=2.0, spike=8.0, spike_frac=0.30, scaffold_frac=0.30,
                     tau=0.9, steps=8, seed=5),
}


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32)
    return f32_to_bf16_bits(x) if dtype == BF16 else x


def widen(x: np.ndarray, dtype: str) -> np.ndarray:
    """Stored values as float64 (exact)."""
    if dtype == BF16:
        return bf16_bits_to_f32(x).astype(np.float64)
    return np.asarray(x, dtype=np.float64)


def _normal(rng, shape, std):
    x = rng.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        x *= np.float32(std)
    return x


def attention_inputs(w: Workload, rng=None, identical_blocks: bool = False):
    """q, prefix_k, prefix_v, block_k, block_v in storage type."""
    rng = np.random.default_rng(w.seed) if rng is None else rng
    q = _normal(rng, (w.N, w.B, w.Hq, w.D), w.qkv_std)
    pk = _normal(rng, (w.L, w.Hkv, w.D), w.qkv_std)
    if w.k_channel_scale:
        pk *= rng.uniform(0.5, 2.0, size=(w.Hkv, w.D)).astype(np.float32)
    pv = _normal(rng, (w.L, w.Hkv, w.D), w.qkv_std)
    bk = _normal(rng, (w.N, w.B, w.Hkv, w.D), w.qkv_std)
    bv = _normal(rng, (w.N, w.B, w.Hkv, w.D), w.qkv_std)
    if identical_blocks:
        q[:] = q[:1]
        bk[:] = bk[:1]
        bv[:] = bv[:1]
    return {k: to_storage(v, w.dtype) for k, v in
            dict(q=q, prefix_k=pk, prefix_v=pv, block_k=bk, block_v=bv).items()}


def scaffold_positions(w: Workload, rng, shared: bool = True) -> np.ndarray:
    """uint8 [N,B]; 1 marks a frozen structural token.

    A fixed output schema puts the scaffold at the same positions in every
    forked rollout, so by default one draw is shared by all N rollouts.
    """
    k = int(round(w.scaffold_frac * w.B))
    out = np.zeros((w.N, w.B), dtype=np.uint8)
    if shared:
        idx = rng.permutation(w.B)[:k]
        out[:, idx] = 1
    else:
        for n in range(w.N):
            out[n, rng.permutation(w.B)[:k]] = 1
    return out


def initial_state(w: Workload, scaffold: np.ndarray, rng, mask_token: int = -1):
    """Start of a block: every value position masked, scaffold ids filled in."""
    mask = (1 - scaffold).astype(np.uint8)
    tokens = np.full((w.N, w.B), mask_token, dtype=np.int32)
    ids = rng.integers(0, max(w.V, 2), size=(w.N, w.B), dtype=np.int32)
    tokens[scaffold == 1] = ids[scaffold == 1]
    return tokens, mask


def step_logits(w: Workload, mask: np.ndarray, rng) -> np.ndarray:
    """Logits [N,B,V] in storage type: noise plus a spike on some masked rows."""
    x = _normal(rng, (w.N, w.B, w.V), w.logit_std)
    hit = (rng.random((w.N, w.B)) < w.spike_frac) & (mask == 1)
    ids = rng.integers(0, w.V, size=(w.N, w.B))
    n_idx, b_idx = np.nonzero(hit)
    x[n_idx, b_idx, ids[n_idx, b_idx]] += np.float32(w.spike)
    return to_storage(x, w.dtype)


def kv_tables(w: Workload, rng):
    """Stand-in for embedding+projection of a committed token: row t of these
    tables is the K (V) row a position takes once token id t is written."""
    tk = _normal(rng, (w.table_rows, w.Hkv, w.D), w.qkv_std)
    tv = _normal(rng, (w.table_rows, w.Hkv, w.D), w.qkv_std)
    return to_storage(tk, w.dtype), to_storage(tv, w.dtype)


def full_step_inputs(w: Workload, n_logit_steps: int | None = None):
    """Everything one workload needs, drawn in the documented order."""
    rng = np.random.default_rng(w.seed)
    d = attention_inputs(w, rng)
    scaffold = scaffold_positions(w, rng)
    tokens, mask = initial_state(w, scaffold, rng)
    d.update(scaffold_mask=scaffold, tokens=tokens, mask=mask)
    if w.V:
        steps = w.steps if n_logit_steps is None else n_logit_steps
        if steps == 1:
            d["logits"] = step_logits(w, mask, rng)
        else:
            # later steps draw their logits lazily (they are large); hand out
            # one child generator per step so the draws do not depend on order
            d["logit_rngs"] = [np.random.default_rng([w.seed, 1000 + s]) for s in range(steps)]
        trng = np.random.default_rng([w.seed, 77])
        d["table_k"], d["table_v"] = kv_tables(w, trng)
    return d


# ---------------------------------------------------------------------------
# Section layout of the paper's output schema (Table 1): value / scaffold
# token counts per section.  Used to shape realistic scaffold masks.
TABLE1_SECTIONS = (("critical_objects", 12, 80), ("explanation", 192, 6),
                   ("future_meta_behavior", 6, 18), ("trajectory", 70, 20))


def table1_block_layout(d: int = 32, rng=None):
    """Split every section into blocks holding at most ``d`` value positions.

    Returns a list of (section, scaffold_mask uint8[len]) per block, where the
    section's scaffold tokens are spread over its blocks and interleaved with
    the value tokens at seeded positions.  The paper gives only the counts,
    not the interleaving, so the positions are synthetic.
    """
    rng = np.random.default_rng(0) if rng is None else rng
    blocks = []
    for name, n_val, n_sc in TABLE1_SECTIONS:
        n_blocks = -(-n_val // d)
        for j in range(n_blocks):
            v = min(d, n_val - j * d)
            s = n_sc // n_blocks + (1 if j < n_sc % n_blocks else 0)
            m = np.zeros(v + s, dtype=np.uint8)
            m[rng.permutation(v + s)[:s]] = 1
            blocks.append((name, m))
    return blocks
