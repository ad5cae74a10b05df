"""fp64 CPU oracle of the block-diffusion denoise step -- TEST INFRASTRUCTURE.

Only tests, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It loads ``liboracle.so`` (plain C,
built from ``fdd_oracle.c`` with gcc) through ctypes and marshals numpy
arrays; all arithmetic is in the C file, whose header cites the passages of
the paper each function follows.  Nothing here imports the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fdd_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_DT = {np.dtype(np.float64): 0, np.dtype(np.float32): 1, np.dtype(np.uint16): 2}


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc -O2 -fopenmp)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".{os.getpid()}.tmp"
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-ffp-contract=off",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c = ctypes
        lib.fddo_block_attn.restype = c.c_int
        lib.fddo_block_attn.argtypes = [c.c_int] * 7 + [c.c_double] + [c.c_void_p] * 6 + [c.c_int64, c.c_void_p]
        lib.fddo_block_attn_ex.restype = c.c_int
        lib.fddo_block_attn_ex.argtypes = [c.c_int] * 7 + [c.c_double, c.c_int] + [c.c_void_p] * 6 + [c.c_int64, c.c_void_p]
        lib.fddo_block_attn_ext.restype = c.c_int
        lib.fddo_block_attn_ext.argtypes = ([c.c_int] * 9 + [c.c_double, c.c_int] + [c.c_void_p] * 8 +
                                            [c.c_int64, c.c_void_p])
        lib.fddo_traj_mean.restype = c.c_int
        lib.fddo_traj_mean.argtypes = [c.c_int, c.c_int, c.c_int, c.c_void_p, c.c_void_p]
        lib.fddo_block_commit.restype = c.c_int
        lib.fddo_block_commit.argtypes = [c.c_int] * 7 + [c.c_void_p] * 4
        lib.fddo_verify_step.restype = c.c_int
        lib.fddo_verify_step.argtypes = [c.c_int, c.c_int, c.c_int64, c.c_int] + [c.c_void_p] * 8
        lib.fddo_verify_step_ex.restype = c.c_int
        lib.fddo_verify_step_ex.argtypes = [c.c_int, c.c_int, c.c_int64, c.c_int] + [c.c_void_p] * 8 + [c.c_float, c.c_uint64]
        lib.fddo_philox4x32_10.restype = None
        lib.fddo_philox4x32_10.argtypes = [c.c_void_p] * 3
        lib.fddo_flog2.restype = c.c_float
        lib.fddo_flog2.argtypes = [c.c_float]
        lib.fddo_sample_key.restype = c.c_float
        lib.fddo_sample_key.argtypes = [c.c_float, c.c_float, c.c_uint64, c.c_uint32, c.c_int64]
        lib.fddo_sample_scale.restype = c.c_float
        lib.fddo_sample_scale.argtypes = [c.c_float]
        lib.fddo_unmask_step.restype = c.c_int
        lib.fddo_unmask_step.argtypes = [c.c_int, c.c_int, c.c_int64, c.c_int, c.c_double] + [c.c_void_p] * 8
        lib.fddo_block_kv_update.restype = c.c_int
        lib.fddo_block_kv_update.argtypes = [c.c_int] * 6 + [c.c_void_p] * 6
        lib.fddo_fork_block.restype = c.c_int
        lib.fddo_fork_block.argtypes = [c.c_int, c.c_size_t, c.c_void_p, c.c_void_p]
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the oracle's parallel loops use (reported with CPU timings)."""
    lib = _load()
    lib.fddo_num_threads.restype = ctypes.c_int
    return int(lib.fddo_num_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _same_storage(*arrs):
    arrs = [np.ascontiguousarray(a) for a in arrs]
    dt = arrs[0].dtype
    if dt not in _DT or any(a.dtype != dt for a in arrs):
        raise TypeError("arrays must share one of float64 / float32 / uint16(bf16 bits)")
    return arrs, _DT[dt]


def block_attn(q, prefix_k, prefix_v, block_k, block_v, scale=None, rows=None, causal_block=False,
               ext_k=None, ext_v=None, E=0):
    """Block-causal shared-prefix attention in fp64.  ``causal_block=True`` makes
    the in-block part causal (the verify pass of scaffold speculative decoding).
    ``ext_k/ext_v`` [N,Ecap,Hkv,D] with ``E`` valid rows per rollout: the blocks a
    rollout has committed since the fork, visible to that rollout only.

    q [N,B,Hq,D], prefix_k/v [L,Hkv,D], block_k/v [N,B,Hkv,D]; float64,
    float32, or uint16 holding bf16 bits.  ``rows``: optional int array
    [R,3] of (n,b,h) to compute only those output rows.
    Returns float64 [N,B,Hq,D] (or [R,D]).
    """
    (q, prefix_k, prefix_v, block_k, block_v), dt = _same_storage(q, prefix_k, prefix_v, block_k, block_v)
    N, B, Hq, D = q.shape
    L, Hkv, _ = prefix_k.shape
    assert prefix_v.shape == (L, Hkv, D) and block_k.shape == (N, B, Hkv, D) and block_v.shape == (N, B, Hkv, D)
    scale = 1.0 / np.sqrt(D) if scale is None else float(scale)
    if rows is None:
        out = np.empty((N, B, Hq, D), dtype=np.float64)
        r, nr = None, 0
    else:
        r = np.ascontiguousarray(rows, dtype=np.int32).reshape(-1, 3)
        nr = r.shape[0]
        out = np.empty((nr, D), dtype=np.float64)
    Ecap = 0
    if E > 0:
        (ext_k, ext_v), dte = _same_storage(ext_k, ext_v)
        assert dte == dt and ext_k.shape == ext_v.shape and ext_k.shape[0] == N and ext_k.shape[2:] == (Hkv, D)
        Ecap = ext_k.shape[1]
    else:
        ext_k = ext_v = None
    rc = _load().fddo_block_attn_ext(N, B, L, int(E), Ecap, Hq, Hkv, D, dt, scale, int(bool(causal_block)), _ptr(q),
                                     _ptr(prefix_k), _ptr(prefix_v), _ptr(ext_k), _ptr(ext_v), _ptr(block_k),
                                     _ptr(block_v), _ptr(r), nr, _ptr(out))
    if rc:
        raise ValueError("fddo_block_attn rejected its arguments")
    return out


def unmask_step(logits, mask, scaffold_mask, tokens, tau):
    """One confidence-threshold unmask iteration; inputs are not modified.

    Returns dict(tokens, mask, confidences (float64, -inf where not
    eligible), candidates, n_unmasked, committed).
    """
    logits = np.ascontiguousarray(logits)
    dt = _DT[logits.dtype]
    N, B, V = logits.shape
    mask = np.array(mask, dtype=np.uint8, order="C", copy=True).reshape(N, B)
    tokens = np.array(tokens, dtype=np.int32, order="C", copy=True).reshape(N, B)
    sc = None if scaffold_mask is None else np.ascontiguousarray(scaffold_mask, dtype=np.uint8).reshape(N, B)
    conf = np.empty((N, B), dtype=np.float64)
    cand = np.empty((N, B), dtype=np.int32)
    nun = np.empty((N,), dtype=np.int32)
    com = np.empty((N, B), dtype=np.uint8)
    rc = _load().fddo_unmask_step(N, B, V, dt, float(tau), _ptr(logits), _ptr(sc), _ptr(mask), _ptr(tokens),
                                  _ptr(conf), _ptr(cand), _ptr(nun), _ptr(com))
    if rc:
        raise ValueError("fddo_unmask_step rejected its arguments")
    return dict(tokens=tokens, mask=mask, confidences=conf, candidates=cand, n_unmasked=nun, committed=com)


def verify_step(ar_logits, mask, scaffold_mask, draft, tokens, temperature=0.0, seed=0):
    """Accept scan of scaffold speculative decoding; inputs are not modified.
    ``temperature`` = 0: greedy verifier; > 0: sampled verifier (Gumbel-max
    with the Philox stream of ``seed``).

    Returns dict(tokens, mask, ar_tokens, n_accepted, accepted).
    """
    ar_logits = np.ascontiguousarray(ar_logits)
    dt = _DT[ar_logits.dtype]
    N, B, V = ar_logits.shape
    mask = np.array(mask, dtype=np.uint8, order="C", copy=True).reshape(N, B)
    tokens = np.array(tokens, dtype=np.int32, order="C", copy=True).reshape(N, B)
    draft = np.ascontiguousarray(draft, dtype=np.int32).reshape(N, B)
    sc = None if scaffold_mask is None else np.ascontiguousarray(scaffold_mask, dtype=np.uint8).reshape(N, B)
    ar = np.empty((N, B), dtype=np.int32)
    nacc = np.empty((N,), dtype=np.int32)
    acc = np.empty((N, B), dtype=np.uint8)
    rc = _load().fddo_verify_step_ex(N, B, V, dt, _ptr(ar_logits), _ptr(sc), _ptr(draft), _ptr(mask),
                                     _ptr(tokens), _ptr(ar), _ptr(nacc), _ptr(acc), float(temperature), int(seed))
    if rc:
        raise ValueError("fddo_verify_step_ex rejected its arguments")
    return dict(tokens=tokens, mask=mask, ar_tokens=ar, n_accepted=nacc, accepted=acc)


def philox4x32_10(counter, key):
    """One block of the sampler's counter-based generator: 4 + 2 words in, 4 words out."""
    c = (ctypes.c_uint32 * 4)(*[int(x) for x in counter])
    k = (ctypes.c_uint32 * 2)(*[int(x) for x in key])
    out = (ctypes.c_uint32 * 4)()
    _load().fddo_philox4x32_10(c, k, out)
    return [int(x) for x in out]


def flog2(x):
    """The sampler's fp32 log2, element by element."""
    lib = _load()
    x = np.asarray(x, dtype=np.float32)
    return np.array([lib.fddo_flog2(float(v)) for v in x.ravel()], dtype=np.float32).reshape(x.shape)


def sample_key(x, temperature, seed, row, v):
    """The sampler's key of one vocabulary entry (fp32)."""
    lib = _load()
    return lib.fddo_sample_key(float(x), lib.fddo_sample_scale(float(temperature)), int(seed), int(row), int(v))


def block_kv_update(tokens, committed, table_k, table_v, block_k, block_v):
    """Returns refreshed copies (block_k, block_v)."""
    (table_k, table_v, block_k, block_v), dt = _same_storage(table_k, table_v, block_k, block_v)
    block_k, block_v = block_k.copy(), block_v.copy()
    N, B, Hkv, D = block_k.shape
    T = table_k.shape[0]
    tokens = np.ascontiguousarray(tokens, dtype=np.int32)
    committed = np.ascontiguousarray(committed, dtype=np.uint8)
    rc = _load().fddo_block_kv_update(N, B, Hkv, D, T, dt, _ptr(tokens), _ptr(committed), _ptr(table_k),
                                      _ptr(table_v), _ptr(block_k), _ptr(block_v))
    if rc:
        raise ValueError("fddo_block_kv_update rejected its arguments")
    return block_k, block_v


def block_commit(block_k, block_v, ext_k, ext_v, E):
    """Returns copies of (ext_k, ext_v) with rows E .. E+B-1 of every rollout set to its block."""
    (block_k, block_v, ext_k, ext_v), dt = _same_storage(block_k, block_v, ext_k, ext_v)
    ext_k, ext_v = ext_k.copy(), ext_v.copy()
    N, B, Hkv, D = block_k.shape
    rc = _load().fddo_block_commit(N, B, int(E), ext_k.shape[1], Hkv, D, dt, _ptr(block_k), _ptr(block_v), _ptr(ext_k),
                                   _ptr(ext_v))
    if rc:
        raise ValueError("fddo_block_commit rejected its arguments")
    return ext_k, ext_v


def traj_mean(traj):
    """Equal-weight mean over the N rollout trajectories; traj [N, ...] float32/float64 -> float64 [...]."""
    traj = np.ascontiguousarray(traj)
    if traj.dtype not in (np.float32, np.float64):
        raise TypeError("trajectories are float32 or float64")
    N = traj.shape[0]
    P = int(np.prod(traj.shape[1:]))
    out = np.empty(traj.shape[1:], dtype=np.float64)
    rc = _load().fddo_traj_mean(N, P, _DT[traj.dtype], _ptr(traj), _ptr(out))
    if rc:
        raise ValueError("fddo_traj_mean rejected its arguments")
    return out


def fork_block(src, N):
    """N private copies of one rollout's block-sized array."""
    src = np.ascontiguousarray(src)
    dst = np.empty((N,) + src.shape, dtype=src.dtype)
    rc = _load().fddo_fork_block(N, src.nbytes, _ptr(src), _ptr(dst))
    if rc:
        raise ValueError("fddo_fork_block rejected its arguments")
    return dst
