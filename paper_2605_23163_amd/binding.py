"""ctypes binding of the C ABI declared in ``include/fdd.h``.

Argument marshalling only: tensors in, pointers and sizes out.  Every step of
the path runs inside the library's HIP kernels; there is no fallback.  torch
is used for device memory and for the current stream.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libfdd.so")
_lib = None

FDD_F32, FDD_BF16 = 0, 1
FDD_ATTN_CAUSAL_BLOCK = 1
EXPORTS = ("fdd_block_attn_workspace", "fdd_block_attn", "fdd_prefix_pack_bytes", "fdd_prefix_pack",
           "fdd_unmask_workspace", "fdd_unmask_step", "fdd_unmask_step_static", "fdd_verify_workspace", "fdd_verify_step",
           "fdd_fork_block", "fdd_block_kv_update", "fdd_block_commit", "fdd_traj_mean", "fdd_profile_attn_events", "fdd_last_error", "fdd_version")


class FddError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"fdd status {code}: {msg}")
        self.code = code


class AttnParams(C.Structure):
    _fields_ = [("N", C.c_int32), ("B", C.c_int32), ("L", C.c_int32), ("Hq", C.c_int32), ("Hkv", C.c_int32),
                ("D", C.c_int32), ("dtype", C.c_int32), ("scale", C.c_float),
                ("q", C.c_void_p), ("prefix_k", C.c_void_p), ("prefix_v", C.c_void_p),
                ("block_k", C.c_void_p), ("block_v", C.c_void_p), ("scaffold_mask", C.c_void_p),
                ("out", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("stream", C.c_void_p), ("splits", C.c_int32), ("flags", C.c_int32),
                ("prefix_v_packed", C.c_void_p), ("ext_k", C.c_void_p), ("ext_v", C.c_void_p),
                ("E", C.c_int32), ("ext_capacity", C.c_int32), ("batch", C.c_int32), ("n_q_positions", C.c_int32),
                ("q_batch_stride", C.c_int64), ("prefix_batch_stride", C.c_int64), ("block_batch_stride", C.c_int64),
                ("ext_batch_stride", C.c_int64), ("out_batch_stride", C.c_int64), ("packed_batch_stride", C.c_size_t),
                ("q_positions", C.c_void_p)]


class UnmaskParams(C.Structure):
    _fields_ = [("N", C.c_int32), ("B", C.c_int32), ("V", C.c_int64), ("dtype", C.c_int32), ("tau", C.c_float),
                ("logits", C.c_void_p), ("scaffold_mask", C.c_void_p), ("mask", C.c_void_p),
                ("tokens", C.c_void_p), ("confidences", C.c_void_p), ("n_unmasked", C.c_void_p),
                ("committed", C.c_void_p), ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t),
                ("stream", C.c_void_p),
                ("refresh_table_k", C.c_void_p), ("refresh_table_v", C.c_void_p),
                ("refresh_block_k", C.c_void_p), ("refresh_block_v", C.c_void_p),
                ("refresh_Hkv", C.c_int32), ("refresh_D", C.c_int32), ("refresh_T", C.c_int32),
                ("refresh_dtype", C.c_int32)]


class VerifyParams(C.Structure):
    _fields_ = [("N", C.c_int32), ("B", C.c_int32), ("V", C.c_int64), ("dtype", C.c_int32), ("temperature", C.c_float),
                ("ar_logits", C.c_void_p), ("scaffold_mask", C.c_void_p), ("draft", C.c_void_p), ("mask", C.c_void_p),
                ("tokens", C.c_void_p), ("n_accepted", C.c_void_p), ("accepted", C.c_void_p),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t), ("stream", C.c_void_p),
                ("seed", C.c_uint64)]


class KvUpdateParams(C.Structure):
    _fields_ = [("N", C.c_int32), ("B", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("T", C.c_int32),
                ("dtype", C.c_int32), ("tokens", C.c_void_p), ("committed", C.c_void_p),
                ("table_k", C.c_void_p), ("table_v", C.c_void_p), ("block_k", C.c_void_p),
                ("block_v", C.c_void_p), ("stream", C.c_void_p)]


class CommitParams(C.Structure):
    _fields_ = [("N", C.c_int32), ("B", C.c_int32), ("Hkv", C.c_int32), ("D", C.c_int32), ("dtype", C.c_int32),
                ("E", C.c_int32), ("ext_capacity", C.c_int32), ("reserved", C.c_int32),
                ("block_k", C.c_void_p), ("block_v", C.c_void_p), ("ext_k", C.c_void_p), ("ext_v", C.c_void_p),
                ("stream", C.c_void_p)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libfdd.so (after torch, so both share one HIP runtime)."""
    global _lib
    if _lib is None:
        import torch  # noqa: F401  -- brings in the HIP runtime the library links against
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2605_23163_amd.build` "
                "(there is no fallback path)")
        lib = C.CDLL(_LIB_PATH)
        lib.fdd_block_attn_workspace.restype = C.c_size_t
        lib.fdd_block_attn_workspace.argtypes = [C.POINTER(AttnParams)]
        lib.fdd_block_attn.restype = C.c_int
        lib.fdd_block_attn.argtypes = [C.POINTER(AttnParams)]
        lib.fdd_prefix_pack_bytes.restype = C.c_size_t
        lib.fdd_prefix_pack_bytes.argtypes = [C.c_int32] * 4
        lib.fdd_prefix_pack.restype = C.c_int
        lib.fdd_prefix_pack.argtypes = [C.c_void_p, C.c_int32, C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_size_t,
                                        C.c_void_p]
        lib.fdd_unmask_workspace.restype = C.c_size_t
        lib.fdd_unmask_workspace.argtypes = [C.POINTER(UnmaskParams)]
        lib.fdd_unmask_step.restype = C.c_int
        lib.fdd_unmask_step.argtypes = [C.POINTER(UnmaskParams)]
        lib.fdd_unmask_step_static.restype = C.c_int
        lib.fdd_unmask_step_static.argtypes = [C.POINTER(UnmaskParams)]
        lib.fdd_verify_workspace.restype = C.c_size_t
        lib.fdd_verify_workspace.argtypes = [C.POINTER(VerifyParams)]
        lib.fdd_verify_step.restype = C.c_int
        lib.fdd_verify_step.argtypes = [C.POINTER(VerifyParams)]
        lib.fdd_fork_block.restype = C.c_int
        lib.fdd_fork_block.argtypes = [C.c_int32, C.c_size_t, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.fdd_block_kv_update.restype = C.c_int
        lib.fdd_block_kv_update.argtypes = [C.POINTER(KvUpdateParams)]
        lib.fdd_traj_mean.restype = C.c_int
        lib.fdd_traj_mean.argtypes = [C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.fdd_block_commit.restype = C.c_int
        lib.fdd_block_commit.argtypes = [C.POINTER(CommitParams)]
        lib.fdd_profile_attn_events.restype = C.c_int
        lib.fdd_profile_attn_events.argtypes = [C.c_void_p, C.c_void_p]
        lib.fdd_last_error.restype = C.c_char_p
        lib.fdd_version.restype = C.c_int
        _lib = lib
    return _lib


def fdd_last_error() -> str:
    return load_library().fdd_last_error().decode()


def fdd_version() -> int:
    return load_library().fdd_version()


def fdd_profile_attn_events(start=None, stop=None):
    """Record two torch.cuda.Event (created with enable_timing=True and already
    recorded once, so that their handles exist) around the main attention
    kernel of every following fdd_block_attn call; None, None clears."""
    a = None if start is None else start.cuda_event
    b = None if stop is None else stop.cuda_event
    _check(load_library().fdd_profile_attn_events(a, b))


def _check(code):
    if code != 0:
        raise FddError(code, fdd_last_error())


def _dtype_code(t):
    import torch
    if t.dtype == torch.bfloat16:
        return FDD_BF16
    if t.dtype == torch.float32:
        return FDD_F32
    raise TypeError(f"unsupported element type {t.dtype}")


def _dev(t, name):
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError(f"{name} must live in GPU memory")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream_ptr(stream):
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream


def _workspace(ws, need, device):
    import torch
    if need == 0:
        return None, 0
    if ws is None:
        ws = torch.empty(need, dtype=torch.uint8, device=device)
    return ws, ws.numel() * ws.element_size()


def _attn_params(q, prefix_k, prefix_v, block_k, block_v, scaffold_mask, out, scale, splits, prefix_v_packed=None,
                 causal_block=False, ext_k=None, ext_v=None, E=0):
    N, B, Hq, D = q.shape
    L, Hkv = prefix_k.shape[0], block_k.shape[2]
    if tuple(prefix_k.shape[1:]) != (Hkv, D) or tuple(prefix_v.shape) != tuple(prefix_k.shape):
        raise ValueError("prefix_k / prefix_v must be [L,Hkv,D]")
    if tuple(block_k.shape) != (N, B, Hkv, D) or tuple(block_v.shape) != (N, B, Hkv, D):
        raise ValueError("block_k / block_v must be [N,B,Hkv,D]")
    dt = _dtype_code(q)
    for t in (prefix_k, prefix_v, block_k, block_v):
        if t.dtype != q.dtype:
            raise TypeError("q, k and v must share one element type")
    p = AttnParams()
    p.N, p.B, p.L, p.Hq, p.Hkv, p.D, p.dtype = N, B, L, Hq, Hkv, D, dt
    p.scale = 0.0 if scale is None else float(scale)
    p.q = _dev(q, "q")
    p.prefix_k = _dev(prefix_k, "prefix_k") if L > 0 else None
    p.prefix_v = _dev(prefix_v, "prefix_v") if L > 0 else None
    p.block_k, p.block_v = _dev(block_k, "block_k"), _dev(block_v, "block_v")
    p.scaffold_mask = _dev(scaffold_mask, "scaffold_mask")
    p.out = _dev(out, "out") if out is not None else None
    p.splits = int(splits)
    p.prefix_v_packed = _dev(prefix_v_packed, "prefix_v_packed")
    p.flags = FDD_ATTN_CAUSAL_BLOCK if causal_block else 0
    p.E = int(E)
    if ext_k is not None:
        if tuple(ext_k.shape) != tuple(ext_v.shape) or ext_k.shape[0] != N or tuple(ext_k.shape[2:]) != (Hkv, D):
            raise ValueError("ext_k / ext_v must be [N,ext_capacity,Hkv,D]")
        if ext_k.dtype != q.dtype or ext_v.dtype != q.dtype:
            raise TypeError("q, k and v must share one element type")
        p.ext_k, p.ext_v, p.ext_capacity = _dev(ext_k, "ext_k"), _dev(ext_v, "ext_v"), ext_k.shape[1]
    return p


def fdd_prefix_pack_bytes(prefix_v) -> int:
    L, Hkv, D = prefix_v.shape
    return load_library().fdd_prefix_pack_bytes(L, Hkv, D, _dtype_code(prefix_v))


def fdd_prefix_pack(prefix_v, packed=None, stream=None):
    """One-time relayout of the prefix V for later fdd_block_attn calls; returns
    the packed buffer (None when there is nothing to pack)."""
    import torch
    lib = load_library()
    L, Hkv, D = prefix_v.shape
    need = lib.fdd_prefix_pack_bytes(L, Hkv, D, _dtype_code(prefix_v))
    if need == 0:
        return None
    if packed is None:
        packed = torch.empty(need, dtype=torch.uint8, device=prefix_v.device)
    _check(lib.fdd_prefix_pack(_dev(prefix_v, "prefix_v"), L, Hkv, D, _dtype_code(prefix_v), _dev(packed, "packed"),
                               packed.numel() * packed.element_size(), _stream_ptr(stream)))
    return packed


def fdd_block_attn_workspace(q, prefix_k, prefix_v, block_k, block_v, splits=0, prefix_v_packed=None,
                             ext_k=None, ext_v=None, E=0, n_q_positions=0) -> int:
    """Workspace bytes of the fdd_block_attn call with these arguments (E and the number of query
    positions count: the work split depends on them)."""
    p = _attn_params(q, prefix_k, prefix_v, block_k, block_v, None, None, None, splits, prefix_v_packed, False,
                     ext_k, ext_v, E)
    p.n_q_positions = int(n_q_positions)
    return load_library().fdd_block_attn_workspace(C.byref(p))


def fdd_block_attn(q, prefix_k, prefix_v, block_k, block_v, scaffold_mask=None, out=None, scale=None,
                   workspace=None, stream=None, splits=0, prefix_v_packed=None, causal_block=False,
                   ext_k=None, ext_v=None, E=0, q_positions=None):
    """out[N,B,Hq,D] = shared-prefix block-causal attention (see include/fdd.h).
    ``causal_block=True`` is the verify pass: causal inside the block.
    ``ext_k/ext_v`` [N,ext_capacity,Hkv,D] with ``E`` valid rows: the blocks each
    rollout has committed since the fork.
    ``q_positions``: int32 device tensor of ascending flat positions n*B+b; only
    their rows of ``out`` are written (pass ``out`` then)."""
    import torch
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    p = _attn_params(q, prefix_k, prefix_v, block_k, block_v, scaffold_mask, out, scale, splits, prefix_v_packed,
                     causal_block, ext_k, ext_v, E)
    if q_positions is not None:
        if q_positions.dtype != torch.int32 or q_positions.dim() != 1 or not q_positions.is_contiguous():
            raise ValueError("q_positions must be a contiguous 1-D int32 tensor")
        p.q_positions = _dev(q_positions, "q_positions")
        p.n_q_positions = q_positions.numel()
    need = lib.fdd_block_attn_workspace(C.byref(p))
    ws, nbytes = _workspace(workspace, need, q.device)
    p.workspace = ws.data_ptr() if ws is not None else None
    p.workspace_bytes = nbytes
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_block_attn(C.byref(p)))
    return out


def _batched_params(q, prefix_k, prefix_v, block_k, block_v, out, scale, splits, prefix_v_packed, causal_block, ext_k, ext_v, E):
    """Parameters of a batch of independent problems: every array has a leading batch dimension."""
    P = q.shape[0]
    for name, t in (("prefix_k", prefix_k), ("prefix_v", prefix_v), ("block_k", block_k), ("block_v", block_v),
                    ("out", out), ("ext_k", ext_k), ("ext_v", ext_v), ("prefix_v_packed", prefix_v_packed)):
        if t is not None and (t.shape[0] != P or not t[0].is_contiguous()):
            raise ValueError(f"{name} must have leading dimension {P} and contiguous problems")
    sub = lambda t: None if t is None else t[0]
    p = _attn_params(q[0], prefix_k[0], prefix_v[0], block_k[0], block_v[0], None, sub(out), scale, splits,
                     sub(prefix_v_packed), causal_block, sub(ext_k), sub(ext_v), E)
    p.batch = P
    if prefix_k.stride(0) != prefix_v.stride(0) or block_k.stride(0) != block_v.stride(0) or \
            (ext_k is not None and ext_k.stride(0) != ext_v.stride(0)):
        raise ValueError("K and V arrays of a batch must share their batch stride")
    p.q_batch_stride, p.out_batch_stride = q.stride(0), (out.stride(0) if out is not None else q[0].numel())
    p.prefix_batch_stride, p.block_batch_stride = prefix_k.stride(0), block_k.stride(0)
    p.ext_batch_stride = ext_k.stride(0) if ext_k is not None else 0
    p.packed_batch_stride = prefix_v_packed.stride(0) * prefix_v_packed.element_size() if prefix_v_packed is not None else 0
    return p


def fdd_block_attn_batched_workspace(q, prefix_k, prefix_v, block_k, block_v, splits=0, prefix_v_packed=None,
                                     ext_k=None, ext_v=None, E=0) -> int:
    p = _batched_params(q, prefix_k, prefix_v, block_k, block_v, None, None, splits, prefix_v_packed, False, ext_k, ext_v, E)
    return load_library().fdd_block_attn_workspace(C.byref(p))


def fdd_block_attn_batched(q, prefix_k, prefix_v, block_k, block_v, out=None, scale=None, workspace=None, stream=None,
                           splits=0, prefix_v_packed=None, causal_block=False, ext_k=None, ext_v=None, E=0):
    """A batch of independent fdd_block_attn problems of one shape in a single launch.  Every array carries a
    leading batch dimension: q [P,N,B,Hq,D], prefix_k/v [P,L,Hkv,D], block_k/v [P,N,B,Hkv,D], and
    prefix_v_packed [P, fdd_prefix_pack_bytes] if given.  Nothing is shared between the problems."""
    import torch
    lib = load_library()
    if out is None:
        out = torch.empty_like(q)
    p = _batched_params(q, prefix_k, prefix_v, block_k, block_v, out, scale, splits, prefix_v_packed, causal_block,
                        ext_k, ext_v, E)
    need = lib.fdd_block_attn_workspace(C.byref(p))
    ws, nbytes = _workspace(workspace, need, q.device)
    p.workspace = ws.data_ptr() if ws is not None else None
    p.workspace_bytes = nbytes
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_block_attn(C.byref(p)))
    return out


def _unmask_params(logits, mask, scaffold_mask, tokens, tau, confidences, n_unmasked, committed, refresh=None):
    N, B, V = logits.shape
    p = UnmaskParams()
    if refresh is not None:
        tk, tv, bk, bv = refresh
        if tuple(bk.shape[:2]) != (N, B) or tk.shape[1:] != bk.shape[2:] or tv.shape != tk.shape or bv.shape != bk.shape:
            raise TypeError("refresh = (table_k [T,Hkv,D], table_v, block_k [N,B,Hkv,D], block_v)")
        p.refresh_table_k, p.refresh_table_v = _dev(tk, "table_k"), _dev(tv, "table_v")
        p.refresh_block_k, p.refresh_block_v = _dev(bk, "block_k"), _dev(bv, "block_v")
        p.refresh_T, p.refresh_Hkv, p.refresh_D = tk.shape[0], tk.shape[1], tk.shape[2]
        p.refresh_dtype = _dtype_code(tk)
    p.N, p.B, p.V, p.dtype, p.tau = N, B, V, _dtype_code(logits), float(tau)
    p.logits = _dev(logits, "logits")
    p.scaffold_mask = _dev(scaffold_mask, "scaffold_mask")
    p.mask, p.tokens = _dev(mask, "mask"), _dev(tokens, "tokens")
    p.confidences = _dev(confidences, "confidences")
    p.n_unmasked = _dev(n_unmasked, "n_unmasked")
    p.committed = _dev(committed, "committed")
    return p


def fdd_unmask_workspace(logits) -> int:
    p = _unmask_params(logits, None, None, None, 0.0, None, None, None)
    return load_library().fdd_unmask_workspace(C.byref(p))


def fdd_unmask_step(logits, mask, scaffold_mask, tau, tokens, confidences=None, n_unmasked=None, committed=None,
                    workspace=None, stream=None, refresh=None):
    """One unmask iteration; ``tokens`` and ``mask`` are updated in place.
    ``refresh`` = (table_k, table_v, block_k, block_v): the K/V rows of the positions
    committed by this call are refreshed by the same launch (what
    ``fdd_block_kv_update`` would do afterwards).

    Returns (tokens, confidences, n_unmasked, committed).
    """
    import torch
    lib = load_library()
    N, B, V = logits.shape
    for t, dt, nm in ((mask, torch.uint8, "mask"), (tokens, torch.int32, "tokens")):
        if t.dtype != dt or tuple(t.shape) != (N, B):
            raise TypeError(f"{nm} must be {dt} [N,B]")
    if scaffold_mask is not None and (scaffold_mask.dtype != torch.uint8 or tuple(scaffold_mask.shape) != (N, B)):
        raise TypeError("scaffold_mask must be uint8 [N,B]")
    dev = logits.device
    if confidences is None:
        confidences = torch.empty((N, B), dtype=torch.float32, device=dev)
    if n_unmasked is None:
        n_unmasked = torch.empty((N,), dtype=torch.int32, device=dev)
    if committed is None:
        committed = torch.empty((N, B), dtype=torch.uint8, device=dev)
    p = _unmask_params(logits, mask, scaffold_mask, tokens, tau, confidences, n_unmasked, committed, refresh)
    need = lib.fdd_unmask_workspace(C.byref(p))
    ws, nbytes = _workspace(workspace, need, dev)
    p.workspace = ws.data_ptr() if ws is not None else None
    p.workspace_bytes = nbytes
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_unmask_step(C.byref(p)))
    return tokens, confidences, n_unmasked, committed


def fdd_unmask_step_static(logits, mask, scaffold_mask, tau, tokens, confidences, n_unmasked, committed, stream=None,
                           refresh=None):
    """``fdd_unmask_step`` without a workspace and without any allocation: every
    output tensor is the caller's, the partial results live in the library's
    built-in device array.  Raises FddError when the shape needs more than that
    array holds."""
    lib = load_library()
    p = _unmask_params(logits, mask, scaffold_mask, tokens, tau, confidences, n_unmasked, committed, refresh)
    p.workspace = None
    p.workspace_bytes = 0
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_unmask_step_static(C.byref(p)))
    return tokens, confidences, n_unmasked, committed


def fdd_verify_workspace(ar_logits, temperature=0.0) -> int:
    """Workspace bytes of the fdd_verify_step call on these logits (the greedy and the sampled verifier differ)."""
    p = VerifyParams()
    p.N, p.B, p.V = ar_logits.shape
    p.dtype, p.temperature = _dtype_code(ar_logits), float(temperature)
    return load_library().fdd_verify_workspace(C.byref(p))


def fdd_verify_step(ar_logits, mask, scaffold_mask, draft, tokens, n_accepted=None, accepted=None, workspace=None,
                    stream=None, temperature=0.0, seed=0):
    """Accept scan of scaffold speculative decoding; ``tokens`` and ``mask`` are
    updated in place.  ``temperature`` > 0 selects the sampled verifier with the
    random stream ``seed``.  Returns (tokens, n_accepted, accepted)."""
    import torch
    lib = load_library()
    N, B, V = ar_logits.shape
    for t, dt, nm in ((mask, torch.uint8, "mask"), (tokens, torch.int32, "tokens"), (draft, torch.int32, "draft")):
        if t.dtype != dt or tuple(t.shape) != (N, B):
            raise TypeError(f"{nm} must be {dt} [N,B]")
    dev = ar_logits.device
    if n_accepted is None:
        n_accepted = torch.empty((N,), dtype=torch.int32, device=dev)
    if accepted is None:
        accepted = torch.empty((N, B), dtype=torch.uint8, device=dev)
    p = VerifyParams()
    p.N, p.B, p.V, p.dtype = N, B, V, _dtype_code(ar_logits)
    p.temperature, p.seed = float(temperature), int(seed)
    p.ar_logits = _dev(ar_logits, "ar_logits")
    p.scaffold_mask = _dev(scaffold_mask, "scaffold_mask")
    p.draft, p.mask, p.tokens = _dev(draft, "draft"), _dev(mask, "mask"), _dev(tokens, "tokens")
    p.n_accepted, p.accepted = _dev(n_accepted, "n_accepted"), _dev(accepted, "accepted")
    need = lib.fdd_verify_workspace(C.byref(p))
    ws, nbytes = _workspace(workspace, need, dev)
    p.workspace = ws.data_ptr() if ws is not None else None
    p.workspace_bytes = nbytes
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_verify_step(C.byref(p)))
    return tokens, n_accepted, accepted


def fdd_fork_block(src, N, dst=None, stream=None):
    """dst[n] = src for n < N: the private block state of N forked rollouts."""
    import torch
    lib = load_library()
    if dst is None:
        dst = torch.empty((N,) + tuple(src.shape), dtype=src.dtype, device=src.device)
    nbytes = src.numel() * src.element_size()
    if dst.numel() * dst.element_size() != N * nbytes:
        raise ValueError("dst must hold N copies of src")
    _check(lib.fdd_fork_block(N, nbytes, _dev(src, "src"), _dev(dst, "dst"), _stream_ptr(stream)))
    return dst


def fdd_block_kv_update(tokens, committed, table_k, table_v, block_k, block_v, stream=None):
    """Refresh block_k / block_v rows of committed positions in place."""
    lib = load_library()
    N, B, Hkv, D = block_k.shape
    p = KvUpdateParams()
    p.N, p.B, p.Hkv, p.D, p.T, p.dtype = N, B, Hkv, D, table_k.shape[0], _dtype_code(block_k)
    p.tokens, p.committed = _dev(tokens, "tokens"), _dev(committed, "committed")
    p.table_k, p.table_v = _dev(table_k, "table_k"), _dev(table_v, "table_v")
    p.block_k, p.block_v = _dev(block_k, "block_k"), _dev(block_v, "block_v")
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_block_kv_update(C.byref(p)))
    return block_k, block_v


def fdd_block_commit(block_k, block_v, ext_k, ext_v, E, stream=None):
    """ext[n, E:E+B] = block[n] for K and V (in place); returns E + B."""
    lib = load_library()
    N, B, Hkv, D = block_k.shape
    p = CommitParams()
    p.N, p.B, p.Hkv, p.D, p.dtype, p.E, p.ext_capacity = N, B, Hkv, D, _dtype_code(block_k), int(E), ext_k.shape[1]
    p.block_k, p.block_v = _dev(block_k, "block_k"), _dev(block_v, "block_v")
    p.ext_k, p.ext_v = _dev(ext_k, "ext_k"), _dev(ext_v, "ext_v")
    p.stream = _stream_ptr(stream)
    _check(lib.fdd_block_commit(C.byref(p)))
    return int(E) + B


def fdd_traj_mean(traj, out=None, stream=None):
    """Equal-weight mean of the N rollout trajectories: traj [N, ...] float32 -> [...]."""
    import torch
    lib = load_library()
    if traj.dtype != torch.float32:
        raise TypeError("trajectories are float32")
    N = traj.shape[0]
    P = traj[0].numel()
    if out is None:
        out = torch.empty(traj.shape[1:], dtype=torch.float32, device=traj.device)
    _check(lib.fdd_traj_mean(N, P, _dev(traj, "traj"), _dev(out, "out"), _stream_ptr(stream)))
    return out
