"""The C ABI on a machine without a GPU: the library loads, exports what
include/fdd.h declares, sizes workspaces on the host, and turns every
host-detectable mistake into an error code without launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2605_23163_amd import binding as bd

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(bd.library_path()):
        from paper_2605_23163_amd import build
        build.build()
    return bd.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "fdd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(fdd_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(bd.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_version_and_empty_error(lib):
    assert lib.fdd_version() == 100


def attn(**kw):
    p = bd.AttnParams()
    base = dict(N=1, B=32, L=2048, Hq=28, Hkv=4, D=128, dtype=bd.FDD_BF16, scale=0.0, q=256, prefix_k=512,
                prefix_v=768, block_k=1024, block_v=1280, out=1536, workspace=4096, workspace_bytes=1 << 30)
    base.update(kw)
    for k, v in base.items():
        setattr(p, k, v)
    return p


def test_attn_workspace_is_host_arithmetic(lib):
    p = attn()
    w = lib.fdd_block_attn_workspace(C.byref(p))
    assert w > 0 and w % 256 == 0
    p1 = attn(splits=1)
    assert lib.fdd_block_attn_workspace(C.byref(p1)) == 0
    p4 = attn(splits=4)
    # 4 KV heads x 1 M-tile x 4 segments x 256 rows x (128 bf16 averages + (m, l) in fp32)
    assert lib.fdd_block_attn_workspace(C.byref(p4)) == 4 * 4 * 256 * (128 * 2 + 2 * 4)
    assert lib.fdd_block_attn_workspace(C.byref(attn(Hq=30))) == 0     # invalid -> 0


@pytest.mark.parametrize("kw,code", [
    (dict(N=0), 2), (dict(B=-1), 2), (dict(L=-1), 2), (dict(Hq=30), 2), (dict(dtype=7), 3), (dict(D=96), 4),
    (dict(splits=65), 4), (dict(flags=2), 4), (dict(q=None), 1), (dict(out=None), 1), (dict(prefix_k=None), 1),
    (dict(block_v=None), 1), (dict(q=264), 4), (dict(out=256), 4), (dict(workspace=None), 5),
    (dict(workspace=4100), 5), (dict(workspace_bytes=16), 5), (dict(scale=float("nan")), 4),
])
def test_attn_rejects_bad_arguments_without_launching(lib, kw, code):
    p = attn(**kw)
    assert lib.fdd_block_attn(C.byref(p)) == code
    assert lib.fdd_last_error().decode().startswith("fdd_block_attn:")
    assert lib.fdd_block_attn(None) == 1


def unmask(**kw):
    p = bd.UnmaskParams()
    base = dict(N=8, B=32, V=152064, dtype=bd.FDD_BF16, tau=0.9, logits=256, mask=512, tokens=768, confidences=1024,
                workspace=4096, workspace_bytes=1 << 30)
    base.update(kw)
    for k, v in base.items():
        setattr(p, k, v)
    return p


def test_unmask_workspace_and_errors(lib):
    assert lib.fdd_unmask_workspace(C.byref(unmask())) > 0
    assert lib.fdd_unmask_workspace(C.byref(unmask(V=0))) == 0
    for kw, code in [(dict(N=0), 2), (dict(V=0), 2), (dict(V=1 << 31), 2), (dict(dtype=3), 3), (dict(logits=None), 1),
                     (dict(mask=None), 1), (dict(tokens=None), 1), (dict(confidences=None), 1), (dict(logits=260), 4),
                     (dict(workspace=None), 5), (dict(workspace_bytes=8), 5), (dict(tau=float("nan")), 4)]:
        assert lib.fdd_unmask_step(C.byref(unmask(**kw))) == code, kw
        assert lib.fdd_last_error().decode().startswith("fdd_unmask_step:")
    assert lib.fdd_unmask_step(None) == 1
    # the optional K/V refresh: all four arrays or none, sane row shape, aligned
    ok = dict(refresh_table_k=512, refresh_table_v=1024, refresh_block_k=2048, refresh_block_v=4096, refresh_Hkv=4,
              refresh_D=128, refresh_T=16, refresh_dtype=bd.FDD_BF16)
    for kw, code in [(dict(refresh_table_v=None), 1), (dict(refresh_block_k=None), 1), (dict(refresh_T=0), 2),
                     (dict(refresh_Hkv=-1), 2), (dict(refresh_dtype=9), 3), (dict(refresh_D=3), 4),
                     (dict(refresh_block_v=4100), 4)]:
        assert lib.fdd_unmask_step(C.byref(unmask(**{**ok, **kw}))) == code, kw
        assert lib.fdd_unmask_step_static(C.byref(unmask(**{**ok, **kw}))) == code, kw


def test_prefix_pack_sizes_and_errors(lib):
    assert lib.fdd_prefix_pack_bytes(16384, 4, 128, bd.FDD_BF16) == 16384 * 4 * 128 * 2
    assert lib.fdd_prefix_pack_bytes(100, 2, 64, bd.FDD_BF16) == 64 * 2 * 64 * 2     # full tiles only
    assert lib.fdd_prefix_pack_bytes(63, 4, 128, bd.FDD_BF16) == 0
    assert lib.fdd_prefix_pack_bytes(4096, 4, 128, bd.FDD_F32) == 0
    assert lib.fdd_prefix_pack(256, 4096, 4, 128, bd.FDD_F32, 512, 1 << 30, None) == 3
    assert lib.fdd_prefix_pack(256, 4096, 4, 96, bd.FDD_BF16, 512, 1 << 30, None) == 4
    assert lib.fdd_prefix_pack(None, 4096, 4, 128, bd.FDD_BF16, 512, 1 << 30, None) == 1
    assert lib.fdd_prefix_pack(256, 4096, 4, 128, bd.FDD_BF16, 512, 1024, None) == 5
    assert lib.fdd_prefix_pack(256, 4096, 0, 128, bd.FDD_BF16, 512, 1 << 30, None) == 2
    assert lib.fdd_prefix_pack(256, 10, 4, 128, bd.FDD_BF16, None, 0, None) == 0       # nothing to pack
    assert lib.fdd_last_error().decode().startswith("fdd_prefix_pack:")


def test_verify_workspace_and_errors(lib):
    def vp(**kw):
        p = bd.VerifyParams()
        base = dict(N=8, B=32, V=152064, dtype=bd.FDD_BF16, ar_logits=256, draft=512, mask=768, tokens=1024,
                    workspace=4096, workspace_bytes=1 << 30)
        base.update(kw)
        for k, v in base.items():
            setattr(p, k, v)
        return p
    # the sampled verifier shares the unmask step's plan; the greedy one (no sums) cuts a row into more pieces
    assert lib.fdd_verify_workspace(C.byref(vp(temperature=1.0))) == lib.fdd_unmask_workspace(C.byref(unmask()))
    greedy = lib.fdd_verify_workspace(C.byref(vp()))
    assert greedy % (8 * 32 * 16) == 0 and greedy >= lib.fdd_unmask_workspace(C.byref(unmask()))
    assert lib.fdd_verify_workspace(C.byref(vp(V=0))) == 0
    for kw, code in [(dict(N=0), 2), (dict(V=1 << 31), 2), (dict(dtype=5), 3), (dict(temperature=-1.0), 4), (dict(temperature=float('nan')), 4), (dict(temperature=float('inf')), 4), (dict(draft=None), 1),
                     (dict(ar_logits=None), 1), (dict(ar_logits=264), 4), (dict(workspace=None), 5), (dict(workspace_bytes=1), 5)]:
        assert lib.fdd_verify_step(C.byref(vp(**kw))) == code, kw
        assert lib.fdd_last_error().decode().startswith("fdd_verify_step:")
    assert lib.fdd_verify_step(None) == 1


def test_bookkeeping_errors(lib):
    assert lib.fdd_fork_block(4, 64, None, 4096, None) == 1
    assert lib.fdd_fork_block(0, 64, 256, 4096, None) == 2
    assert lib.fdd_fork_block(4, 6, 256, 4096, None) == 4
    assert lib.fdd_fork_block(4, 64, 256, 300, None) == 4        # overlap
    p = bd.KvUpdateParams()
    for k, v in dict(N=2, B=4, Hkv=4, D=128, T=16, dtype=1, tokens=256, committed=512, table_k=1024, table_v=2048,
                     block_k=4096, block_v=8192).items():
        setattr(p, k, v)
    p.T = 0
    assert lib.fdd_block_kv_update(C.byref(p)) == 2
    p.T, p.table_k = 16, None
    assert lib.fdd_block_kv_update(C.byref(p)) == 1
    p.table_k, p.dtype = 1024, 9
    assert lib.fdd_block_kv_update(C.byref(p)) == 3
    assert lib.fdd_block_kv_update(None) == 1


def test_extension_and_commit_errors(lib):
    # attention with a per-rollout extension: every host-detectable mistake is a status code
    for kw, code in [(dict(E=-1), 2), (dict(E=8, ext_capacity=4, ext_k=2048, ext_v=2304), 2),
                     (dict(E=8, ext_capacity=8), 1), (dict(E=8, ext_capacity=8, ext_k=2048, ext_v=2056), 4),
                     (dict(E=8, ext_capacity=1 << 30, ext_k=2048, ext_v=2304), 2)]:
        assert lib.fdd_block_attn(C.byref(attn(**kw))) == code, kw
        assert lib.fdd_last_error().decode().startswith("fdd_block_attn:")
    # a batch of problems: strides must cover one problem and keep 16-byte alignment
    ok = dict(batch=3, q_batch_stride=1 * 32 * 28 * 128, out_batch_stride=1 * 32 * 28 * 128,
              block_batch_stride=1 * 32 * 4 * 128, prefix_batch_stride=2048 * 4 * 128)
    assert lib.fdd_block_attn_workspace(C.byref(attn(**ok))) > 0
    for kw, code in [(dict(ok, q_batch_stride=100), 2), (dict(ok, prefix_batch_stride=2048 * 4 * 128 + 4), 2),
                     (dict(ok, batch=-1), 2), (dict(ok, batch=20000), 2), (dict(ok, n_q_positions=1), 1),
                     (dict(ok, n_q_positions=-1), 2), (dict(ok, n_q_positions=33), 2), (dict(ok, n_q_positions=4, q_positions=8194), 4),
                     (dict(ok, prefix_v_packed=8192, packed_batch_stride=100), 2)]:
        assert lib.fdd_block_attn(C.byref(attn(**kw))) == code, kw
    # E = 0 ignores the extension pointers
    assert lib.fdd_block_attn_workspace(C.byref(attn(E=0, ext_capacity=64, ext_k=2048, ext_v=2304))) == \
        lib.fdd_block_attn_workspace(C.byref(attn()))
    assert lib.fdd_block_attn_workspace(C.byref(attn(E=64, ext_capacity=64, ext_k=2048, ext_v=2304))) > 0

    def cp(**kw):
        p = bd.CommitParams()
        base = dict(N=4, B=32, Hkv=4, D=128, dtype=bd.FDD_BF16, E=32, ext_capacity=96, block_k=256, block_v=512,
                    ext_k=1024, ext_v=2048)
        base.update(kw)
        for k, v in base.items():
            setattr(p, k, v)
        return p
    for kw, code in [(dict(N=0), 2), (dict(E=65), 2), (dict(E=-1), 2), (dict(dtype=7), 3), (dict(reserved=1), 4),
                     (dict(ext_k=None), 1), (dict(block_v=None), 1), (dict(ext_v=2056), 4), (dict(Hkv=1, D=4, dtype=bd.FDD_BF16), 4)]:
        assert lib.fdd_block_commit(C.byref(cp(**kw))) == code, kw
        assert lib.fdd_last_error().decode().startswith("fdd_block_commit:")
    assert lib.fdd_block_commit(None) == 1


def test_traj_mean_errors(lib):
    assert lib.fdd_traj_mean(4, 40, None, 4096, None) == 1
    assert lib.fdd_traj_mean(0, 40, 256, 4096, None) == 2
    assert lib.fdd_traj_mean(4, 0, 256, 4096, None) == 2
    assert lib.fdd_traj_mean(4, 40, 258, 4096, None) == 4
    assert lib.fdd_last_error().decode().startswith("fdd_traj_mean:")


def test_binding_refuses_host_tensors():
    import torch
    q = torch.zeros(1, 8, 4, 64)
    k = torch.zeros(16, 1, 64)
    b = torch.zeros(1, 8, 1, 64)
    with pytest.raises(ValueError, match="GPU memory"):
        bd.fdd_block_attn(q, k, k, b, b, out=torch.zeros_like(q))
