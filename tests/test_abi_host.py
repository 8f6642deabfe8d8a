"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, computes the slopes, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import numpy as np
import pytest

from paper_2312_17482_amd import binding as mb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
lib = mb.raw()
A = 4096            # a fake, 16-byte aligned "device pointer": must never be dereferenced by these calls


def declared_symbols():
    names = []
    for fn in os.listdir(os.path.join(ROOT, "include")):
        if fn.endswith(".h"):
            text = open(os.path.join(ROOT, "include", fn)).read()
            names += re.findall(r"MB_API\s+[\w\s\*]+?\b(mb_\w+)\s*\(", text)
    return names


def test_library_exports_every_declared_symbol():
    names = declared_symbols()
    assert len(names) >= 10 and set(names) == set(mb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    assert mb.mb_version() >= 100


def test_slopes_against_fixture():
    rows = [l.split() for l in open(os.path.join(ROOT, "tests", "golden", "alibi_slopes.txt"))
            if l.strip() and not l.startswith("#")]
    for n, h, p, q in rows:
        s = mb.mb_alibi_slopes(int(n)).numpy()
        assert s.dtype == np.float32 and s.shape == (int(n),)
        assert s[int(h) - 1] == np.float32(2.0 ** (-int(p) / int(q)))
    with pytest.raises(mb.MosaicAttnError) as e:
        mb.mb_alibi_slopes(0)
    assert e.value.status == mb.MB_ERR_INVALID_ARG and "H=0" in str(e.value)
    assert lib.mb_alibi_slopes(4, None) == mb.MB_ERR_INVALID_ARG


def fwd_args(**over):
    a = dict(q=A, k=A, v=A, qs=768, ks=768, vs=768, cu=A, B=2, T=64, max_seqlen=32, H=12, D=64, slopes=A,
             scale=0.125, dt=mb.MB_BF16, o=A, os=768, lse=A, ws=None, wsb=0, klens=None, rows=None, plan=None,
             stream=None)
    a.update(over)
    return [a[x] for x in ("q", "k", "v", "qs", "ks", "vs", "cu", "B", "T", "max_seqlen", "H", "D", "slopes", "scale",
                           "dt", "o", "os", "lse", "ws", "wsb", "klens", "rows", "plan", "stream")]


def bwd_args(**over):
    a = dict(do=A, q=A, k=A, v=A, o=A, lse=A, dos=768, qs=768, ks=768, vs=768, os=768, cu=A, B=2, T=64,
             max_seqlen=32, H=12, D=64, slopes=A, scale=0.125, dt=mb.MB_BF16, dq=A, dk=A, dv=A, dqs=768, dks=768,
             dvs=768, ws=A, wsb=1 << 20, klens=None, rows=None, plan=None, stream=None)
    a.update(over)
    return [a[x] for x in ("do", "q", "k", "v", "o", "lse", "dos", "qs", "ks", "vs", "os", "cu", "B", "T",
                           "max_seqlen", "H", "D", "slopes", "scale", "dt", "dq", "dk", "dv", "dqs", "dks", "dvs",
                           "ws", "wsb", "klens", "rows", "plan", "stream")]


@pytest.mark.parametrize("over,status,needle", [
    (dict(q=None), mb.MB_ERR_INVALID_ARG, "q is NULL"),
    (dict(lse=None), mb.MB_ERR_INVALID_ARG, "lse is NULL"),
    (dict(k=A + 2), mb.MB_ERR_INVALID_ARG, "16-byte"),
    (dict(H=0), mb.MB_ERR_INVALID_ARG, "positive"),
    (dict(T=-1), mb.MB_ERR_INVALID_ARG, "negative"),
    (dict(D=256), mb.MB_ERR_UNSUPPORTED, "head_dim"),
    (dict(D=12, dt=mb.MB_BF16, qs=768), mb.MB_ERR_UNSUPPORTED, "multiple of 8"),
    (dict(qs=100), mb.MB_ERR_INVALID_ARG, "smaller than H*D"),
    (dict(vs=772), mb.MB_ERR_INVALID_ARG, "multiple of 16 bytes"),
    (dict(ks=1 << 24), mb.MB_ERR_UNSUPPORTED, "exceeds 2^24"),
    (dict(dt=7), mb.MB_ERR_INVALID_ARG, "dtype"),
    (dict(scale=float("nan")), mb.MB_ERR_INVALID_ARG, "finite"),
    (dict(max_seqlen=0), mb.MB_ERR_INVALID_ARG, "max_seqlen"),
    (dict(dt=mb.MB_F32, D=16, H=2, max_seqlen=1 << 20), mb.MB_ERR_UNSUPPORTED, "max_seqlen"),
    (dict(rows=A + 4), mb.MB_ERR_INVALID_ARG, "token_rows"),
    (dict(max_seqlen=512), mb.MB_ERR_WORKSPACE, "workspace"),                       # any-length kernels need their plan
    (dict(max_seqlen=512, ws=A, wsb=64), mb.MB_ERR_WORKSPACE, "needed"),
    (dict(max_seqlen=512, ws=A + 4, wsb=1 << 20), mb.MB_ERR_INVALID_ARG, "workspace is not 16-byte"),
    (dict(max_seqlen=1 << 23), mb.MB_ERR_UNSUPPORTED, "2^22"),
    (dict(klens=A + 2), mb.MB_ERR_INVALID_ARG, "key_lens is not 4-byte"),
    (dict(plan=A + 8), mb.MB_ERR_INVALID_ARG, "plan is not 16-byte"),
    (dict(klens=A, dt=mb.MB_F32, D=16, H=2, qs=32, ks=32, vs=32, os=32), mb.MB_ERR_UNSUPPORTED, "key_lens"),
])
def test_fwd_rejects_bad_arguments_without_launching(over, status, needle):
    assert lib.mb_alibi_attn_fwd(*fwd_args(**over)) == status
    assert needle in mb.mb_last_error()


@pytest.mark.parametrize("over,status,needle", [
    (dict(do=None), mb.MB_ERR_INVALID_ARG, "dout is NULL"),
    (dict(dv=None), mb.MB_ERR_INVALID_ARG, "dv is NULL"),
    (dict(dqs=8), mb.MB_ERR_INVALID_ARG, "smaller than H*D"),
    (dict(dos=1 << 25), mb.MB_ERR_UNSUPPORTED, "exceeds 2^24"),
    (dict(ws=None), mb.MB_ERR_WORKSPACE, "workspace"),
    (dict(wsb=16), mb.MB_ERR_WORKSPACE, "needed"),
    (dict(ws=A + 4), mb.MB_ERR_INVALID_ARG, "workspace is not 16-byte"),
    (dict(D=200), mb.MB_ERR_UNSUPPORTED, "head_dim"),
])
def test_bwd_rejects_bad_arguments_without_launching(over, status, needle):
    assert lib.mb_alibi_attn_bwd(*bwd_args(**over)) == status
    assert needle in mb.mb_last_error()


def static_bwd_args(**over):
    a = bwd_args(**over)
    return a[:26] + a[28:]          # the same list without workspace and workspace_bytes


@pytest.mark.parametrize("over,status,needle", [
    (dict(do=None), mb.MB_ERR_INVALID_ARG, "dout is NULL"),
    (dict(dks=8), mb.MB_ERR_INVALID_ARG, "smaller than H*D"),
    (dict(rows=A + 4), mb.MB_ERR_INVALID_ARG, "token_rows"),
    # 16 heads x 300000 token rows of Delta = 19.2 MB: more than the static array holds
    (dict(T=300000, H=16, qs=1024, ks=1024, vs=1024, os=1024, dos=1024, dqs=1024, dks=1024, dvs=1024, max_seqlen=512),
     mb.MB_ERR_WORKSPACE, "static array holds"),
])
def test_static_bwd_rejects_bad_arguments_and_sizes_beyond_its_array_without_launching(over, status, needle):
    assert lib.mb_alibi_attn_bwd_static(*static_bwd_args(**over)) == status
    assert needle in mb.mb_last_error()
    assert lib.mb_alibi_attn_bwd_static(*static_bwd_args(B=0, T=0, do=None)) == mb.MB_OK


def test_degenerate_sizes_are_ok_and_touch_nothing():
    # T == 0 / B == 0: MB_OK before any pointer is looked at or anything is launched
    assert lib.mb_alibi_attn_fwd(*fwd_args(T=0, q=None, k=None, v=None, o=None, lse=None)) == mb.MB_OK
    assert lib.mb_alibi_attn_bwd(*bwd_args(B=0, T=0, do=None, ws=None, wsb=0)) == mb.MB_OK
    assert mb.mb_last_error() == ""
    assert lib.mb_unpad(None, None, 0, None, 768, mb.MB_BF16, None, None) == mb.MB_OK
    assert lib.mb_pad(None, None, 0, None, 0, 128, 768, mb.MB_BF16, None, None) == mb.MB_OK


def test_plan_rejects_bad_arguments_without_launching():
    need = mb.mb_attn_plan_bytes(64, 512, 12)
    assert need >= 64 * 12 * 4 * 16 and need % 256 == 0 and mb.mb_attn_plan_bytes(64, 512, 0) == 0
    assert need == mb.mb_alibi_attn_fwd_workspace_bytes(64, 32768, 512, 12, 64, mb.MB_BF16)
    for args, status, needle in (((None, None, 64, 512, 12, A, need, None), mb.MB_ERR_INVALID_ARG, "cu_seqlens is NULL"),
                                 ((A, None, 64, 512, 12, None, need, None), mb.MB_ERR_WORKSPACE, "needed"),
                                 ((A, None, 64, 512, 12, A, need - 1, None), mb.MB_ERR_WORKSPACE, "needed"),
                                 ((A, None, 64, 512, 12, A + 8, need, None), mb.MB_ERR_INVALID_ARG, "16-byte"),
                                 ((A, A + 2, 64, 512, 12, A, need, None), mb.MB_ERR_INVALID_ARG, "key_lens"),
                                 ((A, None, 64, 512, 0, A, need, None), mb.MB_ERR_INVALID_ARG, "positive"),
                                 ((A, None, -1, 512, 12, A, need, None), mb.MB_ERR_INVALID_ARG, "negative")):
        assert lib.mb_attn_plan(*args) == status
        assert needle in mb.mb_last_error()


def test_workspace_query():
    need = mb.mb_alibi_attn_bwd_workspace_bytes(256, 27000, 128, 12, 64, mb.MB_BF16)
    assert need >= 12 * 27000 * 4 and need % 256 == 0
    # the any-length kernels add their work plan: 8 lists of 16-byte items, one per (sequence, head, 128 tokens)
    plan = mb.mb_alibi_attn_fwd_workspace_bytes(64, 32768, 512, 12, 64, mb.MB_BF16)
    assert plan >= 64 * 12 * 4 * 16 and plan % 256 == 0
    assert mb.mb_alibi_attn_bwd_workspace_bytes(64, 32768, 512, 12, 64, mb.MB_BF16) >= 12 * 32768 * 4 + plan
    assert mb.mb_alibi_attn_fwd_workspace_bytes(256, 32768, 128, 12, 64, mb.MB_BF16) == 0      # single-tile kernel
    assert mb.mb_alibi_attn_fwd_workspace_bytes(4, 128, 32, 2, 16, mb.MB_F32) == 0              # generic kernels
    assert mb.mb_alibi_attn_bwd_workspace_bytes(1, 1, 1, 0, 64, mb.MB_BF16) == 0
    assert mb.mb_alibi_attn_bwd_workspace_bytes(1, 1, 1, 1, 64, 9) == 0


@pytest.mark.parametrize("args,status,needle", [
    ((None, A, 16, None, 768, mb.MB_BF16, A, None), mb.MB_ERR_INVALID_ARG, "padded is NULL"),
    ((A, A, 16, None, 100, mb.MB_BF16, A, None), mb.MB_ERR_INVALID_ARG, "16 bytes"),
    ((A, A, -1, None, 768, mb.MB_BF16, A, None), mb.MB_ERR_INVALID_ARG, "negative"),
    ((A, A, 16, None, 0, mb.MB_BF16, A, None), mb.MB_ERR_INVALID_ARG, "positive"),
    ((A, A + 8, 16, None, 768, mb.MB_BF16, A, None), mb.MB_ERR_INVALID_ARG, "aligned"),
])
def test_unpad_rejects_bad_arguments(args, status, needle):
    assert lib.mb_unpad(*args) == status
    assert needle in mb.mb_last_error()


def test_pad_and_index_reject_bad_arguments():
    assert lib.mb_pad(A, A, 100, None, 2, 8, 768, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG   # T_cap > B*L
    assert "exceeds B*L" in mb.mb_last_error()
    assert lib.mb_pad(A, A, 4, None, 2, 8, 768, mb.MB_BF16, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_unpad_index(None, 2, 8, A, A, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert "mask is NULL" in mb.mb_last_error()
    assert lib.mb_unpad_index(A, -1, 8, A, A, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_unpad_index(A, 1 << 16, 1 << 16, A, A, A, A, None) == mb.MB_ERR_UNSUPPORTED
    assert lib.mb_unpad_index(A, 2, 8, A, A, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_read_meta(None, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_zero_padding(A, 100, None, 2, 8, 768, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_zero_padding(A, 4, None, 2, 8, 768, mb.MB_BF16, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_zero_padding(None, 0, None, 0, 8, 768, mb.MB_BF16, None, None) == mb.MB_OK


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2312_17482_amd")
    for dirpath, _, files in os.walk(pkg):
        for fn in files:
            if fn.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, fn)).read()
                assert not re.search(r"^\s*(from|import)\s+\S*oracle", text, re.M), "%s imports the oracle" % fn
                assert "mosaic_oracle" not in text, "%s names the oracle module" % fn


def test_layernorm_rejects_bad_arguments():
    assert lib.mb_add_layernorm_fwd(A, A, A, A, 16, None, 100, 1e-5, mb.MB_BF16, A, A, A, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert "16 bytes" in mb.mb_last_error()
    assert lib.mb_add_layernorm_fwd(A, A, A, A, 16, None, 4096, 1e-5, mb.MB_BF16, A, A, A, A, None, None) == mb.MB_ERR_UNSUPPORTED
    assert lib.mb_add_layernorm_fwd(A, A, A, A, 16, None, 768, -1.0, mb.MB_BF16, A, A, A, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_add_layernorm_fwd(A, A, A, A, 16, None, 768, 1e-5, mb.MB_BF16, A, None, A, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert "s is NULL" in mb.mb_last_error()
    assert lib.mb_add_layernorm_fwd(None, None, A, A, 16, None, 768, 1e-5, mb.MB_BF16, A, None, A, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_add_layernorm_fwd(None, None, None, None, 0, None, 768, 1e-5, mb.MB_BF16, None, None, None, None, None, None) == mb.MB_OK
    need = mb.mb_add_layernorm_bwd_workspace_bytes(768)
    assert need == 1024 * 2 * 768 * 4 and mb.mb_add_layernorm_bwd_workspace_bytes(0) == 0
    assert lib.mb_add_layernorm_bwd(A, A, A, A, A, 16, None, 768, mb.MB_BF16, A, A, A, A, need - 1, None, None) == mb.MB_ERR_WORKSPACE
    assert lib.mb_add_layernorm_bwd(A, A, A, A, A, 16, None, 768, mb.MB_BF16, A, None, A, A, need, None, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_add_layernorm_fwd(A, A, A, A, 16, None, 768, 1e-5, mb.MB_BF16, A, A, A, A, A + 2, None) == mb.MB_ERR_INVALID_ARG
    assert "y_rows" in mb.mb_last_error()
    assert lib.mb_add_layernorm_bwd(A, A, A, A, A, 16, None, 768, mb.MB_BF16, A, A, A, A, need, A + 1, None) == mb.MB_ERR_INVALID_ARG
    assert "dy_rows" in mb.mb_last_error()


def test_geglu_rejects_bad_arguments():
    f = lib.mb_geglu_fwd
    assert f(A, A, A, 16, None, 768, 3072, mb.MB_F32, A, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, A, 16, None, 768, 3072, 7, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, -1, None, 768, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, 16, None, 0, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, 16, None, 700, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, A, 16, None, 768, 3000, mb.MB_BF16, A, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, A, 1 << 20, None, 768, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_UNSUPPORTED     # 2^31 elements
    assert f(None, A, A, 16, None, 768, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, 16, None, 768, 3072, mb.MB_BF16, A, None, None) == mb.MB_ERR_INVALID_ARG
    assert f(A + 8, A, A, 16, None, 768, 3072, mb.MB_BF16, A, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(None, None, None, 0, None, 768, 3072, mb.MB_BF16, None, None, None) == mb.MB_OK


def test_linear_and_gelu_gate_reject_bad_arguments():
    f = lib.mb_linear_fwd
    assert f(A, A, 16, None, 768, 3072, mb.MB_F32, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, 16, None, 700, 3072, mb.MB_BF16, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, 16, None, 768, 3000, mb.MB_BF16, A, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, -2, None, 768, 3072, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, None, 16, None, 768, 3072, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert f(None, None, 0, None, 768, 3072, mb.MB_BF16, None, None) == mb.MB_OK
    g = lib.mb_gelu_gate
    assert g(A, A, 3072, 16, None, 3072, mb.MB_F32, A, None) == mb.MB_ERR_UNSUPPORTED
    assert g(A, A, 3070, 16, None, 3072, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert g(A, A, 3072, 16, None, 3076, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert g(A, A + 2, 3072, 16, None, 3072, mb.MB_BF16, A, None) == mb.MB_ERR_INVALID_ARG
    assert g(None, None, 3072, 0, None, 3072, mb.MB_BF16, None, None) == mb.MB_OK


def test_traffic_probe_rejects_bad_arguments():
    assert lib.mb_probe_bwd_traffic(A, A, A, None, A, 4, 12, None) == mb.MB_ERR_INVALID_ARG and "dqkv is NULL" in mb.mb_last_error()
    assert lib.mb_probe_bwd_traffic(A, A, A, A, A, 4, 0, None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_probe_bwd_traffic(None, None, None, None, None, 0, 12, None) == mb.MB_OK


def test_probe_rejects_bad_arguments():
    w = ctypes.c_double(0.0)
    assert lib.mb_probe_ceiling(3, 10, A, ctypes.byref(w), None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_probe_ceiling(0, 0, A, ctypes.byref(w), None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_probe_ceiling(0, 10, None, ctypes.byref(w), None) == mb.MB_ERR_INVALID_ARG
    assert lib.mb_probe_ceiling(0, 10, A, None, None) == mb.MB_ERR_INVALID_ARG


def test_geglu_bwd_rejects_bad_arguments():
    f = lib.mb_geglu_bwd
    need = mb.mb_geglu_bwd_workspace_bytes(512, 768, 3072)
    assert need > 2 * 512 * 6144 * 2 and need % 256 == 0
    assert mb.mb_geglu_bwd_workspace_bytes(512, 768, 3000) == 0
    assert f(A, A, A, A, A, None, 512, None, 768, 3072, mb.MB_BF16, A, A, A, A, need - 1, None) == mb.MB_ERR_WORKSPACE
    assert f(A, A, A, A, A, None, 512, None, 768, 3072, mb.MB_BF16, A, A, A, None, need, None) == mb.MB_ERR_WORKSPACE
    assert f(A, A, A, A, A, None, 512, None, 768, 3072, mb.MB_BF16, A, A, A, A + 16, need, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, A, A, None, 512, None, 768, 3200, mb.MB_BF16, A, A, A, A, need, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, A, A, A, None, 512, None, 768, 3072, mb.MB_F32, A, A, A, A, need, None) == mb.MB_ERR_UNSUPPORTED
    assert f(A, A, A, A, A, None, 512, None, 768, 3072, mb.MB_BF16, A, None, A, A, need, None) == mb.MB_ERR_INVALID_ARG
    assert f(None, A, A, A, A, None, 512, None, 768, 3072, mb.MB_BF16, A, A, A, A, need, None) == mb.MB_ERR_INVALID_ARG
    assert f(A, A, A, A, A, A + 4, 512, None, 768, 3072, mb.MB_BF16, A, A, A, A, need, None) == mb.MB_ERR_INVALID_ARG
