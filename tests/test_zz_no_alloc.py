"""mb_alibi_attn_bwd_static (the backward on the library's fixed scratch array, for callers that cannot allocate)
gives bit for bit what mb_alibi_attn_bwd gives with a workspace of the caller's: two calls in a row, the second
on a smaller input, through the raw C ABI; then the oracle's tolerance on the second."""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2312_17482_amd import workloads as wl
from tests.helpers import err_stats, to_dev

pytestmark = pytest.mark.gpu


def _packed_case(mb, seed, lengths, L, H):
    c = wl.random_attention_case(seed, lengths, L, H, 64, std=0.5, bf16=True)
    B = len(lengths)
    mask = torch.from_numpy(c["mask"]).cuda()
    seqlens, cu, indices, meta = mb.mb_unpad_index(mask)
    T, mx = mb.mb_read_meta(meta)
    qkv = mb.mb_unpad(to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(B * L, 3 * H * 64), True), indices,
                      B * L, meta)[:T].view(T, 3, H, 64)
    dout = mb.mb_unpad(to_dev(c["do"].reshape(B * L, H * 64), True), indices, B * L, meta)[:T].view(T, H, 64)
    return c, cu, T, mx, qkv, dout


def _both(mb, c, cu, T, mx, qkv, dout, H):
    lib = mb.raw()
    slopes = mb.mb_alibi_slopes(H).cuda()
    o, lse = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, mx, slopes, c["scale"])
    ref = torch.full((T, 3, H, 64), 3.0, dtype=torch.bfloat16, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, mx, slopes, c["scale"],
                         dq=ref[:, 0], dk=ref[:, 1], dv=ref[:, 2])
    got = torch.full((T, 3, H, 64), 5.0, dtype=torch.bfloat16, device="cuda")
    B = cu.numel() - 1
    st = lib.mb_alibi_attn_bwd_static(
        dout.data_ptr(), qkv[:, 0].data_ptr(), qkv[:, 1].data_ptr(), qkv[:, 2].data_ptr(), o.data_ptr(), lse.data_ptr(),
        H * 64, 3 * H * 64, 3 * H * 64, 3 * H * 64, H * 64, cu.data_ptr(), B, T, mx, H, 64, slopes.data_ptr(),
        float(c["scale"]), mb.MB_BF16, got[:, 0].data_ptr(), got[:, 1].data_ptr(), got[:, 2].data_ptr(),
        3 * H * 64, 3 * H * 64, 3 * H * 64, None, None, None, torch.cuda.current_stream().cuda_stream)
    assert st == mb.MB_OK, mb.mb_last_error()
    torch.cuda.synchronize()
    assert torch.equal(got, ref), "static-scratch backward differs from the workspace backward"
    return got


@pytest.mark.parametrize("family,first,second,L", [
    ("any-length kernels", [700, 129, 300, 64, 1, 512], [130, 257, 5], 700),       # these use the scratch array
    ("single-tile kernel", [128, 77, 1, 100, 128, 31], [64, 9], 128),              # this one does not touch it
])
def test_static_scratch_backward_equals_workspace_backward_twice(family, first, second, L):
    from paper_2312_17482_amd import binding as mb
    print("no-alloc backward:", family, flush=True)
    H = 3
    case1 = _packed_case(mb, 901, first, L, H)
    _both(mb, *case1, H)
    c, cu, T, mx, qkv, dout = _packed_case(mb, 902, second, L, H)        # smaller input on the same array
    got = _both(mb, c, cu, T, mx, qkv, dout, H)
    # and the second call's result is right, not merely equal: oracle tolerance (bf16: 2e-2 max-abs, 1e-2 rel. Frobenius)
    dQ, dK, dV = orc.attention_bwd(c["do"], c["q"], c["k"], c["v"], c["mask"], orc.alibi_slopes(H), c["scale"])
    idx = np.flatnonzero(c["mask"].reshape(-1))
    for i, ref in enumerate((dQ, dK, dV)):
        ma, rf = err_stats(got[:, i].double().cpu().numpy(), ref.reshape(-1, H, 64)[idx])
        assert ma <= 2e-2 and rf <= 1e-2, (family, i, ma, rf)
