"""Shared test plumbing: runs the HIP path through the binding, and the oracle beside it."""
import numpy as np
import torch

from oracle import mosaic_oracle as orc


def to_dev(x: np.ndarray, bf16: bool) -> torch.Tensor:
    t = torch.from_numpy(np.ascontiguousarray(x))
    if bf16:
        t = t.to(torch.bfloat16)          # exact: the values are already bf16-representable
    return t.cuda()


def run_hip_path(mb, batch, slopes_host: torch.Tensor, bf16: bool, scale=None):
    """unpad_index -> unpad(fused QKV, dO) -> fwd -> bwd -> pad(O), pad(dQKV), all through the C ABI.

    Returns numpy arrays in the padded layout [B, L, H, D] (float64) plus the index maps.
    """
    q, k, v, do, mask = batch["q"], batch["k"], batch["v"], batch["do"], batch["mask"]
    B, L, H, D = q.shape
    scale = batch["scale"] if scale is None else scale
    mask_d = torch.from_numpy(mask.astype(np.int32)).cuda()
    seqlens, cu, indices, meta = mb.mb_unpad_index(mask_d)
    T, max_seqlen = mb.mb_read_meta(meta)
    qkv_padded = to_dev(np.concatenate([q.reshape(B * L, H * D), k.reshape(B * L, H * D), v.reshape(B * L, H * D)], axis=1), bf16)
    do_padded = to_dev(do.reshape(B * L, H * D), bf16)
    qkv = mb.mb_unpad(qkv_padded, indices, B * L, meta)[:T].view(T, 3, H, D)
    dout = mb.mb_unpad(do_padded, indices, B * L, meta)[:T].view(T, H, D)
    slopes = slopes_host.cuda()
    out = {"seqlens": seqlens.cpu().numpy(), "cu": cu.cpu().numpy(), "indices": indices[:T].cpu().numpy(),
           "T": T, "max_seqlen": max_seqlen}
    if T == 0:
        return out
    o, lse = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, max_seqlen, slopes, scale)
    dqkv = torch.empty_like(qkv)
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, max_seqlen, slopes, scale,
                         dq=dqkv[:, 0], dk=dqkv[:, 1], dv=dqkv[:, 2])
    o_pad = mb.mb_pad(o.view(T, H * D), indices, B * L, meta, B, L)
    dqkv_pad = mb.mb_pad(dqkv.view(T, 3 * H * D), indices, B * L, meta, B, L).view(B, L, 3, H, D)
    torch.cuda.synchronize()
    out.update(o=o_pad.view(B, L, H, D).double().cpu().numpy(), lse=lse.double().cpu().numpy(),
               dq=dqkv_pad[:, :, 0].double().cpu().numpy(), dk=dqkv_pad[:, :, 1].double().cpu().numpy(),
               dv=dqkv_pad[:, :, 2].double().cpu().numpy(),
               o_packed=o, lse_dev=lse, dqkv_packed=dqkv)
    return out


def run_oracle(batch, slopes64: np.ndarray, scale=None, seq_ids=None):
    """Oracle on the padded layout; with seq_ids, each chosen sequence is cropped to its own length
    first (padding width does not change the result) so long, sparse batches stay cheap."""
    scale = batch["scale"] if scale is None else scale
    q, k, v, do, mask = batch["q"], batch["k"], batch["v"], batch["do"], batch["mask"]
    if seq_ids is None:
        O, LSE = orc.attention_fwd(q, k, v, mask, slopes64, scale)
        dQ, dK, dV = orc.attention_bwd(do, q, k, v, mask, slopes64, scale)
        return {"o": O, "lse": LSE, "dq": dQ, "dk": dK, "dv": dV}
    res = {}
    for b in seq_ids:
        n = int(batch["lengths"][b])
        if n == 0:
            continue
        m1 = np.ones((1, n), dtype=np.int32)
        O, LSE = orc.attention_fwd(q[b:b + 1, :n], k[b:b + 1, :n], v[b:b + 1, :n], m1, slopes64, scale)
        dQ, dK, dV = orc.attention_bwd(do[b:b + 1, :n], q[b:b + 1, :n], k[b:b + 1, :n], v[b:b + 1, :n], m1, slopes64, scale)
        res[b] = {"o": O[0], "lse": LSE[0], "dq": dQ[0], "dk": dK[0], "dv": dV[0]}
    return res


def err_stats(got: np.ndarray, ref: np.ndarray):
    diff = got - ref
    max_abs = float(np.max(np.abs(diff))) if diff.size else 0.0
    denom = float(np.linalg.norm(ref.ravel()))
    rel_f = float(np.linalg.norm(diff.ravel()) / denom) if denom > 0 else float(np.linalg.norm(diff.ravel()))
    return max_abs, rel_f
