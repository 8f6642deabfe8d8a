"""ctypes binding of libmosaicattn.so: same names as the C ABI, argument marshalling only.

Tensors are torch tensors used purely as device buffers (data_ptr, shape, stride); every step of
the path runs inside the HIP library.  Importing this module raises if the library is not built:
there is no CPU or PyTorch fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import c_char_p, c_float, c_int, c_int64, c_size_t, c_void_p

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libmosaicattn.so")
if not os.path.exists(_LIB_PATH):
    raise ImportError(
        "libmosaicattn.so is not built (%s). Run `python -c 'import __graft_entry__ as g; g.build()'`." % _LIB_PATH)
_lib = ctypes.CDLL(_LIB_PATH)

MB_OK, MB_ERR_INVALID_ARG, MB_ERR_UNSUPPORTED, MB_ERR_WORKSPACE, MB_ERR_HIP = range(5)
MB_F32, MB_BF16 = 0, 1

EXPORTS = ("mb_last_error", "mb_version", "mb_alibi_slopes", "mb_unpad_index", "mb_read_meta", "mb_unpad",
           "mb_pad", "mb_zero_padding", "mb_alibi_attn_fwd", "mb_alibi_attn_fwd_workspace_bytes",
           "mb_alibi_attn_bwd_workspace_bytes",
           "mb_alibi_attn_bwd", "mb_add_layernorm_fwd", "mb_add_layernorm_bwd_workspace_bytes",
           "mb_add_layernorm_bwd", "mb_geglu_fwd", "mb_geglu_bwd_workspace_bytes", "mb_geglu_bwd", "mb_linear_fwd", "mb_gelu_gate", "mb_probe_ceiling",
           "mb_alibi_attn_bwd_static", "mb_device_status", "mb_attn_plan_bytes", "mb_attn_plan", "mb_probe_bwd_traffic")

_lib.mb_last_error.restype = c_char_p
_lib.mb_last_error.argtypes = []
_lib.mb_version.restype = c_int
_lib.mb_version.argtypes = []
_lib.mb_alibi_slopes.restype = c_int
_lib.mb_alibi_slopes.argtypes = [c_int, c_void_p]
_lib.mb_unpad_index.restype = c_int
_lib.mb_unpad_index.argtypes = [c_void_p, c_int, c_int, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
_lib.mb_read_meta.restype = c_int
_lib.mb_read_meta.argtypes = [c_void_p, c_void_p, c_void_p]
_lib.mb_unpad.restype = c_int
_lib.mb_unpad.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_int, c_int, c_void_p, c_void_p]
_lib.mb_pad.restype = c_int
_lib.mb_pad.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
_lib.mb_zero_padding.restype = c_int
_lib.mb_zero_padding.argtypes = [c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_int, c_void_p, c_void_p]
_lib.mb_alibi_attn_fwd.restype = c_int
_lib.mb_alibi_attn_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, c_int64, c_void_p, c_int, c_int,
                                   c_int, c_int, c_int, c_void_p, c_float, c_int, c_void_p, c_int64, c_void_p,
                                   c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_void_p]
_lib.mb_attn_plan_bytes.restype = c_size_t
_lib.mb_attn_plan_bytes.argtypes = [c_int, c_int, c_int]
_lib.mb_attn_plan.restype = c_int
_lib.mb_attn_plan.argtypes = [c_void_p, c_void_p, c_int, c_int, c_int, c_void_p, c_size_t, c_void_p]
_lib.mb_alibi_attn_fwd_workspace_bytes.restype = c_size_t
_lib.mb_alibi_attn_fwd_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int, c_int]
_lib.mb_alibi_attn_bwd_workspace_bytes.restype = c_size_t
_lib.mb_alibi_attn_bwd_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int, c_int, c_int]
_lib.mb_alibi_attn_bwd.restype = c_int
_lib.mb_alibi_attn_bwd.argtypes = ([c_void_p] * 6 + [c_int64] * 5 + [c_void_p] + [c_int] * 5 + [c_void_p, c_float, c_int]
                                   + [c_void_p] * 3 + [c_int64] * 3
                                   + [c_void_p, c_size_t, c_void_p, c_void_p, c_void_p, c_void_p])
_lib.mb_alibi_attn_bwd_static.restype = c_int
_lib.mb_alibi_attn_bwd_static.argtypes = ([c_void_p] * 6 + [c_int64] * 5 + [c_void_p] + [c_int] * 5
                                          + [c_void_p, c_float, c_int] + [c_void_p] * 3 + [c_int64] * 3
                                          + [c_void_p, c_void_p, c_void_p, c_void_p])
_lib.mb_device_status.restype = c_int
_lib.mb_device_status.argtypes = [c_void_p]
MB_STATIC_SCRATCH_BYTES = 16 << 20

_lib.mb_add_layernorm_fwd.restype = c_int
_lib.mb_add_layernorm_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_int, c_float, c_int,
                                      c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p]
_lib.mb_add_layernorm_bwd_workspace_bytes.restype = c_size_t
_lib.mb_add_layernorm_bwd_workspace_bytes.argtypes = [c_int]
_lib.mb_add_layernorm_bwd.restype = c_int
_lib.mb_add_layernorm_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_int, c_int,
                                      c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p, c_void_p]
_lib.mb_geglu_bwd_workspace_bytes.restype = c_size_t
_lib.mb_geglu_bwd_workspace_bytes.argtypes = [c_int, c_int, c_int, c_int]
_lib.mb_geglu_bwd.restype = c_int
_lib.mb_geglu_bwd.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_int, c_int, c_int,
                              c_void_p, c_void_p, c_void_p, c_void_p, c_size_t, c_void_p]
_lib.mb_probe_bwd_traffic.restype = c_int
_lib.mb_probe_bwd_traffic.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p, c_void_p, c_int, c_int, c_void_p]
_lib.mb_probe_ceiling.restype = c_int
_lib.mb_probe_ceiling.argtypes = [c_int, c_int, c_void_p, c_void_p, c_void_p]
_lib.mb_linear_fwd.restype = c_int
_lib.mb_linear_fwd.argtypes = [c_void_p, c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p]
_lib.mb_gelu_gate.restype = c_int
_lib.mb_gelu_gate.argtypes = [c_void_p, c_void_p, c_int64, c_int, c_void_p, c_int, c_int, c_void_p, c_void_p]
_lib.mb_geglu_fwd.restype = c_int
_lib.mb_geglu_fwd.argtypes = [c_void_p, c_void_p, c_void_p, c_int, c_void_p, c_int, c_int, c_int, c_void_p, c_void_p,
                              c_void_p]


class MosaicAttnError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__("libmosaicattn status %d: %s" % (status, message))
        self.status = status


def raw():
    """The ctypes library handle, for tests of the C ABI itself."""
    return _lib


def _check(status: int) -> None:
    if status != MB_OK:
        raise MosaicAttnError(status, _lib.mb_last_error().decode())


def _ptr(t) -> int | None:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return MB_F32
    if t.dtype == torch.bfloat16:
        return MB_BF16
    raise TypeError("unsupported dtype %s" % t.dtype)


def _row_stride(t: torch.Tensor) -> int:
    """[T, H, D] view with contiguous (H, D): returns the token stride in elements."""
    assert t.dim() == 3 and t.stride(2) == 1 and t.stride(1) == t.shape[2], "need [T, H, D] with dense (H, D)"
    return t.stride(0) if t.shape[0] > 1 else max(t.stride(0), t.shape[1] * t.shape[2])


def mb_version() -> int:
    return _lib.mb_version()


def mb_last_error() -> str:
    return _lib.mb_last_error().decode()


def mb_alibi_slopes(H: int) -> torch.Tensor:
    """Host tensor [H] float32 of the head slopes."""
    out = torch.empty(max(H, 0), dtype=torch.float32)
    _check(_lib.mb_alibi_slopes(H, out.data_ptr() if H > 0 else None))
    return out


def mb_unpad_index(mask: torch.Tensor):
    """mask [B, L] int32 on the GPU -> (seqlens [B], cu_seqlens [B+1], indices [B*L] (first T valid), meta [2])."""
    assert mask.dtype == torch.int32 and mask.dim() == 2 and mask.is_contiguous()
    B, L = mask.shape
    dev = mask.device
    seqlens = torch.empty(max(B, 1), dtype=torch.int32, device=dev)[:B]
    cu = torch.empty(B + 1, dtype=torch.int32, device=dev)
    indices = torch.empty(max(B * L, 1), dtype=torch.int32, device=dev)[:B * L]
    meta = torch.empty(2, dtype=torch.int32, device=dev)
    _check(_lib.mb_unpad_index(_ptr(mask), B, L, _ptr(seqlens), _ptr(cu), _ptr(indices), _ptr(meta), _stream()))
    return seqlens, cu, indices, meta


def mb_read_meta(meta: torch.Tensor):
    host = (ctypes.c_int32 * 2)()
    _check(_lib.mb_read_meta(_ptr(meta), ctypes.addressof(host), _stream()))
    return int(host[0]), int(host[1])


def mb_unpad(padded: torch.Tensor, indices: torch.Tensor, T_cap: int, meta, out: torch.Tensor | None = None):
    """padded [B*L, W] (any leading shape flattened by the caller) -> packed [T_cap, W]; rows < T written."""
    assert padded.dim() == 2 and padded.is_contiguous()
    W = padded.shape[1]
    if out is None:
        out = torch.empty((T_cap, W), dtype=padded.dtype, device=padded.device)
    assert out.is_contiguous() and out.shape[1] == W and out.shape[0] >= T_cap
    _check(_lib.mb_unpad(_ptr(padded), _ptr(indices), T_cap, _ptr(meta), W, _dtype_code(padded), _ptr(out), _stream()))
    return out


def mb_pad(packed: torch.Tensor, indices: torch.Tensor, T_cap: int, meta, B: int, L: int,
           out: torch.Tensor | None = None):
    """packed [>=T, W] -> padded [B*L, W], zero at padded positions."""
    assert packed.dim() == 2 and packed.is_contiguous()
    W = packed.shape[1]
    if out is None:
        out = torch.empty((B * L, W), dtype=packed.dtype, device=packed.device)
    assert out.is_contiguous() and tuple(out.shape) == (B * L, W)
    _check(_lib.mb_pad(_ptr(packed), _ptr(indices), T_cap, _ptr(meta), B, L, W, _dtype_code(packed), _ptr(out),
                       _stream()))
    return out


def mb_zero_padding(padded: torch.Tensor, indices: torch.Tensor, T_cap: int, meta, B: int, L: int):
    """Zero the rows of padded [B*L, W] that `indices` does not list."""
    assert padded.dim() == 2 and padded.is_contiguous() and padded.shape[0] == B * L
    _check(_lib.mb_zero_padding(_ptr(indices), T_cap, _ptr(meta), B, L, padded.shape[1], _dtype_code(padded),
                                _ptr(padded), _stream()))
    return padded


def mb_alibi_attn_fwd(q, k, v, cu_seqlens, max_seqlen: int, slopes, softmax_scale: float, out=None, lse=None,
                      token_rows=None, T=None, workspace=None, key_lens=None, plan=None):
    """q, k, v: [T, H, D] views (token stride free).  Returns (o [T, H, D], lse [H, T] float32).
    With token_rows the views are over a padded batch ([B*L, H, D]) and T (the lse pitch) must be given."""
    _, H, D = q.shape
    T = q.shape[0] if T is None else T
    B = cu_seqlens.numel() - 1
    if out is None:
        out = torch.empty((q.shape[0], H, D), dtype=q.dtype, device=q.device)
    if lse is None:
        lse = torch.empty((H, T), dtype=torch.float32, device=q.device)
    need = 0 if plan is not None else mb_alibi_attn_fwd_workspace_bytes(B, T, max_seqlen, H, D, _dtype_code(q))
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    _check(_lib.mb_alibi_attn_fwd(_ptr(q), _ptr(k), _ptr(v), _row_stride(q), _row_stride(k), _row_stride(v),
                                  _ptr(cu_seqlens), B, T, max_seqlen, H, D, _ptr(slopes), float(softmax_scale),
                                  _dtype_code(q), _ptr(out), _row_stride(out), _ptr(lse), _ptr(workspace),
                                  0 if workspace is None else workspace.numel(), _ptr(key_lens), _ptr(token_rows),
                                  _ptr(plan), _stream()))
    return out, lse


def mb_attn_plan_bytes(B: int, max_seqlen: int, H: int) -> int:
    return int(_lib.mb_attn_plan_bytes(B, max_seqlen, H))


def mb_attn_plan(cu_seqlens, max_seqlen: int, H: int, key_lens=None, plan=None):
    """Builds the work plan of the any-length attention kernels once for a batch; returns the plan buffer."""
    B = cu_seqlens.numel() - 1
    need = mb_attn_plan_bytes(B, max_seqlen, H)
    if plan is None:
        plan = torch.empty(max(need, 16), dtype=torch.uint8, device=cu_seqlens.device)
    _check(_lib.mb_attn_plan(_ptr(cu_seqlens), _ptr(key_lens), B, max_seqlen, H, _ptr(plan), plan.numel(), _stream()))
    return plan


def mb_alibi_attn_fwd_workspace_bytes(B, T, max_seqlen, H, D, dtype_code) -> int:
    return int(_lib.mb_alibi_attn_fwd_workspace_bytes(B, T, max_seqlen, H, D, dtype_code))


def mb_alibi_attn_bwd_workspace_bytes(B, T, max_seqlen, H, D, dtype_code) -> int:
    return int(_lib.mb_alibi_attn_bwd_workspace_bytes(B, T, max_seqlen, H, D, dtype_code))


def mb_alibi_attn_bwd(dout, q, k, v, o, lse, cu_seqlens, max_seqlen: int, slopes, softmax_scale: float,
                      dq=None, dk=None, dv=None, workspace=None, token_rows=None, T=None, key_lens=None, plan=None):
    """Returns (dq, dk, dv), each [T, H, D] (padded-batch views when token_rows is given)."""
    R, H, D = q.shape
    T = R if T is None else T
    B = cu_seqlens.numel() - 1
    dq = torch.empty((R, H, D), dtype=q.dtype, device=q.device) if dq is None else dq
    dk = torch.empty((R, H, D), dtype=q.dtype, device=q.device) if dk is None else dk
    dv = torch.empty((R, H, D), dtype=q.dtype, device=q.device) if dv is None else dv
    need = mb_alibi_attn_bwd_workspace_bytes(B, T, max_seqlen, H, D, _dtype_code(q))
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    _check(_lib.mb_alibi_attn_bwd(_ptr(dout), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _row_stride(dout),
                                  _row_stride(q), _row_stride(k), _row_stride(v), _row_stride(o), _ptr(cu_seqlens),
                                  B, T, max_seqlen, H, D, _ptr(slopes), float(softmax_scale), _dtype_code(q),
                                  _ptr(dq), _ptr(dk), _ptr(dv), _row_stride(dq), _row_stride(dk), _row_stride(dv),
                                  _ptr(workspace), workspace.numel(), _ptr(key_lens), _ptr(token_rows), _ptr(plan),
                                  _stream()))
    return dq, dk, dv


def mb_alibi_attn_bwd_static(dout, q, k, v, o, lse, cu_seqlens, max_seqlen: int, slopes, softmax_scale: float,
                             dq, dk, dv, token_rows=None, T=None, key_lens=None, plan=None):
    """mb_alibi_attn_bwd on the library's static scratch array.  This wrapper allocates nothing either:
    the outputs dq, dk, dv must be given."""
    R, H, D = q.shape
    T = R if T is None else T
    B = cu_seqlens.numel() - 1
    _check(_lib.mb_alibi_attn_bwd_static(_ptr(dout), _ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), _row_stride(dout),
                                         _row_stride(q), _row_stride(k), _row_stride(v), _row_stride(o),
                                         _ptr(cu_seqlens), B, T, max_seqlen, H, D, _ptr(slopes), float(softmax_scale),
                                         _dtype_code(q), _ptr(dq), _ptr(dk), _ptr(dv), _row_stride(dq),
                                         _row_stride(dk), _row_stride(dv), _ptr(key_lens), _ptr(token_rows), _ptr(plan),
                                         _stream()))
    return dq, dk, dv


def mb_device_status() -> None:
    """Raises MosaicAttnError(MB_ERR_INVALID_ARG) if an attention call since the last check met a sequence
    longer than its max_seqlen; clears the device's sticky word.  Synchronises the current stream."""
    _check(_lib.mb_device_status(_stream()))


def mb_add_layernorm_fwd(x, r, gamma, beta, eps: float, T_cap=None, meta=None, y=None, s=None, mean=None, rstd=None,
                         y_rows=None):
    """x, r: [rows, W] (r may be None).  Returns (y, s, mean, rstd); s is x itself when r is None.
    With y_rows, y must be given: a padded batch whose row y_rows[t] receives the result of token t."""
    assert x.dim() == 2 and x.is_contiguous()
    rows, W = x.shape
    T_cap = rows if T_cap is None else T_cap
    assert y_rows is None or y is not None
    y = torch.empty_like(x) if y is None else y
    if r is not None and s is None:
        s = torch.empty_like(x)
    mean = torch.empty(rows, dtype=torch.float32, device=x.device) if mean is None else mean
    rstd = torch.empty(rows, dtype=torch.float32, device=x.device) if rstd is None else rstd
    _check(_lib.mb_add_layernorm_fwd(_ptr(x), _ptr(r), _ptr(gamma), _ptr(beta), T_cap, _ptr(meta), W, float(eps),
                                     _dtype_code(x), _ptr(y), _ptr(s) if r is not None else None, _ptr(mean),
                                     _ptr(rstd), _ptr(y_rows), _stream()))
    return y, (s if r is not None else x), mean, rstd


def mb_add_layernorm_bwd_workspace_bytes(W: int) -> int:
    return int(_lib.mb_add_layernorm_bwd_workspace_bytes(W))


def mb_add_layernorm_bwd(dy, s, gamma, mean, rstd, T_cap=None, meta=None, ds=None, dgamma=None, dbeta=None,
                         workspace=None, dy_rows=None):
    """Returns (ds [rows, W], dgamma [W] float32, dbeta [W] float32).
    With dy_rows, dy is a padded batch and token t's row is dy[dy_rows[t]]."""
    rows, W = s.shape
    T_cap = rows if T_cap is None else T_cap
    ds = torch.empty_like(s) if ds is None else ds
    dgamma = torch.empty(W, dtype=torch.float32, device=s.device) if dgamma is None else dgamma
    dbeta = torch.empty(W, dtype=torch.float32, device=s.device) if dbeta is None else dbeta
    if workspace is None:
        workspace = torch.empty(mb_add_layernorm_bwd_workspace_bytes(W), dtype=torch.uint8, device=s.device)
    _check(_lib.mb_add_layernorm_bwd(_ptr(dy), _ptr(s), _ptr(gamma), _ptr(mean), _ptr(rstd), T_cap, _ptr(meta), W,
                                     _dtype_code(s), _ptr(ds), _ptr(dgamma), _ptr(dbeta), _ptr(workspace),
                                     workspace.numel(), _ptr(dy_rows), _stream()))
    return ds, dgamma, dbeta


def mb_geglu_fwd(x, w1v, w2, T_cap=None, meta=None, act=None, y=None):
    """x [rows, hidden]; w1v [2*inter, hidden] (W1 transposed over V transposed); w2 [hidden, inter] (W2
    transposed).  Returns (y [rows, hidden], act [rows, inter])."""
    assert x.dim() == 2 and x.is_contiguous() and w1v.is_contiguous() and w2.is_contiguous()
    rows, hidden = x.shape
    inter = w2.shape[1]
    assert tuple(w1v.shape) == (2 * inter, hidden) and tuple(w2.shape) == (hidden, inter)
    T_cap = rows if T_cap is None else T_cap
    act = torch.empty((rows, inter), dtype=x.dtype, device=x.device) if act is None else act
    y = torch.empty_like(x) if y is None else y
    _check(_lib.mb_geglu_fwd(_ptr(x), _ptr(w1v), _ptr(w2), T_cap, _ptr(meta), hidden, inter, _dtype_code(x),
                             _ptr(act), _ptr(y), _stream()))
    return y, act


def mb_linear_fwd(x, wt, T_cap=None, meta=None, y=None):
    """y = x @ wt.T for x [rows, n_in], wt [n_out, n_in]."""
    assert x.dim() == 2 and x.is_contiguous() and wt.is_contiguous() and wt.shape[1] == x.shape[1]
    rows, n_in = x.shape
    n_out = wt.shape[0]
    T_cap = rows if T_cap is None else T_cap
    y = torch.empty((rows, n_out), dtype=x.dtype, device=x.device) if y is None else y
    _check(_lib.mb_linear_fwd(_ptr(x), _ptr(wt), T_cap, _ptr(meta), n_in, n_out, _dtype_code(x), _ptr(y), _stream()))
    return y


def mb_gelu_gate(h, gate, T_cap=None, meta=None, act=None):
    """act = GeLU(h) * gate; h and gate are [rows, inter] views with the same row stride (two buffers, or
    the halves of one [rows, 2*inter] buffer)."""
    assert h.dim() == 2 and h.shape == gate.shape and h.stride(1) == 1 and gate.stride(1) == 1
    assert h.stride(0) == gate.stride(0)
    rows, inter = h.shape
    T_cap = rows if T_cap is None else T_cap
    act = torch.empty((rows, inter), dtype=h.dtype, device=h.device) if act is None else act
    _check(_lib.mb_gelu_gate(_ptr(h), _ptr(gate), h.stride(0), T_cap, _ptr(meta), inter, _dtype_code(h), _ptr(act),
                             _stream()))
    return act


def mb_probe_ceiling(kind: int, iters: int, out) -> float:
    """Enqueues one probe launch (0: bf16 MFMA, 1: fp32 FMA, 2: fp32 exp); returns its work (flops or exps)."""
    work = ctypes.c_double(0.0)
    _check(_lib.mb_probe_ceiling(kind, iters, _ptr(out), ctypes.byref(work), _stream()))
    return work.value


def mb_probe_bwd_traffic(qkv, dout, o, dqkv, cu_seqlens) -> None:
    """Enqueues the traffic-only twin of the single-tile backward: qkv [T, 3, H, 64], dout / o [T, H, 64] read,
    dqkv [T, 3, H, 64] overwritten with meaningless values."""
    H = dout.shape[1]
    assert qkv.is_contiguous() and dout.is_contiguous() and o.is_contiguous() and dqkv.is_contiguous()
    _check(_lib.mb_probe_bwd_traffic(_ptr(qkv), _ptr(dout), _ptr(o), _ptr(dqkv), _ptr(cu_seqlens),
                                     cu_seqlens.numel() - 1, H, _stream()))


def mb_geglu_bwd_workspace_bytes(T_cap: int, hidden: int, inter: int, dtype_code: int = MB_BF16) -> int:
    return int(_lib.mb_geglu_bwd_workspace_bytes(T_cap, hidden, inter, dtype_code))


def mb_geglu_bwd(dy, x, w1v, w2, act, hg=None, T_cap=None, meta=None, dx=None, dw1v=None, dw2=None, workspace=None):
    """Returns (dx [rows, hidden], dw1v [2*inter, hidden] float32, dw2 [hidden, inter] float32).  hg: the stored
    [rows, 2*inter] projections of the unfused forward, or None to have them computed again."""
    assert hg is None or hg.is_contiguous()
    rows, hidden = x.shape
    inter = w2.shape[1]
    T_cap = rows if T_cap is None else T_cap
    dx = torch.empty_like(x) if dx is None else dx
    dw1v = torch.empty((2 * inter, hidden), dtype=torch.float32, device=x.device) if dw1v is None else dw1v
    dw2 = torch.empty((hidden, inter), dtype=torch.float32, device=x.device) if dw2 is None else dw2
    if workspace is None:
        workspace = torch.empty(max(mb_geglu_bwd_workspace_bytes(T_cap, hidden, inter, _dtype_code(x)), 256),
                                dtype=torch.uint8, device=x.device)
    _check(_lib.mb_geglu_bwd(_ptr(dy), _ptr(x), _ptr(w1v), _ptr(w2), _ptr(act), _ptr(hg), T_cap, _ptr(meta), hidden, inter,
                             _dtype_code(x), _ptr(dx), _ptr(dw1v), _ptr(dw2), _ptr(workspace), workspace.numel(),
                             _stream()))
    return dx, dw1v, dw2
