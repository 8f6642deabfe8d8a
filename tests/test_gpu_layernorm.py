"""GPU parity of Add & LayerNorm (bf16 storage) against the CPU oracle, through the C ABI.

Tolerances: the stored sum s bit-exact; y and ds (bf16) max-abs <= 2e-2 and relative Frobenius <= 1e-2;
mean / rstd relative 1e-5; dgamma / dbeta (fp32 sums of products of the same bf16 inputs) relative
Frobenius <= 1e-4.  fp32 storage: 1e-5 throughout."""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2312_17482_amd import workloads as wl
from tests.helpers import err_stats

pytestmark = pytest.mark.gpu
EPS = 1e-5        # the usual BERT LayerNorm epsilon... a small constant; the paper does not state one


@pytest.fixture(scope="module")
def mb():
    assert torch.cuda.is_available()
    from paper_2312_17482_amd import binding
    return binding


def make(seed, T, W, bf16=True):
    rng = np.random.default_rng(seed)
    rd = wl.round_to_bf16 if bf16 else (lambda a: a)
    x = rd(rng.standard_normal((T, W), dtype=np.float32) * 1.5)
    r = rd(rng.standard_normal((T, W), dtype=np.float32) + 0.3)
    gamma = rd(1.0 + 0.2 * rng.standard_normal(W, dtype=np.float32))
    beta = rd(0.1 * rng.standard_normal(W, dtype=np.float32))
    dy = rd(rng.standard_normal((T, W), dtype=np.float32))
    return x, r, gamma, beta, dy


def dev(a, bf16):
    t = torch.from_numpy(np.ascontiguousarray(a))
    return (t.to(torch.bfloat16) if bf16 else t).cuda()


@pytest.mark.parametrize("T,W,residual", [(1000, 768, True), (1, 1024, True), (4097, 64, True), (333, 2048, True),
                                          (517, 768, False), (26963, 768, True), (300, 256, True)])
def test_layernorm_bf16_parity(mb, T, W, residual):
    print("layernorm bf16 T=%d W=%d residual=%s" % (T, W, residual), flush=True)
    x, r, gamma, beta, dy = make(7, T, W)
    y_ref, s_ref, mean_ref, rstd_ref = orc.add_layernorm_fwd(x, r if residual else None, gamma, beta, EPS)
    ds_ref, dg_ref, db_ref = orc.add_layernorm_bwd(dy, s_ref, gamma, EPS)
    guard = 3
    xd, rd_, gd, bd, dyd = (dev(a, True) for a in (x, r, gamma, beta, dy))
    y = torch.full((T + guard, W), 9.0, dtype=torch.bfloat16, device="cuda")
    s = torch.full((T + guard, W), 9.0, dtype=torch.bfloat16, device="cuda")
    y_, s_, mean, rstd = mb.mb_add_layernorm_fwd(xd, rd_ if residual else None, gd, bd, EPS, y=y[:T],
                                                 s=s[:T] if residual else None)
    ds = torch.full((T + guard, W), 9.0, dtype=torch.bfloat16, device="cuda")
    _, dgamma, dbeta = mb.mb_add_layernorm_bwd(dyd, s_, gd, mean, rstd, ds=ds[:T])
    torch.cuda.synchronize()
    assert torch.all(y[T:] == 9.0) and torch.all(ds[T:] == 9.0) and torch.all(s[T:] == 9.0)
    assert np.array_equal(s_.double().cpu().numpy(), s_ref), "stored sum is not bit-exact"
    for name, got, ref in (("y", y[:T], y_ref), ("ds", ds[:T], ds_ref)):
        ma, rf = err_stats(got.double().cpu().numpy(), ref)
        assert ma <= 2e-2 and rf <= 1e-2, "%s max_abs=%.3e rel_fro=%.3e" % (name, ma, rf)
    assert np.allclose(mean.double().cpu().numpy(), mean_ref, rtol=1e-5, atol=1e-6)
    assert np.allclose(rstd.double().cpu().numpy(), rstd_ref, rtol=1e-5)
    for name, got, ref in (("dgamma", dgamma, dg_ref), ("dbeta", dbeta, db_ref)):
        ma, rf = err_stats(got.double().cpu().numpy(), ref)
        assert rf <= 1e-4, "%s rel_fro=%.3e" % (name, rf)
    # deterministic column sums
    _, dg2, db2 = mb.mb_add_layernorm_bwd(dyd, s_, gd, mean, rstd)
    assert torch.equal(dg2, dgamma) and torch.equal(db2, dbeta)


def test_layernorm_fp32_and_device_side_row_count(mb):
    T_cap, T, W = 900, 611, 256
    x, r, gamma, beta, dy = make(8, T_cap, W, bf16=False)
    meta = torch.tensor([T, 0], dtype=torch.int32, device="cuda")
    xd, rd_, gd, bd, dyd = (dev(a, False) for a in (x, r, gamma, beta, dy))
    y = torch.full((T_cap, W), 9.0, device="cuda")
    s = torch.full((T_cap, W), 9.0, device="cuda")
    _, _, mean, rstd = mb.mb_add_layernorm_fwd(xd, rd_, gd, bd, EPS, meta=meta, y=y, s=s)
    ds = torch.full((T_cap, W), 9.0, device="cuda")
    _, dgamma, dbeta = mb.mb_add_layernorm_bwd(dyd, s, gd, mean, rstd, meta=meta, ds=ds)
    torch.cuda.synchronize()
    assert torch.all(y[T:] == 9.0) and torch.all(s[T:] == 9.0) and torch.all(ds[T:] == 9.0)
    y_ref, s_ref, _, _ = orc.add_layernorm_fwd(x[:T], r[:T], gamma, beta, EPS, round_sum=False)
    ds_ref, dg_ref, db_ref = orc.add_layernorm_bwd(dy[:T], s_ref, gamma, EPS)
    for got, ref in ((y[:T], y_ref), (s[:T], s_ref), (ds[:T], ds_ref), (dgamma, dg_ref), (dbeta, db_ref)):
        ma, rf = err_stats(got.double().cpu().numpy(), ref)
        assert rf <= 1e-5 and ma <= 1e-4


def test_layernorm_empty_input_writes_zero_column_sums(mb):
    W = 64
    lib = mb.raw()
    dg = torch.full((W,), 5.0, device="cuda")
    db = torch.full((W,), 5.0, device="cuda")
    ws = torch.empty(mb.mb_add_layernorm_bwd_workspace_bytes(W), dtype=torch.uint8, device="cuda")
    assert lib.mb_add_layernorm_bwd(None, None, None, None, None, 0, None, W, mb.MB_BF16, None, dg.data_ptr(),
                                    db.data_ptr(), ws.data_ptr(), ws.numel(), None, None) == 0
    torch.cuda.synchronize()
    assert torch.all(dg == 0) and torch.all(db == 0)


@pytest.mark.parametrize("bf16,W,holes", [(True, 768, False), (True, 1024, True), (False, 96, True)])
def test_layernorm_reads_and_writes_a_padded_batch_directly(mb, bf16, W, holes):
    """y_rows / dy_rows: the scatter of mb_pad in the forward's stores and the gather of mb_unpad in the
    backward's loads give bit for bit what the explicit calls give, for suffix padding and for masks with holes."""
    rng = np.random.default_rng(11)
    B, L = 9, 37
    if holes:
        mask = (rng.random((B, L)) < 0.7).astype(np.int32)
    else:
        mask = wl.suffix_mask(rng.integers(0, L + 1, size=B), L)
    mask[3] = 0
    maskd = torch.from_numpy(mask).cuda()
    _, _, indices, meta = mb.mb_unpad_index(maskd)
    T = int(mask.sum())
    x, r, gamma, beta, dy = make(5, T, W, bf16)
    xd, rd_, gd, bd, dyd = (dev(a, bf16) for a in (x, r, gamma, beta, dy))
    # explicit: packed LayerNorm, then mb_pad
    y, s, mean, rstd = mb.mb_add_layernorm_fwd(xd, rd_, gd, bd, EPS)
    y_padded = mb.mb_pad(y, indices, T, None, B, L)
    # fused: rows scattered by the LayerNorm itself, padding rows zeroed separately
    y2 = torch.full((B * L, W), 7.0, dtype=xd.dtype, device="cuda")
    _, s2, mean2, rstd2 = mb.mb_add_layernorm_fwd(xd, rd_, gd, bd, EPS, y=y2, y_rows=indices)
    mb.mb_zero_padding(y2, indices, T, None, B, L)
    assert torch.equal(y2.view(torch.uint8), y_padded.view(torch.uint8))
    assert torch.equal(s2, s) and torch.equal(mean2, mean) and torch.equal(rstd2, rstd)
    # backward: dy handed over as a padded batch
    dy_padded = mb.mb_pad(dyd, indices, T, None, B, L)
    dy_padded[torch.from_numpy(mask.reshape(-1) == 0).cuda()] = float("nan")   # padding rows must not be read
    ds, dg, db = mb.mb_add_layernorm_bwd(dyd, s, gd, mean, rstd)
    ds2, dg2, db2 = mb.mb_add_layernorm_bwd(dy_padded, s, gd, mean, rstd, dy_rows=indices)
    assert torch.equal(ds2, ds) and torch.equal(dg2, dg) and torch.equal(db2, db)
    # ... and the fused calls agree with the oracle on this very case
    idx = np.flatnonzero(mask.reshape(-1))
    y_ref, s_ref, mean_ref, rstd_ref = orc.add_layernorm_fwd(x, r, gamma, beta, EPS, round_sum=bf16)
    ds_ref, dg_ref, db_ref = orc.add_layernorm_bwd(dy, s_ref, gamma, EPS)
    y_got = y2.double().cpu().numpy()
    tol_abs, tol_rel = (2e-2, 1e-2) if bf16 else (1e-4, 1e-5)
    ma, rf = err_stats(y_got[idx], y_ref)
    assert ma <= tol_abs and rf <= tol_rel, "y (scattered) max_abs=%.3e rel_fro=%.3e" % (ma, rf)
    pad_rows = np.setdiff1d(np.arange(B * L), idx)
    assert not y2.view(torch.int16 if bf16 else torch.int32).cpu().numpy()[pad_rows].any()
    ma, rf = err_stats(ds2.double().cpu().numpy(), ds_ref)
    assert ma <= tol_abs and rf <= tol_rel, "ds (gathered dy) max_abs=%.3e rel_fro=%.3e" % (ma, rf)
    for name, g_, ref in (("dgamma", dg2, dg_ref), ("dbeta", db2, db_ref)):
        _, rf = err_stats(g_.double().cpu().numpy(), ref)
        assert rf <= (1e-4 if bf16 else 1e-5), "%s rel_fro=%.3e" % (name, rf)
