"""GPU parity of the GeGLU feed-forward (forward) against the CPU oracle, through the C ABI.

Tolerances (bf16 storage, fp32 accumulation): for the stored activation a = GeLU(x W1) (*) x V and for y,
max-abs <= 2e-2 and relative Frobenius <= 1e-2, and in addition max-abs <= 2^-6 * max|ref| so that cases
with small outputs are held to the same relative standard.  One case with O(1) weights has |a| up to ~10,
where a correctly rounded bf16 value is already off by 2^-9 relative: there the absolute bound is
max(2e-2, 2^-7 * max|ref|)."""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2312_17482_amd import workloads as wl
from tests.helpers import err_stats

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def mb():
    assert torch.cuda.is_available()
    from paper_2312_17482_amd import binding
    return binding


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).cuda()


def check(name, got, ref, wide=False):
    ma, rf = err_stats(got.double().cpu().numpy(), ref)
    top = float(np.abs(ref).max())
    bound = max(2e-2, 2.0 ** -7 * top) if wide else min(2e-2, max(2.0 ** -6 * top, 1e-30))
    assert ma <= bound and rf <= 1e-2, "%s max_abs=%.3e (bound %.3e) rel_fro=%.3e" % (name, ma, bound, rf)


def run_case(mb, seed, T, hidden, inter, w_std=0.02, T_cap=None, wide=False):
    case = wl.random_ffn_case(seed, T if T_cap is None else T_cap, hidden, inter, w_std)
    x, w1v, w2 = case["x"], case["w1v"], case["w2"]
    y_ref, a_ref = orc.geglu_fwd(x[:T], w1v[:inter], w1v[inter:], w2)
    rows = x.shape[0]
    guard = 2
    act = torch.full((rows + guard, inter), 9.0, dtype=torch.bfloat16, device="cuda")
    y = torch.full((rows + guard, hidden), 9.0, dtype=torch.bfloat16, device="cuda")
    meta = None if T_cap is None else torch.tensor([T, 0], dtype=torch.int32, device="cuda")
    mb.mb_geglu_fwd(dev(x), dev(w1v), dev(w2), meta=meta, act=act[:rows], y=y[:rows])
    torch.cuda.synchronize()
    assert torch.all(act[T:] == 9.0) and torch.all(y[T:] == 9.0), "rows at or beyond T were written"
    check("act", act[:T], a_ref, wide)
    check("y", y[:T], y_ref, wide)
    return act, y


@pytest.mark.parametrize("T,hidden,inter", [(1, 256, 128), (37, 256, 384), (256, 256, 128), (257, 512, 256),
                                            (700, 768, 3072), (1300, 1024, 4096), (2049, 256, 640)])
def test_geglu_forward_parity(mb, T, hidden, inter):
    print("geglu T=%d hidden=%d inter=%d" % (T, hidden, inter), flush=True)
    run_case(mb, 11, T, hidden, inter)


def test_geglu_forward_unit_scale_weights(mb):
    print("geglu unit-scale weights", flush=True)
    run_case(mb, 12, 600, 768, 3072, w_std=1.0 / np.sqrt(768.0), wide=True)


def test_geglu_forward_device_side_row_count(mb):
    print("geglu capacity mode", flush=True)
    run_case(mb, 13, 1111, 768, 3072, T_cap=1536)
    run_case(mb, 14, 256, 256, 128, T_cap=1024)      # whole workgroups beyond T


def test_geglu_forward_full_size_and_repeatable(mb):
    """The feed-forward of the benchmark batch: 26963 packed tokens, hidden 768, intermediate 3072."""
    print("geglu full size", flush=True)
    case = wl.random_ffn_case(15, 26963, 768, 3072)
    y_ref, a_ref = orc.geglu_fwd(case["x"], case["w1v"][:3072], case["w1v"][3072:], case["w2"])
    xd, wd, w2d = dev(case["x"]), dev(case["w1v"]), dev(case["w2"])
    y, act = mb.mb_geglu_fwd(xd, wd, w2d)
    y2, act2 = mb.mb_geglu_fwd(xd, wd, w2d)
    torch.cuda.synchronize()
    check("act", act, a_ref)
    check("y", y, y_ref)
    assert torch.equal(y, y2) and torch.equal(act, act2)


def test_geglu_empty_input(mb):
    x = torch.empty((0, 768), dtype=torch.bfloat16, device="cuda")
    w1v = torch.zeros((6144, 768), dtype=torch.bfloat16, device="cuda")
    w2 = torch.zeros((768, 3072), dtype=torch.bfloat16, device="cuda")
    y, act = mb.mb_geglu_fwd(x, w1v, w2)
    assert y.shape == (0, 768) and act.shape == (0, 3072)
    # T = 0 on the device with a non-zero capacity: nothing is written
    xx = torch.zeros((512, 768), dtype=torch.bfloat16, device="cuda")
    yy = torch.full((512, 768), 9.0, dtype=torch.bfloat16, device="cuda")
    aa = torch.full((512, 3072), 9.0, dtype=torch.bfloat16, device="cuda")
    meta = torch.zeros(2, dtype=torch.int32, device="cuda")
    mb.mb_geglu_fwd(xx, w1v, w2, meta=meta, act=aa, y=yy)
    torch.cuda.synchronize()
    assert torch.all(yy == 9.0) and torch.all(aa == 9.0)


@pytest.mark.parametrize("T,n_in,n_out", [(300, 768, 6144), (513, 3072, 768), (64, 128, 192), (1000, 256, 1024),
                                          (257, 640, 384), (400, 768, 30528)])   # last: the paper's vocabulary size
def test_linear_forward_parity(mb, T, n_in, n_out):
    print("linear T=%d n_in=%d n_out=%d" % (T, n_in, n_out), flush=True)
    rng = np.random.default_rng(21)
    x = wl.round_to_bf16(rng.standard_normal((T, n_in), dtype=np.float32))
    wt = wl.round_to_bf16(rng.standard_normal((n_out, n_in), dtype=np.float32) / np.float32(np.sqrt(n_in)))
    y = torch.full((T + 2, n_out), 9.0, dtype=torch.bfloat16, device="cuda")
    mb.mb_linear_fwd(dev(x), dev(wt), y=y[:T])
    torch.cuda.synchronize()
    assert torch.all(y[T:] == 9.0)
    check("y", y[:T], orc.linear_fwd(x, wt), wide=True)


def test_gelu_gate_parity_and_unfused_arrangements(mb):
    """The activation pass alone, and the two unfused arrangements of the appendix on GLU implementations
    (two projections; one double-width projection, sliced) against the oracle and against the fused call."""
    print("gelu gate / unfused arrangements", flush=True)
    T, hidden, inter = 900, 768, 3072
    case = wl.random_ffn_case(22, T, hidden, inter)
    x, w1v, w2 = case["x"], case["w1v"], case["w2"]
    y_ref, a_ref = orc.geglu_fwd(x, w1v[:inter], w1v[inter:], w2)
    xd, wd, w2d = dev(x), dev(w1v), dev(w2)
    # activation pass on given h, g (wide range, both signs)
    rng = np.random.default_rng(23)
    h = wl.round_to_bf16(rng.standard_normal((T, inter), dtype=np.float32) * 2.5)
    g = wl.round_to_bf16(rng.standard_normal((T, inter), dtype=np.float32))
    act = mb.mb_gelu_gate(dev(h), dev(g))
    check("gelu_gate", act, orc.gelu_gate(h, g), wide=True)
    # (C) one double-width projection, stored and sliced
    hg = mb.mb_linear_fwd(xd, wd)
    act_c = mb.mb_gelu_gate(hg[:, :inter], hg[:, inter:])
    y_c = mb.mb_linear_fwd(act_c, w2d)
    # (B) two separate projections
    h_b = mb.mb_linear_fwd(xd, wd[:inter].contiguous())
    g_b = mb.mb_linear_fwd(xd, wd[inter:].contiguous())
    act_b = mb.mb_gelu_gate(h_b, g_b)
    y_b = mb.mb_linear_fwd(act_b, w2d)
    y_f, act_f = mb.mb_geglu_fwd(xd, wd, w2d)
    torch.cuda.synchronize()
    # (the unfused arrangements store x W1 and x V in bf16 before the activation: one more rounding per
    # factor than the fused call, hence the bound that scales with the largest value for them)
    for name, a_, y_, wide in (("sliced", act_c, y_c, True), ("separate", act_b, y_b, True), ("fused", act_f, y_f, False)):
        check("act " + name, a_, a_ref, wide)
        check("y " + name, y_, y_ref, wide)
    assert torch.equal(act_b, act_c) and torch.equal(y_b, y_c)     # same arithmetic, different buffers
    # capacity mode of the pieces
    meta = torch.tensor([500, 0], dtype=torch.int32, device="cuda")
    yy = torch.full((T, inter), 9.0, dtype=torch.bfloat16, device="cuda")
    mb.mb_linear_fwd(xd, wd[:inter].contiguous(), meta=meta, y=yy)
    aa = torch.full((T, inter), 9.0, dtype=torch.bfloat16, device="cuda")
    mb.mb_gelu_gate(hg[:, :inter], hg[:, inter:], meta=meta, act=aa)
    torch.cuda.synchronize()
    assert torch.all(yy[500:] == 9.0) and torch.equal(yy[:500], h_b[:500])
    assert torch.all(aa[500:] == 9.0) and torch.equal(aa[:500], act_c[:500])


def check_f32(name, got, ref):
    ma, rf = err_stats(got.double().cpu().numpy(), ref)
    top = float(np.abs(ref).max())
    assert rf <= 1e-2 and ma <= 2.0 ** -6 * top, "%s max_abs=%.3e (max|ref| %.3e) rel_fro=%.3e" % (name, ma, top, rf)


@pytest.mark.parametrize("T,hidden,inter,w_std", [(300, 256, 256, 0.05), (1000, 768, 3072, 0.02), (65, 512, 768, 0.04),
                                                  (2500, 768, 3072, 0.02)])
def test_geglu_backward_parity(mb, T, hidden, inter, w_std):
    """dx (bf16) and the fp32 weight gradients against the oracle's textbook derivative.  Weight gradients are
    sums over T tokens of products of bf16-rounded factors: relative Frobenius <= 1e-2, max-abs <= 2^-6 max|ref|."""
    print("geglu backward T=%d hidden=%d inter=%d" % (T, hidden, inter), flush=True)
    case = wl.random_ffn_case(31, T, hidden, inter, w_std)
    x, w1v, w2, dy = case["x"], case["w1v"], case["w2"], case["dy"]
    dx_ref, dw1_ref, dv_ref, dw2_ref = orc.geglu_bwd(dy, x, w1v[:inter], w1v[inter:], w2)
    xd, wd, w2d, dyd = dev(x), dev(w1v), dev(w2), dev(dy)
    y, act = mb.mb_geglu_fwd(xd, wd, w2d)
    guard = 2
    dx = torch.full((T + guard, hidden), 9.0, dtype=torch.bfloat16, device="cuda")
    _, dw1v, dw2 = mb.mb_geglu_bwd(dyd, xd, wd, w2d, act, dx=dx[:T])
    torch.cuda.synchronize()
    assert torch.all(dx[T:] == 9.0)
    check("dx", dx[:T], dx_ref, wide=True)
    check_f32("dw1", dw1v[:inter], dw1_ref)
    check_f32("dv", dw1v[inter:], dv_ref)
    check_f32("dw2", dw2, dw2_ref)
    # run-to-run identical (fixed summation order)
    dx2, dw1v2, dw22 = mb.mb_geglu_bwd(dyd, xd, wd, w2d, act)
    torch.cuda.synchronize()
    assert torch.equal(dx2, dx[:T]) and torch.equal(dw1v2, dw1v) and torch.equal(dw22, dw2)
    # with the projections handed over by the unfused forward instead of computed again: same numbers
    hg = mb.mb_linear_fwd(xd, wd)
    dx3, dw1v3, dw23 = mb.mb_geglu_bwd(dyd, xd, wd, w2d, act, hg=hg)
    torch.cuda.synchronize()
    assert torch.equal(dx3, dx[:T]) and torch.equal(dw1v3, dw1v) and torch.equal(dw23, dw2)


def test_geglu_backward_device_side_row_count_and_empty(mb):
    print("geglu backward capacity mode", flush=True)
    T_cap, T, hidden, inter = 1024, 333, 256, 512
    case = wl.random_ffn_case(32, T_cap, hidden, inter, 0.05)
    x, w1v, w2, dy = case["x"], case["w1v"], case["w2"], case["dy"]
    dx_ref, dw1_ref, dv_ref, dw2_ref = orc.geglu_bwd(dy[:T], x[:T], w1v[:inter], w1v[inter:], w2)
    xd, wd, w2d, dyd = dev(x), dev(w1v), dev(w2), dev(dy)
    meta = torch.tensor([T, 0], dtype=torch.int32, device="cuda")
    y, act = mb.mb_geglu_fwd(xd, wd, w2d, meta=meta)
    dx = torch.full((T_cap, hidden), 9.0, dtype=torch.bfloat16, device="cuda")
    _, dw1v, dw2 = mb.mb_geglu_bwd(dyd, xd, wd, w2d, act, meta=meta, dx=dx)
    torch.cuda.synchronize()
    assert torch.all(dx[T:] == 9.0)
    check("dx", dx[:T], dx_ref, wide=True)
    check_f32("dw1", dw1v[:inter], dw1_ref)
    check_f32("dv", dw1v[inter:], dv_ref)
    check_f32("dw2", dw2, dw2_ref)
    # no tokens at all: weight gradients are zeros, dx untouched
    meta0 = torch.zeros(2, dtype=torch.int32, device="cuda")
    dx0 = torch.full((T_cap, hidden), 9.0, dtype=torch.bfloat16, device="cuda")
    _, dw1v0, dw20 = mb.mb_geglu_bwd(dyd, xd, wd, w2d, act, meta=meta0, dx=dx0)
    torch.cuda.synchronize()
    assert torch.all(dx0 == 9.0) and torch.all(dw1v0 == 0) and torch.all(dw20 == 0)
