"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded inputs.

Tolerances: integer/index/byte results bit-exact.  bf16 attention outputs and gradients: max-abs
<= 2e-2 and relative Frobenius <= 1e-2.  fp32 path: max-abs <= 1e-4, relative Frobenius <= 1e-5.
Row log-sum-exp: max-abs <= 1e-3 (bf16 inputs) / 1e-4 (fp32).
"""
import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2312_17482_amd import workloads as wl
from tests.helpers import err_stats, run_hip_path, run_oracle, to_dev

pytestmark = pytest.mark.gpu

BF16_TOL = (2e-2, 1e-2)
F32_TOL = (1e-4, 1e-5)


@pytest.fixture(scope="module")
def mb():
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    from paper_2312_17482_amd import binding
    return binding


def check_index_maps(got, mask):
    lengths, cu, idx, T, mx = orc.unpad_index(mask)
    assert got["T"] == T and got["max_seqlen"] == mx
    assert np.array_equal(got["seqlens"], lengths)
    assert np.array_equal(got["cu"], cu)
    assert np.array_equal(got["indices"], idx)


def compare_attention(got, ref, mask, tol, lse_tol, label, abs_floor_ulps=False):
    """abs_floor_ulps: for stress cases whose outputs are much larger than 1, the absolute bound is
    widened to 2^-7 of the largest reference magnitude (a correctly rounded bf16 value of magnitude M
    is already off by up to M * 2^-8: half a unit in the last of its 8 bits); the benchmark workloads never use this."""
    valid = mask != 0
    report = {}
    for key in ("o", "dq", "dk", "dv"):
        assert np.all(got[key][~valid] == 0), "%s: %s not zero at padded rows" % (label, key)
        assert np.all(np.isfinite(got[key])), "%s: %s has non-finite values" % (label, key)
        ma, rf = err_stats(got[key][valid], ref[key][valid])
        report[key] = (ma, rf)
        tol_abs = max(tol[0], 2.0 ** -7 * float(np.max(np.abs(ref[key][valid])))) if abs_floor_ulps else tol[0]
        assert ma <= tol_abs and rf <= tol[1], "%s: %s max_abs=%.3e rel_fro=%.3e" % (label, key, ma, rf)
    B, L = mask.shape
    idx = np.flatnonzero(mask.reshape(-1))
    lse_ref = np.transpose(ref["lse"], (1, 0, 2)).reshape(ref["lse"].shape[1], B * L)[:, idx]   # [H, T]
    d = float(np.max(np.abs(got["lse"] - lse_ref)))
    assert d <= lse_tol, "%s: lse max_abs=%.3e" % (label, d)
    print(label, {k: "%.2e/%.2e" % v for k, v in report.items()}, "lse %.2e" % d, flush=True)


# ------------------------------------------------------------------ index maps and row copies
@pytest.mark.parametrize("seed,B,L,p", [(0, 4, 32, 0.5), (1, 7, 300, 0.9), (2, 1, 1, 1.0), (3, 5, 16, 0.0),
                                        (4, 3, 1000, 1.0), (5, 300, 17, 0.3), (6, 2, 5000, 0.01), (7, 256, 128, 0.8),
                                        (8, 600, 128, 0.7), (9, 3, 40000, 0.5), (10, 512, 128, 1.0), (11, 1, 65536, 0.9),
                                        (12, 65536, 1, 0.5), (13, 1000, 65, 0.2), (14, 1, 63, 1.0)])
def test_unpad_index_arbitrary_masks_bit_exact(mb, seed, B, L, p):
    print("unpad_index seed=%d B=%d L=%d p=%.2f" % (seed, B, L, p), flush=True)
    mask = wl.random_mask(seed, B, L, p)
    mask[mask != 0] = np.random.default_rng(seed).integers(-3, 9, size=int(mask.sum())) * 2 + 1   # any nonzero keeps
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(mask).cuda())
    T, mx = mb.mb_read_meta(meta)
    got = {"T": T, "max_seqlen": mx, "seqlens": seqlens.cpu().numpy(), "cu": cu.cpu().numpy(),
           "indices": indices[:T].cpu().numpy()}
    check_index_maps(got, mask)


def test_unpad_index_leaves_tail_untouched_and_handles_empty_batch(mb):
    mask = wl.suffix_mask(np.array([3, 0, 5]), 8)
    B, L = mask.shape
    indices = torch.full((B * L,), -7, dtype=torch.int32, device="cuda")
    seqlens = torch.empty(B, dtype=torch.int32, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    meta = torch.empty(2, dtype=torch.int32, device="cuda")
    lib = mb.raw()
    assert lib.mb_unpad_index(torch.from_numpy(mask).cuda().data_ptr(), B, L, seqlens.data_ptr(), cu.data_ptr(),
                              indices.data_ptr(), meta.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert indices[:8].tolist() == [0, 1, 2, 16, 17, 18, 19, 20] and torch.all(indices[8:] == -7)
    assert cu.tolist() == [0, 3, 3, 8] and meta.tolist() == [8, 5]
    assert lib.mb_unpad_index(None, 0, 8, None, cu.data_ptr(), None, meta.data_ptr(), None) == 0
    torch.cuda.synchronize()
    assert cu[0].item() == 0 and meta.tolist() == [0, 0]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("seed,B,L,W,p", [(0, 4, 32, 32, 0.6), (1, 9, 77, 768, 0.8), (2, 3, 50, 2304, 0.5),
                                          (3, 2, 40, 8, 1.0), (4, 2, 40, 8, 0.0), (5, 64, 128, 1024, 0.8)])
def test_unpad_pad_rows_bit_exact(mb, dtype, seed, B, L, W, p):
    print("unpad/pad seed=%d B=%d L=%d W=%d p=%.1f %s" % (seed, B, L, W, p, dtype), flush=True)
    mask = wl.random_mask(seed + 100, B, L, p)
    _, _, idx, T, _ = orc.unpad_index(mask)
    rng = np.random.default_rng(seed)
    X = wl.round_to_bf16(rng.standard_normal((B, L, W), dtype=np.float32))
    X[0, 0, 0] = np.nan if mask[0, 0] == 0 else X[0, 0, 0]        # garbage in a padded row must not leak
    Xd = torch.from_numpy(X).to(dtype).cuda().view(B * L, W)
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(mask).cuda())
    sentinel = 12288.0
    packed = torch.full((B * L + 3, W), sentinel, dtype=dtype, device="cuda")
    mb.mb_unpad(Xd, indices, B * L, meta, out=packed)
    ref = orc.unpad(X, idx)
    got = packed.float().cpu().numpy()
    assert np.array_equal(got[:T], ref.astype(np.float32)), "gather mismatch"
    assert np.all(got[T:] == sentinel), "rows beyond T were touched"
    padded = torch.full((B * L, W), sentinel, dtype=dtype, device="cuda")
    mb.mb_pad(packed, indices, B * L, meta, B, L, out=padded)
    ref_pad = orc.pad(ref, idx, B, L).astype(np.float32)
    gotp = padded.float().cpu().numpy().reshape(B, L, W)
    assert np.array_equal(gotp, ref_pad)
    # padded positions are all-zero BITS (not -0.0)
    raw = padded.view(torch.int16 if dtype == torch.bfloat16 else torch.int32).cpu().numpy().reshape(B, L, W)
    assert np.all(raw[mask == 0] == 0)
    # without meta (host-known T): same result
    if T > 0:
        packed2 = torch.full((T, W), sentinel, dtype=dtype, device="cuda")
        mb.mb_unpad(Xd, indices, T, None, out=packed2)
        assert torch.equal(packed2, packed[:T])


# ------------------------------------------------------------------ slopes
@pytest.mark.parametrize("H", [1, 2, 8, 12, 16, 24])
def test_slopes_equal_the_oracles_rounded_to_float(mb, H):
    """"Attention with Linear Biases" paragraph: geometric slopes with ratio 2^(-8/H).  The product's values
    are the oracle's doubles rounded to float, for power-of-two and other head counts alike; every parity
    test below hands the oracle ITS OWN slopes and the kernels the product's."""
    assert np.array_equal(mb.mb_alibi_slopes(H).numpy(), orc.alibi_slopes(H).astype(np.float32))


# ------------------------------------------------------------------ attention, fp32 generic path
def test_tiny_fp32_full_path(mb):
    b = wl.make_batch("tiny")
    slopes = mb.mb_alibi_slopes(2)
    assert np.array_equal(slopes.numpy(), orc.alibi_slopes(2).astype(np.float32))
    got = run_hip_path(mb, b, slopes, bf16=False)
    check_index_maps(got, b["mask"])
    ref = run_oracle(b, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, b["mask"], F32_TOL, 1e-4, "tiny fp32")


@pytest.mark.parametrize("D,H,lengths,L", [(16, 2, [1, 2, 65, 64, 0, 130], 130), (128, 1, [33, 7], 40), (4, 3, [200], 200)])
def test_generic_fp32_shapes(mb, D, H, lengths, L):
    c = wl.random_attention_case(21, lengths, L, H, D)
    slopes = mb.mb_alibi_slopes(H)
    got = run_hip_path(mb, c, slopes, bf16=False)
    check_index_maps(got, c["mask"])
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, c["mask"], F32_TOL, 1e-4, "generic fp32 D=%d" % D)


def test_fp32_scale_one_matches_eq1_literally(mb):
    """Eq. 1 as printed has no 1/sqrt(d): scale = 1."""
    c = wl.random_attention_case(22, [9, 31], 31, 2, 16, std=0.5)
    slopes = mb.mb_alibi_slopes(2)
    got = run_hip_path(mb, c, slopes, bf16=False, scale=1.0)
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)), scale=1.0)
    compare_attention(got, ref, c["mask"], F32_TOL, 1e-4, "fp32 scale=1")


# ------------------------------------------------------------------ attention, bf16 matrix-core path
@pytest.mark.parametrize("name,lengths,L,H,std,v_std", [
    ("ragged-small", [5, 17, 32, 9, 1, 0, 33, 64, 31, 128, 127, 97], 128, 3, 1.0, 1.0),
    ("sharp", [128, 100, 60, 16], 128, 4, 1.0, 1.0),
    ("soft", [128, 77, 128, 19], 128, 12, 0.125, 0.125),
    # logits of a few hundred: exercises the max subtraction; V kept O(1) because the absolute
    # tolerance is stated for O(1) outputs (bf16 rounding alone is 2^-9 relative)
    ("large-logits", [128, 45, 90], 128, 2, 4.0, 0.5),
    ("multi-tile", [129, 300, 257, 64, 511, 1], 512, 2, 0.5, 0.5),
])
def test_bf16_attention_cases(mb, name, lengths, L, H, std, v_std):
    print("bf16 case", name, flush=True)
    c = wl.random_attention_case(31, lengths, L, H, 64, std=std, bf16=True, v_std=v_std)
    slopes = mb.mb_alibi_slopes(H)
    got = run_hip_path(mb, c, slopes, bf16=True)
    check_index_maps(got, c["mask"])
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 " + name, abs_floor_ulps=(name == "large-logits"))


def test_bf16_zero_slopes_and_scale_one(mb):
    c = wl.random_attention_case(32, [128, 50, 3], 128, 2, 64, std=0.3, bf16=True)
    slopes = torch.zeros(2)
    got = run_hip_path(mb, c, slopes, bf16=True, scale=1.0)
    ref = run_oracle(c, np.zeros(2), scale=1.0)
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 zero slopes")


@pytest.mark.parametrize("name", ["bert_base", "bert_large"])
def test_bf16_full_size_workloads(mb, name):
    """The benchmark's workloads at full size, every sequence and head checked."""
    print("full-size", name, flush=True)
    b = wl.make_batch(name)
    H = b["workload"].H
    slopes = mb.mb_alibi_slopes(H)
    got = run_hip_path(mb, b, slopes, bf16=True)
    check_index_maps(got, b["mask"])
    ref = run_oracle(b, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, b["mask"], BF16_TOL, 1e-3, name)


@pytest.mark.parametrize("name,nseq", [("long512", 12), ("ragged2048", 6)])
def test_bf16_long_workloads_sampled(mb, name, nseq):
    """Long workloads at full size on the GPU; the oracle checks a sample of sequences (each cropped
    to its own length, which does not change its result), always including the longest and shortest."""
    print("full-size sampled", name, flush=True)
    b = wl.make_batch(name)
    H, L = b["workload"].H, b["workload"].L
    slopes = mb.mb_alibi_slopes(H)
    got = run_hip_path(mb, b, slopes, bf16=True)
    check_index_maps(got, b["mask"])
    order = np.argsort(b["lengths"])
    pick = sorted(set([int(order[0]), int(order[-1])] + [int(x) for x in np.random.default_rng(5).choice(len(order), nseq, replace=False)]))
    ref = run_oracle(b, orc.alibi_slopes(H), seq_ids=pick)
    for key in ("o", "dq", "dk", "dv"):
        assert np.all(got[key][b["mask"] == 0] == 0) and np.all(np.isfinite(got[key]))
    for s in pick:
        n = int(b["lengths"][s])
        for key in ("o", "dq", "dk", "dv"):
            ma, rf = err_stats(got[key][s, :n], ref[s][key])
            assert ma <= BF16_TOL[0] and rf <= BF16_TOL[1], "%s seq %d (len %d) %s: %.3e %.3e" % (name, s, n, key, ma, rf)
        lse_got = got["lse"][:, got["cu"][s]:got["cu"][s + 1]]
        assert np.max(np.abs(lse_got - ref[s]["lse"])) <= 1e-3
    print(name, "sampled sequences", pick, "ok", flush=True)


def test_bf16_run_to_run_bitwise_identical(mb):
    b = wl.make_batch("bert_base", batch=32)
    slopes = mb.mb_alibi_slopes(12)
    a = run_hip_path(mb, b, slopes, bf16=True)
    c = run_hip_path(mb, b, slopes, bf16=True)
    assert torch.equal(a["o_packed"], c["o_packed"]) and torch.equal(a["lse_dev"], c["lse_dev"])
    assert torch.equal(a["dqkv_packed"], c["dqkv_packed"])


def test_bf16_outputs_do_not_write_outside_their_rows(mb):
    """Guard rows after T and the gap columns of a strided output stay untouched."""
    c = wl.random_attention_case(33, [100, 28], 128, 2, 64, std=0.5, bf16=True)
    B, L, H, D = c["q"].shape
    mask_d = torch.from_numpy(c["mask"]).cuda()
    seqlens, cu, indices, meta = mb.mb_unpad_index(mask_d)
    T, mx = mb.mb_read_meta(meta)
    qkv = to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(B * L, 3 * H * D), True)
    qkv = mb.mb_unpad(qkv, indices, B * L, meta)[:T].view(T, 3, H, D)
    dout = mb.mb_unpad(to_dev(c["do"].reshape(B * L, H * D), True), indices, B * L, meta)[:T].view(T, H, D)
    slopes = mb.mb_alibi_slopes(H).cuda()
    guard = 777.0
    obuf = torch.full((T + 4, 2, H, D), guard, dtype=torch.bfloat16, device="cuda")      # stride 2*H*D, slot 0 used
    lse = torch.full((H, T), guard, dtype=torch.float32, device="cuda")
    o, _ = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, mx, slopes, c["scale"], out=obuf[:T, 0], lse=lse)
    gbuf = torch.full((T + 4, 4, H, D), guard, dtype=torch.bfloat16, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, mx, slopes, c["scale"],
                         dq=gbuf[:T, 0], dk=gbuf[:T, 1], dv=gbuf[:T, 2])
    torch.cuda.synchronize()
    assert torch.all(obuf[T:] == guard) and torch.all(obuf[:T, 1] == guard) and not torch.any(obuf[:T, 0] == guard)
    assert torch.all(gbuf[T:] == guard) and torch.all(gbuf[:T, 3] == guard)
    assert not torch.any(lse == guard)
    # strided result equals the dense one
    o2, lse2 = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, mx, slopes, c["scale"])
    assert torch.equal(o2, obuf[:T, 0]) and torch.equal(lse2, lse)


@pytest.mark.parametrize("bf16,D,L", [(True, 64, 128), (True, 64, 300), (False, 16, 64)])
def test_capacity_mode_needs_no_host_round_trip(mb, bf16, D, L):
    """T passed as the capacity B*L and max_seqlen as L (nothing read back from the device) gives the
    same bits as passing the exact token count, and rows past the last real token stay untouched."""
    lengths = [L, 17, 0, L // 2, 33]
    c = wl.random_attention_case(41, lengths, L, 2, D, std=0.5, bf16=bf16)
    B, _, H, _ = c["q"].shape
    cap = B * L
    tdt = torch.bfloat16 if bf16 else torch.float32
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(c["mask"]).cuda())
    qkv = mb.mb_unpad(to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(cap, 3 * H * D), bf16), indices, cap, meta).view(cap, 3, H, D)
    dout = mb.mb_unpad(to_dev(c["do"].reshape(cap, H * D), bf16), indices, cap, meta).view(cap, H, D)
    slopes = mb.mb_alibi_slopes(H).cuda()
    guard = 3.0
    o_cap = torch.full((cap, H, D), guard, dtype=tdt, device="cuda")
    lse_cap = torch.full((H, cap), guard, dtype=torch.float32, device="cuda")
    mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, L, slopes, c["scale"], out=o_cap, lse=lse_cap)
    g_cap = torch.full((cap, 3, H, D), guard, dtype=tdt, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o_cap, lse_cap, cu, L, slopes, c["scale"],
                         dq=g_cap[:, 0], dk=g_cap[:, 1], dv=g_cap[:, 2])
    T, mx = mb.mb_read_meta(meta)
    assert T == sum(lengths)
    o_ex, lse_ex = mb.mb_alibi_attn_fwd(qkv[:T, 0], qkv[:T, 1], qkv[:T, 2], cu, mx, slopes, c["scale"])
    g_ex = torch.empty((T, 3, H, D), dtype=tdt, device="cuda")
    mb.mb_alibi_attn_bwd(dout[:T], qkv[:T, 0], qkv[:T, 1], qkv[:T, 2], o_ex, lse_ex, cu, mx, slopes, c["scale"],
                         dq=g_ex[:, 0], dk=g_ex[:, 1], dv=g_ex[:, 2])
    torch.cuda.synchronize()
    assert torch.equal(o_cap[:T], o_ex) and torch.equal(lse_cap[:, :T], lse_ex) and torch.equal(g_cap[:T], g_ex)
    assert torch.all(o_cap[T:] == guard) and torch.all(lse_cap[:, T:] == guard) and torch.all(g_cap[T:] == guard)


@pytest.mark.parametrize("bf16,D,L,holes", [(True, 64, 128, False), (True, 64, 128, True), (True, 64, 300, False),
                                             (True, 64, 300, True), (True, 64, 700, False), (True, 64, 700, True),
                                             (False, 16, 64, False), (True, 32, 40, False)])
def test_token_rows_mode_equals_explicit_unpad_and_pad(mb, bf16, D, L, holes):
    """Attention reading and writing the padded batch directly (token_rows = indices) + mb_zero_padding
    gives bit-for-bit what mb_unpad -> attention -> mb_pad gives."""
    print("token_rows bf16=%s D=%d L=%d holes=%s" % (bf16, D, L, holes), flush=True)
    lengths = [L, 17, 0, L // 2, 33, 1]
    c = wl.random_attention_case(51, lengths, L, 2, D, std=0.5, bf16=bf16)
    if holes:   # any 0/1 mask: the kept tokens of a row form its sequence
        c["mask"] = wl.random_mask(52, len(lengths), L, 0.7)
    B, _, H, _ = c["q"].shape
    cap = B * L
    tdt = torch.bfloat16 if bf16 else torch.float32
    slopes_h = mb.mb_alibi_slopes(H)
    ref = run_hip_path(mb, c, slopes_h, bf16=bf16)            # explicit unpad -> attention -> pad
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(c["mask"]).cuda())
    qkv_p = to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(cap, 3 * H * D), bf16).view(cap, 3, H, D)
    do_p = to_dev(c["do"].reshape(cap, H * D), bf16).view(cap, H, D)
    slopes = slopes_h.cuda()
    garbage = 5.0
    o_p = torch.full((cap, H, D), garbage, dtype=tdt, device="cuda")
    lse = torch.full((H, cap), garbage, dtype=torch.float32, device="cuda")
    mb.mb_alibi_attn_fwd(qkv_p[:, 0], qkv_p[:, 1], qkv_p[:, 2], cu, L, slopes, c["scale"], out=o_p, lse=lse,
                         token_rows=indices, T=cap)
    mb.mb_zero_padding(o_p.view(cap, H * D), indices, cap, meta, B, L)
    g_p = torch.full((cap, 3, H, D), garbage, dtype=tdt, device="cuda")
    mb.mb_alibi_attn_bwd(do_p, qkv_p[:, 0], qkv_p[:, 1], qkv_p[:, 2], o_p, lse, cu, L, slopes, c["scale"],
                         dq=g_p[:, 0], dk=g_p[:, 1], dv=g_p[:, 2], token_rows=indices, T=cap)
    mb.mb_zero_padding(g_p.view(cap, 3 * H * D), indices, cap, meta, B, L)
    torch.cuda.synchronize()
    T = ref["T"]
    assert np.array_equal(o_p.double().cpu().numpy().reshape(B, L, H, D), ref["o"])
    got = g_p.double().cpu().numpy().reshape(B, L, 3, H, D)
    assert np.array_equal(got[:, :, 0], ref["dq"]) and np.array_equal(got[:, :, 1], ref["dk"])
    assert np.array_equal(got[:, :, 2], ref["dv"])
    assert np.array_equal(lse[:, :T].double().cpu().numpy(), ref["lse"]) and torch.all(lse[:, T:] == garbage)
    # ... and the padded-layout results agree with the oracle.  The kept tokens of a batch row form its
    # sequence and positions are those inside that sequence, so for a mask with holes the oracle is given the
    # kept tokens moved to the front of their row (a plain numpy gather), which is a suffix-padded batch.
    mask = c["mask"]
    lens = mask.astype(bool).sum(1)
    cc = {key: np.zeros_like(c[key]) for key in ("q", "k", "v", "do")}
    for b in range(B):
        keep = np.flatnonzero(mask[b])
        for key in cc:
            cc[key][b, :len(keep)] = c[key][b, keep]
    cc.update(mask=wl.suffix_mask(lens, L), scale=c["scale"], lengths=lens)
    oref = run_oracle(cc, orc.alibi_slopes(H))
    tol = BF16_TOL if bf16 else F32_TOL
    fused = {"o": o_p.double().cpu().numpy().reshape(B, L, H, D), "dq": got[:, :, 0], "dk": got[:, :, 1],
             "dv": got[:, :, 2]}
    for key, arr in fused.items():
        for b in range(B):
            keep = np.flatnonzero(mask[b])
            if len(keep) == 0:
                continue
            ma, rf = err_stats(arr[b, keep], oref[key][b, :len(keep)])
            # (a one-token sequence has dQ = dK = 0 up to fp64 round-off: no relative error to speak of)
            assert ma <= tol[0] and (rf <= tol[1] or ma <= 1e-7), \
                "token_rows vs oracle %s row %d: %.3e %.3e" % (key, b, ma, rf)
        assert np.all(arr[mask == 0] == 0)


@pytest.mark.parametrize("scale", [-0.2, 0.0])
def test_bf16_nonpositive_scale_takes_the_generic_kernels(mb, scale):
    """The matrix-core kernels need scale > 0; any other finite scale must still be computed correctly."""
    c = wl.random_attention_case(61, [70, 128, 5], 128, 2, 64, std=0.5, bf16=True)
    slopes = mb.mb_alibi_slopes(2)
    got = run_hip_path(mb, c, slopes, bf16=True, scale=scale)
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)), scale=scale)
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 scale=%g" % scale)


def test_all_sequences_empty_and_single_token_batches(mb):
    """Capacity mode with no real token at all: nothing is written, nothing faults; then B = 1, n = 1."""
    B, L, H, D = 3, 64, 2, 64
    cap = B * L
    mask = torch.zeros((B, L), dtype=torch.int32, device="cuda")
    seqlens, cu, indices, meta = mb.mb_unpad_index(mask)
    assert mb.mb_read_meta(meta) == (0, 0) and cu.tolist() == [0, 0, 0, 0]
    x = torch.full((cap, 3, H, D), 2.0, dtype=torch.bfloat16, device="cuda")
    o = torch.full((cap, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((H, cap), 7.0, dtype=torch.float32, device="cuda")
    slopes = mb.mb_alibi_slopes(H).cuda()
    for msl in (L, 1000):        # single-tile kernels, then the any-length kernels
        mb.mb_alibi_attn_fwd(x[:, 0], x[:, 1], x[:, 2], cu, msl, slopes, 0.125, out=o, lse=lse)
        g = torch.full((cap, 3, H, D), 7.0, dtype=torch.bfloat16, device="cuda")
        mb.mb_alibi_attn_bwd(o, x[:, 0], x[:, 1], x[:, 2], o, lse, cu, msl, slopes, 0.125, dq=g[:, 0], dk=g[:, 1], dv=g[:, 2])
        torch.cuda.synchronize()
        assert torch.all(o == 7.0) and torch.all(lse == 7.0) and torch.all(g == 7.0)
    padded = mb.mb_pad(o.view(cap, H * D), indices, cap, meta, B, L)
    assert torch.all(padded == 0)
    c = wl.random_attention_case(62, [1], 1, 1, 64, bf16=True)
    got = run_hip_path(mb, c, mb.mb_alibi_slopes(1), bf16=True)
    ref = run_oracle(c, orc.alibi_slopes(1))
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "single token")
    assert np.array_equal(got["o"][0, 0], c["v"][0, 0].astype(np.float64))      # O = V for a length-1 sequence


@pytest.mark.parametrize("bf16,D,lengths,promised", [(True, 64, [100, 140, 64], 128),     # single-tile kernels
                                                     (True, 64, [100, 300, 600], 384),   # any-length kernels
                                                     (False, 16, [20, 50, 7], 32)])       # generic kernels
def test_sequence_longer_than_max_seqlen_is_skipped_and_reported(mb, bf16, D, lengths, promised):
    """An understated max_seqlen must not truncate silently: the sequences that fit are computed as usual, a
    longer one is skipped (its rows of o and of the gradients untouched, its rows of lse NaN) and
    mb_device_status reports MB_ERR_INVALID_ARG once, then MB_OK again."""
    H = 2
    L = max(lengths)
    c = wl.random_attention_case(91, lengths, L, H, D, std=0.5, bf16=bf16)
    B = len(lengths)
    tdt = torch.bfloat16 if bf16 else torch.float32
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(c["mask"]).cuda())
    T, mx = mb.mb_read_meta(meta)
    qkv = mb.mb_unpad(to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(B * L, 3 * H * D), bf16), indices,
                      B * L, meta)[:T].view(T, 3, H, D)
    dout = mb.mb_unpad(to_dev(c["do"].reshape(B * L, H * D), bf16), indices, B * L, meta)[:T].view(T, H, D)
    slopes = mb.mb_alibi_slopes(H).cuda()
    mb.mb_device_status()                                     # clean before
    o_ok, lse_ok = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, mx, slopes, c["scale"])
    g_ok = torch.empty((T, 3, H, D), dtype=tdt, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o_ok, lse_ok, cu, mx, slopes, c["scale"],
                         dq=g_ok[:, 0], dk=g_ok[:, 1], dv=g_ok[:, 2])
    mb.mb_device_status()                                     # a correct bound raises nothing
    guard = 9.0
    o = torch.full((T, H, D), guard, dtype=tdt, device="cuda")
    lse = torch.full((H, T), guard, dtype=torch.float32, device="cuda")
    mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, promised, slopes, c["scale"], out=o, lse=lse)
    with pytest.raises(mb.MosaicAttnError) as e:
        mb.mb_device_status()
    assert e.value.status == mb.MB_ERR_INVALID_ARG and "max_seqlen" in str(e.value)
    mb.mb_device_status()                                     # reading it cleared it
    g = torch.full((T, 3, H, D), guard, dtype=tdt, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o_ok, lse_ok, cu, promised, slopes, c["scale"],
                         dq=g[:, 0], dk=g[:, 1], dv=g[:, 2])
    with pytest.raises(mb.MosaicAttnError):
        mb.mb_device_status()
    cu_h = cu.tolist()
    for b, n in enumerate(lengths):
        sl = slice(cu_h[b], cu_h[b + 1])
        if n <= promised:     # computed as with the right bound (possibly by the other kernel family: tolerance)
            assert torch.allclose(o[sl].float(), o_ok[sl].float(), atol=2e-2, rtol=0)
            assert torch.allclose(lse[:, sl], lse_ok[:, sl], atol=1e-3, rtol=0)
            assert torch.allclose(g[sl].float(), g_ok[sl].float(), atol=2e-2, rtol=0)
        else:                 # skipped, visibly
            assert torch.all(o[sl] == guard) and torch.all(torch.isnan(lse[:, sl])) and torch.all(g[sl] == guard)


@pytest.mark.parametrize("L,lengths", [(128, [128, 17, 64, 33, 1, 0, 96, 127]), (300, [300, 17, 150, 33, 1, 0, 129, 256]),
                                       (64, [5, 64, 32, 31])])
def test_padded_batch_with_key_mask_equals_the_oracle_on_real_tokens(mb, L, lengths):
    """Attention over the PADDED batch with a key-padding mask (what the paper's own code ran: appendix on sequence
    length): every sequence has L tokens (cu_seqlens = 0, L, 2L, ...), key_lens = the real lengths.  No unpadding
    anywhere.  On the real tokens O, lse, dQ, dK, dV equal the oracle's padded-with-mask result; padding tokens get
    zero dK and dV; padding content (large values) does not leak.  The upstream gradient is zero at padding rows,
    as in a training step whose loss ignores them."""
    H, D = 2, 64
    c = wl.random_attention_case(95, lengths, L, H, D, std=0.5, bf16=True)
    B = len(lengths)
    pad = c["mask"] == 0
    for key in ("q", "k", "v"):
        c[key][pad] = 60.0                       # garbage at padding positions must not leak
    c["do"][pad] = 0.0
    x = to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(B * L, 3, H, D), True)
    do = to_dev(c["do"].reshape(B * L, H, D), True)
    cu = torch.arange(0, B * L + 1, L, dtype=torch.int32, device="cuda")
    klens = torch.tensor(lengths, dtype=torch.int32, device="cuda")
    slopes = mb.mb_alibi_slopes(H).cuda()
    guard = 5.0
    o = torch.full((B * L, H, D), guard, dtype=torch.bfloat16, device="cuda")
    lse = torch.full((H, B * L), guard, dtype=torch.float32, device="cuda")
    mb.mb_alibi_attn_fwd(x[:, 0], x[:, 1], x[:, 2], cu, L, slopes, c["scale"], out=o, lse=lse, key_lens=klens)
    g = torch.full((B * L, 3, H, D), guard, dtype=torch.bfloat16, device="cuda")
    mb.mb_alibi_attn_bwd(do, x[:, 0], x[:, 1], x[:, 2], o, lse, cu, L, slopes, c["scale"], dq=g[:, 0], dk=g[:, 1],
                         dv=g[:, 2], key_lens=klens)
    mb.mb_device_status()
    ref = run_oracle(c, orc.alibi_slopes(H))
    real = c["mask"] != 0
    got = {"o": o.double().cpu().numpy().reshape(B, L, H, D)}
    gg = g.double().cpu().numpy().reshape(B, L, 3, H, D)
    got.update(dq=gg[:, :, 0], dk=gg[:, :, 1], dv=gg[:, :, 2])
    for key in ("o", "dq", "dk", "dv"):
        assert np.all(np.isfinite(got[key])), key
        ma, rf = err_stats(got[key][real], ref[key][real])
        assert ma <= BF16_TOL[0] and rf <= BF16_TOL[1], "padded+mask %s: %.3e %.3e" % (key, ma, rf)
    lse_got = lse.double().cpu().numpy().reshape(H, B, L).transpose(1, 0, 2)        # [B, H, L]
    realh = np.broadcast_to(real[:, None, :], lse_got.shape)
    assert np.max(np.abs(lse_got[realh] - ref["lse"][realh])) <= 1e-3
    for b, n in enumerate(lengths):
        if n == 0:       # a sequence without keys is skipped: nothing written
            assert np.all(got["o"][b] == guard) and np.all(gg[b] == guard)
        else:            # padding tokens are no keys: zero dK, dV; zero upstream gradient: zero dQ
            assert np.all(got["dk"][b, n:] == 0) and np.all(got["dv"][b, n:] == 0) and np.all(got["dq"][b, n:] == 0)


@pytest.mark.parametrize("limit_keys", [False, True])
def test_plan_built_once_gives_the_same_bits_as_plans_built_per_call(mb, limit_keys):
    """mb_attn_plan once per batch, then forward and backward with `plan`: bit for bit what the calls give when
    each builds its own plan (any-length kernels; with and without key_lens), with no forward workspace and a
    backward workspace that only holds Delta."""
    lengths = [700, 129, 300, 64, 1, 0, 512, 257, 640]
    L, H, D = 700, 3, 64
    c = wl.random_attention_case(97, lengths, L, H, D, std=0.5, bf16=True)
    B = len(lengths)
    seqlens, cu, indices, meta = mb.mb_unpad_index(torch.from_numpy(c["mask"]).cuda())
    T, mx = mb.mb_read_meta(meta)
    qkv = mb.mb_unpad(to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(B * L, 3 * H * D), True), indices,
                      B * L, meta)[:T].view(T, 3, H, D)
    dout = mb.mb_unpad(to_dev(c["do"].reshape(B * L, H * D), True), indices, B * L, meta)[:T].view(T, H, D)
    slopes = mb.mb_alibi_slopes(H).cuda()
    klens = torch.tensor([max(1, n // 2) for n in lengths], dtype=torch.int32, device="cuda") if limit_keys else None
    o1, lse1 = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, mx, slopes, c["scale"], key_lens=klens)
    g1 = torch.zeros((T, 3, H, D), dtype=torch.bfloat16, device="cuda")
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o1, lse1, cu, mx, slopes, c["scale"], dq=g1[:, 0],
                         dk=g1[:, 1], dv=g1[:, 2], key_lens=klens)
    plan = mb.mb_attn_plan(cu, mx, H, key_lens=klens)
    lib = mb.raw()
    o2 = torch.zeros_like(o1)
    lse2 = torch.zeros_like(lse1)
    st = lib.mb_alibi_attn_fwd(qkv[:, 0].data_ptr(), qkv[:, 1].data_ptr(), qkv[:, 2].data_ptr(), 3 * H * D, 3 * H * D,
                               3 * H * D, cu.data_ptr(), B, T, mx, H, D, slopes.data_ptr(), float(c["scale"]), mb.MB_BF16,
                               o2.data_ptr(), H * D, lse2.data_ptr(), None, 0, None if klens is None else klens.data_ptr(),
                               None, plan.data_ptr(), torch.cuda.current_stream().cuda_stream)
    assert st == mb.MB_OK, mb.mb_last_error()       # no workspace at all
    g2 = torch.zeros_like(g1)
    ws = torch.empty(H * T * 4 + 256, dtype=torch.uint8, device="cuda")               # Delta only
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o2, lse2, cu, mx, slopes, c["scale"], dq=g2[:, 0],
                         dk=g2[:, 1], dv=g2[:, 2], key_lens=klens, plan=plan, workspace=ws)
    mb.mb_device_status()
    assert torch.equal(o1, o2) and torch.equal(lse1, lse2) and torch.equal(g1, g2)


@pytest.mark.parametrize("lengths,L,H,limit_keys", [([300, 0, 129, 128, 513, 64, 1], 513, 3, False),
                                                     ([700, 20, 256, 255, 257], 700, 12, True),
                                                     (list(range(1, 41)) * 15, 200, 2, False)])
def test_work_plan_lists_every_tile_exactly_once(mb, lengths, L, H, limit_keys):
    """The work plan of the any-length kernels is scheduling, not arithmetic, so what can be checked is that it is
    VALID: read back, its 8 lists (8 int32 counts, then 8 x cap items of 4 int32: first packed token, length,
    tile | head << 16, keys) together name every (sequence, head, tile of 128 tokens) that has work exactly once,
    with the sequence's own start, length and key count; sequences without tokens or without keys are absent;
    and, for up to 512 sequences (more are taken in the order given), pair p = rank * H + head, ranks longest first,
    sits in list p % 16 or 15 - p % 16 and inside a list lengths never increase."""
    B = len(lengths)
    print("plan B=%d L=%d H=%d limit_keys=%s" % (B, L, H, limit_keys), flush=True)
    lens = np.asarray(lengths, dtype=np.int64)
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lens)]), dtype=torch.int32, device="cuda")
    klens_np = np.maximum(lens - np.arange(B) % 3 * 40, 0) if limit_keys else lens
    klens = torch.tensor(klens_np, dtype=torch.int32, device="cuda") if limit_keys else None
    plan = mb.mb_attn_plan(cu, L, H, key_lens=klens)
    torch.cuda.synchronize()
    mb.mb_device_status()
    words = plan.view(torch.int32).cpu().numpy()
    cap = 2 * ((B * H + 15) // 16) * ((L + 127) // 128)   # items a list can hold: the pairs it can get x the most tiles
    assert 32 + 8 * cap * 16 <= mb.mb_attn_plan_bytes(B, L, H)
    counts = words[:8]
    assert np.all(counts >= 0) and np.all(counts <= cap)
    starts = np.concatenate([[0], np.cumsum(lens)])[:B]
    expected = {}
    for b in range(B):
        if lens[b] > 0 and klens_np[b] > 0:
            for h in range(H):
                for t in range((lens[b] + 127) // 128):
                    expected[(int(starts[b]), h, t)] = (int(lens[b]), int(min(klens_np[b], lens[b])))
    order = sorted(range(B), key=lambda b: (-lens[b], b))   # longest first, ties by index
    rank = {b: r for r, b in enumerate(order)}
    seq_of_start = {int(starts[b]): b for b in range(B) if lens[b] > 0}
    seen = set()
    for c in range(8):
        items = words[8 + c * cap * 4: 8 + (c * cap + int(counts[c])) * 4].reshape(-1, 4)
        if B <= 512:
            assert np.all(np.diff(items[:, 1]) <= 0), "list %d is not longest first" % c
        for start, n, th, nk in items.tolist():
            key = (start, th >> 16, th & 0xffff)
            assert key in expected and key not in seen, "list %d: item %s" % (c, key)
            assert expected[key] == (n, nk)
            seen.add(key)
            if B <= 512:
                pair = rank[seq_of_start[start]] * H + (th >> 16)
                assert c in (pair % 16, 15 - pair % 16)
    assert len(seen) == len(expected)


def test_bf16_tile_boundary_lengths(mb):
    """Lengths on both sides of every tile boundary of the any-length kernels (32, 64, 128) in one batch."""
    lengths = [31, 32, 33, 63, 64, 65, 95, 96, 97, 127, 128, 129, 191, 192, 193, 255, 256, 257, 2, 0]
    c = wl.random_attention_case(71, lengths, 257, 2, 64, std=0.7, bf16=True, v_std=0.5)
    slopes = mb.mb_alibi_slopes(2)
    got = run_hip_path(mb, c, slopes, bf16=True)
    check_index_maps(got, c["mask"])
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 tile boundaries")


@pytest.mark.parametrize("B", [300, 530])
def test_bf16_many_sequences_through_the_any_length_kernels(mb, B):
    """More sequences than one pass of the longest-first ranking covers (256 candidates per pass), and more
    than it is applied to at all (512): mostly very short sequences, many of equal length, two long ones."""
    rng = np.random.default_rng(77 + B)
    lengths = [int(x) for x in rng.integers(0, 13, size=B)]
    lengths[B // 3] = 130
    lengths[B - 2] = 129
    c = wl.random_attention_case(300 + B, lengths, 130, 1, 64, std=0.7, bf16=True, v_std=0.5)
    slopes = mb.mb_alibi_slopes(1)
    got = run_hip_path(mb, c, slopes, bf16=True)
    check_index_maps(got, c["mask"])
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 %d sequences" % B)


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_bf16_random_shapes(mb, seed):
    """Random batch sizes, head counts and lengths (both kernel families, chosen by the longest sequence)."""
    rng = np.random.default_rng(1000 + seed)
    B = int(rng.integers(1, 9))
    H = int(rng.integers(1, 5))
    L = int(rng.choice([48, 128, 200, 400]))
    lengths = [int(x) for x in rng.integers(0, L + 1, size=B)]
    lengths[int(rng.integers(B))] = L
    print("random shapes seed=%d B=%d H=%d L=%d lengths=%s" % (seed, B, H, L, lengths), flush=True)
    c = wl.random_attention_case(2000 + seed, lengths, L, H, 64, std=0.6, bf16=True, v_std=0.6)
    slopes = mb.mb_alibi_slopes(H)
    got = run_hip_path(mb, c, slopes, bf16=True)
    check_index_maps(got, c["mask"])
    ref = run_oracle(c, orc.alibi_slopes(len(slopes)))
    compare_attention(got, ref, c["mask"], BF16_TOL, 1e-3, "bf16 random %d" % seed)


@pytest.mark.parametrize("n,B", [(2000, 3000), (100, 60000)])
def test_bf16_buffers_beyond_four_gigabytes(mb, n, B):
    """Packed QKV of 9.2 GB (6 million tokens x 3 x 4 heads x 64): element offsets pass 2^32, so every row
    address must be formed in 64 bits.  Both kernel families (n = 2000: any-length, n = 100: single tile);
    the oracle checks the first, a middle and the last sequence, which sit at the two ends of the buffers."""
    H, D = 4, 64
    T = n * B
    print("large buffers n=%d B=%d T=%d" % (n, B, T), flush=True)
    dev, bf = "cuda", torch.bfloat16
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    qkv = torch.empty((T, 3, H, D), dtype=bf, device=dev)
    dout = torch.empty((T, H, D), dtype=bf, device=dev)
    step = 1 << 20
    for t0 in range(0, T, step):   # filled in pieces: no fp32 copy of the whole buffer
        t1 = min(T, t0 + step)
        qkv[t0:t1] = (torch.randn((t1 - t0, 3, H, D), device=dev, generator=gen) * 0.5).to(bf)
        dout[t0:t1] = torch.randn((t1 - t0, H, D), device=dev, generator=gen).to(bf)
    cu = torch.arange(0, T + 1, n, dtype=torch.int32, device=dev)
    slopes = mb.mb_alibi_slopes(H).to(dev)
    o, lse = mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, n, slopes, 0.125)
    dqkv = torch.empty_like(qkv)
    mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, n, slopes, 0.125,
                         dq=dqkv[:, 0], dk=dqkv[:, 1], dv=dqkv[:, 2])
    torch.cuda.synchronize()
    s64 = orc.alibi_slopes(H)
    ones = np.ones((1, n), dtype=np.int32)
    for b in (0, B // 2, B - 1):
        sl = slice(b * n, (b + 1) * n)
        q, k, v = (qkv[sl, i].float().cpu().numpy()[None] for i in range(3))
        do = dout[sl].float().cpu().numpy()[None]
        O, LSE = orc.attention_fwd(q, k, v, ones, s64, 0.125)
        dQ, dK, dV = orc.attention_bwd(do, q, k, v, ones, s64, 0.125)
        for name, got, ref in (("o", o[sl], O[0]), ("dq", dqkv[sl, 0], dQ[0]), ("dk", dqkv[sl, 1], dK[0]),
                               ("dv", dqkv[sl, 2], dV[0])):
            ma, rf = err_stats(got.float().cpu().numpy().astype(np.float64), ref)
            assert ma <= BF16_TOL[0] and rf <= BF16_TOL[1], "seq %d %s: %.3e %.3e" % (b, name, ma, rf)
        assert np.max(np.abs(lse[:, sl].cpu().numpy() - LSE[0])) <= 1e-3
    del qkv, dqkv, dout, o, lse
    torch.cuda.empty_cache()


@pytest.mark.parametrize("lengths,L", [([70, 128, 1], 128), ([130, 5], 140)])
def test_bf16_rows_sixteen_megabytes_apart(mb, lengths, L):
    """Row strides of 2^23 elements: a sequence's rows no longer lie within 2^31 bytes of its first, so both kernel
    families must form every row address per lane in 64 bits instead of using 32-bit buffer offsets.  The results
    are the bits of the same case in dense tensors, which is checked against the oracle."""
    H, D, stride = 2, 64, 1 << 23
    print("wide rows lengths=%s" % lengths, flush=True)
    c = wl.random_attention_case(321, lengths, L, H, D, std=0.5, bf16=True)
    ref = run_oracle(c, orc.alibi_slopes(H))
    mask = c["mask"] != 0
    T = int(mask.sum())
    dev, bf = "cuda", torch.bfloat16
    cu = torch.tensor(np.concatenate([[0], np.cumsum(lengths)]), dtype=torch.int32, device=dev)
    slopes = mb.mb_alibi_slopes(H).to(dev)
    dense = {k: torch.from_numpy(c[k][mask]).to(bf).to(dev) for k in ("q", "k", "v", "do")}   # [T, H, D]

    def wide(src=None):
        buf = torch.empty(T * stride, dtype=bf, device=dev)
        view = buf.as_strided((T, H, D), (stride, D, 1))
        if src is not None:
            view.copy_(src)
        return view
    res = {}
    for kind in ("dense", "wide"):
        t = dense if kind == "dense" else {k: wide(x) for k, x in dense.items()}
        mk = (lambda: torch.empty((T, H, D), dtype=bf, device=dev)) if kind == "dense" else wide
        o, dq, dk, dv = mk(), mk(), mk(), mk()
        _, lse = mb.mb_alibi_attn_fwd(t["q"], t["k"], t["v"], cu, L, slopes, c["scale"], out=o)
        mb.mb_alibi_attn_bwd(t["do"], t["q"], t["k"], t["v"], o, lse, cu, L, slopes, c["scale"], dq=dq, dk=dk, dv=dv)
        torch.cuda.synchronize()
        mb.mb_device_status()
        res[kind] = {"o": o.contiguous(), "dq": dq.contiguous(), "dk": dk.contiguous(), "dv": dv.contiguous(), "lse": lse}
        del t, o, dq, dk, dv
        torch.cuda.empty_cache()
    for key in ("o", "dq", "dk", "dv", "lse"):
        assert torch.equal(res["dense"][key], res["wide"][key]), key
    for key in ("o", "dq", "dk", "dv"):
        ma, rf = err_stats(res["dense"][key].float().cpu().numpy().astype(np.float64), ref[key][mask])
        assert ma <= BF16_TOL[0] and (rf <= BF16_TOL[1] or ma <= 1e-7), "%s: %.3e %.3e" % (key, ma, rf)


def test_unpad_pad_buffers_beyond_four_gigabytes(mb):
    """Gather and scatter on a padded batch of 13.8 GB (3 million rows of 4608 bytes): bit-exact against
    torch's index_select / index_copy, which also checks the index maps of a 3000 x 1000 mask."""
    B, L, W = 3000, 1000, 2304
    dev = "cuda"
    gen = torch.Generator(device=dev)
    gen.manual_seed(5)
    mask = (torch.rand((B, L), device=dev, generator=gen) < 0.8).to(torch.int32)
    seqlens, cu, indices, meta = mb.mb_unpad_index(mask)
    T = int(mask.sum().item())
    assert torch.equal(indices[:T].long(), torch.nonzero(mask.view(-1)).view(-1))
    assert int(cu[-1].item()) == T and torch.equal(seqlens, mask.sum(1).to(torch.int32))
    padded = torch.empty((B * L, W), dtype=torch.bfloat16, device=dev)
    step = 1 << 18
    for r0 in range(0, B * L, step):
        r1 = min(B * L, r0 + step)
        padded[r0:r1] = torch.randn((r1 - r0, W), device=dev, generator=gen).to(torch.bfloat16)
    packed = mb.mb_unpad(padded, indices, T, None)
    assert torch.equal(packed, padded.index_select(0, indices[:T].long()))
    back = mb.mb_pad(packed, indices, T, None, B, L)
    keep = mask.view(-1) != 0
    assert torch.equal(back[keep], packed) and not bool(back[~keep].view(torch.int16).any())
    del padded, packed, back
    torch.cuda.empty_cache()


@pytest.mark.parametrize("L", [128, 300])
def test_whole_path_replays_from_a_hip_graph(mb, L):
    """The library allocates nothing, never synchronises and enqueues only kernels, so the whole path can be
    captured in a HIP graph: three replays, with eager runs and synchronisation between them, each give the
    bits of the eager run (both kernel families)."""
    lengths = [L, 17, 0, L // 2, 33, 1, L - 1, 64]
    c = wl.random_attention_case(81, lengths, L, 2, 64, std=0.5, bf16=True)
    B, _, H, D = c["q"].shape
    cap = B * L
    bf = torch.bfloat16
    mask = torch.from_numpy(c["mask"]).cuda()
    qkv_p = to_dev(np.stack([c["q"], c["k"], c["v"]], axis=2).reshape(cap, 3 * H * D), True)
    do_p = to_dev(c["do"].reshape(cap, H * D), True)
    slopes = mb.mb_alibi_slopes(H).cuda()
    qkv = torch.empty((cap, 3, H, D), dtype=bf, device="cuda")
    dout = torch.empty((cap, H, D), dtype=bf, device="cuda")
    o = torch.empty((cap, H, D), dtype=bf, device="cuda")
    dqkv = torch.empty((cap, 3, H, D), dtype=bf, device="cuda")
    o_pad = torch.empty((cap, H * D), dtype=bf, device="cuda")
    g_pad = torch.empty((cap, 3 * H * D), dtype=bf, device="cuda")
    lse = torch.empty((H, cap), dtype=torch.float32, device="cuda")
    ws = torch.empty(mb.mb_alibi_attn_bwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16), dtype=torch.uint8, device="cuda")
    ws_f = torch.empty(max(16, mb.mb_alibi_attn_fwd_workspace_bytes(B, cap, L, H, D, mb.MB_BF16)), dtype=torch.uint8,
                       device="cuda")
    seqlens = torch.empty(B, dtype=torch.int32, device="cuda")
    cu = torch.empty(B + 1, dtype=torch.int32, device="cuda")
    indices = torch.empty(cap, dtype=torch.int32, device="cuda")
    meta = torch.empty(2, dtype=torch.int32, device="cuda")
    lib = mb.raw()

    def path():   # capacity mode: no host round trip anywhere
        assert lib.mb_unpad_index(mask.data_ptr(), B, L, seqlens.data_ptr(), cu.data_ptr(), indices.data_ptr(),
                                  meta.data_ptr(), torch.cuda.current_stream().cuda_stream) == 0
        mb.mb_unpad(qkv_p, indices, cap, meta, out=qkv.view(cap, 3 * H * D))
        mb.mb_unpad(do_p, indices, cap, meta, out=dout.view(cap, H * D))
        mb.mb_alibi_attn_fwd(qkv[:, 0], qkv[:, 1], qkv[:, 2], cu, L, slopes, c["scale"], out=o, lse=lse, workspace=ws_f)
        mb.mb_alibi_attn_bwd(dout, qkv[:, 0], qkv[:, 1], qkv[:, 2], o, lse, cu, L, slopes, c["scale"],
                             dq=dqkv[:, 0], dk=dqkv[:, 1], dv=dqkv[:, 2], workspace=ws)
        mb.mb_pad(o.view(cap, H * D), indices, cap, meta, B, L, out=o_pad)
        mb.mb_pad(dqkv.view(cap, 3 * H * D), indices, cap, meta, B, L, out=g_pad)

    path()
    torch.cuda.synchronize()
    ref_o, ref_g = o_pad.clone(), g_pad.clone()
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            path()
    torch.cuda.synchronize()
    for _ in range(3):
        o_pad.fill_(7.0)
        g_pad.fill_(7.0)
        qkv.fill_(1.0)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(o_pad, ref_o) and torch.equal(g_pad, ref_g)
        path()                      # eager work between replays
        torch.cuda.synchronize()
        assert torch.equal(o_pad, ref_o) and torch.equal(g_pad, ref_g)
