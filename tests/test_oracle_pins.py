"""Pins for the CPU oracle: each test checks oracle/ against something other than itself --
closed forms, invariants, finite differences, brute force, hand-worked fixtures, or a library
routine -- so that a dropped term, wrong sign, wrong index or transposed operand fails one."""
import os

import numpy as np
import pytest
import torch

from oracle import mosaic_oracle as orc
from paper_2312_17482_amd import workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _case(seed, lengths, L, H, D, std=1.0):
    c = wl.random_attention_case(seed, lengths, L, H, D, std)
    rng = np.random.default_rng(seed + 7)
    c["slopes"] = rng.uniform(0.01, 0.7, size=H)
    return c


# ---------------------------------------------------------------- P1: softmax rows, LSE
def test_rows_sum_to_one_and_lse_consistent():
    c = _case(1, [5, 17, 32, 9, 1], 32, 3, 8)
    O, LSE, P = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"], return_probs=True)
    pos = np.arange(32)
    for b, n in enumerate(c["lengths"]):
        assert np.allclose(P[b, :, :n, :].sum(-1), 1.0, atol=1e-14)
        assert np.all(P[b, :, :, n:] == 0) and np.all(P[b, :, n:, :] == 0)
        for h in range(3):
            q, k = c["q"][b, :n, h].astype(np.float64), c["k"][b, :n, h].astype(np.float64)
            S = c["scale"] * np.einsum("id,jd->ij", q, k) - c["slopes"][h] * np.abs(pos[:n, None] - pos[None, :n])
            assert np.allclose(np.exp(S - LSE[b, h, :n, None]), P[b, h, :n, :n], atol=1e-13)


# ---------------------------------------------------------------- P2: length-1 sequence
def test_length_one_sequence():
    c = _case(2, [1, 1], 8, 2, 4)
    O, LSE = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    dQ, dK, dV = orc.attention_bwd(c["do"], c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    for b in range(2):
        assert np.allclose(O[b, 0], c["v"][b, 0], atol=1e-15)
        assert np.allclose(LSE[b, :, 0], c["scale"] * np.sum(c["q"][b, 0].astype(np.float64) * c["k"][b, 0], axis=-1))
        assert np.allclose(dV[b, 0], c["do"][b, 0])
        assert np.all(dQ[b] == 0) and np.all(dK[b] == 0)
        assert np.all(O[b, 1:] == 0) and np.all(dV[b, 1:] == 0)


# ---------------------------------------------------------------- P3: zero slopes, identical keys
def test_zero_slope_identical_keys_gives_mean_of_v():
    c = _case(3, [7, 12], 12, 2, 4)
    c["k"][:] = c["k"][:, :1]            # every key equals the first key of its sequence
    O, _ = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], np.zeros(2), c["scale"])
    for b, n in enumerate(c["lengths"]):
        mean_v = c["v"][b, :n].astype(np.float64).mean(axis=0)
        assert np.allclose(O[b, :n], mean_v[None], atol=1e-14)


# ---------------------------------------------------------------- P4: padding is inert
def test_padding_content_and_width_do_not_matter():
    lengths = [5, 17, 32, 9]
    c = _case(4, lengths, 32, 2, 8)
    args = (c["mask"], c["slopes"], c["scale"])
    O, LSE = orc.attention_fwd(c["q"], c["k"], c["v"], *args)
    grads = orc.attention_bwd(c["do"], c["q"], c["k"], c["v"], *args)
    # (a) poison pads with NaN, (b) widen L to 40
    big = {}
    for key in ("q", "k", "v", "do"):
        t = np.full((4, 40, 2, 8), np.nan, dtype=np.float64)
        for b, n in enumerate(lengths):
            t[b, :n] = c[key][b, :n]
        big[key] = t
    mask40 = wl.suffix_mask(np.array(lengths), 40)
    O2, LSE2 = orc.attention_fwd(big["q"], big["k"], big["v"], mask40, c["slopes"], c["scale"])
    grads2 = orc.attention_bwd(big["do"], big["q"], big["k"], big["v"], mask40, c["slopes"], c["scale"])
    for b, n in enumerate(lengths):
        assert np.array_equal(O2[b, :n], O[b, :n]) and np.all(O2[b, n:] == 0)
        assert np.array_equal(LSE2[b, :, :n], LSE[b, :, :n])
        for g2, g in zip(grads2, grads):
            assert np.allclose(g2[b, :n], g[b, :n], atol=1e-14) and np.all(g2[b, n:] == 0)
    # (c) each sequence alone, unpadded, dense: same numbers
    for b, n in enumerate(lengths):
        one = {k_: c[k_][b:b + 1, :n] for k_ in ("q", "k", "v", "do")}
        m1 = np.ones((1, n), dtype=np.int32)
        O1, LSE1 = orc.attention_fwd(one["q"], one["k"], one["v"], m1, c["slopes"], c["scale"])
        g1 = orc.attention_bwd(one["do"], one["q"], one["k"], one["v"], m1, c["slopes"], c["scale"])
        assert np.allclose(O1[0], O[b, :n], atol=1e-14)
        assert np.allclose(LSE1[0], LSE[b, :, :n], atol=1e-14)
        for x1, x in zip(g1, grads):
            assert np.allclose(x1[0], x[b, :n], atol=1e-13)


# ---------------------------------------------------------------- P5: closed form for the ALiBi bias
@pytest.mark.parametrize("n,m", [(1, 0.3), (6, 0.25), (19, 2.0 ** -4), (32, 0.9)])
def test_alibi_closed_form_identical_keys(n, m):
    """All keys equal => scores are c - m|i-j|; with r = exp(-m) and 1-based i,
    Z_i = (1 + r - r^i - r^(n+1-i)) / (1 - r), P_ij = r^|i-j| / Z_i, LSE_i = c + ln Z_i."""
    rng = np.random.default_rng(5)
    D, L = 4, n + 3
    q = rng.standard_normal((1, L, 1, D))
    k = np.broadcast_to(rng.standard_normal((1, 1, 1, D)), (1, L, 1, D)).copy()
    v = rng.standard_normal((1, L, 1, D))
    mask = wl.suffix_mask(np.array([n]), L)
    scale = 0.37
    O, LSE, P = orc.attention_fwd(q, k, v, mask, np.array([m]), scale, return_probs=True)
    r = np.exp(-m)
    i = np.arange(1, n + 1, dtype=np.float64)
    Z = (1 + r - r ** i - r ** (n + 1 - i)) / (1 - r)
    dist = np.abs(i[:, None] - i[None, :])
    P_ref = r ** dist / Z[:, None]
    c = scale * np.einsum("id,d->i", q[0, :n, 0], k[0, 0, 0])
    assert np.allclose(P[0, 0, :n, :n], P_ref, atol=1e-14)
    assert np.allclose(LSE[0, 0, :n], c + np.log(Z), atol=1e-13)
    assert np.allclose(O[0, :n, 0], P_ref @ v[0, :n, 0], atol=1e-14)
    # the bias must favour near tokens: weights decay monotonically away from the diagonal
    if n >= 3:
        assert P[0, 0, 0, 0] > P[0, 0, 0, 1] > P[0, 0, 0, 2]
        assert P[0, 0, n - 1, n - 1] > P[0, 0, n - 1, n - 2] > P[0, 0, n - 1, n - 3]


# ---------------------------------------------------------------- P6: slopes
def test_slopes_match_fixture():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "alibi_slopes.txt")) if l.strip() and not l.startswith("#")]
    assert len(rows) > 20
    for n, h, p, q in rows:
        n, h, p, q = int(n), int(h), int(p), int(q)
        got = orc.alibi_slopes(n)
        assert got.shape == (n,)
        expect = 2.0 ** (-(p / q))
        assert abs(got[h - 1] - expect) <= 1e-15 * expect
        if q == 1:
            assert got[h - 1] == 2.0 ** (-p)             # exact power of two
    s = orc.alibi_slopes(12)
    assert np.allclose(s[1:] / s[:-1], 2.0 ** (-8 / 12), rtol=1e-14)   # the stated ratio
    assert s[0] == s[1] / s[0] or abs(s[0] - s[1] / s[0]) < 1e-15       # first term = ratio


# ---------------------------------------------------------------- P7: symmetry
def test_reversal_symmetry_and_permutation_invariance():
    lengths = [11, 6]
    c = _case(7, lengths, 11, 2, 4)
    O, LSE = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    rev = {}
    for key in ("q", "k", "v"):
        t = c[key].copy()
        for b, n in enumerate(lengths):
            t[b, :n] = c[key][b, :n][::-1]
        rev[key] = t
    Or, LSEr = orc.attention_fwd(rev["q"], rev["k"], rev["v"], c["mask"], c["slopes"], c["scale"])
    for b, n in enumerate(lengths):
        assert np.allclose(Or[b, :n], O[b, :n][::-1], atol=1e-14)
        assert np.allclose(LSEr[b, :, :n], LSE[b, :, :n][:, ::-1], atol=1e-14)
    # zero slopes: jointly permuting keys and values changes nothing
    zero = np.zeros(2)
    O0, _ = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], zero, c["scale"])
    perm = np.random.default_rng(0).permutation(6)
    k2, v2 = c["k"].copy(), c["v"].copy()
    k2[1, :6] = c["k"][1, :6][perm]
    v2[1, :6] = c["v"][1, :6][perm]
    O1, _ = orc.attention_fwd(c["q"], k2, v2, c["mask"], zero, c["scale"])
    assert np.allclose(O1, O0, atol=1e-14)
    # ... but with a nonzero slope it must change (the bias sees positions)
    O2, _ = orc.attention_fwd(c["q"], k2, v2, c["mask"], c["slopes"], c["scale"])
    assert np.abs(O2[1, :6] - O[1, :6]).max() > 1e-3


# ---------------------------------------------------------------- P8: finite differences
def _loss(q, k, v, do, mask, slopes, scale):
    O, _ = orc.attention_fwd(q, k, v, mask, slopes, scale)
    return float(np.sum(O * np.where(mask[:, :, None, None] != 0, do, 0.0)))


@pytest.mark.parametrize("which", ["tiny", "random"])
def test_backward_matches_central_differences(which):
    if which == "tiny":
        b = wl.make_batch("tiny")
        slopes = orc.alibi_slopes(2)
        q, k, v, do = (b[x].astype(np.float64) for x in ("q", "k", "v", "do"))
        mask, scale = b["mask"], b["scale"]
    else:
        c = _case(8, [3, 9, 1, 6], 9, 3, 5)
        slopes = c["slopes"]
        q, k, v, do = (c[x].astype(np.float64) for x in ("q", "k", "v", "do"))
        mask, scale = c["mask"], 0.61
    dQ, dK, dV = orc.attention_bwd(do, q, k, v, mask, slopes, scale)
    rng = np.random.default_rng(11)
    eps = 1e-5
    for name, X, G in (("q", q, dQ), ("k", k, dK), ("v", v, dV)):
        # directional derivatives along random directions + a few single coordinates
        for trial in range(6):
            if trial < 3:
                U = rng.standard_normal(X.shape)
            else:
                U = np.zeros_like(X)
                bb = int(rng.integers(X.shape[0]))
                n = int(np.count_nonzero(mask[bb]))
                U[bb, int(rng.integers(n)), int(rng.integers(X.shape[2])), int(rng.integers(X.shape[3]))] = 1.0
            args = {"q": q, "k": k, "v": v}
            plus, minus = dict(args), dict(args)
            plus[name] = X + eps * U
            minus[name] = X - eps * U
            fd = (_loss(plus["q"], plus["k"], plus["v"], do, mask, slopes, scale)
                  - _loss(minus["q"], minus["k"], minus["v"], do, mask, slopes, scale)) / (2 * eps)
            an = float(np.sum(G * U))
            assert abs(fd - an) <= 1e-7 * max(1.0, abs(an)), (name, trial, fd, an)
    # gradient is exactly zero at padded positions
    for G in (dQ, dK, dV):
        assert np.all(G[mask == 0] == 0)


# ---------------------------------------------------------------- P9: backward identities
def test_backward_identities():
    lengths = [9, 4, 13]
    c = _case(9, lengths, 13, 2, 6)
    dQ, dK, dV = orc.attention_bwd(c["do"], c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    q, k, do = (c[x].astype(np.float64) for x in ("q", "k", "do"))
    for b, n in enumerate(lengths):
        for h in range(2):
            # loss depends on q, k only through q k^T  =>  <q, dq> = <k, dk>
            assert np.isclose(np.sum(q[b, :n, h] * dQ[b, :n, h]), np.sum(k[b, :n, h] * dK[b, :n, h]), atol=1e-12)
            # rows of P sum to one  =>  sum_j dV_j = sum_i dO_i
            assert np.allclose(dV[b, :n, h].sum(0), do[b, :n, h].sum(0), atol=1e-12)
    # adding a constant vector to every key of a sequence shifts each score row by a constant:
    # softmax is unchanged, so dQ.(that vector) summed over ... => sum_j dK_j = 0 per (b, h)
    for b, n in enumerate(lengths):
        assert np.allclose(dK[b, :n].sum(0), 0.0, atol=1e-12)


# ---------------------------------------------------------------- P10: library routine
def test_forward_and_backward_match_torch_sdpa_fp64():
    lengths = [10, 7]
    L, H, D = 10, 3, 8
    c = _case(10, lengths, L, H, D)
    slopes, scale = c["slopes"], c["scale"]
    O, _ = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], slopes, scale)
    dQ, dK, dV = orc.attention_bwd(c["do"], c["q"], c["k"], c["v"], c["mask"], slopes, scale)
    for b, n in enumerate(lengths):
        tq, tk, tv = (torch.tensor(c[x][b, :n].astype(np.float64)).permute(1, 0, 2).contiguous().requires_grad_(True)
                      for x in ("q", "k", "v"))                                      # [H, n, D]
        pos = torch.arange(n, dtype=torch.float64)
        bias = -torch.tensor(slopes)[:, None, None] * (pos[:, None] - pos[None, :]).abs()[None]
        out = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=bias, scale=scale)
        out.backward(torch.tensor(c["do"][b, :n].astype(np.float64)).permute(1, 0, 2))
        assert np.allclose(out.detach().permute(1, 0, 2).numpy(), O[b, :n], atol=1e-13)
        for g, ref in ((tq.grad, dQ), (tk.grad, dK), (tv.grad, dV)):
            assert np.allclose(g.permute(1, 0, 2).numpy(), ref[b, :n], atol=1e-13)


# ---------------------------------------------------------------- P11: index maps
def _parse_fixture():
    out = {}
    for line in open(os.path.join(GOLDEN, "tiny_index_map.txt")):
        if line.startswith("#") or not line.strip():
            continue
        key, *vals = line.split()
        out[key] = vals
    idx = []
    for r in out["indices"]:
        a, b = r.split(":")
        idx.extend(range(int(a), int(b) + 1))
    return ([int(x) for x in out["lengths"]], [int(x) for x in out["cu_seqlens"]], idx,
            int(out["total_tokens"][0]), int(out["max_seqlen"][0]))


def test_index_maps_tiny_fixture():
    lengths, cu, idx, T, mx = _parse_fixture()
    b = wl.make_batch("tiny")
    assert list(b["lengths"]) == lengths
    got = orc.unpad_index(b["mask"])
    assert list(got[0]) == lengths and list(got[1]) == cu and list(got[2]) == idx
    assert got[3] == T and got[4] == mx
    assert got[1].dtype == np.int32 and got[2].dtype == np.int32


@pytest.mark.parametrize("seed,B,L,p", [(0, 3, 7, 0.5), (1, 8, 33, 0.8), (2, 1, 1, 1.0), (3, 5, 16, 0.0),
                                        (4, 5, 16, 1.0), (5, 2, 130, 0.3), (6, 64, 5, 0.05)])
def test_index_maps_brute_force(seed, B, L, p):
    mask = wl.random_mask(seed, B, L, p)
    mask[mask != 0] = np.random.default_rng(seed).integers(1, 5, size=int(mask.sum()))  # any nonzero keeps
    lengths, cu, idx, T, mx = orc.unpad_index(mask)
    assert np.array_equal(idx, np.flatnonzero(mask.reshape(-1)))
    assert np.array_equal(lengths, (mask != 0).sum(1))
    assert cu[0] == 0 and np.array_equal(np.diff(cu), lengths) and cu[-1] == T == np.count_nonzero(mask)
    assert mx == (lengths.max() if B else 0)
    assert np.all(np.diff(idx) > 0)
    X = np.random.default_rng(seed + 1).standard_normal((B, L, 3))
    Y = orc.unpad(X, idx)
    assert Y.shape == (T, 3)
    back = orc.pad(Y, idx, B, L)
    assert np.array_equal(back, X * (mask != 0)[:, :, None])
    assert np.array_equal(orc.unpad(back, idx), Y)
    assert np.array_equal(Y, X.reshape(B * L, 3)[np.flatnonzero(mask.reshape(-1))])


def test_unpadded_equals_masked_padded():
    """Packed tokens of sequence b are the rows cu[b]..cu[b+1]-1, at positions 0..len-1."""
    lengths = [5, 17, 32, 9]
    c = _case(12, lengths, 32, 2, 8)
    O, _ = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    _, cu, idx, T, _ = orc.unpad_index(c["mask"])
    Op = orc.unpad(O, idx)
    qp, kp, vp = (orc.unpad(c[x], idx) for x in ("q", "k", "v"))
    for b, n in enumerate(lengths):
        s, e = cu[b], cu[b + 1]
        one = orc.attention_fwd(qp[None, s:e], kp[None, s:e], vp[None, s:e], np.ones((1, n), np.int32), c["slopes"], c["scale"])[0]
        assert np.allclose(one[0], Op[s:e], atol=1e-14)


# ---------------------------------------------------------------- P12: numerics of the oracle itself
def test_shift_invariance_and_large_logits():
    c = _case(13, [8, 3], 8, 2, 4)
    O, LSE = orc.attention_fwd(c["q"], c["k"], c["v"], c["mask"], c["slopes"], c["scale"])
    # adding one vector u to every key shifts row i of the scores by scale*q_i.u: P and O unchanged
    u = np.random.default_rng(3).standard_normal(4)
    O2, LSE2 = orc.attention_fwd(c["q"], c["k"] + u, c["v"], c["mask"], c["slopes"], c["scale"])
    assert np.allclose(O2, O, atol=1e-13)
    shift = c["scale"] * np.einsum("blhd,d->bhl", c["q"].astype(np.float64), u)
    for b, n in enumerate(c["lengths"]):
        assert np.allclose(LSE2[b, :, :n], LSE[b, :, :n] + shift[b, :, :n], atol=1e-12)
    # huge logits: no overflow, rows still sum to one, output is (nearly) the argmax row of V
    Ob, LSEb, Pb = orc.attention_fwd(c["q"] * 1e3, c["k"], c["v"], c["mask"], c["slopes"], c["scale"], return_probs=True)
    assert np.all(np.isfinite(Ob)) and np.all(np.isfinite(LSEb[0])) and np.allclose(Pb[0].sum(-1), 1.0, atol=1e-14)


def test_attention_oracle_rejects_non_suffix_padding():
    c = _case(14, [4], 6, 1, 2)
    bad = c["mask"].copy()
    bad[0, 1] = 0
    with pytest.raises(ValueError):
        orc.attention_fwd(c["q"], c["k"], c["v"], bad, c["slopes"], c["scale"])


# ---------------------------------------------------------------- input generators
def test_workload_recipes():
    b = wl.make_batch("bert_base", batch=64)
    w = b["workload"]
    assert b["q"].shape == (64, 128, 12, 64) and b["mask"].shape == (64, 128)
    assert np.all((b["lengths"] >= 16) & (b["lengths"] <= 128))
    assert np.array_equal(wl.round_to_bf16(b["q"]), b["q"])           # already bf16-representable
    assert abs(float(b["q"].std()) - 0.125) < 2e-3 and abs(float(b["do"].std()) - 1.0) < 1e-2
    b2 = wl.make_batch("bert_base", batch=64)
    assert np.array_equal(b2["lengths"], b["lengths"]) and np.array_equal(b2["k"], b["k"])   # seeded
    full = wl.draw_lengths(wl.WORKLOADS["bert_base"], np.random.default_rng(1))
    assert 0.45 < np.mean(full == 128) < 0.75
    l5 = wl.draw_lengths(wl.WORKLOADS["ragged2048"], np.random.default_rng(2))
    assert l5.min() >= 8 and l5.max() <= 2048
    # round-to-nearest-even at the bf16 boundary
    x = np.array([1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20], dtype=np.float32)
    assert np.array_equal(wl.round_to_bf16(x), np.array([1.0, 1.0 + 2.0 ** -6, 1.0 + 2.0 ** -7], dtype=np.float32))


# ---------------------------------------------------------------- Add & LayerNorm (bf16 storage)
def _ln_case(seed, T, W):
    rng = np.random.default_rng(seed)
    x = wl.round_to_bf16(rng.standard_normal((T, W), dtype=np.float32) * 1.5)
    r = wl.round_to_bf16(rng.standard_normal((T, W), dtype=np.float32) + 0.3)
    gamma = wl.round_to_bf16(1.0 + 0.2 * rng.standard_normal(W, dtype=np.float32))
    beta = wl.round_to_bf16(0.1 * rng.standard_normal(W, dtype=np.float32))
    dy = wl.round_to_bf16(rng.standard_normal((T, W), dtype=np.float32))
    return x, r, gamma, beta, dy


def test_layernorm_forward_pins():
    x, r, gamma, beta, _ = _ln_case(1, 7, 48)
    y, s, mean, rstd = orc.add_layernorm_fwd(x, r, np.ones(48), np.zeros(48), 0.0)
    # normalised rows have mean 0 and variance 1
    assert np.allclose(y.mean(1), 0, atol=1e-13) and np.allclose((y ** 2).mean(1), 1, atol=1e-12)
    # the stored sum is the exact sum rounded to bf16 (the generator's rounding is an independent routine)
    assert np.array_equal(s, wl.round_to_bf16((x.astype(np.float64) + r).astype(np.float32)).astype(np.float64))
    # affine invariance (eps = 0): LN(a s + b) = LN(s) for a > 0; sign flip for a < 0
    y1, *_ = orc.add_layernorm_fwd(3.0 * s + 5.0, None, gamma, beta, 0.0)
    y0, *_ = orc.add_layernorm_fwd(s, None, gamma, beta, 0.0)
    ym, *_ = orc.add_layernorm_fwd(-2.0 * s, None, gamma, np.zeros(48), 0.0)
    yz, *_ = orc.add_layernorm_fwd(s, None, gamma, np.zeros(48), 0.0)
    assert np.allclose(y1, y0, atol=1e-12) and np.allclose(ym, -yz, atol=1e-12)
    # library routine, float64, with eps
    t = torch.nn.functional.layer_norm(torch.tensor(s), (48,), torch.tensor(gamma.astype(np.float64)),
                                       torch.tensor(beta.astype(np.float64)), 1e-5)
    y2, _, mean2, rstd2 = orc.add_layernorm_fwd(s, None, gamma, beta, 1e-5)
    assert np.allclose(t.numpy(), y2, atol=1e-13)
    assert np.allclose(mean2, s.mean(1)) and np.allclose(rstd2, 1 / np.sqrt(s.var(1) + 1e-5))
    # a constant row: variance 0, output = beta (eps keeps it finite)
    yc, *_ = orc.add_layernorm_fwd(np.full((1, 48), 2.5), None, gamma, beta, 1e-5)
    assert np.allclose(yc[0], beta, atol=1e-12)


def test_layernorm_backward_pins():
    x, r, gamma, beta, dy = _ln_case(2, 6, 40)
    eps = 1e-5
    _, s, _, _ = orc.add_layernorm_fwd(x, r, gamma, beta, eps)
    ds, dg, db = orc.add_layernorm_bwd(dy, s, gamma, eps)
    # library autograd, float64
    ts = torch.tensor(s, requires_grad=True)
    tg = torch.tensor(gamma.astype(np.float64), requires_grad=True)
    tb = torch.tensor(beta.astype(np.float64), requires_grad=True)
    torch.nn.functional.layer_norm(ts, (40,), tg, tb, eps).backward(torch.tensor(dy.astype(np.float64)))
    assert np.allclose(ts.grad.numpy(), ds, atol=1e-12) and np.allclose(tg.grad.numpy(), dg, atol=1e-12)
    assert np.allclose(tb.grad.numpy(), db, atol=1e-12)
    # central differences along random directions
    rng = np.random.default_rng(3)
    loss = lambda s_, g_, b_: float(np.sum(orc.add_layernorm_fwd(s_, None, g_, b_, eps)[0] * dy))
    g64, b64 = gamma.astype(np.float64), beta.astype(np.float64)
    for _ in range(3):
        U = rng.standard_normal(s.shape)
        fd = (loss(s + 1e-6 * U, g64, b64) - loss(s - 1e-6 * U, g64, b64)) / 2e-6
        assert abs(fd - np.sum(ds * U)) <= 1e-6 * max(1.0, abs(fd))
        u = rng.standard_normal(40)
        fd = (loss(s, g64 + 1e-6 * u, b64) - loss(s, g64 - 1e-6 * u, b64)) / 2e-6
        assert abs(fd - np.sum(dg * u)) <= 1e-6 * max(1.0, abs(fd))
    # the normalisation removes the mean and the scale of each row: ds is orthogonal to 1 and to xhat
    xhat = (s - s.mean(1, keepdims=True)) / np.sqrt(s.var(1, keepdims=True) + eps)
    assert np.allclose(ds.sum(1), 0, atol=1e-12)
    assert np.allclose((ds * xhat).sum(1) / 40, 0, atol=1e-4)      # exactly 0 only for eps = 0
    ds0, _, _ = orc.add_layernorm_bwd(dy, s, gamma, 0.0)
    xhat0 = (s - s.mean(1, keepdims=True)) / np.sqrt(s.var(1, keepdims=True))
    assert np.allclose((ds0 * xhat0).sum(1), 0, atol=1e-11)
    assert np.allclose(db, dy.sum(0))


# --------------------------------------------------------------------------- GeGLU feed-forward (Eq. 2)
def test_gelu_pins():
    import math
    z = np.linspace(-6.0, 6.0, 241)
    y = orc.gelu(z)
    # closed values: GeLU(0) = 0; Phi(1) = 0.841344746068543 (standard normal table)
    assert orc.gelu(np.array([0.0]))[0] == 0.0
    assert abs(orc.gelu(np.array([1.0]))[0] - 0.841344746068543) < 1e-15
    assert abs(orc.gelu(np.array([-1.0]))[0] + (1.0 - 0.841344746068543)) < 1e-15
    # Phi(z) + Phi(-z) = 1  =>  GeLU(z) - GeLU(-z) = z
    np.testing.assert_allclose(y - orc.gelu(-z), z, atol=1e-15)
    # brute force: Phi(z) = 1/2 + integral_0^z phi(t) dt by composite Simpson on 2000 panels
    def phi_int(zz):
        n = 2000
        t = np.linspace(0.0, zz, n + 1)
        f = np.exp(-0.5 * t * t) / math.sqrt(2.0 * math.pi)
        return 0.5 + (zz / n) / 3.0 * (f[0] + f[-1] + 4.0 * f[1:-1:2].sum() + 2.0 * f[2:-1:2].sum())
    for zz in (-3.3, -1.7, -0.4, 0.25, 0.9, 2.2, 4.1):
        assert abs(orc.gelu(np.array([zz]))[0] - zz * phi_int(zz)) < 1e-12
    # another library's erf, and torch's exact gelu in float64
    np.testing.assert_allclose(y, [0.5 * t * (1.0 + math.erf(t / math.sqrt(2.0))) for t in z], atol=1e-15)
    np.testing.assert_allclose(y, torch.nn.functional.gelu(torch.from_numpy(z), approximate="none").numpy(), atol=1e-15)
    # not the tanh fit: the two differ by up to ~5e-4 near |z| = 2
    assert np.abs(y - torch.nn.functional.gelu(torch.from_numpy(z), approximate="tanh").numpy()).max() > 1e-4
    # limits and derivative
    assert abs(orc.gelu(np.array([12.0]))[0] - 12.0) < 1e-15 and abs(orc.gelu(np.array([-12.0]))[0]) < 1e-15
    eps = 1e-6
    np.testing.assert_allclose(orc.gelu_grad(z), (orc.gelu(z + eps) - orc.gelu(z - eps)) / (2 * eps), atol=1e-9)


def _geglu_case(seed, T, hidden, inter):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((T, hidden))
    w1 = rng.standard_normal((inter, hidden)) / np.sqrt(hidden)
    v = rng.standard_normal((inter, hidden)) / np.sqrt(hidden)
    w2 = rng.standard_normal((hidden, inter)) / np.sqrt(inter)
    dy = rng.standard_normal((T, hidden))
    return x, w1, v, w2, dy


def test_geglu_forward_pins():
    x, w1, v, w2, _ = _geglu_case(3, 7, 5, 11)
    y, a = orc.geglu_fwd(x, w1, v, w2)
    assert y.shape == (7, 5) and a.shape == (7, 11)
    # element by element from the definition, with plain loops and math.erf
    import math
    for t in (0, 3, 6):
        for j in (0, 4, 10):
            h = sum(x[t, c] * w1[j, c] for c in range(5))
            g = sum(x[t, c] * v[j, c] for c in range(5))
            assert abs(a[t, j] - 0.5 * h * (1.0 + math.erf(h / math.sqrt(2.0))) * g) < 1e-14
        for c in (0, 2, 4):
            assert abs(y[t, c] - sum(a[t, j] * w2[c, j] for j in range(11))) < 1e-13
    # library composition in float64 (linear layers store [out_features, in_features])
    F = torch.nn.functional
    tx, tw1, tv, tw2 = (torch.from_numpy(t) for t in (x, w1, v, w2))
    ref = F.linear(F.gelu(F.linear(tx, tw1)) * F.linear(tx, tv), tw2)
    np.testing.assert_allclose(y, ref.numpy(), atol=1e-13)
    # the fused layout of the appendix on GLU implementations: one projection of twice the width, then a slice
    both = F.linear(tx, torch.cat([tw1, tv], dim=0))
    ref2 = F.linear(F.gelu(both[:, :11]) * both[:, 11:], tw2)
    np.testing.assert_allclose(y, ref2.numpy(), atol=1e-13)
    # special cases: zero gate matrix -> zero output; the gate is linear in V; rows are independent;
    # swapping W1 and V changes the result (the nonlinearity sits on the W1 branch only)
    assert np.all(orc.geglu_fwd(x, w1, 0 * v, w2)[0] == 0)
    np.testing.assert_allclose(orc.geglu_fwd(x, w1, 3.0 * v, w2)[0], 3.0 * y, atol=1e-13)
    np.testing.assert_allclose(orc.geglu_fwd(x[2:3], w1, v, w2)[0], y[2:3], atol=1e-14)
    assert np.abs(orc.geglu_fwd(x, v, w1, w2)[0] - y).max() > 1e-2
    # identity output projection and a gate that is constantly 1 reduce to GeLU of a linear layer
    w2i = np.eye(11)
    vi = np.zeros((11, 5)); xi = x.copy(); xi[:, 0] = 1.0; vi[:, 0] = 1.0
    np.testing.assert_allclose(orc.geglu_fwd(xi, w1, vi, w2i)[0], orc.gelu(xi @ w1.T), atol=1e-14)


def test_unfused_pieces_compose_to_geglu():
    """The three arrangements of the appendix on GLU implementations are the same function: two separate
    projections, one double-width projection that is sliced, and Eq. 2 as written."""
    x, w1, v, w2, _ = _geglu_case(9, 6, 4, 10)
    y, a = orc.geglu_fwd(x, w1, v, w2)
    h, g = orc.linear_fwd(x, w1), orc.linear_fwd(x, v)
    # linear_fwd element by element
    for t, j in ((0, 0), (5, 9), (3, 4)):
        assert abs(h[t, j] - sum(x[t, c] * w1[j, c] for c in range(4))) < 1e-14
    np.testing.assert_allclose(orc.gelu_gate(h, g), a, atol=1e-14)
    np.testing.assert_allclose(orc.linear_fwd(orc.gelu_gate(h, g), w2), y, atol=1e-13)
    hg = orc.linear_fwd(x, np.concatenate([w1, v], axis=0))
    np.testing.assert_allclose(orc.linear_fwd(orc.gelu_gate(hg[:, :10], hg[:, 10:]), w2), y, atol=1e-13)
    # gelu_gate is GeLU on the first argument only
    np.testing.assert_allclose(orc.gelu_gate(h, np.ones_like(h)), orc.gelu(h), atol=0)
    assert np.abs(orc.gelu_gate(g, h) - a).max() > 1e-3


def test_geglu_backward_pins():
    x, w1, v, w2, dy = _geglu_case(5, 6, 4, 9)
    dx, dw1, dv, dw2 = orc.geglu_bwd(dy, x, w1, v, w2)
    # torch autograd in float64
    F = torch.nn.functional
    ts = [torch.from_numpy(t).clone().requires_grad_(True) for t in (x, w1, v, w2)]
    out = F.linear(F.gelu(F.linear(ts[0], ts[1])) * F.linear(ts[0], ts[2]), ts[3])
    (out * torch.from_numpy(dy)).sum().backward()
    for mine, t in zip((dx, dw1, dv, dw2), ts):
        np.testing.assert_allclose(mine, t.grad.numpy(), atol=1e-12)
    # central finite differences of the scalar loss, a few entries of every argument
    def loss(x_, w1_, v_, w2_):
        return float((orc.geglu_fwd(x_, w1_, v_, w2_)[0] * dy).sum())
    args = [x, w1, v, w2]
    eps = 1e-6
    for which, grad in enumerate((dx, dw1, dv, dw2)):
        for idx in ((0, 0), (1, 2), (grad.shape[0] - 1, grad.shape[1] - 1)):
            plus = [t.copy() for t in args]; minus = [t.copy() for t in args]
            plus[which][idx] += eps; minus[which][idx] -= eps
            fd = (loss(*plus) - loss(*minus)) / (2 * eps)
            assert abs(fd - grad[idx]) < 1e-7 * max(1.0, abs(fd)), (which, idx, fd, grad[idx])
