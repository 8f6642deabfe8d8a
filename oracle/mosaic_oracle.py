"""Plain CPU fp64 oracle for the unpad -> ALiBi attention -> pad path.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package imports this file;
only tests, the smoke check and the benchmark's cpu_baseline leg may call it.
It shares no code with the HIP kernels.

What it computes is the plain definition, on the PADDED [B, L] layout with a
mask, in float64:

* attention weights of the paper's Eq. 1 (section "Modifications to the
  Attention Mechanism"): softmax over keys of  scale * q_i.k_j - m_h * |i - j|,
  bidirectional, with the bias symmetric in the token distance;
* head slopes m_h forming a geometric sequence with ratio 2^(-8/H) (same
  section), first term equal to the ratio;
* the removal and restoration of padding tokens described in the "Unpadding"
  paragraph: all real tokens of a batch concatenated in order into one sequence.

The backward pass is the textbook derivative of that forward for the scalar
loss sum(O * dO); the paper prints no backward formula.

Readings taken where the paper is silent (each is also listed in the design
document): the 1/sqrt(d) factor is an explicit `scale` argument (Eq. 1 omits
it); positions are those of the padded row, which for suffix padding equal the
positions inside the packed sequence; masks are int, nonzero = real token;
indices are ascending flat positions b*L + l; logsumexp is the natural log.

Beyond the attention path the file holds the two neighbouring sublayers of the
encoder block in the same plain style: the residual add + LayerNorm with 2-byte
storage ("Low Precision LayerNorm" paragraph) and the GeGLU feed-forward of Eq. 2.

Every function here is pinned by tests/test_oracle_pins.py against closed
forms, invariants, finite differences, brute force and a library routine.
"""
from __future__ import annotations

import numpy as np


# --------------------------------------------------------------------------- slopes
def alibi_slopes(H: int) -> np.ndarray:
    """m_h = 2^(-8 h / H) for h = 1..H (geometric, ratio 2^(-8/H)); float64."""
    return np.array([2.0 ** (-8.0 * h / H) for h in range(1, H + 1)], dtype=np.float64)


# --------------------------------------------------------------------------- index maps
def unpad_index(mask: np.ndarray):
    """Index maps of the "Unpadding" paragraph, by a plain double loop.

    mask: [B, L] integers, nonzero = real token.
    Returns (lengths [B], cu_seqlens [B+1], indices [T], T, max_seqlen), int32/ints.
    """
    mask = np.asarray(mask)
    B, L = mask.shape
    lengths = np.zeros(B, dtype=np.int32)
    cu = np.zeros(B + 1, dtype=np.int32)
    indices = []
    for b in range(B):
        n = 0
        for l in range(L):
            if mask[b, l] != 0:
                indices.append(b * L + l)
                n += 1
        lengths[b] = n
        cu[b + 1] = cu[b] + n
    T = int(cu[B])
    max_seqlen = int(lengths.max()) if B > 0 else 0
    return lengths, cu, np.array(indices, dtype=np.int32), T, max_seqlen


def unpad(X: np.ndarray, indices: np.ndarray) -> np.ndarray:
    """packed[t, ...] = X.reshape(B*L, ...)[indices[t], ...]; X is [B, L, ...]."""
    flat = X.reshape((X.shape[0] * X.shape[1],) + X.shape[2:])
    out = np.empty((len(indices),) + flat.shape[1:], dtype=X.dtype)
    for t, p in enumerate(indices):
        out[t] = flat[p]
    return out


def pad(Y: np.ndarray, indices: np.ndarray, B: int, L: int) -> np.ndarray:
    """padded.reshape(B*L, ...)[indices[t]] = Y[t]; every other row is exactly zero."""
    flat = np.zeros((B * L,) + Y.shape[1:], dtype=Y.dtype)
    for t, p in enumerate(indices):
        flat[p] = Y[t]
    return flat.reshape((B, L) + Y.shape[1:])


# --------------------------------------------------------------------------- attention
def _check_suffix(mask_row: np.ndarray) -> int:
    n = int(np.count_nonzero(mask_row))
    if np.count_nonzero(mask_row[:n]) != n:
        raise ValueError("attention oracle expects padding as a suffix of each row")
    return n


def _scores(q, k, slope, scale, valid):
    """S[i, j] = scale * q_i.k_j - slope * |i - j|; -inf where key j is padding."""
    L = q.shape[0]
    pos = np.arange(L, dtype=np.float64)
    S = scale * (q @ k.T) - slope * np.abs(pos[:, None] - pos[None, :])
    S[:, ~valid] = -np.inf
    return S


def attention_fwd(Q, K, V, mask, slopes, scale, return_probs=False):
    """Masked, padded attention with symmetric ALiBi bias (Eq. 1).

    Q, K, V: [B, L, H, D]; mask [B, L]; slopes [H]; returns O [B, L, H, D]
    (zero at padded rows), LSE [B, H, L] (natural log; NaN at padded rows) and,
    on request, P [B, H, L, L] (zero at padded rows/columns).
    """
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, L, H, D = Q.shape
    O = np.zeros((B, L, H, D))
    LSE = np.full((B, H, L), np.nan)
    P_all = np.zeros((B, H, L, L)) if return_probs else None
    for b in range(B):
        n = _check_suffix(np.asarray(mask[b]))
        valid = np.asarray(mask[b]) != 0
        if n == 0:
            continue
        for h in range(H):
            S = _scores(Q[b, :, h], K[b, :, h], float(slopes[h]), scale, valid)
            M = S.max(axis=1, keepdims=True)
            E = np.exp(S - M)
            Z = E.sum(axis=1, keepdims=True)
            P = E / Z
            P[~valid, :] = 0.0
            v = np.where(valid[:, None], V[b, :, h], 0.0)    # pad content may be anything, even NaN
            O[b, :, h] = P @ v
            LSE[b, h, valid] = (M + np.log(Z))[valid, 0]
            if return_probs:
                P_all[b, h] = P
    if return_probs:
        return O, LSE, P_all
    return O, LSE


def attention_bwd(dO, Q, K, V, mask, slopes, scale):
    """Gradient of sum(O * dO) w.r.t. Q, K, V for attention_fwd.  All [B, L, H, D].

    Delta_i = sum_d dO_id O_id;  dV_j = sum_i P_ij dO_i;  dP_ij = dO_i . V_j;
    dS_ij = P_ij (dP_ij - Delta_i);  dQ_i = scale sum_j dS_ij K_j;
    dK_j = scale sum_i dS_ij Q_i.  Padded rows/columns contribute nothing and
    dO at padded rows is ignored.  The slopes are constants: no gradient.
    """
    dO = np.asarray(dO, dtype=np.float64)
    Q = np.asarray(Q, dtype=np.float64)
    K = np.asarray(K, dtype=np.float64)
    V = np.asarray(V, dtype=np.float64)
    B, L, H, D = Q.shape
    dQ = np.zeros_like(Q)
    dK = np.zeros_like(K)
    dV = np.zeros_like(V)
    for b in range(B):
        n = _check_suffix(np.asarray(mask[b]))
        valid = np.asarray(mask[b]) != 0
        if n == 0:
            continue
        for h in range(H):
            S = _scores(Q[b, :, h], K[b, :, h], float(slopes[h]), scale, valid)
            M = S.max(axis=1, keepdims=True)
            E = np.exp(S - M)
            P = E / E.sum(axis=1, keepdims=True)
            P[~valid, :] = 0.0
            g = np.where(valid[:, None], dO[b, :, h], 0.0)
            v = np.where(valid[:, None], V[b, :, h], 0.0)   # pad content may be anything, even NaN
            k = np.where(valid[:, None], K[b, :, h], 0.0)
            q = np.where(valid[:, None], Q[b, :, h], 0.0)
            o = P @ v
            delta = np.sum(g * o, axis=1, keepdims=True)
            dV[b, :, h] = P.T @ g
            dP = g @ v.T
            dS = P * (dP - delta)
            dQ[b, :, h] = scale * (dS @ k)
            dK[b, :, h] = scale * (dS.T @ q)
    return dQ, dK, dV


# --------------------------------------------------------------------------- Add & LayerNorm in bf16 storage
# Paper, "Low Precision LayerNorm" paragraph and the "Add & Norm" boxes of Figure 1A: LayerNorm reads and
# writes bfloat16 instead of float32 (it is bandwidth-bound, so halving the bytes is the point).  The
# paper fixes storage, not the internal arithmetic; the reading taken is: the residual sum s = x + r is a
# stored bf16 tensor (rounded to nearest even), the statistics and the normalisation are evaluated from
# that stored s in full precision, and y is rounded once when stored.  This oracle keeps everything after
# the rounding of s in float64 and leaves the final rounding of y to the comparison tolerance.
def _round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Nearest-even rounding of float64 values to bfloat16 (returned as float64)."""
    f32 = np.asarray(x, dtype=np.float64).astype(np.float32)          # exact for sums of two bf16 values
    u = f32.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).astype(np.float64)


def add_layernorm_fwd(x, r, gamma, beta, eps, round_sum=True):
    """s = x + r (r may be None), y = (s - mean) / sqrt(var + eps) * gamma + beta over the last axis,
    var = mean((s - mean)^2).  x, r: [T, W]; gamma, beta: [W].  Returns (y, s, mean [T], rstd [T])."""
    s = np.asarray(x, dtype=np.float64)
    if r is not None:
        s = s + np.asarray(r, dtype=np.float64)
        if round_sum:
            s = _round_to_bf16(s)
    mean = s.mean(axis=1)
    var = ((s - mean[:, None]) ** 2).mean(axis=1)
    rstd = 1.0 / np.sqrt(var + eps)
    y = (s - mean[:, None]) * rstd[:, None] * np.asarray(gamma, dtype=np.float64) + np.asarray(beta, dtype=np.float64)
    return y, s, mean, rstd


def add_layernorm_bwd(dy, s, gamma, eps):
    """Gradient of sum(y * dy) for add_layernorm_fwd with respect to s (= to x and to r), gamma and beta.
    xhat = (s - mean) rstd, g = dy * gamma:  ds = rstd * (g - mean(g) - xhat * mean(g * xhat)),
    dgamma = sum_t dy * xhat, dbeta = sum_t dy."""
    dy = np.asarray(dy, dtype=np.float64)
    s = np.asarray(s, dtype=np.float64)
    mean = s.mean(axis=1, keepdims=True)
    var = ((s - mean) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + eps)
    xhat = (s - mean) * rstd
    g = dy * np.asarray(gamma, dtype=np.float64)
    ds = rstd * (g - g.mean(axis=1, keepdims=True) - xhat * (g * xhat).mean(axis=1, keepdims=True))
    return ds, (dy * xhat).sum(axis=0), dy.sum(axis=0)


# --------------------------------------------------------------------------- GeGLU feed-forward
def gelu(z: np.ndarray) -> np.ndarray:
    """Gaussian-error linear unit, the exact form z * Phi(z) with Phi the standard normal
    distribution function, Phi(z) = (1 + erf(z / sqrt 2)) / 2 (section "Gated Linear Units": the
    paper names GeLU and gives no formula; the exact form is the reading taken, not the tanh fit)."""
    from scipy.special import erf
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * z * (1.0 + erf(z / np.sqrt(2.0)))


def gelu_grad(z: np.ndarray) -> np.ndarray:
    """d/dz [z Phi(z)] = Phi(z) + z phi(z), phi the standard normal density."""
    from scipy.special import erf
    z = np.asarray(z, dtype=np.float64)
    return 0.5 * (1.0 + erf(z / np.sqrt(2.0))) + z * np.exp(-0.5 * z * z) / np.sqrt(2.0 * np.pi)


def linear_fwd(x, wt):
    """Bias-free linear layer y = x W with wt = W transposed ([out_features, in_features]); float64."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(wt, dtype=np.float64).T


def gelu_gate(h, g):
    """GeLU(h) (*) g, elementwise: the activation of Eq. 2 between the projections."""
    return gelu(h) * np.asarray(g, dtype=np.float64)


def geglu_fwd(x, w1, v, w2):
    """Eq. 2:  y = (GeLU(x W1) (*) x V) W2, no bias terms, float64.

    x [T, hidden]; w1, v [inter, hidden] and w2 [hidden, inter] hold the TRANSPOSES of the paper's W1, V
    and W2 (the [out_features, in_features] storage of a linear layer), so x W1 is x @ w1.T.
    Returns (y [T, hidden], a [T, inter]) with a = GeLU(x W1) (*) x V, the tensor between the two
    projections."""
    x, w1, v, w2 = (np.asarray(t, dtype=np.float64) for t in (x, w1, v, w2))
    h = x @ w1.T
    g = x @ v.T
    a = gelu(h) * g
    return a @ w2.T, a


def geglu_bwd(dy, x, w1, v, w2):
    """Textbook derivative of geglu_fwd for the scalar loss sum(y * dy) (the paper prints none).
    Returns (dx, dw1, dv, dw2) in the layouts of x, w1, v, w2."""
    dy, x, w1, v, w2 = (np.asarray(t, dtype=np.float64) for t in (dy, x, w1, v, w2))
    h = x @ w1.T
    g = x @ v.T
    a = gelu(h) * g
    da = dy @ w2                    # [T, inter]
    dw2 = dy.T @ a                  # [hidden, inter]
    dh = da * g * gelu_grad(h)
    dg = da * gelu(h)
    dx = dh @ w1 + dg @ v
    return dx, dh.T @ x, dg.T @ x, dw2
