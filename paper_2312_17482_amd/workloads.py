"""Seeded synthetic inputs for the unpad -> ALiBi attention -> pad path.

This module only draws random numbers and shapes them; it contains none of the
method's arithmetic (no softmax, no bias, no slopes, no index maps), so both
the HIP path's tests and the CPU oracle's tests may take their inputs from it.

The five workloads stand in for microbatches of a C4-like corpus truncated at
max_len tokens (paper section "Pretraining Optimizations", Data paragraph, and
the sequence-length sweep of the appendix): the corpus itself is not available,
so sequence lengths are drawn from the stated synthetic mixtures.

Everything is numpy on the host. Tensors are returned as float32 arrays whose
values are exactly representable in the workload's storage type (bf16 values
are rounded to nearest-even here, once), so a GPU path that stores bf16 and an
fp64 oracle both start from identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Dict, Tuple

import numpy as np

BASE_SEED = 20231217


@dataclass(frozen=True)
class Workload:
    name: str
    cfg: int          # 1-based position in the configuration list
    B: int            # sequences in the batch
    L: int            # max_len (padded length)
    H: int            # attention heads
    D: int            # head dimension
    dtype: str        # "f32" or "bf16": storage type of Q/K/V/dO
    qkv_std: float    # standard deviation of Q, K, V entries
    lengths: str      # name of the length recipe


WORKLOADS: Dict[str, Workload] = {
    "tiny": Workload("tiny", 1, 4, 32, 2, 16, "f32", 1.0, "fixed_tiny"),
    "bert_base": Workload("bert_base", 2, 256, 128, 12, 64, "bf16", 0.125, "mix60"),
    "bert_large": Workload("bert_large", 3, 256, 128, 16, 64, "bf16", 0.125, "mix60"),
    "long512": Workload("long512", 4, 64, 512, 12, 64, "bf16", 0.125, "uniform64"),
    "ragged2048": Workload("ragged2048", 5, 16, 2048, 16, 64, "bf16", 0.125, "lognormal"),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    rounded = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "values are not bf16-representable"
    return (u >> np.uint32(16)).astype(np.uint16)


def draw_lengths(w: Workload, rng: np.random.Generator) -> np.ndarray:
    if w.lengths == "fixed_tiny":
        return np.array([5, 17, 32, 9], dtype=np.int32)
    if w.lengths == "mix60":
        full = rng.random(w.B) < 0.6
        short = rng.integers(16, w.L, size=w.B)          # uniform integer in [16, L-1]
        return np.where(full, w.L, short).astype(np.int32)
    if w.lengths == "uniform64":
        return rng.integers(64, w.L + 1, size=w.B).astype(np.int32)
    if w.lengths == "lognormal":
        raw = np.rint(rng.lognormal(mean=6.0, sigma=0.8, size=w.B))
        return np.clip(raw, 8, w.L).astype(np.int32)
    raise ValueError(w.lengths)


def suffix_mask(lengths: np.ndarray, L: int) -> np.ndarray:
    """[B, L] int32 mask: 1 for the first lengths[b] positions of row b, else 0."""
    return (np.arange(L, dtype=np.int32)[None, :] < np.asarray(lengths)[:, None]).astype(np.int32)


def make_batch(name: str, seed_offset: int = 0, batch: int | None = None, full_length: bool = False) -> dict:
    """Draw one batch of the named workload.

    Returns a dict with: workload, lengths [B], mask [B,L] int32, q/k/v/do
    [B,L,H,D] float32 (padded layout, pad rows hold random values too, which the
    path must ignore), scale (1/sqrt(D)).  `batch` overrides B (a sub-batch drawn
    with the same recipe) for cases an fp64 CPU check must finish quickly.
    """
    w = WORKLOADS[name]
    if batch is not None:
        w = Workload(w.name, w.cfg, batch, w.L, w.H, w.D, w.dtype, w.qkv_std, w.lengths)
        if w.lengths == "fixed_tiny":
            assert batch == 4
    rng = np.random.default_rng(BASE_SEED + w.cfg + 1000 * seed_offset)
    lengths = draw_lengths(w, rng)
    if full_length:          # no padding at all: every sequence has max_len tokens (kernel capability runs)
        lengths = np.full(w.B, w.L, dtype=np.int32)
    shape = (w.B, w.L, w.H, w.D)
    out = {"workload": w, "lengths": lengths, "mask": suffix_mask(lengths, w.L)}
    for key, std in (("q", w.qkv_std), ("k", w.qkv_std), ("v", w.qkv_std), ("do", 1.0)):
        t = rng.standard_normal(shape, dtype=np.float32) * np.float32(std)
        out[key] = round_to_bf16(t) if w.dtype == "bf16" else t
    out["scale"] = 1.0 / float(np.sqrt(w.D))
    return out


def random_attention_case(seed: int, lengths, L: int, H: int, D: int, std: float = 1.0,
                          bf16: bool = False, v_std: float | None = None) -> dict:
    """Free-form case for parity/edge tests: explicit lengths, suffix mask, Q,K ~ N(0,std^2),
    V ~ N(0,v_std^2) (v_std defaults to std), dO ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    lengths = np.asarray(lengths, dtype=np.int32)
    shape = (len(lengths), L, H, D)
    out = {"lengths": lengths, "mask": suffix_mask(lengths, L)}
    for key, s in (("q", std), ("k", std), ("v", std if v_std is None else v_std), ("do", 1.0)):
        t = rng.standard_normal(shape, dtype=np.float32) * np.float32(s)
        out[key] = round_to_bf16(t) if bf16 else t
    out["scale"] = 1.0 / float(np.sqrt(D))
    return out


def random_ffn_case(seed: int, T: int, hidden: int, inter: int, w_std: float = 0.02) -> dict:
    """Inputs of the feed-forward sublayer, rounded to bf16: x ~ N(0,1) (what a LayerNorm hands over),
    weights ~ N(0, w_std^2) in [out_features, in_features] storage (0.02 = the usual BERT initialisation;
    the paper states none), w1v = W1 transposed stacked over V transposed, dy ~ N(0,1)."""
    rng = np.random.default_rng(seed)
    x = round_to_bf16(rng.standard_normal((T, hidden), dtype=np.float32))
    w1v = round_to_bf16(rng.standard_normal((2 * inter, hidden), dtype=np.float32) * np.float32(w_std))
    w2 = round_to_bf16(rng.standard_normal((hidden, inter), dtype=np.float32) * np.float32(w_std))
    dy = round_to_bf16(rng.standard_normal((T, hidden), dtype=np.float32))
    return {"x": x, "w1v": w1v, "w2": w2, "dy": dy, "hidden": hidden, "inter": inter}


def random_mask(seed: int, B: int, L: int, keep_prob: float) -> np.ndarray:
    """Arbitrary 0/1 mask (holes allowed) for the index-map tests."""
    rng = np.random.default_rng(seed)
    return (rng.random((B, L)) < keep_prob).astype(np.int32)


def attention_flops(lengths: np.ndarray, H: int, D: int) -> Tuple[float, float]:
    """(forward, backward) multiply-add flops on real tokens: 4 and 10 times H*D*sum(len^2)."""
    s2 = float(np.sum(np.asarray(lengths, dtype=np.float64) ** 2))
    return 4.0 * H * D * s2, 10.0 * H * D * s2
