"""The pins have teeth: a copy of the oracle with ONE planted mistake (made on the CPU by editing a copy of
its source text; the oracle itself is never touched) must fail the pin named beside it.

Each entry: (what is planted, the exact source text replaced, its replacement, the pin test that must fail, its
arguments).  A pin "fails" when it raises AssertionError with the mutant in place of the oracle.
"""
import importlib.util
import os
import types

import pytest

from tests import test_oracle_pins as pins

ORACLE_SRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "oracle", "mosaic_oracle.py")

MISTAKES = [
    ("bias added instead of subtracted (Eq. 1)",
     "scale * (q @ k.T) - slope * np.abs(", "scale * (q @ k.T) + slope * np.abs(",
     "test_alibi_closed_form_identical_keys", (19, 2.0 ** -4)),
    ("one-sided (causal-style) distance instead of |i - j|",
     "np.abs(pos[:, None] - pos[None, :])", "np.maximum(pos[:, None] - pos[None, :], 0.0)",
     "test_reversal_symmetry_and_permutation_invariance", ()),
    ("scores with transposed operands",
     "scale * (q @ k.T) -", "scale * (k @ q.T) -",
     "test_forward_and_backward_match_torch_sdpa_fp64", ()),
    ("slopes start one term early (m_0 = 1)",
     "for h in range(1, H + 1)]", "for h in range(0, H)]",
     "test_slopes_match_fixture", ()),
    ("scale missing in dK",
     "dK[b, :, h] = scale * (dS.T @ q)", "dK[b, :, h] = (dS.T @ q)",
     "test_backward_matches_central_differences", ("random",)),
    ("Delta dropped from dS",
     "dS = P * (dP - delta)", "dS = P * dP",
     "test_backward_identities", ()),
    ("P not transposed in dV",
     "dV[b, :, h] = P.T @ g", "dV[b, :, h] = P @ g",
     "test_backward_matches_central_differences", ("tiny",)),
    ("dQ contracted with queries instead of keys",
     "dQ[b, :, h] = scale * (dS @ k)", "dQ[b, :, h] = scale * (dS @ q)",
     "test_forward_and_backward_match_torch_sdpa_fp64", ()),
    ("padded keys not masked",
     "    S[:, ~valid] = -np.inf\n", "",
     "test_padding_content_and_width_do_not_matter", ()),
    ("indices off by one position",
     "indices.append(b * L + l)", "indices.append(b * L + l + 1)",
     "test_index_maps_tiny_fixture", ()),
    ("cu_seqlens is an inclusive instead of an exclusive prefix sum",
     "cu[b + 1] = cu[b] + n", "cu[b] = (cu[b - 1] if b else 0) + n",
     "test_index_maps_tiny_fixture", ()),
    ("log-sum-exp without the row maximum",
     "LSE[b, h, valid] = (M + np.log(Z))[valid, 0]", "LSE[b, h, valid] = (np.log(Z))[valid, 0]",
     "test_rows_sum_to_one_and_lse_consistent", ()),
]


def _mutant(old: str, new: str) -> types.ModuleType:
    src = open(ORACLE_SRC).read()
    assert src.count(old) == 1, "planted-mistake anchor must occur exactly once in the oracle: %r" % old
    spec = importlib.util.spec_from_loader("mosaic_oracle_mutant", loader=None)
    mod = importlib.util.module_from_spec(spec)
    exec(compile(src.replace(old, new), ORACLE_SRC + " (mutant)", "exec"), mod.__dict__)
    return mod


@pytest.mark.parametrize("what,old,new,pin,args", MISTAKES, ids=[m[0] for m in MISTAKES])
def test_planted_mistake_fails_its_pin(monkeypatch, what, old, new, pin, args):
    getattr(pins, pin)(*args)                       # the pin passes on the oracle as it stands
    monkeypatch.setattr(pins, "orc", _mutant(old, new))
    with pytest.raises(AssertionError):
        getattr(pins, pin)(*args)
