"""Comparison helpers for the GPU-vs-oracle parity tests (tolerances and the near-tie protocol).

Tolerances (stated by the task definition, restated here so that the tests are self-contained):
  * scores, similarities and merged features: max relative error 1e-3 for bf16 inputs with fp32
    accumulation, 1e-5 for fp32 inputs;
  * boundaries, index sets and gathered tensors: bit-exact, where index sets are compared outside a
    band of relative width 1e-3 around the selection threshold; disagreements inside the band are
    reported, never silent.

The named configurations and the bench configuration are held to exactly these bars (frame scores relative
to the oracle's own value, bf16 merged features within one ulp).  Random sweeps draw inputs whose signed
terms can cancel to a result orders of magnitude below the terms; only there the error is measured against
the magnitude of the terms (frame_score_scale, assert_pooled_bf16).
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

RTOL = {"bf16": 1e-3, "f32": 1e-5}
BAND = 1e-3


def assert_rel(got, want, rtol, what, scale=None):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    ref = np.abs(want) if scale is None else np.broadcast_to(np.asarray(scale, dtype=np.float64), want.shape)
    err = np.abs(got - want)
    bad = err > rtol * ref
    if bad.any():
        i = int(np.argmax(err / np.maximum(ref, 1e-300)))
        raise AssertionError(f"{what}: {int(bad.sum())} of {bad.size} beyond rtol {rtol}; worst at {i}: "
                             f"got {got.ravel()[i]!r} want {want.ravel()[i]!r}")
    return float((err / np.maximum(ref, 1e-300)).max()) if err.size else 0.0


def frame_score_scale(V, t):
    """Per frame, the mean over its tokens of |cos(token, t)|: the magnitude of the N signed terms that
    Eq. 5 averages.  The rounding error of a frame score is relative to this magnitude, not to the score
    itself, which can cancel to orders of magnitude less.  A tolerance scale only, never an expected value."""
    V = np.asarray(V, dtype=np.float64)
    t = np.asarray(t, dtype=np.float64).reshape(-1)
    den = np.linalg.norm(V, axis=2) * np.linalg.norm(t)
    cos = np.divide(V @ t, den, out=np.zeros_like(den), where=den >= 1e-12)
    return np.abs(cos).mean(axis=1)


def assert_rows_close(got, want, rtol, what):
    """|g - o|_inf <= rtol * |o_row|_inf per row (element-wise relative error is meaningless near 0)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, f"{what}: shape {got.shape} vs {want.shape}"
    if got.size == 0:
        return 0.0
    scale = np.abs(want).max(axis=1, keepdims=True)
    err = np.abs(got - want)
    worst = float((err / np.maximum(scale, 1e-300)).max())
    assert worst <= rtol, f"{what}: worst row-relative error {worst:.3e} > {rtol}"
    return worst


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers at |x| (8 significant bits)."""
    x = np.abs(np.asarray(x, dtype=np.float64))
    _, e = np.frexp(np.maximum(x, 2.0 ** -126))
    return np.ldexp(1.0, e - 8)


def assert_pooled_bf16(got, exact_mean, vmax, cells, what):
    """bf16 output of the pooled merge: fp32 accumulation of `cells` inputs, one division, one rounding to
    bf16.  The result lies within one bf16 ulp of the exact mean plus the fp32 accumulation error, which is at
    most cells * 2^-24 * max|input| for the mean of `cells` sequential additions; that term only shows where
    the inputs of a window cancel and the mean is orders of magnitude below them.  Apart from rare double
    rounding flips (fp32 mean -> bf16 against fp64 mean -> bf16) the result equals the rounded exact mean."""
    got = np.asarray(got, dtype=np.float64)
    exact_mean = np.asarray(exact_mean, dtype=np.float64)
    assert got.shape == exact_mean.shape, f"{what}: shape {got.shape} vs {exact_mean.shape}"
    tol = bf16_ulp(exact_mean) + cells * 2.0 ** -24 * float(vmax)
    err = np.abs(got - exact_mean)
    assert (err <= tol).all(), f"{what}: pooled bf16 token further than one ulp (+ fp32 accumulation) from the exact mean"
    return err


def assert_pooled_bf16_strict(got, exact_mean, what):
    """The plain bar for a bf16 merged feature: within one bf16 ulp of the exact mean.  Used on the named
    configurations, whose windows do not cancel; the random sweeps use assert_pooled_bf16."""
    got = np.asarray(got, dtype=np.float64)
    exact_mean = np.asarray(exact_mean, dtype=np.float64)
    assert got.shape == exact_mean.shape, f"{what}: shape {got.shape} vs {exact_mean.shape}"
    err = np.abs(got - exact_mean)
    assert (err <= bf16_ulp(exact_mean)).all(), f"{what}: pooled bf16 token further than one ulp from the exact mean"
    return err


def near_tie_report(scores_oracle: np.ndarray, token_seg: np.ndarray, quotas: Sequence[int],
                    kept_gpu: np.ndarray, kept_oracle: np.ndarray) -> Dict[str, int]:
    """Compare two kept sets segment by segment.  Outside the band |score - tau| <= 1e-3 |tau| around
    the oracle's threshold tau (its quota-th largest score) the sets must be identical."""
    s = np.asarray(scores_oracle, dtype=np.float64)
    seg = np.asarray(token_seg)
    g = np.zeros(s.shape[0], dtype=bool); g[np.asarray(kept_gpu, dtype=np.int64)] = True
    o = np.zeros(s.shape[0], dtype=bool); o[np.asarray(kept_oracle, dtype=np.int64)] = True
    report = dict(band_population=0, disagreements_in_band=0)
    for si, quota in enumerate(quotas):
        members = np.nonzero(seg == si)[0]
        assert int(g[members].sum()) == int(quota), f"segment {si}: GPU kept {int(g[members].sum())}, quota {quota}"
        if quota == 0 or quota == len(members):
            assert np.array_equal(g[members], o[members])
            continue
        tau = np.sort(s[members])[::-1][quota - 1]
        in_band = np.abs(s[members] - tau) <= BAND * abs(tau)
        diff = g[members] != o[members]
        assert not (diff & ~in_band).any(), (
            f"segment {si}: kept sets differ outside the near-tie band at "
            f"{members[np.nonzero(diff & ~in_band)[0][:5]].tolist()}")
        report["band_population"] += int(in_band.sum())
        report["disagreements_in_band"] += int(diff.sum())
    return report
