"""Tolerance of the attention parity tests (bf16 path vs. the float64 oracle).

Both conditions must hold for every (row, head) output vector:
  * max-abs:  max_d |g - o| <= 2e-2
  * row-normalised max-rel: max_d |g - o| / max_d |o| <= 1e-2
The second is needed because with N(0,1) inputs and long contexts outputs are ~1e-2 in magnitude, so
the absolute bound alone would accept an all-zero result, while an element-wise relative bound is
unbounded near zero crossings.
"""
import numpy as np

MAX_ABS = 2e-2
MAX_REL = 1e-2


def check(got: np.ndarray, want: np.ndarray, what: str = "") -> None:
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got - want).max(axis=-1)
    ref = np.abs(want).max(axis=-1)
    rel = err / np.maximum(ref, 1e-30)
    worst = np.unravel_index(np.argmax(rel), rel.shape)
    assert err.max() <= MAX_ABS, f"{what}: max-abs {err.max():.3e} > {MAX_ABS}"
    assert rel.max() <= MAX_REL, f"{what}: row-normalised max-rel {rel.max():.3e} at {worst} > {MAX_REL}"
