"""Shared comparison helpers for the GPU parity tests."""
import numpy as np

# tolerance on the fp16 block output, as stated for this build's north star
MAX_ABS = 2e-2
REL_L2 = 5e-3


def errors(got, want):
    got = np.asarray(got, dtype=np.float64).ravel()
    want = np.asarray(want, dtype=np.float64).ravel()
    assert got.shape == want.shape
    assert np.isfinite(got).all(), "non-finite values in the GPU output"
    return float(np.abs(got - want).max()), float(np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30))


def assert_block_close(got, want, what=""):
    ma, rl = errors(got, want)
    assert ma <= MAX_ABS and rl <= REL_L2, f"{what}: max-abs {ma:.3e} (<= {MAX_ABS}), rel-L2 {rl:.3e} (<= {REL_L2})"
    return ma, rl


def assert_fp16_rows_match(got, want, what="", max_fraction=0.02):
    """Appended K/V rows: both sides round an fp32-or-better value to fp16, so
    they are equal except where the two accumulations straddle a rounding
    boundary; then they differ by one fp16 step."""
    g = np.asarray(got, dtype=np.float16)
    w = np.asarray(want, dtype=np.float16)
    assert g.shape == w.shape and np.isfinite(g.astype(np.float32)).all(), what
    diff = g != w
    step = np.spacing(np.abs(w).astype(np.float16)).astype(np.float64)
    # near zero an fp16 step is far below the fp32 accumulation error of an
    # O(1)-magnitude dot product, hence the small absolute term
    assert (np.abs(g.astype(np.float64) - w.astype(np.float64)) <= step + 1e-5).all(), f"{what}: more than one fp16 step apart"
    assert diff.mean() <= max_fraction, f"{what}: {diff.mean():.3%} of appended values differ"
