"""Comparison helpers shared by the GPU parity tests (no method arithmetic)."""
import numpy as np

CENT_RTOL = 1e-5     # centroid coordinates: |a-b| <= 1e-5*max(|a|,|b|) + 1e-6
CENT_ATOL = 1e-6     # (absolute floor: z-scored features have means near 0)
REL = 1e-5           # mu, ucb, objective: pure relative


def assert_cent_close(got, want, what="centroids"):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    tol = CENT_RTOL * np.maximum(np.abs(got), np.abs(want)) + CENT_ATOL
    bad = np.abs(got - want) > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside tolerance, worst " \
                          f"{np.abs(got - want).max():.3e}"


def assert_rel_close(got, want, rel=REL, what="values"):
    got = np.asarray(got, np.float64)
    want = np.asarray(want, np.float64)
    assert got.shape == want.shape, what
    # non-finite entries (+inf, -inf, NaN) must match exactly
    fin = np.isfinite(want)
    np.testing.assert_array_equal(np.isnan(got), np.isnan(want), err_msg=what)
    np.testing.assert_array_equal(got[~fin & ~np.isnan(want)], want[~fin & ~np.isnan(want)],
                                  err_msg=what)
    err = np.abs(got[fin] - want[fin])
    tol = rel * np.maximum(np.abs(want[fin]), np.abs(got[fin]))
    bad = err > tol
    assert not bad.any(), f"{what}: {bad.sum()} of {bad.size} outside {rel} relative, worst " \
                          f"{(err / np.maximum(np.abs(want[fin]), 1e-300)).max():.3e}"


def search_of(seg_off):
    """Search index of every candidate."""
    seg_off = np.asarray(seg_off)
    return np.repeat(np.arange(len(seg_off) - 1), np.diff(seg_off))


def compare_step(b, gpu, ora, what=""):
    """Strict single-step parity: assignments equal on every candidate the
    oracle did not flag as a near-tie, counts equal in searches without flagged
    candidates, centroids and objective within tolerance.  Returns the number of
    flagged candidates on which the two differ (allowed, reported)."""
    diff = gpu["assign"] != ora.assign
    unflagged_bad = diff & (ora.flag == 0)
    assert not unflagged_bad.any(), f"{what}: {unflagged_bad.sum()} unflagged assignments differ"
    sid = search_of(b.seg_off)
    flagged_searches = np.unique(sid[ora.flag != 0])
    diverged = np.unique(sid[diff])
    clean_k = np.ones(b.Ksum, bool)
    for g in flagged_searches:
        clean_k[b.koff[g]:b.koff[g + 1]] = False
    np.testing.assert_array_equal(gpu["counts"][clean_k], ora.counts[clean_k], err_msg=what)
    same_k = np.ones(b.Ksum, bool)
    for g in diverged:
        same_k[b.koff[g]:b.koff[g + 1]] = False
    assert_cent_close(gpu["cent"][same_k], ora.cent[same_k], what + " centroids")
    nonempty = np.diff(b.seg_off) > 0
    assert_rel_close(gpu["objective"][nonempty], ora.objective[nonempty], what=what + " objective")
    return int(diff.sum())
