"""Pins of the oracle's two "next row" functions: class draws from the prior / mixture sampling (Eq. 5) and the
one-way ANOVA F-statistic per channel (Section 4).  CPU only."""
import numpy as np
import pytest
from scipy import stats

import oracle as O
from paper_2102_10485_amd import synth


# ---- class draws -----------------------------------------------------------------------------------------

def test_draw_labels_matches_searchsorted_on_the_cumulative_prior():
    rng = np.random.default_rng(1)
    for K in (2, 10, 100, 1000):
        prior = rng.random(K) + 0.01
        u = rng.random(5000).astype(np.float32)
        rc, lab = O.draw_labels(prior, u)
        assert rc == 0
        cdf = np.cumsum(prior / prior.sum())            # same running sums, same order
        want = np.minimum(np.searchsorted(cdf, u.astype(np.float64), side="right"), K - 1)
        np.testing.assert_array_equal(lab, want)


def test_draw_labels_boundaries_and_zero_probability_classes():
    # exact binary fractions: the cumulative values are 0.25, 0.25, 0.75, 1.0
    prior = [0.25, 0.0, 0.5, 0.25]
    u = np.array([0.0, 0.2499999, 0.25, 0.5, 0.7499999, 0.75, 0.9999999], np.float32)
    rc, lab = O.draw_labels(prior, u)
    assert rc == 0
    np.testing.assert_array_equal(lab, [0, 0, 2, 2, 2, 3, 3])          # u equal to a cumulative value goes to the next class
    rc, lab = O.draw_labels([0.0, 0.0, 1.0, 0.0], np.array([0.0, 0.5, 0.9999999], np.float32))
    np.testing.assert_array_equal(lab, [2, 2, 2])                       # classes of probability zero are never drawn
    rc, lab = O.draw_labels([3.0, 1.0], np.array([0.74, 0.76], np.float32))   # unnormalised prior
    np.testing.assert_array_equal(lab, [0, 1])


def test_draw_labels_rejects_bad_priors():
    u = np.zeros(4, np.float32)
    assert O.draw_labels([0.0, 0.0], u)[0] == -1
    assert O.draw_labels([0.5, -0.1, 0.6], u)[0] == -1


def test_draw_labels_frequencies_follow_the_prior():
    rng = np.random.default_rng(2)
    prior = np.array([0.05, 0.15, 0.3, 0.5])
    n = 200000
    rc, lab = O.draw_labels(prior, rng.random(n).astype(np.float32))
    freq = np.bincount(lab, minlength=4) / n
    sigma = np.sqrt(prior * (1 - prior) / n)
    assert np.all(np.abs(freq - prior) < 5 * sigma)


def test_sample_is_the_per_label_generator_applied_to_the_drawn_labels():
    spec = synth.SPECS["tiny"]
    K = 3
    orc = O.Oracle(spec, K, K)
    rng = np.random.default_rng(3)
    n = 12
    z = rng.normal(size=(n, spec["z_dim"]))
    u = rng.random(n).astype(np.float32)
    prior = [0.2, 0.5, 0.3]
    rc, img, lab = orc.sample(prior, u, z, use_running_stats=1)
    assert rc == 0
    np.testing.assert_array_equal(lab, O.draw_labels(prior, u)[1])
    # every image equals what its label's generator alone makes of its noise row (running statistics: rows independent)
    for k in range(K):
        rows = np.where(lab == k)[0]
        if rows.size == 0:
            continue
        rc2, alone = orc.generate(np.full(rows.size, k, np.int32), z[rows], use_running_stats=1)
        np.testing.assert_allclose(img[rows], alone, rtol=0, atol=1e-13)
    # a prior concentrated on one label uses only that label's generator
    rc, img1, lab1 = orc.sample([0.0, 0.0, 1.0], u, z, use_running_stats=1)
    assert np.all(lab1 == 2)
    rc2, alone = orc.generate(np.full(n, 2, np.int32), z, use_running_stats=1)
    np.testing.assert_allclose(img1, alone, rtol=0, atol=1e-13)
    orc.close()


# ---- ANOVA ------------------------------------------------------------------------------------------------

def _const_images(values, C=1, hw=4):
    """One constant image per value."""
    v = np.asarray(values, np.float32)
    return np.broadcast_to(v[:, None, None, None], (v.size, C, hw, hw)).copy()


def test_anova_worked_example():
    # groups {1,2,3}, {2,3,4}, {5,6,7}: means 2, 3, 6, grand mean 11/3; SSB = 3 (25/9 + 4/9 + 49/9) = 26, df 2;
    # SSW = 2 + 2 + 2 = 6, df 6; F = 13
    lab = np.array([0, 0, 0, 1, 1, 1, 2, 2, 2], np.int32)
    rc, F = O.anova_f(lab, _const_images([1, 2, 3, 2, 3, 4, 5, 6, 7]), 3)
    assert rc == 0
    np.testing.assert_allclose(F, [13.0], rtol=1e-12)


def test_anova_matches_library_routine_and_two_group_t_test():
    rng = np.random.default_rng(4)
    n, K, C = 600, 7, 3
    lab = rng.integers(0, K, n).astype(np.int32)
    img = (rng.normal(size=(n, C, 6, 6)) + 0.2 * lab[:, None, None, None] * np.array([1.0, 0.3, 0.0])[None, :, None, None]).astype(np.float32)
    rc, F = O.anova_f(lab, img, K)
    assert rc == 0
    x = img.astype(np.float64).mean(axis=(2, 3))
    want = [stats.f_oneway(*[x[lab == k, c] for k in range(K)]).statistic for c in range(C)]
    np.testing.assert_allclose(F, want, rtol=1e-6)
    # two groups: F is the square of the pooled-variance t statistic
    lab2 = (lab % 2).astype(np.int32)
    rc, F2 = O.anova_f(lab2, img, 2)
    t = [stats.ttest_ind(x[lab2 == 0, c], x[lab2 == 1, c], equal_var=True).statistic for c in range(C)]
    np.testing.assert_allclose(F2, np.square(t), rtol=1e-8)


def test_anova_invariances_and_degenerate_cases():
    rng = np.random.default_rng(5)
    n, K = 300, 5
    lab = rng.integers(0, K, n).astype(np.int32)
    img = rng.normal(size=(n, 2, 4, 4)) * 0.25 + 0.125 * lab[:, None, None, None]
    img = (np.round(img * 1024.0) / 1024.0).astype(np.float32)      # few mantissa bits: 4 x + 2 is exact in fp32
    rc, F = O.anova_f(lab, img, K)
    rc, Fs = O.anova_f(lab, img * 4.0 + 2.0, K)                 # exact in binary: affine maps leave F unchanged
    np.testing.assert_allclose(Fs, F, rtol=1e-9)
    # the same images under every label: no between-class variation
    base = rng.normal(size=(20, 1, 4, 4)).astype(np.float32)
    rc, F0 = O.anova_f(np.repeat(np.arange(3), 20).astype(np.int32), np.tile(base, (3, 1, 1, 1)), 3)
    assert rc == 0 and abs(F0[0]) < 1e-20
    # samples with labels outside [0, n_labels) are ignored
    lab_bad = np.concatenate([lab, np.array([-1, K, 99], np.int32)])
    img_bad = np.concatenate([img, 100.0 * np.ones((3, 2, 4, 4), np.float32)])
    rc, Fb = O.anova_f(lab_bad, img_bad, K)
    np.testing.assert_allclose(Fb, F, rtol=1e-12)
    # fewer than two classes present: no statistic
    assert O.anova_f(np.zeros(10, np.int32), img[:10], K)[0] == -1


def test_anova_of_the_synthetic_workloads_is_large():
    """The stand-in images carry a per-label offset, so their F is far above 1 - the property the paper reports for
    its datasets (F between 22 and 400)."""
    work = synth.Workload(1)
    lab = work.labels()
    rc, F = O.anova_f(lab, work.images(lab), work.n_labels)
    assert rc == 0 and np.all(F > 10.0)
