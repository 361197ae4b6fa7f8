"""Pins for the oracle's schedule policy (Sec. 3.3 overview, Sec. 4.1) and intermediate prediction
(Sec. 3.1, Eq. 2 and Eq. 3).

The schedule pins are the paper's two settings written out by hand; the Eq. 2 pins are a library
routine (torch-CPU bilinear interpolation plus an add), closed forms (constant maps, equal sizes,
linearity) and the cases in which the unfolded sum of Eq. 3 must agree with the recursion.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as TF

from oracle import fastvar_oracle as O


def test_schedule_of_the_thirteen_step_model_by_hand():
    # Sec. 4.1: N = 4, ratios 40 / 50 / 100 / 100 %; 13 square scales up to 64x64.
    sides = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)
    keep, structure, cached = O.schedule_plan([(s, s) for s in sides], (0.4, 0.5, 1.0, 1.0))
    assert keep[:9] == [1, 4, 16, 36, 64, 144, 256, 400, 576]          # structure stage: every token
    assert keep[9:] == [614, 800, 0, 0]                                # 0.6*1024 = 614.4, 0.5*1600, skipped, skipped
    assert structure == [True] * 9 + [False] * 4
    assert cached == 8                                                 # step K-N = 9, counted from 0; the 24x24 map


def test_schedule_with_two_pruned_steps_by_hand():
    # Sec. 4.1: N = 2, ratios 50 / 75 %; a non-square schedule to catch an h/w mix-up.
    sizes = [(1, 1), (2, 3), (4, 6), (8, 12), (16, 24)]
    keep, structure, cached = O.schedule_plan(sizes, (0.5, 0.75))
    assert keep == [1, 6, 24, 48, 96]
    assert structure == [True, True, True, False, False]
    assert cached == 2


def test_schedule_degenerate_cases():
    sizes = [(1, 1), (2, 2), (3, 3)]
    assert O.schedule_plan(sizes, ()) == ([1, 4, 9], [True] * 3, -1)             # nothing pruned, nothing cached
    keep, structure, cached = O.schedule_plan(sizes, (0.0, 0.5, 1.0))            # every step pruned: no cached step
    assert keep == [1, 2, 0] and structure == [False] * 3 and cached == -1
    assert O.schedule_plan([(5, 5)], (0.5,))[0] == [13]                           # 12.5 rounds half up
    with pytest.raises(AssertionError):
        O.schedule_plan(sizes, (0.1, 0.2, 0.3, 0.4))


def test_residual_accumulate_matches_library_interpolate_plus_add():
    rng = np.random.default_rng(5)
    for (hp, wp, h, w) in [(2, 3, 5, 7), (4, 4, 6, 6), (8, 8, 16, 16), (3, 5, 3, 5), (6, 6, 4, 4)]:
        B, C = 2, 5
        r = rng.standard_normal((B, hp * wp, C))
        f = rng.standard_normal((B, h * w, C))
        t = torch.from_numpy(r).reshape(B, hp, wp, C).permute(0, 3, 1, 2)
        up = TF.interpolate(t, size=(h, w), mode="bilinear", align_corners=False)
        want = up.permute(0, 2, 3, 1).reshape(B, h * w, C).numpy() + f
        np.testing.assert_allclose(O.residual_accumulate(r, hp, wp, f, h, w), want, rtol=0, atol=1e-12)


def test_residual_accumulate_closed_forms():
    rng = np.random.default_rng(6)
    B, C = 2, 3
    f1 = rng.standard_normal((B, 4, C))
    # first step: r_1 = f_1
    np.testing.assert_array_equal(O.residual_accumulate(None, 0, 0, f1, 2, 2), f1)
    # equal sizes: interpolation is the identity, so the step is a plain add
    f2 = rng.standard_normal((B, 4, C))
    np.testing.assert_allclose(O.residual_accumulate(f1, 2, 2, f2, 2, 2), f1 + f2, rtol=0, atol=1e-15)
    # a constant map stays that constant at any size
    c = np.broadcast_to(rng.standard_normal((B, 1, C)), (B, 6, C))
    f3 = rng.standard_normal((B, 35, C))
    np.testing.assert_allclose(O.residual_accumulate(c, 2, 3, f3, 5, 7) - f3, np.broadcast_to(c[:, :1], (B, 35, C)),
                               rtol=0, atol=1e-14)
    # a skipped step (ratio 100 %) is the interpolation alone
    np.testing.assert_array_equal(O.residual_accumulate(f1, 2, 2, None, 4, 4), O.upsample_bilinear(f1, 2, 2, 4, 4))
    # linear in both arguments
    a, b = rng.standard_normal((B, 6, C)), rng.standard_normal((B, 6, C))
    lhs = O.residual_accumulate(2.0 * a - b, 2, 3, 3.0 * f3, 5, 7)
    rhs = 2.0 * O.residual_accumulate(a, 2, 3, 0 * f3, 5, 7) - O.residual_accumulate(b, 2, 3, 0 * f3, 5, 7) + 3.0 * f3
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=1e-13)


def _chain(fs, sizes, skip=()):
    r, prev = None, (0, 0)
    for i, (f, (h, w)) in enumerate(zip(fs, sizes)):
        r = O.residual_accumulate(r, prev[0], prev[1], None if i in skip else f, h, w)
        prev = (h, w)
    return r


def test_recursion_and_unfolded_sum_agree_where_resampling_composes():
    rng = np.random.default_rng(7)
    B, C = 1, 2
    # (a) two steps: one hop each, so Eq. 2 and Eq. 3 are the same expression
    sizes = [(2, 2), (5, 3)]
    fs = [rng.standard_normal((B, h * w, C)) for h, w in sizes]
    np.testing.assert_allclose(_chain(fs, sizes), O.cumulative_prediction(fs, sizes, 2), rtol=0, atol=1e-14)
    # (b) constant residual maps at every scale: every hop preserves constants
    sizes = [(1, 1), (2, 3), (4, 4), (7, 5)]
    consts = rng.standard_normal((len(sizes), C))
    fs = [np.broadcast_to(consts[i], (B, h * w, C)).copy() for i, (h, w) in enumerate(sizes)]
    want = np.broadcast_to(consts.sum(0), (B, 35, C))
    np.testing.assert_allclose(_chain(fs, sizes), want, rtol=0, atol=1e-13)
    np.testing.assert_allclose(O.cumulative_prediction(fs, sizes, 4), want, rtol=0, atol=1e-13)
    # (c) a repeated size is an identity hop
    sizes = [(2, 2), (2, 2), (4, 4)]
    fs = [rng.standard_normal((B, h * w, C)) for h, w in sizes]
    np.testing.assert_allclose(_chain(fs, sizes), O.cumulative_prediction(fs, sizes, 3), rtol=0, atol=1e-14)
    # (d) and in general they differ: two bilinear hops are not one
    sizes = [(2, 2), (3, 3), (8, 8)]
    fs = [rng.standard_normal((B, h * w, C)) for h, w in sizes]
    assert np.abs(_chain(fs, sizes) - O.cumulative_prediction(fs, sizes, 3)).max() > 1e-3


def test_skipped_steps_at_the_end_only_resample_the_last_prediction():
    rng = np.random.default_rng(8)
    sizes = [(2, 2), (4, 4), (6, 6), (8, 8)]
    fs = [rng.standard_normal((1, h * w, 3)) for h, w in sizes]
    r2 = _chain(fs[:2], sizes[:2])
    got = _chain(fs, sizes, skip=(2, 3))
    want = O.upsample_bilinear(O.upsample_bilinear(r2, 4, 4, 6, 6), 6, 6, 8, 8)
    np.testing.assert_allclose(got, want, rtol=0, atol=1e-14)


def test_planted_mistakes_are_caught():
    rng = np.random.default_rng(9)
    r = rng.standard_normal((1, 6, 2))
    f = rng.standard_normal((1, 20, 2))
    good = O.residual_accumulate(r, 2, 3, f, 4, 5)
    t = torch.from_numpy(r).reshape(1, 2, 3, 2).permute(0, 3, 1, 2)
    lib = TF.interpolate(t, size=(4, 5), mode="bilinear", align_corners=False).permute(0, 2, 3, 1).reshape(1, 20, 2).numpy()
    assert np.abs(good - (lib + f)).max() < 1e-12
    assert np.abs(good - lib).max() > 1e-2                      # residual dropped
    assert np.abs(good - (lib - f)).max() > 1e-2                # wrong sign
    swapped = O.upsample_bilinear(r, 3, 2, 4, 5) + f            # h and w of the previous map exchanged
    assert np.abs(good - swapped).max() > 1e-2
