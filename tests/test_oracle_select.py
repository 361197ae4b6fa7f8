"""Pins for the oracle's pivotal token selection (Sec. 3.3, Eq. 4-5, Alg. 1).

None of these re-types the oracle's vectorised formula: they use explicit
Python loops, exhaustive sorts, closed forms and invariants.
"""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def brute_scores(x):
    """Eq. 4-5 as scalar loops over python floats."""
    B, N, D = x.shape
    s = [[0.0] * N for _ in range(B)]
    for b in range(B):
        for n in range(N):
            acc = 0.0
            for c in range(D):
                mean_c = math.fsum(float(x[b, m, c]) for m in range(N)) / N
                d = float(x[b, n, c]) - mean_c
                acc += d * d
            s[b][n] = acc
    return np.array(s)


def brute_topk(scores, k):
    """Exhaustive: sort (score desc, index asc) pairs, take k, return ascending."""
    pairs = sorted(((-float(s), i) for i, s in enumerate(scores)))
    return sorted(i for _, i in pairs[:k])


@pytest.mark.parametrize("shape", [(1, 9, 4), (2, 6, 3), (3, 12, 8)])
def test_scores_match_scalar_loops(shape):
    rng = np.random.default_rng(7)
    x = rng.standard_normal(shape)
    np.testing.assert_allclose(O.pivotal_scores(x), brute_scores(x), rtol=1e-12, atol=1e-14)


def test_dc_component_is_mean_over_positions_not_channels():
    # a map whose channel c is the constant c: mean must be [0,1,2..], scores 0.
    x = np.tile(np.arange(5.0)[None, None, :], (2, 7, 1))
    np.testing.assert_array_equal(O.dc_component(x), np.tile(np.arange(5.0), (2, 1)))
    np.testing.assert_array_equal(O.pivotal_scores(x), np.zeros((2, 7)))


def test_scores_shift_invariant_and_per_sample():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 16, 8))
    s0 = O.pivotal_scores(x)
    shift = rng.standard_normal((2, 1, 8)) * 10
    np.testing.assert_allclose(O.pivotal_scores(x + shift), s0, rtol=1e-10, atol=1e-10)
    # samples are independent: changing sample 1 leaves sample 0 alone
    x2 = x.copy()
    x2[1] *= 3.0
    np.testing.assert_array_equal(O.pivotal_scores(x2)[0], s0[0])


def test_score_sum_equals_N_times_total_variance():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((2, 25, 6)) * 2 + 1
    s = O.pivotal_scores(x)
    for b in range(2):
        want = x.shape[1] * np.var(x[b], axis=0).sum()       # library routine, biased
        assert abs(s[b].sum() - want) <= 1e-10 * want


def test_score_is_squared_norm_not_norm():
    # one token displaced by (3,4) from three tokens at the origin.
    x = np.zeros((1, 4, 2))
    x[0, 0] = [3.0, 4.0]
    # mean = (0.75, 1.0); token0 deviates by (2.25, 3.0); others by (0.75, 1.0)
    s = O.pivotal_scores(x)[0]
    assert s[0] == pytest.approx(2.25 ** 2 + 3.0 ** 2)
    assert s[1] == pytest.approx(0.75 ** 2 + 1.0 ** 2)


def test_constant_map_scores_exactly_zero_for_bf16_inputs():
    x = synth.token_map(5, 2, 16, 16, 64, kind="constant")
    s = O.pivotal_scores(x)
    assert np.all(s == 0.0)
    idx, rank, _ = O.select_pivotal(x, 100)
    np.testing.assert_array_equal(idx, np.tile(np.arange(100, dtype=np.int32), (2, 1)))


@pytest.mark.parametrize("N,k", [(1, 1), (5, 0), (5, 5), (7, 3), (8, 4)])
def test_topk_vs_exhaustive_all_small_tie_patterns(N, k):
    # every score vector over {0,1,2}: covers all tie patterns for tiny N
    for vals in itertools.product([0.0, 1.0, 2.0], repeat=N):
        s = np.array([vals], dtype=np.float32)
        got = O.topk_indices(s, k)[0].tolist()
        assert got == brute_topk(vals, k)


def test_topk_random_vs_exhaustive_and_properties():
    rng = np.random.default_rng(0)
    for trial in range(50):
        N = int(rng.integers(1, 200))
        k = int(rng.integers(0, N + 1))
        # coarse values so ties are common
        s = np.round(rng.standard_normal((2, N)) * 3).astype(np.float32) ** 2
        idx = O.topk_indices(s, k)
        for b in range(2):
            assert idx[b].tolist() == brute_topk(s[b], k)
            assert len(set(idx[b].tolist())) == k
            if 0 < k < N:
                kept = np.zeros(N, bool)
                kept[idx[b]] = True
                assert s[b][kept].min() >= s[b][~kept].max()


def test_select_rank_is_inverse_of_idx():
    x = synth.token_map(1, 2, 8, 8, 32)
    idx, rank, s32 = O.select_pivotal(x, 20)
    assert s32.dtype == np.float32 and idx.dtype == np.int32 and rank.dtype == np.int32
    for b in range(2):
        assert np.all(np.diff(idx[b]) > 0)
        assert (rank[b] >= 0).sum() == 20
        np.testing.assert_array_equal(rank[b, idx[b]], np.arange(20))
    xk = O.gather_tokens(x, idx)
    for b in range(2):
        for j in range(20):
            np.testing.assert_array_equal(xk[b, j], x[b, idx[b, j]])


def test_spiked_positions_are_the_ones_selected():
    # smooth map + large spikes at known places: PTS must pick exactly those.
    rng = np.random.default_rng(2)
    N, D = 64, 16
    x = np.ones((1, N, D)) * 0.5 + rng.standard_normal((1, N, D)) * 1e-3
    spikes = [3, 17, 40, 63]
    x[0, spikes] += 5.0 * rng.choice([-1.0, 1.0], size=(4, D))
    idx, _, _ = O.select_pivotal(x, 4)
    assert idx[0].tolist() == spikes


def test_keep_count_values():
    # the non-integer products the workloads contain
    assert O.keep_count(576, 0.6) == 346
    assert O.keep_count(1024, 0.4) == 410
    assert O.keep_count(4096, 0.4) == 1638
    assert O.keep_count(9216, 0.3) == 2765
    assert O.keep_count(4096, 0.1) == 410
    assert O.keep_count(4096, 0.5) == 2048
    assert O.keep_count(10, 0.0) == 0 and O.keep_count(10, 1.0) == 10
    assert O.keep_count(10, 1.7) == 10 and O.keep_count(10, -0.2) == 0
    for w in synth.WORKLOADS.values():
        assert O.keep_count(w.N, w.keep_ratio) == w.k, w.name


def test_golden_hand_worked_selection():
    """tests/golden/pts_ctr_2x2.txt: Eq. 4-6 evaluated by hand on a 2x2 map."""
    g = _read_golden("pts_ctr_2x2.txt")
    x = np.array(g["x"]).reshape(1, 4, 2)
    np.testing.assert_allclose(O.dc_component(x)[0], g["mean"], rtol=0, atol=1e-15)
    np.testing.assert_allclose(O.pivotal_scores(x)[0], g["score"], rtol=1e-15)
    idx, rank, _ = O.select_pivotal(x, 2)
    assert idx[0].tolist() == [int(v) for v in g["idx_k2"]]
    assert rank[0].tolist() == [int(v) for v in g["rank_k2"]]


def _read_golden(name):
    out = {}
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if not line:
                continue
            key, vals = line.split(":")
            out[key.strip()] = [float(v) for v in vals.split()]
    return out
