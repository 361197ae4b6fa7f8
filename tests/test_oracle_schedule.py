"""Pins for the oracle's stack-level scale step (Fig. 2(a); Sec. 3.3, overview): structure steps run
every block unpruned and capture the per-block outputs at the cached step, texture steps run
selection / block / restoration per block from that block's own cached map.

It is a composition of parts that are pinned on their own, so the pins here are about the wiring:
what feeds what, which cache grows by how much, which map is captured.
"""
import numpy as np

from oracle import fastvar_oracle as O
from test_oracle_block_restore import DIMS, _rand_weights


def _setup(seed, n_layers=3, B=2, h=5, w=4, hc=2, wc=3, L0=7):
    rng = np.random.default_rng(seed)
    Ws = [_rand_weights(seed * 10 + l) for l in range(n_layers)]
    x = rng.standard_normal((B, h * w, DIMS.D))
    kc = [rng.standard_normal((B, L0, DIMS.H, DIMS.dh)) for _ in Ws]
    vc = [rng.standard_normal((B, L0, DIMS.H, DIMS.dh)) for _ in Ws]
    cm = [rng.standard_normal((B, hc * wc, DIMS.D)) for _ in Ws]
    return Ws, x, kc, vc, cm, (h, w, hc, wc, L0)


def test_texture_step_is_the_chain_of_single_block_steps():
    Ws, x, kc, vc, cm, (h, w, hc, wc, L0) = _setup(1)
    k = 9
    r = O.scale_step(x, h, w, k, Ws, DIMS.H, kc, vc, cm, hc, wc, structure=False)
    cur = x
    for l, W in enumerate(Ws):
        s = O.step(cur, h, w, k, W, DIMS.H, kc[l], vc[l], cm[l], hc, wc)
        # each block restores from its OWN cached map and appends only its kept tokens' K/V
        np.testing.assert_array_equal(r["k_caches"][l][:, :L0], kc[l])
        np.testing.assert_array_equal(r["k_caches"][l][:, L0:], s["k_new"])
        np.testing.assert_array_equal(r["v_caches"][l][:, L0:], s["v_new"])
        assert r["k_caches"][l].shape[1] == L0 + k
        cur = s["y"]
    np.testing.assert_array_equal(r["y"], cur)
    np.testing.assert_array_equal(r["idx"], s["idx"])
    assert r["captured"] is None


def test_structure_step_is_the_dense_stack_and_captures_every_block():
    Ws, x, kc, vc, cm, (h, w, hc, wc, L0) = _setup(2)
    N = h * w
    r = O.scale_step(x, h, w, N, Ws, DIMS.H, kc, vc, None, 0, 0, structure=True, capture=True)
    cur = x
    for l, W in enumerate(Ws):
        cur, kn, vn = O.block_forward_pruned(cur, W, DIMS.H, kc[l], vc[l])
        np.testing.assert_array_equal(r["captured"][l], cur)
        assert r["k_caches"][l].shape[1] == L0 + N
        np.testing.assert_array_equal(r["k_caches"][l][:, L0:], kn)
    np.testing.assert_array_equal(r["y"], cur)
    assert r["idx"] is None
    # a texture step that keeps everything gives the same maps: restoration has nothing to fill
    t = O.scale_step(x, h, w, N, Ws, DIMS.H, kc, vc, cm, hc, wc, structure=False)
    np.testing.assert_allclose(t["y"], r["y"], rtol=1e-12, atol=1e-12)


def test_skipped_step_leaves_the_last_blocks_upsampled_cache_and_no_new_keys():
    Ws, x, kc, vc, cm, (h, w, hc, wc, L0) = _setup(3)
    r = O.scale_step(x, h, w, 0, Ws, DIMS.H, kc, vc, cm, hc, wc, structure=False)
    np.testing.assert_array_equal(r["y"], O.upsample_bilinear(cm[-1], hc, wc, h, w))
    assert all(c.shape[1] == L0 for c in r["k_caches"])


def test_captured_maps_feed_the_next_texture_step():
    """Two steps of a schedule: capture at a 3x3 structure step, prune at the 5x5 step after it."""
    Ws, _, kc, vc, _, _ = _setup(4, n_layers=2, L0=4)
    rng = np.random.default_rng(40)
    x3 = rng.standard_normal((2, 9, DIMS.D))
    x5 = rng.standard_normal((2, 25, DIMS.D))
    a = O.scale_step(x3, 3, 3, 9, Ws, DIMS.H, kc, vc, None, 0, 0, structure=True, capture=True)
    b = O.scale_step(x5, 5, 5, 10, Ws, DIMS.H, a["k_caches"], a["v_caches"], a["captured"], 3, 3, structure=False)
    assert b["k_caches"][0].shape[1] == 4 + 9 + 10
    # pruned slots of the result come from the LAST block's captured map, upsampled 3x3 -> 5x5
    up = O.upsample_bilinear(a["captured"][-1], 3, 3, 5, 5)
    for s in range(2):
        rest = np.setdiff1d(np.arange(25), b["idx"][s])
        np.testing.assert_array_equal(b["y"][s, rest], up[s, rest])
        assert np.abs(b["y"][s, b["idx"][s]] - up[s, b["idx"][s]]).max() > 1e-3


def test_skipped_step_with_an_empty_cache_is_the_upsampled_map():
    # degenerate corner: no kept tokens and no cached keys at all (Sec. 4.1: a 100 % ratio skips the step)
    Ws, x, kc, vc, cm, (h, w, hc, wc, L0) = _setup(5, n_layers=1, L0=0)
    r = O.step(x, h, w, 0, Ws[0], DIMS.H, kc[0], vc[0], cm[0], hc, wc)
    np.testing.assert_array_equal(r["y"], O.upsample_bilinear(cm[0], hc, wc, h, w))
    assert r["k_new"].shape[1] == 0 and r["idx"].shape[1] == 0
