"""Pins of the oracle's axial 2-D rotary embedding (the positional term of the backbones Sec. 4.1 names;
the paper prints no formula, so the pins are the properties that define a rotary embedding): identity at
the origin, a plain plane rotation per pair, norm preservation, composition of angles, dependence of q.k
on the position difference only (per axis), the frequency ladder, and its place in the block."""
import math

import numpy as np

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import synth


def test_angles_origin_axes_and_frequency_ladder():
    h, w, dh, base = 5, 7, 16, 100.0
    a = O.rope2d_angles(h, w, dh, base)
    assert a.shape == (h * w, dh // 2)
    assert np.all(a[0] == 0.0)                                   # token (0, 0): no rotation
    q = dh // 4
    for i in range(h):
        for j in range(w):
            n = i * w + j
            for t in range(q):                                   # written out, not vectorised
                assert a[n, t] == i * base ** (-(t / q))         # row half
                assert a[n, q + t] == j * base ** (-(t / q))     # column half
    # first pair of each half turns by the coordinate itself
    assert a[3 * w + 2, 0] == 3.0 and a[3 * w + 2, q] == 2.0
    # a column step leaves the row half alone and vice versa
    assert np.array_equal(a[2 * w + 1, :q], a[2 * w + 6, :q])
    assert np.array_equal(a[1 * w + 4, q:], a[4 * w + 4, q:])


def test_angles_on_a_reference_grid():
    # a 4x4 map laid over an 8x8 reference: coordinates 0, 2, 4, 6
    a = O.rope2d_angles(4, 4, 8, 10000.0, ref_h=8, ref_w=8)
    b = O.rope2d_angles(8, 8, 8, 10000.0)
    for i in range(4):
        for j in range(4):
            assert np.allclose(a[i * 4 + j], b[(2 * i) * 8 + 2 * j], rtol=0, atol=0)


def test_rotation_of_a_unit_pair_and_layout():
    # one head of 4 dims = two pairs; pair 0 turned by 0.3, pair 1 by -1.1
    v = np.zeros((1, 1, 4))
    v[0, 0] = [1.0, 0.0, 0.0, 2.0]
    ang = np.array([[0.3, -1.1]])
    r = O.apply_rope(v, ang)[0, 0]
    want = [math.cos(0.3), math.sin(0.3), -2.0 * math.sin(-1.1), 2.0 * math.cos(-1.1)]
    assert np.allclose(r, want, rtol=0, atol=1e-15)
    # the same angles for every head
    v2 = np.random.default_rng(0).standard_normal((3, 2, 4))
    r2 = O.apply_rope(v2, np.tile(ang, (3, 1)))
    assert np.allclose(r2[:, 0], O.apply_rope(v2[:, :1], np.tile(ang, (3, 1)))[:, 0])
    assert np.allclose(r2[:, 1], O.apply_rope(v2[:, 1:], np.tile(ang, (3, 1)))[:, 0])


def test_identity_norm_and_composition():
    rng = np.random.default_rng(1)
    v = rng.standard_normal((6, 3, 16))
    a = rng.uniform(-4, 4, (6, 8))
    b = rng.uniform(-4, 4, (6, 8))
    assert np.array_equal(O.apply_rope(v, np.zeros((6, 8))), v)
    r = O.apply_rope(v, a)
    # every pair keeps its length, hence every vector
    assert np.allclose(r[..., 0::2] ** 2 + r[..., 1::2] ** 2, v[..., 0::2] ** 2 + v[..., 1::2] ** 2, atol=1e-12)
    assert np.allclose(O.apply_rope(r, b), O.apply_rope(v, a + b), atol=1e-12)
    assert np.allclose(O.apply_rope(r, -a), v, atol=1e-12)


def test_scores_depend_on_the_position_difference_only():
    """q at (i1, j1), k at (i2, j2): the dot product after rotation equals the one at
    (i1 + s, j1 + t), (i2 + s, j2 + t) for any shift, and changes when only one of them moves."""
    h = w = 12
    dh = 32
    ang = O.rope2d_angles(h, w, dh, 50.0)
    rng = np.random.default_rng(2)
    q = rng.standard_normal((1, 1, dh))
    k = rng.standard_normal((1, 1, dh))

    def score(pq, pk):
        nq, nk = pq[0] * w + pq[1], pk[0] * w + pk[1]
        return float(np.sum(O.apply_rope(q, ang[nq:nq + 1]) * O.apply_rope(k, ang[nk:nk + 1])))

    s0 = score((2, 3), (5, 1))
    for s, t in [(1, 0), (0, 4), (3, 5), (6, 7)]:
        assert abs(score((2 + s, 3 + t), (5 + s, 1 + t)) - s0) < 1e-11
    assert abs(score((3, 3), (5, 1)) - s0) > 1e-3
    assert abs(score((2, 3), (5, 2)) - s0) > 1e-3
    # equal positions: the plain dot product
    assert abs(score((4, 9), (4, 9)) - float(np.sum(q * k))) < 1e-12


def test_block_with_rope_places_it_on_q_and_new_keys_only():
    dims = synth.BlockDims(D=32, H=2, dh=16, F=64)
    B, h, w, k, L0 = 2, 4, 5, 7, 6
    x = synth.token_map(3, B, h, w, dims.D)
    W = synth.block_weights(3, dims)
    kp, vp = synth.kv_prior(3, B, L0, dims.H, dims.dh)
    idx, _, _ = O.select_pivotal(x, k)
    xk = O.gather_tokens(x, idx)
    ang = O.rope2d_angles(h, w, dims.dh, 100.0)
    rope = np.stack([ang[idx[b]] for b in range(B)])            # gathered like the tokens
    y1, k1, v1, p1 = O.block_forward_pruned(xk, W, dims.H, kp, vp, rope=rope, return_parts=True)
    y0, k0, v0, p0 = O.block_forward_pruned(xk, W, dims.H, kp, vp, return_parts=True)
    assert np.array_equal(v1, v0)                                # values are not turned
    assert np.allclose(k1, O.apply_rope(k0, rope), atol=1e-12)   # appended keys are the turned ones
    assert np.allclose(p1["q"], O.apply_rope(p0["q"], rope), atol=1e-12)
    assert not np.allclose(y1, y0)
    # independent evaluation of one output row: attention written out for token 0 of sample 0
    b, m = 0, 0
    Kall = np.concatenate([kp[b].astype(np.float64), k1[b]], axis=0)
    Vall = np.concatenate([vp[b].astype(np.float64), v1[b]], axis=0)
    o = np.zeros(dims.D)
    for hd in range(dims.H):
        sc = np.array([np.dot(p1["q"][b, m, hd], Kall[l, hd]) for l in range(Kall.shape[0])]) / math.sqrt(dims.dh)
        pr = np.exp(sc - sc.max())
        pr /= pr.sum()
        o[hd * dims.dh:(hd + 1) * dims.dh] = pr @ Vall[:, hd]
    assert np.allclose(p1["o"][b, m], o, atol=1e-12)
    # with every kept token at one common position and no earlier keys, rotation cancels in q.k
    same = np.tile(ang[7:8], (B, k, 1))
    e = np.zeros((B, 0, dims.H, dims.dh))
    ya, _, _ = O.block_forward_pruned(xk, W, dims.H, e, e, rope=same)
    yb, _, _ = O.block_forward_pruned(xk, W, dims.H, e, e)
    assert np.allclose(ya, yb, atol=1e-10)
