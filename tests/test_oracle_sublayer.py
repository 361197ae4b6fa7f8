"""Pins for the oracle's sub-layer wiring (Fig. 2(b); Sec. 3.3, implementation
paragraph: a selection / restoration pair around the attention layer and
another around the FFN layer).

The two half-layers are pinned against torch-CPU library routines written
independently here, against special cases with known answers, and against the
whole block (already pinned on its own): with the same kept set and no
restoration in between they compose to it.  The step is pinned by the cases in
which its result is known without running it: everything kept (the dense block,
whatever the caches hold), nothing kept (the upsampled FFN cache), kept slots
carrying the layer outputs unchanged.
"""
import numpy as np
import torch
import torch.nn.functional as TF

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import synth
from test_oracle_block_restore import DIMS, _rand_weights


def _t(a):
    return torch.from_numpy(np.asarray(a, np.float64))


def test_ffn_sublayer_matches_torch_library_routines():
    rng = np.random.default_rng(3)
    W = _rand_weights(4)
    x = rng.standard_normal((2, 9, DIMS.D))
    a = TF.layer_norm(_t(x), (DIMS.D,), _t(W["ln2_g"]), _t(W["ln2_b"]), 1e-6)
    ref = _t(x) + TF.linear(TF.gelu(TF.linear(a, _t(W["w_fc1"]), _t(W["b_fc1"]))), _t(W["w_fc2"]), _t(W["b_fc2"]))
    np.testing.assert_allclose(O.ffn_sublayer_pruned(x, W, 1e-6), ref.numpy(), rtol=1e-11, atol=1e-11)


def test_attention_sublayer_matches_torch_library_routines():
    rng = np.random.default_rng(5)
    W = _rand_weights(6)
    B, k, L0, D, H, dh = 2, 7, 5, DIMS.D, DIMS.H, DIMS.dh
    x = rng.standard_normal((B, k, D))
    kc = rng.standard_normal((B, L0, H, dh))
    vc = rng.standard_normal((B, L0, H, dh))
    a = TF.layer_norm(_t(x), (D,), _t(W["ln1_g"]), _t(W["ln1_b"]), 1e-6)
    q, kn, vn = TF.linear(a, _t(W["w_qkv"]), _t(W["b_qkv"])).split(D, dim=-1)
    hd = lambda z: z.reshape(B, k, H, dh)
    K = torch.cat([_t(kc), hd(kn)], dim=1).transpose(1, 2)
    V = torch.cat([_t(vc), hd(vn)], dim=1).transpose(1, 2)
    o = TF.scaled_dot_product_attention(hd(q).transpose(1, 2), K, V).transpose(1, 2).reshape(B, k, D)
    ref = _t(x) + TF.linear(o, _t(W["w_proj"]), _t(W["b_proj"]))
    h, k_new, v_new = O.attention_sublayer_pruned(x, W, H, kc, vc, 1e-6)
    np.testing.assert_allclose(h, ref.numpy(), rtol=1e-10, atol=1e-10)
    np.testing.assert_allclose(k_new, hd(kn).numpy(), rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(v_new, hd(vn).numpy(), rtol=1e-12, atol=1e-12)


def test_half_layers_special_cases():
    rng = np.random.default_rng(7)
    W = _rand_weights(8)
    x = rng.standard_normal((1, 6, DIMS.D))
    kc = rng.standard_normal((1, 4, DIMS.H, DIMS.dh))
    vc = rng.standard_normal((1, 4, DIMS.H, DIMS.dh))
    # zero output projections: each half returns its input plus the output bias (the residual path)
    Wz = dict(W, w_proj=np.zeros_like(W["w_proj"]), w_fc2=np.zeros_like(W["w_fc2"]))
    h, _, _ = O.attention_sublayer_pruned(x, Wz, DIMS.H, kc, vc)
    np.testing.assert_allclose(h, x + W["b_proj"], atol=1e-13)
    np.testing.assert_allclose(O.ffn_sublayer_pruned(x, Wz), x + W["b_fc2"], atol=1e-13)
    # the FFN half is token-wise: a permutation of the tokens permutes the outputs
    perm = rng.permutation(6)
    np.testing.assert_allclose(O.ffn_sublayer_pruned(x[:, perm], W), O.ffn_sublayer_pruned(x, W)[:, perm],
                               atol=1e-13)
    # the attention half uses LN1, the FFN half LN2: swapping the two parameter sets changes both
    Ws = dict(W, ln1_g=W["ln2_g"], ln1_b=W["ln2_b"], ln2_g=W["ln1_g"], ln2_b=W["ln1_b"])
    assert np.abs(O.ffn_sublayer_pruned(x, Ws) - O.ffn_sublayer_pruned(x, W)).max() > 1e-3
    assert np.abs(O.attention_sublayer_pruned(x, Ws, DIMS.H, kc, vc)[0] - h).max() > 1e-3


def test_half_layers_compose_to_the_block():
    rng = np.random.default_rng(9)
    W = _rand_weights(10)
    B, k, L0 = 2, 8, 6
    xk = rng.standard_normal((B, k, DIMS.D))
    kc = rng.standard_normal((B, L0, DIMS.H, DIMS.dh))
    vc = rng.standard_normal((B, L0, DIMS.H, DIMS.dh))
    y, kn, vn = O.block_forward_pruned(xk, W, DIMS.H, kc, vc)
    h, kn2, vn2 = O.attention_sublayer_pruned(xk, W, DIMS.H, kc, vc)
    np.testing.assert_allclose(O.ffn_sublayer_pruned(h, W), y, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(kn, kn2)
    np.testing.assert_array_equal(vn, vn2)


def _step_inputs(seed, h=6, w=5, hc=3, wc=3, L0=9, B=2):
    rng = np.random.default_rng(seed)
    N = h * w
    x = rng.standard_normal((B, N, DIMS.D))
    kc = rng.standard_normal((B, L0, DIMS.H, DIMS.dh))
    vc = rng.standard_normal((B, L0, DIMS.H, DIMS.dh))
    ca = rng.standard_normal((B, hc * wc, DIMS.D))
    cf = rng.standard_normal((B, hc * wc, DIMS.D))
    return x, kc, vc, ca, cf, (h, w, hc, wc, N)


def test_step_sublayer_everything_kept_is_the_dense_block():
    W = _rand_weights(11)
    x, kc, vc, ca, cf, (h, w, hc, wc, N) = _step_inputs(12)
    r = O.step_sublayer(x, h, w, N, N, W, DIMS.H, kc, vc, ca, cf, hc, wc)
    dense, kn, vn = O.block_forward_pruned(x, W, DIMS.H, kc, vc)
    np.testing.assert_allclose(r["y"], dense, rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(r["idx_attn"], np.tile(np.arange(N), (2, 1)))
    np.testing.assert_array_equal(r["idx_ffn"], np.tile(np.arange(N), (2, 1)))
    np.testing.assert_allclose(r["k_new"], kn, atol=1e-13)


def test_step_sublayer_nothing_kept_is_the_upsampled_ffn_cache():
    W = _rand_weights(13)
    x, kc, vc, ca, cf, (h, w, hc, wc, N) = _step_inputs(14)
    r = O.step_sublayer(x, h, w, 0, 0, W, DIMS.H, kc, vc, ca, cf, hc, wc)
    np.testing.assert_array_equal(r["y"], O.upsample_bilinear(cf, hc, wc, h, w))
    np.testing.assert_array_equal(r["x_mid"], O.upsample_bilinear(ca, hc, wc, h, w))
    assert r["k_new"].shape[1] == 0


def test_step_sublayer_slots_and_second_selection():
    W = _rand_weights(15)
    x, kc, vc, ca, cf, (h, w, hc, wc, N) = _step_inputs(16)
    ka, kf = 13, 8
    r = O.step_sublayer(x, h, w, ka, kf, W, DIMS.H, kc, vc, ca, cf, hc, wc)
    up_a, up_f = O.upsample_bilinear(ca, hc, wc, h, w), O.upsample_bilinear(cf, hc, wc, h, w)
    for b in range(2):
        ia, jf = r["idx_attn"][b], r["idx_ffn"][b]
        # the first selection is taken on x, the second on the restored map between the halves
        np.testing.assert_array_equal(ia, O.select_pivotal(x[b:b + 1], ka)[0][0])
        np.testing.assert_array_equal(jf, O.select_pivotal(r["x_mid"][b:b + 1], kf)[0][0])
        # kept slots carry the layer outputs, the others the upsampled cache of the same layer
        np.testing.assert_array_equal(r["x_mid"][b, ia], r["hk"][b])
        np.testing.assert_array_equal(r["y"][b, jf], r["yk"][b])
        rest_a = np.setdiff1d(np.arange(N), ia)
        rest_f = np.setdiff1d(np.arange(N), jf)
        np.testing.assert_array_equal(r["x_mid"][b, rest_a], up_a[b, rest_a])
        np.testing.assert_array_equal(r["y"][b, rest_f], up_f[b, rest_f])
    # the FFN half reads the restored map: kept outputs equal the FFN layer on its gathered rows
    yk = O.ffn_sublayer_pruned(O.gather_tokens(r["x_mid"], r["idx_ffn"]), W)
    np.testing.assert_allclose(r["yk"], yk, atol=1e-13)
    # only the attention half's kept tokens enter the cache
    assert r["k_new"].shape[1] == ka
    # a map handed in for the middle replaces the oracle's own (used when checking a device run)
    r2 = O.step_sublayer(x, h, w, ka, kf, W, DIMS.H, kc, vc, ca, cf, hc, wc, x_mid=r["x_mid"] + 0.0)
    np.testing.assert_array_equal(r2["y"], r["y"])
