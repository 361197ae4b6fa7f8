"""GPU parity of the block's kernels one at a time (LayerNorm, GEMM epilogues,
QKV GEMM with cache append, attention) against the oracle's matching functions.
Bar: max |gpu - oracle| / max |oracle| <= 2e-2 per output tensor."""
import numpy as np
import pytest
import torch

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth
from gpu_util import DEV, cache_rows, from_dev_bf16, make_caches, max_rel, to_dev_bf16

pytestmark = pytest.mark.gpu
TOL = 2e-2


def rnd(rng, *shape, scale=1.0):
    return synth.round_bf16((rng.standard_normal(shape) * scale).astype(np.float32))


@pytest.mark.parametrize("B,N,k,D", [(1, 16, 5, 64), (2, 63, 20, 200), (1, 256, 128, 1024), (3, 100, 37, 1920),
                                     (1, 64, 9, 2048), (1, 8, 3, 8192)])
def test_layernorm_and_gather(B, N, k, D):
    print(f"[layernorm] B={B} N={N} k={k} D={D}", flush=True)
    rng = np.random.default_rng(D + k)
    x = rnd(rng, B, N, D, scale=2.0) + 0.5
    x = synth.round_bf16(x)
    g, bt = rnd(rng, D) * 0.1 + 1, rnd(rng, D) * 0.1
    g, bt = synth.round_bf16(g.astype(np.float32)), synth.round_bf16(bt.astype(np.float32))
    idx = np.stack([np.sort(rng.permutation(N)[:k]) for _ in range(B)]).astype(np.int32)
    out = torch.full((B, k, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    fb.fastvar_layernorm(to_dev_bf16(x), torch.from_numpy(idx).to(DEV), B, N, k, D, to_dev_bf16(g),
                         to_dev_bf16(bt), 1e-6, out)
    ref = O.layer_norm(O.gather_tokens(x, idx), g, bt, 1e-6)
    assert max_rel(from_dev_bf16(out), ref) <= 2.0 ** -8 * 1.01
    # plain (no gather) on the first k rows of each sample stacked
    flat = np.ascontiguousarray(x[:, :k]).reshape(1, B * k, D)
    out2 = torch.full((1, B * k, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    fb.fastvar_layernorm(to_dev_bf16(flat), None, 1, 0, B * k, D, to_dev_bf16(g), to_dev_bf16(bt), 1e-6, out2)
    assert max_rel(from_dev_bf16(out2), O.layer_norm(flat, g, bt, 1e-6)) <= 2.0 ** -8 * 1.01


GEMM_CASES = [
    # M, N, K  (small tile config unless M/256 * N/256 >= 224)
    (128, 128, 64), (100, 192, 128), (37, 520, 192), (300, 1000, 256), (129, 136, 64),
    (1, 64, 64), (2048, 2048, 512), (1792, 8192, 128), (1800, 8200, 64), (3280, 1920, 192),
]


@pytest.mark.parametrize("M,N,K", GEMM_CASES)
@pytest.mark.parametrize("epi", [fb.EPI_BIAS_RES, fb.EPI_BIAS_GELU])
def test_gemm_epilogues(M, N, K, epi):
    print(f"[gemm] M={M} N={N} K={K} epilogue={epi}", flush=True)
    rng = np.random.default_rng(M * 7 + N * 3 + K + epi)
    A, W = rnd(rng, M, K), rnd(rng, N, K, scale=0.2)
    bias, res = rnd(rng, N), rnd(rng, M, N)
    out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device=DEV)
    fb.fastvar_gemm_bf16(to_dev_bf16(A), to_dev_bf16(W), to_dev_bf16(bias), to_dev_bf16(res), M, N, K, epi, out)
    torch.cuda.synchronize()
    lin = O.linear(A, W, bias)
    ref = lin + res if epi == fb.EPI_BIAS_RES else O.gelu(lin)
    got = from_dev_bf16(out)
    assert not np.isnan(got).any()
    assert max_rel(got, ref) <= 2.0 ** -7, (M, N, K, epi)
    # no bias
    out.fill_(float("nan"))
    fb.fastvar_gemm_bf16(to_dev_bf16(A), to_dev_bf16(W), None, to_dev_bf16(res), M, N, K, epi, out)
    lin = O.linear(A, W, None)
    ref = lin + res if epi == fb.EPI_BIAS_RES else O.gelu(lin)
    assert max_rel(from_dev_bf16(out), ref) <= 2.0 ** -7


def test_gemm_exact_small_integers():
    """Small-integer operands: every product and sum is exact, so the layout must be too."""
    print("[gemm] exact integer check", flush=True)
    rng = np.random.default_rng(0)
    M, N, K = 200, 328, 128
    A = rng.integers(-2, 3, (M, K)).astype(np.float32)
    W = rng.integers(-2, 3, (N, K)).astype(np.float32)
    res = np.zeros((M, N), np.float32)
    out = torch.empty((M, N), dtype=torch.bfloat16, device=DEV)
    fb.fastvar_gemm_bf16(to_dev_bf16(A), to_dev_bf16(W), None, to_dev_bf16(res), M, N, K, fb.EPI_BIAS_RES, out)
    ref = A.astype(np.float64) @ W.astype(np.float64).T
    assert np.abs(ref).max() < 256          # representable in bf16
    np.testing.assert_array_equal(from_dev_bf16(out).astype(np.float64), ref)


@pytest.mark.parametrize("dims,B,k,L0,L_cap", [
    (synth.BlockDims(192, 3, 64, 320), 2, 37, 29, 104),
    (synth.BlockDims(256, 2, 128, 512), 3, 70, 45, 128),
    (synth.D16, 1, 128, 424, 688),
    (synth.INF2B, 1, 300, 0, 304),
    # more tiles than one round of workgroups (the launch walks its tiles itself), ragged last row tiles
    (synth.INF2B, 2, 1500, 100, 1608),
    (synth.D30, 8, 410, 70, 480),
])
def test_qkv_gemm_appends_to_caches(dims, B, k, L0, L_cap):
    print(f"[qkv] D={dims.D} H={dims.H} dh={dims.dh} B={B} k={k} L0={L0}", flush=True)
    rng = np.random.default_rng(k)
    D = dims.D
    a = rnd(rng, B, k, D)
    W, bias = rnd(rng, 3 * D, D, scale=0.05), rnd(rng, 3 * D, scale=0.1)
    kp, vp = synth.kv_prior(1, B, L0, dims.H, dims.dh)
    kc, vc = make_caches(kp, vp, L_cap)
    kc0, vc0 = kc.clone(), vc.clone()
    q = torch.full((B, k, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    fb.fastvar_qkv_gemm(to_dev_bf16(a), to_dev_bf16(W), to_dev_bf16(bias), B, k, d, q, kc, vc, L0, L_cap)
    torch.cuda.synchronize()
    ref = O.linear(a, W, bias)
    assert max_rel(from_dev_bf16(q), ref[..., :D]) <= 2.0 ** -7
    kg, vg = cache_rows(kc, vc, L0, L0 + k)
    assert max_rel(kg, ref[..., D:2 * D].reshape(B, k, dims.H, dims.dh)) <= 2.0 ** -7
    assert max_rel(vg, ref[..., 2 * D:].reshape(B, k, dims.H, dims.dh)) <= 2.0 ** -7
    kb, kb0, vb, vb0 = (t.view(torch.int16) for t in (kc, kc0, vc, vc0))
    assert torch.equal(kb[:, :, :L0], kb0[:, :, :L0]) and torch.equal(kb[:, :, L0 + k:], kb0[:, :, L0 + k:])
    assert torch.equal(vb[..., :L0], vb0[..., :L0]) and torch.equal(vb[..., L0 + k:], vb0[..., L0 + k:])


ATT_CASES = [
    # H, dh, B, k, L, L_cap
    (2, 128, 1, 32, 64, 64), (2, 128, 1, 33, 65, 72), (3, 64, 2, 37, 66, 104), (2, 128, 3, 70, 115, 128),
    (16, 64, 1, 128, 552, 688), (1, 64, 1, 1, 1, 8), (2, 64, 1, 5, 200, 200), (16, 128, 1, 200, 1000, 1000),
    (16, 64, 4, 1024, 1124, 1128),   # two query blocks per wave
    (16, 128, 1, 4096, 300, 304),    # 256-query workgroups of the pipelined kernel, three tiles, ragged
    # 128-query workgroups of the pipelined kernel: exactly / just over three tiles, tails of 1 and 7
    (16, 128, 1, 1024, 384, 384), (16, 128, 1, 1000, 385, 392), (16, 128, 1, 1024, 1001, 1008),
    (16, 128, 2, 520, 1023, 1024),
    (16, 128, 2, 2048, 200, 200),    # 256-query workgroups, four 64-key tiles, the last one shifted
    # head dim 64 with 256-query workgroups of the pipelined kernel (eight groups per step instead of
    # sixteen; chosen from 1024 keys on, where 256-query tiles pad no further than 128-query ones):
    # whole tiles, tails of 1 and 7 keys, ragged query counts
    (16, 64, 8, 256, 1024, 1024), (16, 64, 4, 410, 1025, 1032), (16, 64, 2, 1000, 1031, 1032),
    (30, 64, 8, 410, 1626, 1632),    # the 512 px model's 32x32 step at full size
    # head dim 64, same shapes just outside that rule: the plain kernel
    (16, 64, 2, 520, 1023, 1024), (16, 64, 4, 346, 1025, 1032), (16, 64, 1, 4096, 300, 304),
]


@pytest.mark.parametrize("H,dh,B,k,L,L_cap", ATT_CASES)
def test_attention_matches_oracle(H, dh, B, k, L, L_cap):
    print(f"[attention] H={H} dh={dh} B={B} k={k} L={L} L_cap={L_cap}", flush=True)
    rng = np.random.default_rng(H * dh + k + L)
    D = H * dh
    q = rnd(rng, B, k, H, dh)
    K, V = rnd(rng, B, L, H, dh), rnd(rng, B, L, H, dh)
    kc, vc = make_caches(K, V, L_cap)
    o = torch.full((B, k, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    d = fb.make_dims(D, H, dh, 64 * ((4 * D) // 64))
    fb.fastvar_attention(to_dev_bf16(q.reshape(B, k, D)), kc, vc, B, k, d, L, L_cap, o)
    torch.cuda.synchronize()
    got = from_dev_bf16(o).reshape(B, k, H, dh)
    assert not np.isnan(got).any()
    for b in range(B):
        ref = O.attention(q[b].astype(np.float64), K[b].astype(np.float64), V[b].astype(np.float64), dh ** -0.5)
        assert max_rel(got[b], ref) <= TOL, (b,)


@pytest.mark.parametrize("dh,k,L", [(128, 1024, 900), (64, 2048, 1100)])
def test_attention_scores_rising_far_above_the_first_tile(dh, k, L):
    """Keys late in the sequence score hundreds of octaves above the first tile's maximum: the
    pipelined kernel's fixed softmax reference overflows and it must fall back to the running maximum."""
    print(f"[attention] rising scores dh={dh} k={k} L={L}", flush=True)
    H, B = 16, 1
    D = H * dh
    rng = np.random.default_rng(11)
    q = rnd(rng, B, k, H, dh)
    K, V = rnd(rng, B, L, H, dh), rnd(rng, B, L, H, dh)
    K[:, 600:] *= 64.0          # a power of two keeps the values bf16; scores reach several hundred
    L_cap = (L + 7) // 8 * 8
    kc, vc = make_caches(K, V, L_cap)
    o = torch.full((B, k, D), float("nan"), dtype=torch.bfloat16, device=DEV)
    d = fb.make_dims(D, H, dh, 4 * D)
    fb.fastvar_attention(to_dev_bf16(q.reshape(B, k, D)), kc, vc, B, k, d, L, L_cap, o)
    got = from_dev_bf16(o).reshape(B, k, H, dh)
    assert not np.isnan(got).any()
    ref = O.attention(q[0].astype(np.float64), K[0].astype(np.float64), V[0].astype(np.float64), dh ** -0.5)
    assert max_rel(got[0], ref) <= TOL


def test_attention_peaked_and_uniform_rows():
    """One-hot attention (huge logit on one key) returns that key's value; equal keys return the mean."""
    print("[attention] peaked / uniform", flush=True)
    H, dh, B, k, L = 2, 64, 1, 40, 150
    D = H * dh
    rng = np.random.default_rng(3)
    K = np.zeros((B, L, H, dh), np.float32)
    V = rnd(rng, B, L, H, dh)
    q = np.zeros((B, k, H, dh), np.float32)
    tgt = rng.integers(0, L, size=k)
    for j in range(L):
        K[0, j, :, j % dh] = 8.0 + (j // dh)      # distinct (direction, length) per key
    for i in range(k):
        q[0, i, :, tgt[i] % dh] = 16.0
    kc, vc = make_caches(K, V, 152)
    o = torch.empty((B, k, D), dtype=torch.bfloat16, device=DEV)
    d = fb.make_dims(D, H, dh, 256, softmax_scale=1.0)
    fb.fastvar_attention(to_dev_bf16(q.reshape(B, k, D)), kc, vc, B, k, d, L, 152, o)
    ref = O.attention(q[0].astype(np.float64), K[0].astype(np.float64), V[0].astype(np.float64), 1.0)
    assert max_rel(from_dev_bf16(o).reshape(k, H, dh), ref) <= TOL
    # uniform: all keys equal -> mean of V
    K[:] = 0.25
    kc, vc = make_caches(K, V, 152)
    fb.fastvar_attention(to_dev_bf16(q.reshape(B, k, D)), kc, vc, B, k, d, L, 152, o)
    want = np.tile(V[0].astype(np.float64).mean(axis=0)[None], (k, 1, 1))
    assert np.max(np.abs(from_dev_bf16(o).reshape(k, H, dh) - want)) <= 2e-2 * np.max(np.abs(want)) + 1e-3
