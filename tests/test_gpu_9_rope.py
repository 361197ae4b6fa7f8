"""GPU parity: rotary positions gathered by the kept index set (the positional term of the backbones of
Sec. 4.1) vs the CPU oracle: the cos/sin table, the QKV GEMM whose epilogue turns q and the new keys, and
the whole block with it.  Bars as for the block: 2e-2 max-relative against the fp64 oracle (bf16 kernels),
values bit-identical to the plain path, cache rows outside the appended window untouched."""
import numpy as np
import pytest
import torch

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth
from gpu_util import (DEV, cache_rows, empty_ws, from_dev_bf16, make_caches, max_rel, to_dev_bf16,
                      upload_weights)

pytestmark = pytest.mark.gpu
TOL = 2e-2
TINY128 = synth.BlockDims(D=256, H=2, dh=128, F=512)
TINY64 = synth.BlockDims(D=192, H=3, dh=64, F=320)


def device_tables(h, w, dh, base, ref_h, ref_w):
    cos = torch.full((h * w, dh // 2), float("nan"), dtype=torch.float32, device=DEV)
    sin = torch.full_like(cos, float("nan"))
    fb.fastvar_rope2d_table(h, w, dh, base, ref_h, ref_w, cos, sin)
    torch.cuda.synchronize()
    return cos, sin


@pytest.mark.parametrize("h,w,dh,base,ref", [(1, 1, 64, 10000.0, (1, 1)), (5, 7, 64, 10000.0, (5, 7)),
                                              (16, 16, 128, 10000.0, (64, 64)), (64, 64, 128, 10000.0, (64, 64)),
                                              (9, 4, 8, 50.0, (18, 12))])
def test_table_matches_oracle(h, w, dh, base, ref):
    print(f"[rope table] {h}x{w} dh={dh} base={base} ref={ref}", flush=True)
    cos, sin = device_tables(h, w, dh, base, ref[0], ref[1])
    ang = O.rope2d_angles(h, w, dh, base, ref[0], ref[1])
    # fp64 evaluation rounded once to fp32; the power is taken as exp(-t/q log base) on the device
    assert np.max(np.abs(cos.cpu().numpy() - np.cos(ang))) <= 2e-6
    assert np.max(np.abs(sin.cpu().numpy() - np.sin(ang))) <= 2e-6
    assert torch.all(cos[0] == 1.0) and torch.all(sin[0] == 0.0)      # the origin is not turned


def check_block_rope(name, dims, B, h, w, k, L0, L_cap, seed, ref=None, rows=None, scale=None):
    print(f"[block+rope] {name} D={dims.D} dh={dims.dh} B={B} N={h*w} k={k} L0={L0}", flush=True)
    N = h * w
    ref = ref or (h, w)
    x_np = synth.token_map(seed, B, h, w, dims.D)
    W = synth.block_weights(seed, dims)
    kp, vp = synth.kv_prior(seed, B, L0, dims.H, dims.dh)
    idx_np = O.select_pivotal(x_np, k)[0] if k < N else np.tile(np.arange(N, dtype=np.int32), (B, 1))
    ang = O.rope2d_angles(h, w, dims.dh, 10000.0, ref[0], ref[1])
    rope = np.stack([ang[idx_np[b]] for b in range(B)])
    cos, sin = device_tables(h, w, dims.dh, 10000.0, ref[0], ref[1])
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F, 1e-6, scale)
    wt, wstruct = upload_weights(W)
    x = to_dev_bf16(x_np)
    idx = torch.from_numpy(idx_np.astype(np.int32)).to(DEV)
    kc, vc = make_caches(kp, vp, L_cap)
    kc0, vc0 = kc.clone(), vc.clone()
    y = torch.full((B, k, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = empty_ws(fb.fastvar_block_workspace_bytes(d, B, k))
    ws.fill_(0xFF)
    fb.fastvar_block_forward_pruned_rope(x, N, idx if k < N else None, B, k, d, wstruct, cos, sin, kc, vc, L0, L_cap,
                                         y, ws)
    torch.cuda.synchronize()
    got = from_dev_bf16(y)
    xk = O.gather_tokens(x_np, idx_np)
    yo, kn, vn = O.block_forward_pruned(xk, W, dims.H, kp, vp, rope=rope, rows=rows, scale=scale)
    y_plain, kn_plain, _ = O.block_forward_pruned(xk, W, dims.H, kp, vp, rows=rows, scale=scale)
    if rows is not None:
        got = got[:, rows]
    kg, vg = cache_rows(kc, vc, L0, L0 + k)
    e = (max_rel(got, yo), max_rel(kg, kn), max_rel(vg, vn))
    print("    max-rel: y %.2e  k_new %.2e  v_new %.2e   (oracle without rope differs by y %.2e  k %.2e)"
          % (e + (max_rel(y_plain, yo), max_rel(kn_plain, kn))), flush=True)
    assert not np.isnan(got).any() and max(e) <= TOL, name
    # the test has teeth: leaving the rotation out, or turning by the wrong slot, is far outside the bar
    if N > 1 and k > 1:
        assert max_rel(kn_plain, kn) > 10 * TOL
    if scale is not None:     # peaked attention: the block output itself tells the two apart
        assert max_rel(y_plain, yo) > 2 * TOL
    # cache rows outside [L0, L0 + k) keep their bits
    kb, kb0 = kc.view(torch.int16), kc0.view(torch.int16)
    vb, vb0 = vc.view(torch.int16), vc0.view(torch.int16)
    assert torch.equal(kb[:, :, :L0], kb0[:, :, :L0]) and torch.equal(kb[:, :, L0 + k:], kb0[:, :, L0 + k:])
    assert torch.equal(vb[:, :, :, :L0], vb0[:, :, :, :L0]) and torch.equal(vb[:, :, :, L0 + k:], vb0[:, :, :, L0 + k:])
    return max_rel(y_plain, yo)


ROPE_CASES = [
    ("tiny64_ragged", TINY64, 2, 7, 9, 37, 29, 104, None),
    ("tiny128_ragged", TINY128, 3, 9, 11, 70, 45, 128, None),
    ("tiny128_keep_all_no_index_list", TINY128, 1, 8, 8, 64, 24, 96, None),
    ("tiny64_single_kept", TINY64, 2, 5, 5, 1, 63, 64, None),
    ("d16_256px_last_on_its_own_grid", synth.D16, 1, 16, 16, 128, 424, 688, None),
    ("d30_s24_b2", synth.D30, 2, 24, 24, 346, 640, 992, (32, 32)),
    ("inf2b_side12_split_k", synth.INF2B, 1, 12, 12, 144, 121, 272, (64, 64)),
    ("inf2b_s40_keep0.6", synth.INF2B, 1, 40, 40, 960, 2521, 3488, (64, 64)),
]


@pytest.mark.parametrize("name,dims,B,h,w,k,L0,L_cap,ref", ROPE_CASES, ids=[c[0] for c in ROPE_CASES])
def test_block_with_rope_matches_oracle(name, dims, B, h, w, k, L0, L_cap, ref):
    check_block_rope(name, dims, B, h, w, k, L0, L_cap, seed=23, ref=ref)


def test_block_with_rope_peaked_attention_output_depends_on_positions():
    """With the synthetic weights the scores are small and attention is close to uniform, so the block output
    moves little when q and k are turned; a large softmax scale makes the output itself position dependent."""
    check_block_rope("tiny128_scale3", TINY128, 2, 9, 11, 70, 0, 72, seed=25, scale=3.0)
    check_block_rope("tiny64_scale16", TINY64, 1, 12, 12, 100, 0, 104, seed=26, scale=16.0)


def test_block_with_rope_headline_size_sampled_rows():
    wl = synth.WORKLOADS[synth.HEADLINE]
    rows = np.unique(np.concatenate([np.arange(0, 2), np.arange(wl.k - 2, wl.k),
                                     np.random.default_rng(6).integers(0, wl.k, 28)]))
    check_block_rope("headline_sampled", wl.dims, 1, wl.h, wl.h, wl.k, wl.L0_full, 8480, seed=24, rows=rows)


@pytest.mark.parametrize("dims,B,h,w,k,L0,L_cap", [
    (synth.D16, 2, 10, 12, 50, 17, 72),
    (synth.INF2B, 2, 48, 48, 1500, 100, 1608),    # more tiles than one round of workgroups
])
def test_qkv_gemm_rope_component_and_values_untouched(dims, B, h, w, k, L0, L_cap):
    """The component entry point with a per-sample index list: q and K turned by the slots' angles, V the
    same bits as the plain QKV GEMM writes."""
    print(f"[qkv+rope] D={dims.D} dh={dims.dh} B={B} N={h*w} k={k}", flush=True)
    N = h * w
    rng = np.random.default_rng(8)
    a_np = synth.round_bf16(rng.standard_normal((B * k, dims.D)).astype(np.float32))
    W = synth.block_weights(8, dims)
    idx_np = np.stack([np.sort(rng.permutation(N)[:k]) for _ in range(B)]).astype(np.int32)
    ang = O.rope2d_angles(h, w, dims.dh)
    cos, sin = device_tables(h, w, dims.dh, 10000.0, h, w)
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    a = to_dev_bf16(a_np)
    wq, bq = to_dev_bf16(W["w_qkv"]), to_dev_bf16(W["b_qkv"])
    idx = torch.from_numpy(idx_np).to(DEV)
    e0 = np.zeros((B, 0, dims.H, dims.dh), np.float32)
    out = []
    for rope in (True, False):
        kc, vc = make_caches(e0, e0, L_cap)
        q = torch.full((B * k, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        if rope:
            fb.fastvar_qkv_gemm_rope(a, wq, bq, idx, B, N, k, d, cos, sin, q, kc, vc, L0, L_cap)
        else:
            fb.fastvar_qkv_gemm(a, wq, bq, B, k, d, q, kc, vc, L0, L_cap)
        torch.cuda.synchronize()
        out.append((from_dev_bf16(q), kc, vc))
    qkv = O.linear(a_np.reshape(B, k, dims.D), W["w_qkv"], W["b_qkv"])
    D = dims.D
    rope_a = np.stack([ang[idx_np[b]] for b in range(B)])
    q_ref = O.apply_rope(qkv[..., :D].reshape(B, k, dims.H, dims.dh), rope_a).reshape(B * k, D)
    k_ref = O.apply_rope(qkv[..., D:2 * D].reshape(B, k, dims.H, dims.dh), rope_a)
    kg, vg = cache_rows(out[0][1], out[0][2], L0, L0 + k)
    assert max_rel(out[0][0], q_ref) <= 2.0 ** -7 and max_rel(kg, k_ref) <= 2.0 ** -7
    assert torch.equal(out[0][2].view(torch.int16)[:, :, :, L0:L0 + k], out[1][2].view(torch.int16)[:, :, :, L0:L0 + k])
    assert max_rel(vg, qkv[..., 2 * D:].reshape(B, k, dims.H, dims.dh)) <= 2.0 ** -7


def test_rope_argument_errors():
    print("[rope] error paths", flush=True)
    cos = torch.zeros((16, 32), dtype=torch.float32, device=DEV)
    sin = torch.zeros_like(cos)
    L = fb.lib()
    st = torch.cuda.current_stream().cuda_stream
    assert L.fastvar_rope2d_table(4, 4, 64, 10000.0, 4, 4, None, sin.data_ptr(), st) == fb.FASTVAR_EINVAL
    assert L.fastvar_rope2d_table(4, 4, 64, -1.0, 4, 4, cos.data_ptr(), sin.data_ptr(), st) == fb.FASTVAR_EINVAL
    assert L.fastvar_rope2d_table(4, 4, 60, 10000.0, 4, 4, cos.data_ptr(), sin.data_ptr(), st) == fb.FASTVAR_EALIGN
    assert L.fastvar_rope2d_table(400, 400, 64, 10000.0, 4, 4, cos.data_ptr(), sin.data_ptr(), st) == fb.FASTVAR_ECAPACITY
    torch.cuda.synchronize()
    assert torch.all(cos == 0)
