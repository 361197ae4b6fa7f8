"""GPU parity: fastvar_scale_step, the stack-level scale step (Fig. 2(a); Sec. 3.3, overview), and the
unpruned block (no index list) it uses in the structure construction stage.

A whole small schedule is run through the library for a one-block stack and compared with the
oracle step by step: caches grow by the kept tokens only, the map captured at the cached step feeds
the pruned steps, a skipped step leaves the upsampled cache.  For several blocks the selection of
block l+1 depends on the device's bf16 output of block l, so the stack is checked against the
library's own single-block entry points, which must give the same bits, and those are checked
against the oracle elsewhere.
"""
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


@pytest.mark.parametrize("dims,B,h,w,L0,L_cap", [(TINY64, 2, 5, 7, 13, 48), (TINY128, 1, 1, 1, 0, 8),
                                                (TINY128, 3, 2, 2, 1, 8), (synth.D16, 1, 16, 16, 424, 680)])
def test_unpruned_block_without_index_list(dims, B, h, w, L0, L_cap):
    print(f"[dense block] D={dims.D} B={B} N={h*w} L0={L0}", flush=True)
    N = h * w
    x_np = synth.token_map(31, B, h, w, dims.D)
    W = synth.block_weights(31, dims)
    kp, vp = synth.kv_prior(31, B, L0, dims.H, dims.dh)
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    wt, wstruct = upload_weights(W)
    x = to_dev_bf16(x_np)
    kc, vc = make_caches(kp, vp, L_cap)
    y = torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
    ws = empty_ws(fb.fastvar_block_workspace_bytes(d, B, N))
    ws.fill_(0xFF)
    fb.fastvar_block_forward_pruned(x, N, None, B, N, d, wstruct, kc, vc, L0, L_cap, y, ws)
    torch.cuda.synchronize()
    ref, kn, vn = O.block_forward_pruned(x_np, W, dims.H, kp, vp)
    got = from_dev_bf16(y)
    kg, vg = cache_rows(kc, vc, L0, L0 + N)
    assert not np.isnan(got).any()
    assert max_rel(got, ref) <= TOL and max_rel(kg, kn) <= TOL and max_rel(vg, vn) <= TOL
    # the same rows as with the identity index list, bit for bit
    kc2, vc2 = make_caches(kp, vp, L_cap)
    y2 = torch.empty_like(y)
    idx = torch.arange(N, dtype=torch.int32, device=DEV).repeat(B, 1)
    fb.fastvar_block_forward_pruned(x, N, idx, B, N, d, wstruct, kc2, vc2, L0, L_cap, y2, ws)
    torch.cuda.synchronize()
    assert torch.equal(y.view(torch.int16), y2.view(torch.int16))
    # an index list may only be left out when every token is kept
    if N > 1:
        with pytest.raises(fb.FastvarError):
            fb.fastvar_block_forward_pruned(x, N, None, B, N - 1, d, wstruct, kc, vc, L0, L_cap, y, ws)


def _stack(dims, n_layers, B, L_cap, hc, wc, seed):
    layers = []
    for l in range(n_layers):
        W = synth.block_weights(seed + l, dims)
        wt, wstruct = upload_weights(W)
        kp, vp = synth.kv_prior(seed + l, B, 0, dims.H, dims.dh)
        kc, vc = make_caches(kp, vp, L_cap)
        cache = torch.full((B, hc * wc, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        layers.append(dict(W=W, wt=wt, w=wstruct, kc=kc, vc=vc, cache=cache))
    return layers


def test_one_block_schedule_matches_oracle_step_by_step():
    """Sides (1,2,3,5,8,11): structure steps 0-3 (capture at the 5x5 step), then keep 0.6, a skipped
    step is replaced by keep 0 at the last scale."""
    dims, B = TINY128, 2
    sides = (1, 2, 3, 5, 8, 11)
    cache_step = 3
    keeps = {4: 0.6, 5: 0.0}
    L_cap = 1 + 4 + 9 + 25 + 64 + 121 + 7
    L_cap = (L_cap + 7) // 8 * 8
    hc = wc = sides[cache_step]
    layers = _stack(dims, 1, B, L_cap, hc, wc, seed=50)
    arr = fb.make_layers(layers)
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    o_k = [np.zeros((B, 0, dims.H, dims.dh))]
    o_v = [np.zeros((B, 0, dims.H, dims.dh))]
    o_cache = None
    kv_len = 0
    for step, side in enumerate(sides):
        N = side * side
        k = N if step <= cache_step else fb.fastvar_keep_count(N, keeps[step])
        print(f"[schedule] step {step} side {side} k={k} kv_len={kv_len}", flush=True)
        x_np = synth.token_map(60 + step, B, side, side, dims.D)
        x = to_dev_bf16(x_np)
        y = torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        idx = torch.full((B, max(k, 1)), -7, dtype=torch.int32, device=DEV)
        ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, k))
        ws.fill_(0xFF)
        new_len = fb.fastvar_scale_step(x, list(sides), list(sides), step, cache_step, B, k, d, arr, kv_len, L_cap,
                                        y, None, idx, ws)
        torch.cuda.synchronize()
        ref = O.scale_step(x_np, side, side, k, [layers[0]["W"]], dims.H, o_k, o_v, o_cache, hc, wc,
                           structure=step <= cache_step, capture=step == cache_step)
        got = from_dev_bf16(y)
        assert new_len == kv_len + k
        assert not np.isnan(got).any()
        assert max_rel(got, ref["y"]) <= TOL, step
        if step > cache_step and 0 < k < N:
            np.testing.assert_array_equal(idx[:, :k].cpu().numpy(), ref["idx"])
        if k > 0:
            kg, vg = cache_rows(layers[0]["kc"], layers[0]["vc"], kv_len, kv_len + k)
            assert max_rel(kg, ref["k_caches"][0][:, kv_len:]) <= TOL
            assert max_rel(vg, ref["v_caches"][0][:, kv_len:]) <= TOL
        if step == cache_step:
            # the captured map is the output itself; the oracle goes on with the device's bf16 copy of it
            assert torch.equal(layers[0]["cache"].view(torch.int16), y.view(torch.int16))
            o_cache = [from_dev_bf16(layers[0]["cache"]).astype(np.float64)]
        # the oracle's caches follow the device's bf16 rows, so that later steps see identical keys
        kall, vall = cache_rows(layers[0]["kc"], layers[0]["vc"], 0, new_len)
        o_k, o_v = [kall.astype(np.float64)], [vall.astype(np.float64)]
        kv_len = new_len
    # the last step kept nothing: the output is the upsampled captured map, within one bf16 rounding
    up = O.upsample_bilinear(o_cache[0], hc, wc, sides[-1], sides[-1])
    assert np.all(np.abs(got - up) <= 2.0 ** -8 * 1.001 * np.abs(up) + 2e-6)


@pytest.mark.parametrize("n_layers,keeps", [(2, (0.45, 0.45)), (3, (0.45, 0.0)), (3, (1.0, 0.3))])
def test_stack_equals_the_single_block_entry_points(n_layers, keeps):
    dims, B = TINY64, 2
    sides = (2, 3, 4, 6, 9)
    cache_step = 2
    hc = wc = sides[cache_step]
    L_cap = 160
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    A = _stack(dims, n_layers, B, L_cap, hc, wc, seed=70)      # through fastvar_scale_step
    Bk = _stack(dims, n_layers, B, L_cap, hc, wc, seed=70)     # block by block
    arr = fb.make_layers(A)
    kv_a = kv_b = 0
    for step, side in enumerate(sides):
        N = side * side
        k = N if step <= cache_step else fb.fastvar_keep_count(N, keeps[step - cache_step - 1])
        print(f"[stack] layers={n_layers} step {step} side {side} k={k}", flush=True)
        x = to_dev_bf16(synth.token_map(80 + step, B, side, side, dims.D))
        y = torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        tmp = torch.full_like(y, float("nan"))
        idx = torch.zeros((B, max(k, 1)), dtype=torch.int32, device=DEV)
        ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, k))
        kv_a = fb.fastvar_scale_step(x, list(sides), list(sides), step, cache_step, B, k, d, arr, kv_a, L_cap, y,
                                     tmp, idx, ws)
        # the same through the single-block calls
        cur = x
        for l, ly in enumerate(Bk):
            out = torch.empty_like(y)
            if step <= cache_step:
                fb.fastvar_block_forward_pruned(cur, N, None, B, N, d, ly["w"], ly["kc"], ly["vc"], kv_b, L_cap, out,
                                                ws)
                if step == cache_step:
                    ly["cache"] = out.clone()
            else:
                idx_b = torch.zeros((B, max(k, 1)), dtype=torch.int32, device=DEV)
                fb.fastvar_step(cur, list(sides), list(sides), step, cache_step, B, k, d, ly["w"], ly["kc"], ly["vc"],
                                kv_b, L_cap, ly["cache"], out, idx_b, ws)
            cur = out
        kv_b += k
        torch.cuda.synchronize()
        assert kv_a == kv_b
        assert torch.equal(y.view(torch.int16), cur.view(torch.int16)), step
        if step > cache_step and 0 < k < N:
            assert torch.equal(idx, idx_b)
        for la, lb in zip(A, Bk):
            assert torch.equal(la["kc"][:, :, :kv_a].view(torch.int16), lb["kc"][:, :, :kv_a].view(torch.int16))
            assert torch.equal(la["vc"][:, :, :, :kv_a].view(torch.int16), lb["vc"][:, :, :, :kv_a].view(torch.int16))
            if step == cache_step:
                assert torch.equal(la["cache"].view(torch.int16), lb["cache"].view(torch.int16))


def test_stack_equals_single_block_calls_at_the_headline_size():
    """Two blocks of the headline step through fastvar_scale_step (where the restoration of a block leaves the
    column sums for the next block's selection) against two fastvar_step calls: same bits."""
    wl = synth.WORKLOADS[synth.HEADLINE]
    dims, B, N, k = wl.dims, 1, wl.N, wl.k
    print(f"[stack] headline size, 2 blocks, N={N} k={k}", flush=True)
    L0, L_cap = wl.L0_full, 8480
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)

    def rn(shape, std=1.0, mean=0.0):
        return (torch.randn(shape, generator=gen, device=DEV) * std + mean).to(torch.bfloat16)

    def make():
        out = []
        g2 = torch.Generator(device=DEV)
        g2.manual_seed(9)
        r = lambda shape, std=1.0, mean=0.0: (torch.randn(shape, generator=g2, device=DEV) * std + mean).to(torch.bfloat16)
        D, F = dims.D, dims.F
        for _ in range(2):
            wt = dict(ln1_g=r((D,), 0.02, 1.0), ln1_b=r((D,), 0.02), w_qkv=r((3 * D, D), 0.02), b_qkv=r((3 * D,), 0.02),
                      w_proj=r((D, D), 0.02), b_proj=r((D,), 0.02), ln2_g=r((D,), 0.02, 1.0), ln2_b=r((D,), 0.02),
                      w_fc1=r((F, D), 0.02), b_fc1=r((F,), 0.02), w_fc2=r((D, F), 0.02), b_fc2=r((D,), 0.02))
            kc = torch.zeros((B, dims.H, L_cap, dims.dh), dtype=torch.bfloat16, device=DEV)
            vc = torch.zeros((B, dims.H, dims.dh, L_cap), dtype=torch.bfloat16, device=DEV)
            kc[:, :, :L0] = r((B, dims.H, L0, dims.dh))
            vc[:, :, :, :L0] = r((B, dims.H, dims.dh, L0))
            out.append(dict(wt=wt, w=fb.make_weights(wt), kc=kc, vc=vc, cache=r((B, wl.hc * wl.hc, D))))
        return out

    x = to_dev_bf16(synth.token_map(5, B, wl.h, wl.h, dims.D))
    sides = list(wl.sides)
    ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, k))
    A, S = make(), make()
    ya, tmp = torch.empty_like(x), torch.empty_like(x)
    ia = torch.zeros((B, k), dtype=torch.int32, device=DEV)
    fb.fastvar_scale_step(x, sides, sides, wl.step, wl.cache_step, B, k, d, fb.make_layers(A), L0, L_cap, ya, tmp, ia, ws)
    cur = x
    for ly in S:
        out = torch.empty_like(x)
        ib = torch.zeros((B, k), dtype=torch.int32, device=DEV)
        fb.fastvar_step(cur, sides, sides, wl.step, wl.cache_step, B, k, d, ly["w"], ly["kc"], ly["vc"], L0, L_cap,
                        ly["cache"], out, ib, ws)
        cur = out
    torch.cuda.synchronize()
    assert torch.equal(ia, ib)
    assert torch.equal(ya.view(torch.int16), cur.view(torch.int16))


@pytest.mark.parametrize("side", [2, 8, 12, 24])
def test_structure_steps_of_the_large_model_across_layers(side):
    """Structure steps of the 2B-class model: few rows, so every GEMM splits K between workgroups, and the
    four GEMMs of a block (different tile counts) and the blocks of the stack reuse one scratch area whose
    arrival counters are cleared once per call.  Three blocks through fastvar_scale_step must give the bits
    of three single-block calls; the first block is also checked against the oracle."""
    dims = synth.INF2B
    B, N, n_layers = 1, side * side, 3
    print(f"[structure step] large model, {n_layers} blocks, N={N}", flush=True)
    L0 = 37
    L_cap = (L0 + N + 7) // 8 * 8
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    x_np = synth.token_map(41, B, side, side, dims.D)
    Ws = [synth.block_weights(41 + l, dims, block=l) for l in range(n_layers)]
    kp, vp = synth.kv_prior(41, B, L0, dims.H, dims.dh)
    up = [upload_weights(W) for W in Ws]
    x = to_dev_bf16(x_np)

    def layers():
        out = []
        for (wt, wstruct) in up:
            kc, vc = make_caches(kp, vp, L_cap)
            out.append(dict(wt=wt, w=wstruct, kc=kc, vc=vc, cache=None))
        return out

    ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, N))
    ws.fill_(0xFF)
    A, S = layers(), layers()
    sides = [side, 2 * side]
    ya = torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
    tmp = torch.empty_like(ya)
    new_len = fb.fastvar_scale_step(x, sides, sides, 0, 1, B, N, d, fb.make_layers(A), L0, L_cap, ya, tmp, None, ws)
    assert new_len == L0 + N
    cur, first = x, None
    for ly in S:
        out = torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV)
        fb.fastvar_block_forward_pruned(cur, N, None, B, N, d, ly["w"], ly["kc"], ly["vc"], L0, L_cap, out, ws)
        first = out if first is None else first
        cur = out
    torch.cuda.synchronize()
    assert not torch.isnan(ya.float()).any()
    assert torch.equal(ya.view(torch.int16), cur.view(torch.int16))
    for la, lb in zip(A, S):
        assert torch.equal(la["kc"].view(torch.int16), lb["kc"].view(torch.int16))
        assert torch.equal(la["vc"].view(torch.int16), lb["vc"].view(torch.int16))
    ref, kn, vn = O.block_forward_pruned(x_np, Ws[0], dims.H, kp, vp)
    assert max_rel(from_dev_bf16(first), ref) <= TOL
    kg, vg = cache_rows(S[0]["kc"], S[0]["vc"], L0, L0 + N)
    assert max_rel(kg, kn) <= TOL and max_rel(vg, vn) <= TOL


def test_timed_scale_step_gives_the_same_result_and_stage_times():
    print("[scale step] stopwatch variant", flush=True)
    dims, B = TINY64, 2
    sides = (2, 3, 5, 8)
    cache_step, L_cap = 1, 128
    hc = wc = sides[cache_step]
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    A = _stack(dims, 3, B, L_cap, hc, wc, seed=95)
    T = _stack(dims, 3, B, L_cap, hc, wc, seed=95)
    la, lt = fb.make_layers(A), fb.make_layers(T)
    kv_a = kv_t = 0
    for step, side in enumerate(sides):
        N = side * side
        k = N if step <= cache_step else fb.fastvar_keep_count(N, 0.5)
        x = to_dev_bf16(synth.token_map(96 + step, B, side, side, dims.D))
        ya, yt = (torch.full((B, N, dims.D), float("nan"), dtype=torch.bfloat16, device=DEV) for _ in range(2))
        tmp = torch.empty_like(ya)
        idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)
        ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, k))
        kv_a = fb.fastvar_scale_step(x, list(sides), list(sides), step, cache_step, B, k, d, la, kv_a, L_cap, ya, tmp, idx, ws)
        kv_t, ms = fb.fastvar_scale_step_timed(x, list(sides), list(sides), step, cache_step, B, k, d, lt, kv_t, L_cap,
                                               yt, tmp, idx, ws)
        # the timed call has waited for the stream: the result is there without a synchronize
        assert kv_a == kv_t
        assert torch.equal(ya.view(torch.int16), yt.view(torch.int16))
        assert set(ms) == set(fb.STAGES)
        pruned = step > cache_step
        for name, v in ms.items():
            # restoration has no launch of its own while something is kept: the pruned rows are filled inside
            # the gather + LayerNorm launch, the kept rows by the block's last GEMM
            if (name == "select" and not pruned) or name == "restore":
                assert v == 0.0, (name, v)
            else:
                assert 0.0 < v < 50.0, (name, v)
    with pytest.raises(fb.FastvarError):
        fb.fastvar_scale_step_timed(x, list(sides), list(sides), 3, cache_step, B, k, d, lt, 999, L_cap, yt, tmp, idx, ws)


def test_scale_step_argument_errors():
    print("[scale step] error paths", flush=True)
    dims, B = TINY64, 1
    sides = [2, 4]
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    layers = _stack(dims, 2, B, 32, 2, 2, seed=90)
    arr = fb.make_layers(layers)
    x = to_dev_bf16(synth.token_map(1, B, 4, 4, dims.D))
    y = torch.zeros((B, 16, dims.D), dtype=torch.bfloat16, device=DEV)
    tmp = torch.zeros_like(y)
    idx = torch.zeros((B, 8), dtype=torch.int32, device=DEV)
    ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, 16, 16))

    def call(**over):
        a = dict(x=x, sched_h=sides, sched_w=sides, step=1, cache_step=0, B=B, k=8, dims=d, layers=arr, kv_len=4,
                 L_cap=32, y_out=y, tmp=tmp, idx_out=idx, ws=ws)
        a.update(over)
        try:
            fb.fastvar_scale_step(**a)
        except fb.FastvarError as e:
            return e.code
        return 0

    assert call(tmp=None) == fb.FASTVAR_EINVAL                 # two blocks need the scratch map
    assert call(y_out=x) == fb.FASTVAR_EINVAL
    assert call(step=0, cache_step=0, k=3) == fb.FASTVAR_EINVAL   # structure steps are unpruned
    assert call(idx_out=None) == fb.FASTVAR_EINVAL
    assert call(kv_len=30) == fb.FASTVAR_ECAPACITY
    assert call(ws=empty_ws(256)) == fb.FASTVAR_EWORKSPACE
    torch.cuda.synchronize()
    assert torch.all(y == 0) and torch.all(tmp == 0)


def _rand_layers(dims, n, B, L0, L_cap, hc, seed):
    g = torch.Generator(device=DEV)
    g.manual_seed(seed)
    r = lambda shape, std=1.0, mean=0.0: (torch.randn(shape, generator=g, device=DEV) * std + mean).to(torch.bfloat16)
    D, F = dims.D, dims.F
    out = []
    for _ in range(n):
        wt = dict(ln1_g=r((D,), 0.02, 1.0), ln1_b=r((D,), 0.02), w_qkv=r((3 * D, D), 0.02), b_qkv=r((3 * D,), 0.02),
                  w_proj=r((D, D), 0.02), b_proj=r((D,), 0.02), ln2_g=r((D,), 0.02, 1.0), ln2_b=r((D,), 0.02),
                  w_fc1=r((F, D), 0.02), b_fc1=r((F,), 0.02), w_fc2=r((D, F), 0.02), b_fc2=r((D,), 0.02))
        kc = torch.zeros((B, dims.H, L_cap, dims.dh), dtype=torch.bfloat16, device=DEV)
        vc = torch.zeros((B, dims.H, dims.dh, L_cap), dtype=torch.bfloat16, device=DEV)
        if L0:
            kc[:, :, :L0] = r((B, dims.H, L0, dims.dh))
            vc[:, :, :, :L0] = r((B, dims.H, dims.dh, L0))
        out.append(dict(wt=wt, w=fb.make_weights(wt), kc=kc, vc=vc, cache=r((B, hc * hc, D))))
    return out


def _two_block_case(case):
    """A two-block stack step of the large model on one of the paths that merge partial results between
    workgroups; returns the call, a poisoner of outputs and scratch, and a snapshot of everything it writes."""
    dims = synth.INF2B
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    if case == "structure_step_split_k":
        B, side, L0 = 1, 12, 121
        N = k = side * side
        sides, step, cache_step, hc = [side, 2 * side], 0, 1, side
    else:
        wl = synth.WORKLOADS[{"headline_two_blocks": synth.HEADLINE, "keep0.25_key_ranges": "inf2b_1024px_s64_keep0.25",
                              "s48_fc2_two_k_slices": "inf2b_1024px_s48_keep0.5"}[case]]
        B, N, k, L0 = 1, wl.N, wl.k, wl.L0_full
        sides, step, cache_step, hc = list(wl.sides), wl.step, wl.cache_step, wl.hc
    L_cap = (L0 + k + 7) // 8 * 8
    layers = _rand_layers(dims, 2, B, L0, L_cap, hc, seed=21)
    arr = fb.make_layers(layers)
    x = to_dev_bf16(synth.token_map(17, B, sides[step], sides[step], dims.D))
    ws = empty_ws(fb.fastvar_step_workspace_bytes(d, B, N, k))
    y = torch.empty((B, N, dims.D), dtype=torch.bfloat16, device=DEV)
    tmp = torch.empty_like(y)
    idx = torch.zeros((B, k), dtype=torch.int32, device=DEV)

    def call():
        fb.fastvar_scale_step(x, sides, sides, step, cache_step, B, k, d, arr, L0, L_cap, y, tmp, idx, ws)

    def poison(run):
        ws.fill_(0xFF if run % 2 else 0x00)
        y.fill_(float("nan"))
        tmp.fill_(float("nan"))

    def snapshot():
        got = [y.view(torch.int16).clone(), tmp.view(torch.int16).clone(), idx.clone()]
        for ly in layers:
            got.append(ly["kc"][:, :, L0:L0 + k].view(torch.int16).clone())
            got.append(ly["vc"][:, :, :, L0:L0 + k].view(torch.int16).clone())
        return got

    return dict(N=N, k=k, L0=L0, y=y, call=call, poison=poison, snapshot=snapshot, keep=(layers, arr, x, ws, tmp, idx))


@pytest.mark.parametrize("case", ["headline_two_blocks", "keep0.25_key_ranges", "structure_step_split_k",
                                  "s48_fc2_two_k_slices"])
def test_same_inputs_give_the_same_bits_every_run(case):
    """Same inputs, same bits: the stack step run 20 times.  The headline step merges two key ranges per
    query tile in its attention; the keep 0.25 step three; the structure step (144 tokens at the large
    model's widths) splits K between workgroups in all four GEMMs; the 48x48 step at keep 0.5 runs FC2 on
    two K slices of 256x128 tiles whose last arriver waits for the other's partial tile.  All of them let the workgroup that
    arrives last combine the partial results, so a result that depended on arrival order, or a partial
    result read before it was complete, would show here as a changed bit.  Stops at the first difference."""
    c = _two_block_case(case)
    print(f"[determinism] {case}: N={c['N']} k={c['k']} L0={c['L0']}, 2 blocks, 20 runs", flush=True)
    first = None
    for run in range(20):
        c["poison"](run)                        # whatever the scratch held before must not matter
        c["call"]()
        torch.cuda.synchronize()
        got = c["snapshot"]()
        y = c["y"]
        if first is None:
            first = got
            assert not torch.isnan(y.float()).any()
            continue
        for i, (a, b) in enumerate(zip(first, got)):
            assert torch.equal(a, b), f"run {run}: tensor {i} differs from the first run"


@pytest.mark.parametrize("case", ["keep0.25_key_ranges", "structure_step_split_k"])
def test_scale_step_replayed_from_a_hip_graph(case):
    """A caller may capture the step into a HIP graph: the library allocates nothing, clears its arrival
    counters with a kernel (not a memset node) and sets function attributes on a first, eager call only.
    The captured step is replayed three times, with eager calls, fills and synchronisations between the
    replays, and every replay is compared bit for bit with the eager result."""
    c = _two_block_case(case)
    print(f"[graph] {case}: N={c['N']} k={c['k']} L0={c['L0']}, 2 blocks, 3 replays", flush=True)
    c["poison"](0)
    c["call"]()
    torch.cuda.synchronize()
    ref = c["snapshot"]()
    assert not torch.isnan(c["y"].float()).any()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        c["call"]()
    for rep in range(3):
        c["poison"](rep + 1)
        g.replay()
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(ref, c["snapshot"]())):
            assert torch.equal(a, b), f"replay {rep}: tensor {i} differs from the eager result"
        c["poison"](rep)
        c["call"]()                              # the program's own eager work between the replays
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(zip(ref, c["snapshot"]())):
            assert torch.equal(a, b), f"eager call after replay {rep}: tensor {i} differs"

