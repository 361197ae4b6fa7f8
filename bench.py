#!/usr/bin/env python3
"""Benchmark of the pruned VAR decoding step on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--wiring block|sublayer]

A step is one pass of the whole hot path -- pivotal token selection, the
transformer block on the kept tokens, cached token restoration -- through every
block of the stack at the last scale of the 1024 px Infinity-2B-style schedule
with keep ratio 0.5 (64x64 map, 2048 kept tokens, 6425 prior cache tokens,
32 blocks with distinct weights, caches and cached maps).  Inputs are seeded
and synthetic and are resident in HBM before the timed region.

Prints ONE JSON line: effective tokens/s (B*N restored tokens per step time),
ms per step, per-kernel timings, the roofline record of the dominant kernel
and the CPU oracle baseline (one block, timed on the host cores).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2503_23367_amd import synth  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def build_state(wl, n_blocks, seed=0, wiring="block"):
    """All device buffers of the workload.  Block 0 comes from the shared
    seeded numpy generators (so the CPU oracle can be fed the same values);
    the remaining blocks are drawn on the GPU with the same distributions."""
    import torch
    from paper_2503_23367_amd import binding as fb
    dev = "cuda:0"
    dims = wl.dims
    B, N, k, L0 = wl.B, wl.N, wl.k, wl.L0_full
    L_cap = (L0 + k + 7) // 8 * 8

    def up(a):
        bits = synth.to_bf16_bits(a).astype(np.int16)
        return torch.from_numpy(bits).to(dev).view(torch.bfloat16).reshape(a.shape)

    host = dict(
        x=synth.token_map(seed, B, wl.h, wl.h, dims.D),
        W=synth.block_weights(seed, dims),
        cache=synth.cached_map(seed, B, wl.hc, wl.hc, dims.D),
        cache_attn=synth.cached_map(seed + 1000, B, wl.hc, wl.hc, dims.D),
    )
    host["kp"], host["vp"] = synth.kv_prior(seed, B, L0, dims.H, dims.dh)

    gen = torch.Generator(device=dev)
    gen.manual_seed(seed + 12345)

    def randn(shape, std=1.0, mean=0.0):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std + mean).to(torch.bfloat16)

    blocks = []
    for blk in range(n_blocks):
        if blk == 0:
            wt = {n: up(a) for n, a in host["W"].items()}
            kc = torch.zeros((B, dims.H, L_cap, dims.dh), dtype=torch.bfloat16, device=dev)
            vc = torch.zeros((B, dims.H, dims.dh, L_cap), dtype=torch.bfloat16, device=dev)
            kc[:, :, :L0] = up(host["kp"]).permute(0, 2, 1, 3)
            vc[:, :, :, :L0] = up(host["vp"]).permute(0, 2, 3, 1)
            cache = up(host["cache"])
            cache_attn = up(host["cache_attn"]) if wiring == "sublayer" else None
        else:
            D, F = dims.D, dims.F
            wt = dict(ln1_g=randn((D,), 0.02, 1.0), ln1_b=randn((D,), 0.02),
                      w_qkv=randn((3 * D, D), 0.02), b_qkv=randn((3 * D,), 0.02),
                      w_proj=randn((D, D), 0.02), b_proj=randn((D,), 0.02),
                      ln2_g=randn((D,), 0.02, 1.0), ln2_b=randn((D,), 0.02),
                      w_fc1=randn((F, D), 0.02), b_fc1=randn((F,), 0.02),
                      w_fc2=randn((D, F), 0.02), b_fc2=randn((D,), 0.02))
            kc = torch.zeros((B, dims.H, L_cap, dims.dh), dtype=torch.bfloat16, device=dev)
            vc = torch.zeros((B, dims.H, dims.dh, L_cap), dtype=torch.bfloat16, device=dev)
            kc[:, :, :L0] = randn((B, dims.H, L0, dims.dh))
            vc[:, :, :, :L0] = randn((B, dims.H, dims.dh, L0))
            cache = randn((B, wl.hc * wl.hc, dims.D))
            cache_attn = randn((B, wl.hc * wl.hc, dims.D)) if wiring == "sublayer" else None
        blocks.append(dict(wt=wt, w=fb.make_weights(wt), kc=kc, vc=vc, cache=cache, cache_attn=cache_attn))

    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)
    ws_bytes = (fb.fastvar_step_sublayer_workspace_bytes(d, B, N, k, k) if wiring == "sublayer"
                else fb.fastvar_step_workspace_bytes(d, B, N, k))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)
    xa = up(host["x"])
    xb = torch.empty_like(xa)
    idx = torch.empty((B, max(k, 1)), dtype=torch.int32, device=dev)
    st = dict(host=host, blocks=blocks, d=d, ws=ws, x_in=xa.clone(), xa=xa, xb=xb, idx=idx, L_cap=L_cap,
              wiring=wiring)
    if wiring == "sublayer":
        st["x_mid"] = torch.empty_like(xa)
        st["idx2"] = torch.empty_like(idx)
    return st


def run_step(wl, st):
    """One pass of the stack at this scale: the output map of a block is the next block's input."""
    from paper_2503_23367_amd import binding as fb
    st["xa"].copy_(st["x_in"])          # same starting map every step (outside the kernels' work)
    sides = list(wl.sides)
    if st["wiring"] == "sublayer":
        src, dst = st["xa"], st["xb"]
        for blk in st["blocks"]:
            fb.fastvar_step_sublayer(src, sides, sides, wl.step, wl.cache_step, wl.B, wl.k, wl.k, st["d"],
                                     blk["w"], blk["kc"], blk["vc"], wl.L0_full, st["L_cap"], blk["cache_attn"],
                                     blk["cache"], st["x_mid"], dst, st["idx"], st["idx2"], st["ws"])
            src, dst = dst, src
        return src
    # the whole stack in one call: every block's caches start at the same prior length
    if "layers" not in st:
        st["layers"] = fb.make_layers(st["blocks"])
        st["tmp"] = st["xa"].new_empty(st["xa"].shape)
    fb.fastvar_scale_step(st["xa"], sides, sides, wl.step, wl.cache_step, wl.B, wl.k, st["d"], st["layers"],
                          wl.L0_full, st["L_cap"], st["xb"], st["tmp"], st["idx"], st["ws"])
    return st["xb"]


def time_kernel(fn, iters):
    """Average duration (ms) of `fn` launched back to back, from HIP events on
    the stream the kernels are enqueued on (torch's current stream)."""
    import torch
    fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def kernel_table(wl, st, iters, block_ms, only=None):
    """Every stage of a block, timed two ways with HIP events on the launch stream.
    `ms`: inside the running step, from the library's own stopwatch variant of the step entry point
    (an event after every stage, averaged over the blocks of the stack and three steps): operands are
    cold, as in the step the headline times, and it is what the rocprofv3 kernel trace of the step
    shows per kernel.  Recording an event between two kernels costs about 3 us of stream time that the
    untimed step does not have; it is taken out again: the difference between the sum of the stage
    times and the untimed step's time per block (`block_ms`), spread evenly over the stages.  `ms_back_to_back`: the same launch through the component entry points, repeated
    back to back (operands cache resident; the stand-alone restore also copies the kept rows, which
    inside the step the last GEMM writes in place)."""
    import torch
    from paper_2503_23367_amd import binding as fb
    dims = wl.dims
    B, N, k, D, F, H, dh = wl.B, wl.N, wl.k, dims.D, dims.F, dims.H, dims.dh
    M, L0, L = B * k, wl.L0_full, wl.L0_full + wl.k
    L_cap = st["L_cap"]
    blk, d = st["blocks"][0], st["d"]
    wt = blk["wt"]
    dev = "cuda:0"
    bf = torch.bfloat16
    sides = list(wl.sides)

    # ---- inside the step
    if "layers" not in st:
        st["layers"] = fb.make_layers(st["blocks"])
        st["tmp"] = st["xa"].new_empty(st["xa"].shape)
    in_step = {}
    reps = 0 if only is not None else 3
    for _ in range(reps):
        st["xa"].copy_(st["x_in"])
        _, ms = fb.fastvar_scale_step_timed(st["xa"], sides, sides, wl.step, wl.cache_step, B, k, d, st["layers"],
                                            L0, L_cap, st["xb"], st["tmp"], st["idx"], st["ws"])
        for n, v in ms.items():
            in_step[n] = in_step.get(n, 0.0) + v / reps

    launched = [n for n, v in in_step.items() if v > 0.0]
    event_ms = max(0.0, (sum(in_step.values()) - block_ms) / len(launched)) if launched else 0.0
    in_step = {n: (max(v - event_ms, 1e-6) if v > 0.0 else 0.0) for n, v in in_step.items()}

    # ---- back to back
    x = st["x_in"]
    idx = st["idx"]
    rank = torch.empty((B, N), dtype=torch.int32, device=dev)
    sel_ws = torch.empty(fb.fastvar_select_workspace_bytes(B, N, D), dtype=torch.uint8, device=dev)
    fb.fastvar_select_pivotal(x, B, wl.h, wl.h, D, k, idx, rank, None, sel_ws)
    a = torch.empty((M, D), dtype=bf, device=dev)
    q = torch.empty((M, D), dtype=bf, device=dev)
    o = torch.empty((M, D), dtype=bf, device=dev)
    h1 = torch.empty((M, D), dtype=bf, device=dev)
    u = torch.empty((M, F), dtype=bf, device=dev)
    yk = torch.empty((M, D), dtype=bf, device=dev)
    y = torch.empty((B, N, D), dtype=bf, device=dev)
    fb.fastvar_layernorm(x, idx, B, N, k, D, wt["ln1_g"], wt["ln1_b"], 1e-6, a)
    b2 = 2  # bytes per bf16
    rows = [
        ("select (colsum+score+topk)", "select", "hbm", B * N * D * b2,
         lambda: fb.fastvar_select_pivotal(x, B, wl.h, wl.h, D, k, idx, rank, None, sel_ws)),
        # inside a pruned step this launch also fills the pruned rows of the restored map (Eq. 6)
        ("gather+layernorm (+fill)", "gather+layernorm 1", "hbm",
         (2 * M * D + (B * (N - k) * D + B * wl.hc * wl.hc * D if k < N else 0)) * b2,
         lambda: fb.fastvar_layernorm(x, idx, B, N, k, D, wt["ln1_g"], wt["ln1_b"], 1e-6, a)),
        ("qkv gemm", "qkv gemm", "mfma", 2.0 * M * D * 3 * D,
         lambda: fb.fastvar_qkv_gemm(a, wt["w_qkv"], wt["b_qkv"], B, k, d, q, blk["kc"], blk["vc"], L0, L_cap)),
        ("attention", "attention", "mfma", 4.0 * B * k * L * D,
         lambda: fb.fastvar_attention(q, blk["kc"], blk["vc"], B, k, d, L, L_cap, o)),
        ("proj gemm", "proj gemm", "mfma", 2.0 * M * D * D,
         lambda: fb.fastvar_gemm_bf16(o, wt["w_proj"], wt["b_proj"], a, M, D, D, fb.EPI_BIAS_RES, h1)),
        ("layernorm 2", "layernorm 2", "hbm", 2 * M * D * b2,
         lambda: fb.fastvar_layernorm(h1, None, 1, 0, M, D, wt["ln2_g"], wt["ln2_b"], 1e-6, q)),
        ("fc1 gemm", "fc1 gemm", "mfma", 2.0 * M * D * F,
         lambda: fb.fastvar_gemm_bf16(q, wt["w_fc1"], wt["b_fc1"], None, M, F, D, fb.EPI_BIAS_GELU, u)),
        ("fc2 gemm", "fc2 gemm", "mfma", 2.0 * M * D * F,
         lambda: fb.fastvar_gemm_bf16(u, wt["w_fc2"], wt["b_fc2"], h1, M, D, F, fb.EPI_BIAS_RES, yk)),
        ("restore", "restore", "hbm", (B * N * D + M * D + B * wl.hc * wl.hc * D) * b2,
         lambda: fb.fastvar_restore(yk, idx, rank, B, k, blk["cache"], wl.hc, wl.hc, wl.h, wl.h, D, y)),
    ]
    if only is not None:
        # profiling aid: the named launch alone, back to back (operands cache resident), nothing else
        for name, stage, bound, work, fn in rows:
            if name == only:
                ms_iso = time_kernel(fn, iters)
                log(f"  {name}: {ms_iso*1e3:.1f} us per launch back to back over {iters} launches")
                return [dict(kernel=name, ms_back_to_back=round(ms_iso, 5), work=work)]
        raise SystemExit(f"bench.py: no stage named {only!r}; stages: {[r[0] for r in rows]}")
    out = []
    log(f"  {'stage':28s} {'in the step':>12s} {'back to back':>13s}   (achieved: from the in-step time)")
    for name, stage, bound, work, fn in rows:
        ms_iso = time_kernel(fn, iters)
        ms = in_step[stage]
        if ms < 1e-4:
            # no launch of its own inside the step (unpruned step: no selection; pruned step: the restoration's
            # fill rides in the gather + LayerNorm launch and the kept rows are written by the last GEMM)
            out.append(dict(kernel=name, bound=bound, ms=0.0, ms_back_to_back=round(ms_iso, 5), work=work,
                            achieved=None, peak=None, unit=None, frac=None, note="no launch of its own in the step"))
            log(f"  {name:28s} {'-':>12s} {ms_iso*1e3:10.1f} us  (no launch of its own inside the step)")
            continue
        if bound == "mfma":
            ach, peak, unit = work / (ms * 1e-3) / 1e12, PEAK_BF16_TFLOPS, "TFLOP/s"
        else:
            ach, peak, unit = work / (ms * 1e-3) / 1e9, PEAK_HBM_GBS, "GB/s"
        out.append(dict(kernel=name, bound=bound, ms=round(ms, 5), ms_back_to_back=round(ms_iso, 5), work=work,
                        achieved=round(ach, 2), peak=peak, unit=unit, frac=round(ach / peak, 4)))
        log(f"  {name:28s} {ms*1e3:9.1f} us {ms_iso*1e3:10.1f} us  {ach:9.1f} {unit:8s} {100*ach/peak:5.1f}% of peak")
    log(f"  (in-step times after taking out {event_ms*1e3:.1f} us of event cost per stage; "
        f"they sum to {sum(in_step.values())*1e3:.1f} us per block)")
    return out


# bench.py's kernel names -> prefix of the device kernel's name in the counter summary
_TRAFFIC_KEYS = {"attention": "attention_pipe_kernel", "qkv gemm": "gemm_nt_kernel<256, 192",
                 "fc1 gemm": "gemm_nt_kernel<256, 256", "restore": "restore_kernel"}


def counter_traffic(workload, kernel):
    """HBM-side bytes per launch of `kernel` from the committed rocprofv3 counter summary of this
    workload (FETCH_SIZE + WRITE_SIZE, scaled by a copy of known size), or None when there is none:
    hardware counters cannot be read from inside this process."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"pmc_traffic_{workload}.txt")
    key = _TRAFFIC_KEYS.get(kernel)
    if key is None or not os.path.exists(path):
        return None
    with open(path) as f:
        for line in f:
            if line.startswith("traffic_bytes " + key):
                return int(line.rsplit("=", 1)[1])
    return None


def cpu_baseline(wl, st, n_blocks, target_seconds=12.0, max_reps=16):
    """The oracle as it stands, on the host cores: one block of the same workload (select + block +
    restore in fp64 NumPy), repeated until about `target_seconds` of CPU work have been timed."""
    from oracle import fastvar_oracle as O
    h = st["host"]
    times = []
    while len(times) < max_reps and (not times or sum(times) < target_seconds):
        t0 = time.perf_counter()
        if st["wiring"] == "sublayer":
            O.step_sublayer(h["x"], wl.h, wl.h, wl.k, wl.k, h["W"], wl.dims.H, h["kp"], h["vp"], h["cache_attn"],
                            h["cache"], wl.hc, wl.hc)
        else:
            O.step(h["x"], wl.h, wl.h, wl.k, h["W"], wl.dims.H, h["kp"], h["vp"], h["cache"], wl.hc, wl.hc)
        times.append(time.perf_counter() - t0)
    dt = sum(times) / len(times)
    cores = len(os.sched_getaffinity(0))
    try:
        from threadpoolctl import threadpool_info
        blas = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas = cores
    est_step = dt * n_blocks
    return dict(value=round(wl.B * wl.N / est_step, 3), unit="tokens/s", cores=min(cores, blas), kind="oracle",
                sample=f"one block of {n_blocks} ({'sub-layer wiring' if st['wiring'] == 'sublayer' else 'select+block+restore'}, fp64 NumPy) run {len(times)} times, "
                       f"{sum(times):.1f} s in all, mean {dt:.2f} s; stack time estimated as block time x {n_blocks}",
                block_seconds=round(dt, 3), affinity_cores=cores, blas_threads=blas)


def schedule_bench(wl, n_blocks, steps, warmup, keeps=(0.6, 0.5, 0.0, 0.0), graphs=False):
    """The whole scale schedule of the workload's model through fastvar_scale_step, twice: every step
    unpruned, and with the last len(keeps) steps pruned to the given keep ratios after a cache capture
    at the step before them (the paper's setting for this model: pruning ratios 40, 50, 100, 100 % on
    the last four steps).  Token maps are seeded synthetic ones per scale (the tokenizer and the
    residual accumulation between scales are outside the library).  graphs: every scale's call is captured
    into a HIP graph once (the library allocates nothing and clears its counters with a kernel, so its calls
    can be captured) and the timed images replay the graphs: the small scales are bound by launches, not by
    work.  Returns a dict for the JSON line."""
    import torch
    from paper_2503_23367_amd import binding as fb
    dev = "cuda:0"
    dims, B, sides = wl.dims, wl.B, list(wl.sides)
    K = len(sides)
    cache_step = K - len(keeps) - 1
    hc = sides[cache_step]
    L_cap = (sum(s * s for s in sides) + 7) // 8 * 8
    gen = torch.Generator(device=dev)
    gen.manual_seed(777)

    def randn(shape, std=1.0, mean=0.0):
        return (torch.randn(shape, generator=gen, device=dev, dtype=torch.float32) * std + mean).to(torch.bfloat16)

    D, F = dims.D, dims.F
    layers = []
    for _ in range(n_blocks):
        wt = dict(ln1_g=randn((D,), 0.02, 1.0), ln1_b=randn((D,), 0.02),
                  w_qkv=randn((3 * D, D), 0.02), b_qkv=randn((3 * D,), 0.02),
                  w_proj=randn((D, D), 0.02), b_proj=randn((D,), 0.02),
                  ln2_g=randn((D,), 0.02, 1.0), ln2_b=randn((D,), 0.02),
                  w_fc1=randn((F, D), 0.02), b_fc1=randn((F,), 0.02),
                  w_fc2=randn((D, F), 0.02), b_fc2=randn((D,), 0.02))
        layers.append(dict(wt=wt, w=fb.make_weights(wt),
                           kc=torch.zeros((B, dims.H, L_cap, dims.dh), dtype=torch.bfloat16, device=dev),
                           vc=torch.zeros((B, dims.H, dims.dh, L_cap), dtype=torch.bfloat16, device=dev),
                           cache=torch.zeros((B, hc * hc, D), dtype=torch.bfloat16, device=dev)))
    arr = fb.make_layers(layers)
    d = fb.make_dims(dims.D, dims.H, dims.dh, dims.F)

    def up(a):
        bits = synth.to_bf16_bits(a).astype(np.int16)
        return torch.from_numpy(bits).to(dev).view(torch.bfloat16).reshape(a.shape)

    xs = [up(synth.token_map(100 + i, B, s, s, D)) for i, s in enumerate(sides)]
    Nmax = sides[-1] ** 2
    y = torch.empty((B, Nmax, D), dtype=torch.bfloat16, device=dev)
    tmp = torch.empty_like(y)
    idx = torch.empty((B, Nmax), dtype=torch.int32, device=dev)

    def k_of(i, pruned):
        N = sides[i] ** 2
        return fb.fastvar_keep_count(N, keeps[i - cache_step - 1]) if pruned and i > cache_step else N

    # one scratch buffer for every step of both runs: the sizes are not monotone in the kept count
    ws_bytes = max(fb.fastvar_step_workspace_bytes(d, B, sides[i] ** 2, k_of(i, pruned))
                   for i in range(K) for pruned in (False, True))
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev)

    captured = {}

    def capture(pruned):
        """One graph per scale; an eager call first, so that nothing happens for the first time under capture."""
        kv = 0
        for i in range(K):
            args = (xs[i], sides, sides, i, cache_step, B, k_of(i, pruned), d, arr, kv, L_cap, y, tmp, idx, ws)
            kv_next = fb.fastvar_scale_step(*args)
            torch.cuda.synchronize()
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                fb.fastvar_scale_step(*args)
            captured[(pruned, i)] = g
            kv = kv_next

    def one_image(pruned, stamps=None):
        kv = 0
        for i in range(K):
            if stamps is not None:
                stamps[i].record()
            if graphs:
                captured[(pruned, i)].replay()
                kv += k_of(i, pruned)
            else:
                kv = fb.fastvar_scale_step(xs[i], sides, sides, i, cache_step, B, k_of(i, pruned), d, arr, kv,
                                           L_cap, y, tmp, idx, ws)
        if stamps is not None:
            stamps[K].record()
        return kv

    out = {}
    for name, pruned in (("unpruned", False), ("fastvar", True)):
        if graphs:
            capture(pruned)
        for _ in range(warmup):
            one_image(pruned)
        torch.cuda.synchronize()
        ev = [[torch.cuda.Event(enable_timing=True) for _ in range(K + 1)] for _ in range(steps)]
        t0 = time.perf_counter()
        for r in range(steps):
            kv = one_image(pruned, ev[r])
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3 / steps
        per_step = [sum(ev[r][i].elapsed_time(ev[r][i + 1]) for r in range(steps)) / steps for i in range(K)]
        out[name] = dict(ms_per_image=round(wall, 3), kv_tokens=kv, ms_per_scale=[round(v, 3) for v in per_step],
                         kept=[k_of(i, pruned) for i in range(K)])
        log(f"{name}: {wall:.2f} ms per image; per scale " + " ".join(f"{v:.2f}" for v in per_step))
    out["speedup"] = round(out["unpruned"]["ms_per_image"] / out["fastvar"]["ms_per_image"], 3)
    out["last_two_scales_share_unpruned"] = round(sum(out["unpruned"]["ms_per_scale"][-2:]) /
                                                  sum(out["unpruned"]["ms_per_scale"]), 3)
    return dict(sides=sides, cache_step=cache_step, keep_ratios=list(keeps), blocks=n_blocks, hip_graphs=bool(graphs),
                **out)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=synth.HEADLINE, choices=sorted(synth.WORKLOADS))
    ap.add_argument("--blocks", type=int, default=0, help="blocks in the stack (default: the workload's)")
    ap.add_argument("--wiring", default="block", choices=("block", "sublayer"),
                    help="one selection/restoration pair around the block (the headline), or one around "
                         "each of its two layers")
    ap.add_argument("--schedule", action="store_true",
                    help="instead of the headline step: the model's whole scale schedule, unpruned and with the "
                         "last four steps pruned (one JSON line of its own)")
    ap.add_argument("--graphs", action="store_true",
                    help="with --schedule: capture every scale's call into a HIP graph once and replay the graphs")
    ap.add_argument("--kernel-iters", type=int, default=20)
    ap.add_argument("--kernel-loop", default=None, metavar="STAGE",
                    help="profiling aid: run only this stage of the kernel table (e.g. 'qkv gemm') back to back "
                         "--kernel-iters times through its component entry point and exit, no step and no JSON "
                         "line: what a counter run of the stage with cache-resident operands is taken from")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-kernel-table", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)

    import torch
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        sys.exit(1)
    from paper_2503_23367_amd import binding as fb
    fb.lib()
    torch.cuda.set_device(0)

    wl = synth.WORKLOADS[args.workload]
    n_blocks = args.blocks or wl.n_blocks
    log(f"workload {wl.name}: B={wl.B} N={wl.N} k={wl.k} L0={wl.L0_full} D={wl.dims.D} blocks={n_blocks}")
    if args.schedule:
        res = schedule_bench(wl, n_blocks, args.steps, args.warmup, graphs=args.graphs)
        print(json.dumps({"metric": "whole scale schedule, transformer stack only: ms per image unpruned vs "
                                    "FastVAR pruning schedule", "value": res["speedup"], "unit": "x (unpruned / pruned)",
                          "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                          "ms_per_step": res["fastvar"]["ms_per_image"], "higher_is_better": True, "scaling": "weak",
                          "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
                          "config": {"workload": wl.name + " (all scales)", **{k: res[k] for k in
                                     ("sides", "cache_step", "keep_ratios", "blocks")}},
                          "schedule": {k: res[k] for k in ("unpruned", "fastvar", "speedup",
                                                             "last_two_scales_share_unpruned", "hip_graphs")}}), flush=True)
        return
    t0 = time.perf_counter()
    st = build_state(wl, n_blocks, wiring=args.wiring)
    torch.cuda.synchronize()
    log(f"inputs resident after {time.perf_counter()-t0:.1f} s; "
        f"HBM in use {torch.cuda.memory_allocated()/2**30:.2f} GiB")

    if args.kernel_loop:
        kernel_table(wl, st, args.kernel_iters, 0.0, only=args.kernel_loop)
        return
    for _ in range(args.warmup):
        run_step(wl, st)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(args.steps):
        run_step(wl, st)
    e1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_ms = e0.elapsed_time(e1) / args.steps
    ms = max(wall_ms, ev_ms)
    log(f"step: {ms:.3f} ms wall ({ev_ms:.3f} ms by events), {ms/n_blocks*1e3:.1f} us per block")

    kernels = [] if (args.no_kernel_table or args.wiring != "block") else kernel_table(wl, st, args.kernel_iters, ms / n_blocks)
    roofline = None
    if kernels:
        dom = max(kernels, key=lambda r: r["ms"])   # rows without a launch of their own have ms = 0
        roofline = dict(kernel=dom["kernel"], bound=dom["bound"], achieved=dom["achieved"], peak=dom["peak"],
                        unit=dom["unit"], frac=dom["frac"], traffic=counter_traffic(wl.name, dom["kernel"]),
                        launch_ms=dom["ms"])
    cpu = None if args.no_cpu_baseline else cpu_baseline(wl, st, n_blocks)

    dims = wl.dims
    M = wl.B * wl.k
    flops_block = 2.0 * M * (4 * dims.D * dims.D + 2 * dims.D * dims.F) + 4.0 * wl.B * wl.k * (wl.L0_full + wl.k) * dims.D
    rec = {
        "metric": "last-scale step ms + effective tokens/s (1024px, keep 0.5); MFMA/HBM % peak",
        "value": round(wl.B * wl.N / (ms * 1e-3), 1),
        "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": wl.name, "B": wl.B, "tokens": wl.N, "kept": wl.k, "prior_cache_tokens": wl.L0_full,
                   "D": dims.D, "heads": dims.H, "head_dim": dims.dh, "mlp": dims.F, "blocks": n_blocks,
                   "wiring": args.wiring,
                   "step": ("select -> block on kept tokens -> restore, every block of the stack"
                            if args.wiring == "block" else
                            "select -> attention layer on kept tokens -> restore -> select -> FFN layer on kept "
                            "tokens -> restore, every block of the stack")},
        "processed_tokens_per_s": round(wl.B * wl.k / (ms * 1e-3), 1),
        "us_per_block": round(ms / n_blocks * 1e3, 2),
        "mfma_frac_whole_block": round(flops_block * n_blocks / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kernels,
    }
    print(json.dumps(rec), flush=True)


if __name__ == "__main__":
    main()
