"""GPU parity: fastvar_select_pivotal vs the CPU oracle (Sec. 3.3, Eq. 4-5).

Bar: index sets bit-exact; both sides take the top-k decision on the score
rounded to fp32; only tokens whose oracle score lies within 1e-6 (relative)
of the k-th largest are exempt when the k-th and (k+1)-th are that close.
Exact ties (constant maps) are not exempt.
"""
import sys

import numpy as np
import pytest
import torch

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth
from gpu_util import DEV, empty_ws, to_dev_bf16

pytestmark = pytest.mark.gpu


def run_select(x_np, h, w, k, want_rank=True, want_score=True):
    B, N, D = x_np.shape
    x = to_dev_bf16(x_np)
    idx = torch.full((B, max(k, 1)), -7, dtype=torch.int32, device=DEV)
    rank = torch.full((B, N), -7, dtype=torch.int32, device=DEV) if want_rank else None
    score = torch.full((B, N), -7.0, dtype=torch.float32, device=DEV) if want_score else None
    ws = empty_ws(fb.fastvar_select_workspace_bytes(B, N, D))
    fb.fastvar_select_pivotal(x, B, h, w, D, k, idx, rank, score, ws)
    torch.cuda.synchronize()
    return (idx[:, :k].cpu().numpy(), None if rank is None else rank.cpu().numpy(),
            None if score is None else score.cpu().numpy())


def check_against_oracle(x_np, h, w, k, name):
    print(f"[select] {name} B={x_np.shape[0]} h={h} w={w} D={x_np.shape[2]} k={k}", flush=True)
    idx_g, rank_g, s_g = run_select(x_np, h, w, k)
    idx_o, rank_o, s_o = O.select_pivotal(x_np, k)
    B, N, _ = x_np.shape
    # scores: fp64 accumulation on both sides, one rounding to fp32
    ulp = np.spacing(np.abs(s_o).astype(np.float32))
    assert np.all(np.abs(s_g.astype(np.float64) - s_o.astype(np.float64)) <= ulp), name
    for b in range(B):
        # self-consistency: the GPU's index set is the stable top-k of its own scores
        own = O.topk_indices(s_g[b:b + 1], k)[0]
        np.testing.assert_array_equal(idx_g[b], own, err_msg=f"{name} sample {b}: not top-k of own scores")
        if not np.array_equal(idx_g[b], idx_o[b]):
            # allowed only for near-ties at the threshold
            srt = np.sort(s_o[b].astype(np.float64))[::-1]
            T, Tn = srt[k - 1], srt[k]
            assert T > 0 and (T - Tn) / T < 1e-6, f"{name} sample {b}: index sets differ without a near-tie"
            near = np.abs(s_o[b].astype(np.float64) - T) <= 1e-6 * T
            a = set(idx_g[b].tolist()) - set(np.nonzero(near)[0].tolist())
            c = set(idx_o[b].tolist()) - set(np.nonzero(near)[0].tolist())
            assert a == c, f"{name} sample {b}: index sets differ outside the near-tie band"
        # rank is the inverse of idx
        want_rank = np.full(N, -1, np.int32)
        want_rank[idx_g[b]] = np.arange(k, dtype=np.int32)
        np.testing.assert_array_equal(rank_g[b], want_rank, err_msg=name)
        assert np.all(np.diff(idx_g[b]) > 0)
    return idx_g, s_g


CASES = [
    # name, B, h, w, D, k, kind
    ("d16_last_scale", 1, 16, 16, 1024, 128, "smooth_spike"),
    ("d30_s24_b8", 8, 24, 24, 1920, 346, "smooth_spike"),
    ("d30_s32_b8", 8, 32, 32, 1920, 410, "smooth_spike"),
    ("ragged_small_D200", 2, 7, 9, 200, 20, "smooth_spike"),
    ("ragged_D520_k1", 3, 5, 13, 520, 1, "smooth_spike"),
    ("single_token", 2, 1, 1, 64, 1, "smooth_spike"),
    ("keep_none", 2, 8, 8, 128, 0, "smooth_spike"),
    ("keep_all", 2, 8, 8, 128, 64, "smooth_spike"),
    ("inf2b_s64_keep0.5", 1, 64, 64, 2048, 2048, "smooth_spike"),
    ("inf2b_s64_keep0.1", 1, 64, 64, 2048, 410, "smooth_spike"),
    ("inf2b_s64_all_spike", 1, 64, 64, 2048, 2048, "all_spike"),
    ("inf2b_s48_b4", 4, 48, 48, 2048, 1152, "smooth_spike"),
    ("inf2b_2k_s128", 1, 128, 128, 2048, 4096, "smooth_spike"),
    ("max_tokens_narrow", 1, 128, 256, 64, 5000, "smooth_spike"),
    ("wide_D8192", 1, 6, 6, 8192, 9, "smooth_spike"),
]


@pytest.mark.parametrize("name,B,h,w,D,k,kind", CASES, ids=[c[0] for c in CASES])
def test_select_matches_oracle(name, B, h, w, D, k, kind):
    x = synth.token_map(11, B, h, w, D, kind=kind)
    check_against_oracle(x, h, w, k, name)


@pytest.mark.parametrize("k", [0, 1, 410, 2048, 4095, 4096])
def test_constant_map_ties_break_to_lowest_index(k):
    print(f"[select] constant map 64x64 k={k}", flush=True)
    x = synth.token_map(3, 2, 64, 64, 2048, kind="constant")
    idx, rank, s = run_select(x, 64, 64, k)
    assert np.all(s == 0.0)
    np.testing.assert_array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (2, 1)))
    want = np.where(np.arange(4096) < k, np.arange(4096), -1).astype(np.int32)
    np.testing.assert_array_equal(rank, np.tile(want, (2, 1)))


def test_many_exact_ties_at_threshold():
    # tokens take only a few distinct values -> scores tie in large groups
    print("[select] quantised map with tie groups", flush=True)
    rng = np.random.default_rng(5)
    base = synth.round_bf16(rng.standard_normal((4, 256)).astype(np.float32))
    pick = rng.integers(0, 4, size=(2, 40 * 40))
    x = base[pick]                                    # [2, 1600, 256]
    for k in (1, 399, 400, 401, 800, 1599):
        check_against_oracle(x, 40, 40, k, f"tie_groups_k{k}")


def test_select_is_bit_reproducible_and_optional_outputs():
    print("[select] reproducibility", flush=True)
    x = synth.token_map(21, 2, 48, 48, 2048)
    i0, r0, s0 = run_select(x, 48, 48, 1152)
    for _ in range(5):
        i1, r1, s1 = run_select(x, 48, 48, 1152)
        assert np.array_equal(i0, i1) and np.array_equal(r0, r1)
        assert np.array_equal(s0.view(np.uint32), s1.view(np.uint32))
    i2, r2, s2 = run_select(x, 48, 48, 1152, want_rank=False, want_score=False)
    assert r2 is None and s2 is None and np.array_equal(i0, i2)


def test_shift_invariance_on_gpu():
    print("[select] DC shift invariance", flush=True)
    rng = np.random.default_rng(9)
    # values on a coarse grid so that x + c stays exactly representable in bf16
    x = (rng.integers(-8, 9, size=(1, 24 * 24, 512)) / 8.0).astype(np.float32)
    c = (rng.integers(-4, 5, size=(1, 1, 512)) / 4.0).astype(np.float32)
    i0, _, s0 = run_select(x, 24, 24, 200)
    i1, _, s1 = run_select(x + c, 24, 24, 200)
    np.testing.assert_array_equal(i0, i1)
    np.testing.assert_array_equal(s0, s1)


def test_select_argument_errors_touch_nothing():
    print("[select] error paths", flush=True)
    x = to_dev_bf16(synth.token_map(1, 1, 4, 4, 64))
    idx = torch.full((1, 16), -7, dtype=torch.int32, device=DEV)
    ws = empty_ws(fb.fastvar_select_workspace_bytes(1, 16, 64))
    L = fb.lib()
    st = torch.cuda.current_stream().cuda_stream
    nb = ws.numel()
    assert L.fastvar_select_pivotal(x.data_ptr(), 1, 4, 4, 64, 17, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(x.data_ptr(), 1, 4, 4, 64, -1, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(None, 1, 4, 4, 64, 4, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal(x.data_ptr(), 1, 4, 4, 64, 4, idx.data_ptr(), None, None, ws.data_ptr(), 16, st) == fb.FASTVAR_EWORKSPACE
    assert L.fastvar_select_pivotal(x.data_ptr() + 2, 1, 4, 4, 64, 4, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_EALIGN
    assert L.fastvar_select_pivotal(x.data_ptr(), 1, 4, 4, 60, 4, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_EALIGN
    assert L.fastvar_select_pivotal(x.data_ptr(), 1, 256, 256, 64, 4, idx.data_ptr(), None, None, ws.data_ptr(), nb, st) == fb.FASTVAR_ECAPACITY
    torch.cuda.synchronize()
    assert torch.all(idx == -7)
