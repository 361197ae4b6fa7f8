"""GPU check of fastvar_select_pivotal_static, the selection entry point that allocates nothing (its scratch
is a device array inside the library): same index set, rank map and scores, bit for bit, as
fastvar_select_pivotal with a caller-provided scratch buffer.  Two calls in a row, the second on a smaller
map (the array keeps the first call's contents), then a third on the first map again; a request beyond the
array's size is refused before anything is launched."""
import numpy as np
import pytest
import torch

from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth
from gpu_util import DEV, empty_ws, to_dev_bf16

pytestmark = pytest.mark.gpu


def _both(x, B, h, w, D, k):
    N = h * w
    out = []
    for static in (False, True):
        idx = torch.full((B, max(k, 1)), -7, dtype=torch.int32, device=DEV)
        rank = torch.full((B, N), -7, dtype=torch.int32, device=DEV)
        score = torch.full((B, N), float("nan"), dtype=torch.float32, device=DEV)
        if static:
            fb.fastvar_select_pivotal_static(x, B, h, w, D, k, idx, rank, score)
        else:
            ws = empty_ws(fb.fastvar_select_workspace_bytes(B, N, D))
            ws.fill_(0xFF)
            fb.fastvar_select_pivotal(x, B, h, w, D, k, idx, rank, score, ws)
        torch.cuda.synchronize()
        out.append((idx.cpu().numpy(), rank.cpu().numpy(), score.cpu().numpy().view(np.uint32)))
    return out


def test_static_scratch_select_equals_the_workspace_one():
    cases = [(1, 64, 64, 2048, 2048, 5),     # the headline map: 2 MiB of partials
             (2, 24, 24, 1920, 346, 6),      # smaller, batched, other width: reuses the array as it was left
             (1, 64, 64, 2048, 410, 5)]      # the first map again, other k
    for B, h, w, D, k, seed in cases:
        print(f"[no-alloc select] B={B} {h}x{w} D={D} k={k}", flush=True)
        x = to_dev_bf16(synth.token_map(seed, B, h, w, D))
        (i0, r0, s0), (i1, r1, s1) = _both(x, B, h, w, D, k)
        assert np.array_equal(i0, i1) and np.array_equal(r0, r1) and np.array_equal(s0, s1)
        assert (i1[:, :k] >= 0).all() and (np.diff(i1[:, :k], axis=1) > 0).all()
    # optional outputs may be NULL (the scores then live in the array too)
    B, h, w, D, k, seed = cases[0]
    x = to_dev_bf16(synth.token_map(seed, B, h, w, D))
    idx = torch.full((B, k), -7, dtype=torch.int32, device=DEV)
    fb.fastvar_select_pivotal_static(x, B, h, w, D, k, idx, None, None)
    torch.cuda.synchronize()
    (i0, _, _), _ = _both(x, B, h, w, D, k)
    assert np.array_equal(idx.cpu().numpy(), i0)


def test_static_scratch_select_refuses_what_does_not_fit():
    B, h, w, D = 4, 128, 128, 2048        # 4 x 256 chunks x 2048 x 8 bytes = 16 MiB of partials
    assert fb.fastvar_select_workspace_bytes(B, h * w, D) > fb.FASTVAR_SELECT_STATIC_BYTES
    x = to_dev_bf16(np.zeros((1, 16, 64), np.float32))    # never read: the sizes are refused first
    idx = torch.full((B, 8), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(fb.FastvarError) as e:
        fb.fastvar_select_pivotal_static(x, B, h, w, D, 8, idx, None, None)
    assert e.value.code == fb.FASTVAR_ECAPACITY
    # the ordinary argument errors, as in fastvar_select_pivotal
    L = fb.lib()
    st = torch.cuda.current_stream().cuda_stream
    assert L.fastvar_select_pivotal_static(None, 1, 4, 4, 64, 4, idx.data_ptr(), None, None, st) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal_static(x.data_ptr(), 1, 4, 4, 64, 17, idx.data_ptr(), None, None, st) == fb.FASTVAR_EINVAL
    assert L.fastvar_select_pivotal_static(x.data_ptr(), 1, 4, 4, 60, 4, idx.data_ptr(), None, None, st) == fb.FASTVAR_EALIGN
    torch.cuda.synchronize()
    assert torch.all(idx == -7)
