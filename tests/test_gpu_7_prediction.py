"""GPU parity: fastvar_residual_accumulate vs the CPU oracle (Sec. 3.1, Eq. 2; skipped steps per Sec. 4.1).

Bar: the device evaluates the bilinear resampling and the add in fp32 on fp32 maps, the oracle in fp64 on the
same values, so every element agrees to a few fp32 roundings of the operands' magnitude
(|err| <= 1e-6 * (max|r_prev| + max|f_k|) per step; a chain of steps is allowed that much per step).
"""
import numpy as np
import pytest
import torch

from oracle import fastvar_oracle as O
from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth
from gpu_util import DEV, to_dev_bf16

pytestmark = pytest.mark.gpu


def _run(r_prev, hp, wp, f_k, h, w, B, C):
    rp = None if r_prev is None else torch.from_numpy(np.ascontiguousarray(r_prev, np.float32)).to(DEV)
    fk = None if f_k is None else to_dev_bf16(f_k)
    out = torch.full((B, h * w, C), float("nan"), dtype=torch.float32, device=DEV)
    fb.fastvar_residual_accumulate(rp, hp, wp, fk, h, w, B, C, out)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def _inputs(seed, B, hp, wp, h, w, C):
    rng = np.random.default_rng(seed)
    r = (3.0 * rng.standard_normal((B, hp * wp, C))).astype(np.float32)
    f = synth.round_bf16(rng.standard_normal((B, h * w, C)).astype(np.float32))
    return r, f


CASES = [  # B, hp, wp, h, w, C
    (1, 1, 1, 2, 2, 4), (2, 24, 24, 32, 32, 32), (1, 48, 48, 64, 64, 32), (3, 5, 3, 7, 9, 8),
    (1, 16, 16, 16, 16, 64), (1, 64, 64, 40, 40, 32), (1, 8, 8, 12, 12, 2048), (2, 3, 7, 11, 5, 12),
    (1, 64, 64, 128, 128, 32),
]


@pytest.mark.parametrize("B,hp,wp,h,w,C", CASES)
def test_residual_accumulate_matches_oracle(B, hp, wp, h, w, C):
    print(f"[residual_accumulate] B={B} prev={hp}x{wp} map={h}x{w} C={C}", flush=True)
    r, f = _inputs(B * 1000 + h, B, hp, wp, h, w, C)
    bound = 1e-6 * (np.abs(r).max() + np.abs(f).max())
    got = _run(r, hp, wp, f, h, w, B, C)
    ref = O.residual_accumulate(r, hp, wp, f, h, w)
    assert not np.isnan(got).any()
    assert np.abs(got - ref).max() <= bound
    # skipped step: interpolation alone
    got = _run(r, hp, wp, None, h, w, B, C)
    assert np.abs(got - O.residual_accumulate(r, hp, wp, None, h, w)).max() <= bound
    # first step: the residual itself, exactly
    got = _run(None, 0, 0, f, h, w, B, C)
    np.testing.assert_array_equal(got, f)


def test_equal_sizes_is_an_exact_add():
    r, f = _inputs(3, 2, 9, 7, 9, 7, 16)
    got = _run(r, 9, 7, f, 9, 7, 2, 16)
    np.testing.assert_array_equal(got, r + f)          # taps coincide, weights are 0: fp32 add of the same operands


def test_thirteen_step_chain_with_the_last_two_steps_skipped():
    sides = synth.WORKLOADS[synth.HEADLINE].sides
    keep, cached = fb.fastvar_schedule_plan(sides, sides, (0.4, 0.5, 1.0, 1.0))
    assert cached == 8 and keep[-2:] == [0, 0]
    B, C = 1, 32
    rng = np.random.default_rng(11)
    fs = [synth.round_bf16(rng.standard_normal((B, s * s, C)).astype(np.float32)) for s in sides]
    dev, ref, prev = None, None, 0
    scale = 0.0
    for i, s in enumerate(sides):
        f = None if keep[i] == 0 else fs[i]
        print(f"[residual chain] step {i} side {s} {'skipped' if f is None else 'residual added'}", flush=True)
        dev = _run(dev, prev, prev, f, s, s, B, C)                 # the device's own fp32 map feeds the next step
        ref = O.residual_accumulate(ref, prev, prev, f, s, s)
        prev = s
        scale += np.abs(fs[i]).max()
        assert np.abs(dev - ref).max() <= 1e-6 * scale * (i + 1)
    assert dev.shape == (B, 64 * 64, C)


def test_argument_errors():
    r = torch.zeros((1, 4, 8), dtype=torch.float32, device=DEV)
    f = torch.zeros((1, 16, 8), dtype=torch.bfloat16, device=DEV)
    out = torch.zeros((1, 16, 8), dtype=torch.float32, device=DEV)

    def code(*a):
        with pytest.raises(fb.FastvarError) as e:
            fb.fastvar_residual_accumulate(*a)
        return e.value.code

    assert code(None, 0, 0, None, 4, 4, 1, 8, out) == fb.FASTVAR_EINVAL          # neither term
    assert code(r, 2, 2, f, 4, 4, 1, 8, None) == fb.FASTVAR_EINVAL
    assert code(r, 0, 2, f, 4, 4, 1, 8, out) == fb.FASTVAR_EINVAL
    assert code(r, 2, 2, f, 4, 4, 1, 6, out) == fb.FASTVAR_EALIGN                 # C not a multiple of 4
    assert code(out, 4, 4, f, 4, 4, 1, 8, out) == fb.FASTVAR_EINVAL               # in place
    assert code(r, 2, 2, f, 256, 256, 1, 8, out) == fb.FASTVAR_ECAPACITY          # 65536 tokens
    assert code(r[:, :, 1:], 2, 2, f, 4, 4, 1, 4, out) == fb.FASTVAR_EALIGN       # pointer off by 4 bytes
