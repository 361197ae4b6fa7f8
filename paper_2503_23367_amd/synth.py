"""Seeded synthetic inputs for the pruned VAR decoding step.

This module only manufactures inputs (token maps, cached maps, prior K/V,
block weights) and names the workload shapes.  It holds none of the method's
arithmetic: no scoring, no selection, no block math, no restoration.  Both the
HIP path's tests/bench and the CPU oracle's tests draw their inputs from here
so that the two sides see bit-identical values.

Every tensor is drawn in fp32 with ``numpy.random.default_rng(seed)`` and then
rounded to the nearest bf16 (ties to even); the fp32 arrays returned are
therefore exactly representable in bf16, and ``to_bf16_bits`` gives the 16-bit
patterns to upload.

The shapes follow the paper's workloads (next-scale-prediction schedules of
VAR-d16/d30 at 256/512 px, Infinity-2B at 1024 px and its zero-shot 2K
extension, Sec. 4.1 / 4.4 / Suppl. A); the values are synthetic stand-ins for
the real models' activations: a smooth low-frequency field plus sparse
high-frequency spikes, which is the structure Sec. 3.2 (Observation 2)
describes for large-scale token maps.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Tuple

import numpy as np

# --------------------------------------------------------------------------
# bf16 helpers (pure bit manipulation)
# --------------------------------------------------------------------------


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round-to-nearest-even."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> fp32 array (exact widening)."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_bf16(a: np.ndarray) -> np.ndarray:
    """fp32 array rounded to the nearest bf16 value, returned as fp32."""
    return from_bf16_bits(to_bf16_bits(a))


# --------------------------------------------------------------------------
# workload shapes
# --------------------------------------------------------------------------


@dataclass(frozen=True)
class BlockDims:
    D: int   # model width
    H: int   # attention heads
    dh: int  # head dim (D == H*dh)
    F: int   # MLP hidden width


@dataclass(frozen=True)
class Workload:
    """One pruned decoding step of one block: a scale of a schedule."""
    name: str
    dims: BlockDims
    sides: Tuple[int, ...]      # square scale schedule (h_k = w_k = sides[k])
    step: int                   # index into sides of the scale being decoded
    cache_step: int             # index of the last unpruned scale (K - N)
    keep_ratio: float
    k: int                      # kept tokens per sample at this step
    B: int = 1
    n_blocks: int = 1
    # keep counts of earlier pruned steps (same order as the schedule tail)
    prior_k: Dict[int, int] = field(default_factory=dict)

    @property
    def h(self) -> int:
        return self.sides[self.step]

    @property
    def N(self) -> int:
        return self.sides[self.step] ** 2

    @property
    def hc(self) -> int:
        return self.sides[self.cache_step]

    @property
    def L0_full(self) -> int:
        """Prior tokens if every earlier scale entered the cache whole."""
        return sum(s * s for s in self.sides[: self.step])

    @property
    def L0_pruned(self) -> int:
        """Prior tokens when earlier pruned scales cached only kept tokens."""
        return sum(self.prior_k.get(i, s * s)
                   for i, s in enumerate(self.sides[: self.step]))


D16 = BlockDims(D=1024, H=16, dh=64, F=4096)
D30 = BlockDims(D=1920, H=30, dh=64, F=7680)
INF2B = BlockDims(D=2048, H=16, dh=128, F=8192)

SIDES_256 = (1, 2, 3, 4, 5, 6, 8, 10, 13, 16)
SIDES_512 = (1, 2, 3, 4, 6, 9, 13, 18, 24, 32)
SIDES_1024 = (1, 2, 4, 6, 8, 12, 16, 20, 24, 32, 40, 48, 64)
SIDES_2K = SIDES_1024 + (80, 96, 128)

WORKLOADS: Dict[str, Workload] = {}


def _add(w: Workload) -> None:
    WORKLOADS[w.name] = w


# VAR-d16-style block, last step of the 256 px schedule.
_add(Workload("d16_256px_s16_keep0.5", D16, SIDES_256, 9, 8, 0.5, 128))
# VAR-d30-style at 512 px, last two scales pruned, batch 8.
_add(Workload("d30_512px_s24_keep0.6", D30, SIDES_512, 8, 7, 0.6, 346, B=8, n_blocks=30))
_add(Workload("d30_512px_s32_keep0.4", D30, SIDES_512, 9, 7, 0.4, 410, B=8, n_blocks=30,
              prior_k={8: 346}))
# Infinity-2B-style at 1024 px, last three scales pruned.
_add(Workload("inf2b_1024px_s40_keep0.6", INF2B, SIDES_1024, 10, 9, 0.6, 960, n_blocks=32))
_add(Workload("inf2b_1024px_s48_keep0.5", INF2B, SIDES_1024, 11, 9, 0.5, 1152, n_blocks=32,
              prior_k={10: 960}))
_add(Workload("inf2b_1024px_s64_keep0.4", INF2B, SIDES_1024, 12, 9, 0.4, 1638, n_blocks=32,
              prior_k={10: 960, 11: 1152}))
# The same three pruned scales at batch 4.
_add(Workload("inf2b_1024px_s40_keep0.6_b4", INF2B, SIDES_1024, 10, 9, 0.6, 960, B=4, n_blocks=32))
_add(Workload("inf2b_1024px_s48_keep0.5_b4", INF2B, SIDES_1024, 11, 9, 0.5, 1152, B=4, n_blocks=32,
              prior_k={10: 960}))
_add(Workload("inf2b_1024px_s64_keep0.4_b4", INF2B, SIDES_1024, 12, 9, 0.4, 1638, B=4, n_blocks=32,
              prior_k={10: 960, 11: 1152}))
# Zero-shot 2K extension of the same stack.
_add(Workload("inf2b_2k_s80_keep0.4", INF2B, SIDES_2K, 13, 12, 0.4, 2560, n_blocks=32))
_add(Workload("inf2b_2k_s96_keep0.3", INF2B, SIDES_2K, 14, 12, 0.3, 2765, n_blocks=32,
              prior_k={13: 2560}))
_add(Workload("inf2b_2k_s128_keep0.25", INF2B, SIDES_2K, 15, 12, 0.25, 4096, n_blocks=32,
              prior_k={13: 2560, 14: 2765}))
# Keep-ratio sweep on the 64x64 last scale at 1024 px (0.5 is the headline).
for _r, _k in ((1.0, 4096), (0.75, 3072), (0.5, 2048), (0.25, 1024), (0.1, 410)):
    _add(Workload(f"inf2b_1024px_s64_keep{_r}", INF2B, SIDES_1024, 12, 9, _r, _k, n_blocks=32))

HEADLINE = "inf2b_1024px_s64_keep0.5"
SMALL = "d16_256px_s16_keep0.5"


# --------------------------------------------------------------------------
# tensors
# --------------------------------------------------------------------------

# tensor ids: seed of a tensor = base_seed + id
_TID = dict(field=1, spike_pos=2, spike_val=3, cached=4, kprior=5, vprior=6,
            ln1_g=10, ln1_b=11, w_qkv=12, b_qkv=13, w_proj=14, b_proj=15,
            ln2_g=16, ln2_b=17, w_fc1=18, b_fc1=19, w_fc2=20, b_fc2=21)


def _rng(base_seed: int, tensor: str, block: int = 0) -> np.random.Generator:
    return np.random.default_rng(base_seed + _TID[tensor] + 100 * block)


def _stretch(field4: np.ndarray, out: int) -> np.ndarray:
    """Piecewise-linear stretch of axis 0 (length 4) to ``out`` samples.

    Input synthesis only: end points map to end points, which is deliberately
    not the resampling convention of the method's restoration step.
    """
    g = field4.shape[0]
    if out == 1:
        return field4[:1].copy()
    pos = np.linspace(0.0, g - 1.0, out)
    lo = np.minimum(np.floor(pos).astype(np.int64), g - 2)
    t = (pos - lo).astype(np.float32)
    shape = (out,) + (1,) * (field4.ndim - 1)
    return field4[lo] * (1.0 - t).reshape(shape) + field4[lo + 1] * t.reshape(shape)


def token_map(base_seed: int, B: int, h: int, w: int, D: int,
              kind: str = "smooth_spike") -> np.ndarray:
    """Current-scale token map x, shape [B, h*w, D], fp32 holding bf16 values.

    kind:
      smooth_spike  4x4 N(0,1) field per channel stretched to h x w, plus
                    N(0,1.5) vectors on a seeded round(0.1*N) positions
      all_spike     the same with spikes on every position
      constant      every token equal to one N(0,1) vector (all scores tie)
    """
    N = h * w
    out = np.empty((B, N, D), dtype=np.float32)
    for b in range(B):
        rf = _rng(base_seed + 1000 * b, "field")
        if kind == "constant":
            v = rf.standard_normal(D, dtype=np.float32)
            out[b] = v[None, :]
            continue
        f4 = rf.standard_normal((4, 4, D), dtype=np.float32)
        f = _stretch(f4, h)                                   # [h,4,D]
        f = np.moveaxis(_stretch(np.moveaxis(f, 1, 0), w), 0, 1)  # [h,w,D]
        xb = f.reshape(N, D).astype(np.float32)
        n_spk = N if kind == "all_spike" else int(round(0.1 * N))
        if kind not in ("smooth_spike", "all_spike"):
            raise ValueError(kind)
        pos = _rng(base_seed + 1000 * b, "spike_pos").permutation(N)[:n_spk]
        val = _rng(base_seed + 1000 * b, "spike_val").standard_normal(
            (n_spk, D), dtype=np.float32) * np.float32(1.5)
        xb[pos] += val
        out[b] = xb
    return round_bf16(out)


def cached_map(base_seed: int, B: int, hc: int, wc: int, D: int) -> np.ndarray:
    """Cached previous-scale layer output, [B, hc*wc, D], N(0,1), bf16 values."""
    a = _rng(base_seed, "cached").standard_normal((B, hc * wc, D), dtype=np.float32)
    return round_bf16(a)


def kv_prior(base_seed: int, B: int, L0: int, H: int, dh: int):
    """Prior-scale keys and values, each [B, L0, H, dh], N(0,1), bf16 values."""
    kk = _rng(base_seed, "kprior").standard_normal((B, L0, H, dh), dtype=np.float32)
    vv = _rng(base_seed, "vprior").standard_normal((B, L0, H, dh), dtype=np.float32)
    return round_bf16(kk), round_bf16(vv)


def block_weights(base_seed: int, dims: BlockDims, block: int = 0) -> Dict[str, np.ndarray]:
    """Weights of one pre-LayerNorm block, bf16 values held in fp32.

    Linear weights are [out_features, in_features]; the fused QKV weight is
    [3D, D] with output rows ordered q (D rows, head-major), k, v.  All
    matrices and biases N(0, 0.02); LayerNorm gain 1 + N(0, 0.02), shift
    N(0, 0.02).
    """
    D, F = dims.D, dims.F

    def n(name, shape, mean=0.0):
        a = _rng(base_seed, name, block).standard_normal(shape, dtype=np.float32)
        return round_bf16(a * np.float32(0.02) + np.float32(mean))

    return dict(
        ln1_g=n("ln1_g", (D,), 1.0), ln1_b=n("ln1_b", (D,)),
        w_qkv=n("w_qkv", (3 * D, D)), b_qkv=n("b_qkv", (3 * D,)),
        w_proj=n("w_proj", (D, D)), b_proj=n("b_proj", (D,)),
        ln2_g=n("ln2_g", (D,), 1.0), ln2_b=n("ln2_b", (D,)),
        w_fc1=n("w_fc1", (F, D)), b_fc1=n("b_fc1", (F,)),
        w_fc2=n("w_fc2", (D, F)), b_fc2=n("b_fc2", (D,)),
    )
