"""Helpers for the GPU parity tests: bf16 upload/download and the library's
physical KV-cache layouts.  Marshalling only, no method arithmetic."""
import numpy as np
import torch

from paper_2503_23367_amd import binding as fb
from paper_2503_23367_amd import synth

DEV = "cuda:0"


def to_dev_bf16(a: np.ndarray) -> torch.Tensor:
    """fp32 array holding bf16-representable values -> bf16 CUDA tensor (bit exact)."""
    bits = synth.to_bf16_bits(a).astype(np.int16)
    return torch.from_numpy(bits).to(DEV).view(torch.bfloat16).reshape(a.shape)


def from_dev_bf16(t: torch.Tensor) -> np.ndarray:
    """bf16 CUDA tensor -> fp32 numpy (exact widening)."""
    bits = t.contiguous().view(torch.int16).cpu().numpy().astype(np.uint16)
    return synth.from_bf16_bits(bits).reshape(tuple(t.shape))


def empty_ws(nbytes: int) -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=DEV)


def make_caches(k_prior: np.ndarray, v_prior: np.ndarray, L_cap: int, poison: bool = True):
    """Logical [B,L0,H,dh] priors -> library layouts k [B,H,L_cap,dh], v [B,H,dh,L_cap].

    Unused positions are filled with NaN bit patterns when `poison` so that any
    read past the valid length shows up in the outputs.
    """
    B, L0, H, dh = k_prior.shape
    fill = float("nan") if poison else 0.0
    kc = torch.full((B, H, L_cap, dh), fill, dtype=torch.bfloat16, device=DEV)
    vc = torch.full((B, H, dh, L_cap), fill, dtype=torch.bfloat16, device=DEV)
    if L0 > 0:
        kc[:, :, :L0, :] = to_dev_bf16(k_prior).permute(0, 2, 1, 3)
        vc[:, :, :, :L0] = to_dev_bf16(v_prior).permute(0, 2, 3, 1)
    return kc, vc


def cache_rows(kc: torch.Tensor, vc: torch.Tensor, lo: int, hi: int):
    """Library caches -> logical fp32 [B, hi-lo, H, dh] for K and V."""
    k = from_dev_bf16(kc[:, :, lo:hi, :].permute(0, 2, 1, 3).contiguous())
    v = from_dev_bf16(vc[:, :, :, lo:hi].permute(0, 3, 1, 2).contiguous())
    return k, v


def upload_weights(W):
    """dict of fp32 arrays -> (dict of bf16 CUDA tensors, BlockWeights struct)."""
    t = {n: to_dev_bf16(a) for n, a in W.items()}
    return t, fb.make_weights(t)


def max_rel(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got-ref| / max |ref| over a tensor."""
    denom = float(np.max(np.abs(ref)))
    return float(np.max(np.abs(np.asarray(got, np.float64) - ref))) / (denom if denom > 0 else 1.0)
