"""ctypes binding of libfastvar.so: same names as the C ABI, argument
marshalling only.  Tensors are torch CUDA tensors used purely as device
buffers; kernels are enqueued on torch's current stream.

There is no fallback: if the shared library is missing `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libfastvar.so")

FASTVAR_OK = 0
FASTVAR_EINVAL = -1
FASTVAR_ECAPACITY = -2
FASTVAR_EWORKSPACE = -3
FASTVAR_EALIGN = -4
FASTVAR_EHIP = -5
FASTVAR_MAX_TOKENS = 32768


class FastvarError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class Dims(C.Structure):
    _fields_ = [("D", C.c_int32), ("H", C.c_int32), ("dh", C.c_int32), ("F", C.c_int32),
                ("ln_eps", C.c_float), ("softmax_scale", C.c_float)]


WEIGHT_FIELDS = ("ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_proj", "b_proj",
                 "ln2_g", "ln2_b", "w_fc1", "b_fc1", "w_fc2", "b_fc2")


class BlockWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_FIELDS]


class Layer(C.Structure):
    _fields_ = [("weights", C.POINTER(BlockWeights)), ("k_cache", C.c_void_p), ("v_cache", C.c_void_p),
                ("cache_map", C.c_void_p)]


_lib = None

EXPORTS = ("fastvar_version", "fastvar_strerror", "fastvar_keep_count", "fastvar_schedule_plan",
           "fastvar_residual_accumulate",
           "fastvar_select_workspace_bytes", "fastvar_block_workspace_bytes",
           "fastvar_restore_workspace_bytes", "fastvar_step_workspace_bytes",
           "fastvar_select_pivotal", "fastvar_select_pivotal_static", "fastvar_block_forward_pruned",
           "fastvar_restore",
           "fastvar_step", "fastvar_scale_step", "fastvar_scale_step_timed",
           "fastvar_step_sublayer_workspace_bytes", "fastvar_attn_forward_pruned",
           "fastvar_ffn_forward_pruned", "fastvar_step_sublayer", "fastvar_layernorm", "fastvar_gemm_bf16",
           "fastvar_qkv_gemm", "fastvar_attention", "fastvar_rope2d_table", "fastvar_qkv_gemm_rope",
           "fastvar_block_forward_pruned_rope")


def lib() -> C.CDLL:
    """Load libfastvar.so (once) and declare the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} not found: build it with `python -m paper_2503_23367_amd.build` "
            "(there is no CPU or PyTorch fallback)")
    L = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    L.fastvar_version.restype = i32
    L.fastvar_strerror.restype = C.c_char_p
    L.fastvar_strerror.argtypes = [i32]
    L.fastvar_keep_count.restype = i32
    L.fastvar_keep_count.argtypes = [i32, C.c_double]
    L.fastvar_select_workspace_bytes.restype = sz
    L.fastvar_select_workspace_bytes.argtypes = [i32, i32, i32]
    L.fastvar_block_workspace_bytes.restype = sz
    L.fastvar_block_workspace_bytes.argtypes = [C.POINTER(Dims), i32, i32]
    L.fastvar_restore_workspace_bytes.restype = sz
    L.fastvar_restore_workspace_bytes.argtypes = [i32, i32]
    L.fastvar_step_workspace_bytes.restype = sz
    L.fastvar_step_workspace_bytes.argtypes = [C.POINTER(Dims), i32, i32, i32]
    L.fastvar_select_pivotal.restype = i32
    L.fastvar_select_pivotal.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp]
    L.fastvar_select_pivotal_static.restype = i32
    L.fastvar_select_pivotal_static.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    L.fastvar_block_forward_pruned.restype = i32
    L.fastvar_block_forward_pruned.argtypes = [vp, i32, vp, i32, i32, C.POINTER(Dims),
                                               C.POINTER(BlockWeights), vp, vp, i32, i32, vp, vp, sz, vp]
    L.fastvar_schedule_plan.restype = i32
    L.fastvar_schedule_plan.argtypes = [C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32, C.POINTER(C.c_double), i32,
                                        C.POINTER(C.c_int32), C.POINTER(C.c_int32)]
    L.fastvar_residual_accumulate.restype = i32
    L.fastvar_residual_accumulate.argtypes = [vp, i32, i32, vp, i32, i32, i32, i32, vp, vp]
    L.fastvar_restore.restype = i32
    L.fastvar_restore.argtypes = [vp, vp, vp, i32, i32, vp, i32, i32, i32, i32, i32, vp, vp, sz, vp]
    L.fastvar_step.restype = i32
    L.fastvar_step.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32, i32, i32, i32, i32,
                               C.POINTER(Dims), C.POINTER(BlockWeights), vp, vp, C.POINTER(C.c_int32), i32,
                               vp, vp, vp, vp, sz, vp]
    L.fastvar_scale_step.restype = i32
    L.fastvar_scale_step.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32, i32, i32, i32, i32,
                                     C.POINTER(Dims), C.POINTER(Layer), i32, C.POINTER(C.c_int32), i32,
                                     vp, vp, vp, vp, sz, vp]
    L.fastvar_scale_step_timed.restype = i32
    L.fastvar_scale_step_timed.argtypes = L.fastvar_scale_step.argtypes + [C.POINTER(C.c_float)]
    L.fastvar_step_sublayer_workspace_bytes.restype = sz
    L.fastvar_step_sublayer_workspace_bytes.argtypes = [C.POINTER(Dims), i32, i32, i32, i32]
    L.fastvar_attn_forward_pruned.restype = i32
    L.fastvar_attn_forward_pruned.argtypes = [vp, i32, vp, i32, i32, C.POINTER(Dims),
                                              C.POINTER(BlockWeights), vp, vp, i32, i32, vp, vp, sz, vp]
    L.fastvar_ffn_forward_pruned.restype = i32
    L.fastvar_ffn_forward_pruned.argtypes = [vp, i32, vp, i32, i32, C.POINTER(Dims),
                                             C.POINTER(BlockWeights), vp, vp, sz, vp]
    L.fastvar_step_sublayer.restype = i32
    L.fastvar_step_sublayer.argtypes = [vp, C.POINTER(C.c_int32), C.POINTER(C.c_int32), i32, i32, i32, i32,
                                        i32, i32, C.POINTER(Dims), C.POINTER(BlockWeights), vp, vp,
                                        C.POINTER(C.c_int32), i32, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    L.fastvar_layernorm.restype = i32
    L.fastvar_layernorm.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, C.c_float, vp, vp]
    L.fastvar_gemm_bf16.restype = i32
    L.fastvar_gemm_bf16.argtypes = [vp, vp, vp, vp, i32, i32, i32, i32, vp, vp]
    L.fastvar_qkv_gemm.restype = i32
    L.fastvar_qkv_gemm.argtypes = [vp, vp, vp, i32, i32, C.POINTER(Dims), vp, vp, vp, i32, i32, vp]
    L.fastvar_attention.restype = i32
    L.fastvar_attention.argtypes = [vp, vp, vp, i32, i32, C.POINTER(Dims), i32, i32, vp, vp]
    L.fastvar_rope2d_table.restype = i32
    L.fastvar_rope2d_table.argtypes = [i32, i32, i32, C.c_double, i32, i32, vp, vp, vp]
    L.fastvar_qkv_gemm_rope.restype = i32
    L.fastvar_qkv_gemm_rope.argtypes = [vp, vp, vp, vp, i32, i32, i32, C.POINTER(Dims), vp, vp, vp, vp, vp, i32, i32, vp]
    L.fastvar_block_forward_pruned_rope.restype = i32
    L.fastvar_block_forward_pruned_rope.argtypes = [vp, i32, vp, i32, i32, C.POINTER(Dims), C.POINTER(BlockWeights),
                                                    vp, vp, vp, vp, i32, i32, vp, vp, sz, vp]
    _lib = L
    return L


# ---------------------------------------------------------------------------
# helpers
# ---------------------------------------------------------------------------

def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str) -> None:
    if rc != FASTVAR_OK:
        raise FastvarError(rc, where)


def strerror(code: int) -> str:
    return lib().fastvar_strerror(code).decode()


def make_dims(D: int, H: int, dh: int, F: int, ln_eps: float = 1e-6,
              softmax_scale: Optional[float] = None) -> Dims:
    if softmax_scale is None:
        softmax_scale = dh ** -0.5
    return Dims(D, H, dh, F, ln_eps, softmax_scale)


def make_weights(tensors: Dict[str, "object"]) -> BlockWeights:
    """Struct of device pointers; keeps no reference, the caller keeps the tensors alive."""
    w = BlockWeights()
    for n in WEIGHT_FIELDS:
        setattr(w, n, _ptr(tensors.get(n)))
    return w


# ---------------------------------------------------------------------------
# the C ABI, name for name
# ---------------------------------------------------------------------------

def fastvar_version() -> int:
    return lib().fastvar_version()


def fastvar_keep_count(N: int, keep_ratio: float) -> int:
    return lib().fastvar_keep_count(N, keep_ratio)


def fastvar_select_workspace_bytes(B: int, N: int, D: int) -> int:
    return lib().fastvar_select_workspace_bytes(B, N, D)


def fastvar_block_workspace_bytes(dims: Dims, B: int, k: int) -> int:
    return lib().fastvar_block_workspace_bytes(C.byref(dims), B, k)


def fastvar_schedule_plan(sched_h, sched_w, prune_ratio):
    """Host call: returns (keep counts per step, cached step index or -1)."""
    K, n = len(sched_h), len(prune_ratio)
    hs = (C.c_int32 * K)(*sched_h)
    ws_ = (C.c_int32 * K)(*sched_w)
    pr = (C.c_double * max(n, 1))(*prune_ratio)
    keep = (C.c_int32 * K)()
    cached = C.c_int32(-2)
    rc = lib().fastvar_schedule_plan(hs, ws_, K, pr if n else None, n, keep, C.byref(cached))
    _check(rc, "fastvar_schedule_plan")
    return list(keep), cached.value


def fastvar_residual_accumulate(r_prev, hp, wp, f_k, h, w, B, Cc, r_out) -> None:
    rc = lib().fastvar_residual_accumulate(_ptr(r_prev), hp, wp, _ptr(f_k), h, w, B, Cc, _ptr(r_out), _stream())
    _check(rc, "fastvar_residual_accumulate")


def fastvar_restore_workspace_bytes(B: int, N: int) -> int:
    return lib().fastvar_restore_workspace_bytes(B, N)


def fastvar_step_workspace_bytes(dims: Dims, B: int, N: int, k: int) -> int:
    return lib().fastvar_step_workspace_bytes(C.byref(dims), B, N, k)


def fastvar_select_pivotal(x, B, h, w, D, k, idx_out, rank_out, score_out, ws) -> None:
    rc = lib().fastvar_select_pivotal(_ptr(x), B, h, w, D, k, _ptr(idx_out), _ptr(rank_out),
                                      _ptr(score_out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                      _stream())
    _check(rc, "fastvar_select_pivotal")


FASTVAR_SELECT_STATIC_BYTES = 8 << 20


def fastvar_select_pivotal_static(x, B, h, w, D, k, idx_out, rank_out, score_out) -> None:
    rc = lib().fastvar_select_pivotal_static(_ptr(x), B, h, w, D, k, _ptr(idx_out), _ptr(rank_out),
                                             _ptr(score_out), _stream())
    _check(rc, "fastvar_select_pivotal_static")


def fastvar_block_forward_pruned(x, N, idx, B, k, dims: Dims, weights: BlockWeights, k_cache, v_cache,
                                 L0, L_cap, y_kept_out, ws) -> None:
    rc = lib().fastvar_block_forward_pruned(_ptr(x), N, _ptr(idx), B, k, C.byref(dims), C.byref(weights),
                                            _ptr(k_cache), _ptr(v_cache), L0, L_cap, _ptr(y_kept_out),
                                            _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                                            _stream())
    _check(rc, "fastvar_block_forward_pruned")


def fastvar_restore(y_kept, idx, rank, B, k, cache_map, hc, wc, h, w, D, y_out, ws=None) -> None:
    rc = lib().fastvar_restore(_ptr(y_kept), _ptr(idx), _ptr(rank), B, k, _ptr(cache_map), hc, wc, h, w, D,
                               _ptr(y_out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                               _stream())
    _check(rc, "fastvar_restore")


def fastvar_step(x, sched_h, sched_w, step, cache_step, B, k, dims: Dims, weights: BlockWeights,
                 k_cache, v_cache, kv_len: int, L_cap, cache_map, y_out, idx_out, ws) -> int:
    """Returns the new cache length."""
    K = len(sched_h)
    sh = (C.c_int32 * K)(*sched_h)
    sw = (C.c_int32 * K)(*sched_w)
    kv = C.c_int32(kv_len)
    rc = lib().fastvar_step(_ptr(x), sh, sw, K, step, cache_step, B, k, C.byref(dims), C.byref(weights),
                            _ptr(k_cache), _ptr(v_cache), C.byref(kv), L_cap, _ptr(cache_map), _ptr(y_out),
                            _ptr(idx_out), _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(),
                            _stream())
    _check(rc, "fastvar_step")
    return kv.value


def make_layers(blocks):
    """Host array of Layer structs from dicts with keys w (BlockWeights), kc, vc, cache (tensors; cache may be
    None).  Keeps no reference to the tensors; the BlockWeights structs must outlive the array."""
    arr = (Layer * len(blocks))()
    for i, b in enumerate(blocks):
        arr[i].weights = C.pointer(b["w"])
        arr[i].k_cache = _ptr(b["kc"])
        arr[i].v_cache = _ptr(b["vc"])
        arr[i].cache_map = _ptr(b.get("cache"))
    return arr


def fastvar_scale_step(x, sched_h, sched_w, step, cache_step, B, k, dims: Dims, layers, kv_len: int, L_cap,
                       y_out, tmp, idx_out, ws) -> int:
    """`layers`: array from make_layers.  Returns the new cache length."""
    K = len(sched_h)
    sh = (C.c_int32 * K)(*sched_h)
    sw = (C.c_int32 * K)(*sched_w)
    kv = C.c_int32(kv_len)
    rc = lib().fastvar_scale_step(_ptr(x), sh, sw, K, step, cache_step, B, k, C.byref(dims), layers, len(layers),
                                  C.byref(kv), L_cap, _ptr(y_out), _ptr(tmp), _ptr(idx_out), _ptr(ws),
                                  0 if ws is None else ws.numel() * ws.element_size(), _stream())
    _check(rc, "fastvar_scale_step")
    return kv.value


STAGES = ("select", "gather+layernorm 1", "qkv gemm", "attention", "proj gemm", "layernorm 2", "fc1 gemm",
          "fc2 gemm", "restore")


def fastvar_scale_step_timed(x, sched_h, sched_w, step, cache_step, B, k, dims: Dims, layers, kv_len: int, L_cap,
                             y_out, tmp, idx_out, ws):
    """fastvar_scale_step that waits for the stream and returns (new cache length, {stage: ms per block})."""
    K = len(sched_h)
    sh = (C.c_int32 * K)(*sched_h)
    sw = (C.c_int32 * K)(*sched_w)
    kv = C.c_int32(kv_len)
    ms = (C.c_float * len(STAGES))()
    rc = lib().fastvar_scale_step_timed(_ptr(x), sh, sw, K, step, cache_step, B, k, C.byref(dims), layers,
                                        len(layers), C.byref(kv), L_cap, _ptr(y_out), _ptr(tmp), _ptr(idx_out),
                                        _ptr(ws), 0 if ws is None else ws.numel() * ws.element_size(), _stream(), ms)
    _check(rc, "fastvar_scale_step_timed")
    return kv.value, {n: float(ms[i]) for i, n in enumerate(STAGES)}


def fastvar_step_sublayer_workspace_bytes(dims: Dims, B: int, N: int, k_attn: int, k_ffn: int) -> int:
    return lib().fastvar_step_sublayer_workspace_bytes(C.byref(dims), B, N, k_attn, k_ffn)


def _nbytes(t) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def fastvar_attn_forward_pruned(x, N, idx, B, k, dims: Dims, weights: BlockWeights, k_cache, v_cache,
                                L0, L_cap, h_kept_out, ws) -> None:
    rc = lib().fastvar_attn_forward_pruned(_ptr(x), N, _ptr(idx), B, k, C.byref(dims), C.byref(weights),
                                           _ptr(k_cache), _ptr(v_cache), L0, L_cap, _ptr(h_kept_out),
                                           _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "fastvar_attn_forward_pruned")


def fastvar_ffn_forward_pruned(x, N, idx, B, k, dims: Dims, weights: BlockWeights, y_kept_out, ws) -> None:
    rc = lib().fastvar_ffn_forward_pruned(_ptr(x), N, _ptr(idx), B, k, C.byref(dims), C.byref(weights),
                                          _ptr(y_kept_out), _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "fastvar_ffn_forward_pruned")


def fastvar_step_sublayer(x, sched_h, sched_w, step, cache_step, B, k_attn, k_ffn, dims: Dims,
                          weights: BlockWeights, k_cache, v_cache, kv_len: int, L_cap, cache_map_attn,
                          cache_map_ffn, x_mid, y_out, idx_attn_out, idx_ffn_out, ws) -> int:
    """Returns the new cache length."""
    K = len(sched_h)
    sh = (C.c_int32 * K)(*sched_h)
    sw = (C.c_int32 * K)(*sched_w)
    kv = C.c_int32(kv_len)
    rc = lib().fastvar_step_sublayer(_ptr(x), sh, sw, K, step, cache_step, B, k_attn, k_ffn, C.byref(dims),
                                     C.byref(weights), _ptr(k_cache), _ptr(v_cache), C.byref(kv), L_cap,
                                     _ptr(cache_map_attn), _ptr(cache_map_ffn), _ptr(x_mid), _ptr(y_out),
                                     _ptr(idx_attn_out), _ptr(idx_ffn_out), _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "fastvar_step_sublayer")
    return kv.value


EPI_BIAS_RES = 1
EPI_BIAS_GELU = 2


def fastvar_layernorm(inp, idx, B, N, k, D, gamma, beta, eps, out) -> None:
    rc = lib().fastvar_layernorm(_ptr(inp), _ptr(idx), B, N, k, D, _ptr(gamma), _ptr(beta), eps, _ptr(out),
                                 _stream())
    _check(rc, "fastvar_layernorm")


def fastvar_gemm_bf16(A, W, bias, residual, M, N, K, epilogue, out) -> None:
    rc = lib().fastvar_gemm_bf16(_ptr(A), _ptr(W), _ptr(bias), _ptr(residual), M, N, K, epilogue, _ptr(out),
                                 _stream())
    _check(rc, "fastvar_gemm_bf16")


def fastvar_qkv_gemm(a, w_qkv, b_qkv, B, k, dims: Dims, q_out, k_cache, v_cache, L0, L_cap) -> None:
    rc = lib().fastvar_qkv_gemm(_ptr(a), _ptr(w_qkv), _ptr(b_qkv), B, k, C.byref(dims), _ptr(q_out),
                                _ptr(k_cache), _ptr(v_cache), L0, L_cap, _stream())
    _check(rc, "fastvar_qkv_gemm")


def fastvar_attention(q, k_cache, v_cache, B, k, dims: Dims, L, L_cap, o) -> None:
    rc = lib().fastvar_attention(_ptr(q), _ptr(k_cache), _ptr(v_cache), B, k, C.byref(dims), L, L_cap,
                                 _ptr(o), _stream())
    _check(rc, "fastvar_attention")


def fastvar_rope2d_table(h, w, dh, base, ref_h, ref_w, cos_out, sin_out) -> None:
    rc = lib().fastvar_rope2d_table(h, w, dh, base, ref_h, ref_w, _ptr(cos_out), _ptr(sin_out), _stream())
    _check(rc, "fastvar_rope2d_table")


def fastvar_qkv_gemm_rope(a, w_qkv, b_qkv, idx, B, N, k, dims: Dims, rope_cos, rope_sin, q_out, k_cache, v_cache,
                          L0, L_cap) -> None:
    rc = lib().fastvar_qkv_gemm_rope(_ptr(a), _ptr(w_qkv), _ptr(b_qkv), _ptr(idx), B, N, k, C.byref(dims),
                                     _ptr(rope_cos), _ptr(rope_sin), _ptr(q_out), _ptr(k_cache), _ptr(v_cache),
                                     L0, L_cap, _stream())
    _check(rc, "fastvar_qkv_gemm_rope")


def fastvar_block_forward_pruned_rope(x, N, idx, B, k, dims: Dims, weights: BlockWeights, rope_cos, rope_sin,
                                      k_cache, v_cache, L0, L_cap, y_kept_out, ws) -> None:
    rc = lib().fastvar_block_forward_pruned_rope(_ptr(x), N, _ptr(idx), B, k, C.byref(dims), C.byref(weights),
                                                 _ptr(rope_cos), _ptr(rope_sin), _ptr(k_cache), _ptr(v_cache),
                                                 L0, L_cap, _ptr(y_kept_out), _ptr(ws), _nbytes(ws), _stream())
    _check(rc, "fastvar_block_forward_pruned_rope")
