"""CPU oracle for one FastVAR pruned decoding step (TEST INFRASTRUCTURE ONLY).

A plain, slow, fp64 NumPy statement of what the hot path computes, written
from the paper (FastVAR, arXiv 2503.23367): pivotal token selection (Sec. 3.3,
Eq. 4-5, Alg. 1 first function), one pre-LayerNorm transformer block on the
kept tokens attending to the multi-scale KV cache (Sec. 3.1 KV-cache remark,
Sec. 3.3: only kept tokens enter the cache), and cached token
restoration (Sec. 3.3, Eq. 6, Alg. 1 second function).

It is the checker, not the product: only tests, the smoke entry and the
benchmark's cpu_baseline leg may import it.  It shares no code with the HIP
path and imports nothing from it.

Pins (tests/test_oracle_*.py): brute-force loops and exhaustive sorts on tiny
maps, closed forms (variance identity, shift invariance, constant maps,
half-pixel bilinear weights), keep-ratio 1.0 == dense block, library routines
of torch-CPU for LayerNorm / attention / GELU / bilinear interpolation, a
hand-worked fixture under tests/golden/, and for the schedule the paper's own
settings (Sec. 4.1) written out by hand.  The paper prints no worked numeric
example of a whole step, so `step` as a composition is pinned only through its
parts: whole-step values are "parity unpinned" against the paper itself.

Readings taken where the paper is silent or inconsistent (also listed in the
design notes):
  * score is the squared L2 distance (Alg. 1) -- same ordering as Eq. 5's norm;
  * the top-k decision is taken on the score rounded to fp32, ties go to the
    lowest token index, the index set is emitted ascending;
  * `interpolate` is bilinear with half-pixel centres, edges clamped, in Eq. 6 and
    in Eq. 2 alike; Eq. 2 is taken as the definition of the intermediate prediction
    and Eq. 3 as its unfolding, exact only where resampling composes (bilinear
    resampling in two hops is not one hop, so the two differ in general);
  * `step` puts one select/restore pair around the whole block;
    `step_sublayer` is the finer wiring of Fig. 2(b), one pair around the
    attention layer and one around the FFN layer, each with its own cached map;
  * the cached map and the block output are post-residual hidden states;
  * block internals (pre-LN, eps, 1/sqrt(dh), erf-GELU, biases) come from the
    workload definition, not the paper;
  * nothing is masked at decode time: queries of the current scale see every
    cached key of earlier scales and every kept key of the current scale;
  * rotary positions (Sec. 4.1 names backbones that use them; the paper gives no
    formula): axial 2-D rotary embedding on q and k, interleaved pairs, the first
    half of the pairs turned by the token's grid row and the second half by its
    grid column, each kept token carrying the position of its own slot in the
    token map (the positions are gathered with the same index set as the tokens);
    cached keys were rotated when they were appended.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Tuple

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64


# ---------------------------------------------------------------------------
# ratio -> count  (Sec. 4.1 gives pruning ratios; keep = 1 - prune)
# ---------------------------------------------------------------------------

def keep_count(N: int, keep_ratio: float) -> int:
    """Number of kept tokens for a keep ratio: round-half-up of keep*N, clamped."""
    k = int(math.floor(float(keep_ratio) * N + 0.5))
    return max(0, min(N, k))


# ---------------------------------------------------------------------------
# Pivotal Token Selection  (Sec. 3.3, Eq. 4, Eq. 5)
# ---------------------------------------------------------------------------

def dc_component(x: np.ndarray) -> np.ndarray:
    """Eq. 4: per-sample, per-channel mean over the h*w token positions.

    x [B, N, D] -> [B, D] (fp64).
    """
    x = np.asarray(x, dtype=F64)
    return x.sum(axis=1) / x.shape[1]


def pivotal_scores(x: np.ndarray) -> np.ndarray:
    """Eq. 5 in the squared form of Alg. 1: s[b,n] = sum_c (x[b,n,c]-mean[b,c])^2.

    Returns fp64 scores [B, N].
    """
    x = np.asarray(x, dtype=F64)
    hf = x - dc_component(x)[:, None, :]          # high-frequency part
    return (hf * hf).sum(axis=-1)


def topk_indices(score32: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest scores per sample, ties to the lowest index.

    score32 [B, N] fp32 -> int32 [B, k], each row ascending.
    A stable descending sort keeps equal scores in ascending index order, so
    its first k entries are exactly the lowest-index winners.
    """
    s = np.asarray(score32, dtype=np.float32)
    B, N = s.shape
    if not 0 <= k <= N:
        raise ValueError("k out of range")
    out = np.empty((B, k), dtype=np.int32)
    for b in range(B):
        order = np.argsort(-s[b].astype(F64), kind="stable")
        out[b] = np.sort(order[:k])
    return out


def select_pivotal(x: np.ndarray, k: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """PTS: (idx [B,k] ascending int32, rank [B,N] int32, score [B,N] fp32).

    rank[b,n] is the position of token n inside idx[b], or -1 if pruned.
    """
    s32 = pivotal_scores(x).astype(np.float32)
    idx = topk_indices(s32, k)
    B, N = s32.shape
    rank = np.full((B, N), -1, dtype=np.int32)
    for b in range(B):
        rank[b, idx[b]] = np.arange(k, dtype=np.int32)
    return idx, rank, s32


def gather_tokens(x: np.ndarray, idx: np.ndarray) -> np.ndarray:
    """x [B,N,D], idx [B,k] -> x_kept [B,k,D] (Alg. 1 gather)."""
    x = np.asarray(x)
    return np.stack([x[b, idx[b]] for b in range(x.shape[0])], axis=0)


# ---------------------------------------------------------------------------
# Transformer block on the kept tokens
# ---------------------------------------------------------------------------

def layer_norm(a: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float) -> np.ndarray:
    """LayerNorm over the last axis, biased variance."""
    a = np.asarray(a, dtype=F64)
    m = a.mean(axis=-1, keepdims=True)
    v = ((a - m) ** 2).mean(axis=-1, keepdims=True)
    return (a - m) / np.sqrt(v + eps) * np.asarray(gamma, F64) + np.asarray(beta, F64)


def gelu(a: np.ndarray) -> np.ndarray:
    """Exact GELU: a * Phi(a) with the Gaussian CDF through erf."""
    a = np.asarray(a, dtype=F64)
    return 0.5 * a * (1.0 + _erf(a / math.sqrt(2.0)))


def linear(a: np.ndarray, w: np.ndarray, b: Optional[np.ndarray]) -> np.ndarray:
    """a [..., in] times w [out, in] transposed, plus bias."""
    y = np.asarray(a, F64) @ np.asarray(w, F64).T
    if b is not None:
        y = y + np.asarray(b, F64)
    return y


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, scale: float) -> np.ndarray:
    """Materialised softmax attention, no mask.

    q [M, H, dh], K/V [L, H, dh] -> [M, H, dh].
    """
    M, H, dh = q.shape
    out = np.empty((M, H, dh), dtype=F64)
    if M == 0:          # no queries (a skipped step): nothing to compute, also with no keys
        return out
    for h in range(H):
        s = (q[:, h, :] @ K[:, h, :].T) * scale          # [M, L]
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p = p / p.sum(axis=-1, keepdims=True)
        out[:, h, :] = p @ V[:, h, :]
    return out


def rope2d_angles(h: int, w: int, dh: int, base: float = 10000.0,
                  ref_h: Optional[int] = None, ref_w: Optional[int] = None) -> np.ndarray:
    """Rotation angles of the axial 2-D rotary embedding for every slot of an h x w token map.

    Returns [h*w, dh/2] (fp64): pair t of a head's dh/2 interleaved pairs (2t, 2t+1) is turned by
    angle[n, t] = pos * base**(-t'/(dh/4)), where for the first dh/4 pairs pos is the row coordinate of
    token n = i*w + j and t' = t, for the other dh/4 pairs pos is the column coordinate and
    t' = t - dh/4.  Coordinates are i * ref_h/h and j * ref_w/w: the grid of this scale laid over a
    reference grid (by default its own, i.e. plain integer coordinates), so that the maps of a
    multi-scale schedule can share one coordinate frame.
    """
    assert dh % 4 == 0
    ref_h = h if ref_h is None else ref_h
    ref_w = w if ref_w is None else ref_w
    q = dh // 4
    freq = np.asarray([float(base) ** (-(t / q)) for t in range(q)], dtype=F64)
    ii = np.repeat(np.arange(h, dtype=F64) * (float(ref_h) / h), w)
    jj = np.tile(np.arange(w, dtype=F64) * (float(ref_w) / w), h)
    return np.concatenate([ii[:, None] * freq[None, :], jj[:, None] * freq[None, :]], axis=1)


def apply_rope(v: np.ndarray, angles: np.ndarray) -> np.ndarray:
    """Turn the interleaved pairs of v [..., T, H, dh] by angles [..., T, dh/2] (the same for every head):
    (a, b) -> (a cos - b sin, a sin + b cos)."""
    v = np.asarray(v, F64)
    c = np.cos(angles)[..., None, :]
    s = np.sin(angles)[..., None, :]
    a, b = v[..., 0::2], v[..., 1::2]
    out = np.empty_like(v)
    out[..., 0::2] = a * c - b * s
    out[..., 1::2] = a * s + b * c
    return out


def block_forward_pruned(xk: np.ndarray, W: Dict[str, np.ndarray], H: int,
                         k_cache: np.ndarray, v_cache: np.ndarray,
                         eps: float = 1e-6, scale: Optional[float] = None,
                         return_parts: bool = False, rows: Optional[np.ndarray] = None,
                         rope: Optional[np.ndarray] = None):
    """One pre-LN block on kept tokens xk [B,k,D].

    k_cache / v_cache [B, L0, H, dh] hold the keys/values of all earlier
    scales.  Keys seen by the kept queries are the cached ones followed by the
    kept tokens' own; only the kept tokens' K/V are appended (Sec. 3.3).

    Returns (yk [B,k,D], k_new [B,k,H,dh], v_new [B,k,H,dh]); with
    return_parts also the dict of intermediates (a1, q, o, h1, a2, u).

    `rows` (positions inside the kept set, the same for every sample) limits
    the outputs to those kept tokens: every kept token still contributes its
    key and value, but queries, attention and the MLP are evaluated only for
    the chosen rows, so single outputs of a large step can be checked.

    `rope` [B, k, dh/2]: rotary angles of the kept tokens (rope2d_angles of the
    token map, gathered with the kept index set).  Queries and new keys are
    turned by them before attention; the returned k_new are the turned keys
    (what enters the cache).  The cached keys are taken as they are.
    """
    xk = np.asarray(xk, F64)
    B, k, D = xk.shape
    dh = D // H
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    a1 = layer_norm(xk, W["ln1_g"], W["ln1_b"], eps)
    qkv = linear(a1, W["w_qkv"], W.get("b_qkv"))
    q = qkv[..., 0 * D:1 * D].reshape(B, k, H, dh)
    kn = qkv[..., 1 * D:2 * D].reshape(B, k, H, dh)
    vn = qkv[..., 2 * D:3 * D].reshape(B, k, H, dh)
    if rope is not None:
        q = apply_rope(q, rope)
        kn = apply_rope(kn, rope)
    if rows is not None:
        rows = np.asarray(rows, dtype=np.int64)
        q = q[:, rows]
        xk = xk[:, rows]
    kq = q.shape[1]
    o = np.empty((B, kq, D), dtype=F64)
    for b in range(B):
        Kall = np.concatenate([np.asarray(k_cache[b], F64), kn[b]], axis=0)
        Vall = np.concatenate([np.asarray(v_cache[b], F64), vn[b]], axis=0)
        o[b] = attention(q[b], Kall, Vall, scale).reshape(kq, D)
    h1 = xk + linear(o, W["w_proj"], W.get("b_proj"))
    a2 = layer_norm(h1, W["ln2_g"], W["ln2_b"], eps)
    u = gelu(linear(a2, W["w_fc1"], W.get("b_fc1")))
    yk = h1 + linear(u, W["w_fc2"], W.get("b_fc2"))
    if return_parts:
        return yk, kn, vn, dict(a1=a1, q=q, o=o, h1=h1, a2=a2, u=u)
    return yk, kn, vn


def attention_sublayer_pruned(xk: np.ndarray, W: Dict[str, np.ndarray], H: int,
                              k_cache: np.ndarray, v_cache: np.ndarray,
                              eps: float = 1e-6, scale: Optional[float] = None):
    """The attention layer of the block on kept tokens xk [B,k,D], with its
    residual: h = xk + proj(attn(LN1(xk))).  Keys and values as in
    block_forward_pruned (cached ones, then the kept tokens' own).

    Returns (h [B,k,D], k_new [B,k,H,dh], v_new [B,k,H,dh]).
    """
    xk = np.asarray(xk, F64)
    B, k, D = xk.shape
    dh = D // H
    if scale is None:
        scale = 1.0 / math.sqrt(dh)
    a = layer_norm(xk, W["ln1_g"], W["ln1_b"], eps)
    qkv = linear(a, W["w_qkv"], W.get("b_qkv"))
    q = qkv[..., :D].reshape(B, k, H, dh)
    kn = qkv[..., D:2 * D].reshape(B, k, H, dh)
    vn = qkv[..., 2 * D:].reshape(B, k, H, dh)
    o = np.empty((B, k, D), dtype=F64)
    for b in range(B):
        keys = np.concatenate([np.asarray(k_cache[b], F64), kn[b]], axis=0)
        vals = np.concatenate([np.asarray(v_cache[b], F64), vn[b]], axis=0)
        o[b] = attention(q[b], keys, vals, scale).reshape(k, D)
    return xk + linear(o, W["w_proj"], W.get("b_proj")), kn, vn


def ffn_sublayer_pruned(xk: np.ndarray, W: Dict[str, np.ndarray], eps: float = 1e-6) -> np.ndarray:
    """The FFN layer of the block on kept tokens xk [B,k,D], with its
    residual: y = xk + fc2(gelu(fc1(LN2(xk))))."""
    xk = np.asarray(xk, F64)
    a = layer_norm(xk, W["ln2_g"], W["ln2_b"], eps)
    u = gelu(linear(a, W["w_fc1"], W.get("b_fc1")))
    return xk + linear(u, W["w_fc2"], W.get("b_fc2"))


# ---------------------------------------------------------------------------
# Cached Token Restoration  (Sec. 3.3, Eq. 6)
# ---------------------------------------------------------------------------

def _taps(n_in: int, n_out: int):
    """Half-pixel-centre linear resampling taps along one axis.

    For output position d the source coordinate is (d+0.5)*n_in/n_out-0.5,
    clamped into [0, n_in-1]; returns (i0, i1, lam) with value
    (1-lam)*src[i0] + lam*src[i1].
    """
    d = np.arange(n_out, dtype=F64)
    src = (d + 0.5) * (float(n_in) / float(n_out)) - 0.5
    src = np.clip(src, 0.0, float(n_in - 1))
    i0 = np.floor(src).astype(np.int64)
    i1 = np.minimum(i0 + 1, n_in - 1)
    return i0, i1, src - i0


def upsample_bilinear(cache_map: np.ndarray, hc: int, wc: int, h: int, w: int) -> np.ndarray:
    """Eq. 6: cache_map [B, hc*wc, D] -> [B, h*w, D], bilinear, fp64."""
    c = np.asarray(cache_map, F64)
    B, Nc, D = c.shape
    assert Nc == hc * wc
    c = c.reshape(B, hc, wc, D)
    r0, r1, lr = _taps(hc, h)
    c0, c1, lc = _taps(wc, w)
    rows = c[:, r0] * (1.0 - lr)[None, :, None, None] + c[:, r1] * lr[None, :, None, None]
    out = rows[:, :, c0] * (1.0 - lc)[None, None, :, None] + rows[:, :, c1] * lc[None, None, :, None]
    return out.reshape(B, h * w, D)


def restore(yk: np.ndarray, idx: np.ndarray, cache_map: np.ndarray,
            hc: int, wc: int, h: int, w: int) -> np.ndarray:
    """CTR: the upsampled cache with the kept outputs scattered in at idx."""
    y = upsample_bilinear(cache_map, hc, wc, h, w)
    yk = np.asarray(yk, F64)
    for b in range(y.shape[0]):
        y[b, idx[b]] = yk[b]
    return y


# ---------------------------------------------------------------------------
# Whole step
# ---------------------------------------------------------------------------

def step(x, h, w, k, W, H, k_cache, v_cache, cache_map, hc, wc,
         eps: float = 1e-6, scale: Optional[float] = None):
    """select -> block on kept tokens -> restore, block granularity.

    Returns dict(idx, rank, score, yk, k_new, v_new, y).
    """
    idx, rank, s32 = select_pivotal(x, k)
    xk = gather_tokens(np.asarray(x, F64), idx)
    yk, kn, vn = block_forward_pruned(xk, W, H, k_cache, v_cache, eps, scale)
    y = restore(yk, idx, cache_map, hc, wc, h, w)
    return dict(idx=idx, rank=rank, score=s32, yk=yk, k_new=kn, v_new=vn, y=y)


def step_sublayer(x, h, w, k_attn, k_ffn, W, H, k_cache, v_cache, cache_attn, cache_ffn, hc, wc,
                  eps: float = 1e-6, scale: Optional[float] = None, x_mid=None):
    """Fig. 2(b): a select/restore pair around the attention layer and another
    around the FFN layer (Sec. 3.3, implementation paragraph), each restoring
    from the cached output of its own layer (Sec. 3.3 overview: per-layer
    outputs of the cached step are kept).

    x_mid, when given, replaces the restored map between the two halves (a
    caller that checks a device run passes the device's own bf16-rounded map, so
    that the second selection is taken on identical values).

    Returns dict(idx_attn, hk, k_new, v_new, x_mid, idx_ffn, yk, y).
    """
    idx_a, _, _ = select_pivotal(x, k_attn)
    xk = gather_tokens(np.asarray(x, F64), idx_a)
    hk, kn, vn = attention_sublayer_pruned(xk, W, H, k_cache, v_cache, eps, scale)
    mid = restore(hk, idx_a, cache_attn, hc, wc, h, w)
    src = mid if x_mid is None else np.asarray(x_mid, F64)
    idx_f, _, _ = select_pivotal(src, k_ffn)
    yk = ffn_sublayer_pruned(gather_tokens(src, idx_f), W, eps)
    y = restore(yk, idx_f, cache_ffn, hc, wc, h, w)
    return dict(idx_attn=idx_a, hk=hk, k_new=kn, v_new=vn, x_mid=mid, idx_ffn=idx_f, yk=yk, y=y)



def scale_step(x, h, w, k, layers, H, k_caches, v_caches, cache_maps, hc, wc, structure, capture=False,
               eps: float = 1e-6, scale: Optional[float] = None):
    """One scale step of a stack of blocks (Fig. 2(a); Sec. 3.3, overview).

    layers: list of weight dicts; k_caches / v_caches: per block [B, L0, H, dh];
    cache_maps: per block [B, hc*wc, D] (unused in the structure stage).
    structure=True: every block runs on all tokens, no selection or restoration
    (the stage is kept as the standard model); with capture the block outputs are
    returned as the new cached maps.  Otherwise each block runs select -> block on
    the kept tokens -> restore from its own cached map; k == N runs it unpruned
    and k == 0 leaves only the upsampled cache.  Only kept tokens enter a cache.

    Returns dict(y, k_caches, v_caches (grown), captured (list or None), idx (of the
    last block, None when nothing was selected)).
    """
    cur = np.asarray(x, F64)
    N = h * w
    new_k, new_v, captured, idx = [], [], ([] if capture else None), None
    for l, W in enumerate(layers):
        if structure or k == N:
            y, kn, vn = block_forward_pruned(cur, W, H, k_caches[l], v_caches[l], eps, scale)
        else:
            r = step(cur, h, w, k, W, H, k_caches[l], v_caches[l], cache_maps[l], hc, wc, eps, scale)
            y, kn, vn, idx = r["y"], r["k_new"], r["v_new"], r["idx"]
        new_k.append(np.concatenate([np.asarray(k_caches[l], F64), kn], axis=1))
        new_v.append(np.concatenate([np.asarray(v_caches[l], F64), vn], axis=1))
        if capture:
            captured.append(y)
        cur = y
    return dict(y=cur, k_caches=new_k, v_caches=new_v, captured=captured, idx=idx)


# ---------------------------------------------------------------------------
# Around the scale step: pruning schedule (Sec. 3.3 overview, Sec. 4.1) and the
# intermediate prediction (Sec. 3.1, Eq. 2, Eq. 3)
# ---------------------------------------------------------------------------

def schedule_plan(sizes, prune_ratios):
    """Which steps are pruned, how many tokens each keeps, and which step is cached.

    sizes: [(h_1, w_1) .. (h_K, w_K)]; prune_ratios: the N ratios of the last N steps,
    in step order (Sec. 4.1: e.g. 40, 50, 100, 100 % with N = 4, or 50, 75 % with N = 2).
    The first K-N steps are the structure stage and keep everything; the per-block
    outputs of the last of them (step K-N, index K-N-1 counted from 0) are what the
    texture steps restore from.  A ratio of 100 % keeps nothing: the step is skipped.
    Returns (keep counts [K], structure flags [K], cached step index or -1 when N == 0
    or N == K).
    """
    K, n = len(sizes), len(prune_ratios)
    assert 0 <= n <= K
    keep, structure = [], []
    for i, (h, w) in enumerate(sizes):
        if i < K - n:
            keep.append(h * w)
            structure.append(True)
        else:
            keep.append(keep_count(h * w, 1.0 - float(prune_ratios[i - (K - n)])))
            structure.append(False)
    cached = K - n - 1 if 0 < n < K else -1
    return keep, structure, cached


def residual_accumulate(r_prev: Optional[np.ndarray], hp: int, wp: int,
                        f_k: Optional[np.ndarray], h: int, w: int) -> np.ndarray:
    """Eq. 2: r_k = interpolate(r_{k-1}, (h, w)) + f_k, maps as [B, h*w, C], fp64.

    r_prev None: the first step, r_1 = f_1.  f_k None: a skipped step (ratio 100 %),
    whose output is the interpolation of the previous intermediate prediction alone.
    `interpolate` is the same bilinear resampling as in Eq. 6 (the paper names no mode).
    """
    if r_prev is None:
        assert f_k is not None
        return np.asarray(f_k, F64).copy()
    up = upsample_bilinear(r_prev, hp, wp, h, w)
    return up if f_k is None else up + np.asarray(f_k, F64)


def cumulative_prediction(fs, sizes, k: int) -> np.ndarray:
    """Eq. 3: r_k = sum_{i<=k} interpolate(f_i, (h_k, w_k)) (k counted from 1)."""
    h, w = sizes[k - 1]
    out = None
    for i in range(k):
        hi, wi = sizes[i]
        t = upsample_bilinear(fs[i], hi, wi, h, w)
        out = t if out is None else out + t
    return out

