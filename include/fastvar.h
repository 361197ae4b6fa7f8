/*
 * fastvar.h -- C ABI of the MI355X (gfx950) pruned VAR decoding step.
 *
 * One large-scale decoding step of a next-scale-prediction VAR transformer
 * with FastVAR's cached token pruning (arXiv 2503.23367, Sec. 3.3, Fig. 2,
 * appendix algorithm):
 *   1. Pivotal Token Selection (PTS): score every token of the current token
 *      map by its squared distance from the map mean (Eq. 4, Eq. 5) and keep
 *      the k highest-scoring tokens.
 *   2. One pre-LayerNorm transformer block on the kept tokens only; their
 *      queries attend to the keys/values of all earlier scales held in the
 *      KV cache plus the kept tokens' own, and only the kept tokens' K/V are
 *      appended to the cache (Sec. 3.1, Sec. 3.3).
 *   3. Cached Token Restoration (CTR): the cached output of the last unpruned
 *      scale is bilinearly upsampled to the current grid (Eq. 6) and the kept
 *      tokens' outputs are scattered into it at the kept positions.
 *
 * Conventions
 *   - Every pointer is a DEVICE pointer unless its comment says "host".
 *   - All activations, weights and caches are bf16 (16-bit patterns); index
 *     arrays are int32; scores are fp32.
 *   - Row-major everywhere.  A token map is [B, h*w, D] with token index
 *     n = i*w + j (row i, column j of the h x w grid).
 *   - The caller owns every buffer.  The library allocates nothing, keeps no
 *     state between calls (one documented exception: the per-device scratch of
 *     fastvar_select_pivotal_static) and never synchronises: each call validates its
 *     arguments on the host, enqueues its kernels on `stream`
 *     (a hipStream_t passed as void*; NULL = the default stream) and returns.
 *   - HIP graphs: a call that has run once eagerly on the device (first use
 *     raises a kernel's LDS limit, which is not a stream operation) may be
 *     captured into a graph: it only launches kernels (its arrival counters
 *     are cleared by a kernel, not by a memset node).  fastvar_scale_step_timed
 *     is the exception: it records events and waits.
 *   - Return value: FASTVAR_OK (0) or a negative FASTVAR_E* code.  Arguments
 *     are checked before anything is launched; on an argument error no output
 *     buffer is touched.
 *   - Pointers must be 16-byte aligned; D must be a multiple of 8.  The block
 *     entry points additionally need D, F multiples of 64, dh in {64, 128}
 *     and L_cap a multiple of 8.
 *
 * KV-cache layout (chosen for the attention kernel's 16-byte LDS reads):
 *   k_cache [B, H, L_cap, dh]   key rows, dh contiguous
 *   v_cache [B, H, dh, L_cap]   value columns, cache position contiguous
 * Rows / columns [0, L0) hold the earlier scales; a block call writes
 * positions [L0, L0+k) and the caller then treats the length as L0+k.
 * A caller that holds keys and values token-major, [B, L, H, dh], fills these
 * caches once with  k_cache = K.permute(0, 2, 1, 3)  (positions [0, L) of an
 * L_cap-long axis) and  v_cache = V.permute(0, 2, 3, 1);  rows the library
 * appends read back as  K[b, l, h, :] = k_cache[b, h, l, :]  and
 * V[b, l, h, :] = v_cache[b, h, :, l].
 *
 * Scratch: there is no single workspace-size function; each entry point has
 * its own (fastvar_select_workspace_bytes, fastvar_block_workspace_bytes,
 * fastvar_restore_workspace_bytes, fastvar_step_workspace_bytes,
 * fastvar_step_sublayer_workspace_bytes), because the selection, the block
 * and the whole step need different buffers and a caller of one stage should
 * not pay for the others.  fastvar_step_workspace_bytes(dims, B, N, k) is the
 * one that covers a whole step.
 */
#ifndef FASTVAR_H
#define FASTVAR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FASTVAR_VERSION 100 /* major*10000 + minor*100 + patch */

enum {
    FASTVAR_OK = 0,
    FASTVAR_EINVAL = -1,     /* null pointer, non-positive size, k outside [0,N], D != H*dh, bad step */
    FASTVAR_ECAPACITY = -2,  /* L0 + k > L_cap, or a size beyond a documented maximum */
    FASTVAR_EWORKSPACE = -3, /* ws_bytes smaller than the matching *_workspace_bytes() */
    FASTVAR_EALIGN = -4,     /* pointer not 16-byte aligned, or a width not a required multiple */
    FASTVAR_EHIP = -5        /* a kernel launch reported an error */
};

/* Largest token map the selection kernel accepts (tokens per sample). */
#define FASTVAR_MAX_TOKENS 32768

/* Block geometry and scalars.  D == H*dh.  ln_eps is LayerNorm's epsilon
 * (biased variance); softmax_scale multiplies q.k (use 1/sqrt(dh)). */
typedef struct fastvar_dims {
    int32_t D;
    int32_t H;
    int32_t dh;
    int32_t F;
    float ln_eps;
    float softmax_scale;
} fastvar_dims;

/* Device pointers to one block's bf16 parameters.  Linear weights are
 * [out_features, in_features] row-major.  w_qkv is [3D, D] with output rows
 * ordered q (D rows, feature = head*dh + d), then k, then v.  Biases may be
 * NULL (treated as zero); everything else must be non-NULL. */
typedef struct fastvar_block_weights {
    const void* ln1_g;  /* [D] */
    const void* ln1_b;  /* [D] */
    const void* w_qkv;  /* [3D, D] */
    const void* b_qkv;  /* [3D] or NULL */
    const void* w_proj; /* [D, D] */
    const void* b_proj; /* [D] or NULL */
    const void* ln2_g;  /* [D] */
    const void* ln2_b;  /* [D] */
    const void* w_fc1;  /* [F, D] */
    const void* b_fc1;  /* [F] or NULL */
    const void* w_fc2;  /* [D, F] */
    const void* b_fc2;  /* [D] or NULL */
} fastvar_block_weights;

/* One block of a stack, for fastvar_scale_step: its weights, its KV cache and
 * its cached output map (Sec. 3.3, overview: the per-layer outputs of the last
 * structure step are saved as the cache). */
typedef struct fastvar_layer {
    const fastvar_block_weights* weights; /* host struct of device pointers */
    void* k_cache;                        /* [B, H, L_cap, dh] bf16 */
    void* v_cache;                        /* [B, H, dh, L_cap] bf16 */
    void* cache_map;                      /* [B, hc*wc, D] bf16, (hc,wc) = sched[cache_step] */
} fastvar_layer;

/* ---- host-only helpers -------------------------------------------------- */

int fastvar_version(void);

/* Static string for an error code. */
const char* fastvar_strerror(int code);

/* Kept-token count for a keep ratio (keep = 1 - pruning ratio, Sec. 4.1):
 * floor(keep_ratio*N + 0.5) evaluated in double, clamped to [0, N].
 * Returns FASTVAR_EINVAL if N < 0. */
int fastvar_keep_count(int N, double keep_ratio);

/* Scratch bytes needed by fastvar_select_pivotal for a [B, N, D] map. */
size_t fastvar_select_workspace_bytes(int B, int N, int D);

/* Scratch bytes needed by fastvar_block_forward_pruned for B*k kept tokens.  Not monotone in k: launches
 * with few workgroups get extra room for partial results that larger ones do not need, so a caller that
 * reuses one buffer over several steps sizes it for the maximum over those steps (the same holds for the
 * step sizes below, which contain this one). */
size_t fastvar_block_workspace_bytes(const fastvar_dims* dims, int B, int k);

/*
 * The pruning schedule as keep counts (Sec. 3.3, overview: the first K-N steps
 * are the structure construction stage and stay unpruned, the per-block
 * outputs of step K-N are cached, the last N steps are pruned; Sec. 4.1: the
 * N progressive pruning ratios, e.g. 40, 50, 100, 100 % or 50, 75 %).  Host
 * function, all pointers host.
 *   sched_h, sched_w  [K] the scale schedule
 *   prune_ratio       [n_pruned] fraction of tokens dropped at each of the last
 *                     n_pruned steps, in step order, each in [0, 1]; 1 drops
 *                     every token (the step is skipped: k = 0)
 *   keep_out          [K] tokens kept per step: h*w for the first K-n_pruned
 *                     steps, fastvar_keep_count(h*w, 1 - ratio) after
 *   cache_step_out    index (from 0) of the cached step, K-n_pruned-1: the
 *                     cache_step argument of the step entry points; -1 when
 *                     n_pruned == 0 (nothing is restored, nothing to cache)
 * FASTVAR_EINVAL: null pointer, K <= 0, a non-positive or too large scale, a
 * ratio outside [0, 1], n_pruned < 0 or n_pruned >= K (no step left to cache).
 */
int fastvar_schedule_plan(const int32_t* sched_h, const int32_t* sched_w, int K, const double* prune_ratio,
                          int n_pruned, int32_t* keep_out, int32_t* cache_step_out);

/* Scratch bytes needed by fastvar_restore when `rank` is NULL (else 0). */
size_t fastvar_restore_workspace_bytes(int B, int N);

/* Scratch bytes needed by fastvar_step (covers all three stages). */
size_t fastvar_step_workspace_bytes(const fastvar_dims* dims, int B, int N, int k);

/* Scratch bytes needed by fastvar_step_sublayer (covers every stage of both halves). */
size_t fastvar_step_sublayer_workspace_bytes(const fastvar_dims* dims, int B, int N, int k_attn, int k_ffn);

/* ---- device entry points ------------------------------------------------ */

/*
 * Pivotal Token Selection (Sec. 3.3, Eq. 4-5; appendix algorithm, first
 * function).
 *   x          [B, h*w, D] bf16   current token map (layer input)
 *   k          tokens to keep per sample, 0 <= k <= h*w <= FASTVAR_MAX_TOKENS
 *   idx_out    [B, k] int32       kept token indices, ascending per sample
 *   rank_out   [B, h*w] int32     position of token n inside idx_out, -1 if
 *                                 pruned; may be NULL
 *   score_out  [B, h*w] fp32      pivotal score; may be NULL
 *   ws         scratch of fastvar_select_workspace_bytes(B, h*w, D) bytes
 * The score is sum_c (x[n,c] - mean[c])^2 with the mean over the h*w
 * positions of the sample, accumulated in fp64 and rounded once to fp32; the
 * top-k decision is taken on that fp32 value, ties going to the lowest token
 * index.  Results are bit-reproducible run to run.
 */
int fastvar_select_pivotal(const void* x, int B, int h, int w, int D, int k,
                           int32_t* idx_out, int32_t* rank_out, float* score_out,
                           void* ws, size_t ws_bytes, void* stream);

/*
 * fastvar_select_pivotal for callers that cannot allocate or provide scratch
 * memory: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and error codes as
 * fastvar_select_pivotal (bit for bit the same idx, rank and score), without
 * ws / ws_bytes: the column-sum partials, the mean and (when score_out is NULL)
 * the scores live in a device array of FASTVAR_SELECT_STATIC_BYTES bytes that
 * is part of the library's code object, one copy per GPU, held until the
 * process ends.  The call allocates nothing and frees nothing.
 *   - FASTVAR_ECAPACITY when fastvar_select_workspace_bytes(B, h*w, D) exceeds
 *     FASTVAR_SELECT_STATIC_BYTES (8 MiB: e.g. B = 1 at 16384 x 2048, B = 2 at
 *     4096 x 2048); nothing is launched then.
 *   - The first call on a device looks up that device's copy of the array
 *     (the one piece of per-process state this library keeps); FASTVAR_EHIP
 *     if the runtime cannot resolve it.
 *   - Every call on a GPU uses the same array, which keeps the last call's
 *     contents; nothing in it has to start at zero (each kernel writes what
 *     the next one reads).  Calls that overlap on one GPU (two streams, two
 *     threads) race on it: serialise them, or use fastvar_select_pivotal with
 *     a scratch buffer per stream.
 */
#define FASTVAR_SELECT_STATIC_BYTES (8u << 20)
int fastvar_select_pivotal_static(const void* x, int B, int h, int w, int D, int k,
                                  int32_t* idx_out, int32_t* rank_out, float* score_out, void* stream);

/*
 * One transformer block on the kept tokens (Sec. 3.3, implementation paragraph:
 * the layer itself is unchanged, it just sees fewer tokens; Sec. 3.1 KV cache).
 *   x          [B, N, D] bf16     current token map
 *   idx        [B, k] int32       kept token indices (from selection)
 *   k_cache    [B, H, L_cap, dh]  bf16, positions [0, L0) valid on entry
 *   v_cache    [B, H, dh, L_cap]  bf16, positions [0, L0) valid on entry
 *   y_kept_out [B, k, D] bf16     block output for the kept tokens
 *   ws         scratch of fastvar_block_workspace_bytes(dims, B, k) bytes
 * Computes xk = x[idx]; h1 = xk + proj(attn(LN1(xk))); y = h1 + fc2(gelu(
 * fc1(LN2(h1)))) with GELU evaluated in its tanh form (within 3e-4 of the erf
 * form, below bf16 resolution); attention is unmasked softmax over
 * cache positions [0, L0+k), the last k of which this call writes.  k == 0
 * is a no-op that returns FASTVAR_OK.  idx may be NULL when k == N: every
 * token is kept, in order -- the unpruned block of the structure construction
 * stage (Sec. 3.3, overview).
 */
int fastvar_block_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k,
                                 const fastvar_dims* dims /* host */,
                                 const fastvar_block_weights* weights /* host struct of device ptrs */,
                                 void* k_cache, void* v_cache, int L0, int L_cap,
                                 void* y_kept_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Cached Token Restoration (Sec. 3.3, Eq. 6; appendix algorithm, second
 * function).
 *   y_kept     [B, k, D] bf16     block output of the kept tokens (NULL ok if k == 0)
 *   idx        [B, k] int32       kept indices, ascending, unique (NULL ok if k == 0)
 *   rank       [B, h*w] int32     inverse map from selection, or NULL to have
 *                                 it rebuilt from idx in `ws`
 *   cache_map  [B, hc*wc, D] bf16 cached output of the last unpruned scale
 *   y_out      [B, h*w, D] bf16   restored map; must not alias any input
 * Kept slots receive the kept outputs bit for bit; every other slot receives
 * the cached map bilinearly resampled at half-pixel centres
 * (src = (dst+0.5)*in/out-0.5 clamped to [0,in-1]), computed in fp32 and
 * rounded once to bf16.  k == 0 gives the pure upsample (a skipped step),
 * k == h*w the pure scatter.
 */
int fastvar_restore(const void* y_kept, const int32_t* idx, const int32_t* rank, int B, int k,
                    const void* cache_map, int hc, int wc, int h, int w, int D,
                    void* y_out, void* ws, size_t ws_bytes, void* stream);

/*
 * Intermediate prediction of the next-scale recursion (Sec. 3.1, Eq. 2):
 * r_out = interpolate(r_prev, (h, w)) + f_k.
 *   r_prev   [B, hp*wp, C] fp32  prediction after the previous step; NULL at
 *                                the first step (then r_out = f_k)
 *   f_k      [B, h*w, C] bf16    the model's output at this step (the residual);
 *                                NULL for a skipped step (pruning ratio 100 %,
 *                                Sec. 4.1: the previous prediction is only
 *                                interpolated to the new size)
 *   r_out    [B, h*w, C] fp32    must not alias r_prev
 * `interpolate` is the bilinear resampling of Eq. 6 (half-pixel centres, edges
 * clamped); the sum is kept in fp32 so that thirteen steps of it do not round
 * thirteen times to bf16.  C % 4 == 0; all pointers device, 16-byte aligned.
 * r_prev and f_k both NULL is FASTVAR_EINVAL.
 */
int fastvar_residual_accumulate(const float* r_prev, int hp, int wp, const void* f_k, int h, int w, int B, int C,
                                float* r_out, void* stream);

/*
 * One whole step for one block: selection, block on kept tokens, restoration
 * (Fig. 2(b) at block granularity).
 *   sched_h, sched_w  host int arrays of length K: the scale schedule
 *   step              index of the scale being decoded; (h,w) = sched[step]
 *   cache_step        index of the scale whose output cache_map holds
 *                     (the last unpruned one, K-N in the paper); < step
 *   kv_len            host in/out: cache length before / after the call
 *   idx_out           [B, k] int32, kept indices (also an output)
 * Other arguments as in the three calls above.
 */
int fastvar_step(const void* x, const int32_t* sched_h /* host */, const int32_t* sched_w /* host */,
                 int K, int step, int cache_step, int B, int k,
                 const fastvar_dims* dims /* host */, const fastvar_block_weights* weights /* host */,
                 void* k_cache, void* v_cache, int32_t* kv_len /* host in/out */, int L_cap,
                 const void* cache_map, void* y_out, int32_t* idx_out,
                 void* ws, size_t ws_bytes, void* stream);

/*
 * One scale step of a whole stack of blocks (Fig. 2(a); Sec. 3.3, overview):
 * the output map of a block is the input of the next.
 *   step <= cache_step  structure construction stage: every block runs
 *                       unpruned (k must equal h*w; no selection, no
 *                       restoration).  At step == cache_step each block's
 *                       output is also written to its cache_map (which must
 *                       then hold [B, h*w, D]): the cache capture.
 *   step >  cache_step  texture filling stage: each block runs selection,
 *                       block on the k kept tokens, restoration from its own
 *                       cache_map, as fastvar_step does (k == h*w runs the
 *                       block unpruned, k == 0 skips it: pure upsample).
 *   layers              host array of n_layers blocks
 *   kv_len              host in/out: every block's cache length before / after
 *   y_out               [B, h*w, D] bf16: output map of the last block
 *   tmp                 [B, h*w, D] bf16 scratch map (may be NULL for one
 *                       block or at the capture step); x, y_out, tmp distinct
 *   idx_out             [B, k] int32: kept indices of the last block (may be
 *                       NULL when k == h*w)
 *   ws                  scratch of fastvar_step_workspace_bytes(dims, B, h*w, k)
 * The token map of a scale is derived from the intermediate prediction
 * (fastvar_residual_accumulate) by the model's tokenizer and embedding, which are
 * outside this library: the caller supplies x.
 */
int fastvar_scale_step(const void* x, const int32_t* sched_h /* host */, const int32_t* sched_w /* host */,
                       int K, int step, int cache_step, int B, int k,
                       const fastvar_dims* dims /* host */, const fastvar_layer* layers /* host */, int n_layers,
                       int32_t* kv_len /* host in/out */, int L_cap,
                       void* y_out, void* tmp, int32_t* idx_out,
                       void* ws, size_t ws_bytes, void* stream);

/* Stages of a block inside the step entry points, for fastvar_scale_step_timed. */
enum {
    FASTVAR_STAGE_SELECT = 0,    /* column sums, scores, top-k */
    FASTVAR_STAGE_LN1 = 1,       /* gather + LayerNorm 1 */
    FASTVAR_STAGE_QKV = 2,       /* QKV GEMM + cache append */
    FASTVAR_STAGE_ATTENTION = 3,
    FASTVAR_STAGE_PROJ = 4,      /* output projection + residual */
    FASTVAR_STAGE_LN2 = 5,
    FASTVAR_STAGE_FC1 = 6,       /* FC1 + GELU */
    FASTVAR_STAGE_FC2 = 7,       /* FC2 + residual */
    FASTVAR_STAGE_RESTORE = 8,
    FASTVAR_N_STAGES = 9
};

/*
 * fastvar_scale_step with a stopwatch: a measurement aid for callers that want the time of each
 * stage inside the running step (the benchmark's roofline figures).  Same arguments and effect;
 * in addition an event is recorded on `stream` after every stage, the call WAITS for the stream
 * to finish (unlike every other entry point) and writes to stage_ms[FASTVAR_N_STAGES] (host) the
 * time of each stage in milliseconds, averaged over the n_layers blocks (at most 256).  Stages that
 * did not run (selection and restoration in structure steps) read 0.  It creates and destroys
 * HIP events.
 */
int fastvar_scale_step_timed(const void* x, const int32_t* sched_h /* host */, const int32_t* sched_w /* host */,
                             int K, int step, int cache_step, int B, int k,
                             const fastvar_dims* dims /* host */, const fastvar_layer* layers /* host */,
                             int n_layers, int32_t* kv_len /* host in/out */, int L_cap,
                             void* y_out, void* tmp, int32_t* idx_out,
                             void* ws, size_t ws_bytes, void* stream, float* stage_ms /* host out */);

/*
 * The two halves of the block, each on its own kept set (Fig. 2(b) and Sec. 3.3,
 * implementation paragraph: the selection / restoration pair wraps each
 * Attention and each FFN layer).  Arguments as in fastvar_block_forward_pruned;
 * both take scratch of fastvar_block_workspace_bytes(dims, B, k) bytes.
 *   attention half:  h_kept_out[B,k,D] = xk + proj(attn(LN1(xk))),  xk = x[idx];
 *                    appends the kept tokens' keys / values at [L0, L0+k)
 *   FFN half:        y_kept_out[B,k,D] = xk + fc2(gelu(fc1(LN2(xk)))),  xk = x[idx]
 * k == 0 is a no-op that returns FASTVAR_OK.
 */
int fastvar_attn_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k,
                                const fastvar_dims* dims /* host */,
                                const fastvar_block_weights* weights /* host struct of device ptrs */,
                                void* k_cache, void* v_cache, int L0, int L_cap,
                                void* h_kept_out, void* ws, size_t ws_bytes, void* stream);
int fastvar_ffn_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k,
                               const fastvar_dims* dims /* host */,
                               const fastvar_block_weights* weights /* host struct of device ptrs */,
                               void* y_kept_out, void* ws, size_t ws_bytes, void* stream);

/*
 * One whole step for one block at sub-layer granularity, the wiring of
 * Fig. 2(b): selection on x, attention half on k_attn kept tokens,
 * restoration from cache_map_attn into x_mid; selection on x_mid, FFN half on
 * k_ffn kept tokens, restoration from cache_map_ffn into y_out.
 *   cache_map_attn, cache_map_ffn  [B, hc*wc, D] bf16: the outputs of this
 *                     block's attention layer and FFN layer (residual stream
 *                     after each) at the cached scale (Sec. 3.3 overview: the
 *                     per-layer outputs of step K-N are saved)
 *   x_mid             [B, h*w, D] bf16, output: the restored map between the
 *                     two halves; must not alias x, y_out or a cache map
 *   idx_attn_out      [B, k_attn] int32, idx_ffn_out [B, k_ffn] int32: the two
 *                     kept sets (outputs)
 *   kv_len            host in/out: grows by k_attn (only the attention half
 *                     writes the cache)
 *   ws                scratch of fastvar_step_sublayer_workspace_bytes(...)
 * Other arguments as in fastvar_step.
 */
int fastvar_step_sublayer(const void* x, const int32_t* sched_h /* host */, const int32_t* sched_w /* host */,
                          int K, int step, int cache_step, int B, int k_attn, int k_ffn,
                          const fastvar_dims* dims /* host */, const fastvar_block_weights* weights /* host */,
                          void* k_cache, void* v_cache, int32_t* kv_len /* host in/out */, int L_cap,
                          const void* cache_map_attn, const void* cache_map_ffn, void* x_mid, void* y_out,
                          int32_t* idx_attn_out, int32_t* idx_ffn_out,
                          void* ws, size_t ws_bytes, void* stream);

/* ---- component entry points ----------------------------------------------
 * The kernels of the block one at a time, with the same launch configuration
 * fastvar_block_forward_pruned uses for the same shapes.  They exist so that
 * each kernel can be checked against the oracle and timed on its own; the
 * block (Sec. 3.3, implementation paragraph: an unchanged transformer layer on
 * fewer tokens; Sec. 3.1 for the KV cache) is their composition.  Same
 * conventions as above; no workspace is needed.
 */

/* out[m,:] = LayerNorm(in[row(m),:]) * gamma + beta for M = B*k rows, biased
 * variance, fp32 statistics.  With idx != NULL row(m) = (m / k) * N + idx[m]
 * (the gather of the kept tokens, appendix algorithm); else row(m) = m. */
int fastvar_layernorm(const void* in, const int32_t* idx, int B, int N, int k, int D,
                      const void* gamma, const void* beta, float eps, void* out, void* stream);

/* out[M,N] = epilogue(A[M,K] * W[N,K]^T + bias); bf16 MFMA, fp32 accumulate.
 * epilogue 1: + residual[M,N];  epilogue 2: GELU (tanh form).  bias may be NULL;
 * residual must be non-NULL for epilogue 1.  K % 64 == 0. */
int fastvar_gemm_bf16(const void* A, const void* W, const void* bias, const void* residual,
                      int M, int N, int K, int epilogue, void* out, void* stream);

/* [q | k | v] = a[B*k, D] * w_qkv[3D, D]^T + b_qkv; q -> q_out [B*k, D]; k and
 * v are appended to the caches at positions [L0, L0+k) (Sec. 3.3: only kept
 * tokens enter the cache). */
int fastvar_qkv_gemm(const void* a, const void* w_qkv, const void* b_qkv, int B, int k,
                     const fastvar_dims* dims /* host */, void* q_out, void* k_cache, void* v_cache,
                     int L0, int L_cap, void* stream);

/*
 * Rotary positions (Sec. 4.1: the backbones the method is applied to, HART and
 * Infinity, carry 2-D rotary position embeddings; the paper gives no formula,
 * the reading is in the design notes).  Axial 2-D rotary embedding on
 * interleaved pairs: pair t of a head's dh/2 pairs (channels 2t, 2t+1) is
 * turned by  pos * base^(-t'/(dh/4)),  the first dh/4 pairs by the grid row of
 * the token's slot (t' = t), the others by its grid column (t' = t - dh/4);
 * coordinates are i * ref_h / h and j * ref_w / w, i.e. the h x w map laid over
 * a ref_h x ref_w reference grid (pass ref = own size for integer coordinates).
 * What makes it part of this path: a kept token keeps the position of its own
 * slot, so the tables are read through the kept index set.
 *
 * fastvar_rope2d_table fills cos_out / sin_out [h*w, dh/2] fp32 (device,
 * 16-byte aligned; dh a multiple of 8) for every slot of the map.
 */
int fastvar_rope2d_table(int h, int w, int dh, double base, int ref_h, int ref_w, float* cos_out, float* sin_out,
                         void* stream);

/* fastvar_qkv_gemm with q and the new keys turned (values are not): row m of
 * `a` is the token at slot idx[m] of its sample's map of N slots (idx [B, k],
 * or NULL when k == N: row t is slot t); tables from fastvar_rope2d_table for
 * that map.  The cache receives the turned keys; earlier cache rows are taken
 * as already turned. */
int fastvar_qkv_gemm_rope(const void* a, const void* w_qkv, const void* b_qkv, const int32_t* idx, int B, int N,
                          int k, const fastvar_dims* dims /* host */, const float* rope_cos, const float* rope_sin,
                          void* q_out, void* k_cache, void* v_cache, int L0, int L_cap, void* stream);

/* fastvar_block_forward_pruned with rotary positions on q and the new keys
 * (same arguments, plus the two tables [N, dh/2] of the map x). */
int fastvar_block_forward_pruned_rope(const void* x, int N, const int32_t* idx, int B, int k,
                                      const fastvar_dims* dims /* host */,
                                      const fastvar_block_weights* weights /* host */, const float* rope_cos,
                                      const float* rope_sin, void* k_cache, void* v_cache, int L0, int L_cap,
                                      void* y_kept_out, void* ws, size_t ws_bytes, void* stream);

/* o[B*k, D] = softmax(q K^T * softmax_scale) V per head over cache positions
 * [0, L), no mask (Sec. 3.1: queries of the current scale see the cached keys
 * of every earlier scale and the current scale's own). */
int fastvar_attention(const void* q, const void* k_cache, const void* v_cache, int B, int k,
                      const fastvar_dims* dims /* host */, int L, int L_cap, void* o, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FASTVAR_H */
