// Host-side launchers of the gfx950 kernels (internal to the library).
// Every launcher enqueues on `stream` and returns; shapes are validated by the
// C-ABI layer before any launcher is called.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <mutex>

namespace fv {

// Raises a kernel's dynamic-LDS limit: a per-function attribute that has to be set once per process before
// the first launch that asks for more than 64 KB.  The once_flag (one per launch site, i.e. per kernel
// instantiation) makes concurrent first calls from several host threads safe.
template <class Kernel>
inline void raise_lds_limit_once(std::once_flag& once, Kernel kernel, size_t bytes) {
    std::call_once(once, [&] {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                                  (int)bytes);
    });
}

// ---- selection (Sec. 3.3, Eq. 4-5) ----
struct SelectPlan {
    int col_tiles;     // column tiles of 512
    int n_chunks;      // row chunks of the column-sum pass
    int rows_per_chunk;
    size_t off_partial;  // fp64 [B, n_chunks, D]
    size_t off_mean;     // fp64 [B, D]
    size_t off_score;    // fp32 [B, N]
    size_t bytes;
};
SelectPlan select_plan(int B, int N, int D);
void launch_select(const void* x, int B, int N, int D, int k, int32_t* idx, int32_t* rank,
                   float* score_out, void* ws, const SelectPlan& plan, hipStream_t stream);

// ---- restoration (Sec. 3.3, Eq. 6) ----
void launch_rank_from_idx(const int32_t* idx, int32_t* rank, int B, int N, int k, hipStream_t stream);
void launch_restore(const void* y_kept, const int32_t* rank, int B, int k, const void* cache_map,
                    int hc, int wc, int h, int w, int D, void* y_out, hipStream_t stream);
// Eq. 2 on fp32 maps [B, h*w, C] (C % 4 == 0): r_out = resample(r_prev [B, hp*wp, C]) + f_k (bf16).
// r_prev or f_k may be null (not both).
void launch_residual_accumulate(const float* r_prev, int hp, int wp, const void* f_k, int h, int w, int B, int C,
                                float* r_out, hipStream_t stream);

// ---- block pieces ----
// xk = x[idx] (optional copy out) and a = LayerNorm(xk); one wave per row.
// rows_out (optional, int32 [B*k]) receives the absolute source row b*N + idx[m] of
// every kept token, for later gathers of the same rows.
void launch_gather_layernorm(const void* x, const int32_t* idx, int B, int N, int k, int D,
                             const void* gamma, const void* beta, float eps, int32_t* rows_out,
                             void* a_out, hipStream_t stream);
// The same launch carrying the restoration's fill as well (Sec. 3.3, Eq. 6): extra workgroups write every
// pruned row (rank[b,n] < 0) of y_out [B, N, D] from cache_map [B, hc*wc, D] resampled to h x w (N = h*w).
// y_out must not be x.  Kept rows of y_out are not touched.
void launch_gather_layernorm_fill(const void* x, const int32_t* idx, int B, int N, int k, int D, const void* gamma,
                                  const void* beta, float eps, int32_t* rows_out, void* a_out, const int32_t* rank,
                                  const void* cache_map, int hc, int wc, int h, int w, void* y_out,
                                  hipStream_t stream);
// a = LayerNorm(rows of `in`), M rows.
void launch_layernorm(const void* in, int M, int D, const void* gamma, const void* beta, float eps,
                      void* a_out, hipStream_t stream);

enum GemmEpilogue {
    EPI_QKV = 0,       // +bias; q -> q_out [M, D]; k, v -> caches at positions L0 + t
    EPI_BIAS_RES = 1,  // out = acc + bias + residual
    EPI_BIAS_GELU = 2  // out = gelu(acc + bias)
};
struct GemmArgs {
    const void* A;     // [M, K] bf16
    const void* W;     // [N, K] bf16
    const void* bias;  // [N] bf16 or null
    int M, N, K;
    // EPI_BIAS_RES / EPI_BIAS_GELU
    void* out;             // [M, N] bf16
    const void* residual;  // [M, N] bf16 (EPI_BIAS_RES), or the gather source when res_idx is set
    const int32_t* res_rows = nullptr;  // optional: the residual of output row m is row res_rows[m] of `residual`
    const int32_t* out_rows = nullptr;  // optional (EPI_BIAS_RES): output row m is written to row out_rows[m] of `out`
    // EPI_QKV
    void* q_out;    // [M, D]
    void* k_cache;  // [B, H, L_cap, dh]
    void* v_cache;  // [B, H, dh, L_cap]
    int D, H, dh, k_tokens, L0, L_cap;
    // EPI_QKV, optional: rotary embedding of q and the new keys.  rope_cos / rope_sin [rope_N, dh/2] fp32
    // (launch_rope2d_table); the slot of output row m is rope_rows[m] % rope_N (a row list that is absolute,
    // b*N + n, or per sample, n, gives the same slot), or with rope_rows == NULL its token index m % k_tokens.
    const float* rope_cos = nullptr;
    const float* rope_sin = nullptr;
    const int32_t* rope_rows = nullptr;
    int rope_N = 0;
    // Optional scratch for the split-K path of shapes with few output tiles (gemm_splitk_plan):
    // [counters | partial tiles]; the counters must be zero on entry and are zero again on exit.
    void* splitk_ws = nullptr;
};
void launch_gemm(GemmEpilogue epi, const GemmArgs& a, hipStream_t stream);

// Split-K plan for a GEMM shape with few output tiles (few rows: the small scales of a schedule, where
// a block is nothing but streaming its weights once): the K range is cut into `splits` slices that run
// as separate workgroups, so that every CU streams a share of the weights; the workgroup that finishes
// a tile last sums the slices in slice order and runs the epilogue.  Up to 256 rows use 64x64 tiles with
// an eight-stage ring (a workgroup's whole K slice, or half of it, is in flight at once), more rows
// 128x128 tiles where K is long; FC2-like shapes a little too tall for those, 256x128 tiles on two slices.
// splits == 1: no scratch needed.
constexpr int kSplitKMaxTiles = 128;   // most output tiles a split-K launch has
struct SplitKPlan {
    int splits;
    int tiles;
    int shape;             // 0: 64x64 tiles, 1: 128x128, 2: 256x128 (count-first exchange)
    int tile_m, tile_n;
    size_t counter_bytes;  // 2 x kSplitKMaxTiles ints (arrivals, ready counts) whatever the shape: GEMMs that share a scratch area share the counters
    size_t bytes;          // counters + partial tiles
};
SplitKPlan gemm_splitk_plan(int M, int N, int K);
// zero the n counters at the head of a split-K scratch area
void launch_zero_i32(int32_t* p, int n, hipStream_t stream);

// cos / sin tables [h*w, dh/2] fp32 of the axial 2-D rotary embedding (see rope.hip).
void launch_rope2d_table(int h, int w, int dh, double base, int ref_h, int ref_w, float* cos_out, float* sin_out,
                         hipStream_t stream);

struct AttnArgs {
    const void* q;        // [B*k, D] bf16 (feature = head*dh + d)
    const void* k_cache;  // [B, H, L_cap, dh]
    const void* v_cache;  // [B, H, dh, L_cap]
    void* o;              // [B*k, D] bf16
    int B, H, dh, k_tokens, L, L_cap;
    float scale;
    // Optional scratch (attention_split_plan) that lets shapes with too few queries to fill the chip
    // split the key range between workgroups; without it every workgroup walks all keys.
    void* split_ws = nullptr;
    size_t split_ws_bytes = 0;   // its size: variants that need more are not considered
};
void launch_attention(const AttnArgs& a, hipStream_t stream);

// Key-range split for attention shapes whose workgroups do not fill whole rounds of 256 CUs (too few
// queries, or a last round that is mostly empty): `splits` workgroups per query tile each take
// `keys_per_split` keys (a multiple of the key tile) and leave unnormalised partial outputs with their
// softmax statistics in scratch; the workgroup that finishes a query tile last merges them (softmax
// partials combine exactly; it adds them in range order, so the result does not depend on who was last).
// The plan is the cheapest of 128- or 256-query workgroups on 2-4 key ranges, for every tile or only for
// the tiles of a part-filled last round (the whole rounds before it stay unsplit), under a simple
// round-count model, if that beats the unsplit launch.  splits == 1: no scratch.  max_bytes != 0: only variants whose
// scratch fits.
struct AttnSplitPlan {
    int splits;
    int keys_per_split;
    bool wide;      // 256-query workgroups (else 128-query ones)
    int full_tiles;        // (sample, head, query tile) triples walked whole by one workgroup (whole rounds of 256)
    int tail_tiles;        // the others, shared by `splits` workgroups each
    int counters;          // arrival counters at the head of the scratch (zero on entry, zero again on exit)
    size_t counter_bytes;
    size_t bytes;          // counters + partial results
};
AttnSplitPlan attention_split_plan(int B, int H, int dh, int k_tokens, int L, size_t max_bytes = 0);

}  // namespace fv
