// C-ABI layer: argument validation, workspace carving and launch order.
// Everything that computes runs in the kernels; this file only checks,
// slices the caller's scratch buffer and enqueues.
#include "../../include/fastvar.h"

#include <hip/hip_runtime.h>
#include <math.h>

#include <mutex>

#include "kernels.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round256(size_t v) { return (v + 255) & ~(size_t)255; }

constexpr int kMaxWidth = 8192;  // LayerNorm keeps a row in registers; score keeps the mean in 64 KB of LDS

struct BlockPlan {
    size_t off_a, off_q, off_h1, off_u, off_rows, off_asplit, asplit_bytes, off_sk, sk_bytes, bytes;
    int sk_counters, asplit_counters;
};

BlockPlan block_plan(const fastvar_dims* d, int B, int k) {
    const size_t M = (size_t)B * (size_t)k;
    BlockPlan p;
    size_t off = 0;
    p.off_a = off;   off += round256(M * d->D * 2);  // LN1 output, later the attention output
    p.off_q = off;   off += round256(M * d->D * 2);  // queries, later the LN2 output
    p.off_h1 = off;  off += round256(M * d->D * 2);  // residual stream after attention
    p.off_u = off;   off += round256(M * d->F * 2);  // MLP hidden
    p.off_rows = off; off += round256(M * 4);        // absolute source row of every kept token
    // partial outputs of an attention whose key range is split between workgroups: sized for the plan
    // of an unbounded cache length (every variant admissible); with the real length the launcher only
    // considers variants that fit into this
    p.asplit_bytes = 0;
    p.asplit_counters = 0;
    if (k > 0) {
        const fv::AttnSplitPlan sp = fv::attention_split_plan(B, d->H, d->dh, k, 1 << 28);
        if (sp.splits > 1) {
            p.asplit_bytes = sp.bytes;
            p.asplit_counters = (int)(sp.counter_bytes / 4);
        }
    }
    p.off_asplit = off; off += round256(p.asplit_bytes);
    // split-K scratch of the GEMMs (only shapes with few output tiles have any): one area, the
    // largest of the four, used by one GEMM at a time
    p.sk_bytes = 0;
    p.sk_counters = 0;
    const int shapes[4][2] = {{3 * d->D, d->D}, {d->D, d->D}, {d->F, d->D}, {d->D, d->F}};
    for (const auto& nk : shapes) {
        const fv::SplitKPlan sk = fv::gemm_splitk_plan((int)M, nk[0], nk[1]);
        if (sk.bytes > p.sk_bytes) p.sk_bytes = sk.bytes;
        if (sk.splits > 1) p.sk_counters = (int)(sk.counter_bytes / 4);
    }
    p.off_sk = off; off += round256(p.sk_bytes);
    p.bytes = off;
    return p;
}

int check_dims(const fastvar_dims* d) {
    if (!d) return FASTVAR_EINVAL;
    if (d->D <= 0 || d->H <= 0 || d->dh <= 0 || d->F <= 0) return FASTVAR_EINVAL;
    if ((long)d->H * d->dh != d->D) return FASTVAR_EINVAL;
    if (!(d->ln_eps >= 0.f) || !(d->softmax_scale > 0.f) || !isfinite(d->softmax_scale)) return FASTVAR_EINVAL;
    if (d->D % 64 != 0 || d->F % 64 != 0) return FASTVAR_EALIGN;
    if (d->dh != 64 && d->dh != 128) return FASTVAR_EALIGN;
    if (d->D > kMaxWidth) return FASTVAR_ECAPACITY;
    return FASTVAR_OK;
}

int check_weights(const fastvar_block_weights* w) {
    if (!w) return FASTVAR_EINVAL;
    const void* need[] = {w->ln1_g, w->ln1_b, w->w_qkv, w->w_proj, w->ln2_g, w->ln2_b, w->w_fc1, w->w_fc2};
    for (const void* p : need) {
        if (!p) return FASTVAR_EINVAL;
        if (!aligned16(p)) return FASTVAR_EALIGN;
    }
    const void* opt[] = {w->b_qkv, w->b_proj, w->b_fc1, w->b_fc2};
    for (const void* p : opt)
        if (p && !aligned16(p)) return FASTVAR_EALIGN;
    return FASTVAR_OK;
}

int check_select(const void* x, int B, int h, int w, int D, int k, const int32_t* idx, const void* ws,
                 size_t ws_bytes) {
    if (!x || B <= 0 || h <= 0 || w <= 0 || D <= 0) return FASTVAR_EINVAL;
    const long N = (long)h * w;
    if (k < 0 || k > N) return FASTVAR_EINVAL;
    if (k > 0 && !idx) return FASTVAR_EINVAL;
    if (N > FASTVAR_MAX_TOKENS || D > kMaxWidth) return FASTVAR_ECAPACITY;
    if ((double)B * (double)N * (double)D >= 2147483648.0 * 4.0) return FASTVAR_ECAPACITY;
    if (D % 8 != 0 || !aligned16(x) || (ws && !aligned16(ws))) return FASTVAR_EALIGN;
    if (!ws || ws_bytes < fastvar_select_workspace_bytes(B, (int)N, D)) return FASTVAR_EWORKSPACE;
    return FASTVAR_OK;
}

int check_block(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* dims,
                const fastvar_block_weights* wts, const void* kc, const void* vc, int L0, int L_cap,
                const void* y, const void* ws, size_t ws_bytes) {
    int rc = check_dims(dims);
    if (rc) return rc;
    rc = check_weights(wts);
    if (rc) return rc;
    if (!x || !kc || !vc || B <= 0 || N <= 0 || k < 0 || k > N || L0 < 0 || L_cap <= 0) return FASTVAR_EINVAL;
    if (k > 0 && (!y || (!idx && k != N))) return FASTVAR_EINVAL;   // no index list: every token kept
    if ((long)L0 + k > L_cap) return FASTVAR_ECAPACITY;
    if (L_cap % 8 != 0) return FASTVAR_EALIGN;
    if (!aligned16(x) || !aligned16(kc) || !aligned16(vc) || (y && !aligned16(y)) || (ws && !aligned16(ws)))
        return FASTVAR_EALIGN;
    // 32-bit element offsets inside the GEMM operand loads
    const double M = (double)B * k;
    const double widest = dims->F > 3 * dims->D ? dims->F : 3 * dims->D;
    if (M * widest >= 2147483648.0 || (double)widest * dims->F >= 2147483648.0) return FASTVAR_ECAPACITY;
    if (k > 0 && (!ws || ws_bytes < fastvar_block_workspace_bytes(dims, B, k))) return FASTVAR_EWORKSPACE;
    return FASTVAR_OK;
}

int check_restore(const void* y_kept, const int32_t* idx, const int32_t* rank, int B, int k, const void* cache,
                  int hc, int wc, int h, int w, int D, const void* y_out, const void* ws, size_t ws_bytes) {
    if (!cache || !y_out || B <= 0 || hc <= 0 || wc <= 0 || h <= 0 || w <= 0 || D <= 0) return FASTVAR_EINVAL;
    const long N = (long)h * w;
    if (k < 0 || k > N) return FASTVAR_EINVAL;
    if (k > 0 && (!y_kept || (!rank && !idx))) return FASTVAR_EINVAL;
    if (y_out == cache || (k > 0 && y_out == y_kept)) return FASTVAR_EINVAL;
    if (N > FASTVAR_MAX_TOKENS) return FASTVAR_ECAPACITY;
    if (D % 8 != 0 || !aligned16(cache) || !aligned16(y_out) || (y_kept && !aligned16(y_kept)))
        return FASTVAR_EALIGN;
    if (k > 0 && !rank) {
        if (!ws || ws_bytes < fastvar_restore_workspace_bytes(B, (int)N)) return FASTVAR_EWORKSPACE;
        if (!aligned16(ws)) return FASTVAR_EALIGN;
    }
    return FASTVAR_OK;
}

int launch_status() { return hipGetLastError() == hipSuccess ? FASTVAR_OK : FASTVAR_EHIP; }

// Scratch of fastvar_select_pivotal_static: part of the code object, so every GPU the library runs on holds
// its own copy at its own address.  In host code the array's name is only a handle for the symbol lookup
// below, never a device address: kernels are given the looked-up pointer.
constexpr int kMaxDevices = 64;
static __device__ __align__(256) unsigned char g_select_scratch[FASTVAR_SELECT_STATIC_BYTES];
static_assert(sizeof(g_select_scratch) == FASTVAR_SELECT_STATIC_BYTES, "header and array agree");
std::mutex g_select_scratch_mu;
void* g_select_scratch_ptr[kMaxDevices] = {};

// Device address of the current device's copy of the array, looked up once per device (with that device
// current, as it is for the caller's launch) and kept.
int select_scratch_address(void** out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return FASTVAR_EHIP;
    std::lock_guard<std::mutex> lock(g_select_scratch_mu);
    if (!g_select_scratch_ptr[dev]) {
        void* p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(g_select_scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return FASTVAR_EHIP;
        }
        g_select_scratch_ptr[dev] = p;
    }
    *out = g_select_scratch_ptr[dev];
    return FASTVAR_OK;
}

// Optional per-stage timing of the step entry points (fastvar_scale_step_timed): when a profile is
// installed for the calling thread, an event is recorded on the launch stream after every stage.
constexpr int kMaxMarks = 1 + FASTVAR_N_STAGES * 256;
struct StepProfile {
    hipEvent_t ev[kMaxMarks];
    int stage[kMaxMarks];
    int n = 0;
};
thread_local StepProfile* g_profile = nullptr;
inline void mark(hipStream_t st, int stage) {
    StepProfile* p = g_profile;
    if (p && p->n < kMaxMarks) {
        (void)hipEventRecord(p->ev[p->n], st);
        p->stage[p->n++] = stage;
    }
}

// The restoration's fill (Sec. 3.3, Eq. 6), handed to the gather launch of the layer it belongs to: the
// pruned rows of y_out [B, h*w, D] are written from cache_map while the kept rows are normalised; the
// layer's last GEMM then scatters the kept rows into y_out, which completes the restored map.
struct Fill {
    const int32_t* rank;
    const void* cache_map;
    int hc, wc, h, w;
    void* y_out;
};

// Rotary tables [N, dh/2] fp32 for the map the block's tokens come from (fastvar_rope2d_table).
struct Rope {
    const float* cos;
    const float* sin;
};

// Attention half of the block on the kept tokens: h1 = x[idx] + proj(attn(LN1(x[idx]))).
// Scratch used: a, q, rows of the block plan.
// `scatter`: h1_out is a [B, N, D] map and row m goes to the kept token's own row of it.
void enqueue_attn(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* d,
                  const fastvar_block_weights* w, void* kc, void* vc, int L0, int L_cap, void* h1_out, void* ws,
                  hipStream_t st, bool scatter = false, const Fill* fill = nullptr, const Rope* rope = nullptr) {
    const BlockPlan bp = block_plan(d, B, k);
    char* base = static_cast<char*>(ws);
    void* buf_a = base + bp.off_a;
    void* buf_q = base + bp.off_q;
    int32_t* rows = reinterpret_cast<int32_t*>(base + bp.off_rows);
    void* sk = bp.sk_bytes ? base + bp.off_sk : nullptr;
    const int M = B * k;

    // a1 = LN1(x[idx]); without an index list every token is kept, in order
    if (idx && fill)
        fv::launch_gather_layernorm_fill(x, idx, B, N, k, d->D, w->ln1_g, w->ln1_b, d->ln_eps, rows, buf_a,
                                         fill->rank, fill->cache_map, fill->hc, fill->wc, fill->h, fill->w,
                                         fill->y_out, st);
    else if (idx)
        fv::launch_gather_layernorm(x, idx, B, N, k, d->D, w->ln1_g, w->ln1_b, d->ln_eps, rows, buf_a, st);
    else
        fv::launch_layernorm(x, M, d->D, w->ln1_g, w->ln1_b, d->ln_eps, buf_a, st);
    mark(st, FASTVAR_STAGE_LN1);
    // q | k | v = a1 * Wqkv^T + b ; k, v appended to the caches at [L0, L0+k)
    fv::GemmArgs g{};
    g.A = buf_a; g.W = w->w_qkv; g.bias = w->b_qkv; g.M = M; g.N = 3 * d->D; g.K = d->D;
    g.q_out = buf_q; g.k_cache = kc; g.v_cache = vc;
    g.D = d->D; g.H = d->H; g.dh = d->dh; g.k_tokens = k; g.L0 = L0; g.L_cap = L_cap;
    g.splitk_ws = sk;
    if (rope) {   // q and the new keys are turned by the angles of each kept token's own slot
        g.rope_cos = rope->cos; g.rope_sin = rope->sin; g.rope_rows = idx ? rows : nullptr; g.rope_N = N;
    }
    fv::launch_gemm(fv::EPI_QKV, g, st);
    mark(st, FASTVAR_STAGE_QKV);
    // o = softmax(q K^T * scale) V over cache positions [0, L0+k)
    fv::AttnArgs at{};
    at.q = buf_q; at.k_cache = kc; at.v_cache = vc; at.o = buf_a;
    at.B = B; at.H = d->H; at.dh = d->dh; at.k_tokens = k; at.L = L0 + k; at.L_cap = L_cap;
    at.scale = d->softmax_scale;
    at.split_ws = bp.asplit_bytes ? base + bp.off_asplit : nullptr;
    at.split_ws_bytes = bp.asplit_bytes;
    fv::launch_attention(at, st);
    mark(st, FASTVAR_STAGE_ATTENTION);
    // h1 = x[idx] + o * Wp^T + bp
    fv::GemmArgs pj{};
    pj.A = buf_a; pj.W = w->w_proj; pj.bias = w->b_proj; pj.M = M; pj.N = d->D; pj.K = d->D;
    pj.out = h1_out; pj.residual = x; pj.res_rows = idx ? rows : nullptr; pj.k_tokens = k;
    pj.out_rows = (scatter && idx) ? rows : nullptr;
    pj.splitk_ws = sk;
    fv::launch_gemm(fv::EPI_BIAS_RES, pj, st);
    mark(st, FASTVAR_STAGE_PROJ);
}

// MLP half: y = s + fc2(gelu(fc1(LN2(s)))), where s = src[idx] (rows gathered from a [B, N, D]
// map) or, with idx == NULL, the contiguous [B*k, D] rows at src.  Scratch used: q, u, rows.
// `scatter_rows`: y is a [B, N, D] map and row m goes to row scatter_rows[m] of it (the absolute row of
// the kept token, as left in the plan's row list by the gather).
void enqueue_ffn(const void* src, int N, const int32_t* idx, int B, int k, const fastvar_dims* d,
                 const fastvar_block_weights* w, void* y, void* ws, hipStream_t st, bool scatter = false,
                 const Fill* fill = nullptr) {
    const BlockPlan bp = block_plan(d, B, k);
    char* base = static_cast<char*>(ws);
    void* buf_q = base + bp.off_q;
    void* buf_u = base + bp.off_u;
    int32_t* rows = reinterpret_cast<int32_t*>(base + bp.off_rows);
    void* sk = bp.sk_bytes ? base + bp.off_sk : nullptr;
    const int M = B * k;

    // a2 = LN2(s)
    if (idx && fill)
        fv::launch_gather_layernorm_fill(src, idx, B, N, k, d->D, w->ln2_g, w->ln2_b, d->ln_eps, rows, buf_q,
                                         fill->rank, fill->cache_map, fill->hc, fill->wc, fill->h, fill->w,
                                         fill->y_out, st);
    else if (idx)
        fv::launch_gather_layernorm(src, idx, B, N, k, d->D, w->ln2_g, w->ln2_b, d->ln_eps, rows, buf_q, st);
    else
        fv::launch_layernorm(src, M, d->D, w->ln2_g, w->ln2_b, d->ln_eps, buf_q, st);
    mark(st, FASTVAR_STAGE_LN2);
    // u = gelu(a2 * W1^T + b1)
    fv::GemmArgs f1{};
    f1.A = buf_q; f1.W = w->w_fc1; f1.bias = w->b_fc1; f1.M = M; f1.N = d->F; f1.K = d->D;
    f1.out = buf_u; f1.k_tokens = k;
    f1.splitk_ws = sk;
    fv::launch_gemm(fv::EPI_BIAS_GELU, f1, st);
    mark(st, FASTVAR_STAGE_FC1);
    // y = s + u * W2^T + b2
    fv::GemmArgs f2{};
    f2.A = buf_u; f2.W = w->w_fc2; f2.bias = w->b_fc2; f2.M = M; f2.N = d->D; f2.K = d->F;
    f2.out = y; f2.residual = src; f2.res_rows = idx ? rows : nullptr; f2.k_tokens = k;
    f2.out_rows = scatter ? rows : nullptr;
    f2.splitk_ws = sk;
    fv::launch_gemm(fv::EPI_BIAS_RES, f2, st);
    mark(st, FASTVAR_STAGE_FC2);
}

// `scatter`: y is the [B, N, D] output map and the kept tokens' outputs go straight to their own rows
// (the row list written by the gather of the attention half is still in the plan when FC2 runs).
// The arrival counters of the split-K scratch (GEMM) and of the key-range split (attention) must be zero
// before the first kernel that uses them; every such kernel leaves them zero again, so once per
// entry-point call is enough.
void zero_splitk_counters(void* ws, const fastvar_dims* d, int B, int k, hipStream_t st) {
    if (k <= 0) return;
    const BlockPlan bp = block_plan(d, B, k);
    if (bp.sk_bytes)
        fv::launch_zero_i32(reinterpret_cast<int32_t*>(static_cast<char*>(ws) + bp.off_sk), bp.sk_counters, st);
    if (bp.asplit_bytes)
        fv::launch_zero_i32(reinterpret_cast<int32_t*>(static_cast<char*>(ws) + bp.off_asplit), bp.asplit_counters, st);
}

void enqueue_block(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* d,
                   const fastvar_block_weights* w, void* kc, void* vc, int L0, int L_cap, void* y, void* ws,
                   hipStream_t st, bool scatter = false, const Fill* fill = nullptr, const Rope* rope = nullptr) {
    void* buf_h1 = static_cast<char*>(ws) + block_plan(d, B, k).off_h1;
    enqueue_attn(x, N, idx, B, k, d, w, kc, vc, L0, L_cap, buf_h1, ws, st, false, idx ? fill : nullptr, rope);
    enqueue_ffn(buf_h1, 0, nullptr, B, k, d, w, y, ws, st, scatter && idx);
}

int check_ffn(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* dims,
              const fastvar_block_weights* wts, const void* y, const void* ws, size_t ws_bytes) {
    int rc = check_dims(dims);
    if (rc) return rc;
    rc = check_weights(wts);
    if (rc) return rc;
    if (!x || B <= 0 || N <= 0 || k < 0 || k > N) return FASTVAR_EINVAL;
    if (k > 0 && (!idx || !y)) return FASTVAR_EINVAL;
    if (!aligned16(x) || (y && !aligned16(y)) || (ws && !aligned16(ws))) return FASTVAR_EALIGN;
    const double M = (double)B * k;
    if (M * dims->F >= 2147483648.0 || (double)dims->D * dims->F >= 2147483648.0) return FASTVAR_ECAPACITY;
    if (k > 0 && (!ws || ws_bytes < fastvar_block_workspace_bytes(dims, B, k))) return FASTVAR_EWORKSPACE;
    return FASTVAR_OK;
}

}  // namespace

extern "C" {

int fastvar_version(void) { return FASTVAR_VERSION; }

const char* fastvar_strerror(int code) {
    switch (code) {
        case FASTVAR_OK: return "ok";
        case FASTVAR_EINVAL: return "invalid argument";
        case FASTVAR_ECAPACITY: return "capacity exceeded";
        case FASTVAR_EWORKSPACE: return "workspace too small";
        case FASTVAR_EALIGN: return "misaligned pointer or unsupported width";
        case FASTVAR_EHIP: return "HIP launch failed";
        default: return "unknown error";
    }
}

int fastvar_keep_count(int N, double keep_ratio) {
    if (N < 0) return FASTVAR_EINVAL;
    if (!(keep_ratio > 0.0)) return 0;
    const double v = floor(keep_ratio * (double)N + 0.5);
    if (v >= (double)N) return N;
    return (int)v;
}

int fastvar_schedule_plan(const int32_t* sched_h, const int32_t* sched_w, int K, const double* prune_ratio,
                          int n_pruned, int32_t* keep_out, int32_t* cache_step_out) {
    if (!sched_h || !sched_w || !keep_out || !cache_step_out || K <= 0) return FASTVAR_EINVAL;
    if (n_pruned < 0 || n_pruned >= K || (n_pruned > 0 && !prune_ratio)) return FASTVAR_EINVAL;
    for (int i = 0; i < K; ++i)
        if (sched_h[i] <= 0 || sched_w[i] <= 0 || (long)sched_h[i] * sched_w[i] > FASTVAR_MAX_TOKENS)
            return FASTVAR_EINVAL;
    for (int j = 0; j < n_pruned; ++j)
        if (!(prune_ratio[j] >= 0.0 && prune_ratio[j] <= 1.0)) return FASTVAR_EINVAL;
    const int first_pruned = K - n_pruned;
    for (int i = 0; i < K; ++i) {
        const int N = sched_h[i] * sched_w[i];
        keep_out[i] = i < first_pruned ? N : fastvar_keep_count(N, 1.0 - prune_ratio[i - first_pruned]);
    }
    *cache_step_out = n_pruned > 0 ? first_pruned - 1 : -1;
    return FASTVAR_OK;
}

size_t fastvar_select_workspace_bytes(int B, int N, int D) {
    if (B <= 0 || N <= 0 || D <= 0) return 0;
    return fv::select_plan(B, N, D).bytes;
}

size_t fastvar_block_workspace_bytes(const fastvar_dims* dims, int B, int k) {
    if (!dims || B <= 0 || k <= 0 || dims->D <= 0 || dims->F <= 0) return 0;
    return block_plan(dims, B, k).bytes;
}

size_t fastvar_restore_workspace_bytes(int B, int N) {
    if (B <= 0 || N <= 0) return 0;
    return round256((size_t)B * N * sizeof(int32_t));
}

size_t fastvar_step_workspace_bytes(const fastvar_dims* dims, int B, int N, int k) {
    if (!dims || B <= 0 || N <= 0) return 0;
    return fastvar_select_workspace_bytes(B, N, dims->D) + fastvar_restore_workspace_bytes(B, N) +
           fastvar_block_workspace_bytes(dims, B, k);
}

int fastvar_select_pivotal(const void* x, int B, int h, int w, int D, int k, int32_t* idx_out,
                           int32_t* rank_out, float* score_out, void* ws, size_t ws_bytes, void* stream) {
    const int rc = check_select(x, B, h, w, D, k, idx_out, ws, ws_bytes);
    if (rc) return rc;
    const int N = h * w;
    const fv::SelectPlan plan = fv::select_plan(B, N, D);
    fv::launch_select(x, B, N, D, k, idx_out, rank_out, score_out, ws, plan, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_select_pivotal_static(const void* x, int B, int h, int w, int D, int k, int32_t* idx_out,
                                  int32_t* rank_out, float* score_out, void* stream) {
    // sizes first: no HIP call is made for a request that cannot be served
    if (B <= 0 || h <= 0 || w <= 0 || D <= 0) return FASTVAR_EINVAL;
    if ((long)h * w > FASTVAR_MAX_TOKENS || D > kMaxWidth) return FASTVAR_ECAPACITY;
    if ((double)B * h * w * D >= 2147483648.0 * 4.0) return FASTVAR_ECAPACITY;
    const size_t need = fastvar_select_workspace_bytes(B, h * w, D);
    if (need > sizeof(g_select_scratch)) return FASTVAR_ECAPACITY;
    void* ws = nullptr;
    int rc = select_scratch_address(&ws);
    if (rc) return rc;
    rc = check_select(x, B, h, w, D, k, idx_out, ws, need);
    if (rc) return rc;
    const int N = h * w;
    fv::launch_select(x, B, N, D, k, idx_out, rank_out, score_out, ws, fv::select_plan(B, N, D),
                      static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_block_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k,
                                 const fastvar_dims* dims, const fastvar_block_weights* weights, void* k_cache,
                                 void* v_cache, int L0, int L_cap, void* y_kept_out, void* ws, size_t ws_bytes,
                                 void* stream) {
    const int rc = check_block(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, y_kept_out, ws,
                               ws_bytes);
    if (rc) return rc;
    if (k == 0) return FASTVAR_OK;
    zero_splitk_counters(ws, dims, B, k, static_cast<hipStream_t>(stream));
    enqueue_block(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, y_kept_out, ws,
                  static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_rope2d_table(int h, int w, int dh, double base, int ref_h, int ref_w, float* cos_out, float* sin_out,
                         void* stream) {
    if (!cos_out || !sin_out || h <= 0 || w <= 0 || ref_h <= 0 || ref_w <= 0 || !(base > 0.0) || !isfinite(base))
        return FASTVAR_EINVAL;
    if ((long)h * w > FASTVAR_MAX_TOKENS) return FASTVAR_ECAPACITY;
    if (dh <= 0 || dh % 8 != 0 || !aligned16(cos_out) || !aligned16(sin_out)) return FASTVAR_EALIGN;
    fv::launch_rope2d_table(h, w, dh, base, ref_h, ref_w, cos_out, sin_out, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_block_forward_pruned_rope(const void* x, int N, const int32_t* idx, int B, int k,
                                      const fastvar_dims* dims, const fastvar_block_weights* weights,
                                      const float* rope_cos, const float* rope_sin, void* k_cache, void* v_cache,
                                      int L0, int L_cap, void* y_kept_out, void* ws, size_t ws_bytes, void* stream) {
    if (!rope_cos || !rope_sin) return FASTVAR_EINVAL;
    if (!aligned16(rope_cos) || !aligned16(rope_sin)) return FASTVAR_EALIGN;
    const int rc = check_block(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, y_kept_out, ws,
                               ws_bytes);
    if (rc) return rc;
    if (k == 0) return FASTVAR_OK;
    const Rope rope{rope_cos, rope_sin};
    zero_splitk_counters(ws, dims, B, k, static_cast<hipStream_t>(stream));
    enqueue_block(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, y_kept_out, ws,
                  static_cast<hipStream_t>(stream), false, nullptr, &rope);
    return launch_status();
}

int fastvar_restore(const void* y_kept, const int32_t* idx, const int32_t* rank, int B, int k,
                    const void* cache_map, int hc, int wc, int h, int w, int D, void* y_out, void* ws,
                    size_t ws_bytes, void* stream) {
    const int rc = check_restore(y_kept, idx, rank, B, k, cache_map, hc, wc, h, w, D, y_out, ws, ws_bytes);
    if (rc) return rc;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int N = h * w;
    if (k > 0 && !rank) {
        int32_t* rebuilt = static_cast<int32_t*>(ws);
        fv::launch_rank_from_idx(idx, rebuilt, B, N, k, st);
        rank = rebuilt;
    }
    fv::launch_restore(y_kept, rank, B, k, cache_map, hc, wc, h, w, D, y_out, st);
    return launch_status();
}

int fastvar_residual_accumulate(const float* r_prev, int hp, int wp, const void* f_k, int h, int w, int B, int C,
                                float* r_out, void* stream) {
    if (!r_out || (!r_prev && !f_k) || B <= 0 || h <= 0 || w <= 0 || C <= 0) return FASTVAR_EINVAL;
    if (r_prev && (hp <= 0 || wp <= 0)) return FASTVAR_EINVAL;
    if ((long)h * w > FASTVAR_MAX_TOKENS || (r_prev && (long)hp * wp > FASTVAR_MAX_TOKENS)) return FASTVAR_ECAPACITY;
    if (C % 4 != 0 || !aligned16(r_out) || (r_prev && !aligned16(r_prev)) || (f_k && !aligned16(f_k)))
        return FASTVAR_EALIGN;
    if (r_out == r_prev) return FASTVAR_EINVAL;
    fv::launch_residual_accumulate(r_prev, hp, wp, f_k, h, w, B, C, r_out, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_step(const void* x, const int32_t* sched_h, const int32_t* sched_w, int K, int step, int cache_step,
                 int B, int k, const fastvar_dims* dims, const fastvar_block_weights* weights, void* k_cache,
                 void* v_cache, int32_t* kv_len, int L_cap, const void* cache_map, void* y_out,
                 int32_t* idx_out, void* ws, size_t ws_bytes, void* stream) {
    if (!sched_h || !sched_w || !kv_len || K <= 0) return FASTVAR_EINVAL;
    if (step < 0 || step >= K || cache_step < 0 || cache_step >= step) return FASTVAR_EINVAL;
    const int h = sched_h[step], w = sched_w[step];
    const int hc = sched_h[cache_step], wc = sched_w[cache_step];
    if (h <= 0 || w <= 0 || hc <= 0 || wc <= 0 || (long)h * w > FASTVAR_MAX_TOKENS) return FASTVAR_EINVAL;
    const int N = h * w;
    const int L0 = *kv_len;
    int rc = check_dims(dims);
    if (rc) return rc;
    const int D = dims->D;
    if (B <= 0 || k < 0 || k > N || y_out == x) return FASTVAR_EINVAL;
    if (!ws) return FASTVAR_EWORKSPACE;
    if (!aligned16(ws)) return FASTVAR_EALIGN;
    if (ws_bytes < fastvar_step_workspace_bytes(dims, B, N, k)) return FASTVAR_EWORKSPACE;

    // scratch: [selection | rank [B,N] | block buffers]
    const size_t sel_bytes = fastvar_select_workspace_bytes(B, N, D);
    const size_t rank_bytes = fastvar_restore_workspace_bytes(B, N);
    char* base = static_cast<char*>(ws);
    void* ws_sel = base;
    int32_t* rank = reinterpret_cast<int32_t*>(base + sel_bytes);
    char* ws_blk = base + sel_bytes + rank_bytes;
    const size_t blk_bytes = ws_bytes - sel_bytes - rank_bytes;
    // Stand-in for a kept-output buffer in the argument checks below (the block's last GEMM writes the
    // kept rows of y_out directly).
    void* yk = k > 0 ? static_cast<void*>(ws_blk + block_plan(dims, B, k).off_q) : nullptr;

    rc = check_select(x, B, h, w, D, k, idx_out, ws_sel, sel_bytes);
    if (rc) return rc;
    rc = check_block(x, N, idx_out, B, k, dims, weights, k_cache, v_cache, L0, L_cap, yk, ws_blk, blk_bytes);
    if (rc) return rc;
    rc = check_restore(yk, idx_out, rank, B, k, cache_map, hc, wc, h, w, D, y_out, nullptr, 0);
    if (rc) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    zero_splitk_counters(ws_blk, dims, B, k, st);
    fv::launch_select(x, B, N, D, k, idx_out, rank, nullptr, ws_sel, fv::select_plan(B, N, D), st);
    // Restoration has no launch of its own: the pruned rows of y_out are filled by extra workgroups of the
    // gather + LayerNorm launch, the kept rows are written by the block's last GEMM.  With nothing kept
    // the step is the upsampled cache.
    const Fill fill{rank, cache_map, hc, wc, h, w, y_out};
    if (k > 0)
        enqueue_block(x, N, idx_out, B, k, dims, weights, k_cache, v_cache, L0, L_cap, y_out, ws_blk, st, true, &fill);
    else
        fv::launch_restore(nullptr, rank, B, k, cache_map, hc, wc, h, w, D, y_out, st);
    rc = launch_status();
    if (rc == FASTVAR_OK) *kv_len = L0 + k;
    return rc;
}

int fastvar_scale_step(const void* x, const int32_t* sched_h, const int32_t* sched_w, int K, int step,
                       int cache_step, int B, int k, const fastvar_dims* dims, const fastvar_layer* layers,
                       int n_layers, int32_t* kv_len, int L_cap, void* y_out, void* tmp, int32_t* idx_out,
                       void* ws, size_t ws_bytes, void* stream) {
    if (!sched_h || !sched_w || !kv_len || !layers || K <= 0 || n_layers <= 0) return FASTVAR_EINVAL;
    if (step < 0 || step >= K || cache_step < 0 || cache_step >= K) return FASTVAR_EINVAL;
    const int h = sched_h[step], w = sched_w[step];
    if (h <= 0 || w <= 0 || (long)h * w > FASTVAR_MAX_TOKENS) return FASTVAR_EINVAL;
    const int N = h * w;
    const bool structure = step <= cache_step;      // structure stage: standard, unpruned
    const bool capture = step == cache_step;
    if (B <= 0 || k < 0 || k > N || (structure && k != N)) return FASTVAR_EINVAL;
    int rc = check_dims(dims);
    if (rc) return rc;
    const int D = dims->D;
    if (!x || !y_out || y_out == x || tmp == x || tmp == y_out) return FASTVAR_EINVAL;
    if (!tmp && n_layers > 1 && !capture) return FASTVAR_EINVAL;
    if (!aligned16(x) || !aligned16(y_out) || (tmp && !aligned16(tmp))) return FASTVAR_EALIGN;
    if (!ws) return FASTVAR_EWORKSPACE;
    if (!aligned16(ws)) return FASTVAR_EALIGN;
    if (ws_bytes < fastvar_step_workspace_bytes(dims, B, N, k)) return FASTVAR_EWORKSPACE;
    const int L0 = *kv_len;
    const bool dense = k == N;
    if (!dense && !idx_out) return FASTVAR_EINVAL;
    const int hc = sched_h[cache_step], wc = sched_w[cache_step];

    const size_t sel_bytes = fastvar_select_workspace_bytes(B, N, D);
    const size_t rank_bytes = fastvar_restore_workspace_bytes(B, N);
    char* base = static_cast<char*>(ws);
    void* ws_sel = base;
    int32_t* rank = reinterpret_cast<int32_t*>(base + sel_bytes);
    char* ws_blk = base + sel_bytes + rank_bytes;
    const size_t blk_bytes = ws_bytes - sel_bytes - rank_bytes;
    void* yk = k > 0 ? static_cast<void*>(ws_blk + block_plan(dims, B, k).off_q) : nullptr;

    // Every layer is checked before the first launch.  Output of layer l: its own cache map at the
    // capture step (the next layer reads it from there), else tmp / y_out alternating so that the last
    // layer writes y_out.
    auto dst_of = [&](int l) -> void* {
        if (capture) return layers[l].cache_map;
        return ((n_layers - 1 - l) % 2 == 0) ? y_out : tmp;
    };
    for (int l = 0; l < n_layers; ++l) {
        const fastvar_layer& ly = layers[l];
        if (!ly.weights || !ly.k_cache || !ly.v_cache) return FASTVAR_EINVAL;
        if ((capture || !structure) && !ly.cache_map) return FASTVAR_EINVAL;
        const void* src = l == 0 ? x : dst_of(l - 1);
        void* dst = dst_of(l);
        if (!aligned16(dst) || dst == x) return FASTVAR_EINVAL;
        if (dense) {
            rc = check_block(src, N, nullptr, B, k, dims, ly.weights, ly.k_cache, ly.v_cache, L0, L_cap, dst, ws_blk,
                             blk_bytes);
        } else {
            rc = check_select(src, B, h, w, D, k, idx_out, ws_sel, sel_bytes);
            if (!rc)
                rc = check_block(src, N, idx_out, B, k, dims, ly.weights, ly.k_cache, ly.v_cache, L0, L_cap, yk,
                                 ws_blk, blk_bytes);
            if (!rc) rc = check_restore(yk, idx_out, rank, B, k, ly.cache_map, hc, wc, h, w, D, dst, nullptr, 0);
        }
        if (rc) return rc;
    }

    hipStream_t st = static_cast<hipStream_t>(stream);
    const fv::SelectPlan sp = fv::select_plan(B, N, D);
    zero_splitk_counters(ws_blk, dims, B, k, st);
    for (int l = 0; l < n_layers; ++l) {
        const fastvar_layer& ly = layers[l];
        const void* src = l == 0 ? x : dst_of(l - 1);
        void* dst = dst_of(l);
        if (dense) {
            enqueue_block(src, N, nullptr, B, k, dims, ly.weights, ly.k_cache, ly.v_cache, L0, L_cap, dst, ws_blk, st);
        } else {
            fv::launch_select(src, B, N, D, k, idx_out, rank, nullptr, ws_sel, sp, st);
            mark(st, FASTVAR_STAGE_SELECT);
            // restoration rides in the block's first launch (pruned rows) and its last (kept rows)
            const Fill fill{rank, ly.cache_map, hc, wc, h, w, dst};
            if (k > 0) {
                enqueue_block(src, N, idx_out, B, k, dims, ly.weights, ly.k_cache, ly.v_cache, L0, L_cap, dst, ws_blk,
                              st, true, &fill);
            } else {
                fv::launch_restore(nullptr, rank, B, k, ly.cache_map, hc, wc, h, w, D, dst, st);
                mark(st, FASTVAR_STAGE_RESTORE);
            }
        }
    }
    if (capture &&
        hipMemcpyAsync(y_out, layers[n_layers - 1].cache_map, (size_t)B * N * D * 2, hipMemcpyDeviceToDevice, st) !=
            hipSuccess)
        return FASTVAR_EHIP;
    rc = launch_status();
    if (rc == FASTVAR_OK) *kv_len = L0 + k;
    return rc;
}

int fastvar_scale_step_timed(const void* x, const int32_t* sched_h, const int32_t* sched_w, int K, int step,
                             int cache_step, int B, int k, const fastvar_dims* dims, const fastvar_layer* layers,
                             int n_layers, int32_t* kv_len, int L_cap, void* y_out, void* tmp, int32_t* idx_out,
                             void* ws, size_t ws_bytes, void* stream, float* stage_ms) {
    if (!stage_ms || n_layers <= 0 || n_layers > 256) return FASTVAR_EINVAL;
    hipStream_t st = static_cast<hipStream_t>(stream);
    StepProfile* prof = new StepProfile;
    const int want = 1 + FASTVAR_N_STAGES * n_layers;
    int made = 0;
    for (; made < want; ++made)
        if (hipEventCreate(&prof->ev[made]) != hipSuccess) break;
    int rc = made == want ? FASTVAR_OK : FASTVAR_EHIP;
    if (rc == FASTVAR_OK) {
        g_profile = prof;
        mark(st, -1);   // start of the step
        rc = fastvar_scale_step(x, sched_h, sched_w, K, step, cache_step, B, k, dims, layers, n_layers, kv_len, L_cap,
                                y_out, tmp, idx_out, ws, ws_bytes, stream);
        g_profile = nullptr;
        if (rc == FASTVAR_OK && hipStreamSynchronize(st) != hipSuccess) rc = FASTVAR_EHIP;
    }
    if (rc == FASTVAR_OK) {
        for (int i = 0; i < FASTVAR_N_STAGES; ++i) stage_ms[i] = 0.f;
        for (int i = 1; i < prof->n; ++i) {
            float ms = 0.f;
            if (hipEventElapsedTime(&ms, prof->ev[i - 1], prof->ev[i]) != hipSuccess) { rc = FASTVAR_EHIP; break; }
            stage_ms[prof->stage[i]] += ms / (float)n_layers;
        }
    }
    for (int i = 0; i < made; ++i) (void)hipEventDestroy(prof->ev[i]);
    delete prof;
    return rc;
}

size_t fastvar_step_sublayer_workspace_bytes(const fastvar_dims* dims, int B, int N, int k_attn, int k_ffn) {
    if (!dims || B <= 0 || N <= 0) return 0;
    // the block scratch is laid out per kept count and its size is not monotone in it (the split plans of
    // the GEMMs and of the attention change with the row count): the larger of the two layouts
    const size_t blk_a = fastvar_block_workspace_bytes(dims, B, k_attn);
    const size_t blk_f = fastvar_block_workspace_bytes(dims, B, k_ffn);
    return fastvar_select_workspace_bytes(B, N, dims->D) + fastvar_restore_workspace_bytes(B, N) +
           (blk_a > blk_f ? blk_a : blk_f);
}

int fastvar_attn_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* dims,
                                const fastvar_block_weights* weights, void* k_cache, void* v_cache, int L0,
                                int L_cap, void* h_kept_out, void* ws, size_t ws_bytes, void* stream) {
    const int rc = check_block(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, h_kept_out, ws,
                               ws_bytes);
    if (rc) return rc;
    if (k == 0) return FASTVAR_OK;
    zero_splitk_counters(ws, dims, B, k, static_cast<hipStream_t>(stream));
    enqueue_attn(x, N, idx, B, k, dims, weights, k_cache, v_cache, L0, L_cap, h_kept_out, ws,
                 static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_ffn_forward_pruned(const void* x, int N, const int32_t* idx, int B, int k, const fastvar_dims* dims,
                               const fastvar_block_weights* weights, void* y_kept_out, void* ws, size_t ws_bytes,
                               void* stream) {
    const int rc = check_ffn(x, N, idx, B, k, dims, weights, y_kept_out, ws, ws_bytes);
    if (rc) return rc;
    if (k == 0) return FASTVAR_OK;
    zero_splitk_counters(ws, dims, B, k, static_cast<hipStream_t>(stream));
    enqueue_ffn(x, N, idx, B, k, dims, weights, y_kept_out, ws, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_step_sublayer(const void* x, const int32_t* sched_h, const int32_t* sched_w, int K, int step,
                          int cache_step, int B, int k_attn, int k_ffn, const fastvar_dims* dims,
                          const fastvar_block_weights* weights, void* k_cache, void* v_cache, int32_t* kv_len,
                          int L_cap, const void* cache_map_attn, const void* cache_map_ffn, void* x_mid,
                          void* y_out, int32_t* idx_attn_out, int32_t* idx_ffn_out, void* ws, size_t ws_bytes,
                          void* stream) {
    if (!sched_h || !sched_w || !kv_len || K <= 0) return FASTVAR_EINVAL;
    if (step < 0 || step >= K || cache_step < 0 || cache_step >= step) return FASTVAR_EINVAL;
    const int h = sched_h[step], w = sched_w[step];
    const int hc = sched_h[cache_step], wc = sched_w[cache_step];
    if (h <= 0 || w <= 0 || hc <= 0 || wc <= 0 || (long)h * w > FASTVAR_MAX_TOKENS) return FASTVAR_EINVAL;
    const int N = h * w;
    const int L0 = *kv_len;
    int rc = check_dims(dims);
    if (rc) return rc;
    const int D = dims->D;
    if (B <= 0 || k_attn < 0 || k_attn > N || k_ffn < 0 || k_ffn > N) return FASTVAR_EINVAL;
    if (!x_mid || x_mid == x || y_out == x || y_out == x_mid) return FASTVAR_EINVAL;
    if (!ws) return FASTVAR_EWORKSPACE;
    if (!aligned16(ws)) return FASTVAR_EALIGN;
    if (ws_bytes < fastvar_step_sublayer_workspace_bytes(dims, B, N, k_attn, k_ffn)) return FASTVAR_EWORKSPACE;

    // scratch: [selection | rank [B,N] | block buffers for max(k_attn, k_ffn)]
    const size_t sel_bytes = fastvar_select_workspace_bytes(B, N, D);
    const size_t rank_bytes = fastvar_restore_workspace_bytes(B, N);
    char* base = static_cast<char*>(ws);
    void* ws_sel = base;
    int32_t* rank = reinterpret_cast<int32_t*>(base + sel_bytes);
    char* ws_blk = base + sel_bytes + rank_bytes;
    const size_t blk_bytes = ws_bytes - sel_bytes - rank_bytes;
    // Kept outputs of either half go to the h1 buffer of its own plan (neither half uses it).
    void* hk = k_attn > 0 ? static_cast<void*>(ws_blk + block_plan(dims, B, k_attn).off_h1) : nullptr;
    void* yk = k_ffn > 0 ? static_cast<void*>(ws_blk + block_plan(dims, B, k_ffn).off_h1) : nullptr;

    rc = check_select(x, B, h, w, D, k_attn, idx_attn_out, ws_sel, sel_bytes);
    if (rc) return rc;
    rc = check_block(x, N, idx_attn_out, B, k_attn, dims, weights, k_cache, v_cache, L0, L_cap, hk, ws_blk,
                     blk_bytes);
    if (rc) return rc;
    rc = check_restore(hk, idx_attn_out, rank, B, k_attn, cache_map_attn, hc, wc, h, w, D, x_mid, nullptr, 0);
    if (rc) return rc;
    rc = check_select(x_mid, B, h, w, D, k_ffn, idx_ffn_out, ws_sel, sel_bytes);
    if (rc) return rc;
    rc = check_ffn(x_mid, N, idx_ffn_out, B, k_ffn, dims, weights, yk, ws_blk, blk_bytes);
    if (rc) return rc;
    rc = check_restore(yk, idx_ffn_out, rank, B, k_ffn, cache_map_ffn, hc, wc, h, w, D, y_out, nullptr, 0);
    if (rc) return rc;

    hipStream_t st = static_cast<hipStream_t>(stream);
    const fv::SelectPlan sp = fv::select_plan(B, N, D);
    zero_splitk_counters(ws_blk, dims, B, k_attn, st);
    fv::launch_select(x, B, N, D, k_attn, idx_attn_out, rank, nullptr, ws_sel, sp, st);
    // each half's restoration rides in its own gather launch (pruned rows) and last GEMM (kept rows)
    const Fill fill_a{rank, cache_map_attn, hc, wc, h, w, x_mid};
    if (k_attn > 0)
        enqueue_attn(x, N, idx_attn_out, B, k_attn, dims, weights, k_cache, v_cache, L0, L_cap, x_mid, ws_blk, st, true,
                     &fill_a);
    else
        fv::launch_restore(nullptr, rank, B, k_attn, cache_map_attn, hc, wc, h, w, D, x_mid, st);
    fv::launch_select(x_mid, B, N, D, k_ffn, idx_ffn_out, rank, nullptr, ws_sel, sp, st);
    zero_splitk_counters(ws_blk, dims, B, k_ffn, st);   // the two halves lay the scratch out for their own k
    const Fill fill_f{rank, cache_map_ffn, hc, wc, h, w, y_out};
    if (k_ffn > 0)
        enqueue_ffn(x_mid, N, idx_ffn_out, B, k_ffn, dims, weights, y_out, ws_blk, st, true, &fill_f);
    else
        fv::launch_restore(nullptr, rank, B, k_ffn, cache_map_ffn, hc, wc, h, w, D, y_out, st);
    rc = launch_status();
    if (rc == FASTVAR_OK) *kv_len = L0 + k_attn;
    return rc;
}

int fastvar_layernorm(const void* in, const int32_t* idx, int B, int N, int k, int D, const void* gamma,
                      const void* beta, float eps, void* out, void* stream) {
    if (!in || !gamma || !beta || !out || B <= 0 || k <= 0 || D <= 0 || !(eps >= 0.f)) return FASTVAR_EINVAL;
    if (idx && N <= 0) return FASTVAR_EINVAL;
    if (D > kMaxWidth) return FASTVAR_ECAPACITY;
    if (D % 8 != 0 || !aligned16(in) || !aligned16(gamma) || !aligned16(beta) || !aligned16(out))
        return FASTVAR_EALIGN;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (idx)
        fv::launch_gather_layernorm(in, idx, B, N, k, D, gamma, beta, eps, nullptr, out, st);
    else
        fv::launch_layernorm(in, B * k, D, gamma, beta, eps, out, st);
    return launch_status();
}

int fastvar_gemm_bf16(const void* A, const void* W, const void* bias, const void* residual, int M, int N, int K,
                      int epilogue, void* out, void* stream) {
    if (!A || !W || !out || M <= 0 || N <= 0 || K <= 0) return FASTVAR_EINVAL;
    if (epilogue != fv::EPI_BIAS_RES && epilogue != fv::EPI_BIAS_GELU) return FASTVAR_EINVAL;
    if (epilogue == fv::EPI_BIAS_RES && !residual) return FASTVAR_EINVAL;
    if (K % 64 != 0 || N % 8 != 0 || !aligned16(A) || !aligned16(W) || !aligned16(out) ||
        (bias && !aligned16(bias)) || (residual && !aligned16(residual)))
        return FASTVAR_EALIGN;
    if ((double)M * K >= 2147483648.0 || (double)N * K >= 2147483648.0 || (double)M * N >= 2147483648.0)
        return FASTVAR_ECAPACITY;
    fv::GemmArgs g{};
    g.A = A; g.W = W; g.bias = bias; g.M = M; g.N = N; g.K = K;
    g.out = out; g.residual = residual; g.k_tokens = M;
    fv::launch_gemm(static_cast<fv::GemmEpilogue>(epilogue), g, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_qkv_gemm(const void* a, const void* w_qkv, const void* b_qkv, int B, int k, const fastvar_dims* dims,
                     void* q_out, void* k_cache, void* v_cache, int L0, int L_cap, void* stream) {
    const int rc = check_dims(dims);
    if (rc) return rc;
    if (!a || !w_qkv || !q_out || !k_cache || !v_cache || B <= 0 || k <= 0 || L0 < 0 || L_cap <= 0)
        return FASTVAR_EINVAL;
    if ((long)L0 + k > L_cap) return FASTVAR_ECAPACITY;
    if (L_cap % 8 != 0 || !aligned16(a) || !aligned16(w_qkv) || !aligned16(q_out) || !aligned16(k_cache) ||
        !aligned16(v_cache) || (b_qkv && !aligned16(b_qkv)))
        return FASTVAR_EALIGN;
    if ((double)B * k * 3.0 * dims->D >= 2147483648.0) return FASTVAR_ECAPACITY;
    fv::GemmArgs g{};
    g.A = a; g.W = w_qkv; g.bias = b_qkv; g.M = B * k; g.N = 3 * dims->D; g.K = dims->D;
    g.q_out = q_out; g.k_cache = k_cache; g.v_cache = v_cache;
    g.D = dims->D; g.H = dims->H; g.dh = dims->dh; g.k_tokens = k; g.L0 = L0; g.L_cap = L_cap;
    fv::launch_gemm(fv::EPI_QKV, g, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_qkv_gemm_rope(const void* a, const void* w_qkv, const void* b_qkv, const int32_t* idx, int B, int N,
                          int k, const fastvar_dims* dims, const float* rope_cos, const float* rope_sin, void* q_out,
                          void* k_cache, void* v_cache, int L0, int L_cap, void* stream) {
    const int rc = check_dims(dims);
    if (rc) return rc;
    if (!a || !w_qkv || !q_out || !k_cache || !v_cache || !rope_cos || !rope_sin || B <= 0 || N <= 0 || k <= 0 ||
        k > N || L0 < 0 || L_cap <= 0 || (!idx && k != N))
        return FASTVAR_EINVAL;
    if ((long)L0 + k > L_cap) return FASTVAR_ECAPACITY;
    if (L_cap % 8 != 0 || !aligned16(a) || !aligned16(w_qkv) || !aligned16(q_out) || !aligned16(k_cache) ||
        !aligned16(v_cache) || (b_qkv && !aligned16(b_qkv)) || !aligned16(rope_cos) || !aligned16(rope_sin))
        return FASTVAR_EALIGN;
    if ((double)B * k * 3.0 * dims->D >= 2147483648.0) return FASTVAR_ECAPACITY;
    fv::GemmArgs g{};
    g.A = a; g.W = w_qkv; g.bias = b_qkv; g.M = B * k; g.N = 3 * dims->D; g.K = dims->D;
    g.q_out = q_out; g.k_cache = k_cache; g.v_cache = v_cache;
    g.D = dims->D; g.H = dims->H; g.dh = dims->dh; g.k_tokens = k; g.L0 = L0; g.L_cap = L_cap;
    g.rope_cos = rope_cos; g.rope_sin = rope_sin; g.rope_rows = idx; g.rope_N = N;
    fv::launch_gemm(fv::EPI_QKV, g, static_cast<hipStream_t>(stream));
    return launch_status();
}

int fastvar_attention(const void* q, const void* k_cache, const void* v_cache, int B, int k,
                      const fastvar_dims* dims, int L, int L_cap, void* o, void* stream) {
    const int rc = check_dims(dims);
    if (rc) return rc;
    if (!q || !k_cache || !v_cache || !o || B <= 0 || k <= 0 || L <= 0 || L_cap <= 0) return FASTVAR_EINVAL;
    if (L > L_cap) return FASTVAR_ECAPACITY;
    if (L_cap % 8 != 0 || !aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(o))
        return FASTVAR_EALIGN;
    fv::AttnArgs at{};
    at.q = q; at.k_cache = k_cache; at.v_cache = v_cache; at.o = o;
    at.B = B; at.H = dims->H; at.dh = dims->dh; at.k_tokens = k; at.L = L; at.L_cap = L_cap;
    at.scale = dims->softmax_scale;
    fv::launch_attention(at, static_cast<hipStream_t>(stream));
    return launch_status();
}

}  // extern "C"
