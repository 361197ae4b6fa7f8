// bf16 MFMA GEMM for the block's four dense contractions (QKV, out-proj, FC1,
// FC2):  C[m,n] = sum_k A[m,k] * W[n,k]  with A [M,K] and W [N,K] both
// K-contiguous (activations are row-major, weights are [out, in]).
//
// Tiling for gfx950: a workgroup of 4 waves owns a BM x BN tile of C; each wave
// owns a (BM/2) x (BN/2) sub-tile built from 32x32x16 bf16 MFMAs with fp32
// accumulators.  K is walked in steps of 64: both operand tiles are copied to
// LDS (double buffered; the next tile's global loads are in flight while the
// current one is multiplied) in rows of 128 bytes whose 16-byte chunks are
// XOR-swizzled with the row index, so the MFMA operand reads (one 16-byte
// ds_read per lane, 32 consecutive rows per half-wave) are conflict free.
//
// Epilogues are fused: bias, residual add, exact GELU, and for the QKV GEMM
// the split into the query buffer and the append into the K / V caches
// (V transposed so that cache positions are contiguous).
#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

constexpr int BK = 64;  // K step; one LDS row = 64 bf16 = 8 chunks of 16 bytes

// Exact-form GELU, v * Phi(v), with erf from the rational approximation of
// Abramowitz & Stegun 7.1.26 (absolute error below 1.5e-7, far under bf16
// resolution); branch free so that the unrolled epilogue stays small.
__device__ __forceinline__ float gelu_erf(float v) {
    const float z = fabsf(v) * 0.70710678118654752440f;
    const float t = __builtin_amdgcn_rcpf(fmaf(0.3275911f, z, 1.0f));
    float poly = fmaf(1.061405429f, t, -1.453152027f);
    poly = fmaf(poly, t, 1.421413741f);
    poly = fmaf(poly, t, -0.284496736f);
    poly = fmaf(poly, t, 0.254829592f);
    const float e = __builtin_amdgcn_exp2f(-z * z * 1.4426950408889634f);
    const float erf_abs = 1.0f - poly * t * e;  // erf(|v|/sqrt2)
    const float erf_v = copysignf(erf_abs, v);
    return 0.5f * v * (1.0f + erf_v);
}

struct GemmParams {
    const bf16_t* A;
    const bf16_t* W;
    const bf16_t* bias;
    int M, N, K;
    bf16_t* out;
    const bf16_t* residual;
    const int32_t* res_idx;  // optional row gather for the residual: row = (m / k_tokens) * res_N + res_idx[m]
    int res_N;
    bf16_t* q_out;
    bf16_t* k_cache;
    bf16_t* v_cache;
    int D, H, dh, k_tokens, L0, L_cap;
    int tiles_m, tiles_n;
};

// Where one output column lands: element address = ptr + b*batch_stride + t*row_stride
// for row m = b*k_tokens + t (for plain [M,N] outputs batch_stride = k_tokens*row_stride).
struct ColDest {
    bf16_t* ptr;
    long batch_stride;
    int row_stride;
};

template <int EPI>
__device__ __forceinline__ ColDest col_dest(const GemmParams& p, int n) {
    ColDest c;
    if (EPI != EPI_QKV) {
        c.ptr = p.out + n;
        c.row_stride = p.N;
        c.batch_stride = (long)p.k_tokens * p.N;
        return c;
    }
    const int sec = n / p.D;
    const int f = n - sec * p.D;
    const int hh = f / p.dh;
    const int d = f - hh * p.dh;
    if (sec == 0) {
        c.ptr = p.q_out + f;
        c.row_stride = p.D;
        c.batch_stride = (long)p.k_tokens * p.D;
    } else if (sec == 1) {  // k_cache [B, H, L_cap, dh]
        c.ptr = p.k_cache + ((size_t)hh * p.L_cap + p.L0) * p.dh + d;
        c.row_stride = p.dh;
        c.batch_stride = (long)p.H * p.L_cap * p.dh;
    } else {  // v_cache [B, H, dh, L_cap]
        c.ptr = p.v_cache + ((size_t)hh * p.dh + d) * p.L_cap + p.L0;
        c.row_stride = 1;
        c.batch_stride = (long)p.H * p.dh * p.L_cap;
    }
    return c;
}

template <int BM, int BN, int EPI>
__global__ __launch_bounds__(256) void gemm_nt_kernel(const GemmParams p) {
    constexpr int T = 256;
    constexpr int WTM = BM / 2, WTN = BN / 2;  // wave tile (2 x 2 waves)
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int A_CH = BM * 8 / T, W_CH = BN * 8 / T;  // 16-byte chunks per thread per tile

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t* sA = reinterpret_cast<u32x4_t*>(smem);  // [2][BM*8]
    u32x4_t* sW = sA + 2 * BM * 8;                   // [2][BN*8]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;

    // Tile id: consecutive workgroup ids are dealt round-robin to the 8 XCDs;
    // undo that so each XCD (own L2) walks a contiguous run of tiles, and walk
    // tiles in groups of 8 tile-rows so neighbours share operand rows.
    int pid = blockIdx.x;
    const int n_tiles = p.tiles_m * p.tiles_n;
    if ((n_tiles & 7) == 0) pid = (pid & 7) * (n_tiles >> 3) + (pid >> 3);
    constexpr int GROUP = 8;
    const int per_group = GROUP * p.tiles_n;
    const int grp = pid / per_group;
    const int first_m = grp * GROUP;
    const int gsize = min(p.tiles_m - first_m, GROUP);
    const int in_grp = pid - grp * per_group;
    const int tm = first_m + in_grp % gsize;
    const int tn = in_grp / gsize;
    const int m0 = tm * BM, n0 = tn * BN;

    // per-thread load slots: chunk column c is fixed, rows step by 32
    const int c = tid & 7;
    const int r_base = tid >> 3;
    const int lds_slot = r_base * 8 + (c ^ (r_base & 7));
    int a_off[A_CH], w_off[W_CH];
#pragma unroll
    for (int i = 0; i < A_CH; ++i) a_off[i] = min(m0 + r_base + 32 * i, p.M - 1) * p.K + c * 8;
#pragma unroll
    for (int i = 0; i < W_CH; ++i) w_off[i] = min(n0 + r_base + 32 * i, p.N - 1) * p.K + c * 8;

    f32x16_t acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = 0.f;

    u32x4_t ra[A_CH], rw[W_CH];
    const int KT = p.K / BK;

#define FV_LOAD_GLOBAL(kt_)                                                      \
    {                                                                            \
        const int k0_ = (kt_) * BK;                                              \
        _Pragma("unroll") for (int i = 0; i < A_CH; ++i)                         \
            ra[i] = *reinterpret_cast<const u32x4_t*>(p.A + a_off[i] + k0_);     \
        _Pragma("unroll") for (int i = 0; i < W_CH; ++i)                         \
            rw[i] = *reinterpret_cast<const u32x4_t*>(p.W + w_off[i] + k0_);     \
    }
#define FV_STORE_LDS(buf_)                                                       \
    {                                                                            \
        u32x4_t* da_ = sA + (buf_) * BM * 8 + lds_slot;                          \
        u32x4_t* dw_ = sW + (buf_) * BN * 8 + lds_slot;                          \
        _Pragma("unroll") for (int i = 0; i < A_CH; ++i) da_[i * 256] = ra[i];   \
        _Pragma("unroll") for (int i = 0; i < W_CH; ++i) dw_[i * 256] = rw[i];   \
    }

    FV_LOAD_GLOBAL(0)
    FV_STORE_LDS(0)
    __syncthreads();

    const int frag_row = lane & 31;
    const int frag_half = lane >> 5;
    const int frag_sw = lane & 7;

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) FV_LOAD_GLOBAL(kt + 1)

        const u32x4_t* a_base = sA + buf * BM * 8 + (wm * WTM + frag_row) * 8;
        const u32x4_t* w_base = sW + buf * BN * 8 + (wn * WTN + frag_row) * 8;
#pragma unroll
        for (int kk = 0; kk < BK / 16; ++kk) {
            const int ch = (2 * kk + frag_half) ^ frag_sw;
            bf16x8_t af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[mi] = *reinterpret_cast<const bf16x8_t*>(a_base + mi * 32 * 8 + ch);
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
                bfr[ni] = *reinterpret_cast<const bf16x8_t*>(w_base + ni * 32 * 8 + ch);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
                    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[mi], bfr[ni], acc[mi][ni], 0, 0, 0);
        }

        if (kt + 1 < KT) FV_STORE_LDS(buf ^ 1)
        __syncthreads();
    }
#undef FV_LOAD_GLOBAL
#undef FV_STORE_LDS

    // Epilogue.  Accumulator register r of lane l holds C[row, col] with
    // col = l % 32 and row = 8*(r/4) + 4*(l/32) + r%4 inside the 32x32 block.
    ColDest cd[NI];
    float bias[NI];
    bool n_ok[NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int n = n0 + wn * WTN + ni * 32 + frag_row;
        n_ok[ni] = n < p.N;
        const int nc = n_ok[ni] ? n : 0;
        cd[ni] = col_dest<EPI>(p, nc);
        bias[ni] = p.bias ? bf16_to_f32(p.bias[nc]) : 0.f;
    }
    static_for<0, MI>([&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
        static_for<0, 16>([&](auto r_c) {
            constexpr int r = decltype(r_c)::value;
            const int m = m0 + wm * WTM + mi * 32 + 8 * (r >> 2) + 4 * frag_half + (r & 3);
            if (m < p.M) {
                const int b = m / p.k_tokens;
                const int t = m - b * p.k_tokens;
                const bf16_t* res_row = nullptr;
                if (EPI == EPI_BIAS_RES) {
                    const size_t rrow = p.res_idx ? (size_t)b * p.res_N + p.res_idx[m] : (size_t)m;
                    res_row = p.residual + rrow * p.N + (n0 + wn * WTN + frag_row);
                }
                static_for<0, NI>([&](auto ni_c) {
                    constexpr int ni = decltype(ni_c)::value;
                    if (n_ok[ni]) {
                        float v = acc[mi][ni][r] + bias[ni];
                        if (EPI == EPI_BIAS_GELU) v = gelu_erf(v);
                        if (EPI == EPI_BIAS_RES) v += bf16_to_f32(res_row[ni * 32]);
                        cd[ni].ptr[(long)b * cd[ni].batch_stride + (long)t * cd[ni].row_stride] =
                            (bf16_t)f32_to_bf16_bits(v);
                    }
                });
            }
        });
    });
}

template <int BM, int BN>
constexpr size_t smem_bytes() {
    return (size_t)2 * (BM + BN) * BK * sizeof(bf16_t);
}

template <int BM, int BN, int EPI>
void launch_cfg(GemmParams& p, hipStream_t stream) {
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    static bool attr_set = false;  // raising the dynamic-LDS limit is per function, once per process
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&gemm_nt_kernel<BM, BN, EPI>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem_bytes<BM, BN>());
        attr_set = true;
    }
    gemm_nt_kernel<BM, BN, EPI><<<dim3(p.tiles_m * p.tiles_n), 256, smem_bytes<BM, BN>(), stream>>>(p);
}

template <int EPI>
void launch_epi(GemmParams& p, hipStream_t stream) {
    // Large tiles only when they still give every CU at least one tile.
    const long big_tiles = (long)((p.M + 255) / 256) * ((p.N + 255) / 256);
    if (big_tiles >= 224)
        launch_cfg<256, 256, EPI>(p, stream);
    else
        launch_cfg<128, 128, EPI>(p, stream);
}

}  // namespace

void launch_gemm(GemmEpilogue epi, const GemmArgs& a, hipStream_t stream) {
    GemmParams p;
    p.A = static_cast<const bf16_t*>(a.A);
    p.W = static_cast<const bf16_t*>(a.W);
    p.bias = static_cast<const bf16_t*>(a.bias);
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.out = static_cast<bf16_t*>(a.out);
    p.residual = static_cast<const bf16_t*>(a.residual);
    p.res_idx = a.res_idx;
    p.res_N = a.res_N;
    p.q_out = static_cast<bf16_t*>(a.q_out);
    p.k_cache = static_cast<bf16_t*>(a.k_cache);
    p.v_cache = static_cast<bf16_t*>(a.v_cache);
    p.D = a.D; p.H = a.H; p.dh = a.dh; p.k_tokens = a.k_tokens; p.L0 = a.L0; p.L_cap = a.L_cap;
    p.tiles_m = p.tiles_n = 0;
    switch (epi) {
        case EPI_QKV: launch_epi<EPI_QKV>(p, stream); break;
        case EPI_BIAS_RES: launch_epi<EPI_BIAS_RES>(p, stream); break;
        case EPI_BIAS_GELU: launch_epi<EPI_BIAS_GELU>(p, stream); break;
    }
}

}  // namespace fv
