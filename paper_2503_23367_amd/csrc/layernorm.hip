// Gather of the kept tokens fused with the block's first LayerNorm, and the
// plain LayerNorm before the MLP.  One wave per token row; the row is held in
// registers (two-pass mean / biased variance in fp32); 16-byte loads and stores.
// HBM bound: reads k*D bf16, writes k*D bf16.
// The gather launch can also carry the restoration's fill (Sec. 3.3, Eq. 6): the pruned slots of the
// restored map depend only on the selection and on the cached map, not on the block's output, so extra
// workgroups of the same launch write them while the first ones normalise the kept rows.
#include "common.h"
#include "kernels.h"
#include "resample.h"

namespace fv {

namespace {

__device__ __forceinline__ void unpack8(const uint4& v, float (&f)[8]) {
    f[0] = bf16_lo(v.x); f[1] = bf16_hi(v.x);
    f[2] = bf16_lo(v.y); f[3] = bf16_hi(v.y);
    f[4] = bf16_lo(v.z); f[5] = bf16_hi(v.z);
    f[6] = bf16_lo(v.w); f[7] = bf16_hi(v.w);
}

// CH = number of 512-column groups held in registers (D <= 512*CH).
// Row m of the output reads input row (idx ? b*N + idx[m] : m), b = m / k; that
// row index is also written to rows_out[m] when asked for.
template <int CH>
__device__ __forceinline__ void layernorm_row(const bf16_t* __restrict__ in, const int32_t* __restrict__ idx, int N,
                                              int k, int M, int D, const bf16_t* __restrict__ gamma,
                                              const bf16_t* __restrict__ beta, float eps,
                                              int32_t* __restrict__ rows_out, bf16_t* __restrict__ out, int m) {
    const int lane = threadIdx.x & 63;
    if (m >= M) return;
    size_t src_row = (size_t)m;
    if (idx) src_row = (size_t)(m / k) * N + idx[m];
    if (rows_out && lane == 0) rows_out[m] = (int32_t)src_row;
    const bf16_t* src = in + src_row * D;

    // All of the row's loads and the gain / shift loads go out together: one memory
    // latency instead of two in a kernel that has little else to hide it with.
    uint4 raw[CH], graw[CH], braw[CH];
#pragma unroll
    for (int g = 0; g < CH; ++g) {
        const int col = g * 512 + lane * 8;
        if (col < D) {
            raw[g] = *reinterpret_cast<const uint4*>(src + col);
            graw[g] = *reinterpret_cast<const uint4*>(gamma + col);
            braw[g] = *reinterpret_cast<const uint4*>(beta + col);
        }
    }
    float v[CH][8];
    float sum = 0.f;
#pragma unroll
    for (int g = 0; g < CH; ++g) {
        const int col = g * 512 + lane * 8;
        if (col < D) {
            unpack8(raw[g], v[g]);
#pragma unroll
            for (int j = 0; j < 8; ++j) sum += v[g][j];
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) v[g][j] = 0.f;
        }
    }
    const float mean = wave_sum(sum) / (float)D;
    float sq = 0.f;
#pragma unroll
    for (int g = 0; g < CH; ++g) {
        const int col = g * 512 + lane * 8;
        if (col < D) {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const float d = v[g][j] - mean;
                sq = fmaf(d, d, sq);
            }
        }
    }
    const float rstd = 1.0f / sqrtf(wave_sum(sq) / (float)D + eps);
#pragma unroll
    for (int g = 0; g < CH; ++g) {
        const int col = g * 512 + lane * 8;
        if (col < D) {
            float gm[8], bt[8];
            unpack8(graw[g], gm);
            unpack8(braw[g], bt);
            float o[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) o[j] = (v[g][j] - mean) * rstd * gm[j] + bt[j];
            uint4 pk;
            pk.x = pack_bf16x2(o[0], o[1]);
            pk.y = pack_bf16x2(o[2], o[3]);
            pk.z = pack_bf16x2(o[4], o[5]);
            pk.w = pack_bf16x2(o[6], o[7]);
            *reinterpret_cast<uint4*>(out + (size_t)m * D + col) = pk;
        }
    }
}

template <int CH>
__global__ __launch_bounds__(256) void layernorm_rows_kernel(const bf16_t* __restrict__ in,
                                                             const int32_t* __restrict__ idx, int N, int k,
                                                             int M, int D, const bf16_t* __restrict__ gamma,
                                                             const bf16_t* __restrict__ beta, float eps,
                                                             int32_t* __restrict__ rows_out,
                                                             bf16_t* __restrict__ out) {
    layernorm_row<CH>(in, idx, N, k, M, D, gamma, beta, eps, rows_out, out, blockIdx.x * 4 + (threadIdx.x >> 6));
}

// The same launch with the restoration's fill behind it: workgroups [0, ln_blocks) normalise the kept rows,
// the others walk the token rows of the restored map (eight per workgroup, two per wave) and write the
// pruned ones (rank < 0) from the cached map; kept rows are left to the block's last GEMM.
struct FillParams {
    const int32_t* rank;      // [B, N]
    const bf16_t* cache_map;  // [B, hc*wc, D]
    bf16_t* y_out;            // [B, N, D]
    int hc, wc, h, w;
    int blocks_per_sample;
};
constexpr int kFillRowsPerWave = 1;

template <int CH>
__global__ __launch_bounds__(256) void gather_layernorm_fill_kernel(const bf16_t* __restrict__ in,
                                                                    const int32_t* __restrict__ idx, int N, int k,
                                                                    int M, int D, const bf16_t* __restrict__ gamma,
                                                                    const bf16_t* __restrict__ beta, float eps,
                                                                    int32_t* __restrict__ rows_out,
                                                                    bf16_t* __restrict__ out, int ln_blocks,
                                                                    const FillParams f) {
    if ((int)blockIdx.x < ln_blocks) {
        layernorm_row<CH>(in, idx, N, k, M, D, gamma, beta, eps, rows_out, out, blockIdx.x * 4 + (threadIdx.x >> 6));
        return;
    }
    const int fb = blockIdx.x - ln_blocks;
    const int b = fb / f.blocks_per_sample;
    const int blk = fb - b * f.blocks_per_sample;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
    for (int rr = 0; rr < kFillRowsPerWave; ++rr) {
        const int n = (blk * 4 + wave) * kFillRowsPerWave + rr;
        if (n >= N) break;
        if (f.rank[(size_t)b * N + n] >= 0) continue;
        fill_pruned_row_any(f.cache_map + (size_t)b * f.hc * f.wc * D, f.hc, f.wc, f.h, f.w, D, n, lane,
                        f.y_out + ((size_t)b * N + n) * D);
    }
}

void dispatch(const void* in, const int32_t* idx, int N, int k, int M, int D, const void* gamma,
              const void* beta, float eps, int32_t* rows_out, void* out, hipStream_t stream) {
    const dim3 grid((M + 3) / 4), block(256);
    const int ch = (D + 511) / 512;
#define FV_LN_CASE(CHV)                                                                                  \
    layernorm_rows_kernel<CHV><<<grid, block, 0, stream>>>(                                              \
        static_cast<const bf16_t*>(in), idx, N, k, M, D, static_cast<const bf16_t*>(gamma),              \
        static_cast<const bf16_t*>(beta), eps, rows_out, static_cast<bf16_t*>(out))
    if (ch <= 1) FV_LN_CASE(1);
    else if (ch <= 2) FV_LN_CASE(2);
    else if (ch <= 4) FV_LN_CASE(4);
    else if (ch <= 8) FV_LN_CASE(8);
    else FV_LN_CASE(16);  // D <= 8192, checked by the caller
#undef FV_LN_CASE
}

}  // namespace

void launch_gather_layernorm(const void* x, const int32_t* idx, int B, int N, int k, int D, const void* gamma,
                             const void* beta, float eps, int32_t* rows_out, void* a_out, hipStream_t stream) {
    dispatch(x, idx, N, k, B * k, D, gamma, beta, eps, rows_out, a_out, stream);
}

void launch_gather_layernorm_fill(const void* x, const int32_t* idx, int B, int N, int k, int D, const void* gamma,
                                  const void* beta, float eps, int32_t* rows_out, void* a_out, const int32_t* rank,
                                  const void* cache_map, int hc, int wc, int h, int w, void* y_out,
                                  hipStream_t stream) {
    const int M = B * k;
    const int ln_blocks = (M + 3) / 4;
    FillParams f;
    f.rank = rank;
    f.cache_map = static_cast<const bf16_t*>(cache_map);
    f.y_out = static_cast<bf16_t*>(y_out);
    f.hc = hc; f.wc = wc; f.h = h; f.w = w;
    f.blocks_per_sample = (N + 4 * kFillRowsPerWave - 1) / (4 * kFillRowsPerWave);
    const dim3 grid(ln_blocks + B * f.blocks_per_sample), block(256);
    const int ch = (D + 511) / 512;
#define FV_LNF_CASE(CHV)                                                                                 \
    gather_layernorm_fill_kernel<CHV><<<grid, block, 0, stream>>>(                                       \
        static_cast<const bf16_t*>(x), idx, N, k, M, D, static_cast<const bf16_t*>(gamma),               \
        static_cast<const bf16_t*>(beta), eps, rows_out, static_cast<bf16_t*>(a_out), ln_blocks, f)
    if (ch <= 1) FV_LNF_CASE(1);
    else if (ch <= 2) FV_LNF_CASE(2);
    else if (ch <= 4) FV_LNF_CASE(4);
    else if (ch <= 8) FV_LNF_CASE(8);
    else FV_LNF_CASE(16);
#undef FV_LNF_CASE
}

void launch_layernorm(const void* in, int M, int D, const void* gamma, const void* beta, float eps, void* a_out,
                      hipStream_t stream) {
    dispatch(in, nullptr, 0, 1, M, D, gamma, beta, eps, nullptr, a_out, stream);
}

}  // namespace fv
