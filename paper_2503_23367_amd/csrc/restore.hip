// Cached Token Restoration (FastVAR Sec. 3.3, Eq. 6 and the scatter that
// follows it): every slot of the restored map is either the kept token's block
// output (a row copy) or the cached previous-scale map resampled bilinearly at
// half-pixel centres.  One pass over the output, one wave per token row,
// 16-byte loads and stores; HBM bound (writes N*D bf16 once).
#include "common.h"
#include "kernels.h"
#include "resample.h"

namespace fv {

namespace {

// rank[b,n] = position of n in the ascending idx[b,:], or -1.  Binary search,
// so no ordering between a fill and a scatter is needed.
__global__ __launch_bounds__(256) void rank_from_idx_kernel(const int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ rank, int N, int k) {
    const int n = blockIdx.x * 256 + threadIdx.x;
    const int b = blockIdx.y;
    if (n >= N) return;
    const int32_t* row = idx + (size_t)b * k;
    int lo = 0, hi = k;  // first position with row[pos] >= n
    while (lo < hi) {
        const int mid = (lo + hi) >> 1;
        if (row[mid] < n) lo = mid + 1; else hi = mid;
    }
    rank[(size_t)b * N + n] = (lo < k && row[lo] == n) ? lo : -1;
}

constexpr int kRowsPerWave = 2;

// grid (ceil(N / (4*kRowsPerWave)), B), block 256.
__global__ __launch_bounds__(256) void restore_kernel(const bf16_t* __restrict__ y_kept,
                                                      const int32_t* __restrict__ rank, int k,
                                                      const bf16_t* __restrict__ cache_map, int hc, int wc,
                                                      int h, int w, int D, bf16_t* __restrict__ y_out) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int b = blockIdx.y;
    const int N = h * w;
    const int groups = (D + 511) >> 9;
#pragma unroll
    for (int rr = 0; rr < kRowsPerWave; ++rr) {
        const int n = (blockIdx.x * 4 + wave) * kRowsPerWave + rr;
        if (n >= N) break;
        const int r = (k > 0) ? rank[(size_t)b * N + n] : -1;
        bf16_t* dst = y_out + ((size_t)b * N + n) * D;
        if (r >= 0) {
            if (!y_kept) continue;   // the kept rows are already in place (written by the block's last GEMM)
            const bf16_t* src = y_kept + ((size_t)b * k + r) * D;
            for (int g = 0; g < groups; ++g) {
                const int col = g * 512 + lane * 8;
                if (col < D)
                    *reinterpret_cast<uint4*>(dst + col) = *reinterpret_cast<const uint4*>(src + col);
            }
        } else {
            fill_pruned_row_any(cache_map + (size_t)b * hc * wc * D, hc, wc, h, w, D, n, lane, dst);
        }
    }
}

// Intermediate prediction (Sec. 3.1, Eq. 2): r_k = interpolate(r_{k-1}, (h, w)) + f_k on fp32 maps of C
// channels.  One thread per four channels of one position; either term may be absent (first step: no
// previous map; skipped step: no residual).  HBM bound: reads 4 taps (neighbouring threads share them
// through the cache) and 8 bytes of residual, writes 16 bytes.
__global__ __launch_bounds__(256) void residual_accumulate_kernel(const float* __restrict__ r_prev, int hp, int wp,
                                                                  const bf16_t* __restrict__ f_k, int h, int w, int C,
                                                                  float* __restrict__ r_out, long total) {
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int c4 = C >> 2;
    const int c = (int)(i % c4) << 2;
    const long t = i / c4;
    const int N = h * w;
    const int n = (int)(t % N);
    const long b = t / N;
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (r_prev) {
        int i0, i1, j0, j1;
        float lr, lc;
        axis_taps(n / w, hp, h, i0, i1, lr);
        axis_taps(n % w, wp, w, j0, j1, lc);
        const float* pb = r_prev + (size_t)b * hp * wp * C + c;
        const float4 c00 = *reinterpret_cast<const float4*>(pb + ((size_t)i0 * wp + j0) * C);
        const float4 c01 = *reinterpret_cast<const float4*>(pb + ((size_t)i0 * wp + j1) * C);
        const float4 c10 = *reinterpret_cast<const float4*>(pb + ((size_t)i1 * wp + j0) * C);
        const float4 c11 = *reinterpret_cast<const float4*>(pb + ((size_t)i1 * wp + j1) * C);
        acc.x = lerp2(c00.x, c01.x, c10.x, c11.x, lr, lc);
        acc.y = lerp2(c00.y, c01.y, c10.y, c11.y, lr, lc);
        acc.z = lerp2(c00.z, c01.z, c10.z, c11.z, lr, lc);
        acc.w = lerp2(c00.w, c01.w, c10.w, c11.w, lr, lc);
    }
    if (f_k) {
        const uint2 v = *reinterpret_cast<const uint2*>(f_k + (size_t)t * C + c);
        acc.x += bf16_lo(v.x);
        acc.y += bf16_hi(v.x);
        acc.z += bf16_lo(v.y);
        acc.w += bf16_hi(v.y);
    }
    *reinterpret_cast<float4*>(r_out + (size_t)t * C + c) = acc;
}

}  // namespace

void launch_rank_from_idx(const int32_t* idx, int32_t* rank, int B, int N, int k, hipStream_t stream) {
    rank_from_idx_kernel<<<dim3((N + 255) / 256, B), 256, 0, stream>>>(idx, rank, N, k);
}

void launch_restore(const void* y_kept, const int32_t* rank, int B, int k, const void* cache_map, int hc,
                    int wc, int h, int w, int D, void* y_out, hipStream_t stream) {
    const int N = h * w;
    const int rows_per_block = 4 * kRowsPerWave;
    restore_kernel<<<dim3((N + rows_per_block - 1) / rows_per_block, B), 256, 0, stream>>>(
        static_cast<const bf16_t*>(y_kept), rank, k, static_cast<const bf16_t*>(cache_map), hc, wc, h, w, D,
        static_cast<bf16_t*>(y_out));
}

void launch_residual_accumulate(const float* r_prev, int hp, int wp, const void* f_k, int h, int w, int B, int C,
                                float* r_out, hipStream_t stream) {
    const long total = (long)B * h * w * (C / 4);
    if (total == 0) return;
    const unsigned blocks = (unsigned)((total + 255) / 256);
    residual_accumulate_kernel<<<blocks, 256, 0, stream>>>(r_prev, hp, wp, static_cast<const bf16_t*>(f_k), h, w, C,
                                                           r_out, total);
}

}  // namespace fv
