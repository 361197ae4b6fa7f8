// Cached Token Restoration (FastVAR Sec. 3.3, Eq. 6 and the scatter that
// follows it): every slot of the restored map is either the kept token's block
// output (a row copy) or the cached previous-scale map resampled bilinearly at
// half-pixel centres.  One pass over the output, one wave per token row,
// 16-byte loads and stores; HBM bound (writes N*D bf16 once).
#include "common.h"
#include "kernels.h"

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

// Source taps of one axis for output position d (half-pixel centres, clamped).
__device__ __forceinline__ void axis_taps(int d, int n_in, int n_out, int& i0, int& i1, float& lam) {
    double src = ((double)d + 0.5) * ((double)n_in / (double)n_out) - 0.5;
    src = fmin(fmax(src, 0.0), (double)(n_in - 1));
    const double f = floor(src);
    i0 = (int)f;
    i1 = min(i0 + 1, n_in - 1);
    lam = (float)(src - f);
}

__device__ __forceinline__ float lerp2(float c00, float c01, float c10, float c11, float lr, float lc) {
    const float top = c00 + lc * (c01 - c00);
    const float bot = c10 + lc * (c11 - c10);
    return top + lr * (bot - top);
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
            int i0, i1, j0, j1;
            float lr, lc;
            axis_taps(n / w, hc, h, i0, i1, lr);
            axis_taps(n % w, wc, w, j0, j1, lc);
            const bf16_t* cb = cache_map + (size_t)b * hc * wc * D;
            const bf16_t* p00 = cb + ((size_t)i0 * wc + j0) * D;
            const bf16_t* p01 = cb + ((size_t)i0 * wc + j1) * D;
            const bf16_t* p10 = cb + ((size_t)i1 * wc + j0) * D;
            const bf16_t* p11 = cb + ((size_t)i1 * wc + j1) * D;
            for (int g = 0; g < groups; ++g) {
                const int col = g * 512 + lane * 8;
                if (col < D) {
                    const uint4 a = *reinterpret_cast<const uint4*>(p00 + col);
                    const uint4 bq = *reinterpret_cast<const uint4*>(p01 + col);
                    const uint4 c = *reinterpret_cast<const uint4*>(p10 + col);
                    const uint4 d = *reinterpret_cast<const uint4*>(p11 + col);
                    uint4 o;
                    o.x = pack_bf16x2(lerp2(bf16_lo(a.x), bf16_lo(bq.x), bf16_lo(c.x), bf16_lo(d.x), lr, lc),
                                      lerp2(bf16_hi(a.x), bf16_hi(bq.x), bf16_hi(c.x), bf16_hi(d.x), lr, lc));
                    o.y = pack_bf16x2(lerp2(bf16_lo(a.y), bf16_lo(bq.y), bf16_lo(c.y), bf16_lo(d.y), lr, lc),
                                      lerp2(bf16_hi(a.y), bf16_hi(bq.y), bf16_hi(c.y), bf16_hi(d.y), lr, lc));
                    o.z = pack_bf16x2(lerp2(bf16_lo(a.z), bf16_lo(bq.z), bf16_lo(c.z), bf16_lo(d.z), lr, lc),
                                      lerp2(bf16_hi(a.z), bf16_hi(bq.z), bf16_hi(c.z), bf16_hi(d.z), lr, lc));
                    o.w = pack_bf16x2(lerp2(bf16_lo(a.w), bf16_lo(bq.w), bf16_lo(c.w), bf16_lo(d.w), lr, lc),
                                      lerp2(bf16_hi(a.w), bf16_hi(bq.w), bf16_hi(c.w), bf16_hi(d.w), lr, lc));
                    *reinterpret_cast<uint4*>(dst + col) = o;
                }
            }
        }
    }
}

// Restoration fused with the column sums the next selection starts with.  Same geometry as the
// selection's own first pass: grid (column tiles of 512, row chunks, B), block 256; wave w of a block
// takes rows r0+w, r0+w+4, ... of its chunk, lane l eight columns, and adds the bf16 values it
// writes (or, for kept rows that are already in place, reads) to fp64 sums in ascending row order;
// the four waves are combined through LDS in the same fixed order.  The partials are therefore bit
// for bit what that pass would compute from y_out.
constexpr int kColsPerTile = 512;
constexpr int kRedStride = 72;

__device__ __forceinline__ void add8d(double (&acc)[8], const uint4& v) {
    acc[0] += (double)bf16_lo(v.x);
    acc[1] += (double)bf16_hi(v.x);
    acc[2] += (double)bf16_lo(v.y);
    acc[3] += (double)bf16_hi(v.y);
    acc[4] += (double)bf16_lo(v.z);
    acc[5] += (double)bf16_hi(v.z);
    acc[6] += (double)bf16_lo(v.w);
    acc[7] += (double)bf16_hi(v.w);
}

__global__ __launch_bounds__(256) void restore_colsum_kernel(const bf16_t* __restrict__ y_kept,
                                                             const int32_t* __restrict__ rank, int k,
                                                             const bf16_t* __restrict__ cache_map, int hc, int wc,
                                                             int h, int w, int D, bf16_t* y_out,
                                                             double* __restrict__ partial, int rows_per_chunk,
                                                             int n_chunks) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = blockIdx.x * kColsPerTile + lane * 8;
    const int b = blockIdx.z;
    const int N = h * w;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(r0 + rows_per_chunk, N);

    double acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0;

    if (col < D) {
        const bf16_t* cb = cache_map + (size_t)b * hc * wc * D + col;
        // Rows are taken eight at a time (one chunk of 32 rows is eight per wave): first every row's
        // rank, then every row's loads, then the arithmetic, so that the memory latencies of the rows
        // overlap instead of adding up.  The sums still see the rows in ascending order.
        constexpr int RB = 8;
        for (int nb = r0 + wave; nb < r1; nb += 4 * RB) {
            int rk[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int n = nb + 4 * i;
                rk[i] = (n < r1 && k > 0) ? rank[(size_t)b * N + n] : -1;
            }
            uint4 t0[RB], t1[RB], t2[RB], t3[RB];
            float lr[RB], lc[RB];
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int n = nb + 4 * i;
                if (n < r1) {
                    if (rk[i] >= 0) {
                        const bf16_t* src = y_kept ? y_kept + ((size_t)b * k + rk[i]) * D + col
                                                   : y_out + ((size_t)b * N + n) * D + col;   // already in place
                        t0[i] = *reinterpret_cast<const uint4*>(src);
                    } else {
                        int i0, i1, j0, j1;
                        axis_taps(n / w, hc, h, i0, i1, lr[i]);
                        axis_taps(n % w, wc, w, j0, j1, lc[i]);
                        t0[i] = *reinterpret_cast<const uint4*>(cb + ((size_t)i0 * wc + j0) * D);
                        t1[i] = *reinterpret_cast<const uint4*>(cb + ((size_t)i0 * wc + j1) * D);
                        t2[i] = *reinterpret_cast<const uint4*>(cb + ((size_t)i1 * wc + j0) * D);
                        t3[i] = *reinterpret_cast<const uint4*>(cb + ((size_t)i1 * wc + j1) * D);
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < RB; ++i) {
                const int n = nb + 4 * i;
                if (n < r1) {
                    bf16_t* dst = y_out + ((size_t)b * N + n) * D + col;
                    uint4 o;
                    if (rk[i] >= 0) {
                        o = t0[i];
                        if (y_kept) *reinterpret_cast<uint4*>(dst) = o;
                    } else {
                        const uint4 a = t0[i], bq = t1[i], c = t2[i], d = t3[i];
                        const float fr = lr[i], fc = lc[i];
                        o.x = pack_bf16x2(lerp2(bf16_lo(a.x), bf16_lo(bq.x), bf16_lo(c.x), bf16_lo(d.x), fr, fc),
                                          lerp2(bf16_hi(a.x), bf16_hi(bq.x), bf16_hi(c.x), bf16_hi(d.x), fr, fc));
                        o.y = pack_bf16x2(lerp2(bf16_lo(a.y), bf16_lo(bq.y), bf16_lo(c.y), bf16_lo(d.y), fr, fc),
                                          lerp2(bf16_hi(a.y), bf16_hi(bq.y), bf16_hi(c.y), bf16_hi(d.y), fr, fc));
                        o.z = pack_bf16x2(lerp2(bf16_lo(a.z), bf16_lo(bq.z), bf16_lo(c.z), bf16_lo(d.z), fr, fc),
                                          lerp2(bf16_hi(a.z), bf16_hi(bq.z), bf16_hi(c.z), bf16_hi(d.z), fr, fc));
                        o.w = pack_bf16x2(lerp2(bf16_lo(a.w), bf16_lo(bq.w), bf16_lo(c.w), bf16_lo(d.w), fr, fc),
                                          lerp2(bf16_hi(a.w), bf16_hi(bq.w), bf16_hi(c.w), bf16_hi(d.w), fr, fc));
                        *reinterpret_cast<uint4*>(dst) = o;
                    }
                    add8d(acc, o);
                }
            }
        }
    }

    __shared__ double red[4][8 * kRedStride];
#pragma unroll
    for (int j = 0; j < 8; ++j) red[wave][j * kRedStride + lane] = acc[j];
    __syncthreads();
#pragma unroll
    for (int e = 0; e < 2; ++e) {
        const int cl = threadIdx.x + e * 256;  // column inside the tile
        const int at = (cl & 7) * kRedStride + (cl >> 3);
        const double s = ((red[0][at] + red[1][at]) + red[2][at]) + red[3][at];
        const int c = blockIdx.x * kColsPerTile + cl;
        if (c < D) partial[((size_t)b * n_chunks + blockIdx.y) * D + c] = s;
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

void launch_restore_colsum(const void* y_kept, const int32_t* rank, int B, int k, const void* cache_map, int hc,
                           int wc, int h, int w, int D, void* y_out, void* select_ws, const SelectPlan& plan,
                           hipStream_t stream) {
    double* partial = reinterpret_cast<double*>(static_cast<char*>(select_ws) + plan.off_partial);
    restore_colsum_kernel<<<dim3(plan.col_tiles, plan.n_chunks, B), 256, 0, stream>>>(
        static_cast<const bf16_t*>(y_kept), rank, k, static_cast<const bf16_t*>(cache_map), hc, wc, h, w, D,
        static_cast<bf16_t*>(y_out), partial, plan.rows_per_chunk, plan.n_chunks);
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
