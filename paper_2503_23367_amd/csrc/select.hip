// Pivotal Token Selection (FastVAR Sec. 3.3, Eq. 4-5): per-channel mean over
// the token positions, squared distance of every token from it, and the k
// highest-scoring tokens per sample.
//
// Four launches, all bit-reproducible (no floating-point atomics):
//   colsum_partial   fp64 column sums of row chunks           (HBM bound: reads x once)
//   colsum_finalize  fixed-order sum of the chunk partials / N (tiny)
//   score            fp64 sum_c (x - mean)^2 per token, one wave per token,
//                    mean staged in LDS, rounded once to fp32  (re-reads x, mostly from cache)
//   topk             one workgroup per sample: MSB-first radix select on the
//                    order-preserving bit pattern of the fp32 score, then an
//                    ordered compaction (ties to the lowest index)
#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

constexpr int kColsPerWave = 512;  // 64 lanes x 8 bf16 (one 16-byte load per lane)
constexpr int kRedStride = 72;     // padded [j][lane] stride of the LDS reduction buffer

__device__ __forceinline__ void add8(double (&acc)[8], const uint4& v) {
    acc[0] += (double)bf16_lo(v.x);
    acc[1] += (double)bf16_hi(v.x);
    acc[2] += (double)bf16_lo(v.y);
    acc[3] += (double)bf16_hi(v.y);
    acc[4] += (double)bf16_lo(v.z);
    acc[5] += (double)bf16_hi(v.z);
    acc[6] += (double)bf16_lo(v.w);
    acc[7] += (double)bf16_hi(v.w);
}

// grid (col_tiles, n_chunks, B), block 256.  Wave w of a block sums rows
// r0+w, r0+w+4, ... of its chunk for the block's 512 columns; the four waves
// are then combined through LDS in a fixed order.
__global__ __launch_bounds__(256) void colsum_partial_kernel(const bf16_t* __restrict__ x,
                                                             double* __restrict__ partial, int N, int D,
                                                             int rows_per_chunk, int n_chunks) {
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int col = blockIdx.x * kColsPerWave + lane * 8;
    const int b = blockIdx.z;
    const int r0 = blockIdx.y * rows_per_chunk;
    const int r1 = min(r0 + rows_per_chunk, N);

    double acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0;

    if (col < D) {
        const bf16_t* base = x + (size_t)b * N * D + col;
        int r = r0 + wave;
        for (; r + 12 < r1; r += 16) {
            const uint4 v0 = *reinterpret_cast<const uint4*>(base + (size_t)(r + 0) * D);
            const uint4 v1 = *reinterpret_cast<const uint4*>(base + (size_t)(r + 4) * D);
            const uint4 v2 = *reinterpret_cast<const uint4*>(base + (size_t)(r + 8) * D);
            const uint4 v3 = *reinterpret_cast<const uint4*>(base + (size_t)(r + 12) * D);
            add8(acc, v0);
            add8(acc, v1);
            add8(acc, v2);
            add8(acc, v3);
        }
        for (; r < r1; r += 4) {
            const uint4 v0 = *reinterpret_cast<const uint4*>(base + (size_t)r * D);
            add8(acc, v0);
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
        const int c = blockIdx.x * kColsPerWave + cl;
        if (c < D) partial[((size_t)b * n_chunks + blockIdx.y) * D + c] = s;
    }
}

// grid (ceil(D/64), B), block 1024: mean[b,c] = (sum of the chunk partials) / N.
// Thread (c = t%64, g = t/64) sums every 16th chunk starting at g, ascending (eight
// independent loads at a time); the sixteen partial sums of a column are then
// added in a fixed order.
constexpr int kFinGroups = 16;
__global__ __launch_bounds__(64 * kFinGroups) void colsum_finalize_kernel(const double* __restrict__ partial,
                                                                          double* __restrict__ mean, int N, int D,
                                                                          int n_chunks) {
    __shared__ double part[kFinGroups][64];
    const int cl = threadIdx.x & 63, g = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + cl;
    const int b = blockIdx.y;
    double s = 0.0;
    if (c < D) {
        const double* p = partial + (size_t)b * n_chunks * D + c;
        int y = g;
        for (; y + 7 * kFinGroups < n_chunks; y += 8 * kFinGroups) {
            double a[8];
#pragma unroll
            for (int j = 0; j < 8; ++j) a[j] = p[(size_t)(y + j * kFinGroups) * D];
#pragma unroll
            for (int j = 0; j < 8; ++j) s += a[j];
        }
        for (; y < n_chunks; y += kFinGroups) s += p[(size_t)y * D];
    }
    part[g][cl] = s;
    __syncthreads();
    if (g == 0 && c < D) {
        double t = part[0][cl];
#pragma unroll
        for (int j = 1; j < kFinGroups; ++j) t += part[j][cl];
        mean[(size_t)b * D + c] = t / (double)N;
    }
}

constexpr int kScoreRowsPerBlock = 16;  // 8 waves x 2 rows: two waves per SIMD cover each other's fp64 chains and loads
constexpr int kScoreThreads = 512;

__device__ __forceinline__ void sqdev8(double& acc, const uint4& v, const double* mu /* stride 64 */) {
    double d;
    d = (double)bf16_lo(v.x) - mu[0 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_hi(v.x) - mu[1 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_lo(v.y) - mu[2 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_hi(v.y) - mu[3 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_lo(v.z) - mu[4 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_hi(v.z) - mu[5 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_lo(v.w) - mu[6 * 64]; acc = fma(d, d, acc);
    d = (double)bf16_hi(v.w) - mu[7 * 64]; acc = fma(d, d, acc);
}

// grid (ceil(N/16), B), block 512, dynamic LDS = round_up(D,512) doubles.
// The mean is staged in LDS as [group of 512 cols][j = col%8][lane = (col%512)/8]
// so that the 64 lanes of a wave read consecutive doubles.
__global__ __launch_bounds__(kScoreThreads) void score_kernel(const bf16_t* __restrict__ x,
                                                    const double* __restrict__ mean,
                                                    float* __restrict__ score, int N, int D) {
    extern __shared__ double mu_s[];
    const int b = blockIdx.y;
    for (int c = threadIdx.x; c < D; c += kScoreThreads) {
        const int g = c >> 9, r = c & 511;
        mu_s[g * 512 + (r & 7) * 64 + (r >> 3)] = mean[(size_t)b * D + c];
    }
    __syncthreads();

    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int groups = (D + 511) >> 9;
    {
        const int n0 = blockIdx.x * kScoreRowsPerBlock + wave * 2;
        const int n1 = n0 + 1;
        const bool ok0 = n0 < N, ok1 = n1 < N;
        const bf16_t* row0 = x + ((size_t)b * N + (ok0 ? n0 : 0)) * D;
        const bf16_t* row1 = x + ((size_t)b * N + (ok1 ? n1 : 0)) * D;
        double acc0 = 0.0, acc1 = 0.0;
        for (int g = 0; g < groups; ++g) {
            const int col = g * 512 + lane * 8;
            if (col < D) {
                const uint4 v0 = *reinterpret_cast<const uint4*>(row0 + col);
                const uint4 v1 = *reinterpret_cast<const uint4*>(row1 + col);
                const double* mu = mu_s + g * 512 + lane;
                sqdev8(acc0, v0, mu);
                sqdev8(acc1, v1, mu);
            }
        }
        acc0 = wave_sum(acc0);
        acc1 = wave_sum(acc1);
        if (lane == 0) {
            if (ok0) score[(size_t)b * N + n0] = (float)acc0;
            if (ok1) score[(size_t)b * N + n1] = (float)acc1;
        }
    }
}

// Order-preserving map of an fp32 bit pattern to an unsigned key.
__device__ __forceinline__ uint32_t float_key(float f) {
    const uint32_t u = __float_as_uint(f);
    return u ^ ((u >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

constexpr int kTopkThreads = 1024;

// grid (B), block 1024, dynamic LDS = N uint32 keys.
__global__ __launch_bounds__(kTopkThreads) void topk_kernel(const float* __restrict__ score, int N, int k,
                                                            int32_t* __restrict__ idx,
                                                            int32_t* __restrict__ rank) {
    extern __shared__ uint32_t keys[];
    __shared__ uint32_t hist[256];
    __shared__ uint32_t sel[2];
    __shared__ uint32_t wave_tot[kTopkThreads / 64];

    const int b = blockIdx.x;
    const int t = threadIdx.x;
    for (int n = t; n < N; n += kTopkThreads) keys[n] = float_key(score[(size_t)b * N + n]);

    // ---- radix select: T = key of the k-th largest, need = how many keys equal to T are kept.
    // Scores of one map usually share their leading bits (same sign, nearby
    // exponents); those bits are found first (AND / OR over all keys) and the
    // 8-bit digit passes only walk the bits below them, which also keeps the
    // LDS histogram atomics from piling onto a single bin.
    uint32_t prefix = 0, mask = 0, k_rem = (uint32_t)k;
    if (k > 0) {
        uint32_t all_and = 0xFFFFFFFFu, all_or = 0u;
        for (int n = t; n < N; n += kTopkThreads) {  // this thread's own entries: no barrier needed yet
            const uint32_t key = keys[n];
            all_and &= key;
            all_or |= key;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            all_and &= __shfl_xor(all_and, o, 64);
            all_or |= __shfl_xor(all_or, o, 64);
        }
        if ((t & 63) == 0) { wave_tot[t >> 6] = all_and; hist[t >> 6] = all_or; }
        __syncthreads();
        for (int wv = 0; wv < kTopkThreads / 64; ++wv) { all_and &= wave_tot[wv]; all_or |= hist[wv]; }
        __syncthreads();
        const uint32_t differ = all_and ^ all_or;           // bits that are not common to all keys
        const int top = differ ? 32 - __clz(differ) : 0;     // number of low bits that may differ
        mask = top >= 32 ? 0u : (0xFFFFFFFFu << top);
        prefix = all_and & mask;
        for (int shift = top - 8; shift > -8; shift -= 8) {
            const int sh = shift < 0 ? 0 : shift;
            const uint32_t dmask = shift < 0 ? ((1u << (shift + 8)) - 1u) : 255u;  // last pass may be narrower
            if (t < 256) hist[t] = 0;
            __syncthreads();
            for (int n = t; n < N; n += kTopkThreads) {
                const uint32_t key = keys[n];
                if ((key & mask) == prefix) atomicAdd(&hist[(key >> sh) & dmask], 1u);
            }
            __syncthreads();
            if (t < 64) {
                const uint32_t h0 = hist[4 * t + 0], h1 = hist[4 * t + 1];
                const uint32_t h2 = hist[4 * t + 2], h3 = hist[4 * t + 3];
                const uint32_t tot = h0 + h1 + h2 + h3;
                uint32_t incl = tot;  // becomes sum over lanes >= t
#pragma unroll
                for (int o = 1; o < 64; o <<= 1) {
                    const uint32_t v = __shfl_down(incl, o, 64);
                    if (t + o < 64) incl += v;
                }
                const uint32_t c3 = incl - tot;  // keys in bins above 4t+3
                const uint32_t c2 = c3 + h3, c1 = c2 + h2, c0 = c1 + h1;
                if (c3 < k_rem && k_rem <= c3 + h3) { sel[0] = 4 * t + 3; sel[1] = k_rem - c3; }
                else if (c2 < k_rem && k_rem <= c2 + h2) { sel[0] = 4 * t + 2; sel[1] = k_rem - c2; }
                else if (c1 < k_rem && k_rem <= c1 + h1) { sel[0] = 4 * t + 1; sel[1] = k_rem - c1; }
                else if (c0 < k_rem && k_rem <= c0 + h0) { sel[0] = 4 * t + 0; sel[1] = k_rem - c0; }
            }
            __syncthreads();
            prefix |= sel[0] << sh;
            mask |= dmask << sh;
            k_rem = sel[1];
        }
    } else {
        __syncthreads();
        prefix = 0xFFFFFFFFu;  // nothing is greater; need = 0 keeps no tie
        k_rem = 0;
    }
    const uint32_t T = prefix, need = k_rem;

    // ---- ordered compaction: thread t owns tokens [t*E, (t+1)*E)
    const int E = (N + kTopkThreads - 1) / kTopkThreads;
    const int lo = min(t * E, N), hi = min(lo + E, N);
    uint32_t cnt = 0;  // (greater << 16) | equal ; both totals <= 32768
    for (int n = lo; n < hi; ++n) {
        const uint32_t key = keys[n];
        cnt += (key > T ? 0x10000u : 0u) + (key == T ? 1u : 0u);
    }
    uint32_t incl = cnt;
    const int lane = t & 63, wave = t >> 6;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const uint32_t v = __shfl_up(incl, o, 64);
        if (lane >= o) incl += v;
    }
    if (lane == 63) wave_tot[wave] = incl;
    __syncthreads();
    uint32_t before = incl - cnt;
    for (int wv = 0; wv < wave; ++wv) before += wave_tot[wv];
    uint32_t gt_before = before >> 16, eq_before = before & 0xFFFFu;
    for (int n = lo; n < hi; ++n) {
        const uint32_t key = keys[n];
        int pos = -1;
        if (key > T) {
            pos = (int)(gt_before + min(eq_before, need));
            ++gt_before;
        } else if (key == T) {
            if (eq_before < need) pos = (int)(gt_before + eq_before);
            ++eq_before;
        }
        if (pos >= 0) idx[(size_t)b * k + pos] = n;
        if (rank) rank[(size_t)b * N + n] = pos;
    }
}

}  // namespace

SelectPlan select_plan(int B, int N, int D) {
    SelectPlan p;
    p.col_tiles = (D + kColsPerWave - 1) / kColsPerWave;
    // 32 rows per chunk (8 per wave) lets a wave issue all of its loads at once;
    // the chunk count is capped at 256 so the fp64 partials stay a small
    // fraction of x (1/8 of its bytes at 32 rows per chunk, less beyond).
    int rows = 32;
    while ((N + rows - 1) / rows > 256) rows *= 2;
    p.rows_per_chunk = rows;
    p.n_chunks = (N + rows - 1) / rows;
    size_t off = 0;
    p.off_partial = off;
    off += (size_t)B * p.n_chunks * D * sizeof(double);
    p.off_mean = off;
    off += (size_t)B * D * sizeof(double);
    p.off_score = off;
    off += (((size_t)B * N * sizeof(float)) + 255) & ~(size_t)255;
    p.bytes = (off + 255) & ~(size_t)255;
    return p;
}

void launch_select(const void* x, int B, int N, int D, int k, int32_t* idx, int32_t* rank, float* score_out,
                   void* ws, const SelectPlan& plan, hipStream_t stream) {
    char* w = static_cast<char*>(ws);
    double* partial = reinterpret_cast<double*>(w + plan.off_partial);
    double* mean = reinterpret_cast<double*>(w + plan.off_mean);
    float* score = score_out ? score_out : reinterpret_cast<float*>(w + plan.off_score);
    const bf16_t* xb = static_cast<const bf16_t*>(x);

    colsum_partial_kernel<<<dim3(plan.col_tiles, plan.n_chunks, B), 256, 0, stream>>>(
        xb, partial, N, D, plan.rows_per_chunk, plan.n_chunks);
    colsum_finalize_kernel<<<dim3((D + 63) / 64, B), 64 * kFinGroups, 0, stream>>>(partial, mean, N, D, plan.n_chunks);
    const size_t mu_bytes = (size_t)plan.col_tiles * 512 * sizeof(double);
    score_kernel<<<dim3((N + kScoreRowsPerBlock - 1) / kScoreRowsPerBlock, B), kScoreThreads, mu_bytes, stream>>>(
        xb, mean, score, N, D);
    static std::once_flag once;  // maps above 16K tokens need more than the default 64 KB of dynamic LDS
    raise_lds_limit_once(once, &topk_kernel, 32768 * sizeof(uint32_t));
    topk_kernel<<<dim3(B), kTopkThreads, (size_t)N * sizeof(uint32_t), stream>>>(score, N, k, idx, rank);
}

}  // namespace fv
