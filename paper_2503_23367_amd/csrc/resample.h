// Device-side pieces of Cached Token Restoration (FastVAR Sec. 3.3, Eq. 6) shared by the kernels that
// fill pruned slots: half-pixel-centre bilinear taps and the fill of one pruned token row.
#pragma once

#include "common.h"

namespace fv {

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

// Eight channels of the four taps -> eight bf16 outputs (one rounding).
__device__ __forceinline__ uint4 lerp8(const uint4& a, const uint4& bq, const uint4& c, const uint4& d, float lr,
                                       float lc) {
    uint4 o;
    o.x = pack_bf16x2(lerp2(bf16_lo(a.x), bf16_lo(bq.x), bf16_lo(c.x), bf16_lo(d.x), lr, lc),
                      lerp2(bf16_hi(a.x), bf16_hi(bq.x), bf16_hi(c.x), bf16_hi(d.x), lr, lc));
    o.y = pack_bf16x2(lerp2(bf16_lo(a.y), bf16_lo(bq.y), bf16_lo(c.y), bf16_lo(d.y), lr, lc),
                      lerp2(bf16_hi(a.y), bf16_hi(bq.y), bf16_hi(c.y), bf16_hi(d.y), lr, lc));
    o.z = pack_bf16x2(lerp2(bf16_lo(a.z), bf16_lo(bq.z), bf16_lo(c.z), bf16_lo(d.z), lr, lc),
                      lerp2(bf16_hi(a.z), bf16_hi(bq.z), bf16_hi(c.z), bf16_hi(d.z), lr, lc));
    o.w = pack_bf16x2(lerp2(bf16_lo(a.w), bf16_lo(bq.w), bf16_lo(c.w), bf16_lo(d.w), lr, lc),
                      lerp2(bf16_hi(a.w), bf16_hi(bq.w), bf16_hi(c.w), bf16_hi(d.w), lr, lc));
    return o;
}

// One wave fills token row n of sample b of the restored map from the cached map cb [hc*wc, D] of that
// sample: the bilinear resampling of Eq. 6, 16 bytes per lane and 512-column group.
// Any width, in passes of at most four groups; the sixteen tap loads of a pass go out before their first
// use, so a pass costs one memory latency, not one per group.
__device__ __forceinline__ void fill_pruned_row_any(const bf16_t* __restrict__ cb, int hc, int wc, int h, int w,
                                                    int D, int n, int lane, bf16_t* __restrict__ dst) {
    for (int c0 = 0; c0 < D; c0 += 2048) {
        const int Dp = min(D - c0, 2048);
        int i0, i1, j0, j1;
        float lr, lc;
        axis_taps(n / w, hc, h, i0, i1, lr);
        axis_taps(n % w, wc, w, j0, j1, lc);
        const bf16_t* p00 = cb + ((size_t)i0 * wc + j0) * D + c0;
        const bf16_t* p01 = cb + ((size_t)i0 * wc + j1) * D + c0;
        const bf16_t* p10 = cb + ((size_t)i1 * wc + j0) * D + c0;
        const bf16_t* p11 = cb + ((size_t)i1 * wc + j1) * D + c0;
        uint4 a[4], bq[4], c[4], d[4];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col = g * 512 + lane * 8;
            if (col < Dp) {
                a[g] = *reinterpret_cast<const uint4*>(p00 + col);
                bq[g] = *reinterpret_cast<const uint4*>(p01 + col);
                c[g] = *reinterpret_cast<const uint4*>(p10 + col);
                d[g] = *reinterpret_cast<const uint4*>(p11 + col);
            }
        }
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int col = g * 512 + lane * 8;
            if (col < Dp) *reinterpret_cast<uint4*>(dst + c0 + col) = lerp8(a[g], bq[g], c[g], d[g], lr, lc);
        }
    }
}

}  // namespace fv
