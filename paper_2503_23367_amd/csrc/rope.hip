// Table of the axial 2-D rotary embedding: cos and sin of the rotation angle of every interleaved pair of
// a head, for every slot of an h x w token map.  Pair t of the dh/2 pairs is turned by
// pos * base^(-t'/(dh/4)): the first dh/4 pairs by the slot's grid row, the others by its grid column
// (t' = t mod dh/4); coordinates are laid over a reference grid (i * ref_h / h, j * ref_w / w).
// The table is what the QKV GEMM's epilogue reads, gathered by the kept index set, to turn q and the
// new keys.  Evaluated in fp64 and rounded once to fp32; tiny (N * dh/2 entries), launch bound.
#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

__global__ __launch_bounds__(256) void rope2d_table_kernel(int h, int w, int half, double log_base, double sh,
                                                           double sw, float* __restrict__ cos_out,
                                                           float* __restrict__ sin_out, int total) {
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= total) return;
    const int n = i / half, t = i - n * half;
    const int q = half >> 1;
    const int tt = t < q ? t : t - q;
    const double pos = t < q ? (double)(n / w) * sh : (double)(n % w) * sw;
    const double ang = pos * exp(-((double)tt / (double)q) * log_base);
    cos_out[i] = (float)cos(ang);
    sin_out[i] = (float)sin(ang);
}

}  // namespace

void launch_rope2d_table(int h, int w, int dh, double base, int ref_h, int ref_w, float* cos_out, float* sin_out,
                         hipStream_t stream) {
    const int half = dh / 2;
    const int total = h * w * half;
    rope2d_table_kernel<<<(total + 255) / 256, 256, 0, stream>>>(h, w, half, log(base), (double)ref_h / (double)h,
                                                                (double)ref_w / (double)w, cos_out, sin_out, total);
}

}  // namespace fv
