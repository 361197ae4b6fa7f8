// Flash-style attention of the kept queries over the multi-scale KV cache
// (all earlier scales followed by the kept tokens of the current one); no mask
// is needed at decode time.  bf16 MFMA with fp32 online softmax.
//
// Orientation: the kernel computes the TRANSPOSED score tile S^T = K * Q^T with
// 32x32x16 MFMAs, so a lane owns one query column: the softmax row statistics
// need only a register reduction plus one exchange between the two half-waves,
// the rescale of the output accumulator is a per-lane scalar, and the
// accumulator registers of S^T are, after conversion to bf16, exactly the
// B operand of the second MFMA  O^T += V^T * P^T.  The contraction index of
// that second product is the key; its lane layout wants 8 consecutive keys per
// lane, which is why the V cache is stored with the cache position contiguous
// ([B,H,dh,L_cap]) and why key rows are placed in LDS with bits 2 and 3 of the
// in-block key index exchanged (the accumulator row order of the first MFMA
// then lines up with 16-byte runs of keys in the V^T tile).
//
// A workgroup of 4 waves owns 128*QB queries of one (sample, head); each wave
// owns 32*QB of them and walks all keys in tiles of 64.  K and V^T tiles are
// staged in LDS (double buffered, XOR-swizzled 16-byte chunks) and shared by
// the four waves.
#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

constexpr int BN = 64;  // keys per tile

struct AttnParams {
    const bf16_t* q;
    const bf16_t* kc;
    const bf16_t* vc;
    bf16_t* o;
    int H, k_tokens, L, L_cap, D;
    float scale_log2e;
};

__device__ __forceinline__ int swap_bits_2_3(int v) {
    return (v & ~12) | ((v & 4) << 1) | ((v & 8) >> 1);
}

// Eight consecutive cache positions of one V^T row; `valid` = how many of them
// lie inside the cache length.  Positions past the length may hold anything
// (even NaN patterns), so they are read as zero.
__device__ __forceinline__ u32x4_t load_v_chunk(const bf16_t* src, int valid) {
    u32x4_t v = {0u, 0u, 0u, 0u};
    if (valid > 0) {
        v = *reinterpret_cast<const u32x4_t*>(src);
        if (valid < 8) {
            v.x = valid >= 2 ? v.x : (v.x & 0xFFFFu);
            v.y = valid >= 4 ? v.y : (valid >= 3 ? (v.y & 0xFFFFu) : 0u);
            v.z = valid >= 6 ? v.z : (valid >= 5 ? (v.z & 0xFFFFu) : 0u);
            v.w = valid >= 7 ? (v.w & 0xFFFFu) : 0u;
        }
    }
    return v;
}

template <int DH, int QB>
__global__ __launch_bounds__(256) void attention_kernel(const AttnParams p) {
    constexpr int KCH = DH / 8;            // 16-byte chunks per key row
    constexpr int KS = DH / 16;            // MFMA k-steps over the head dim
    constexpr int DB = DH / 32;            // 32-row blocks of O^T
    constexpr int K_LD = BN * KCH / 256;   // K-tile chunks per thread
    constexpr int V_LD = DH * 8 / 256;     // V^T-tile chunks per thread
    constexpr int K_TILE = BN * KCH;       // u32x4_t per K tile
    constexpr int V_TILE = DH * 8;         // u32x4_t per V^T tile

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t* sK = reinterpret_cast<u32x4_t*>(smem);  // [2][K_TILE]
    u32x4_t* sV = sK + 2 * K_TILE;                 // [2][V_TILE]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int li = lane & 31;   // query column / operand row
    const int hf = lane >> 5;   // half-wave
    const int sw = lane & 7;    // swizzle key of this lane's operand row
    const int head = blockIdx.y;
    const int b = blockIdx.z;
    const int q_base = blockIdx.x * (128 * QB) + wave * (32 * QB);

    const bf16_t* kc = p.kc + ((size_t)b * p.H + head) * p.L_cap * DH;
    const bf16_t* vc = p.vc + ((size_t)b * p.H + head) * DH * (size_t)p.L_cap;

    // Q^T operand fragments: lane (li, hf) holds q[query li][16*ks + 8*hf .. +8)
    bf16x8_t qf[QB][KS];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qrow = min(q_base + qb * 32 + li, p.k_tokens - 1);
        const bf16_t* src = p.q + ((size_t)b * p.k_tokens + qrow) * p.D + head * DH + hf * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) qf[qb][ks] = *reinterpret_cast<const bf16x8_t*>(src + ks * 16);
    }

    f32x16_t acc[DB][QB];
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[db][qb][r] = 0.f;
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; }

    const int KT = (p.L + BN - 1) / BN;
    u32x4_t rk[K_LD], rv[V_LD];

#define FV_LOAD_GLOBAL(kt_)                                                                         \
    {                                                                                               \
        const int key0_ = (kt_) * BN;                                                               \
        _Pragma("unroll") for (int i = 0; i < K_LD; ++i) {                                          \
            const int q_ = tid + 256 * i;                                                           \
            const int key_ = min(key0_ + q_ / KCH, p.L - 1);                                        \
            rk[i] = *reinterpret_cast<const u32x4_t*>(kc + (size_t)key_ * DH + (q_ % KCH) * 8);     \
        }                                                                                           \
        _Pragma("unroll") for (int i = 0; i < V_LD; ++i) {                                          \
            const int q_ = tid + 256 * i;                                                           \
            const int kpos_ = key0_ + (q_ & 7) * 8;                                                 \
            rv[i] = load_v_chunk(vc + (size_t)(q_ >> 3) * p.L_cap + kpos_, p.L - kpos_);            \
        }                                                                                           \
    }
#define FV_STORE_LDS(buf_)                                                                          \
    {                                                                                               \
        _Pragma("unroll") for (int i = 0; i < K_LD; ++i) {                                          \
            const int q_ = tid + 256 * i;                                                           \
            const int row_ = q_ / KCH, c_ = q_ % KCH;                                               \
            const int slot_ = (row_ & ~31) | swap_bits_2_3(row_ & 31);                              \
            sK[(buf_) * K_TILE + slot_ * KCH + (c_ ^ (slot_ & 7))] = rk[i];                         \
        }                                                                                           \
        _Pragma("unroll") for (int i = 0; i < V_LD; ++i) {                                          \
            const int q_ = tid + 256 * i;                                                           \
            const int d_ = q_ >> 3, c_ = q_ & 7;                                                    \
            sV[(buf_) * V_TILE + d_ * 8 + (c_ ^ (d_ & 7))] = rv[i];                                 \
        }                                                                                           \
    }

    FV_LOAD_GLOBAL(0)
    FV_STORE_LDS(0)
    __syncthreads();

    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) FV_LOAD_GLOBAL(kt + 1)

        // ---- S^T = K * Q^T for 64 keys x 32*QB queries
        f32x16_t s[2][QB];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int r = 0; r < 16; ++r) s[kb][qb][r] = 0.f;
        const u32x4_t* k_base = sK + buf * K_TILE;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const bf16x8_t a = *reinterpret_cast<const bf16x8_t*>(
                    k_base + (kb * 32 + li) * KCH + ((2 * ks + hf) ^ sw));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    s[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[qb][ks], s[kb][qb], 0, 0, 0);
            }
        }

        // ---- mask keys past the cache length (last tile only)
        if (kt == KT - 1 && (p.L & (BN - 1)) != 0) {
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int srow = 8 * (r >> 2) + 4 * hf + (r & 3);
                    const int key = kt * BN + kb * 32 + swap_bits_2_3(srow);
                    if (key >= p.L) {
#pragma unroll
                        for (int qb = 0; qb < QB; ++qb) s[kb][qb][r] = -INFINITY;
                    }
                }
        }

        // ---- online softmax, one query per lane (two half-waves share a query)
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float mx = s[0][qb][0];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) mx = fmaxf(mx, s[kb][qb][r]);
            mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
            const float m_new = fmaxf(m_run[qb], mx * p.scale_log2e);
            const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
            m_run[qb] = m_new;
            float lsum = 0.f;
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][r], p.scale_log2e, -m_new));
                    s[kb][qb][r] = pv;
                    lsum += pv;
                }
            l_run[qb] = l_run[qb] * alpha + lsum;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[db][qb][r] *= alpha;
            }
        }

        // ---- O^T += V^T * P^T
        const u32x4_t* v_base = sV + buf * V_TILE;
#pragma unroll
        for (int t = 0; t < 4; ++t) {
            bf16x8_t pf[QB];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int j = 0; j < 8; ++j) pf[qb][j] = (__bf16)s[t >> 1][qb][(t & 1) * 8 + j];
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                const bf16x8_t vf = *reinterpret_cast<const bf16x8_t*>(
                    v_base + (db * 32 + li) * 8 + ((2 * t + hf) ^ sw));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
                    acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb], acc[db][qb], 0, 0, 0);
            }
        }

        if (kt + 1 < KT) FV_STORE_LDS(buf ^ 1)
        __syncthreads();
    }

    // ---- normalise and store: lane (li, hf) register r of block db is
    // o[query li][32*db + 8*(r/4) + 4*hf + r%4]
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
        const float inv = 1.0f / l_tot;
        const int qrow = q_base + qb * 32 + li;
        if (qrow < p.k_tokens) {
            bf16_t* dst = p.o + ((size_t)b * p.k_tokens + qrow) * p.D + head * DH + 4 * hf;
#pragma unroll
            for (int db = 0; db < DB; ++db)
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    uint2 pk;
                    pk.x = pack_bf16x2(acc[db][qb][4 * g + 0] * inv, acc[db][qb][4 * g + 1] * inv);
                    pk.y = pack_bf16x2(acc[db][qb][4 * g + 2] * inv, acc[db][qb][4 * g + 3] * inv);
                    *reinterpret_cast<uint2*>(dst + db * 32 + 8 * g) = pk;
                }
        }
    }
}

template <int DH, int QB>
void launch_cfg(const AttnParams& p, int B, hipStream_t stream) {
    constexpr size_t smem = (size_t)2 * (BN * (DH / 8) + DH * 8) * sizeof(u32x4_t);
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<DH, QB>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int per_wg = 128 * QB;
    attention_kernel<DH, QB><<<dim3((p.k_tokens + per_wg - 1) / per_wg, p.H, B), 256, smem, stream>>>(p);
}

}  // namespace

void launch_attention(const AttnArgs& a, hipStream_t stream) {
    AttnParams p;
    p.q = static_cast<const bf16_t*>(a.q);
    p.kc = static_cast<const bf16_t*>(a.k_cache);
    p.vc = static_cast<const bf16_t*>(a.v_cache);
    p.o = static_cast<bf16_t*>(a.o);
    p.H = a.H; p.k_tokens = a.k_tokens; p.L = a.L; p.L_cap = a.L_cap; p.D = a.H * a.dh;
    p.scale_log2e = a.scale * 1.4426950408889634f;
    // Two query blocks per wave halve the LDS traffic per MFMA but halve the
    // number of workgroups; take them only when the grid still covers the chip.
    const long wgs2 = (long)((a.k_tokens + 255) / 256) * a.H * a.B;
    const bool wide = wgs2 >= 256;
    if (a.dh == 128) {
        if (wide) launch_cfg<128, 2>(p, a.B, stream); else launch_cfg<128, 1>(p, a.B, stream);
    } else {
        if (wide) launch_cfg<64, 2>(p, a.B, stream); else launch_cfg<64, 1>(p, a.B, stream);
    }
}

}  // namespace fv
