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
// Work split: a wave owns 32*QB queries (QB = 2 halves the LDS traffic per
// MFMA: every K / V^T fragment read feeds two MFMAs).  A workgroup has
// QG * KSPLIT waves: QG query groups, and KSPLIT waves per group that each take
// a different 64-key slice of every (64*KSPLIT)-key tile and are merged at the
// end (softmax partials combine exactly).  KSPLIT = 2 keeps all SIMDs busy when
// there are too few queries for one wave per SIMD.
//
// K and V^T tiles go global -> LDS directly (no register staging), double
// buffered; 16-byte chunks are XOR-swizzled with the row so operand reads are
// conflict free.
#include <stdlib.h>

#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

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

// Value held by the lane 32 positions away (the other half-wave), through the
// cross-half swap instruction instead of an LDS round trip.
__device__ __forceinline__ float other_half(float v) {
    const uint32_t u = __float_as_uint(v);
    const auto r = __builtin_amdgcn_permlane32_swap(u, u, false, false);
    // after the swap r[0] = {low half, low half} and r[1] = {high half, high half}
    return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

constexpr int attn_waitcnt(int vm, bool lgkm) {
    return (vm & 0xF) | ((vm >> 4) << 14) | (0x7 << 4) | ((lgkm ? 0x0 : 0xF) << 8);
}

template <int DH, int QB, int QG, int KSPLIT>
__global__ __launch_bounds__(QG * KSPLIT * 64, 1) void attention_kernel(const AttnParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int WAVES = QG * KSPLIT;
    constexpr int BN = 64 * KSPLIT;        // keys per tile
    constexpr int KCH = DH / 8;            // 16-byte chunks per key row
    constexpr int KS = DH / 16;            // MFMA k-steps over the head dim
    constexpr int DB = DH / 32;            // 32-row blocks of O^T
    constexpr int VCH = BN / 8;            // 16-byte chunks per V^T row
    constexpr int K_TILE = BN * KCH;       // chunks per K tile
    constexpr int V_TILE = DH * VCH;       // chunks per V^T tile
    constexpr int K_RPI = 64 / KCH;        // key rows per 64-lane direct-to-LDS load
    constexpr int V_RPI = 64 / VCH;        // V^T rows per load
    constexpr int K_LD = BN / K_RPI / WAVES;   // loads per wave per tile
    constexpr int V_LD = DH / V_RPI / WAVES;
    static_assert(K_LD >= 1 && V_LD >= 1, "tile too small for this many waves");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t* lds = reinterpret_cast<u32x4_t*>(smem);  // [2][K tile] then [2][V^T tile]
    typedef __attribute__((address_space(3))) void* lds_ptr_t;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qg = wave / KSPLIT;       // query group
    const int kh = wave % KSPLIT;       // key slice inside a tile
    const int li = lane & 31;           // query column / operand row
    const int hf = lane >> 5;           // half-wave
    const int sw = lane & 7;            // swizzle key of this lane's operand row
    const int head = blockIdx.y;
    const int b = blockIdx.z;
    const int q_base = blockIdx.x * (QG * 32 * QB) + qg * (32 * QB);

    const bf16_t* kc = p.kc + ((size_t)b * p.H + head) * p.L_cap * DH;
    const bf16_t* vc = p.vc + ((size_t)b * p.H + head) * DH * (size_t)p.L_cap;

    // ---- per-lane source descriptors of the direct-to-LDS loads.  Load j of this
    // wave is instruction ij = wave + WAVES*j of the tile; it fills 1 KB of LDS,
    // lane l landing at chunk 64*ij + l.
    int k_key[K_LD], k_col[K_LD];   // key inside the tile, element offset inside the row
    int v_row[V_LD], v_col[V_LD];   // element offset of the V^T row, key offset inside the tile
#pragma unroll
    for (int j = 0; j < K_LD; ++j) {
        const int slot = (wave + WAVES * j) * K_RPI + lane / KCH;  // LDS row
        const int c = (lane % KCH) ^ (slot & 7);                   // logical chunk stored at this position
        k_key[j] = (slot & ~31) | swap_bits_2_3(slot & 31);
        k_col[j] = c * 8;
    }
#pragma unroll
    for (int j = 0; j < V_LD; ++j) {
        const int d = (wave + WAVES * j) * V_RPI + lane / VCH;
        const int c = (lane % VCH) ^ (d & 7);
        v_row[j] = d * p.L_cap;
        v_col[j] = c * 8;
    }
    const int last_chunk = ((p.L - 1) >> 3) << 3;  // start of the last 8-key run that holds a valid key

    // K tiles and V^T tiles live in separate two-stage rings: the second MFMA of
    // a tile is deferred to the next iteration (see the schedule below), so
    // iteration k consumes K tile k and V^T tile k-1.
#define FV_ISSUE_K(kt_)                                                                             \
    {                                                                                               \
        const int key0_ = (kt_) * BN;                                                               \
        u32x4_t* sk_ = lds + ((kt_) & 1) * K_TILE + wave * 64;                                      \
        _Pragma("unroll") for (int j = 0; j < K_LD; ++j) {                                          \
            const int key_ = min(key0_ + k_key[j], p.L - 1);                                        \
            __builtin_amdgcn_global_load_lds(kc + key_ * DH + k_col[j],                             \
                                             (lds_ptr_t)(sk_ + j * (WAVES * 64)), 16, 0, 0);        \
        }                                                                                           \
    }
#define FV_ISSUE_V(kt_)                                                                             \
    {                                                                                               \
        const int key0_ = (kt_) * BN;                                                               \
        u32x4_t* sv_ = lds + 2 * K_TILE + ((kt_) & 1) * V_TILE + wave * 64;                         \
        _Pragma("unroll") for (int j = 0; j < V_LD; ++j) {                                          \
            const int kpos_ = min(key0_ + v_col[j], last_chunk);                                    \
            __builtin_amdgcn_global_load_lds(vc + v_row[j] + kpos_,                                 \
                                             (lds_ptr_t)(sv_ + j * (WAVES * 64)), 16, 0, 0);        \
        }                                                                                           \
    }
    // Cache positions at or past the length may hold anything (even NaN patterns),
    // and 0 * NaN would poison the output: after its own loads of a partial tile
    // have landed, each lane zeroes the out-of-range positions of its V^T chunks.
#define FV_FIX_TAIL(kt_)                                                                            \
    {                                                                                               \
        __builtin_amdgcn_s_waitcnt(attn_waitcnt(0, true));                                          \
        const int key0_ = (kt_) * BN;                                                               \
        u32x4_t* sv_ = lds + 2 * K_TILE + ((kt_) & 1) * V_TILE + wave * 64 + lane;                  \
        _Pragma("unroll") for (int j = 0; j < V_LD; ++j) {                                          \
            const int valid_ = p.L - (key0_ + v_col[j]);                                            \
            if (valid_ < 8) {                                                                       \
                u32x4_t v_ = sv_[j * (WAVES * 64)];                                                 \
                v_.x = valid_ >= 2 ? v_.x : (valid_ >= 1 ? (v_.x & 0xFFFFu) : 0u);                  \
                v_.y = valid_ >= 4 ? v_.y : (valid_ >= 3 ? (v_.y & 0xFFFFu) : 0u);                  \
                v_.z = valid_ >= 6 ? v_.z : (valid_ >= 5 ? (v_.z & 0xFFFFu) : 0u);                  \
                v_.w = valid_ >= 7 ? (v_.w & 0xFFFFu) : 0u;                                         \
                sv_[j * (WAVES * 64)] = v_;                                                         \
            }                                                                                       \
        }                                                                                           \
    }
    // Own loads landed, own LDS reads done, then the workgroup barrier: publishes
    // the tiles just fetched and frees the stages the next iteration refills.
#define FV_PUBLISH()                                                                                \
    {                                                                                               \
        asm volatile("" ::: "memory");                                                              \
        __builtin_amdgcn_s_waitcnt(attn_waitcnt(0, true));                                          \
        __builtin_amdgcn_s_barrier();                                                               \
        asm volatile("" ::: "memory");                                                              \
    }

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
    const bool ragged = (p.L % BN) != 0;

    f32x16_t s_cur[2][QB];   // scores of tile k (this wave's 64-key slice: two 32-key blocks)
    f32x16_t s_nxt[2][QB];   // scores of tile k+1, produced while tile k is in the softmax
    bf16x8_t pf_[4][QB];     // probabilities of tile k-1 as the B operand of the second MFMA

    // S^T = K Q^T of tile kt_ into dst_ (prologue only; no overlap needed)
#define FV_QK_ONLY(kt_, dst_)                                                                       \
    {                                                                                               \
        const u32x4_t* k_base_ = lds + ((kt_) & 1) * K_TILE + (kh * 64) * KCH;                      \
        _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                            \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                       \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) dst_[kb][qb][r] = 0.f;               \
        _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                           \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) {                                      \
                const bf16x8_t a_ = *reinterpret_cast<const bf16x8_t*>(                             \
                    k_base_ + (kb * 32 + li) * KCH + ((2 * ks + hf) ^ sw));                         \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    dst_[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a_, qf[qb][ks], dst_[kb][qb], 0, 0, 0); \
            }                                                                                       \
    }
    // O^T += V^T P^T of tile kt_ alone (after the last iteration)
#define FV_PV_ONLY(kt_)                                                                             \
    {                                                                                               \
        const u32x4_t* v_base_ = lds + 2 * K_TILE + ((kt_) & 1) * V_TILE + kh * 8;                  \
        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                               \
            _Pragma("unroll") for (int db = 0; db < DB; ++db) {                                     \
                const bf16x8_t vf_ = *reinterpret_cast<const bf16x8_t*>(                            \
                    v_base_ + (db * 32 + li) * VCH + ((2 * t + hf) ^ sw));                          \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf_, pf_[t][qb], acc[db][qb], 0, 0, 0); \
            }                                                                                       \
    }

    // One iteration k of the software pipeline, three tiles in flight in one wave:
    //   matrix pipe : O^T += V^T P^T of tile k-1 (HAS_PV_), then S^T = K Q^T of tile k+1 (HAS_QK_)
    //   vector pipe : online softmax of tile k (s_cur -> new probabilities, running max / sum)
    // The two streams are independent inside the iteration.  The body is cut into
    // slices, one per operand fragment: the QB MFMAs that consume the fragment,
    // the LDS read of the fragment DEPTH slices ahead, and a small piece of the
    // softmax (a few VALU ops and exps fit under a 32-clock MFMA for free).
    // A scheduling fence after each slice keeps the compiler from regrouping them.
    // The rescale of O by the new maximum comes after the PV MFMAs of the iteration.
#define FV_SCUR(e_) s_cur[((e_) % 32) / 16][(e_) / 32][(e_) % 16]
#define FV_LOAD_FRAG(i_)                                                                            \
    {                                                                                               \
        if ((i_) < NV_) {                                                                           \
            fr_[(i_)] = *reinterpret_cast<const bf16x8_t*>(                                         \
                v_base_ + ((((i_) % DB)) * 32 + li) * VCH + ((2 * ((i_) / DB) + hf) ^ sw));         \
        } else {                                                                                    \
            fr_[(i_)] = *reinterpret_cast<const bf16x8_t*>(                                         \
                k_base_ + ((((i_) - NV_) % 2) * 32 + li) * KCH + ((2 * (((i_) - NV_) / 2) + hf) ^ sw)); \
        }                                                                                           \
    }
#define FV_ITER(kt_, HAS_PV_, HAS_QK_, MASK_)                                                       \
    {                                                                                               \
        constexpr int NV_ = (HAS_PV_) ? 4 * DB : 0;                                                 \
        constexpr int NK_ = (HAS_QK_) ? 2 * KS : 0;                                                 \
        constexpr int NF_ = NV_ + NK_;                                                              \
        constexpr int DEPTH_ = NF_ < 4 ? NF_ : 4;                                                   \
        constexpr int NE_ = 32 * QB;           /* score elements per lane */                        \
        constexpr int NMAX_ = 4;               /* slices that carry the max reduction */            \
        constexpr int EPS_ = 2 * QB;           /* elements exponentiated per later slice */         \
        const u32x4_t* v_base_ = lds + 2 * K_TILE + (((kt_) + 1) & 1) * V_TILE + kh * 8;            \
        const u32x4_t* k_base_ = lds + (((kt_) + 1) & 1) * K_TILE + (kh * 64) * KCH;                \
        bf16x8_t fr_[NF_ > 0 ? NF_ : 1];                                                            \
        if (MASK_) {                                                                                \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                    \
                    const int srow_ = 8 * (r >> 2) + 4 * hf + (r & 3);                              \
                    const int key_ = (kt_) * BN + kh * 64 + kb * 32 + swap_bits_2_3(srow_);         \
                    if (key_ >= p.L) {                                                              \
                        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) s_cur[kb][qb][r] = -INFINITY; \
                    }                                                                               \
                }                                                                                   \
        }                                                                                           \
        if (HAS_QK_) {                                                                              \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) s_nxt[kb][qb][r] = 0.f;          \
        }                                                                                           \
        _Pragma("unroll") for (int i = 0; i < DEPTH_; ++i) FV_LOAD_FRAG(i)                          \
        float mx_[QB], m_use_[QB], alpha_[QB], lsum_[QB];                                           \
        bf16x8_t pnew_[4][QB];                                                                      \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) { mx_[qb] = -INFINITY; lsum_[qb] = 0.f; } \
        constexpr int NSL_ = NF_ > (NMAX_ + 1 + NE_ / EPS_) ? NF_ : (NMAX_ + 1 + NE_ / EPS_);      \
        _Pragma("unroll") for (int i = 0; i < NSL_; ++i) {                                          \
            /* matrix stream */                                                                     \
            if (i < NV_) {                                                                          \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    acc[i % DB][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                      \
                        fr_[i < NF_ ? i : 0], pf_[i / DB][qb], acc[i % DB][qb], 0, 0, 0);           \
            } else if (i < NF_) {                                                                   \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    s_nxt[(i - NV_) % 2][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(             \
                        fr_[i < NF_ ? i : 0], qf[qb][((i - NV_) / 2) % KS], s_nxt[(i - NV_) % 2][qb], 0, 0, 0); \
            }                                                                                       \
            if (i + DEPTH_ < NF_) FV_LOAD_FRAG(i + DEPTH_)                                          \
            /* vector stream */                                                                     \
            if (i < NMAX_) {                                                                        \
                _Pragma("unroll") for (int e = i * (NE_ / NMAX_); e < (i + 1) * (NE_ / NMAX_); ++e) \
                    mx_[e / 32] = fmaxf(mx_[e / 32], FV_SCUR(e));                                   \
            } else if (i == NMAX_) {                                                                \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                 \
                    const float mxa_ = fmaxf(mx_[qb], other_half(mx_[qb]));                         \
                    /* a slice that is entirely past the length keeps the old maximum */           \
                    const float m_new_ = fmaxf(m_run[qb], mxa_ * p.scale_log2e);                    \
                    m_use_[qb] = (m_new_ == -INFINITY) ? 0.f : m_new_;                              \
                    alpha_[qb] = __builtin_amdgcn_exp2f(m_run[qb] - m_use_[qb]);                    \
                    m_run[qb] = m_new_;                                                             \
                }                                                                                   \
            } else if ((i - NMAX_ - 1) * EPS_ < NE_) {                                              \
                _Pragma("unroll") for (int e = (i - NMAX_ - 1) * EPS_; e < (i - NMAX_) * EPS_; ++e) { \
                    const float pv_ = __builtin_amdgcn_exp2f(fmaf(FV_SCUR(e), p.scale_log2e, -m_use_[e / 32])); \
                    lsum_[e / 32] += pv_;                                                           \
                    pnew_[2 * ((e % 32) / 16) + ((e % 16) >> 3)][e / 32][e & 7] = (__bf16)pv_;      \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        /* the interleaving the scheduler must produce: slice by slice, what the slice holds */     \
        _Pragma("unroll") for (int i = 0; i < NSL_; ++i) {                                          \
            if (i < NF_) __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);                        \
            if (i + DEPTH_ < NF_) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                \
            if (i < NMAX_) {                                                                        \
                __builtin_amdgcn_sched_group_barrier(0x002, (NE_ / NMAX_) / 2, 0);                  \
            } else if (i == NMAX_) {                                                                \
                __builtin_amdgcn_sched_group_barrier(0x002, 8 * QB, 0);                             \
                __builtin_amdgcn_sched_group_barrier(0x400, QB, 0);                                 \
            } else if ((i - NMAX_ - 1) * EPS_ < NE_) {                                              \
                __builtin_amdgcn_sched_group_barrier(0x002, EPS_, 0);                               \
                __builtin_amdgcn_sched_group_barrier(0x400, EPS_, 0);                               \
                __builtin_amdgcn_sched_group_barrier(0x002, EPS_ + EPS_ / 2, 0);                    \
            }                                                                                       \
        }                                                                                           \
        /* keep the softmax results in this basic block (otherwise the compiler sinks their */      \
        /* computation below the conditional rescale, out of reach of the interleaving) */          \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                         \
            asm volatile("" : "+v"(lsum_[qb]), "+v"(alpha_[qb]));                                   \
            _Pragma("unroll") for (int t = 0; t < 4; ++t) asm volatile("" : "+v"(pnew_[t][qb]));    \
        }                                                                                           \
        /* ---- end of iteration: running sum, rescale of O, rotate the pipeline registers */       \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                         \
            l_run[qb] = l_run[qb] * alpha_[qb] + lsum_[qb];                                         \
            if (__any(alpha_[qb] != 1.0f)) {                                                        \
                _Pragma("unroll") for (int db = 0; db < DB; ++db)                                   \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[db][qb][r] *= alpha_[qb];    \
            }                                                                                       \
            _Pragma("unroll") for (int t = 0; t < 4; ++t) pf_[t][qb] = pnew_[t][qb];                \
            if (HAS_QK_) {                                                                          \
                _Pragma("unroll") for (int kb = 0; kb < 2; ++kb) s_cur[kb][qb] = s_nxt[kb][qb];     \
            }                                                                                       \
        }                                                                                           \
    }

    // ---- schedule.  Iteration k fetches K tile k+2 and V^T tile k, and needs
    // K tile k+1 and V^T tile k-1 in LDS (two-stage rings each).
    FV_ISSUE_K(0)
    if (KT > 1) FV_ISSUE_K(1)
    FV_PUBLISH()
    FV_QK_ONLY(0, s_cur)
    FV_PUBLISH()  // stage 0 of the K ring is refilled next: every wave must be done with tile 0

    if (KT == 1) {
        FV_ISSUE_V(0)
        FV_ITER(0, false, false, true)
        if (ragged) FV_FIX_TAIL(0)
        FV_PUBLISH()
    } else {
        // iteration 0: nothing to multiply by V yet
        if (KT > 2) FV_ISSUE_K(2)
        FV_ISSUE_V(0)
        FV_ITER(0, false, true, false)
        FV_PUBLISH()
        int kt = 1;
        for (; kt + 2 < KT; ++kt) {  // steady state
            FV_ISSUE_K(kt + 2)
            FV_ISSUE_V(kt)
            FV_ITER(kt, true, true, false)
            FV_PUBLISH()
        }
        if (kt + 1 < KT) {  // iteration KT-2: no further K tile to fetch
            FV_ISSUE_V(kt)
            FV_ITER(kt, true, true, false)
            FV_PUBLISH()
            ++kt;
        }
        // iteration KT-1: last tile in the softmax (masked), no next tile
        FV_ISSUE_V(kt)
        FV_ITER(kt, true, false, true)
        if (ragged) FV_FIX_TAIL(kt)
        FV_PUBLISH()
    }
    FV_PV_ONLY(KT - 1)
#undef FV_ITER
#undef FV_SCUR
#undef FV_LOAD_FRAG
#undef FV_QK_ONLY
#undef FV_PV_ONLY
#undef FV_ISSUE_K
#undef FV_ISSUE_V
#undef FV_FIX_TAIL

    // ---- merge the key slices of a query group (exact: online-softmax partials
    // combine as m = max, l = sum l_i 2^(m_i - m), O = sum O_i 2^(m_i - m))
    if (KSPLIT > 1) {
        FV_PUBLISH()  // everyone is done with the operand tiles
        float* xch = reinterpret_cast<float*>(smem) + qg * ((DB * 16 + 2) * QB * 64);
        for (int src = 1; src < KSPLIT; ++src) {
            if (kh == src) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    float* base = xch + qb * ((DB * 16 + 2) * 64) + lane;
                    base[0] = m_run[qb];
                    base[64] = l_run[qb];
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r) base[(2 + db * 16 + r) * 64] = acc[db][qb][r];
                }
            }
            FV_PUBLISH()
            if (kh == 0) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const float* base = xch + qb * ((DB * 16 + 2) * 64) + lane;
                    const float m_o = base[0], l_o = base[64];
                    const float m_new = fmaxf(m_run[qb], m_o);
                    const float m_use = (m_new == -INFINITY) ? 0.f : m_new;
                    const float a_me = __builtin_amdgcn_exp2f(m_run[qb] - m_use);
                    const float a_o = __builtin_amdgcn_exp2f(m_o - m_use);
                    m_run[qb] = m_new;
                    l_run[qb] = l_run[qb] * a_me + l_o * a_o;
#pragma unroll
                    for (int db = 0; db < DB; ++db)
#pragma unroll
                        for (int r = 0; r < 16; ++r)
                            acc[db][qb][r] = acc[db][qb][r] * a_me + base[(2 + db * 16 + r) * 64] * a_o;
                }
            }
            if (src + 1 < KSPLIT) FV_PUBLISH()
        }
    }
#undef FV_PUBLISH

    // ---- normalise and store: lane (li, hf) register r of block db is
    // o[query li][32*db + 8*(r/4) + 4*hf + r%4]
    if (kh == 0) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const float l_tot = l_run[qb] + other_half(l_run[qb]);
            const float inv = 1.0f / l_tot;
            const int qrow = q_base + qb * 32 + li;
            if (qrow < p.k_tokens) {
                bf16_t* dst = p.o + ((size_t)b * p.k_tokens + qrow) * p.D + head * DH + 4 * hf;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2_t pk;
                        pk.x = pack_bf16x2(acc[db][qb][4 * g + 0] * inv, acc[db][qb][4 * g + 1] * inv);
                        pk.y = pack_bf16x2(acc[db][qb][4 * g + 2] * inv, acc[db][qb][4 * g + 3] * inv);
                        *reinterpret_cast<u32x2_t*>(dst + db * 32 + 8 * g) = pk;
                    }
            }
        }
    }
#endif
}

template <int DH, int QB, int QG, int KSPLIT>
void launch_cfg(const AttnParams& p, int B, hipStream_t stream) {
    constexpr size_t tile_bytes = (size_t)2 * (64 * KSPLIT * (DH / 8) + DH * (8 * KSPLIT)) * 16;
    constexpr size_t merge_bytes = KSPLIT > 1 ? (size_t)QG * (DH / 32 * 16 + 2) * QB * 64 * 4 : 0;
    constexpr size_t smem = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
    static bool attr_set = false;
    if (!attr_set) {
        (void)hipFuncSetAttribute(reinterpret_cast<const void*>(&attention_kernel<DH, QB, QG, KSPLIT>),
                                  hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        attr_set = true;
    }
    const int per_wg = QG * 32 * QB;
    attention_kernel<DH, QB, QG, KSPLIT>
        <<<dim3((p.k_tokens + per_wg - 1) / per_wg, p.H, B), QG * KSPLIT * 64, smem, stream>>>(p);
}

int attn_cfg_override() {
    static int v = -2;
    if (v == -2) {
        const char* e = getenv("FASTVAR_ATTN_CFG");
        v = e ? atoi(e) : -1;
    }
    return v;
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
    // One wave per 64 queries; when that leaves SIMDs idle (fewer than ~1 wave per
    // SIMD on 256 CUs), split the keys of each tile over two waves instead.
    const long waves = (long)((a.k_tokens + 63) / 64) * a.H * a.B;
    int cfg = waves >= 900 ? 0 : 1;
    if (attn_cfg_override() >= 0) cfg = attn_cfg_override();
    if (a.dh == 128) {
        switch (cfg) {
            case 0: launch_cfg<128, 2, 4, 1>(p, a.B, stream); break;
            case 1: launch_cfg<128, 2, 2, 2>(p, a.B, stream); break;
            case 2: launch_cfg<128, 1, 4, 1>(p, a.B, stream); break;
            case 3: launch_cfg<128, 1, 2, 2>(p, a.B, stream); break;
            default: launch_cfg<128, 1, 4, 2>(p, a.B, stream); break;
        }
    } else {
        switch (cfg) {
            case 0: launch_cfg<64, 2, 4, 1>(p, a.B, stream); break;
            case 1: launch_cfg<64, 2, 2, 2>(p, a.B, stream); break;
            case 2: launch_cfg<64, 1, 4, 1>(p, a.B, stream); break;
            case 3: launch_cfg<64, 1, 2, 2>(p, a.B, stream); break;
            default: launch_cfg<64, 1, 4, 2>(p, a.B, stream); break;
        }
    }
}

}  // namespace fv
