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

// XOR key that spreads the 16-byte chunks of consecutive rows over all 64 LDS
// banks (256 bytes): a 16-byte-per-lane read is served 16 lanes at a time, so 16
// consecutive rows must land in 16 different chunk columns.  Rows of 256 bytes
// (16 chunks) use the low 4 row bits; rows of 128 bytes (8 chunks, two rows per
// bank sweep) use row bits 1-3.
template <int CPR>
__device__ __forceinline__ int chunk_key(int row) {
    static_assert(CPR == 8 || CPR == 16, "rows of 128 or 256 bytes");
    return CPR == 16 ? (row & 15) : ((row >> 1) & 7);
}

#ifndef ATTN_SPAN_FULL
#define ATTN_SPAN_FULL 0
#endif
#ifndef ATTN_VF_SPLIT
#define ATTN_VF_SPLIT 0
#endif
constexpr int attn_waitcnt(int vm, bool lgkm) {
    return (vm & 0xF) | ((vm >> 4) << 14) | (0x7 << 4) | ((lgkm ? 0x0 : 0xF) << 8);
}

template <int DH, int QB, int QG, int KSPLIT>
__global__ __launch_bounds__(QG * KSPLIT * 64, (QB == 1 ? 2 : 1)) void attention_kernel(const AttnParams p) {
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
    const int sw_k = chunk_key<DH / 8>(lane & 31);          // swizzle keys of this lane's operand rows
    const int sw_v = chunk_key<8 * KSPLIT>(lane & 31);
    // Workgroup -> (query tile, head, sample).  Consecutive workgroup ids are dealt
    // round-robin to the 8 XCDs, each with its own L2; undo that so an XCD works on
    // a contiguous run of (head, query tile) pairs: the workgroups that stream the
    // same head's K / V then share one L2 instead of pulling it into all eight.
    int wg = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int n_wg = gridDim.x * gridDim.y * gridDim.z;
    if ((n_wg & 7) == 0) wg = (wg & 7) * (n_wg >> 3) + (wg >> 3);
    const int q_tile = wg % gridDim.x;
    const int head = (wg / gridDim.x) % gridDim.y;
    const int b = wg / (gridDim.x * gridDim.y);
    const int q_base = q_tile * (QG * 32 * QB) + qg * (32 * QB);

    const bf16_t* kc = p.kc + ((size_t)b * p.H + head) * p.L_cap * DH;
    const bf16_t* vc = p.vc + ((size_t)b * p.H + head) * DH * (size_t)p.L_cap;

    const int KT = (p.L + BN - 1) / BN;
    const bool ragged = (p.L % BN) != 0;

    // ---- per-lane byte offsets of the direct-to-LDS loads, relative to the start of
    // a tile (K: key row kt*BN of this head; V^T: cache position kt*BN of row 0).
    // Load j of this wave is instruction ij = wave + WAVES*j of the tile; it fills
    // 1 KB of LDS, lane l landing at chunk 64*ij + l.  The offsets are the same for
    // every full tile (the scalar base pointer advances), so a load costs no vector
    // arithmetic; the last tile has its own set, clamped to the valid length.
    uint32_t k_off[K_LD], k_off_last[K_LD], v_off[V_LD], v_off_last[V_LD];
    int v_col[V_LD];  // key offset inside the tile of this lane's V^T chunk
    {
        const int last_chunk = ((p.L - 1) >> 3) << 3;  // start of the last 8-key run that holds a valid key
        const int key_last0 = (KT - 1) * BN;
#pragma unroll
        for (int j = 0; j < K_LD; ++j) {
            const int slot = (wave + WAVES * j) * K_RPI + lane / KCH;  // LDS row
            const int c = (lane % KCH) ^ chunk_key<KCH>(slot);         // logical chunk stored at this position
            const int key = (slot & ~31) | swap_bits_2_3(slot & 31);   // key inside the tile
            k_off[j] = (uint32_t)(key * DH + c * 8) * 2u;
            k_off_last[j] = (uint32_t)((min(key_last0 + key, p.L - 1) - key_last0) * DH + c * 8) * 2u;
        }
#pragma unroll
        for (int j = 0; j < V_LD; ++j) {
            const int d = (wave + WAVES * j) * V_RPI + lane / VCH;     // V^T row
            const int c = (lane % VCH) ^ chunk_key<VCH>(d);
            v_col[j] = c * 8;
            v_off[j] = (uint32_t)(d * p.L_cap + c * 8) * 2u;
            v_off_last[j] = (uint32_t)(d * p.L_cap + min(key_last0 + c * 8, last_chunk) - key_last0) * 2u;
        }
    }

    // K tiles and V^T tiles live in separate two-stage rings: the second MFMA of
    // a tile is deferred to the next iteration (see the schedule below), so
    // iteration k consumes K tile k and V^T tile k-1.
    //
    // The loads are written as inline assembly on purpose: after the compiler's own
    // direct-to-LDS builtin it drains the whole LDS queue (lgkmcnt(0)) before the
    // next operand use, which would undo the read-ahead of the matrix phase.
    // Completion is tracked by hand: every path waits for vmcnt(0) before the
    // barrier that publishes the tile.
#define FV_DMA16(base_, off_, lds_chunk_ptr_)                                                       \
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"                                \
                 :                                                                                  \
                 : "s"((uint32_t)(uintptr_t)(lds_ptr_t)(lds_chunk_ptr_)), "v"(off_), "s"(base_)    \
                 : "memory", "m0")
    // The same load, pinned in the instruction stream: it takes a register of the
    // surrounding arithmetic as a pass-through operand, so it is scheduled after
    // that value's producer and before its consumers.
#define FV_DMA16_AT(base_, off_, lds_chunk_ptr_, reg_)                                              \
    asm volatile("s_mov_b32 m0, %1\n\tglobal_load_lds_dwordx4 %2, %3"                                \
                 : "+v"(reg_)                                                                       \
                 : "s"((uint32_t)(uintptr_t)(lds_ptr_t)(lds_chunk_ptr_)), "v"(off_), "s"(base_)    \
                 : "memory", "m0")
    // One of this wave's loads (j_ in [0, K_LD + V_LD): K rows of tile ktk_ first, then
    // V^T rows of tile ktv_)
#define FV_ISSUE_ONE_AT(ktk_, ktv_, j_, reg_)                                                       \
    {                                                                                               \
        if ((j_) < K_LD) {                                                                          \
            const int jk_ = (j_) < K_LD ? (j_) : 0;                                                 \
            const uint32_t off_ = ((ktk_) == KT - 1) ? k_off_last[jk_] : k_off[jk_];                \
            FV_DMA16_AT(kc + (size_t)(ktk_) * (BN * DH), off_,                                      \
                        lds + ((ktk_) & 1) * K_TILE + wave * 64 + jk_ * (WAVES * 64), reg_);        \
        } else {                                                                                    \
            const int jv_ = (j_) >= K_LD ? (j_) - K_LD : 0;                                         \
            const uint32_t off_ = ((ktv_) == KT - 1) ? v_off_last[jv_] : v_off[jv_];                \
            FV_DMA16_AT(vc + (size_t)(ktv_) * BN, off_,                                             \
                        lds + 2 * K_TILE + ((ktv_) & 1) * V_TILE + wave * 64 + jv_ * (WAVES * 64), reg_); \
        }                                                                                           \
    }
#define FV_ISSUE_ONE(ktk_, ktv_, j_)                                                                \
    {                                                                                               \
        if ((j_) < K_LD) {                                                                          \
            const int jk_ = (j_) < K_LD ? (j_) : 0;                                                 \
            const uint32_t off_ = ((ktk_) == KT - 1) ? k_off_last[jk_] : k_off[jk_];                \
            FV_DMA16(kc + (size_t)(ktk_) * (BN * DH), off_,                                         \
                     lds + ((ktk_) & 1) * K_TILE + wave * 64 + jk_ * (WAVES * 64));                 \
        } else {                                                                                    \
            const int jv_ = (j_) >= K_LD ? (j_) - K_LD : 0;                                         \
            const uint32_t off_ = ((ktv_) == KT - 1) ? v_off_last[jv_] : v_off[jv_];                \
            FV_DMA16(vc + (size_t)(ktv_) * BN, off_,                                                \
                     lds + 2 * K_TILE + ((ktv_) & 1) * V_TILE + wave * 64 + jv_ * (WAVES * 64));    \
        }                                                                                           \
    }
#define FV_ISSUE_K(kt_) _Pragma("unroll") for (int j = 0; j < K_LD; ++j) FV_ISSUE_ONE(kt_, 0, j)
#define FV_ISSUE_V(kt_) _Pragma("unroll") for (int j = K_LD; j < K_LD + V_LD; ++j) FV_ISSUE_ONE(0, kt_, j)
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

    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16_t s_[2][QB];   // scores of this wave's 64-key slice (two 32-key blocks)
    bf16x8_t pf_[4][QB];  // probabilities as the B operand of the second MFMA (four 16-key steps)

    // Matrix phase of iteration kt_: O^T += V^T P^T for tile kt_-1 (if HAS_PV_),
    // then S^T = K Q^T for tile kt_, on this wave's 64-key slice.  All operand
    // fragments come from LDS; their reads run DEPTH fragments ahead of the MFMAs
    // that consume them (the scheduler is given the interleaving explicitly), so
    // LDS latency hides behind the matrix pipe.  Consecutive MFMAs alternate
    // accumulators.
#define FV_MATRIX(kt_, HAS_PV_, LOAD_K_, LOAD_V_)                                                   \
    {                                                                                               \
        constexpr int NV_ = (HAS_PV_) ? 4 * DB : 0;                                                 \
        constexpr int NK_ = 2 * KS;                                                                 \
        constexpr int DEPTH_ = 4;                                                                   \
        /* The next tiles' direct-to-LDS loads (K tile kt_+1, V^T tile kt_) are issued */           \
        /* between the operand reads below: program order against LDS reads is kept, so */          \
        /* they end up spread between the MFMAs instead of queueing up in front of them. */         \
        constexpr int JLO_ = (LOAD_K_) ? 0 : K_LD;                                                  \
        constexpr int JHI_ = (LOAD_V_) ? K_LD + V_LD : K_LD;                                        \
        constexpr int NJ_ = JHI_ > JLO_ ? JHI_ - JLO_ : 0;                                          \
        constexpr int NFR_ = NV_ + NK_;                                                             \
        constexpr int SPAN_ = (ATTN_SPAN_FULL || NJ_ > NFR_ / 2) ? NFR_ : NFR_ / 2;                 \
        const u32x4_t* v_base_ = lds + 2 * K_TILE + (((kt_) + 1) & 1) * V_TILE;                     \
        const u32x4_t* k_base_ = lds + ((kt_) & 1) * K_TILE + (kh * 64) * KCH;                      \
        bf16x8_t fr_[NV_ + NK_];                                                                    \
        _Pragma("unroll") for (int i = 0; i < NFR_; ++i) {                                          \
            if (i < NV_)                                                                            \
                fr_[i] = *reinterpret_cast<const bf16x8_t*>(                                        \
                    v_base_ + ((i % DB) * 32 + li) * VCH + ((kh * 8 + 2 * (i / DB) + hf) ^ sw_v));  \
            else                                                                                    \
                fr_[i] = *reinterpret_cast<const bf16x8_t*>(                                        \
                    k_base_ + (((i - NV_) % 2) * 32 + li) * KCH + ((2 * ((i - NV_) / 2) + hf) ^ sw_k)); \
            /* the loads go between the first SPAN_ fragment reads, evenly: early enough */       \
            /* to land before the end-of-iteration barrier */                                       \
            if (NJ_ > 0 && i < SPAN_ && ((i + 1) * NJ_) / SPAN_ > (i * NJ_) / SPAN_)                \
                FV_ISSUE_ONE((kt_) + 1, (kt_), JLO_ + (i * NJ_) / SPAN_)                            \
        }                                                                                           \
        if (HAS_PV_) {                                                                              \
            _Pragma("unroll") for (int t = 0; t < 4; ++t)                                           \
                _Pragma("unroll") for (int db = 0; db < DB; ++db)                                   \
                    _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                               \
                        acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                      \
                            fr_[t * DB + db], pf_[t][qb], acc[db][qb], 0, 0, 0);                    \
        }                                                                                           \
        _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                           \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    s_[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                           \
                        fr_[NV_ + ks * 2 + kb], qf[qb][ks], ks == 0 ? zero16 : s_[kb][qb], 0, 0, 0); \
        __builtin_amdgcn_sched_group_barrier(0x100, DEPTH_, 0);                                     \
        _Pragma("unroll") for (int i = 0; i < NV_ + NK_ - DEPTH_; ++i) {                            \
            __builtin_amdgcn_sched_group_barrier(0x008, QB, 0);                                     \
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                      \
        }                                                                                           \
        __builtin_amdgcn_sched_group_barrier(0x008, DEPTH_ * QB, 0);                                \
    }
    // O^T += V^T P^T alone (after the last tile)
#define FV_PV_LAST(kt_)                                                                             \
    {                                                                                               \
        const u32x4_t* v_base_ = lds + 2 * K_TILE + ((kt_) & 1) * V_TILE;                           \
        _Pragma("unroll") for (int t = 0; t < 4; ++t)                                               \
            _Pragma("unroll") for (int db = 0; db < DB; ++db) {                                     \
                const bf16x8_t vf_ = *reinterpret_cast<const bf16x8_t*>(                            \
                    v_base_ + (db * 32 + li) * VCH + ((kh * 8 + 2 * t + hf) ^ sw_v));               \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                                   \
                    acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf_, pf_[t][qb], acc[db][qb], 0, 0, 0); \
            }                                                                                       \
    }
    // online softmax of the scores of tile kt_: s_ -> pf_, running max / sum, rescale of O.
    // LOAD_K_ / LOAD_V_: this wave's loads of K tile ktl_+1 / V^T tile ktl_ are issued
    // from inside the exponential loop, one every few elements, instead of in a burst
    // (a burst from several waves at once fills the texture-address queue and the
    // waves sit in it).  The wave raises its issue priority for the duration: its
    // many short vector instructions then win the issue slot over the matrix-phase
    // wave sharing the SIMD, which needs one slot per 32-cycle MFMA only.
#define FV_SOFTMAX(kt_, MASK_, LOAD_K_, LOAD_V_, ktl_)                                              \
    {                                                                                               \
        __builtin_amdgcn_s_setprio(1);                                                              \
        constexpr int JLO_ = (LOAD_K_) ? 0 : K_LD;                                                  \
        constexpr int JHI_ = (LOAD_V_) ? K_LD + V_LD : K_LD;                                        \
        constexpr int NJ_ = JHI_ > JLO_ ? JHI_ - JLO_ : 0;                                          \
        constexpr int EVERY_ = NJ_ > 0 ? (32 / NJ_ > 0 ? 32 / NJ_ : 1) : 1;                         \
        static_assert(NJ_ <= 32, "at most one load per score element");                             \
        if (MASK_) {                                                                                \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                    \
                    const int srow_ = 8 * (r >> 2) + 4 * hf + (r & 3);                              \
                    const int key_ = (kt_) * BN + kh * 64 + kb * 32 + swap_bits_2_3(srow_);         \
                    if (key_ >= p.L) {                                                              \
                        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) s_[kb][qb][r] = -INFINITY; \
                    }                                                                               \
                }                                                                                   \
        }                                                                                           \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                         \
            float mx_ = s_[0][qb][0];                                                               \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) mx_ = fmaxf(mx_, s_[kb][qb][r]);     \
            mx_ = fmaxf(mx_, other_half(mx_));                                                      \
            /* a slice that is entirely past the length keeps the old maximum */                   \
            const float m_new_ = fmaxf(m_run[qb], mx_ * p.scale_log2e);                             \
            const float m_use_ = (m_new_ == -INFINITY) ? 0.f : m_new_;                              \
            const float alpha_ = __builtin_amdgcn_exp2f(m_run[qb] - m_use_);                        \
            m_run[qb] = m_new_;                                                                     \
            float lsum_ = 0.f;                                                                      \
            _Pragma("unroll") for (int kb = 0; kb < 2; ++kb)                                        \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                    \
                    float pv_ = __builtin_amdgcn_exp2f(fmaf(s_[kb][qb][r], p.scale_log2e, -m_use_)); \
                    const int e_ = kb * 16 + r;                                                     \
                    if (qb == 0 && NJ_ > 0 && e_ % EVERY_ == 0 && e_ / EVERY_ < NJ_)                \
                        FV_ISSUE_ONE_AT((ktl_) + 1, (ktl_), JLO_ + e_ / EVERY_, pv_)                \
                    pf_[2 * kb + (r >> 3)][qb][r & 7] = (__bf16)pv_;                                \
                    lsum_ += pv_;                                                                   \
                }                                                                                   \
            l_run[qb] = l_run[qb] * alpha_ + lsum_;                                                 \
            if (__any(alpha_ != 1.0f)) {                                                            \
                _Pragma("unroll") for (int db = 0; db < DB; ++db)                                   \
                    _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[db][qb][r] *= alpha_;        \
            }                                                                                       \
        }                                                                                           \
        __builtin_amdgcn_s_setprio(0);                                                              \
    }
    // ---- schedule.  Iteration k fetches K tile k+1 and V^T tile k and needs
    // K tile k and V^T tile k-1.  Every wave does, per tile, a matrix phase
    // (PV of the previous tile, then QK of this one) and a vector phase (softmax
    // of this tile).  With two waves per SIMD (8-wave workgroups) the waves of
    // the second half run the phases in the opposite order, so that on every SIMD
    // one wave is in its matrix phase while the other is in its vector phase
    // (both start each iteration together at the barrier).
    const bool vector_first = (WAVES == 8) && (wave >= 4);

    FV_ISSUE_K(0)
    FV_PUBLISH()

    if (!vector_first) {
        // iteration 0
        if (KT > 1) { FV_MATRIX(0, false, true, true) } else { FV_MATRIX(0, false, false, true) }
        if (KT == 1) { FV_SOFTMAX(0, true, false, false, 0) } else { FV_SOFTMAX(0, false, false, false, 0) }
        if (KT == 1 && ragged) FV_FIX_TAIL(0)
        FV_PUBLISH()
        int kt = 1;
        for (; kt + 1 < KT; ++kt) {
            FV_MATRIX(kt, true, true, true)
            FV_SOFTMAX(kt, false, false, false, 0)
            FV_PUBLISH()
        }
        if (kt < KT) {  // last tile
            FV_MATRIX(kt, true, false, true)
            FV_SOFTMAX(kt, true, false, false, 0)
            if (ragged) FV_FIX_TAIL(kt)
            FV_PUBLISH()
        }
        FV_PV_LAST(KT - 1)
    } else {
        // vector-first waves fetch at the start of the iteration (their matrix phase
        // comes last, right before the barrier)
        if (KT > 1) { FV_MATRIX(0, false, true, true) } else { FV_MATRIX(0, false, false, true) }
        if (KT == 1 && ragged) FV_FIX_TAIL(0)
        FV_PUBLISH()
        int kt = 1;
        for (; kt + 1 < KT; ++kt) {
            if (ATTN_VF_SPLIT) {
                FV_SOFTMAX(kt - 1, false, true, false, kt)
                FV_MATRIX(kt, true, false, true)
            } else {
                FV_SOFTMAX(kt - 1, false, true, true, kt)
                FV_MATRIX(kt, true, false, false)
            }
            FV_PUBLISH()
        }
        if (kt < KT) {  // last tile
            FV_SOFTMAX(kt - 1, false, false, true, kt)
            FV_MATRIX(kt, true, false, false)
            if (ragged) FV_FIX_TAIL(kt)
            FV_PUBLISH()
        }
        FV_SOFTMAX(KT - 1, true, false, false, 0)
        FV_PV_LAST(KT - 1)
    }
#undef FV_MATRIX
#undef FV_PV_LAST
#undef FV_SOFTMAX
#undef FV_ISSUE_K
#undef FV_ISSUE_ONE
#undef FV_ISSUE_ONE_AT
#undef FV_DMA16_AT
#undef FV_DMA16
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
    // One wave per 32 queries, two waves per SIMD: with enough queries two 4-wave
    // workgroups share a CU; otherwise an 8-wave workgroup splits the keys of each
    // tile between two waves per query group.
    const long waves = (long)((a.k_tokens + 31) / 32) * a.H * a.B;
    int cfg = waves >= 1800 ? 2 : 4;
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
