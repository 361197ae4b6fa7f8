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

// Every query tile's counters have a 128-byte line of their own: the workgroups of different tiles count and
// poll at the same time, and atomics on one line are served one after the other.
constexpr int kCounterStride = 32;

struct AttnParams {
    const bf16_t* q;
    const bf16_t* kc;
    const bf16_t* vc;
    bf16_t* o;
    int H, k_tokens, L, L_cap, D;
    float scale_log2e;
    // key-range split between workgroups (pipelined kernel instantiated with KVS): of the launch's
    // (sample, head, query tile) triples, counted in that order, the first full_tiles are walked whole by
    // one workgroup each; each of the other tail_tiles is shared by `splits` workgroups
    int q_tiles, splits, keys_per_split, full_tiles, tail_tiles;
    float* part;   // [tail tile][split][1 + DB*QB*4 vectors][QG*64 lanes][4] fp32
    int* split_cnt;   // [tail tile][kCounterStride] arrival counters, zero between launches
    int* split_ready; // [tail tile][kCounterStride] ranges whose partial result is complete in memory, zero between launches
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
        constexpr int SPAN_ = (NJ_ > NFR_ / 2) ? NFR_ : NFR_ / 2;                                   \
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
            FV_SOFTMAX(kt - 1, false, true, true, kt)
            FV_MATRIX(kt, true, false, false)
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

// ---------------------------------------------------------------------------------------------
// Software-pipelined variant for long key sequences (L > 2 tiles): one wave per SIMD owns 64
// queries, so every K / V^T fragment read from LDS feeds two MFMAs, and the softmax of one
// 32-key block is interleaved, inside the same wave, with the MFMAs of its neighbours:
//   step s:  softmax(block s)   |   S(block s+1) = K Q^T   |   O^T += V^T P^T (block s-1)
// About four vector instructions fit in the shadow of one 32-cycle MFMA, which is what the
// softmax of a 32x64 block needs per MFMA of the two products around it.  Scores and
// probabilities are double buffered by name (two instantiations of the step), a wave's 64-key
// slice of a tile is two steps, and there is one barrier per tile, between the two steps:
// it publishes K tile kt+1 and V^T tile kt (fetched during the previous tile's second step) and
// frees K tile kt and V^T tile kt-1, whose stages the second step refills.
// The last tile is shifted back so that it ends at the (8-aligned) end of the cache: it never
// reads past L_cap, its leading keys (already seen) and the up to 7 positions past L are masked.
// KVS: the key range is also split between workgroups (consecutive query-tile ids of the grid's x
// dimension are the same tile's splits); each works on keys [split*keys_per_split, ...) as if they
// were the whole cache; the workgroup that arrives last at the tile merges the ranges, the others leave
// their unnormalised output and statistics for it.
template <int DH, int QG, int KSPLIT, bool KVS = false>
__global__ __launch_bounds__(QG * KSPLIT * 64, 1) void attention_pipe_kernel(const AttnParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int QB = 2;
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
    static_assert(K_LD >= 1 && V_LD >= 1 && K_LD + V_LD <= 2 * DB + KS, "one load per operand read at most");
    static_assert(WAVES * K_RPI % 32 == 0 || WAVES * K_RPI == 16, "key rows of a wave's loads must differ by a constant");

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
    const int sw_k = chunk_key<KCH>(li);
    const int sw_v = chunk_key<VCH>(li);
    int wg = blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
    const int n_wg = gridDim.x * gridDim.y * gridDim.z;
    if ((n_wg & 7) == 0) wg = (wg & 7) * (n_wg >> 3) + (wg >> 3);  // XCD-aware order, as above
    int q_tile = wg % gridDim.x, head = (wg / gridDim.x) % gridDim.y, b = wg / (gridDim.x * gridDim.y);
    int split = 0, nsp = 1, tail_idx = 0;   // key range, ranges of this tile, index among the shared tiles
    if (KVS) {
        // a one-dimensional launch: full_tiles workgroups that walk all keys of their tile, then `splits`
        // workgroups for each of the other tiles, range by range (the tiles of a head, which share its
        // K / V, stay next to each other in both parts, and each part is dealt to the XCDs in runs)
        const int F = p.full_tiles, R = p.tail_tiles;
        const int lin = blockIdx.x;
        int t;
        if (lin < F) {
            t = (F & 7) == 0 ? (lin & 7) * (F >> 3) + (lin >> 3) : lin;
        } else {
            const int n = R * p.splits;
            int r = lin - F;
            if ((n & 7) == 0) r = (r & 7) * (n >> 3) + (r >> 3);
            split = r / R;
            tail_idx = r - split * R;
            t = F + tail_idx;
            nsp = p.splits;
        }
        q_tile = t % p.q_tiles;
        head = (t / p.q_tiles) % p.H;
        b = t / (p.q_tiles * p.H);
    }
    const int q_base = q_tile * (QG * 32 * QB) + qg * (32 * QB);
    const int key_first = (KVS && nsp > 1) ? split * p.keys_per_split : 0;    // a multiple of the key tile
    const int L = (KVS && nsp > 1) ? min(p.L - key_first, p.keys_per_split) : p.L;   // keys of this workgroup

    const bf16_t* kc = p.kc + (((size_t)b * p.H + head) * p.L_cap + key_first) * DH;
    const bf16_t* vc = p.vc + ((size_t)b * p.H + head) * DH * (size_t)p.L_cap + key_first;

    const int KT = (L + BN - 1) / BN;                   // >= 3, checked by the launcher
    const int last_start = ((L + 7) & ~7) - BN;         // first key of the shifted last tile
    const int last_first_new = (KT - 1) * BN;           // keys before this one were seen in tile KT-2
#define FP_TILE_START(kt_) ((kt_) == KT - 1 ? last_start : (kt_) * BN)

    // Per-lane byte offsets of this wave's loads inside a tile; load j adds a scalar constant.
    uint32_t k_off0, v_off0;
    int v_col0;   // key offset inside the tile of this lane's V^T chunk (the same for every load)
    {
        const int slot = wave * K_RPI + lane / KCH;
        const int c = (lane % KCH) ^ chunk_key<KCH>(slot);
        const int key = (slot & ~31) | swap_bits_2_3(slot & 31);
        k_off0 = (uint32_t)(key * DH + c * 8) * 2u;
        const int d = wave * V_RPI + lane / VCH;
        const int cv = (lane % VCH) ^ chunk_key<VCH>(d);
        v_col0 = cv * 8;
        v_off0 = (uint32_t)(d * p.L_cap + cv * 8) * 2u;
    }
#define FP_DMA16(base_, off_, lds_chunk_ptr_)                                                       \
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"                                \
                 :                                                                                  \
                 : "s"((uint32_t)(uintptr_t)(lds_ptr_t)(lds_chunk_ptr_)), "v"(off_), "s"(base_)    \
                 : "memory", "m0")
    // load j_ of this wave: K rows of tile ktk_ for j_ < K_LD, then V^T rows of tile ktv_
#define FP_ISSUE_ONE(ktk_, ktv_, j_)                                                                \
    {                                                                                               \
        if ((j_) < K_LD) {                                                                          \
            FP_DMA16(kc + ((size_t)FP_TILE_START(ktk_) + (j_) * (WAVES * K_RPI)) * DH, k_off0,      \
                     lds + ((ktk_) & 1) * K_TILE + wave * 64 + (j_) * (WAVES * 64));                \
        } else {                                                                                    \
            FP_DMA16(vc + (size_t)((j_) - K_LD) * (WAVES * V_RPI) * p.L_cap + FP_TILE_START(ktv_), v_off0, \
                     lds + 2 * K_TILE + ((ktv_) & 1) * V_TILE + wave * 64 + ((j_) - K_LD) * (WAVES * 64)); \
        }                                                                                           \
    }
    // zero the V^T LDS positions of tile KT-1 that lie at or past the length (they may hold NaN
    // patterns and 0 * NaN would poison the output); own loads have landed (vmcnt(0) before)
#define FP_FIX_TAIL()                                                                               \
    {                                                                                               \
        u32x4_t* sv_ = lds + 2 * K_TILE + ((KT - 1) & 1) * V_TILE + wave * 64 + lane;               \
        const int valid_ = L - (last_start + v_col0);                                             \
        if (valid_ < 8) {                                                                           \
            _Pragma("unroll") for (int j = 0; j < V_LD; ++j) {                                      \
                u32x4_t v_ = sv_[j * (WAVES * 64)];                                                 \
                v_.x = valid_ >= 2 ? v_.x : (valid_ >= 1 ? (v_.x & 0xFFFFu) : 0u);                  \
                v_.y = valid_ >= 4 ? v_.y : (valid_ >= 3 ? (v_.y & 0xFFFFu) : 0u);                  \
                v_.z = valid_ >= 6 ? v_.z : (valid_ >= 5 ? (v_.z & 0xFFFFu) : 0u);                  \
                v_.w = valid_ >= 7 ? (v_.w & 0xFFFFu) : 0u;                                         \
                sv_[j * (WAVES * 64)] = v_;                                                         \
            }                                                                                       \
        }                                                                                           \
    }
#define FP_PUBLISH()                                                                                \
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

    const f32x16_t zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    f32x16_t acc[DB][QB];
    float m_run[QB], l_run[QB];
    f32x16_t sa_[QB], sb_[QB];        // scores of two consecutive 32-key blocks
    bf16x8_t pa_[2][QB], pb_[2][QB];  // their probabilities as B operands (two 16-key steps each)
    bf16x8_t fe_[16], fo_[16];        // operand fragments of the first / second step of a tile

    // S = K Q^T accumulates in vector registers (the softmax reads it there); the MFMA is written
    // as inline assembly because the compiler's own form of it, in a kernel this large, puts every
    // MFMA result in the accumulator file and copies it out again for the vector unit.
    // The query operand is taken from the accumulator file (it is used by these MFMAs only, and the
    // 64 registers it would occupy are what the vector file is short of).
    // The leading wait states stand in for the ones the compiler inserts before its own MFMAs
    // (it cannot see through the assembly: without them the results are wrong); they cost nothing,
    // the wave is waiting for the matrix pipe at that point anyway.
#define FP_MFMA_S0(S_, a_, b_) \
    asm("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, 0" : "=&v"(S_) : "v"(a_), "a"(b_))
#define FP_MFMA_S(S_, a_, b_) \
    asm("s_nop 1\n\tv_mfma_f32_32x32x16_bf16 %0, %1, %2, %0" : "+v"(S_) : "v"(a_), "a"(b_))

    // The exponentials of a block are numbered e = 16*qb + r (32 per step).  A half-group starts
    // one or two of them (multiply-add), takes the exp2 of those the half-group before it started
    // and consumes the ones before that (row-sum add; bf16 pack once a pair is complete): the wave
    // issues in order, so a value must not be used in the half-group that computes it.
    // (each value is pinned where it is computed: the optimiser would otherwise sink the packs and
    // the row-sum adds to the end of the step, out of the MFMAs' shadow and with 32 values alive)
#define FP_ARG(S_, e_)                                                                              \
    px_[e_] = fmaf(S_[(e_) / 16][(e_) % 16], p.scale_log2e, -m_use_[(e_) / 16]);                    \
    asm volatile("" : "+v"(px_[e_]));
#define FP_EXP(e_)                                                                                  \
    pe_[e_] = __builtin_amdgcn_exp2f(px_[e_]);                                                      \
    asm volatile("" : "+v"(pe_[e_]));
#define FP_CONSUME(P_, e_)                                                                          \
    {                                                                                               \
        lsum_[(e_) / 16] += pe_[e_];                                                                \
        asm volatile("" : "+v"(lsum_[(e_) / 16]));                                                  \
        if ((e_) % 2 == 1) {                                                                        \
            uint32_t pk_ = pack_bf16x2(pe_[(e_) - 1], pe_[e_]);                                     \
            asm volatile("" : "+v"(pk_));                                                           \
            pw_[((e_) / 16) * 8 + ((e_) % 16) / 2] = pk_;                                           \
        }                                                                                           \
    }
    // Half-group hh_ (two per group, 2 * NG_ per step) starts elements [FP_E0(hh_), FP_E0(hh_+1)) of the
    // 32.  With the running maximum the first eight half-groups are busy with the maxima and the
    // elements are spread over the others (16 groups: 2,1,1,2,...; 8 groups: four each); in fast mode
    // every half-group starts the same number (one or two).
#define FP_E0(RESC_, hh_)                                                                           \
    ((hh_) < 0 ? 0                                                                                  \
     : (RESC_) ? ((hh_) < 8 ? 0                                                                     \
                  : NG_ == 16 ? ((hh_) - 8) + (((hh_) - 8) + 2) / 3                                 \
                              : (((hh_) - 8) * 4 > 32 ? 32 : ((hh_) - 8) * 4))                      \
               : ((hh_) * (16 / NG_) > 32 ? 32 : (hh_) * (16 / NG_)))
#define FP_HALF(RESC_, S_, P_, hh_)                                                                 \
    {                                                                                               \
        constexpr int x0_ = FP_E0(RESC_, hh_), x1_ = FP_E0(RESC_, (hh_) + 1);                       \
        constexpr int e0_ = FP_E0(RESC_, (hh_) - 1), e1_ = x0_;                                     \
        constexpr int c0_ = FP_E0(RESC_, (hh_) - 2), c1_ = e0_;                                     \
        static_for<x0_, x1_>([&](auto e_c) { constexpr int e = decltype(e_c)::value; FP_ARG(S_, e) }); \
        static_for<e0_, e1_>([&](auto e_c) { constexpr int e = decltype(e_c)::value; FP_EXP(e) });  \
        static_for<c0_, c1_>([&](auto e_c) { constexpr int e = decltype(e_c)::value; FP_CONSUME(P_, e) }); \
    }
    // One step.  S_SM_/P_SM_: block whose softmax is taken (scores in, probabilities out; first key
    // key0_sm_, MASK_ for blocks of the last tile).  DO_QK_: S_QK_ = K Q^T for the 32 key rows at
    // kbase_.  DO_PV_: O^T += V^T P^T with P_PV_ and the V^T chunks vchunk0_ .. +3 of the tile at
    // vbase_.  LOAD_K_ / LOAD_V_: this wave's loads of K tile ktk_ / V^T tile ktv_ go out, one per
    // group.  The step is written as 16 groups that the scheduler may not mix: two MFMAs (one
    // operand fragment, both query blocks), the read of the fragment DEPTH groups ahead, one load,
    // and a slice of the softmax: groups 0-3 take the row maxima (masking first where needed),
    // groups 4-15 the exponentials, two at a time.
    // RESC_ = true: online softmax with a running maximum; the output accumulator is rescaled under
    // a branch when the maximum moves.  RESC_ = false (fast mode): the maximum stays where the first
    // tile left it (softmax is shift invariant; fp32 has the range), so there are no maxima to take,
    // the step is branch free and the accumulator never leaves the accumulator file.  Should a later
    // score exceed the reference by so much that exp2 endangers the fp32 range, the row sum shows it
    // and the caller repeats the whole computation with RESC_ = true.
    // group g_ of a step (a literal, so that every index below is a compile-time constant)
#define FP_G(g_, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, \
             LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_)           \
    if constexpr ((g_) < NG_) {                                                                     \
        constexpr int gg = (g_);                                                                    \
        constexpr int f = gg + DEPTH_;      /* operand fragment read in this group */               \
        if ((BAR_) && gg == NG_ - DEPTH_) {                                                         \
            /* every read of the old tiles has been issued: publish the tiles fetched during the */ \
            /* previous step, free the old ones (the next step's first operands come from the new) */ \
            asm volatile("" ::: "memory");                                                          \
            __builtin_amdgcn_s_waitcnt(attn_waitcnt(0, true));                                      \
            if ((MASK_) && ((L & 7) != 0)) FP_FIX_TAIL()                                          \
            FP_PUBLISH()                                                                            \
        }                                                                                           \
        if (f < NV_ && (DO_PV_))                                                                    \
            FR_[f < NV_ ? f : 0] = *reinterpret_cast<const bf16x8_t*>(                              \
                (vbase_) + ((f % DB) * 32 + li) * VCH + (((vchunk0_) + 2 * (f / DB) + hf) ^ sw_v)); \
        if (f >= NV_ && f < NG_ && (DO_QK_))                                                        \
            FR_[f < NG_ ? f : 0] = *reinterpret_cast<const bf16x8_t*>(                              \
                (kbase_) + li * KCH + ((2 * (f - NV_) + hf) ^ sw_k));                               \
        if (f >= NG_ && (N_DO_PV_))         /* the first operands of the next step */               \
            NFR_[f >= NG_ ? f - NG_ : 0] = *reinterpret_cast<const bf16x8_t*>(                      \
                (nvbase_) + (((f >= NG_ ? f - NG_ : 0) % DB) * 32 + li) * VCH +                     \
                (((nvchunk0_) + 2 * ((f >= NG_ ? f - NG_ : 0) / DB) + hf) ^ sw_v));                 \
        {                                                                                           \
            if (gg < NJ_) FP_ISSUE_ONE(ktk_, ktv_, JLO_ + gg)                                       \
            /* two halves, each one MFMA (query block 0, then 1) with its share of the softmax: */  \
            /* the wave issues in order, so the vector work must sit between the two MFMAs */      \
            /* ---- first half */                                                                   \
            if (gg < NV_ && (DO_PV_))                                                               \
                acc[gg % DB][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                          \
                    FR_[gg], P_PV_[(gg / DB) % 2][0], acc[gg % DB][0], 0, 0, 0);                    \
            if (gg == NV_ && (DO_QK_)) FP_MFMA_S0(S_QK_[0], FR_[gg], qf[0][0]);                     \
            if (gg > NV_ && (DO_QK_)) FP_MFMA_S(S_QK_[0], FR_[gg], qf[0][gg > NV_ ? gg - NV_ : 0]); \
            if ((MASK_) && (gg == 0 || gg == 2)) {                                                  \
                constexpr int qb = gg / 2 % 2;                                                      \
                _Pragma("unroll") for (int r = 0; r < 16; ++r) {                                    \
                    const int key_ = (key0_sm_) + swap_bits_2_3(8 * (r >> 2) + 4 * hf + (r & 3));   \
                    if (key_ >= L || key_ < last_first_new) S_SM_[qb][r] = -INFINITY;             \
                }                                                                                   \
            }                                                                                       \
            if ((RESC_) && (gg == 1 || gg == 3)) {                                                  \
                /* two independent chains over the first eight scores */                            \
                constexpr int qb = gg / 2 % 2;                                                      \
                mxa_ = fmaxf(fmaxf(S_SM_[qb][0], S_SM_[qb][1]), S_SM_[qb][2]);                      \
                mxb_ = fmaxf(fmaxf(S_SM_[qb][3], S_SM_[qb][4]), S_SM_[qb][5]);                      \
                mxa_ = fmaxf(fmaxf(mxa_, S_SM_[qb][6]), S_SM_[qb][7]);                              \
            }                                                                                       \
            FP_HALF(RESC_, S_SM_, P_SM_, 2 * gg)                                                    \
            __builtin_amdgcn_sched_barrier(0);                                                      \
            /* ---- second half */                                                                  \
            if (gg < NV_ && (DO_PV_))                                                               \
                acc[gg % DB][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(                          \
                    FR_[gg], P_PV_[(gg / DB) % 2][1], acc[gg % DB][1], 0, 0, 0);                    \
            if (gg == NV_ && (DO_QK_)) FP_MFMA_S0(S_QK_[1], FR_[gg], qf[1][0]);                     \
            if (gg > NV_ && (DO_QK_)) FP_MFMA_S(S_QK_[1], FR_[gg], qf[1][gg > NV_ ? gg - NV_ : 0]); \
            if ((RESC_) && (gg == 1 || gg == 3)) {                                                  \
                constexpr int qb = gg / 2 % 2;                                                      \
                mxb_ = fmaxf(fmaxf(mxb_, S_SM_[qb][8]), S_SM_[qb][9]);                              \
                mxa_ = fmaxf(fmaxf(mxa_, S_SM_[qb][10]), S_SM_[qb][11]);                            \
                mxb_ = fmaxf(fmaxf(mxb_, S_SM_[qb][12]), S_SM_[qb][13]);                            \
                mxa_ = fmaxf(fmaxf(mxa_, S_SM_[qb][14]), S_SM_[qb][15]);                            \
                float mx_ = fmaxf(mxa_, mxb_);                                                      \
                mx_ = fmaxf(mx_, other_half(mx_));                                                  \
                const float m_new_ = fmaxf(m_run[qb], mx_ * p.scale_log2e);                         \
                m_use_[qb] = (m_new_ == -INFINITY) ? 0.f : m_new_;                                  \
                alpha_[qb] = __builtin_amdgcn_exp2f(m_run[qb] - m_use_[qb]);                        \
                m_run[qb] = m_new_;                                                                 \
            }                                                                                       \
            FP_HALF(RESC_, S_SM_, P_SM_, 2 * gg + 1)                                                \
            __builtin_amdgcn_sched_barrier(0);                                                      \
        }                                                                                           \
    }
#define FP_STEP(RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, \
                LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_)        \
    {                                                                                               \
        constexpr int NV_ = 2 * DB;                                                                 \
        constexpr int NG_ = 2 * DB + KS;           /* groups = fragments */                         \
        static_assert(NG_ == 16 || NG_ == 8, "the group list below is written for 16 or 8 groups"); \
        constexpr int JLO_ = (LOAD_K_) ? 0 : K_LD;                                                  \
        constexpr int JHI_ = (LOAD_V_) ? K_LD + V_LD : K_LD;                                        \
        constexpr int NJ_ = JHI_ > JLO_ ? JHI_ - JLO_ : 0;                                          \
        constexpr int DEPTH_ = NV_ < 6 ? NV_ : 6;  /* the fragments read ahead into the next step are V^T ones */ \
        float m_use_[QB], alpha_[QB], lsum_[QB], px_[32], pe_[32], mxa_ = 0.f, mxb_ = 0.f;          \
        uint32_t pw_[16];          /* packed probabilities: [qb][r / 2] */                         \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                         \
            m_use_[qb] = m_run[qb];   /* fast mode: the reference stays; else replaced in groups 1, 3 */ \
            alpha_[qb] = 1.0f;                                                                      \
            lsum_[qb] = 0.f;                                                                        \
        }                                                                                           \
        FP_G(0, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(1, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(2, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(3, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(4, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(5, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(6, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(7, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(8, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(9, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(10, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(11, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(12, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(13, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(14, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        FP_G(15, RESC_, S_SM_, P_SM_, key0_sm_, MASK_, DO_QK_, S_QK_, kbase_, DO_PV_, P_PV_, vbase_, vchunk0_, LOAD_K_, ktk_, LOAD_V_, ktv_, FR_, NFR_, N_DO_PV_, nvbase_, nvchunk0_, BAR_) \
        /* what the last half-groups left in flight */                                              \
        static_for<FP_E0(RESC_, 2 * NG_ - 1), 32>([&](auto e_c) { constexpr int e = decltype(e_c)::value; FP_EXP(e) }); \
        static_for<FP_E0(RESC_, 2 * NG_ - 2), 32>([&](auto e_c) { constexpr int e = decltype(e_c)::value; FP_CONSUME(P_SM_, e) }); \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                         \
            if (RESC_) l_run[qb] = l_run[qb] * alpha_[qb] + lsum_[qb];                              \
            else l_run[qb] += lsum_[qb];                                                            \
            _Pragma("unroll") for (int t = 0; t < 2; ++t) {                                         \
                const u32x4_t w_ = {pw_[qb * 8 + t * 4 + 0], pw_[qb * 8 + t * 4 + 1],               \
                                    pw_[qb * 8 + t * 4 + 2], pw_[qb * 8 + t * 4 + 3]};              \
                P_SM_[t][qb] = __builtin_bit_cast(bf16x8_t, w_);                                    \
            }                                                                                       \
        }                                                                                           \
        if (RESC_) {                                                                                \
            /* O is relative to the old maximum */                                                  \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                     \
                if (__any(alpha_[qb] != 1.0f)) {                                                    \
                    _Pragma("unroll") for (int db = 0; db < DB; ++db)                               \
                        _Pragma("unroll") for (int r = 0; r < 16; ++r) acc[db][qb][r] *= alpha_[qb]; \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
    }
    // One tile = two steps.  FIRST_: no previous block to multiply; HAS_K2_: K tile kt+2 exists;
    // HAS_NEXT_: tile kt+1 exists; LAST_: this is the shifted last tile.  The barrier sits inside
    // the first step, after its last read of the old tiles.
#define FP_TILE(RESC_, kt_, FIRST_, HAS_K2_, HAS_NEXT_, LAST_)                                      \
    {                                                                                               \
        const int start_ = FP_TILE_START(kt_) + kh * 64;                                            \
        const u32x4_t* ks_ = lds + ((kt_) & 1) * K_TILE + (kh * 64) * KCH;       /* K tile kt */     \
        const u32x4_t* kn_ = lds + (((kt_) + 1) & 1) * K_TILE + (kh * 64) * KCH; /* K tile kt+1 */   \
        const u32x4_t* vp_ = lds + 2 * K_TILE + (((kt_) + 1) & 1) * V_TILE;      /* V^T tile kt-1 */ \
        const u32x4_t* vs_ = lds + 2 * K_TILE + ((kt_) & 1) * V_TILE;            /* V^T tile kt */   \
        /* first step: softmax(kt,0); S(kt,1); PV(kt-1,1); next step starts with V^T(kt) block 0 */ \
        FP_STEP(RESC_, sa_, pa_, start_, LAST_, true, sb_, ks_ + 32 * KCH, !(FIRST_), pb_, vp_, kh * 8 + 4, \
                false, 0, false, 0, fe_, fo_, true, vs_, kh * 8, true)                              \
        /* second step: softmax(kt,1); S(kt+1,0); PV(kt,0); fetch K tile kt+2 and V^T tile kt+1; */ \
        /* next step starts with V^T(kt) block 1 */                                                 \
        FP_STEP(RESC_, sb_, pb_, start_ + 32, LAST_, HAS_NEXT_, sa_, kn_, true, pa_, vs_, kh * 8,   \
                HAS_K2_, (kt_) + 2, HAS_NEXT_, (kt_) + 1, fo_, fe_, HAS_NEXT_, vs_, kh * 8 + 4, false) \
    }
    // The whole pass over the keys.  The first tile always runs with the running maximum (it
    // establishes the reference); REST_ selects the mode of the others.
#define FP_RUN(REST_)                                                                               \
    {                                                                                               \
        _Pragma("unroll") for (int db = 0; db < DB; ++db)                                           \
            _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) acc[db][qb] = zero16;                 \
        _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) { m_run[qb] = -INFINITY; l_run[qb] = 0.f; } \
        /* K tiles 0 and 1, V^T tile 0; first score block */                                        \
        _Pragma("unroll") for (int j = 0; j < K_LD; ++j) FP_ISSUE_ONE(0, 0, j)                      \
        _Pragma("unroll") for (int j = 0; j < K_LD; ++j) FP_ISSUE_ONE(1, 0, j)                      \
        _Pragma("unroll") for (int j = K_LD; j < K_LD + V_LD; ++j) FP_ISSUE_ONE(0, 0, j)            \
        FP_PUBLISH()                                                                                \
        {                                                                                           \
            const u32x4_t* k0_ = lds + (kh * 64) * KCH;                                             \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                     \
                const bf16x8_t kf_ =                                                                \
                    *reinterpret_cast<const bf16x8_t*>(k0_ + li * KCH + ((2 * ks + hf) ^ sw_k));    \
                _Pragma("unroll") for (int qb = 0; qb < QB; ++qb) {                                 \
                    if (ks == 0) FP_MFMA_S0(sa_[qb], kf_, qf[qb][ks]);                              \
                    else FP_MFMA_S(sa_[qb], kf_, qf[qb][ks]);                                       \
                }                                                                                   \
            }                                                                                       \
        }                                                                                           \
        FP_TILE(true, 0, true, true, true, false)                                                   \
        int kt = 1;                                                                                 \
        for (; kt + 2 < KT; ++kt) FP_TILE(REST_, kt, false, true, true, false)                      \
        FP_TILE(REST_, kt, false, false, true, false) /* kt = KT-2 */                               \
        ++kt;                                                                                       \
        FP_TILE(REST_, kt, false, false, false, true) /* kt = KT-1 */                               \
        {   /* O^T += V^T P^T for the very last block (KT-1, 1) */                                  \
            const u32x4_t* vs_ = lds + 2 * K_TILE + ((KT - 1) & 1) * V_TILE;                        \
            _Pragma("unroll") for (int t = 0; t < 2; ++t)                                           \
                _Pragma("unroll") for (int db = 0; db < DB; ++db) {                                 \
                    const bf16x8_t vf_ = *reinterpret_cast<const bf16x8_t*>(                        \
                        vs_ + (db * 32 + li) * VCH + ((kh * 8 + 4 + 2 * t + hf) ^ sw_v));           \
                    _Pragma("unroll") for (int qb = 0; qb < QB; ++qb)                               \
                        acc[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf_, pb_[t][qb],      \
                                                                              acc[db][qb], 0, 0, 0); \
                }                                                                                   \
        }                                                                                           \
    }

    FP_RUN(false)
    {
        // Did any score of any wave rise far enough above its reference to endanger the fp32 range?
        // Then a row sum is huge, infinite or NaN (each fails the comparison the right way round)
        // and every wave repeats the pass with the running maximum.
        int* flag = reinterpret_cast<int*>(smem);
        FP_PUBLISH()   // all waves are done with the tiles
        if (tid == 0) *flag = 0;
        FP_PUBLISH()
        if (!(l_run[0] < 0x1p100f) || !(l_run[1] < 0x1p100f)) *flag = 1;
        FP_PUBLISH()
        const int redo = *flag;
        FP_PUBLISH()   // the flag's LDS word is tile memory again
        if (redo) FP_RUN(true)
    }
#undef FP_RUN
#undef FP_TILE
#undef FP_STEP
#undef FP_G
#undef FP_HALF
#undef FP_E0
#undef FP_CONSUME
#undef FP_EXP
#undef FP_ARG
#undef FP_MFMA_S
#undef FP_MFMA_S0
#undef FP_FIX_TAIL
#undef FP_ISSUE_ONE
#undef FP_DMA16
#undef FP_TILE_START

    // ---- merge the key slices of a query group, normalise and store (as in the kernel above)
    if (KSPLIT > 1) {
        FP_PUBLISH()  // everyone is done with the operand tiles
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
            FP_PUBLISH()
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
            if (src + 1 < KSPLIT) FP_PUBLISH()
        }
    }
#undef FP_PUBLISH
    if (KVS && nsp > 1) {
        // A key range first counts itself in at the query tile's counter.  Every range but the last to arrive
        // then leaves its partial result (statistics, then the accumulator), waits until its stores have been
        // acknowledged and reports ready; the last to arrive keeps its own part in registers, waits for the
        // others' reports (they are running and past their key loops, so the wait is short and always ends; it
        // is bounded all the same) and combines all ranges exactly, in range order, normalises and stores.
        // Against every range storing before it counts: a range's worth less of traffic, and the last
        // arriver's own stores are off the launch's critical path.  The partials go out and come back as
        // 16 bytes per lane with the device-scope cache policy (written through to, and read from, the
        // memory side of the chip's eight L2s, where they are coherent by themselves); counter and ready
        // count are device-scope relaxed atomics.
        // Layout per (query tile, range): [vector][QG*64 lanes][4 floats]; vector 0 holds the statistics
        // (running maxima, then row sums, of the lane's two query blocks), vector 1 + (db*QB + qb)*4 + g
        // the accumulator registers 4g .. 4g+3 of block (db, qb).
        static_assert(QB == 2, "the statistics of the two query blocks fill one 16-byte vector");
        constexpr int VECS = 1 + DB * QB * 4;
        constexpr int kDeviceScope = 16;   // cache-policy bit of the buffer accesses below
        const size_t tile_id = (size_t)tail_idx;
        const uint32_t vstride = (uint32_t)VECS * (QG * 64) * 16;     // bytes per (tile, range)
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            reinterpret_cast<char*>(p.part) + tile_id * p.splits * (size_t)vstride, 0, 0x7FFFFFFF, 0x00020000);
        const uint32_t lane_off = (uint32_t)(qg * 64 + lane) * 16u;
        float l_tot[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) l_tot[qb] = l_run[qb] + other_half(l_run[qb]);
        int* flag = reinterpret_cast<int*>(smem);
        __syncthreads();                 // the flag's LDS word was tile or merge memory
        if (tid == 0)
            *flag = __hip_atomic_fetch_add(p.split_cnt + tile_id * kCounterStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int arrived = *flag;
        if (arrived != p.splits - 1) {
            if (kh == 0) {
                const uint32_t mine = (uint32_t)split * vstride + lane_off;
                const f32x4_t st = {m_run[0], m_run[1], l_tot[0], l_tot[1]};
                __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4_t, st), rsrc, mine, 0, kDeviceScope);
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const f32x4_t v = {acc[db][qb][4 * g + 0], acc[db][qb][4 * g + 1], acc[db][qb][4 * g + 2],
                                               acc[db][qb][4 * g + 3]};
                            __builtin_amdgcn_raw_buffer_store_b128(
                                __builtin_bit_cast(u32x4_t, v), rsrc,
                                mine + (uint32_t)(1 + (db * QB + qb) * 4 + g) * (QG * 64 * 16), 0, kDeviceScope);
                        }
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(attn_waitcnt(0, true));   // own stores acknowledged
            __syncthreads();
            if (tid == 0)
                __hip_atomic_fetch_add(p.split_ready + tile_id * kCounterStride, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (tid == 0) {
            // about a microsecond per look; the bound is never reached by a launch that is making progress
            for (int looks = 0; looks < (1 << 20); ++looks) {
                if (__hip_atomic_load(p.split_ready + tile_id * kCounterStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                    p.splits - 1)
                    break;
                __builtin_amdgcn_s_sleep(8);
            }
            // ready for the next launch
            __hip_atomic_store(p.split_cnt + tile_id * kCounterStride, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.split_ready + tile_id * kCounterStride, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        if (kh != 0) return;
        if (p.splits == 2) {
            // Two ranges: the other range's statistics and all 32 accumulator vectors of a lane are fetched
            // together (one round trip to the memory side, 0.9 us, instead of one per accumulator block), then
            // summed in range order, r = fma(w1, part1, w0 * part0), whichever of the two this workgroup holds
            // in registers: the result does not depend on who arrived last.
            const int other = split ^ 1;
            f32x4_t pv[VECS];
#pragma unroll
            for (int vi = 0; vi < VECS; ++vi)
                pv[vi] = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                         rsrc, (uint32_t)other * vstride + lane_off +
                                                                   (uint32_t)vi * (QG * 64 * 16), 0, kDeviceScope));
            __builtin_amdgcn_sched_barrier(0);   // every load is out before the first use
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                const float m_o = pv[0][qb], l_o = pv[0][2 + qb];
                const float m = fmaxf(m_run[qb], m_o);
                const float w_me = __builtin_amdgcn_exp2f(m_run[qb] - m), w_o = __builtin_amdgcn_exp2f(m_o - m);
                const float w0 = split == 0 ? w_me : w_o, w1 = split == 0 ? w_o : w_me;
                const float l0 = split == 0 ? l_tot[qb] : l_o, l1 = split == 0 ? l_o : l_tot[qb];
                const float inv = 1.0f / __builtin_fmaf(w1, l1, w0 * l0);
                const int qrow = q_base + qb * 32 + li;
                bf16_t* dst = p.o + ((size_t)b * p.k_tokens + min(qrow, p.k_tokens - 1)) * p.D + head * DH + 4 * hf;
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    float o[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const float mine = acc[db][qb][r], theirs = pv[1 + (db * QB + qb) * 4 + r / 4][r % 4];
                        const float p0 = split == 0 ? mine : theirs, p1 = split == 0 ? theirs : mine;
                        o[r] = __builtin_fmaf(w1, p1, w0 * p0);
                    }
                    if (qrow < p.k_tokens) {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            u32x2_t pk;
                            pk.x = pack_bf16x2(o[4 * g + 0] * inv, o[4 * g + 1] * inv);
                            pk.y = pack_bf16x2(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
                            *reinterpret_cast<u32x2_t*>(dst + db * 32 + 8 * g) = pk;
                        }
                    }
                }
            }
            return;
        }
        // statistics of every range (at most four), own from registers
        float ms[4][QB], ls[4][QB];
        for (int s2 = 0; s2 < p.splits; ++s2) {
            f32x4_t st = {m_run[0], m_run[1], l_tot[0], l_tot[1]};
            if (s2 != split)
                st = __builtin_bit_cast(f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                                     rsrc, (uint32_t)s2 * vstride + lane_off, 0, kDeviceScope));
            ms[s2 & 3][0] = st[0]; ms[s2 & 3][1] = st[1];
            ls[s2 & 3][0] = st[2]; ls[s2 & 3][1] = st[3];
        }
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            float ws[4];
            float m = m_run[qb];
            for (int s2 = 0; s2 < p.splits; ++s2) m = fmaxf(m, ms[s2 & 3][qb]);
            float l = 0.f;
            for (int s2 = 0; s2 < p.splits; ++s2) {
                ws[s2 & 3] = __builtin_amdgcn_exp2f(ms[s2 & 3][qb] - m);
                l += ws[s2 & 3] * ls[s2 & 3][qb];
            }
            const float inv = 1.0f / l;
            const int qrow = q_base + qb * 32 + li;
            bf16_t* dst = p.o + ((size_t)b * p.k_tokens + min(qrow, p.k_tokens - 1)) * p.D + head * DH + 4 * hf;
#pragma unroll
            for (int db = 0; db < DB; ++db) {
                float o[16];
#pragma unroll
                for (int r = 0; r < 16; ++r) o[r] = 0.f;
                for (int s2 = 0; s2 < p.splits; ++s2) {
                    float v[16];
                    if (s2 == split) {
#pragma unroll
                        for (int r = 0; r < 16; ++r) v[r] = acc[db][qb][r];
                    } else {
#pragma unroll
                        for (int g = 0; g < 4; ++g) {
                            const f32x4_t t = __builtin_bit_cast(
                                f32x4_t, __builtin_amdgcn_raw_buffer_load_b128(
                                             rsrc,
                                             (uint32_t)s2 * vstride + lane_off +
                                                 (uint32_t)(1 + (db * QB + qb) * 4 + g) * (QG * 64 * 16),
                                             0, kDeviceScope));
                            v[4 * g + 0] = t[0]; v[4 * g + 1] = t[1]; v[4 * g + 2] = t[2]; v[4 * g + 3] = t[3];
                        }
                    }
#pragma unroll
                    for (int r = 0; r < 16; ++r) o[r] += ws[s2 & 3] * v[r];
                }
                if (qrow < p.k_tokens) {
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        u32x2_t pk;
                        pk.x = pack_bf16x2(o[4 * g + 0] * inv, o[4 * g + 1] * inv);
                        pk.y = pack_bf16x2(o[4 * g + 2] * inv, o[4 * g + 3] * inv);
                        *reinterpret_cast<u32x2_t*>(dst + db * 32 + 8 * g) = pk;
                    }
                }
            }
        }
        return;
    }
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

template <int DH, int QG, int KSPLIT>
void launch_pipe(const AttnParams& p, int B, hipStream_t stream) {
    constexpr size_t tile_bytes = (size_t)2 * (64 * KSPLIT * (DH / 8) + DH * (8 * KSPLIT)) * 16;
    constexpr size_t merge_bytes = KSPLIT > 1 ? (size_t)QG * (DH / 32 * 16 + 2) * 2 * 64 * 4 : 0;
    constexpr size_t smem = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
    static std::once_flag once;
    raise_lds_limit_once(once, &attention_pipe_kernel<DH, QG, KSPLIT>, smem);
    const int per_wg = QG * 64;
    attention_pipe_kernel<DH, QG, KSPLIT>
        <<<dim3((p.k_tokens + per_wg - 1) / per_wg, p.H, B), QG * KSPLIT * 64, smem, stream>>>(p);
}

// the pipelined kernel with the key range split between `p.splits` workgroups per query tile
template <int DH, int QG, int KSPLIT>
void launch_pipe_split(const AttnParams& p, int B, hipStream_t stream) {
    constexpr size_t tile_bytes = (size_t)2 * (64 * KSPLIT * (DH / 8) + DH * (8 * KSPLIT)) * 16;
    constexpr size_t merge_bytes = KSPLIT > 1 ? (size_t)QG * (DH / 32 * 16 + 2) * 2 * 64 * 4 : 0;
    constexpr size_t smem = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
    static std::once_flag once;
    raise_lds_limit_once(once, &attention_pipe_kernel<DH, QG, KSPLIT, true>, smem);
    (void)B;
    attention_pipe_kernel<DH, QG, KSPLIT, true>
        <<<dim3(p.full_tiles + p.tail_tiles * p.splits), QG * KSPLIT * 64, smem, stream>>>(p);
}

template <int DH, int QB, int QG, int KSPLIT>
void launch_cfg(const AttnParams& p, int B, hipStream_t stream) {
    constexpr size_t tile_bytes = (size_t)2 * (64 * KSPLIT * (DH / 8) + DH * (8 * KSPLIT)) * 16;
    constexpr size_t merge_bytes = KSPLIT > 1 ? (size_t)QG * (DH / 32 * 16 + 2) * QB * 64 * 4 : 0;
    constexpr size_t smem = tile_bytes > merge_bytes ? tile_bytes : merge_bytes;
    static std::once_flag once;
    raise_lds_limit_once(once, &attention_kernel<DH, QB, QG, KSPLIT>, smem);
    const int per_wg = QG * 32 * QB;
    attention_kernel<DH, QB, QG, KSPLIT>
        <<<dim3((p.k_tokens + per_wg - 1) / per_wg, p.H, B), QG * KSPLIT * 64, smem, stream>>>(p);
}

// Tuning builds only (-DFASTVAR_DEV_KNOBS, never the product library, which reads no environment and keeps
// no state): FASTVAR_ATTN_WIDE=0 turns the 256-query variants of the key-range split off, FASTVAR_ATTN_CFG
// forces a kernel configuration.
bool attn_wide_enabled() {
#ifdef FASTVAR_DEV_KNOBS
    const char* e = getenv("FASTVAR_ATTN_WIDE");
    return !e || atoi(e) != 0;
#else
    return true;
#endif
}

int attn_cfg_override() {
#ifdef FASTVAR_DEV_KNOBS
    const char* e = getenv("FASTVAR_ATTN_CFG");
    return e ? atoi(e) : -1;
#else
    return -1;
#endif
}

}  // namespace

AttnSplitPlan attention_split_plan(int B, int H, int dh, int k_tokens, int L, size_t max_bytes) {
    AttnSplitPlan sp{1, 0, false, 0, 0, 0, 0, 0};
    if (dh != 128 || L <= 256 || k_tokens <= 0) return sp;
    const long wg128 = (long)((k_tokens + 127) / 128) * H * B;
    // With fewer than 128 workgroups of 128 queries the unsplit launch is the plain kernel's 64-query workgroups
    // (keys split in two inside the workgroup), which the model below does not describe; over a short cache
    // they win (400 / 576 queries over 921 / 1497 keys: 22.3 / 29.3 us against 25.5 / 33.7 on two / three
    // ranges), over a long one the ranges do (410 queries over 6835 keys).
    if (wg128 < 128 && L < 2048) return sp;
    const long wg256 = (long)((k_tokens + 255) / 256) * H * B;
    const size_t per_query_row = (size_t)(1 + 4 * 2 * 4) * 64 * 16;   // per wave of 64 queries: 33 vectors of 16 bytes per lane
    // The counters take the same room whichever variant is chosen (one per 128-query tile, the larger count).
    // (two per tile: arrivals, and ranges whose partial result is complete)
    const size_t counter_bytes = (size_t)wg128 * 8 * kCounterStride;
    auto ranges_ok = [&](int s, int bn, int& per) {
        per = (((L + s - 1) / s) + bn - 1) / bn * bn;          // whole key tiles
        return per > 2 * bn && L - (s - 1) * per > 2 * bn;     // every range has at least three tiles
    };
    // Time model, in units of one 128-query workgroup walking all L keys: workgroups run in rounds of 256
    // (one per CU); a 256-query workgroup takes 1.86 units (twice the work, about 7 % faster); a workgroup
    // on one of s key ranges takes 1/s of that plus its prologue, its partial output and the merge: 4 % for
    // two ranges, 18 % per extra range beyond (with three rounds of workgroups the split lost in every
    // case tried, so at most two are considered).  Unsplit, the launcher below takes the cheaper of the
    // two workgroup sizes.
    auto rounds = [](long wgs) { return (double)((wgs + 255) / 256); };
    const double kWide = 1.86;
    double best = rounds(wg128) < kWide * rounds(wg256) ? rounds(wg128) : kWide * rounds(wg256);
    best *= 0.97;    // a split has to win by more than the model's noise
    for (int wide = 0; wide <= (attn_wide_enabled() ? 1 : 0); ++wide) {
        // with fewer than 128 workgroups of 128 queries the unsplit launch is the plain kernel's 64-query
        // workgroups, which the model above does not describe and 256-query workgroups do not beat
        if (wide && wg128 < 128) continue;
        const long wg = wide ? wg256 : wg128;
        for (int s = 2; s <= 4; ++s) {
            int per;
            if (wg * s > 512 || !ranges_ok(s, wide ? 64 : 128, per)) continue;
            const size_t bytes = counter_bytes + (size_t)wg * s * (wide ? 4 : 2) * per_query_row;
            if (max_bytes && bytes > max_bytes) continue;
            // one round of 128-query workgroups, or two ranges: the figures above; three or four ranges of
            // 256-query workgroups, or two rounds: the fixed cost per range weighs more the shorter the
            // range (measured with cold caches at 3.7-19 K keys: a loss below about 6 K keys)
            const bool plain_case = wg * s <= 256 && (!wide || s == 2);
            const double overhead = plain_case ? (s == 2 ? 0.04 : 0.18 * (s - 1)) : (s - 1) * (0.1 + 900.0 / L);
            const double cost = (wide ? kWide : 1.0) * rounds(wg * s) / s * (1.0 + overhead);
            if (cost < best) {
                best = cost;
                sp.splits = s; sp.keys_per_split = per; sp.wide = wide != 0;
                sp.full_tiles = 0; sp.tail_tiles = (int)wg;
                sp.counters = (int)wg; sp.counter_bytes = counter_bytes; sp.bytes = bytes;
            }
        }
    }
    // (only where no launch with every tile split beat the unsplit one: where one did, the mixed launch lost
    // to it: 2560 kept tokens over 13 K keys, three ranges in two rounds 251 us, mixed 273)
    if (sp.splits > 1) return sp;
    for (int wide = 0; wide <= (attn_wide_enabled() ? 1 : 0); ++wide) {
        if (wide && wg128 < 128) continue;
        const long wg = wide ? wg256 : wg128;
        // Whole rounds unsplit, the part-filled last round on s key ranges each: 576 workgroups (1152 kept
        // tokens, 16 heads, four samples) are two rounds of 256 plus 64 tiles on four ranges, two and a
        // quarter rounds instead of three.  The shared tiles are the last ones of the launch; they start as
        // the full ones drain.  A part-filled round costs less than the model's full round (with a quarter
        // of the CUs idle the others ran 15 % faster: 3072 kept tokens, 192 workgroups of 256 queries), and a
        // 256-query workgroup then costs about 1.6 units, not 1.86; measured, the mixed launch lost 4-7 %
        // where this model saw it 4 % ahead (3072 and 2765 kept tokens) and won 7 % where it saw 20 %
        // (4 x 1152), so it has to be 12 % ahead of the unsplit launch to be taken.
        const long full = (wg / 256) * 256, rem = wg - full;
        if (full == 0 || rem == 0) continue;
        const double kWideMixed = 1.6;
        const double unsplit = rounds(wg128) < kWideMixed * rounds(wg256) ? rounds(wg128) : kWideMixed * rounds(wg256);
        for (int s = 2; s <= 4; ++s) {
            int per;
            if (rem * s > 256 || !ranges_ok(s, wide ? 64 : 128, per)) continue;
            const size_t bytes = counter_bytes + (size_t)rem * s * (wide ? 4 : 2) * per_query_row;
            if (max_bytes && bytes > max_bytes) continue;
            const double overhead = s == 2 ? 0.06 : 0.18 * (s - 1);
            const double cost = (wide ? kWideMixed : 1.0) * ((double)(full / 256) + (1.0 + overhead) / s);
            if (cost < 0.88 * unsplit && cost < best) {
                best = cost;
                sp.splits = s; sp.keys_per_split = per; sp.wide = wide != 0;
                sp.full_tiles = (int)full; sp.tail_tiles = (int)rem;
                sp.counters = (int)wg; sp.counter_bytes = counter_bytes; sp.bytes = bytes;
            }
        }
    }
    return sp;
}

void launch_attention(const AttnArgs& a, hipStream_t stream) {
    AttnParams p;
    p.q = static_cast<const bf16_t*>(a.q);
    p.kc = static_cast<const bf16_t*>(a.k_cache);
    p.vc = static_cast<const bf16_t*>(a.v_cache);
    p.o = static_cast<bf16_t*>(a.o);
    p.H = a.H; p.k_tokens = a.k_tokens; p.L = a.L; p.L_cap = a.L_cap; p.D = a.H * a.dh;
    p.scale_log2e = a.scale * 1.4426950408889634f;
    p.q_tiles = (a.k_tokens + 127) / 128; p.splits = 1; p.keys_per_split = 0; p.part = nullptr; p.split_cnt = nullptr; p.split_ready = nullptr;
    p.full_tiles = p.tail_tiles = 0;
    if (a.split_ws && attn_cfg_override() < 0) {
        const AttnSplitPlan sp = attention_split_plan(a.B, a.H, a.dh, a.k_tokens, a.L, a.split_ws_bytes);
        if (sp.splits > 1) {
            p.splits = sp.splits; p.keys_per_split = sp.keys_per_split;
            p.full_tiles = sp.full_tiles; p.tail_tiles = sp.tail_tiles;
            p.split_cnt = static_cast<int*>(a.split_ws);
            p.split_ready = p.split_cnt + sp.counter_bytes / 8;
            p.part = reinterpret_cast<float*>(static_cast<char*>(a.split_ws) + sp.counter_bytes);
            if (sp.wide) {
                p.q_tiles = (a.k_tokens + 255) / 256;
                launch_pipe_split<128, 4, 1>(p, a.B, stream);
            } else {
                launch_pipe_split<128, 2, 2>(p, a.B, stream);
            }
            return;
        }
    }
    // Head dim 128 and more than two key tiles: the software-pipelined kernel (64 queries per wave),
    // with 128-query workgroups (two query groups x two key slices) or 256-query workgroups (four query
    // groups), whichever needs less time for its rounds of workgroups; with fewer than 128 workgroups
    // of 128 queries, 64-query workgroups of the plain kernel (one wave per 32 queries, keys split in two).
    // Otherwise one wave per 32 queries, two waves per SIMD: with enough queries two 4-wave workgroups
    // share a CU; with fewer an 8-wave workgroup splits the keys of each tile between two waves per
    // query group.
    const long waves = (long)((a.k_tokens + 31) / 32) * a.H * a.B;
    const long wg256 = (long)((a.k_tokens + 255) / 256) * a.H * a.B;
    const long wg128 = (long)((a.k_tokens + 127) / 128) * a.H * a.B;
    int cfg = waves >= 1800 ? 2 : 4;
    if (a.dh == 128 && a.L > 256) {
        // rounds of workgroups on 256 CUs; a 256-query workgroup does twice the work about 7 % faster
        const long rounds128 = (wg128 + 255) / 256, rounds256 = (wg256 + 255) / 256;
        if (wg128 < 128) cfg = 3;   // too few queries for half the chip: 64-query workgroups, keys split in two
        else cfg = 1.86 * (double)rounds256 < (double)rounds128 ? 6 : 5;
    }
    if (a.dh == 64 && a.L >= 1024 && wg256 >= 128 && (a.k_tokens + 255) / 256 * 2 == (a.k_tokens + 127) / 128) {
        // Head dim 64 is bound by the softmax, not the matrix pipe, and the pipelined kernel gains less:
        // its 256-query workgroups win (by 5-20 % on 8 x 30 heads, 1024-3072 keys) where they pad the
        // queries no further than 128-query workgroups would and the key loop is long enough to pay
        // for the longer prologue; the plain kernel wins elsewhere.
        cfg = 6;
    }
    if (attn_cfg_override() >= 0) cfg = attn_cfg_override();
    // the software-pipelined kernel needs at least three key tiles
    if ((cfg == 5 || cfg == 6) && a.L <= 2 * (cfg == 5 ? 128 : 64)) cfg = 4;
    if (a.dh == 128) {
        switch (cfg) {
            case 0: launch_cfg<128, 2, 4, 1>(p, a.B, stream); break;
            case 1: launch_cfg<128, 2, 2, 2>(p, a.B, stream); break;
            case 2: launch_cfg<128, 1, 4, 1>(p, a.B, stream); break;
            case 3: launch_cfg<128, 1, 2, 2>(p, a.B, stream); break;
            case 5: launch_pipe<128, 2, 2>(p, a.B, stream); break;
            case 6: launch_pipe<128, 4, 1>(p, a.B, stream); break;
            default: launch_cfg<128, 1, 4, 2>(p, a.B, stream); break;
        }
    } else {
        switch (cfg) {
            case 0: launch_cfg<64, 2, 4, 1>(p, a.B, stream); break;
            case 1: launch_cfg<64, 2, 2, 2>(p, a.B, stream); break;
            case 2: launch_cfg<64, 1, 4, 1>(p, a.B, stream); break;
            case 3: launch_cfg<64, 1, 2, 2>(p, a.B, stream); break;
            case 5: launch_pipe<64, 2, 2>(p, a.B, stream); break;
            case 6: launch_pipe<64, 4, 1>(p, a.B, stream); break;
            default: launch_cfg<64, 1, 4, 2>(p, a.B, stream); break;
        }
    }
}

}  // namespace fv
