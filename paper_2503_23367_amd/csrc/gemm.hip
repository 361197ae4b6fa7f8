// bf16 MFMA GEMM for the block's four dense contractions (QKV, out-proj, FC1,
// FC2):  C[m,n] = sum_k A[m,k] * W[n,k]  with A [M,K] and W [N,K] both
// K-contiguous (activations are row-major, weights are [out, in]).
//
// Tiling for gfx950: a workgroup of 4 or 8 waves owns a BM x BN tile of C; each
// wave owns a sub-tile built from 32x32x16 bf16 MFMAs with fp32 accumulators.
// K is walked in tiles of BK: both operand tiles are copied global -> LDS by
// direct-to-LDS loads into a ring of STAGES stages (the next tiles' loads are in
// flight while the current one is multiplied), in rows whose 16-byte chunks are
// XOR-swizzled with the row index so that the MFMA operand reads (one 16-byte
// ds_read per lane, 32 consecutive rows per half-wave) are conflict free.
//
// Epilogues are fused: bias, residual add, GELU, and for the QKV GEMM the
// split into the query buffer and the append into the K / V caches
// (V transposed so that cache positions are contiguous).
#include <stdio.h>
#include <stdlib.h>

#include <mutex>
#include "common.h"
#include "kernels.h"

namespace fv {

namespace {

// GELU in its tanh form written as a sigmoid: v * sigma(2u), u = sqrt(2/pi) (v + 0.044715 v^3).
// It deviates from the erf form by at most 3e-4 in absolute value (near |v| = 2),
// far below the bf16 resolution of the outputs, and costs 7 instructions where
// an erf approximation costs about 20: the epilogue is pure VALU time that no
// MFMA overlaps.
__device__ __forceinline__ float gelu_fast(float v) {
    // -2u log2(e), the factor folded into the two coefficients
    constexpr float c1 = -1.4426950408889634f * 1.5957691216057308f;
    constexpr float c3 = c1 * 0.044715f;
    const float v2 = v * v;
    const float e = __builtin_amdgcn_exp2f(v * fmaf(c3, v2, c1));                         // exp(-2u)
    return v * __builtin_amdgcn_rcpf(1.0f + e);
}

// Internal fourth epilogue: EPI_QKV with the rotary embedding of q and the new keys (an instantiation of its
// own, so that the plain QKV GEMM carries none of its registers).
constexpr int EPI_QKV_ROPE = 3;
constexpr bool is_qkv(int epi) { return epi == EPI_QKV || epi == EPI_QKV_ROPE; }

struct GemmParams {
    const bf16_t* A;
    const bf16_t* W;
    const bf16_t* bias;
    int M, N, K;
    bf16_t* out;
    const bf16_t* residual;
    const int32_t* res_rows;  // optional row gather for the residual: row of output row m is res_rows[m]
    const int32_t* out_rows;  // optional row scatter of the output (EPI_BIAS_RES): row m goes to row out_rows[m]
    bf16_t* q_out;
    bf16_t* k_cache;
    bf16_t* v_cache;
    int D, H, dh, k_tokens, L0, L_cap;
    const float* rope_cos;     // optional [rope_N, dh/2] tables: q and the new keys are turned in the epilogue
    const float* rope_sin;
    const int32_t* rope_rows;  // slot of output row m = rope_rows[m] % rope_N (NULL: its token index)
    int rope_N;
    int tiles_m, tiles_n;
    int splits;        // split-K slices (grid.y); 1 unless the kernel is instantiated with SK
    float* sk_part;    // [tile][slice][BM*BN] fp32 partial tiles, accumulator-register order
    int* sk_cnt;       // [tile] arrival counters, zero between launches
    int* sk_ready;     // [tile] slices whose partial tile is complete in memory (CF kernels), zero between launches
};

// s_waitcnt immediate (gfx9 encoding): wait until at most `vm` vector-memory
// operations are outstanding; lgkm = true also waits for all LDS/scalar ops.
constexpr int waitcnt_imm(int vm, bool lgkm) {
    return (vm & 0xF) | ((vm >> 4) << 14) | (0x7 << 4) | ((lgkm ? 0x0 : 0xF) << 8);
}

// XOR key that spreads the 16-byte chunks of consecutive rows over all 64 LDS
// banks (256 bytes): a 16-byte-per-lane read is served 16 lanes at a time, so 16
// consecutive rows must land in 16 different chunk columns.  Rows of 128 bytes
// (8 chunks, two rows per bank sweep) use row bits 1-3; rows of 64 bytes (4
// chunks, four rows per sweep) use row bits 2-3.
template <int CPR>
__device__ __forceinline__ int swz(int row) {
    return CPR == 8 ? ((row >> 1) & 7) : ((row >> 2) & 3);
}

// WGM x WGN waves tile the BM x BN block; KG such groups of waves split every K
// tile between them (group g takes the g-th run of 16-wide k-steps) and are
// summed through LDS at the end.  Eight waves (two per SIMD) cover each other's
// barrier, load and LDS waits where the tile gives one wave per SIMD too little
// independent work.
// SK: the K range is also split between workgroups (blockIdx.y); every workgroup leaves its partial
// tile in scratch memory, and the one that arrives last at the tile's counter adds the slices up, in
// slice order (so the sum does not depend on who was last), and runs the epilogue.  Nobody waits.
// CF (with SK; large partial tiles): the slices count themselves in first, only the earlier arrivers
// store, and the last one polls for their stores: see the epilogue.
template <int EPI, int KG, bool SK>
constexpr bool kPersistent = !SK && KG == 1 && is_qkv(EPI);

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, int KG, int EPI, bool SK = false, bool CF = false>
__global__ __launch_bounds__(64 * WGM * WGN * KG) void gemm_nt_kernel(const GemmParams p) {
#if defined(__HIP_DEVICE_COMPILE__)  // the host pass only needs the launch stub
    constexpr int NWQ = WGM * WGN;             // waves per k-group
    constexpr int NW = NWQ * KG;               // waves per workgroup
    constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
    constexpr int MI = WTM / 32, NI = WTN / 32;
    constexpr int CPR = BK / 8;                // 16-byte chunks per LDS row
    constexpr int RPI = 64 / CPR;              // rows covered by one 64-lane direct-to-LDS load
    constexpr int KK = BK / 16 / KG;           // MFMA k-steps per tile and k-group
    constexpr int A_LD = BM / RPI / NW, W_LD = BN / RPI / NW;  // loads per wave per tile
    constexpr int LPT = A_LD + W_LD;
    constexpr int A_TILE = BM * CPR, W_TILE = BN * CPR;      // 16-byte chunks per stage
    constexpr int STAGE = A_TILE + W_TILE;
    static_assert(WTM % 32 == 0 && WTN % 32 == 0 && (BK / 16) % KG == 0, "wave tiles are made of 32x32x16 MFMAs");
    static_assert(A_LD * RPI * NW == BM && W_LD * RPI * NW == BN && NW % 2 == 0, "loads must tile the stage");
    // When a stage is refilled.  EARLY: at the hand-over that frees it, all of the tile's loads at once (LPR
    // after each operand read), so they have STAGES-1 whole tiles of matrix work to land in: what a ring of two
    // stages needs.  Otherwise spread over the k-steps of the following tile, one load per operand read: a
    // quarter to three quarters of a tile later, which deeper rings can afford, and gentler on the hand-over.
#ifndef FV_GEMM_EARLY_MAX_STAGES
#define FV_GEMM_EARLY_MAX_STAGES 2
#endif
    constexpr bool EARLY = STAGES <= FV_GEMM_EARLY_MAX_STAGES || KK == 1;
    constexpr int LPR = (LPT + MI + NI - 1) / (MI + NI);
    static_assert(EARLY || (LPT + KK - 2) / (KK - 1) <= MI + NI, "one load per operand read at most");
    static_assert((STAGES - 1) * LPT <= 63, "vmcnt is 6 bits");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    u32x4_t* lds = reinterpret_cast<u32x4_t*>(smem);  // [STAGES][A tile | W tile]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int kg = wave / NWQ;                 // k-group
    const int wq = wave % NWQ;                 // position in the wave grid
    const int wm = wq / WGN, wn = wq % WGN;
    const int kk0 = kg * KK;                   // first k-step of this group inside a tile

    // Tile id: consecutive workgroup ids are dealt round-robin to the 8 XCDs;
    // undo that so each XCD (own L2) walks a contiguous run of tiles, and walk
    // tiles in groups of 8 tile-rows so neighbours share operand rows.
    // A QKV launch with more tiles than the chip holds workgroups at a time is persistent: the grid is one
    // round of workgroups, and workgroup i takes tiles i, i + grid, ... (the grid is a multiple of 8, so
    // a workgroup's tiles stay in its XCD's run).  What that buys is the overlap at the seam: the next
    // tile's first stages are fetched while this tile's epilogue runs, which needs no LDS.  It pays for the
    // QKV epilogue, the longest (2-byte stores into the transposed V cache): 3-4 % of the launch at 3072 to
    // 6552 rows; the other epilogues are short enough that the hardware's own hand-over from a finished
    // workgroup to the next does as well (measured: +-2 %), so they keep one workgroup per tile.
    constexpr bool PERSIST = kPersistent<EPI, KG, SK>;
    const int n_tiles = p.tiles_m * p.tiles_n;
    int m0, n0;
#define FV_TILE_COORDS(vpid_)                                                                   \
    {                                                                                           \
        int pid_ = (vpid_);                                                                     \
        if ((n_tiles & 7) == 0) pid_ = (pid_ & 7) * (n_tiles >> 3) + (pid_ >> 3);              \
        constexpr int GROUP = 8;                                                                \
        const int per_group_ = GROUP * p.tiles_n;                                               \
        const int grp_ = pid_ / per_group_;                                                     \
        const int first_m_ = grp_ * GROUP;                                                      \
        const int gsize_ = min(p.tiles_m - first_m_, GROUP);                                    \
        const int in_grp_ = pid_ - grp_ * per_group_;                                           \
        m0 = (first_m_ + in_grp_ % gsize_) * BM;                                                \
        n0 = (in_grp_ / gsize_) * BN;                                                           \
    }
    int vpid = blockIdx.x;
    FV_TILE_COORDS(vpid)
    static_assert(!SK || KG == 1, "split-K across workgroups is written for one k-group");
    const int n_splits = SK ? p.splits : 1;
    const int split = SK ? (int)blockIdx.y : 0;
    const int KT = p.K / BK / n_splits;          // K tiles of this workgroup
    const bf16_t* const Ab = p.A + (size_t)split * KT * BK;
    const bf16_t* const Wb = p.W + (size_t)split * KT * BK;

    // Direct-to-LDS loads: one instruction moves 64 x 16 bytes into a contiguous
    // 1 KB of LDS (lane l lands at base + 16 l), i.e. RPI whole tile rows.  The
    // swizzle is applied on the global side: lane l fetches the chunk that
    // belongs at its LDS position.  Load j of a wave covers tile rows
    // (wave + NW j) * RPI + ld_row; the key of such a row does not depend on j
    // (RPI is 8 or 16, NW is even and the key uses row bits below 4).
    const int ld_row = lane / CPR;
    const int ld_chunk = (lane % CPR) ^ swz<CPR>(wave * RPI + ld_row);
    // Per-lane byte offsets of the loads; they do not change along K (the scalar
    // base pointer advances instead), so a load costs no vector arithmetic.
    uint32_t a_off[A_LD], w_off[W_LD];
#define FV_TILE_OFFSETS()                                                                       \
    {                                                                                           \
        _Pragma("unroll") for (int j = 0; j < A_LD; ++j)                                        \
            a_off[j] = (uint32_t)(min(m0 + (wave + NW * j) * RPI + ld_row, p.M - 1) * p.K + ld_chunk * 8) * 2u; \
        _Pragma("unroll") for (int j = 0; j < W_LD; ++j)                                        \
            w_off[j] = (uint32_t)(min(n0 + (wave + NW * j) * RPI + ld_row, p.N - 1) * p.K + ld_chunk * 8) * 2u; \
    }
    FV_TILE_OFFSETS()

    // The loads are issued through inline assembly: the compiler's own model of
    // this instruction makes it drain every outstanding LDS operation before the
    // next operand use, which would serialise the operand reads behind it.
    // Completion is tracked by hand (vmcnt before the barrier that publishes a tile).
    typedef __attribute__((address_space(3))) void* lds_ptr_t;
#define FV_DMA16(base_, off_, lds_chunk_ptr_)                                                   \
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2"                            \
                 :                                                                              \
                 : "s"((uint32_t)(uintptr_t)(lds_ptr_t)(lds_chunk_ptr_)), "v"(off_), "s"(base_) \
                 : "memory", "m0")
    // Load q of a tile (A loads first, then W) into ring stage stage_.
#define FV_ISSUE_Q(kt_, stage_, q_)                                                             \
    {                                                                                           \
        if ((q_) < A_LD)                                                                        \
            FV_DMA16(Ab + (size_t)(kt_) * BK, a_off[(q_) < A_LD ? (q_) : 0],                   \
                     lds + (stage_) * STAGE + wave * 64 + (q_) * (NW * 64));                    \
        else                                                                                    \
            FV_DMA16(Wb + (size_t)(kt_) * BK, w_off[(q_) >= A_LD ? (q_) - A_LD : 0],           \
                     lds + (stage_) * STAGE + A_TILE + wave * 64 + ((q_) - A_LD) * (NW * 64));  \
    }
#define FV_ISSUE_TILE(kt_, stage_)                                                              \
    _Pragma("unroll") for (int q = 0; q < LPT; ++q) FV_ISSUE_Q(kt_, stage_, q)

    const int frag_row = lane & 31;
    const int frag_half = lane >> 5;
    const int a_row = wm * WTM + frag_row;  // + 32 mi
    const int w_row = wn * WTN + frag_row;  // + 32 ni
    const int frag_sw = swz<CPR>(frag_row);

#define FV_LOAD_FRAGS(dst_a_, dst_w_, stage_, kk_)                                              \
    {                                                                                           \
        const u32x4_t* sa_ = lds + (stage_) * STAGE;                                            \
        const u32x4_t* sw_ = sa_ + A_TILE;                                                      \
        const int ch_ = (2 * (kk0 + (kk_)) + frag_half) ^ frag_sw;                              \
        _Pragma("unroll") for (int mi = 0; mi < MI; ++mi)                                       \
            dst_a_[mi] = *reinterpret_cast<const bf16x8_t*>(sa_ + (a_row + 32 * mi) * CPR + ch_); \
        _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                       \
            dst_w_[ni] = *reinterpret_cast<const bf16x8_t*>(sw_ + (w_row + 32 * ni) * CPR + ch_); \
    }
    // The same operand reads with the loads of a whole tile issued between them, LPR after each read
    // (putting reads between the loads keeps the texture-address queue from filling up and stalling the wave).
#define FV_LOAD_FRAGS_ISSUE(dst_a_, dst_w_, stage_, kk_, kt_, fill_)                            \
    {                                                                                           \
        const u32x4_t* sa_ = lds + (stage_) * STAGE;                                            \
        const u32x4_t* sw_ = sa_ + A_TILE;                                                      \
        const int ch_ = (2 * (kk0 + (kk_)) + frag_half) ^ frag_sw;                              \
        _Pragma("unroll") for (int g = 0; g < MI + NI; ++g) {                                   \
            if (g < MI)                                                                         \
                dst_a_[g < MI ? g : 0] =                                                        \
                    *reinterpret_cast<const bf16x8_t*>(sa_ + (a_row + 32 * g) * CPR + ch_);     \
            else                                                                                \
                dst_w_[g >= MI ? g - MI : 0] =                                                  \
                    *reinterpret_cast<const bf16x8_t*>(sw_ + (w_row + 32 * (g - MI)) * CPR + ch_); \
            _Pragma("unroll") for (int u = 0; u < LPR; ++u)                                     \
                if (g * LPR + u < LPT) FV_ISSUE_Q(kt_, fill_, g * LPR + u)                      \
        }                                                                                       \
    }

    // ... and with slice part_ of nparts_ of a tile's loads, one load after each read.
#define FV_LOAD_FRAGS_ISSUE_PART(dst_a_, dst_w_, stage_, kk_, kt_, fill_, part_, nparts_)       \
    {                                                                                           \
        const u32x4_t* sa_ = lds + (stage_) * STAGE;                                            \
        const u32x4_t* sw_ = sa_ + A_TILE;                                                      \
        const int ch_ = (2 * (kk0 + (kk_)) + frag_half) ^ frag_sw;                              \
        const int q_lo_ = (part_) * LPT / (nparts_), q_hi_ = ((part_) + 1) * LPT / (nparts_); \
        _Pragma("unroll") for (int g = 0; g < MI + NI; ++g) {                                   \
            if (g < MI)                                                                         \
                dst_a_[g < MI ? g : 0] =                                                        \
                    *reinterpret_cast<const bf16x8_t*>(sa_ + (a_row + 32 * g) * CPR + ch_);     \
            else                                                                                \
                dst_w_[g >= MI ? g - MI : 0] =                                                  \
                    *reinterpret_cast<const bf16x8_t*>(sw_ + (w_row + 32 * (g - MI)) * CPR + ch_); \
            if (q_lo_ + g < q_hi_) FV_ISSUE_Q(kt_, fill_, q_lo_ + g)                            \
        }                                                                                       \
    }

    // ---- prologue: AHEAD tiles in flight (EARLY: every stage of the ring)
    constexpr int AHEAD = EARLY ? STAGES : STAGES - 1;
#define FV_ISSUE_PROLOGUE()                                                                     \
    _Pragma("unroll") for (int s = 0; s < AHEAD; ++s)                                           \
        if (s < KT) FV_ISSUE_TILE(s, s)
    FV_ISSUE_PROLOGUE()
    bool first_tile = true;
    for (;;) {   // the tiles of this workgroup
    // The accumulators start from the bias, which saves the epilogue an add per element; with K split between
    // k-groups or workgroups only the first slice carries it.  (Accumulator blocks hold C transposed, see the
    // epilogue: register r of a lane is column 8*(r/4) + 4*(lane/32) + r%4 of the block.)
    f32x16_t acc[MI][NI];
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        float b16[16];
#pragma unroll
        for (int g = 0; g < 4; ++g) {
            const int n = n0 + wn * WTN + ni * 32 + 8 * g + 4 * (lane >> 5);
            u32x2_t bb = {0u, 0u};
            if (p.bias && n < p.N && kg == 0 && split == 0) bb = *reinterpret_cast<const u32x2_t*>(p.bias + n);
            b16[4 * g + 0] = bf16_lo(bb.x); b16[4 * g + 1] = bf16_hi(bb.x);
            b16[4 * g + 2] = bf16_lo(bb.y); b16[4 * g + 3] = bf16_hi(bb.y);
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mi][ni][r] = b16[r];
    }

    // ---- wait for the first K tile.  (A later tile of a persistent workgroup waits for everything: its
    // loads went out before the previous epilogue's stores and residual loads, and the counter says
    // nothing about the order in which loads and stores complete.)
    if (first_tile && KT >= AHEAD)
        __builtin_amdgcn_s_waitcnt(waitcnt_imm((AHEAD - 1) * LPT, true));
    else
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
    asm volatile("" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");

    bf16x8_t fa[2][MI], fw[2][NI];
    FV_LOAD_FRAGS(fa[0], fw[0], 0, 0)

#define FV_MFMA_ROWS(cur_, mi_lo_, mi_hi_)                                                      \
    _Pragma("unroll") for (int mi = (mi_lo_); mi < (mi_hi_); ++mi)                              \
        _Pragma("unroll") for (int ni = 0; ni < NI; ++ni)                                       \
            acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[cur_][ni], fa[cur_][mi],   \
                                                                  acc[mi][ni], 0, 0, 0);
#define FV_INTERLEAVE(mfma_per_read_, with_dma_)                                                \
    _Pragma("unroll") for (int g = 0; g < MI + NI; ++g) {                                       \
        __builtin_amdgcn_sched_group_barrier(0x008, (mfma_per_read_), 0); /* MFMA */            \
        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                /* DS read */         \
        if (with_dma_) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0); /* direct-to-LDS load */ \
    }
    // One K tile.  Software pipeline inside the wave: the operand reads of the
    // next k-step are interleaved with the MFMAs of the current one (the
    // scheduler is told the pattern), so LDS latency hides behind the matrix
    // pipe.  HANDOVER_: a next tile exists, so the last k-step waits for it (this
    // wave's loads: the counter, at most WAITN_ loads of later tiles still in
    // flight; the other waves' loads: the barrier, which also tells everyone that
    // this tile's stage is no longer being read) and preloads its first operands.
    // MORE_: a further tile is fetched, AHEAD tiles on: into the stage this tile
    // leaves, at its hand-over (EARLY), or into the stage the tile before it left,
    // during its first k-steps.  The body is branch free on purpose: the
    // accumulators must stay in one register class across the loop.
#define FV_TILE_BODY(MORE_, HANDOVER_, WAITN_)                                                  \
    {                                                                                           \
        int next_stage_ = stage + 1;                                                            \
        if (next_stage_ == STAGES) next_stage_ = 0;                                             \
        int fill_ = stage + STAGES - 1;                                                         \
        if (fill_ >= STAGES) fill_ -= STAGES;                                                   \
        _Pragma("unroll") for (int kk = 0; kk < KK; ++kk) {                                     \
            const int cur_ = kk & 1, nxt_ = cur_ ^ 1;                                           \
            if (kk + 1 < KK) {                                                                  \
                if ((MORE_) && !EARLY)                                                          \
                    FV_LOAD_FRAGS_ISSUE_PART(fa[nxt_], fw[nxt_], stage, kk + 1, kt + AHEAD, fill_, kk, KK - 1) \
                else                                                                            \
                    FV_LOAD_FRAGS(fa[nxt_], fw[nxt_], stage, kk + 1)                            \
                FV_MFMA_ROWS(cur_, 0, MI)                                                       \
                FV_INTERLEAVE((MI * NI) / (MI + NI), false)                                     \
            } else if (HANDOVER_) {                                                             \
                __builtin_amdgcn_s_waitcnt(waitcnt_imm((WAITN_), true));                        \
                asm volatile("" ::: "memory");                                                  \
                __builtin_amdgcn_s_barrier();                                                   \
                asm volatile("" ::: "memory");                                                  \
                if ((MORE_) && EARLY)                                                           \
                    FV_LOAD_FRAGS_ISSUE(fa[nxt_], fw[nxt_], next_stage_, 0, kt + AHEAD, stage)  \
                else                                                                            \
                    FV_LOAD_FRAGS(fa[nxt_], fw[nxt_], next_stage_, 0)                           \
                FV_MFMA_ROWS(cur_, 0, MI)                                                       \
                FV_INTERLEAVE((MI * NI) / (MI + NI), false)                                     \
            } else {                                                                            \
                FV_MFMA_ROWS(cur_, 0, MI)                                                       \
            }                                                                                   \
        }                                                                                       \
        stage = next_stage_;                                                                    \
    }

    int stage = 0;  // stage of tile kt
    int kt = 0;
    for (; kt + AHEAD < KT; ++kt) FV_TILE_BODY(true, true, (STAGES - 2) * LPT)
    // the ring drains: r tiles are left after this one, r-1 of them may still be in flight at the hand-over
    static_for<0, AHEAD - 1>([&](auto i_c) {
        constexpr int r = AHEAD - 1 - decltype(i_c)::value;
        if (KT - 1 - kt == r) {
            FV_TILE_BODY(false, true, (r - 1) * LPT)
            ++kt;
        }
    });
    FV_TILE_BODY(false, false, 0)

    // ---- the seam of a persistent workgroup: once every wave has read its last operands, the next tile's
    // first stages are fetched; the epilogue of this tile (m0e, n0e) runs under their flight
    const int m0e = m0, n0e = n0;
    const int vnext = vpid + (int)gridDim.x;
    const bool has_next = PERSIST && vnext < n_tiles;
    if (has_next) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(63, true));
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
        FV_TILE_COORDS(vnext)
        FV_TILE_OFFSETS()
        FV_ISSUE_PROLOGUE()
    }

    // ---- Epilogue, from registers.  The MFMAs take the W fragment as their first operand, so an accumulator
    // block holds C transposed: register r of lane l is C[row, col] with row = l % 32 and
    // col = 8*(r/4) + 4*(l/32) + r%4 inside a 32x32 block: a lane owns one output row and four runs of four
    // consecutive columns.  GELU, residual (an 8-byte load per run) and rotary turn are applied in fp32, the
    // runs are rounded once to bf16, and one half-wave exchange (v_permlane32_swap) per pair of runs leaves
    // every lane with two runs of eight consecutive columns: two 16-byte stores per block, no staging through
    // LDS and no barrier between the main loop and the stores (a wave that is done stores while the others
    // still multiply).  The V section of the QKV GEMM is stored along the token axis of the transposed cache:
    // there consecutive lanes are consecutive tokens, 2-byte stores that a half-wave makes 64 contiguous bytes.
    constexpr int XCH = KG > 1 ? MI * NI * 16 * 64 * NWQ : 0;  // floats handed over by the other k-groups
    static_assert(XCH * 4 <= STAGES * (BM + BN) * BK * 2, "the k-group exchange must fit in the tile LDS");
    if (KG > 1 || SK) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
        __builtin_amdgcn_s_barrier();  // every wave is done reading operand tiles: LDS is free for the exchange
        asm volatile("" ::: "memory");
    }
    if (KG > 1) {
        // Sum the k-groups: group g > 0 writes its accumulators (register-major, lane
        // contiguous), group 0 adds them; only group 0 goes on to the epilogue.
        float* xch = reinterpret_cast<float*>(smem) + wq * (MI * NI * 16 * 64) + lane;
        for (int g = 1; g < KG; ++g) {
            if (kg == g) {
                static_for<0, MI * NI * 16>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    xch[i * 64] = acc[i / (NI * 16)][(i / 16) % NI][i % 16];
                });
            }
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            if (kg == 0) {
                static_for<0, MI * NI * 16>([&](auto i_c) {
                    constexpr int i = decltype(i_c)::value;
                    acc[i / (NI * 16)][(i / 16) % NI][i % 16] += xch[i * 64];
                });
            }
            if (g + 1 < KG) {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));
                __builtin_amdgcn_s_barrier();
                asm volatile("" ::: "memory");
            }
        }
        if (kg != 0) return;  // no barrier follows
    }
    if (SK && CF) {
        // Large partial tiles (256x128 fp32 = 128 KB): count first, store only if not last.  A slice counts
        // itself in at the tile's counter; every slice but the last to arrive then leaves its partial tile,
        // waits until its stores have been acknowledged and reports ready; the last to arrive keeps its own
        // accumulators, polls the ready count (the others are running and past their K loops: the wait is short
        // and always ends, and it is bounded all the same), adds the slices up in slice order and runs the
        // epilogue.  Half the stores of the other order, and none on the last arriver's path.  (For the few-KB
        // partials of the few-row shapes a poll costs more than the stores it saves: they keep the order below.)
        float* part = p.sk_part + ((size_t)blockIdx.x * n_splits) * (BM * BN) + wq * 64 + lane;
        int* flag = reinterpret_cast<int*>(smem);
        if (tid == 0)
            *flag = __hip_atomic_fetch_add(p.sk_cnt + blockIdx.x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int arrived = *flag;
        if (arrived != n_splits - 1) {
            float* mine = part + (size_t)split * (BM * BN);
            static_for<0, MI>([&](auto mi_c) {
                constexpr int mi = decltype(mi_c)::value;
                if (m0e + wm * WTM + mi * 32 < p.M) {
                    static_for<0, NI * 16>([&](auto j_c) {
                        constexpr int j = decltype(j_c)::value;
                        __hip_atomic_store(mine + (mi * NI * 16 + j) * (NWQ * 64), acc[mi][j / 16][j % 16],
                                           __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    });
                }
            });
            asm volatile("" ::: "memory");
            __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));   // own stores acknowledged
            __syncthreads();
            if (tid == 0)
                __hip_atomic_fetch_add(p.sk_ready + blockIdx.x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            return;
        }
        if (tid == 0) {
            // about a microsecond per look; the bound is never reached by a launch that is making progress
            for (int looks = 0; looks < (1 << 20); ++looks) {
                if (__hip_atomic_load(p.sk_ready + blockIdx.x, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) ==
                    n_splits - 1)
                    break;
                __builtin_amdgcn_s_sleep(8);
            }
            // ready for the next launch
            __hip_atomic_store(p.sk_cnt + blockIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __hip_atomic_store(p.sk_ready + blockIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        __syncthreads();
        // slice order, this workgroup's own slice from its registers
        static_for<0, MI>([&](auto mi_c) {
            constexpr int mi = decltype(mi_c)::value;
            if (m0e + wm * WTM + mi * 32 < p.M) {
                float sum[NI * 16];
                _Pragma("unroll") for (int j = 0; j < NI * 16; ++j) sum[j] = 0.f;
                for (int sl = 0; sl < n_splits; ++sl) {
                    if (sl == split) {
                        static_for<0, NI * 16>([&](auto j_c) {
                            constexpr int j = decltype(j_c)::value;
                            sum[j] += acc[mi][j / 16][j % 16];
                        });
                    } else {
                        const float* src = part + (size_t)sl * (BM * BN) + (mi * NI * 16) * (NWQ * 64);
                        float v[NI * 16];
                        _Pragma("unroll") for (int j = 0; j < NI * 16; ++j)
                            v[j] = __hip_atomic_load(src + j * (NWQ * 64), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        _Pragma("unroll") for (int j = 0; j < NI * 16; ++j) sum[j] += v[j];
                    }
                }
                static_for<0, NI * 16>([&](auto j_c) {
                    constexpr int j = decltype(j_c)::value;
                    acc[mi][j / 16][j % 16] = sum[j];
                });
            }
        });
    }
    if (SK && !CF) {
        // Leave this slice's partial tile (register-major, lane contiguous), then count arrivals;
        // 32-row blocks that lie entirely past M (most of the tile at the small scales) are skipped.
        // The partial tiles and the counter are written and read with device-scope atomic accesses
        // (relaxed): those are coherent across the chip's L2s by themselves, so no cache write-back
        // or invalidate is needed (a device-scope fence in each of 256 workgroups costs 7 us per
        // GEMM here).  Order: every thread waits until its own stores have been acknowledged, the
        // barrier collects the workgroup, and only then one thread counts the workgroup in.
        float* part = p.sk_part + ((size_t)blockIdx.x * n_splits) * (BM * BN) + wq * 64 + lane;
        float* mine = part + (size_t)split * (BM * BN);
        static_for<0, MI>([&](auto mi_c) {
            constexpr int mi = decltype(mi_c)::value;
            if (m0e + wm * WTM + mi * 32 < p.M) {
                static_for<0, NI * 16>([&](auto j_c) {
                    constexpr int j = decltype(j_c)::value;
                    __hip_atomic_store(mine + (mi * NI * 16 + j) * (NWQ * 64), acc[mi][j / 16][j % 16],
                                       __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                });
            }
        });
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(waitcnt_imm(0, true));   // own stores acknowledged
        int* flag = reinterpret_cast<int*>(smem);
        __syncthreads();
        if (tid == 0)
            *flag = __hip_atomic_fetch_add(p.sk_cnt + blockIdx.x, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __syncthreads();
        const int arrived = *flag;
        __syncthreads();                 // the flag's LDS word is staging memory below
        if (arrived != n_splits - 1) return;
        // sum the slices in slice order; several slices' loads in flight at a time (128 registers' worth)
        static_for<0, MI>([&](auto mi_c) {
            constexpr int mi = decltype(mi_c)::value;
            if (m0e + wm * WTM + mi * 32 < p.M) {
                float sum[NI * 16];
                _Pragma("unroll") for (int j = 0; j < NI * 16; ++j) sum[j] = 0.f;
                constexpr int SG = 8 / NI > 0 ? 8 / NI : 1;
                for (int s0 = 0; s0 < n_splits; s0 += SG) {
                    float v[SG][NI * 16];
                    _Pragma("unroll") for (int g = 0; g < SG; ++g) {
                        const int sl = min(s0 + g, n_splits - 1);
                        const float* src = part + (size_t)sl * (BM * BN) + (mi * NI * 16) * (NWQ * 64);
                        _Pragma("unroll") for (int j = 0; j < NI * 16; ++j)
                            v[g][j] = __hip_atomic_load(src + j * (NWQ * 64), __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                    _Pragma("unroll") for (int g = 0; g < SG; ++g) {
                        if (s0 + g < n_splits) {
                            _Pragma("unroll") for (int j = 0; j < NI * 16; ++j) sum[j] += v[g][j];
                        }
                    }
                }
                static_for<0, NI * 16>([&](auto j_c) {
                    constexpr int j = decltype(j_c)::value;
                    acc[mi][j / 16][j % 16] = sum[j];
                });
            }
        });
        if (tid == 0)   // ready for the next launch
            __hip_atomic_store(p.sk_cnt + blockIdx.x, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    const int lrow = lane & 31;            // output row inside a 32-row block
    static_for<0, MI>([&](auto mi_c) {
        constexpr int mi = decltype(mi_c)::value;
        const int m = m0e + wm * WTM + mi * 32 + lrow;
        const bool row_ok = m < p.M;
        const int mc = row_ok ? m : p.M - 1;
        // (sample, token) of this lane's row, where its output goes and where its residual comes from
        int bq = 0, tq = mc;
        if (is_qkv(EPI)) {
            bq = mc / p.k_tokens;
            tq = mc - bq * p.k_tokens;
        }
        size_t orow = (size_t)mc, rrow = (size_t)mc;
        if (EPI == EPI_BIAS_RES) {
            if (p.out_rows) orow = (size_t)p.out_rows[mc];
            if (p.res_rows) rrow = (size_t)p.res_rows[mc];
        }
        int slot = tq;   // rotary: the token's slot in its map
        if (EPI == EPI_QKV_ROPE && p.rope_rows) slot = p.rope_rows[mc] % p.rope_N;
        static_for<0, NI>([&](auto ni_c) {
            constexpr int ni = decltype(ni_c)::value;
            const int nb = n0e + wn * WTN + ni * 32;      // first column of the block (wave uniform)
            if (nb >= p.N) return;                       // N % 32 may be non-zero only past whole 8-column groups: checked per group below
            // QKV: section, head and channel of the block's first column (wave uniform: scalar arithmetic); the
            // 32 columns of a block lie in one section and one head (D and dh are multiples of 32)
            int sec = 0, f0 = 0, hh0 = 0, d0 = 0;
            if (is_qkv(EPI)) {
                sec = nb / p.D;
                f0 = nb - sec * p.D;
                hh0 = f0 / p.dh;
                d0 = f0 - hh0 * p.dh;
            }
            if (is_qkv(EPI) && sec == 2) {
                // V section: v_cache[b, head, d, L0 + t], consecutive lanes = consecutive tokens
                if (row_ok) {
                    bf16_t* const v0 = p.v_cache + (((size_t)bq * p.H + hh0) * p.dh + d0) * p.L_cap + p.L0 + tq;
                    static_for<0, 16>([&](auto r_c) {
                        constexpr int r = decltype(r_c)::value;
                        const int col = 8 * (r >> 2) + 4 * frag_half + (r & 3);
                        if (nb + col < p.N) v0[(size_t)col * p.L_cap] = (bf16_t)f32_to_bf16_bits(acc[mi][ni][r]);
                    });
                }
                return;
            }
            // four runs of four columns -> packed bf16 pairs
            uint32_t pk[4][2];
            static_for<0, 4>([&](auto g_c) {
                constexpr int g = decltype(g_c)::value;
                const int n = nb + 8 * g + 4 * frag_half;     // first column of this lane's run
                float v[4] = {acc[mi][ni][4 * g + 0], acc[mi][ni][4 * g + 1], acc[mi][ni][4 * g + 2], acc[mi][ni][4 * g + 3]};
                if (EPI == EPI_BIAS_GELU) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[j] = gelu_fast(v[j]);
                }
                if (EPI == EPI_BIAS_RES && n < p.N) {
                    const u32x2_t rr = *reinterpret_cast<const u32x2_t*>(p.residual + rrow * p.N + n);
                    v[0] += bf16_lo(rr.x); v[1] += bf16_hi(rr.x);
                    v[2] += bf16_lo(rr.y); v[3] += bf16_hi(rr.y);
                }
                if (EPI == EPI_QKV_ROPE && n < p.N) {
                    // two interleaved pairs of one head, turned by the angles of the token's slot
                    const int d = d0 + 8 * g + 4 * frag_half;
                    const size_t at = (size_t)slot * (p.dh >> 1) + (d >> 1);
                    const f32x2_t cs = *reinterpret_cast<const f32x2_t*>(p.rope_cos + at);
                    const f32x2_t sn = *reinterpret_cast<const f32x2_t*>(p.rope_sin + at);
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const float a = v[2 * j], b = v[2 * j + 1];
                        v[2 * j] = a * cs[j] - b * sn[j];
                        v[2 * j + 1] = a * sn[j] + b * cs[j];
                    }
                }
                pk[g][0] = pack_bf16x2(v[0], v[1]);
                pk[g][1] = pack_bf16x2(v[2], v[3]);
            });
            // exchange between the half-waves: the lower half gives its odd runs and takes the upper half's
            // even runs, so that the lower half holds columns 0-7 and 16-23 of its row, the upper half 8-15
            // and 24-31
#pragma unroll
            for (int pr = 0; pr < 2; ++pr)
#pragma unroll
                for (int c = 0; c < 2; ++c) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(pk[2 * pr][c], pk[2 * pr + 1][c], false, false);
                    pk[2 * pr][c] = sw[0];
                    pk[2 * pr + 1][c] = sw[1];
                }
#pragma unroll
            for (int pr = 0; pr < 2; ++pr) {
                const int n8 = nb + 16 * pr + 8 * frag_half;      // first of this lane's eight columns
                if (row_ok && n8 < p.N) {
                    const u32x4_t o = {pk[2 * pr][0], pk[2 * pr][1], pk[2 * pr + 1][0], pk[2 * pr + 1][1]};
                    bf16_t* dst;
                    if (is_qkv(EPI)) {
                        const int off = 16 * pr + 8 * frag_half;
                        if (sec == 0)   // q_out [B*k, D]
                            dst = p.q_out + ((size_t)bq * p.k_tokens + tq) * p.D + f0 + off;
                        else            // k_cache [B, H, L_cap, dh]
                            dst = p.k_cache + (((size_t)bq * p.H + hh0) * p.L_cap + p.L0 + tq) * p.dh + d0 + off;
                    } else {
                        dst = p.out + orow * p.N + n8;
                    }
                    *reinterpret_cast<u32x4_t*>(dst) = o;
                }
            }
        });
    });
    if (!has_next) break;
    vpid = vnext;
    first_tile = false;
    }   // the tiles of this workgroup
#undef FV_TILE_BODY
#undef FV_INTERLEAVE
#undef FV_MFMA_ROWS
#undef FV_ISSUE_PROLOGUE
#undef FV_ISSUE_TILE
#undef FV_ISSUE_Q
#undef FV_DMA16
#undef FV_LOAD_FRAGS_ISSUE_PART
#undef FV_LOAD_FRAGS_ISSUE
#undef FV_LOAD_FRAGS
#undef FV_TILE_OFFSETS
#undef FV_TILE_COORDS
#endif
}

// Compute units of the current device (asked once per process and device).
inline int compute_units() {
    static std::mutex mu;
    static int cus[64] = {0};
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    std::lock_guard<std::mutex> lock(mu);
    if (cus[dev] == 0) {
        int n = 0;
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cus[dev] = n;
    }
    return cus[dev];
}

template <int BM, int BN, int BK, int STAGES, int WGM, int WGN, int KG, int EPI, bool SK = false, bool CF = false>
void launch_cfg(GemmParams& p, hipStream_t stream) {
    constexpr size_t smem = (size_t)STAGES * (BM + BN) * BK * sizeof(bf16_t);
    p.tiles_m = (p.M + BM - 1) / BM;
    p.tiles_n = (p.N + BN - 1) / BN;
    static std::once_flag once;  // raising the dynamic-LDS limit is per function, once per process
    raise_lds_limit_once(once, &gemm_nt_kernel<BM, BN, BK, STAGES, WGM, WGN, KG, EPI, SK, CF>, smem);
    if (!SK) p.splits = 1;
    // one round of workgroups when there are more tiles than the chip holds at a time (the kernel then walks
    // the rest itself); as many workgroups per CU as fit into its 160 KB of LDS
    int grid = p.tiles_m * p.tiles_n;
    if (kPersistent<EPI, KG, SK>) {
        constexpr int per_cu = (int)((160u << 10) / smem) > 0 ? (int)((160u << 10) / smem) : 1;
        const int slots = compute_units() * per_cu;
        if (grid > slots && slots % 8 == 0) grid = slots;
    }
    gemm_nt_kernel<BM, BN, BK, STAGES, WGM, WGN, KG, EPI, SK, CF>
        <<<dim3(grid, SK ? p.splits : 1), 64 * WGM * WGN * KG, smem, stream>>>(p);
}

__global__ void zero_i32_kernel(int32_t* p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

// Tuning builds only (-DFASTVAR_DEV_KNOBS, never the product library, which reads no environment and keeps
// no state): FASTVAR_GEMM_CFG (all epilogues) or FASTVAR_GEMM_CFG<e> (epilogue e = 0, 1, 2) forces a tile
// configuration; unset means the heuristic below.
int gemm_cfg_override(int epi) {
#ifdef FASTVAR_DEV_KNOBS
    char name[32];
    snprintf(name, sizeof(name), "FASTVAR_GEMM_CFG%d", epi);
    const char* e = getenv(name);
    if (!e) e = getenv("FASTVAR_GEMM_CFG");
    return e ? atoi(e) : -1;
#else
    (void)epi;
    return -1;
#endif
}

// Tile choice.  What the measurements on the block's shapes say (inside the running step):
//  * what a tile's loads need is time to land.  A ring refilled during the tile after the hand-over gives them
//    STAGES-2 tiles and a fraction: nothing to speak of with two stages, which is all that 256x256 and 256x192
//    tiles fit into 160 KB.  Those rings are therefore refilled at the hand-over itself (one whole tile ahead:
//    256x192 at 2048 rows 60 -> 52 us, 256x256 68 -> 61 us); rings of three and four stages, which have the
//    time anyway, lose 3-5 % to the burst of loads at the hand-over and keep the spread refill.
//  * 256x128 tiles with eight waves of 64x64 and three stages are as fast per output element as the wide tiles
//    and twice as fine grained; the same tile with two stages and the spread refill, or with 32-wide K tiles in
//    four or six stages (twice the hand-overs), is 20-25 % slower; 128x128 with 128-wide K tiles in two stages
//    20 % slower than with 64-wide ones in four.
//  * 256x256 (QKV: 256x192, N = 3D divides evenly) wins where its tiles fill whole rounds of the 256 CUs, as
//    at 2048 kept tokens; 128x128 tiles with eight waves of 64x32 and four stages where the wide tiles would
//    leave CUs idle (N = D: out-proj, FC2); 192x128 (four waves of 96x64, three stages) where it makes the
//    tile count come out even (3072 rows x 2048 columns = 256 tiles).
//  * a part-filled last round costs less than a full one (fewer workgroups share the memory system and the
//    power budget).
//  * shapes that give at most 128 tiles of 128x128 (few rows) use 128x64 tiles, at most 64 use 64x64 tiles:
//    more workgroups streaming the weights beat the better operand reuse of the larger tile.
// The choice is the candidate with the least modelled time, rounds * (fix + K tiles * per-tile), a part-filled
// round counting 0.85 + 0.29 * fill; the constants are a least-squares fit to the in-step times of the four
// GEMMs of fifteen workloads under each configuration (residual 7 % rms; the picks cost 0.3 % more than the
// best measured configuration of every shape would).
int gemm_choose_cfg(bool qkv, int M, int N, int K) {
    const long tiles128 = (long)((M + 127) / 128) * ((N + 127) / 128);
    if (tiles128 <= 64) return 16;
    if (tiles128 <= 128) return 17;
    struct Cand { int cfg, bm, bn, slots; double fix, per_kt; };
    const Cand cands[] = {
        {qkv ? 12 : 11, 256, qkv ? 192 : 256, 256, 4.0, qkv ? 1.33 : 1.60},
        {32, 256, 128, 256, 10.3, 0.714},
        {34, 192, 128, 256, 9.5, 0.575},
        {40, 128, 128, 256, 6.2, 0.456},
        {6, 128, 128, 512, 8.0, 1.0},     // two workgroups per CU share its time
    };
    const double KT = (double)K / 64.0;
    int best_cfg = 6;
    double best = 1e30;
    for (const Cand& c : cands) {
        double per_kt = c.per_kt;
        if (c.bm == 256 && c.bn >= 192) {
            // the two-stage wide tiles lose ground on long K ranges (1.8 us per K tile at K = 8192) and were
            // never ahead on narrow outputs (N = D: eight tile columns, 4 x 1638 rows 80.7 us against 64.7 modelled
            // for 256x128)
            if ((N + c.bn - 1) / c.bn < 16) continue;
            if (KT > 32.0) per_kt += 0.003 * (KT - 32.0);
        }
        const long tiles = (long)((M + c.bm - 1) / c.bm) * ((N + c.bn - 1) / c.bn);
        const long full = tiles / c.slots, rem = tiles - full * c.slots;
        const double rounds = (double)full + (rem ? 0.85 + 0.29 * (double)rem / c.slots : 0.0);
        const double t = rounds * (c.fix + KT * per_kt);
        if (t < best) { best = t; best_cfg = c.cfg; }
    }
    return best_cfg;
}

template <int EPI>
void launch_epi(GemmParams& p, hipStream_t stream) {
    int cfg = gemm_choose_cfg(is_qkv(EPI), p.M, p.N, p.K);
    constexpr int knob = EPI == EPI_QKV_ROPE ? (int)EPI_QKV : EPI;
    if (gemm_cfg_override(knob) >= 0) cfg = gemm_cfg_override(knob);
    if (p.sk_part && gemm_cfg_override(knob) < 0) {
        // few output tiles: split K between workgroups (the caller sized the scratch with the same plan)
        const SplitKPlan sk = gemm_splitk_plan(p.M, p.N, p.K);
        if (sk.splits > 1) {
            p.splits = sk.splits;
            if (sk.shape == 0) launch_cfg<64, 64, 64, 8, 2, 2, 1, EPI, true>(p, stream);
            // (128x128: two long slices run best on the eight-wave four-stage tile, four short ones on the
            // four-wave three-stage one: FC2 at 576 / 960 rows 48.9 -> 46.5 / 49.6 -> 48.0 us, at 400 rows 33.9 vs 35.1)
            else if (sk.shape == 1 && sk.splits == 2) launch_cfg<128, 128, 64, 4, 2, 4, 1, EPI, true>(p, stream);
            else if (sk.shape == 1) launch_cfg<128, 128, 64, 3, 2, 2, 1, EPI, true>(p, stream);
            else launch_cfg<256, 128, 64, 3, 4, 2, 1, EPI, true, true>(p, stream);
            return;
        }
    }
    switch (cfg) {
        case 11: launch_cfg<256, 256, 64, 2, 2, 4, 1, EPI>(p, stream); break;
        case 12: launch_cfg<256, 192, 64, 2, 4, 2, 1, EPI>(p, stream); break;
        case 16: launch_cfg<64, 64, 64, 4, 2, 2, 1, EPI>(p, stream); break;
        case 17: launch_cfg<128, 64, 64, 3, 2, 2, 1, EPI>(p, stream); break;
        case 32: launch_cfg<256, 128, 64, 3, 4, 2, 1, EPI>(p, stream); break;
        case 34: launch_cfg<192, 128, 64, 3, 2, 2, 1, EPI>(p, stream); break;
        case 40: launch_cfg<128, 128, 64, 4, 2, 4, 1, EPI>(p, stream); break;
#ifdef FASTVAR_DEV_KNOBS
        case 7: launch_cfg<128, 128, 64, 3, 2, 2, 1, EPI>(p, stream); break;
        case 37: launch_cfg<256, 128, 64, 2, 4, 2, 1, EPI>(p, stream); break;
        case 39: launch_cfg<256, 128, 32, 4, 4, 2, 1, EPI>(p, stream); break;
#endif
        default: launch_cfg<128, 128, 64, 2, 2, 2, 1, EPI>(p, stream); break;   // 6: two workgroups per CU
    }
}

}  // namespace

SplitKPlan gemm_splitk_plan(int M, int N, int K) {
    SplitKPlan sk;
    // Up to 256 rows the tiles are 64x64 (eight stages): at those row counts the GEMMs stream their weights,
    // and what counts is how many workgroups pull on them.  Measured inside 32-block steps of the large model
    // (us per launch, 144 / 256 rows): out-proj 13.1 / 14.1 against 21.0 / 21.1 with 128x128 tiles on four
    // slices, FC2 23.4 / 28.4 against 31.4 / 35.3.  Above that, 128x128 tiles split K only where K is long
    // (FC2): with K = 2048 a slice is 8-16 K tiles and the summing costs more than it saves (out-proj at
    // 400 / 576 rows: 21.3 / 23.8 split, 14.9 / 20.6 whole).
    const bool small = M <= 256;
    sk.shape = small ? 0 : 1;
    const int t = small ? 64 : 128;
    sk.tile_m = sk.tile_n = t;
    sk.tiles = ((M + t - 1) / t) * ((N + t - 1) / t);
    sk.splits = 1;
    const int KT = K / 64;
    const int min_kt = small ? 2 : 4;   // K tiles a slice must keep
    // a short K range is over before the slices' summing would pay for itself
    static_assert(kSplitKMaxTiles >= 128 && (kSplitKMaxTiles * 4) % 256 == 0, "covers the tile-count limit below");
    if (K >= (small ? 2048 : 4096) && sk.tiles <= 128)
        while (sk.splits < (small ? 8 : 4) && sk.tiles * sk.splits * 2 <= 256 &&
               KT % (sk.splits * 2) == 0 && KT / (sk.splits * 2) >= min_kt)
            sk.splits *= 2;   // (more slices than that cost more to sum than they save)
    if (sk.splits == 1 && !small && K >= 8192 && KT % 2 == 0) {
        // A long K over a narrow output with a few too many rows for the above (FC2 at 1100-1500 rows): 128x128
        // tiles would fill a little over half of the chip, at the lowest efficiency of the tile shapes; 256x128
        // tiles on two K slices fill two thirds to three quarters of it and run the main loop a quarter faster,
        // and with the count-first exchange (see the kernel) their 128 KB partial tiles cost less than that
        // gain: 1152 rows 68.7 -> 60.2 us.  With more tiles the exchanged bytes win: 1638 rows 70.1 -> 69.1,
        // 2048 rows 73.1 -> 79.7 (32 MB of partial tiles); those stay on 128x128 tiles unsplit.
        const int tiles = ((M + 255) / 256) * ((N + 127) / 128);
        if (tiles * 2 >= 160 && tiles * 2 <= 192) {
            sk.shape = 2;
            sk.tile_m = 256; sk.tile_n = 128;
            sk.tiles = tiles;
            sk.splits = 2;
        }
    }
    // The counter area has one size for every shape (the most tiles the conditions above admit): the
    // GEMMs of a block share one scratch area, and a partial tile of one must never land on a counter
    // of another.
    sk.counter_bytes = sk.splits > 1 ? (size_t)kSplitKMaxTiles * 8 : 0;   // arrivals, then ready counts
    sk.bytes = sk.splits > 1 ? sk.counter_bytes + (size_t)sk.tiles * sk.splits * sk.tile_m * sk.tile_n * 4 : 0;
    return sk;
}

void launch_zero_i32(int32_t* p, int n, hipStream_t stream) {
    if (n > 0) zero_i32_kernel<<<(n + 255) / 256, 256, 0, stream>>>(p, n);
}

void launch_gemm(GemmEpilogue epi, const GemmArgs& a, hipStream_t stream) {
    GemmParams p;
    p.A = static_cast<const bf16_t*>(a.A);
    p.W = static_cast<const bf16_t*>(a.W);
    p.bias = static_cast<const bf16_t*>(a.bias);
    p.M = a.M; p.N = a.N; p.K = a.K;
    p.out = static_cast<bf16_t*>(a.out);
    p.residual = static_cast<const bf16_t*>(a.residual);
    p.res_rows = a.res_rows;
    p.out_rows = a.out_rows;
    p.q_out = static_cast<bf16_t*>(a.q_out);
    p.k_cache = static_cast<bf16_t*>(a.k_cache);
    p.v_cache = static_cast<bf16_t*>(a.v_cache);
    p.D = a.D; p.H = a.H; p.dh = a.dh; p.k_tokens = a.k_tokens; p.L0 = a.L0; p.L_cap = a.L_cap;
    p.rope_cos = a.rope_cos; p.rope_sin = a.rope_sin; p.rope_rows = a.rope_rows; p.rope_N = a.rope_N;
    p.tiles_m = p.tiles_n = 0;
    p.splits = 1;
    p.sk_part = nullptr;
    p.sk_cnt = nullptr;
    p.sk_ready = nullptr;
    if (a.splitk_ws) {
        const SplitKPlan sk = gemm_splitk_plan(a.M, a.N, a.K);
        if (sk.splits > 1) {
            p.sk_cnt = static_cast<int*>(a.splitk_ws);
            p.sk_ready = p.sk_cnt + kSplitKMaxTiles;
            p.sk_part = reinterpret_cast<float*>(static_cast<char*>(a.splitk_ws) + sk.counter_bytes);
        }
    }
    switch (epi) {
        case EPI_QKV:
            if (a.rope_cos) launch_epi<EPI_QKV_ROPE>(p, stream);
            else launch_epi<EPI_QKV>(p, stream);
            break;
        case EPI_BIAS_RES: launch_epi<EPI_BIAS_RES>(p, stream); break;
        case EPI_BIAS_GELU: launch_epi<EPI_BIAS_GELU>(p, stream); break;
    }
}

}  // namespace fv
