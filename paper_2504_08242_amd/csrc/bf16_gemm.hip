// bf16 GEMM  C[M, N] = A[M, K] * W[N, K]^T  for gfx950 with fused epilogues.
//
// Shape of the problem.  A chunk has at most a few hundred rows (M = n_tokens) while N is the layer
// width, so the work per compute unit is small: about 44 K outputs for the gate/up projection of a
// 512-token chunk on 256 CUs.  The kernel therefore gives every CU ONE tall tile, 256 rows by up to
// 192 columns, held entirely in accumulators (the register file of a CU is 512 KB), and sizes the
// tile width so that the number of tiles matches the number of CUs.  That is the largest tile the
// problem allows, which is what keeps the L2 -> LDS traffic per flop low.
//
//   * Waves form a WM x WN grid over the tile; a wave owns 8/WM row blocks x NB/WN column blocks of
//     32 x 32.  Measured at M = 512: eight waves (4 x 2, two per SIMD, 64 x 96 each) beat four waves of
//     128 x 96 (2 x 2) by 20 % although the latter read a third less from LDS: with one wave per SIMD
//     every wait of that wave idles the matrix pipe, with two the other wave's MFMAs cover it.
//     (The 16x16x32 form sustains only ~70 % of the 32x32x16 rate on this chip, measured.)
//   * K advances in stages of 32 through an LDS ring (as many slots as fit, at most 8) filled by direct global->LDS loads
//     (16 bytes per lane, no register staging).  A stage holds two K/16 sub-steps; the fragments of
//     one sub-step are read from LDS while the matrix cores work on the other.
//   * LDS rows are 64 bytes (32 bf16).  Four rows form a 256-byte super-row; chunk c of row r sits at
//     16-byte slot ((4*(r&3) + c) ^ ((r>>2)&3)) of super-row r>>2, so that 16 consecutive rows read at
//     one chunk column touch all 64 banks exactly once.
//   * Both operands are stored pre-tiled as [rows/32 row blocks][K/32 stages][2 KB], each 2 KB block being
//     the LDS image of its 32 rows x 32 columns, swizzle included (W at stage creation, activations by
//     the kernels that produce them).  A wave-wide load instruction then copies 1 KB of consecutive
//     bytes, which the L2 -> LDS path moves about three times faster than 16 pieces of 64 bytes, and a
//     workgroup streams each row block of W front to back in long sequential bursts.
//   * Workgroup ids are decoded so that the tiles sharing a slice of W run on the same XCD (same L2).
//   * The epilogues that write bf16 rows (QKV with rotary embedding and cache append, gate/up with SwiGLU) compute the
//     transposed product W A^T instead: the fragments are the same registers, only the MFMA's operand order changes,
//     and a lane then holds 16 output features of one token instead of 16 tokens of one feature.  With the weight
//     rows ordered for it at pack time a lane finishes its outputs alone (rotary partners, gate and up of a feature
//     sit in the same lane) and writes 16-byte pieces straight from registers.  The earlier epilogues went through a
//     wave-private LDS strip behind a workgroup barrier; measured at 512 rows: gate/up 85.8 -> 83.0 us, QKV unchanged
//     (its epilogue is bound by draining 16.7 MB of scattered 16-byte stores, with or without the strip).
//
// MFMA 32x32x16 bf16 operand layout (lane = 32*hh + c):
//   A: lane supplies A[m = c][k = 8*hh + e], e < 8;  B: lane supplies B[k = 8*hh + e][n = c];
//   D: lane holds D[m = 8*(i/4) + 4*hh + (i%4)][n = c] in register i < 16.
#include <cstdio>
#include <type_traits>
#include <utility>

#include "bf16_common.h"

namespace jup {
namespace {

constexpr int G_BK = 32;

constexpr int kLdsBudget = 160 * 1024;

template <int BMB, int NB, int WM, int WN>
struct Shape {
    static constexpr int BM = 32 * BMB;             // rows of the tile: 256 for prefill-sized chunks, 128, 64 or 32 for
                                                    // short ones (a short chunk is bound by streaming the weights:
                                                    // MFMAs on rows that do not exist would only slow that down)
    static constexpr int NBW = NB / WN;             // column blocks per wave
    static constexpr int MBW = BMB / WM;            // row blocks per wave
    static constexpr int WAVES = WM * WN;
    static constexpr int ROWS = BM + 32 * NB;       // LDS rows per stage: A rows then W rows
    static constexpr int STAGE_BYTES = ROWS * 64;
    static constexpr int LOADERS = WAVES;           // every wave fetches its share of a stage between its MFMAs
    static constexpr int THREADS = 64 * WAVES;
    static constexpr int NL = ROWS / 16;            // 1 KB load units (16 rows) per stage, dealt round-robin to the loading waves
    static constexpr int LPW = (NL + LOADERS - 1) / LOADERS;  // load instructions per stage of the waves that have the most
    static constexpr int REM = NL % LOADERS;        // loading waves below REM issue LPW loads, the others LPW - 1 (0: all LPW)
    static_assert(NB % WN == 0 && BMB % WM == 0, "tile does not split evenly over the waves");
    // as many ring slots as LDS holds (at most 8: the in-flight count must fit the 6-bit vmcnt)
    static constexpr int STAGES = kLdsBudget / STAGE_BYTES > 8 ? 8 : kLdsBudget / STAGE_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(STAGES >= 4 && (STAGES - 2) * LPW < 64, "ring depth");
};

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// s_waitcnt with only the vector-memory counter constrained.
template <int N>
__device__ inline void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit field");
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}
__device__ inline void wait_lgkmcnt0() { __builtin_amdgcn_s_waitcnt(0xC07F); }  // lgkmcnt(0), others free

// Instruction-order hints.  A burst of LDS reads or of global->LDS loads keeps the wave's issue port busy
// for hundreds of cycles while the matrix pipe drains, so memory instructions are dealt out one (or two)
// after each MFMA.  Masks: 0x008 MFMA, 0x100 LDS read, 0x010 vector memory.
template <int MASK>
__device__ __forceinline__ void sched_one() {
    __builtin_amdgcn_sched_group_barrier(MASK, 1, 0);
}
template <int DS, int LO, int HI>
__device__ __forceinline__ void sched_mem_ops() {  // memory ops number LO..HI-1 of a half: LDS reads first
    if constexpr (LO < HI) {
        if constexpr (LO < DS) sched_one<0x100>();
        else sched_one<0x010>();
        sched_mem_ops<DS, LO + 1, HI>();
    }
}
// One half stage: M MFMAs with DS LDS reads and VM vector-memory loads spread evenly behind them.
template <int M, int DS, int VM, int m = 0>
__device__ __forceinline__ void sched_half() {
    if constexpr (m < M) {
        sched_one<0x008>();
        sched_mem_ops<DS, (DS + VM) * m / M, (DS + VM) * (m + 1) / M>();
        sched_half<M, DS, VM, m + 1>();
    }
}

// Waits until at most g of this wave's load groups (one group = the CNT loads of one stage) are still in
// flight; more than ST - 3 are never allowed to be.
template <int ST, int CNT>
__device__ __forceinline__ void wait_groups(int g) {
    if (g >= ST - 3) wait_vmcnt<(ST - 3) * CNT>();
    else if (g == 4) wait_vmcnt<(ST > 7 ? 4 : 0) * CNT>();
    else if (g == 3) wait_vmcnt<(ST > 6 ? 3 : 0) * CNT>();
    else if (g == 2) wait_vmcnt<(ST > 5 ? 2 : 0) * CNT>();
    else if (g == 1) wait_vmcnt<1 * CNT>();
    else wait_vmcnt<0>();
}

// Fragments of one K/16 sub-step of a wave: MB row blocks, NB column blocks.
template <int MB, int NB>
struct Frags {
    bf16x8 a[MB];
    bf16x8 b[NB];
};

template <int BMB, int NB, int WM, int WN, int EPI>
__global__ __launch_bounds__(64 * WM * WN) void gemm_bf16(const GemmArgs a) {
    using S = Shape<BMB, NB, WM, WN>;
    constexpr int G_BM = S::BM;
    constexpr int NBW = S::NBW, MBW = S::MBW;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wm = wave % WM, wn = wave / WM;  // wave owns row blocks [wm MBW, +MBW) x column blocks [wn NBW, +NBW)
    const int lw = wave;

    // ---- which tile ---------------------------------------------------------------------------------
    // Workgroup b runs on XCD b % 8.  Tiles are numbered so that each XCD owns one contiguous range of
    // them, M tiles fastest: the workgroups that read the same weight rows (all M tiles of an N tile) and
    // neighbouring N tiles (same activation rows) then share one L2.
    int mt, grp;
    {
        const int q = gridDim.x >> 3, r = gridDim.x & 7;
        const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
        const int tile = xcd * q + min(xcd, r) + local;
        mt = tile % a.m_tiles;
        grp = tile / a.m_tiles;
    }
    const int nt = grp % a.n_tiles, split = grp / a.n_tiles;
    const int m0 = mt * G_BM, n0 = nt * a.n_stride;
    const int KT = a.kt_per_split;

    // ---- global -> LDS load slots of this wave --------------------------------------------------------
    // A stage is ROWS/4 super-rows of 256 bytes (4 rows of 64 bytes), A rows first, then W rows.  One load
    // instruction moves four super-rows: lane i's 16 bytes land at byte 16 i of the instruction's 1 KB.
    // Unit j of a stage = rows [16j, 16j+16) of the LDS image = 1 KB that is contiguous in the tiled operand
    // too (half a 2 KB block), so one load instruction is a wave-uniform base plus 16 bytes per lane.  Unit
    // j = q * LOADERS + lw belongs to loading wave lw; HAS_LAST says whether its unit q = LPW-1 exists.
    const char* ubase[S::LPW];
    const int kt_total = a.K / G_BK;
    const unsigned lane16 = lane * 16;
#pragma unroll
    for (int q = 0; q < S::LPW; ++q) {
        const int j = min(q * S::LOADERS + lw, S::NL - 1);
        const u16* base;
        int blk;
        if (j < G_BM / 16) {
            blk = min(m0 / 32 + (j >> 1), (a.M + 31) / 32 - 1);  // blocks past M repeat the last one
            base = a.A;
        } else {
            blk = min(n0 / 32 + ((j - G_BM / 16) >> 1), a.N / 32 - 1);  // blocks past N repeat the last one
            base = a.W;
        }
        ubase[q] = uniform_ptr((const char*)(base + ((size_t)blk * kt_total + (size_t)split * KT) * 1024 + (j & 1) * 512));
    }
    // (the 64-row tiles and the four-wave 128-row tiles are the ones short chunks run; the eight-wave 128-row tiles serve
    // 512-row chunks, whose K loop does not afford the branch below: 2 us per launch, measured)
    constexpr bool kShortChunkTile = BMB <= 2 || (BMB == 4 && WM * WN == 4);
    const bool nt_weights = a.m_tiles == 1 && !a.shared_gpu;
    auto issue_one = [&](int q, int stage, int kt) {
        const auto* src = (const __attribute__((address_space(1))) void*)(uniform_ptr(ubase[q] + (size_t)kt * 2048) + lane16);
        auto* dst = (__attribute__((address_space(3))) void*)(smem + stage * S::STAGE_BYTES + (q * S::LOADERS + lw) * 1024);
        // A chunk of up to 128 tokens alone on the chip streams every weight exactly once (one M tile): its weight units
        // are fetched with the non-temporal hint, so that the stream does not push the KV cache and the activations
        // out of L2 and the last-level cache.  Measured on the 7B shapes: gate/up at 5 rows 36.1 -> 32.5 us, the
        // attention launch behind the projections 15.0 -> 12.4 us, a 5-token call 6.59 -> 5.95 ms per 8 branches, 128-token
        // chunks +6 %.  Not for the tiles of longer chunks (the branch costs their K loop 2.5 % and a second M tile re-reads
        // the weights from L2) and not inside an overlapped call (the other chunks find the weights in the caches).
        if (kShortChunkTile && nt_weights && q * S::LOADERS + lw >= G_BM / 16) __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 2);
        else __builtin_amdgcn_global_load_lds(src, dst, 16, 0, 0);
    };
    auto issue = [&](auto has_last, int stage, int kt) {
        constexpr int CNT = S::REM == 0 || decltype(has_last)::value ? S::LPW : S::LPW - 1;
#pragma unroll
        for (int q = 0; q < CNT; ++q) issue_one(q, stage, kt);
    };

    constexpr bool FETCH = true;

    // ---- LDS -> register fragment addresses -------------------------------------------------------------
    // Fragment row = 32*block + c (c = lane & 31), chunk = 2*ks + hh.  Block bases are multiples of 32,
    // so the swizzle term depends on the lane and on ks only: address = lane part + constant.
    const int c = lane & 31, hh = lane >> 5;
    int lane_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        lane_off[ks] = (c >> 2) * 256 + ((((c & 3) << 2) + 2 * ks + hh) ^ ((c >> 2) & 3)) * 16;
    const int a_base = wm * MBW * 2048, b_base = G_BM * 64 + wn * NBW * 2048;
    // Read number t of a sub-step, in the order the MFMAs need them: a[0], b[0], the other a, the other b.
    auto load_frag_one = [&](Frags<MBW, NBW>& f, int stage, int ks, int t) {
        const unsigned char* sb = smem + stage * S::STAGE_BYTES + lane_off[ks];
        if (t == 0) f.a[0] = *(const bf16x8*)(sb + a_base);
        else if (t == 1) f.b[0] = *(const bf16x8*)(sb + b_base);
        else if (t < MBW + 1) f.a[t - 1] = *(const bf16x8*)(sb + a_base + (t - 1) * 2048);
        else f.b[t - MBW] = *(const bf16x8*)(sb + b_base + (t - MBW) * 2048);
    };
    auto load_frags = [&](Frags<MBW, NBW>& f, int stage, int ks) {
        const unsigned char* sb = smem + stage * S::STAGE_BYTES + lane_off[ks];
#pragma unroll
        for (int mb = 0; mb < MBW; ++mb) f.a[mb] = *(const bf16x8*)(sb + a_base + mb * 2048);
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) f.b[nb] = *(const bf16x8*)(sb + b_base + nb * 2048);
    };

    f32x16 acc[MBW][NBW];
#pragma unroll
    for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;


    // ---- prologue: fill all but one slot of the ring, fetch the first fragments -----------------------------
    constexpr int ST = S::STAGES;
    Frags<MBW, NBW> f0, f1;
    // The whole K loop exists once per load count (waves with and without the last load unit), so that no
    // load sits under a condition: a branch inside the loop would also cut it into scheduling regions.
    auto k_loop = [&](auto has_last) {
    constexpr int CNT = !FETCH ? 0 : S::REM == 0 || decltype(has_last)::value ? S::LPW : S::LPW - 1;  // loads per stage
    if constexpr (FETCH) {
#pragma unroll
        for (int s = 0; s < ST - 1; ++s)
            if (s < KT) issue(has_last, s, s);
        if (KT >= ST - 1) wait_vmcnt<(ST - 2) * CNT>();  // stage 0 landed, the others may be in flight
        else wait_vmcnt<0>();
    }
    __builtin_amdgcn_s_barrier();
    load_frags(f0, 0, 0);
    wait_lgkmcnt0();

    // Stage kt.  On entry f0 holds its sub-step 0.  The barrier at the top publishes stage kt+1 (whose
    // sub-step 0 is prefetched in the second half) and retires stage kt-1, which every wave finished
    // reading half a stage ago; that slot is refilled with stage kt+ST-1 right away.  The barrier falls
    // while the previous stage's last MFMAs are still in the pipe, and each half issues 2 + NB fragment
    // reads under 2 * NB MFMAs.
    //
    // STEADY stages (kt + ST - 1 < KT) have no conditions at all; the main loop runs ST of them per trip
    // with the ring slots as compile-time constants, so a trip is one straight run of instructions (taken
    // branches starve the MFMA pipe: the instruction buffer refills while nothing issues).
    // REFILL: the slot behind (pstage) is reloaded with stage kt+ST-1.  LAST: no stage follows (nothing is
    // prefetched and nothing waited for at the top).
    auto do_stage = [&](auto refill, auto last, int kt, int stage, int pstage, int nstage) {
        constexpr bool REFILL = decltype(refill)::value, LAST = decltype(last)::value;
        if (REFILL) {
            if (FETCH) wait_vmcnt<(ST - 3) * CNT>();
            __builtin_amdgcn_s_barrier();
        } else if (!LAST) {
            if (FETCH) wait_groups<ST, CNT>(KT - 1 - (kt + 1));  // stages issued after kt+1 may stay in flight
            __builtin_amdgcn_s_barrier();
        }
        // Memory instructions are dealt out between the MFMAs, and the compiler's scheduler is fenced at
        // every step: a burst of LDS reads or global->LDS loads would hold the wave's issue port while the
        // matrix pipe runs dry.  Fragment reads come first in a half, the global->LDS loads after them
        // (spreading the loads among the reads, or keeping the last MFMAs free of both, measured slower).
        constexpr int NM = MBW * NBW;
        constexpr int V1 = REFILL && FETCH ? (CNT + 1) / 2 : 0;
        constexpr int V2 = REFILL && FETCH ? CNT - V1 : 0;
        auto half = [&]<int... M>(std::integer_sequence<int, M...>, auto second) {
            constexpr bool SECOND = decltype(second)::value;
            constexpr int RD = SECOND && LAST ? 0 : MBW + NBW;
            constexpr int V = SECOND ? V2 : V1;
            constexpr int TOT = RD + V;
            auto step = [&](auto mi) {
                constexpr int m = decltype(mi)::value;
                const Frags<MBW, NBW>& use = SECOND ? f1 : f0;
                // QKV and gate/up compute the TRANSPOSED block (W A^T: the weight fragment as the MFMA's first operand),
                // so that a lane ends up with 16 output features of ONE token: see the epilogues
                if constexpr (EPI == EPI_PARTIAL)
                    acc[m % MBW][m / MBW] = mfma32(use.a[m % MBW], use.b[m / MBW], acc[m % MBW][m / MBW]);
                else
                    acc[m % MBW][m / MBW] = mfma32(use.b[m / MBW], use.a[m % MBW], acc[m % MBW][m / MBW]);
                __builtin_amdgcn_sched_barrier(0);
                if constexpr (TOT > 0) {
#pragma unroll
                    for (int t = TOT * m / NM; t < TOT * (m + 1) / NM; ++t) {
                        if (t >= RD) {
                            issue_one((SECOND ? V1 : 0) + t - RD, pstage, kt + ST - 1);
                        } else {
                            if (SECOND) load_frag_one(f0, nstage, 0, t);
                            else load_frag_one(f1, stage, 1, t);
                        }
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
            };
            (step(std::integral_constant<int, M>{}), ...);
        };
        half(std::make_integer_sequence<int, NM>{}, std::false_type{});
        half(std::make_integer_sequence<int, NM>{}, std::true_type{});
        // f0 (next stage) has had the last MFMAs to arrive; waiting here keeps the next stage's reads out of
        // the wait and leaves no LDS read of this wave outstanding at the barrier.
        wait_lgkmcnt0();
    };
    int kt = 0;
    for (; kt + 2 * ST - 1 <= KT; kt += ST) {  // ST refilling stages per trip, slots as compile-time constants
        [&]<int... I>(std::integer_sequence<int, I...>) {
            (do_stage(std::true_type{}, std::false_type{}, kt + I, I, (I + ST - 1) % ST, (I + 1) % ST), ...);
        }(std::make_integer_sequence<int, ST>{});
    }
    // The rest, with the slots as run-time values: the remaining refilling stages, the stages that only drain
    // the ring, and the last one.  One loop per kind (a single loop that branches between them makes the
    // compiler shuffle all accumulators at every merge).
    int stage = 0;
    auto next_slot = [&](int sl) { return sl + 1 == ST ? 0 : sl + 1; };
    auto prev_slot = [&](int sl) { return sl == 0 ? ST - 1 : sl - 1; };
    for (; kt + ST - 1 < KT; ++kt, stage = next_slot(stage))
        do_stage(std::true_type{}, std::false_type{}, kt, stage, prev_slot(stage), next_slot(stage));
    for (; kt + 1 < KT; ++kt, stage = next_slot(stage))
        do_stage(std::false_type{}, std::false_type{}, kt, stage, prev_slot(stage), next_slot(stage));
    if (kt < KT) do_stage(std::false_type{}, std::true_type{}, kt, stage, prev_slot(stage), next_slot(stage));
    };
    if constexpr (S::REM == 0 || !FETCH) {
        k_loop(std::true_type{});
    } else {
        if (wave < S::REM) k_loop(std::true_type{});
        else k_loop(std::false_type{});
    }

    // ---- epilogues ---------------------------------------------------------------------------------------
    // Lane (c, hh) holds, for block (mb, nb), column n0 + 32 nb + c and rows row0(mb) + 8*(i/4) + 4*hh + (i%4).
    const int n_end = min(n0 + a.n_stride, a.N);  // columns [n0, n_end) belong to this tile
    constexpr int WROWS = 32 * MBW;  // rows of this wave
    const int row_base = m0 + wm * WROWS + 4 * hh;
    const int nw0 = n0 + wn * NBW * 32;  // first column of this wave
    auto row_of = [&](int mb, int i) { return row_base + mb * 32 + 8 * (i >> 2) + (i & 3); };

    if (EPI == EPI_PARTIAL) {
        float* pbase = a.partial + (size_t)split * a.M * a.N + nw0 + c;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            if (nw0 + nb * 32 + c >= n_end) continue;
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int m = row_of(mb, i);
                    if (m < a.M) pbase[(size_t)m * a.N + nb * 32] = acc[mb][nb][i];
                }
        }
    } else if (EPI == EPI_SWIGLU) {
        // Transposed block: lane (c, hh) holds, for block (mb, nb), token m = row block mb, row c, and the packed weight
        // rows 8*(i/4) + 4*hh + (i%4) of the 32-row block nb.  The pack kernel orders those rows so that a lane's
        // registers 0..7 are the gate projections of 8 consecutive features and 8..15 their up projections (block nb
        // = features 16 nb .. 16 nb + 15, lanes of half hh the features 8 hh .. 8 hh + 7 of them).  A lane therefore
        // finishes 8 outputs of one token by itself and stores them as one 16-byte chunk of the tiled activation
        // layout: no exchange between lanes, no LDS, no barrier.
        const int half_n = a.N >> 1;
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int col = nw0 + nb * 32;  // first packed column of the block
            if (col >= n_end) continue;
            const int chunk = (col >> 4) + hh;  // 16-byte chunk of the output row: features 8 * chunk ..
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int m = m0 + wm * WROWS + mb * 32 + c;
                if (m >= a.M) continue;
                u32x4 out;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const float g0 = acc[mb][nb][2 * e], g1 = acc[mb][nb][2 * e + 1];
                    const float u0 = acc[mb][nb][8 + 2 * e], u1 = acc[mb][nb][8 + 2 * e + 1];
                    out[e] = pack_bf16x2(g0 * __builtin_amdgcn_rcpf(1.0f + __expf(-g0)) * u0,
                                         g1 * __builtin_amdgcn_rcpf(1.0f + __expf(-g1)) * u1);
                }
                *(u32x4*)(a.act + tiled_offset(m, chunk, half_n >> 5)) = out;
            }
        }
    } else {  // EPI_QKV
        // Transposed block, as above.  A 32-row block of a Q or K head holds 16 rotary indices and their partners 64
        // further on, ordered by the pack kernel so that a lane's registers 0..7 are the indices F .. F + 7 (F = 16 j
        // + 8 hh for block j of the head) and registers 8..15 their partners F + 64 ..: the lane rotates its 8 pairs and
        // stores two 16-byte pieces.  A block of V holds 32 consecutive features, a lane 16 of them (16 hh ..).
#pragma unroll
        for (int nb = 0; nb < NBW; ++nb) {
            const int col = nw0 + nb * 32;  // packed column of the block: one (q|k|v, head, j) for all lanes
            if (col >= n_end) continue;
            const int which = col / a.d_model;
            const int in_model = col - which * a.d_model;
            const int head = in_model >> 7, j = (in_model & 127) >> 5;
            const int f_lo = which == 2 ? 32 * j + 16 * hh : 16 * j + 8 * hh;  // first feature of registers 0..7
            const int f_hi = which == 2 ? f_lo + 8 : f_lo + 64;                  // ... of registers 8..15
#pragma unroll
            for (int mb = 0; mb < MBW; ++mb) {
                const int m = m0 + wm * WROWS + mb * 32 + c;
                if (m >= a.M) continue;
                u16* dst;
                if (which == 0) {
                    dst = a.q_out + (size_t)m * a.d_model + head * 128;
                } else if (!a.branches) {
                    dst = kv_slot_bf16(a.kv, a.layer, which - 1, head, a.n_heads, a.pos0 + m);
                } else {  // row m is token t of branch b: that branch's cache and position
                    const int b = m / a.branches->n_tok, t = m - b * a.branches->n_tok;
                    dst = kv_slot_bf16(a.branches->kv[b], a.layer, which - 1, head, a.n_heads, a.branches->pos0[b] + t);
                }
                u32x4 lo, hi;
                if (which == 2) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        lo[e] = pack_bf16x2(acc[mb][nb][2 * e], acc[mb][nb][2 * e + 1]);
                        hi[e] = pack_bf16x2(acc[mb][nb][8 + 2 * e], acc[mb][nb][8 + 2 * e + 1]);
                    }
                } else {
                    const float4* rp = (const float4*)(a.rope + (size_t)m * 64 + f_lo);  // 8 (cos, sin) pairs
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float4 cs = rp[e];  // (cos, sin) of indices f_lo + 2 e, f_lo + 2 e + 1
                        const float l0 = acc[mb][nb][2 * e], l1 = acc[mb][nb][2 * e + 1];
                        const float h0 = acc[mb][nb][8 + 2 * e], h1 = acc[mb][nb][8 + 2 * e + 1];
                        // lo' = lo cos - hi sin ; hi' = hi cos + lo sin
                        lo[e] = pack_bf16x2(l0 * cs.x - h0 * cs.y, l1 * cs.z - h1 * cs.w);
                        hi[e] = pack_bf16x2(h0 * cs.x + l0 * cs.y, h1 * cs.z + l1 * cs.w);
                    }
                }
                *(u32x4*)(dst + f_lo) = lo;
                *(u32x4*)(dst + f_hi) = hi;
            }
        }
    }
}

// ---- host side: tiling policy and launch -----------------------------------------------------------------

constexpr int kCUs = 256;

int div_up(int x, int y) { return (x + y - 1) / y; }

// Row blocks of the tile for a chunk of M tokens.
int pick_row_blocks(int M) { return M > 128 ? 8 : M > 64 ? 4 : 2; }

template <int BMB, int NB, int WM, int WN, int EPI>
hipError_t launch(GemmArgs a, hipStream_t s) {
    a.n_stride = 32 * NB;
    a.n_tiles = div_up(a.N, a.n_stride);
    a.m_tiles = div_up(a.M, 32 * BMB);
    a.kt_per_split = a.K / G_BK / a.splits;
    const int grid = a.m_tiles * a.n_tiles * a.splits;
    using S = Shape<BMB, NB, WM, WN>;
    hipLaunchKernelGGL((gemm_bf16<BMB, NB, WM, WN, EPI>), dim3(grid), dim3(S::THREADS), S::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <int BMB, int NB, int WM, int WN, int EPI>
hipError_t configure_one() {
    return hipFuncSetAttribute((const void*)gemm_bf16<BMB, NB, WM, WN, EPI>,
                               hipFuncAttributeMaxDynamicSharedMemorySize, Shape<BMB, NB, WM, WN>::LDS_BYTES);
}

}  // namespace

// Instantiations: (row blocks, column blocks, wave grid) per epilogue.  256-row tiles for prefill-sized
// chunks; 128- and 64-row tiles with narrow N for short chunks, where the grid must be wide enough to keep
// every CU streaming weights.
#define JUP_GEMM_SHAPES(X)                                                          \
    X(8, 1, 4, 1, EPI_QKV) X(8, 2, 4, 1, EPI_QKV) X(8, 3, 8, 1, EPI_QKV) X(8, 6, 4, 2, EPI_QKV)            \
    X(4, 2, 4, 1, EPI_QKV) X(2, 2, 2, 2, EPI_QKV) X(4, 3, 4, 1, EPI_QKV) X(4, 6, 4, 2, EPI_QKV) \
    X(8, 2, 4, 1, EPI_SWIGLU) X(8, 3, 4, 1, EPI_SWIGLU) X(8, 4, 4, 2, EPI_SWIGLU) X(8, 6, 4, 2, EPI_SWIGLU) X(8, 8, 4, 2, EPI_SWIGLU) \
    X(4, 4, 4, 1, EPI_SWIGLU) X(2, 4, 2, 2, EPI_SWIGLU) X(1, 3, 1, 3, EPI_SWIGLU) X(1, 4, 1, 4, EPI_SWIGLU) X(4, 3, 4, 1, EPI_SWIGLU) X(2, 3, 2, 3, EPI_SWIGLU) X(4, 6, 4, 1, EPI_SWIGLU) X(2, 6, 2, 3, EPI_SWIGLU) \
    X(8, 4, 4, 2, EPI_PARTIAL) X(8, 8, 4, 2, EPI_PARTIAL) X(4, 4, 4, 1, EPI_PARTIAL) X(4, 4, 4, 2, EPI_PARTIAL) X(2, 4, 2, 2, EPI_PARTIAL) X(2, 2, 2, 2, EPI_PARTIAL) X(4, 2, 4, 1, EPI_PARTIAL)

hipError_t gemm_configure() {
    hipError_t e = hipSuccess;
    auto acc = [&](hipError_t r) { if (e == hipSuccess) e = r; };
#define X(BMB, NB, WM, WN, EPI) acc(configure_one<BMB, NB, WM, WN, EPI>());
    JUP_GEMM_SHAPES(X)
#undef X
    return e;
}

// The projections whose N (= d_model) alone cannot fill the chip are split along K; the fp32 partial sums are
// added up, in split order, by the reduce + norm kernel that follows.
namespace {
// splits for tiles of 32*nb columns: the largest count up to 8 that keeps the grid within one round of workgroups
// and divides the K stages evenly (powers of two on the 7B shapes; d = 5120 and FFN 13824 also allow 5, 3 and 6)
int splits_for(int M, int N, int K, int nb) {
    const int tiles = div_up(M, 32 * pick_row_blocks(M)) * div_up(N, 32 * nb);
    int splits = 1;
    for (int s = 2; s <= 8; ++s)
        if (tiles * s <= kCUs && (K / G_BK) % s == 0) splits = s;
    return splits;
}
}  // namespace

// Column blocks of the partial-sum tile.  Short chunks take 64-column tiles instead of 128 when the wide tile
// would leave a workgroup only a few K stages (fill and drain of its pipeline would dominate): half the
// splits, so half the partial sums to write and to read back.  Measured on the 7B shapes: 64-row chunks O
// 13.3 -> 12.5 us, down 23.0 -> 22.3 us, reduce + norm 8.2 -> 7.6 us; 128-row chunks O 18.2 -> 15.8 us (down,
// with 43 stages per workgroup, keeps the wide tile: 28.3 vs 29.5 us).
int gemm_partial_col_blocks(int M, int N, int K) {
    const int bmb = pick_row_blocks(M);
    if (bmb >= 8) return 4;
    const int stages_wide = K / G_BK / splits_for(M, N, K, 4);
    return stages_wide < (bmb == 2 ? 64 : 32) ? 2 : 4;
}

// shared: another chunk's kernels run beside this launch (overlapped multi-chunk call).  Filling the chip with one
// launch then matters less than the work per output: at most two splits (half or a quarter of the partial sums to
// write and read back, longer K loops per workgroup); the CUs a launch leaves free go to the other chunks.
// Measured on the 7B shapes with four lanes: 4 x 512 tokens 274k -> 286k tokens/s, 8 x 256 tokens 204k -> 224k,
// 16 x 128 and 8 x 64 tokens +3-4 % (no split at all: -4 % there); alone on the chip the same cap costs 8 % (one
// launch then has to fill it).
// The output projection of a prefill-sized chunk (K no longer than N, 129 to 512 rows) alone on the chip: 128 x 128
// tiles with two splits (four for up to 256 rows) instead of 256 x 128 tiles with four.  The K loop is a little slower
// (a third more LDS traffic per flop), but half the partial sums are written and read back: measured at 512 rows of the 7B shapes, O
// projection 28.3 -> 29.4 us, the reduce + norm pass behind it 13.7 -> 10.2 us, the prompt +1.5 %.  (The same for the
// down projection, whose K loop is 2.7 times as long, measured slower: 52.3 -> 59.4 us.)
static bool square_prefill_projection(int M, int N, int K, bool shared) {
    // (the down projection too for up to 256 rows: four splits of 86 stages instead of eight of 43; measured at 256
    // rows 35.9 -> 36.5 us, the reduce + norm pass behind it reads half the partial sums, the prompt as 8 x 256 +1.5 %)
    return !shared && M > 128 && M <= 512 && (K <= N || M <= 256);  // (longer chunks keep the tall tile)
}

int gemm_plan_splits(int M, int N, int K, bool shared) {
    if (square_prefill_projection(M, N, K, shared)) {
        const int tiles = div_up(M, 128) * div_up(N, 128);
        int splits = 1;
        // (up to 256 rows two splits would leave half of the CUs idle: four; measured at 256 rows, O projection
        // 25.7 -> 21.1 us, the reduce + norm pass behind it 9.8 -> 10.8 us)
        const int cap = M <= 256 ? 4 : 2;
        while (tiles * splits * 2 <= kCUs && (K / G_BK) % (splits * 2) == 0 && splits < cap) splits *= 2;
        return splits;
    }
    // beside other chunks' kernels: the widest tile of the chunk's row count (see launch_gemm_partial)
    const int nb = shared ? (pick_row_blocks(M) >= 8 ? 8 : 4) : gemm_partial_col_blocks(M, N, K);
    const int s = splits_for(M, N, K, nb);
    const int cap = shared ? 2 : 8;
    return s > cap ? cap : s;
}

namespace {
// Among the instantiated widths (in 32-column blocks) of the 256-row tile, the one with the least work on the
// busiest CU: rounds of workgroups x time of one tile.  A tile's time grows with its width plus a fixed part
// (pipeline fill and drain, epilogue, and the 256 rows of A it streams whatever its width) worth about two
// column blocks: without it many narrow tiles look cheapest, and they re-read A once per tile (measured at
// M = 2048: 1.66 GB fetched per launch and 445 us with 64-column tiles, against 325 us expected from M = 1024).
// Ties go to the wider tile.
int pick_blocks(int M, int N, const int* cands, int n_cands) {
    const int m_tiles = div_up(M, 256);
    int best = cands[0];
    long best_cost = -1;
    for (int i = 0; i < n_cands; ++i) {
        const int nb = cands[i];
        const long tiles = (long)m_tiles * div_up(N, 32 * nb);
        const long cost = div_up((int)tiles, kCUs) * (long)(32 * nb + 64);
        if (best_cost < 0 || cost <= best_cost) { best = nb; best_cost = cost; }
    }
    return best;
}
}  // namespace

// ---- which instantiation serves a launch ------------------------------------------------------------------
struct TileShape {
    int bmb, nb, wm, wn;  // row blocks, column blocks, waves along M, waves along N
};

namespace {

TileShape pick_qkv(int M, int N, bool shared_gpu) {
    const int bmb = pick_row_blocks(M);
    // 128-token chunks beside other chunks' kernels: 96-column tiles (half again as much work per workgroup; alone on
    // the chip 64 columns win, 24.0 vs 28.8 us at 64 rows).  Measured with four lanes: 13B shapes, 8 x 128 tokens
    // +2 %; 7B shapes, 16 x 128 tokens +0-1 %; 192 columns +4 % and -1 %; 64-token chunks no difference either way.
    if (shared_gpu && bmb == 4) return {4, 3, 4, 1};
    if (bmb == 2) return {2, 2, 2, 2};
    if (bmb == 4) return {4, 2, 4, 1};
    // 129 to 256 rows alone on the chip: 128 x 96 tiles instead of 256 x 64 (at N = 12288 256 workgroups instead of 192,
    // and 14 KB instead of 20 KB through the fill path per stage); measured at 256 rows: 48.9 -> 42.8 us
    if (!shared_gpu && M > 128 && M <= 256) return {4, 3, 4, 1};
    static const int cands[] = {1, 2, 3};
    const int nb = pick_blocks(M, N, cands, 3);
    // Beside another chunk's kernels (overlapped multi-chunk call) half as many tiles of twice the width do the
    // same work in a quarter less CU time, and the other chunk uses the CUs they leave free: 76 us instead of 59 us
    // for this launch alone, but +1.7 % for the 4 x 512 prompt.  Alone on the chip the narrow tile wins (-6 %).
    if (nb == 3 && shared_gpu && M > 256) return {8, 6, 4, 2};
    // 385 to 512 rows alone on the chip: 128 x 192 tiles fill the same 256 CUs with 11 % fewer bytes through the fill
    // path per stage (20 KB against 22.5 KB); measured at 512 rows: 59.5 -> 57.8 us
    if (nb == 3 && M > 384 && M <= 512) return {4, 6, 4, 2};
    if (nb == 3) return {8, 3, 8, 1};  // 8 waves of 32 x 96: measured 1.3 % faster than 4 of 64 x 96
    if (nb == 2) return {8, 2, 4, 1};
    return {8, 1, 4, 1};
}

TileShape pick_swiglu(int M, int N, bool shared_gpu) {
    const int bmb = pick_row_blocks(M);
    // A short chunk is bound by streaming the weights, and every CU that streams adds bandwidth: the narrower
    // tile (96 columns) when its tiles still fit one round of workgroups (measured at 64 rows, N = 22016:
    // 230 workgroups 38.0 us, 172 workgroups of 128 columns 40.9 us, 344 of 64 columns 47.1 us).
    // Beside other chunks' kernels (overlapped multi-chunk call) the opposite holds: 192-column tiles, fewer and
    // longer-running workgroups, and the other chunks take the CUs they leave (64-token chunks +1.5 %, 128-token
    // chunks +2.5 %, the 13B shapes +4 % over 128 columns, which in turn beat 96 by 2-6 % there).
    if (shared_gpu && bmb == 2) return {2, 6, 2, 3};
    if (shared_gpu && bmb == 4) return {4, 6, 4, 1};
    const bool narrow = div_up(N, 96) <= kCUs;
    // Up to 32 rows: a tile of one row block (32 x 96 or 32 x 128, one wave per column block) leaves the fill path to the
    // weights; measured at 5 rows, N = 22016: 32.5 -> 31.5 us.  (The same for QKV and the O / down projections, on two
    // waves of 32 x 32: QKV 22.8 -> 23.4 us, O / down no different: they keep the 64-row tile.)
    if (bmb == 2 && M <= 32) return narrow ? TileShape{1, 3, 1, 3} : TileShape{1, 4, 1, 4};
    if (bmb == 2) return narrow ? TileShape{2, 3, 2, 3} : TileShape{2, 4, 2, 2};
    if (bmb == 4) return narrow ? TileShape{4, 3, 4, 1} : TileShape{4, 4, 4, 1};
    static const int cands[] = {2, 3, 4, 6};
    const int nb = pick_blocks(M, N, cands, 4);
    // beside other chunks' kernels: the widest tile (see pick_qkv); 256 x 256 over 256 x 192: +1.9 %
    if (nb == 6 && shared_gpu) return {8, 8, 4, 2};
    if (nb == 6) return {8, 6, 4, 2};
    if (nb == 4) return {8, 4, 4, 2};
    if (nb == 3) return {8, 3, 4, 1};
    return {8, 2, 4, 1};
}

TileShape pick_partial(int M, int N, int K, bool shared_gpu) {
    // (eight waves of 32 x 64 on the 128 x 128 tile: two per SIMD; 29.85 -> 28.8 us against four waves of 32 x 128)
    if (square_prefill_projection(M, N, K, shared_gpu)) return {4, 4, 4, 2};
    const int bmb = pick_row_blocks(M);
    // (short chunks beside other chunks' kernels keep the 128-column tile: 64-token chunks +3 %, 128-token +5 %)
    const bool narrow = gemm_partial_col_blocks(M, N, K) == 2 && !shared_gpu;
    if (bmb == 2) return narrow ? TileShape{2, 2, 2, 2} : TileShape{2, 4, 2, 2};
    if (bmb == 4) return narrow ? TileShape{4, 2, 4, 1} : TileShape{4, 4, 4, 1};
    // beside other chunks' kernels: the widest tile, as for QKV and gate/up (256 x 256 over 256 x 128: +2.4 %)
    if (shared_gpu) return {8, 8, 4, 2};
    return {8, 4, 4, 2};
}

template <int EPI>
hipError_t dispatch(TileShape t, const GemmArgs& a, hipStream_t s) {
#define X(BMB, NB, WM, WN, E)                                                         \
    if constexpr (E == EPI)                                                           \
        if (t.bmb == BMB && t.nb == NB && t.wm == WM && t.wn == WN) return launch<BMB, NB, WM, WN, EPI>(a, s);
    JUP_GEMM_SHAPES(X)
#undef X
    return hipErrorInvalidConfiguration;  // a shape the pick functions name but the list above does not hold
}

}  // namespace

hipError_t launch_gemm_qkv(GemmArgs a, hipStream_t s) {
    a.splits = 1;
    return dispatch<EPI_QKV>(pick_qkv(a.M, a.N, a.shared_gpu), a, s);
}

hipError_t launch_gemm_swiglu(GemmArgs a, hipStream_t s) {
    a.splits = 1;
    return dispatch<EPI_SWIGLU>(pick_swiglu(a.M, a.N, a.shared_gpu), a, s);
}

hipError_t launch_gemm_partial(GemmArgs a, hipStream_t s) {
    a.splits = gemm_plan_splits(a.M, a.N, a.K, a.shared_gpu);
    return dispatch<EPI_PARTIAL>(pick_partial(a.M, a.N, a.K, a.shared_gpu), a, s);
}

// "gemm_bf16<row blocks,column blocks,waves along M,waves along N,epilogue>" of the launch a projection of M rows takes
void gemm_kernel_name(GemmKind kind, int M, int d_model, int d_ffn, bool shared_gpu, char* buf, size_t size) {
    TileShape t{};
    int epi = EPI_PARTIAL;
    switch (kind) {
        case GEMM_QKV: t = pick_qkv(M, 3 * d_model, shared_gpu); epi = EPI_QKV; break;
        case GEMM_GATE_UP: t = pick_swiglu(M, 2 * d_ffn, shared_gpu); epi = EPI_SWIGLU; break;
        case GEMM_O: t = pick_partial(M, d_model, d_model, shared_gpu); break;
        case GEMM_DOWN: t = pick_partial(M, d_model, d_ffn, shared_gpu); break;
    }
    snprintf(buf, size, "gemm_bf16<%d,%d,%d,%d,%d>", t.bmb, t.nb, t.wm, t.wn, epi);
}

}  // namespace jup
