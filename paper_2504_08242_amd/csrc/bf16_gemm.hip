// bf16 GEMM  C[M, N] = A[M, K] * W[N, K]^T  for gfx950 with fused epilogues.
//
// Shape of the problem.  A chunk has at most a few hundred rows (M = n_tokens) while N is the layer
// width, so the work per compute unit is small: about 44 K outputs for the gate/up projection of a
// 512-token chunk on 256 CUs.  The kernel therefore gives every CU ONE tall tile, 256 rows by up to
// 192 columns, held entirely in accumulators (the register file of a CU is 512 KB), and sizes the
// tile width so that the number of tiles matches the number of CUs.  That is the largest tile the
// problem allows, which is what keeps the L2 -> LDS traffic per flop low.
//
//   * 4 waves; wave w owns rows [64w, 64w+64) x all NB 32-column blocks: 2*NB MFMA 32x32x16 per K/16.
//     (The 16x16x32 form sustains only ~70 % of the 32x32x16 rate on this chip, measured.)
//   * K advances in stages of 32 through a 5-stage LDS ring filled by direct global->LDS loads
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
//
// MFMA 32x32x16 bf16 operand layout (lane = 32*hh + c):
//   A: lane supplies A[m = c][k = 8*hh + e], e < 8;  B: lane supplies B[k = 8*hh + e][n = c];
//   D: lane holds D[m = 8*(i/4) + 4*hh + (i%4)][n = c] in register i < 16.
#include <type_traits>
#include <utility>

#include "bf16_common.h"

// 0 = product code.  Timing experiments only (results are garbage): bit 0 = no refills of the LDS ring,
// bit 1 = no MFMA, bit 2 = no fragment reads in the loop, bit 3 = no barrier in the loop.
#ifndef GEMM_EXPERIMENT
#define GEMM_EXPERIMENT 0
#endif

namespace jup {
namespace {

constexpr int G_BM = 256, G_BK = 32;
constexpr int kLdsBudget = 160 * 1024;

template <int NB>
struct Shape {
    static constexpr int ROWS = G_BM + 32 * NB;     // LDS rows per stage: A rows then W rows
    static constexpr int STAGE_BYTES = ROWS * 64;
    static constexpr int N_LOAD = ROWS / 16;        // wave-wide load instructions per stage (1 KB each)
    static constexpr int LPW = (N_LOAD + 3) / 4;    // per wave (the last ones may repeat a neighbour's)
    // as many ring slots as LDS holds (at most 8: the in-flight count must fit the 6-bit vmcnt)
    static constexpr int STAGES = kLdsBudget / STAGE_BYTES > 8 ? 8 : kLdsBudget / STAGE_BYTES;
    static constexpr int LDS_BYTES = STAGES * STAGE_BYTES;
    static_assert(STAGES >= 4 && (STAGES - 2) * LPW < 64, "ring depth");
};

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
#if GEMM_EXPERIMENT & 2
    c[0] += (float)a[0] * (float)b[0];
    return c;
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
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

// Fragments of one K/16 sub-step of a wave: 2 row blocks, NB column blocks.
template <int NB>
struct Frags {
    bf16x8 a[2];
    bf16x8 b[NB];
};

template <int NB, int EPI>
__global__ __launch_bounds__(256) void gemm_bf16(const GemmArgs a) {
    using S = Shape<NB>;
    extern __shared__ __attribute__((aligned(1024))) unsigned char smem[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    // ---- which tile ---------------------------------------------------------------------------------
    int mt, grp;
    if (a.xcd_swizzle) {
        const int xcd = blockIdx.x & 7, local = blockIdx.x >> 3;
        mt = local % a.m_tiles;
        grp = xcd + 8 * (local / a.m_tiles);
    } else {
        mt = blockIdx.x % a.m_tiles;
        grp = blockIdx.x / a.m_tiles;
    }
    const int nt = grp % a.n_tiles, split = grp / a.n_tiles;
    const int m0 = mt * G_BM, n0 = nt * a.n_stride;
    const int KT = a.kt_per_split;

    // ---- global -> LDS load slots of this wave --------------------------------------------------------
    // Instruction j covers LDS rows [16j, 16j+16) = 1 KB; lane i lands at byte 16*i of it, which is
    // super-row i>>4, slot i&15, i.e. row 16j + 4*(i>>4) + ((i&15)>>2), chunk (i&3) ^ (i>>4).
    const u16* gp[S::LPW];
    int ldst[S::LPW];  // LDS byte offset inside a stage
    const int kt_total = a.K / G_BK;
#pragma unroll
    for (int q = 0; q < S::LPW; ++q) {
        const int j = min(wave + 4 * q, S::N_LOAD - 1);
        // Both operands are pre-tiled: an instruction copies half of a 2 KB block, lanes in address order.
        if (j < G_BM / 16) {
            const int blk = min(m0 / 32 + (j >> 1), (a.M + 31) / 32 - 1);  // blocks past M repeat the last one
            gp[q] = a.A + ((size_t)blk * kt_total + (size_t)split * KT) * 1024 + (j & 1) * 512 + lane * 8;
        } else {
            const int jw = j - G_BM / 16;
            const int blk = min(n0 / 32 + (jw >> 1), a.N / 32 - 1);  // blocks past N repeat the last one
            gp[q] = a.W + ((size_t)blk * kt_total + (size_t)split * KT) * 1024 + (jw & 1) * 512 + lane * 8;
        }
        ldst[q] = j * 1024;
    }
    auto issue = [&](int stage, int kt) {
#pragma unroll
        for (int q = 0; q < S::LPW; ++q) {
            __builtin_amdgcn_global_load_lds(
                (const __attribute__((address_space(1))) void*)(gp[q] + (size_t)kt * 1024),
                (__attribute__((address_space(3))) void*)(smem + stage * S::STAGE_BYTES + ldst[q]), 16, 0, 0);
        }
    };

    // ---- LDS -> register fragment addresses -------------------------------------------------------------
    // Fragment row = 32*block + c (c = lane & 31), chunk = 2*ks + hh.  Block bases are multiples of 32,
    // so the swizzle term depends on the lane and on ks only: address = lane part + constant.
    const int c = lane & 31, hh = lane >> 5;
    int lane_off[2];
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
        lane_off[ks] = (c >> 2) * 256 + ((((c & 3) << 2) + 2 * ks + hh) ^ ((c >> 2) & 3)) * 16;
    const int a_base = wave * (64 * 64), b_base = G_BM * 64;
    auto load_frags = [&](Frags<NB>& f, int stage, int ks) {
        const unsigned char* sb = smem + stage * S::STAGE_BYTES + lane_off[ks];
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) f.a[mb] = *(const bf16x8*)(sb + a_base + mb * 2048);
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) f.b[nb] = *(const bf16x8*)(sb + b_base + nb * 2048);
    };

    f32x16 acc[2][NB];
#pragma unroll
    for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int nb = 0; nb < NB; ++nb)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[mb][nb][r] = 0.f;

    auto mma = [&](const Frags<NB>& f, int nb_lo, int nb_hi) {
#pragma unroll
        for (int nb = nb_lo; nb < nb_hi; ++nb)
#pragma unroll
            for (int mb = 0; mb < 2; ++mb) acc[mb][nb] = mfma32(f.a[mb], f.b[nb], acc[mb][nb]);
    };

    // ---- prologue: fill all but one slot of the ring, fetch the first fragments -----------------------------
    constexpr int ST = S::STAGES;
#pragma unroll
    for (int s = 0; s < ST - 1; ++s)
        if (s < KT) issue(s, s);
    if (KT >= ST - 1) wait_vmcnt<(ST - 2) * S::LPW>();  // stage 0 landed, the others may be in flight
    else wait_vmcnt<0>();
    __builtin_amdgcn_s_barrier();
    Frags<NB> f0, f1;
    load_frags(f0, 0, 0);
    wait_lgkmcnt0();

    // Waits until at most g of this wave's load groups (one group = one stage) are still in flight.
    auto wait_groups = [&](int g) {
        if (g >= ST - 3) wait_vmcnt<(ST - 3) * S::LPW>();
        else if (g == 4) wait_vmcnt<(ST > 7 ? 4 : 0) * S::LPW>();
        else if (g == 3) wait_vmcnt<(ST > 6 ? 3 : 0) * S::LPW>();
        else if (g == 2) wait_vmcnt<(ST > 5 ? 2 : 0) * S::LPW>();
        else if (g == 1) wait_vmcnt<1 * S::LPW>();
        else wait_vmcnt<0>();
    };

    // Stage kt.  On entry f0 holds its sub-step 0.  The barrier at the top publishes stage kt+1 (whose
    // sub-step 0 is prefetched in the second half) and retires stage kt-1, which every wave finished
    // reading half a stage ago; that slot is refilled with stage kt+ST-1 right away.  The barrier falls
    // while the previous stage's last MFMAs are still in the pipe, and each half issues 2 + NB fragment
    // reads under 2 * NB MFMAs.
    //
    // STEADY stages (kt + ST - 1 < KT) have no conditions at all; the main loop runs ST of them per trip
    // with the ring slots as compile-time constants, so a trip is one straight run of instructions (taken
    // branches starve the MFMA pipe: the instruction buffer refills while nothing issues).
    auto do_stage = [&](auto steady, int kt, int stage, int pstage, int nstage) {
        constexpr bool STEADY = decltype(steady)::value;
        if (STEADY) {
            wait_vmcnt<(ST - 3) * S::LPW>();
            if (!(GEMM_EXPERIMENT & 8)) __builtin_amdgcn_s_barrier();
            if (!(GEMM_EXPERIMENT & 1)) issue(pstage, kt + ST - 1);
        } else if (kt + 1 < KT) {
            wait_groups(KT - 1 - (kt + 1));  // stages issued after kt+1 may stay in flight
            if (!(GEMM_EXPERIMENT & 8)) __builtin_amdgcn_s_barrier();
            if (!(GEMM_EXPERIMENT & 1) && kt + ST - 1 < KT) issue(pstage, kt + ST - 1);
        }
        if (!(GEMM_EXPERIMENT & 4) || kt == 0) load_frags(f1, stage, 1);
        mma(f0, 0, NB);
        if (!(GEMM_EXPERIMENT & 4) && (STEADY || kt + 1 < KT)) load_frags(f0, nstage, 0);
        mma(f1, 0, NB);
        if (STEADY && GEMM_EXPERIMENT == 0) {
            sched_half<2 * NB, 2 + NB, (S::LPW + 1) / 2>();
            sched_half<2 * NB, 2 + NB, S::LPW / 2>();
        }
        // f0 (next stage) has had the last MFMAs to arrive; waiting here keeps the next stage's reads out of
        // the wait and leaves no LDS read of this wave outstanding at the barrier.
        wait_lgkmcnt0();
    };
    int kt = 0;
    for (; kt + 2 * ST - 1 <= KT; kt += ST) {  // every stage of the trip is steady
        [&]<int... I>(std::integer_sequence<int, I...>) {
            (do_stage(std::true_type{}, kt + I, I, (I + ST - 1) % ST, (I + 1) % ST), ...);
        }(std::make_integer_sequence<int, ST>{});
    }
    for (int stage = 0; kt < KT; ++kt) {  // the last few stages, with the tail conditions
        const int nstage = stage + 1 == ST ? 0 : stage + 1;
        const int pstage = stage == 0 ? ST - 1 : stage - 1;
        do_stage(std::false_type{}, kt, stage, pstage, nstage);
        stage = nstage;
    }

    // ---- epilogues ---------------------------------------------------------------------------------------
    // Lane (c, hh) holds, for block (mb, nb), column n0 + 32 nb + c and rows row0(mb) + 8*(i/4) + 4*hh + (i%4).
    const int n_end = min(n0 + a.n_stride, a.N);  // columns [n0, n_end) belong to this tile
    const int row_base = m0 + wave * 64 + 4 * hh;
    auto row_of = [&](int mb, int i) { return row_base + mb * 32 + 8 * (i >> 2) + (i & 3); };

    if (EPI == EPI_PARTIAL) {
        float* pbase = a.partial + (size_t)split * a.M * a.N + n0 + c;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            if (n0 + nb * 32 + c >= n_end) continue;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int m = row_of(mb, i);
                    if (m < a.M) pbase[(size_t)m * a.N + nb * 32] = acc[mb][nb][i];
                }
        }
    } else if (EPI == EPI_SWIGLU) {
        // packed column 2j = gate_j, 2j+1 = up_j: the even lane pairs with its right neighbour
        const int half_n = a.N >> 1;
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int n = n0 + nb * 32 + c;
            const bool col_ok = !(c & 1) && n < n_end;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float own = acc[mb][nb][i];
                    const float other = __builtin_bit_cast(
                        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, own), 0xB1, 0xF, 0xF, true));
                    const int m = row_of(mb, i);
                    if (col_ok && m < a.M)
                        a.act[tiled_offset(m, n >> 4, half_n >> 5) + ((n >> 1) & 7)] = f2bf(own / (1.0f + __expf(-own)) * other);
                }
        }
    } else {  // EPI_QKV
        // Packed column 32j + 16a + c' of a Q/K head is rotary index 16j + c' + 64a: lanes c and c ^ 16 of
        // one block hold the partners i and i + 64.  V columns keep their order.
#pragma unroll
        for (int nb = 0; nb < NB; ++nb) {
            const int col = n0 + nb * 32;  // packed column of the block: one (q|k|v, head, j) for all lanes
            const bool blk_ok = col < n_end;
            const int which = col / a.d_model;
            const int in_model = col - which * a.d_model;
            const int head = in_model >> 7, j = (in_model & 127) >> 5;
            const int hi = c >> 4, i_lo = 16 * j + (c & 15);
            // destination of row m is dst + m * stride
            u16* dst;
            size_t stride;
            if (which == 0) {
                dst = a.q_out + head * 128 + i_lo + 64 * hi;
                stride = a.d_model;
            } else {
                dst = kv_slot_bf16(a.kv, a.layer, which - 1, head, a.n_heads, a.pos0) + (which == 2 ? 32 * j + c : i_lo + 64 * hi);
                stride = 128;
            }
            const float2* rp = a.rope + i_lo;
#pragma unroll
            for (int mb = 0; mb < 2; ++mb)
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const float own = acc[mb][nb][i];
                    const float other = __shfl_xor(own, 16, 64);
                    const int m = row_of(mb, i);
                    if (!blk_ok || m >= a.M) continue;
                    float out = own;
                    if (which != 2) {
                        const float2 cs = rp[(size_t)m * 64];
                        // lo' = lo cos - hi sin ; hi' = hi cos + lo sin
                        out = hi ? own * cs.x + other * cs.y : own * cs.x - other * cs.y;
                    }
                    dst[(size_t)m * stride] = f2bf(out);
                }
        }
    }
}

// ---- host side: tiling policy and launch -----------------------------------------------------------------

constexpr int kCUs = 256;

template <int NB, int EPI>
hipError_t launch(const GemmArgs& a, hipStream_t s) {
    const int grid = a.m_tiles * a.n_tiles * a.splits;
    hipLaunchKernelGGL((gemm_bf16<NB, EPI>), dim3(grid), dim3(256), Shape<NB>::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <int NB, int EPI>
hipError_t configure_one() {
    return hipFuncSetAttribute((const void*)gemm_bf16<NB, EPI>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               Shape<NB>::LDS_BYTES);
}

void finish_plan(GemmArgs& a) {
    a.m_tiles = (a.M + G_BM - 1) / G_BM;
    const int total = a.m_tiles * a.n_tiles * a.splits;
    a.xcd_swizzle = (total % (8 * a.m_tiles)) == 0;
    a.kt_per_split = a.K / G_BK / a.splits;
}

int div_up(int x, int y) { return (x + y - 1) / y; }

}  // namespace

hipError_t gemm_configure() {
    hipError_t e = hipSuccess;
    auto acc = [&](hipError_t r) { if (e == hipSuccess) e = r; };
    acc(configure_one<1, EPI_QKV>());
    acc(configure_one<2, EPI_QKV>());
    acc(configure_one<3, EPI_QKV>());
    acc(configure_one<2, EPI_SWIGLU>());
    acc(configure_one<3, EPI_SWIGLU>());
    acc(configure_one<4, EPI_SWIGLU>());
    acc(configure_one<6, EPI_SWIGLU>());
    acc(configure_one<4, EPI_PARTIAL>());
    return e;
}

// K splits for the projections whose N (= d_model) alone cannot fill the chip.
int gemm_plan_splits(int M, int N, int K) {
    const int m_tiles = (M + G_BM - 1) / G_BM;
    const int n_tiles = div_up(N, 128);
    int splits = 1;
    // double while it keeps the grid within one wave of workgroups and the K stages divide evenly
    while (m_tiles * n_tiles * splits * 2 <= kCUs && (K / G_BK) % (splits * 2) == 0 && splits < 8) splits *= 2;
    return splits;
}

namespace {
// Among the instantiated widths (in 32-column blocks), the one with the least work on the busiest CU:
// rounds of workgroups x rows streamed per tile.  Ties go to the wider tile (fewer re-reads of A).
int pick_blocks(int M, int N, const int* cands, int n_cands) {
    const int m_tiles = (M + G_BM - 1) / G_BM;
    int best = cands[0];
    long best_cost = -1;
    for (int i = 0; i < n_cands; ++i) {
        const int nb = cands[i];
        const long tiles = (long)m_tiles * div_up(N, 32 * nb);
        const long cost = div_up((int)tiles, kCUs) * (long)(32 * nb);
        if (best_cost < 0 || cost <= best_cost) { best = nb; best_cost = cost; }
    }
    return best;
}
}  // namespace

hipError_t launch_gemm_qkv(GemmArgs a, hipStream_t s) {
    static const int cands[] = {1, 2, 3};
    const int nb = pick_blocks(a.M, a.N, cands, 3);
    a.splits = 1;
    a.n_stride = 32 * nb;
    a.n_tiles = div_up(a.N, a.n_stride);
    finish_plan(a);
    if (nb == 3) return launch<3, EPI_QKV>(a, s);
    if (nb == 2) return launch<2, EPI_QKV>(a, s);
    return launch<1, EPI_QKV>(a, s);
}

hipError_t launch_gemm_swiglu(GemmArgs a, hipStream_t s) {
    static const int cands[] = {2, 3, 4, 6};
    const int nb = pick_blocks(a.M, a.N, cands, 4);
    a.splits = 1;
    a.n_stride = 32 * nb;
    a.n_tiles = div_up(a.N, a.n_stride);
    finish_plan(a);
    if (nb == 6) return launch<6, EPI_SWIGLU>(a, s);
    if (nb == 4) return launch<4, EPI_SWIGLU>(a, s);
    if (nb == 3) return launch<3, EPI_SWIGLU>(a, s);
    return launch<2, EPI_SWIGLU>(a, s);
}

hipError_t launch_gemm_partial(GemmArgs a, hipStream_t s) {
    a.splits = gemm_plan_splits(a.M, a.N, a.K);
    a.n_stride = 128;
    a.n_tiles = div_up(a.N, 128);
    finish_plan(a);
    return launch<4, EPI_PARTIAL>(a, s);
}

}  // namespace jup
