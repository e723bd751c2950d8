// Chunk attention of the bf16 path: the chunk's queries against the cached prefix plus the causal
// triangle inside the chunk (Jupiter paper, Sec. IV-A.2, Fig. 4b), MFMA 32x32x16 with online softmax.  The
// same kernel serves the batched outline branches (Sec. V-B: one chunk per branch, each with its own cache)
// and the token tree of a speculative step (Sec. V-A: inside the chunk a query sees its ancestors only).
//
// One workgroup = NQ*32 queries of one head: 4*NQ computing waves plus four waves that only fetch.  Computing
// wave 4*qb + g owns the block qb of 32 queries and the key quarter g, i.e. the 32-key tiles g, g+4, ... of
// the keys the workgroup can see.  The waves of a key quarter (one per query block) share that quarter's
// tiles in LDS; loader wave g keeps them one tile ahead with direct global->LDS loads, and all waves meet at
// ONE workgroup barrier per round.  With 64 accumulator registers per wave three waves fit a SIMD (two
// computing, one loading): while one waits for LDS or works through its softmax on the vector ALU the other
// has the matrix pipe, and no computing wave is held by the issue of a global->LDS load (each holds the
// issuing wave for about a hundred cycles).  Each wave computes the TRANSPOSED products
//     S^T[key][query] = K Q^T        (A = K tile rows, B = Q, held in registers for the whole kernel)
//     O^T[dh][query] += V^T P^T      (A = V^T, read from the row-major V tile with the transposing LDS
//                                     load; B = P^T taken straight from the S^T accumulators)
// so that a lane always owns one query column and the softmax statistics are per-lane scalars.  The
// partial results of the four key quarters are merged at the end with the usual log-sum-exp weights.
//
// The running maximum is lazy: it moves only when a tile's maximum exceeds it by more than 8 (in log2
// units), so the accumulators are rescaled a few times per kernel instead of once per tile; the exponentials
// stay below 2^8, far inside bf16/fp32 range, and the final normalisation removes the common factor.
//
// Key splits.  A decode-sized chunk behind a long cached sequence (Sec. V: a few tokens per step against the whole
// prompt and everything generated so far) has one query block per head, far fewer workgroups than the chip has
// CUs, and each would walk the whole cache alone.  Such a launch splits the key tiles of a query block into up to 8
// contiguous ranges, one workgroup each (blockIdx.y).  Every workgroup leaves its un-normalised result and softmax
// statistics in a scratch buffer and counts itself in; the one that finds all others counted merges the ranges IN
// RANGE ORDER with the log-sum-exp weights and writes the output, so the result does not depend on which workgroup
// came last (bitwise reproducible), no workgroup ever waits for another, and there is no second launch.
//
// MFMA 32x32x16 bf16 operand layout (lane = 32*hh + c):
//   A: lane supplies A[m = c][k = 8*hh + e], e < 8;  B: lane supplies B[k = 8*hh + e][n = c];
//   D: lane holds D[m = 8*(i/4) + 4*hh + (i%4)][n = c] in register i < 16.
// A lane (query column c, half hh) therefore holds S^T for keys 8*(i/4) + 4*hh + (i%4), i < 16.  The PV
// MFMA number ks (0/1) consumes registers 8ks..8ks+7: its contraction index 8*hh + e stands for key
// 16ks + 8*(e/4) + 4*hh + (e%4), and the V^T fragment is assembled for exactly that key order.
//
// ds_read_b64_tr_b16 (measured on gfx950): within each group of 16 lanes, lane i receives as element r
// (r < 4) element (i & 3) of the 8 bytes addressed by lane 4r + (i >> 2) of the group.
#include "bf16_common.h"

namespace jup {
namespace {

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Row of D held in accumulator register i by a lane of half hh.
__device__ inline int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

constexpr int kKT = 32;                 // keys per tile
constexpr int kTileBytes = kKT * 256;   // one K or V tile: 32 rows of 128 bf16
constexpr int kSlotBytes = 2 * kTileBytes;
constexpr int kWaveLds = 2 * kSlotBytes;  // two slots (K + V each) per key partition = 32 KB
// dynamic LDS: the merge at the end needs KP fp32 [32 NQ][132] regions plus the statistics; KP * NQ = 8 at most, so
// the sizes below (KP = 4 partitions of 64 queries, or 2 of 128) cover every instantiation
constexpr int kStatOffset = 4 * 64 * 132 * 4;               // softmax statistics (past the tile slots and the regions)
static_assert(kStatOffset >= 4 * kWaveLds, "the statistics are written while other waves still read their slots");
constexpr int kAttLds = kStatOffset + 2 * 4 * 64 * 4;
static_assert(kAttLds >= 4 * kWaveLds && kAttLds <= 160 * 1024, "LDS budget");

// LDS tile layouts (rows of 256 bytes = 16 chunks of 16 bytes):
//   K: chunk ch of row r at position ch ^ (r & 15)            (16 consecutive rows, same chunk: 16 banksets)
//   V: chunk ch of row r at position (((ch >> 2) ^ (r & 3)) << 2) | (ch & 3)   (4 consecutive rows spread
//      their 64-byte groups over the four 64-byte bank groups for the transposing reads)

// Transposing 8-byte LDS read, issued as text so that the compiler's wait-count pass does not treat it as a
// read that may alias the global->LDS loads in flight (it would drain them all before every read, which
// undoes the prefetch).  The compiler does not know that a result is pending either: every use of the
// results is preceded by wait_tr_reads() on the registers concerned.
template <int OFF>
__device__ inline u32x2 ds_read_tr16(unsigned addr) {
    u32x2 r;
    asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r) : "v"(addr), "n"(OFF));
    return r;
}
// Waits until at most N LDS reads issued after the ones that fill v are still in flight; v is named as
// an operand so that no use of it can be moved above the wait.
template <int N>
__device__ inline void wait_tr_reads(u32x4& v) {
    asm volatile("s_waitcnt lgkmcnt(%1)" : "+v"(v) : "n"(N));
}

// max over the two 32-lane halves (lanes i and i ^ 32 get the same result) on the vector ALU: the swap
// leaves {x.lo, x.lo} in one register and {x.hi, x.hi} in the other.
__device__ inline float max_across_halves(float x) {
    const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
    return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}

template <int NQ, int LPQ = 1, int KP = 4>
__global__ __launch_bounds__(64 * KP * (NQ + LPQ)) void chunk_attention_bf16(const u16* __restrict__ q, u16* __restrict__ o,
                                                                  int n, int d_model, int n_heads, int pos0_arg,
                                                                  KvView kv_arg, int layer, float scale_log2e,
                                                                  const BranchTable* __restrict__ branches,
                                                                  const TreeTable* __restrict__ tree,
                                                                  float* __restrict__ split_buf, int* __restrict__ split_count) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Waves 0 .. 4 NQ - 1 compute (key quarter g, query block qb); the last four waves only fetch tiles, one per
    // key quarter.  A global->LDS load holds the issuing wave for about a hundred cycles (the address path of a
    // CU takes 64 bytes per clock, and all quarters refill at the same moment): issued by the computing waves,
    // the loads of a round cost them as much as the round's arithmetic.
    // LPQ = 2: two loader waves per key quarter, one for the K part of a tile and one for the V part (a single wave
    // issues a 1 KB load every 64 cycles at best; with one query block per workgroup the round is as long as
    // the fill, and two loaders halve it).
    // KP = number of key partitions (4 quarters, or 2 halves for 128 queries per workgroup: each tile then serves
    // twice the queries, which halves the bytes filled per flop).
    static_assert(KP * NQ <= 8 && (KP == 2 || KP == 4), "LDS regions and statistics are sized for 8 x 32 query rows");
    const bool loader = wave >= KP * NQ;
    const int g = wave % KP, qb = loader ? 0 : wave / KP;
    const int lpart = LPQ == 2 ? (wave - KP * NQ) / KP : -1;  // loader: 0 = K only, 1 = V only, -1 = both
    const int c = lane & 31, hh = lane >> 5;
    const int head = blockIdx.x % n_heads;
    const int q_blocks = (n + NQ * 32 - 1) / (NQ * 32);
    const int bq = blockIdx.x / n_heads;
    const int branch = bq / q_blocks;  // 0 without a branch table
    const int q0 = (q_blocks - 1 - bq % q_blocks) * (NQ * 32);
    const int row0 = branch * n;
    // (the same for every lane; read out of the vector registers a table load leaves them in, which the tile loop
    // cannot spare)
    const int pos0 = __builtin_amdgcn_readfirstlane(branches ? branches->pos0[branch] : pos0_arg);
    KvView kv = branches ? branches->kv[branch] : kv_arg;
    kv.own = (void*)uniform_ptr((const char*)kv.own);
    kv.parent = (const void*)uniform_ptr((const char*)kv.parent);
    kv.n_shared = __builtin_amdgcn_readfirstlane(kv.n_shared);
    kv.own_cap = __builtin_amdgcn_readfirstlane(kv.own_cap);
    kv.parent_cap = __builtin_amdgcn_readfirstlane(kv.parent_cap);
    q += (size_t)row0 * d_model;
    const int q_last = min(q0 + NQ * 32, n) - 1;  // last real query of this workgroup
    const int n_keys = pos0 + q_last + 1;
    const int n_tiles = (n_keys + kKT - 1) / kKT;
    const int last_key = n_keys - 1;
    // tiles before it need no mask: they lie below every query's diagonal (in a token tree: before the chunk)
    const int first_masked_tile = tree ? pos0 / kKT : (pos0 + q0 + 1) / kKT;

    unsigned char* grp = lds + g * kWaveLds;  // this key quarter's two slots (K tile + V tile each)
    const unsigned grp_addr = __builtin_amdgcn_readfirstlane(lds_byte_address(lds)) + g * kWaveLds;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + head;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + head;

    // key splits over workgroups: this one owns the tiles [t_lo, t_hi) of the query block
    // (never more than the launch provides: a launch that does not split has gridDim.y = 1)
    const int n_splits = min(att_key_splits(n, n_tiles), (int)gridDim.y);
    const int ks = blockIdx.y;
    if (ks >= n_splits) return;  // (a branch or query block with fewer keys than the longest of the launch)
    const int t_lo = (int)((long)ks * n_tiles / n_splits), t_hi = (int)((long)(ks + 1) * n_tiles / n_splits);
    const int n_own = t_hi - t_lo;
    const int cnt = n_own > g ? (n_own - g + KP - 1) / KP : 0;  // tiles of this key partition
    const int max_cnt = (n_own + KP - 1) / KP;                  // of partition 0: every wave runs that many rounds
    if (loader) {
        // The whole life of a loader wave: one tile ahead of the computing waves, the same barriers as they.
        // Tile fill (loader waves).  Load j covers rows 4j..4j+3 (1 KB of LDS); lane i lands at
        // row 4j + (i >> 4), position i & 15, and fetches the chunk that belongs there.
        const int lrow = lane >> 4, lp = lane & 15;
        const u16* k_own = (const u16*)kv.own + plane_k * (size_t)kv.own_cap * 128;
        const u16* v_own = (const u16*)kv.own + plane_v * (size_t)kv.own_cap * 128;
        const u16* k_par = (const u16*)kv.parent + plane_k * (size_t)kv.parent_cap * 128;
        const u16* v_par = (const u16*)kv.parent + plane_v * (size_t)kv.parent_cap * 128;
        auto fill_part = [&](int tile, int slot, bool v_part) __attribute__((always_inline)) {
            const unsigned dst = grp_addr + slot * kSlotBytes + (v_part ? kTileBytes : 0);
            const u16* par = v_part ? v_par : k_par;
            const u16* own = v_part ? v_own : k_own;
            const int key0 = tile * kKT;
            if (key0 + kKT - 1 <= last_key && (key0 >= kv.n_shared || key0 + kKT <= kv.n_shared)) {
                const bool shared = key0 < kv.n_shared;
                const char* base = uniform_ptr((const char*)((shared ? par : own) + (size_t)(shared ? key0 : key0 - kv.n_shared) * 128));
                const unsigned vch = (((lp >> 2) ^ lrow) << 2) | (lp & 3);
    #pragma unroll
                for (int j = 0; j < 8; ++j)
                    load_to_lds_16(base + j * 1024, lrow * 256 + (v_part ? vch : (lp ^ (4 * (j & 3) + lrow))) * 16,
                                   dst + j * 1024);
            } else {
    #pragma unroll
                for (int j = 0; j < 8; ++j) {
                    const int r = 4 * j + lrow;
                    const int key = min(key0 + r, last_key);
                    const bool shared = key < kv.n_shared;
                    const unsigned row_off = (unsigned)(shared ? key : key - kv.n_shared) * 128u;  // elements, < 2^31
                    const unsigned ch = v_part ? ((((lp >> 2) ^ (r & 3)) << 2) | (lp & 3)) : (lp ^ (r & 15));
                    load_to_lds_16((shared ? par : own) + row_off + ch * 8, dst + j * 1024);
                }
            }
        };
        auto fill = [&](int tile, int slot) __attribute__((always_inline)) {
            if (lpart != 1) fill_part(tile, slot, false);
            if (lpart != 0) fill_part(tile, slot, true);
        };
        if (cnt > 0) fill(t_lo + g, 0);
        for (int it = 0; it < max_cnt; ++it) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the tile of this round has landed
            __builtin_amdgcn_s_barrier();                     // ... and the other slot is free
            if (it + 1 < cnt) fill(t_lo + g + KP * (it + 1), (it + 1) & 1);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // the two barriers of the merge
        __syncthreads();
        if (n_splits > 1) {  // ... and the two of the merge across workgroups
            __syncthreads();
            __syncthreads();
        }
        return;
    }

    // Q fragments (B operand of S^T) straight from global memory: lane = query column, 8 consecutive dh per k-step.
    bf16x8 qf[8];
    {
        const int qrow = min(q0 + qb * 32 + c, n - 1);
        const u16* qp = q + (size_t)qrow * d_model + head * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[ks] = *(const bf16x8*)(qp + 16 * ks);
    }
    f32x16 oacc[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) oacc[db][r] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;

    const unsigned k_lane = c * 256 + ((hh ^ (c & 15)) * 16);
    const int G = lane >> 4, s = lane & 15;
    const int vt_row = 4 * (G >> 1) + (s >> 2);
    unsigned v_lane[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_lane[db] = vt_row * 256 + ((db ^ (vt_row & 3)) << 6) + (2 * (G & 1) + ((s & 3) >> 1)) * 16 + 8 * (s & 1);

    const int q_abs = pos0 + q0 + qb * 32 + c;  // cache entry of this lane's query
    // token tree: bit j = the query sees token j of the chunk (its ancestors and itself)
    const unsigned long long q_sees = tree ? tree->sees[min(q0 + qb * 32 + c, n - 1)] : 0ull;

    for (int it = 0; it < max_cnt; ++it) {
        // One barrier per round: the loader arrives when the tile of this round has landed, the computing waves
        // when they are done with the other slot, which the loader then refills.
        __builtin_amdgcn_s_barrier();
        if (it >= cnt) continue;
        const int tile = t_lo + g + KP * it, slot = it & 1;
        const unsigned char* k_base = grp + slot * kSlotBytes;
        const unsigned v_base = grp_addr + slot * kSlotBytes + kTileBytes;

        // ---- S^T = K Q^T ---------------------------------------------------------------------------------------
        f32x16 sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
#pragma unroll
        for (int half = 0; half < 2; ++half) {  // four fragments at a time: 168 registers per wave is the budget
            bf16x8 kf[4];
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) kf[ks] = *(const bf16x8*)(k_base + (k_lane ^ (32 * (4 * half + ks))));
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) sacc = mfma32(kf[ks], qf[4 * half + ks], sacc);
        }

        // ---- online softmax (a lane owns one query column) -------------------------------------------------------
        float sv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) sv[r] = sacc[r];
        if (tile >= first_masked_tile) {  // the tile reaches some query's diagonal (a few tiles per workgroup)
            asm volatile("");             // keeps this a branch: merged into selects it would run for every tile
            const int key0 = tile * kKT;
            if (tree) {
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int rel = key0 + acc_row(r, hh) - pos0;  // index of the key's token inside the chunk
                    if (rel >= 0 && (rel >= kMaxTreeTokens || !((q_sees >> (rel & 63)) & 1))) sv[r] = -INFINITY;
                }
            } else {
#pragma unroll
                for (int r = 0; r < 16; ++r)
                    if (key0 + acc_row(r, hh) > q_abs) sv[r] = -INFINITY;
            }
        }
        float mt = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) mt = fmaxf(mt, sv[r]);
        mt = max_across_halves(mt) * scale_log2e;  // the scale is positive
        const bool grow = mt > m_run + 8.0f;       // lazy reference maximum
        const float m_new = grow ? mt : m_run;
        const float m_safe = m_new == -INFINITY ? 0.f : m_new;
        const float alpha = grow ? __builtin_amdgcn_exp2f(m_run - m_safe) : 1.0f;
        const bool rescale = grow && m_run != -INFINITY;
        float ps = 0.f;
        bf16x8 pf[2];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float p = __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], scale_log2e, -m_safe));
            ps += p;
            pf[r >> 3][r & 7] = (__bf16)p;
        }
        l_run = l_run * alpha + ps;
        m_run = m_new;
        if (__any(rescale)) {
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[db][r] *= alpha;
        }

        // ---- O^T += V^T P^T ----------------------------------------------------------------------------------------
        u32x4 vf[8];
        [&]<int... F>(std::integer_sequence<int, F...>) {
            (([&] {
                 constexpr int db = F / 2, ks = F % 2;
                 const u32x2 lo = ds_read_tr16<(16 * ks) * 256>(v_base + v_lane[db]);
                 const u32x2 hi = ds_read_tr16<(16 * ks + 8) * 256>(v_base + v_lane[db]);
                 vf[F] = (u32x4){lo[0], lo[1], hi[0], hi[1]};
             }()),
             ...);
        }(std::make_integer_sequence<int, 8>{});
        [&]<int... F>(std::integer_sequence<int, F...>) {
            (([&] {
                 wait_tr_reads<14 - 2 * F>(vf[F]);
                 oacc[F / 2] = mfma32(__builtin_bit_cast(bf16x8, vf[F]), pf[F % 2], oacc[F / 2]);
             }()),
             ...);
        }(std::make_integer_sequence<int, 8>{});
    }

    // ---- merge the key partitions of every query block -------------------------------------------------------------
    constexpr int kORow = 132;
    constexpr int QR = 32 * NQ;                             // query rows of the workgroup
    constexpr int kRegion = QR * kORow;                     // floats per key partition: [QR queries][132]
    static_assert(KP * kRegion * 4 <= kStatOffset, "merge regions overlap the statistics");
    // The lane indices of the merge are derived afresh from a copy of the thread id that the compiler cannot see through:
    // nothing the merge needs is then computed (and kept in registers) before the tile loop, whose register budget
    // is exhausted (one value too many there spills a Q fragment, reloaded in every round).
    int tid_m = tid;
    asm volatile("" : "+v"(tid_m));
    const int c_m = tid_m & 31, hh_m = (tid_m >> 5) & 1;
    float* obuf = (float*)lds;
    float* stat_m = (float*)(lds + kStatOffset);            // [KP][QR]
    float* stat_l = stat_m + KP * QR;
    {
        const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
        if (hh_m == 0) {
            stat_m[g * QR + qb * 32 + c_m] = m_run;
            stat_l[g * QR + qb * 32 + c_m] = l_tot;
        }
    }
    __syncthreads();  // statistics visible; every wave is done with the tile slots
    {
        float m_all = -INFINITY;
#pragma unroll
        for (int w = 0; w < KP; ++w) m_all = fmaxf(m_all, stat_m[w * QR + qb * 32 + c_m]);
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < KP; ++w) {
            const float mw = stat_m[w * QR + qb * 32 + c_m];
            l_all += mw == -INFINITY ? 0.f : stat_l[w * QR + qb * 32 + c_m] * exp2f(mw - m_all);
        }
        // one workgroup for all keys: normalised here; key splits: left un-normalised for the merge across workgroups
        const float wscale = m_run == -INFINITY ? 0.f : exp2f(m_run - m_all) / (n_splits > 1 ? 1.0f : l_all);
        float* mine = obuf + g * kRegion + (qb * 32 + c_m) * kORow;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
                *(float4*)(mine + db * 32 + 8 * gg + 4 * hh_m) =
                    make_float4(oacc[db][4 * gg] * wscale, oacc[db][4 * gg + 1] * wscale,
                                oacc[db][4 * gg + 2] * wscale, oacc[db][4 * gg + 3] * wscale);
        if (n_splits > 1 && g == 0 && hh_m == 0) {  // statistics of this key range, one pair per query row
            store_coherent2(split_buf + ((size_t)(blockIdx.x * gridDim.y + ks) * QR + qb * 32 + c_m) * kAttSplitRow + 128,
                            m_all, l_all);
        }
    }
    __syncthreads();
    for (int idx = tid_m; idx < QR * 16; idx += 64 * KP * NQ) {  // the computing threads (tid < 64 KP NQ)
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        const float* src = obuf + qr * kORow + ch * 8;
        float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
#pragma unroll
        for (int w = 1; w < KP; ++w) {
            const float4 a2 = *(const float4*)(src + w * kRegion), b2 = *(const float4*)(src + w * kRegion + 4);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
        }
        if (n_splits > 1) {
            float* dst = split_buf + ((size_t)(blockIdx.x * gridDim.y + ks) * QR + qr) * kAttSplitRow + ch * 8;
            store_coherent2(dst, a.x, a.y);
            store_coherent2(dst + 2, a.z, a.w);
            store_coherent2(dst + 4, b.x, b.y);
            store_coherent2(dst + 6, b.z, b.w);
            continue;
        }
        u32x4 out;
        out[0] = pack_bf16x2(a.x, a.y); out[1] = pack_bf16x2(a.z, a.w);
        out[2] = pack_bf16x2(b.x, b.y); out[3] = pack_bf16x2(b.z, b.w);
        *(u32x4*)(o + tiled_offset(row0 + qrow, head * 16 + ch, d_model >> 5)) = out;
    }
    if (n_splits == 1) return;

    // ---- merge the key ranges of the query block across workgroups ---------------------------------------------------
    // Every wave waits until its (chip-coherent) stores have been performed, the workgroup counts itself in, and the
    // workgroup that finds all others already counted does the merge.  Nobody waits for anybody.
    wait_stores_performed();
    __syncthreads();
    int* flag = (int*)(lds + kStatOffset);  // (the statistics in LDS are no longer needed)
    if (tid_m == 0) {
        const int before = arrive_coherent(split_count + blockIdx.x);
        *flag = before == n_splits - 1;
        if (before == n_splits - 1) split_count[blockIdx.x] = 0;  // ready for the next launch on this stream
    }
    __syncthreads();
    if (!*flag) return;
    const float* base = split_buf + (size_t)blockIdx.x * gridDim.y * QR * kAttSplitRow;
    for (int idx = tid_m; idx < QR * 16; idx += 64 * KP * NQ) {
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        // (max, sum) of every key range: at most 8, loops unrolled under a condition so that the array stays in
        // registers; all loads first, then the sums in range order, whoever came last
        static_assert(att_max_splits(1) <= 8, "the merge holds at most 8 ranges");
        float2 stat[8], val[8][4];  // every load is issued before the first is used: they come from memory, not L2
#pragma unroll
        for (int sp = 0; sp < 8; ++sp)
            if (sp < n_splits) {
                const float* row = base + ((size_t)sp * QR + qr) * kAttSplitRow;
                stat[sp] = load_coherent2(row + 128);
#pragma unroll
                for (int e = 0; e < 4; ++e) val[sp][e] = load_coherent2(row + ch * 8 + 2 * e);
            }
        float m_all = -INFINITY;
#pragma unroll
        for (int sp = 0; sp < 8; ++sp)
            if (sp < n_splits) m_all = fmaxf(m_all, stat[sp].x);
        float l_all = 0.f;
        float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int sp = 0; sp < 8; ++sp)
            if (sp < n_splits && stat[sp].x != -INFINITY) {  // (-inf: a range this query sees nothing of)
                const float w = exp2f(stat[sp].x - m_all);
                l_all += stat[sp].y * w;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    acc[2 * e] += val[sp][e].x * w;
                    acc[2 * e + 1] += val[sp][e].y * w;
                }
            }
        const float inv = 1.0f / l_all;
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = pack_bf16x2(acc[2 * e] * inv, acc[2 * e + 1] * inv);
        *(u32x4*)(o + tiled_offset(row0 + qrow, head * 16 + ch, d_model >> 5)) = out;
    }
}

}  // namespace

hipError_t attention_configure() {
    hipError_t e = hipFuncSetAttribute((const void*)chunk_attention_bf16<1, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kAttLds);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void*)chunk_attention_bf16<4, 2, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                            kAttLds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)chunk_attention_bf16<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               kAttLds);
}

// Block sizes: 4 NQ computing waves + 4 loader waves per part loaded separately.  Chunks of up to 64 tokens run
// one query block per workgroup with separate K and V loaders (decode-sized attention is a chain of short
// rounds, each as long as its tile fill); longer chunks two query blocks sharing every tile.
namespace {
// a split launch must fit the scratch the workspace reserves for it (it does by construction: see att_split_rows)
bool split_fits(const AttScratch& sc, int wgs, int splits, int query_rows) {
    return splits == 1 || ((size_t)wgs * splits * query_rows <= sc.rows && (size_t)wgs <= sc.counters);
}
}  // namespace

hipError_t launch_chunk_attention(const u16* q, u16* o, int n, int d_model, int n_heads, int pos0, const KvView& kv,
                                  int layer, hipStream_t s, AttScratch sc, const TreeTable* tree, bool shared_gpu) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    const BranchTable* none = nullptr;
    // Beside other chunks' kernels (overlapped multi-chunk call): 128 queries per workgroup against two key halves,
    // half as many workgroups, each tile filled once for twice the queries.  Alone on the chip this is slower (half
    // the CUs idle: 33.7 vs 20.1 us at 512 queries over 1536 cached keys); beside other chunks it takes a sixth less
    // CU time: 4 x 512 tokens +2.4 %, no difference at 256-token chunks.
    if (shared_gpu && n > 256) {
        hipLaunchKernelGGL((chunk_attention_bf16<4, 2, 2>), dim3((n + 127) / 128 * n_heads), dim3(768), kAttLds, s, q, o,
                           n, d_model, n_heads, pos0, kv, layer, scale_log2e, none, tree, sc.split_buf, sc.split_count);
        return hipGetLastError();
    }
    // chunks of up to 256 tokens behind a long cached sequence: several workgroups per query block (key splits)
    const int splits = att_key_splits(n, (pos0 + n + kKT - 1) / kKT);
    // 32 queries per workgroup up to 64 tokens, and up to 128 when the launch has the chip to itself (twice the
    // workgroups of the 64-query variant, which a launch this small needs more than shared tile fills: measured on
    // 128-token chunks, 7B shapes 18.4 -> 17.0 us, 13B shapes 14.6 -> 13.0 us; inside an overlapped call the same
    // choice costs 2-3.5 %, at 256 tokens it gains nothing)
    if (n <= (shared_gpu ? 64 : 128)) {
        const int wgs = (n + 31) / 32 * n_heads;
        if (!split_fits(sc, wgs, splits, 32)) return hipErrorInvalidValue;
        hipLaunchKernelGGL((chunk_attention_bf16<1, 2>), dim3(wgs, splits), dim3(768), kAttLds, s, q, o, n, d_model,
                           n_heads, pos0, kv, layer, scale_log2e, none, tree, sc.split_buf, sc.split_count);
    } else {
        const int wgs = (n + 63) / 64 * n_heads;
        if (!split_fits(sc, wgs, splits, 64)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3(wgs, splits), dim3(768), kAttLds, s, q, o, n, d_model, n_heads,
                           pos0, kv, layer, scale_log2e, none, tree, sc.split_buf, sc.split_count);
    }
    return hipGetLastError();
}

hipError_t launch_branch_attention(const u16* q, u16* o, int n, int n_branches, int d_model, int n_heads,
                                   const BranchTable* branches, int max_keys, int layer, hipStream_t s, AttScratch sc) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    const KvView none{};
    const TreeTable* no_tree = nullptr;
    const int splits = att_key_splits(n, (max_keys + kKT - 1) / kKT);  // of the branch with the most keys
    if (n <= 64) {
        const int wgs = n_branches * ((n + 31) / 32) * n_heads;
        if (!split_fits(sc, wgs, splits, 32)) return hipErrorInvalidValue;
        hipLaunchKernelGGL((chunk_attention_bf16<1, 2>), dim3(wgs, splits), dim3(768), kAttLds, s, q, o, n, d_model,
                           n_heads, 0, none, layer, scale_log2e, branches, no_tree, sc.split_buf, sc.split_count);
    } else {
        const int wgs = n_branches * ((n + 63) / 64) * n_heads;
        if (!split_fits(sc, wgs, splits, 64)) return hipErrorInvalidValue;
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3(wgs, splits), dim3(768), kAttLds, s, q, o, n, d_model, n_heads,
                           0, none, layer, scale_log2e, branches, no_tree, sc.split_buf, sc.split_count);
    }
    return hipGetLastError();
}

}  // namespace jup
