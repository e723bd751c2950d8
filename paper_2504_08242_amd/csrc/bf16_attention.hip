// Chunk attention of the bf16 path: the chunk's queries against the cached prefix plus the causal
// triangle inside the chunk (Jupiter paper, Sec. IV-A.2, Fig. 4b), MFMA 32x32x16 with online softmax.
//
// One workgroup = QB*32 queries of one head, 4 waves.  The waves split the key range: wave w takes the
// 32-key tiles w, w+4, ... of the keys this query block can see.  Each wave runs a private two-slot
// LDS pipeline filled by direct global->LDS loads, so the main loop has no workgroup barrier, and it is
// software-pipelined: the K fragments of the next tile are fetched from LDS under the P V products of
// this one, the V^T fragments under the K Q^T products, and a slot is refilled (two tiles ahead) as soon
// as its last fragment has been read.  Each wave computes the TRANSPOSED products
//     S^T[key][query] = K Q^T        (A = K tile rows, B = Q)
//     O^T[dh][query] += V^T P^T      (A = V^T, read from the row-major V tile with the transposing LDS
//                                     load; B = P^T taken straight from the S^T accumulators)
// so that a lane always owns one query column and the softmax statistics are per-lane scalars.  The
// four partial results are merged at the end with the usual log-sum-exp weights.
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

// 1 = timing experiments only (the output is then overwritten with cycle counters): wave 0 of every
// workgroup accumulates the cycles it spends in the parts of the tile loop.
#ifndef ATT_TIMELINE
#define ATT_TIMELINE 0
#endif
// Timing experiments only (results are garbage): bit 0 = the query fragments are not read (the key
// fragment stands in), bit 1 = no MFMA, bit 2 = no exponentials, bit 3 = V^T fragments are not read,
// bit 4 = slots are not refilled inside the loop.
#ifndef ATT_EXPERIMENT
#define ATT_EXPERIMENT 0
#endif
#if ATT_TIMELINE
#define ATT_T(var) const unsigned long long var = __builtin_amdgcn_s_memtime()
#else
#define ATT_T(var)
#endif

namespace jup {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
#if ATT_EXPERIMENT & 2
    c[0] += (float)a[0] * (float)b[0];
    return c;
#else
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
#endif
}
// Row of D held in accumulator register i by a lane of half hh.
__device__ inline int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

template <int N>
__device__ inline void wait_vmcnt() {
    __builtin_amdgcn_s_waitcnt((N & 0xF) | ((N >> 4) << 14) | 0x0F70);
}

constexpr int kKT = 32;                 // keys per tile
constexpr int kTileBytes = kKT * 256;   // one K or V tile: 32 rows of 128 bf16
constexpr int kSlotBytes = 2 * kTileBytes;
constexpr int kWaveLds = 2 * kSlotBytes;  // two slots (K + V each) per wave = 32 KB
// dynamic LDS: the merge at the end needs four fp32 [64][132] regions plus the statistics
constexpr int kStatOffset = 4 * 64 * 132 * 4;               // softmax statistics of the four waves (past the tile slots)
constexpr int kQOffset = kStatOffset + 2 * 4 * 64 * 4;      // the block's queries follow: [64 rows][256 B], K-tile layout
static_assert(kStatOffset >= 4 * kWaveLds, "the statistics are written while other waves still read their slots");
constexpr int kAttLds = kQOffset + 64 * 256;
static_assert(kAttLds >= 4 * kWaveLds && kAttLds <= 160 * 1024, "LDS budget");

// LDS tile layouts (rows of 256 bytes = 16 chunks of 16 bytes):
//   K: chunk ch of row r at position ch ^ (r & 15)            (16 consecutive rows, same chunk: 16 banksets)
//   V: chunk ch of row r at position (((ch >> 2) ^ (r & 3)) << 2) | (ch & 3)   (4 consecutive rows spread
//      their 64-byte groups over the four 64-byte bank groups for the transposing reads)
__device__ inline int k_pos(int r, int ch) { return ch ^ (r & 15); }
__device__ inline int v_pos(int r, int ch) { return (((ch >> 2) ^ (r & 3)) << 2) | (ch & 3); }

// LDS byte address of a pointer into the workgroup's dynamic LDS.
__device__ inline unsigned lds_addr(const void* p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}

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

template <int QB>
__global__ __launch_bounds__(256) void chunk_attention_bf16(const u16* __restrict__ q, u16* __restrict__ o, int n,
                                                            int d_model, int n_heads, int pos0_arg, KvView kv_arg,
                                                            int layer, float scale_log2e,
                                                            const BranchTable* __restrict__ branches) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, hh = lane >> 5;
    // Workgroup b runs on XCD b % 8: heads vary fastest so that every query block of a head reads that
    // head's keys and values through the same L2; the longest query blocks (most visible keys) start first.
    // A batched-branch launch runs the grid of one chunk once per branch: rows [branch * n, +n) of q and o,
    // that branch's cache and starting position.
    const int head = blockIdx.x % n_heads;
    const int q_blocks = (n + QB * 32 - 1) / (QB * 32);
    const int bq = blockIdx.x / n_heads;
    const int branch = bq / q_blocks;  // 0 without a branch table
    const int q0 = (q_blocks - 1 - bq % q_blocks) * (QB * 32);
    const int row0 = branch * n;       // first row of this chunk in q and o
    const int pos0 = branches ? branches->pos0[branch] : pos0_arg;
    const KvView kv = branches ? branches->kv[branch] : kv_arg;
    q += (size_t)row0 * d_model;
    const int q_last = min(q0 + QB * 32, n) - 1;  // last real query of this block
    const int n_keys = pos0 + q_last + 1;         // keys 0 .. n_keys-1 are visible to the block
    const int n_tiles = (n_keys + kKT - 1) / kKT;
    const int last_key = n_keys - 1;   // rows past it are loaded from it and masked
    const int first_masked_tile = (pos0 + q0 + 1) / kKT;  // tiles before it lie below every query's diagonal

    unsigned char* my = lds + wave * kWaveLds;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + head;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + head;

    f32x16 oacc[QB][4];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int r = 0; r < 16; ++r) oacc[qb][db][r] = 0.f;
    }

    // Tile fill: 8 wave-wide loads for K and 8 for V.  Load j covers rows 4j..4j+3 (1 KB of LDS); lane i
    // lands at row 4j + (i >> 4), position i & 15, and fetches the chunk that belongs there.  A tile that
    // lies inside one cache segment and below the last visible key (all but two or three) is a wave-uniform
    // base plus a per-lane constant; the others compute every row's address.
    const int lrow = lane >> 4, lp = lane & 15;
    // plane bases of the two cache segments (the parent's is never dereferenced when nothing is shared)
    const u16* k_own = (const u16*)kv.own + plane_k * (size_t)kv.own_cap * 128;
    const u16* v_own = (const u16*)kv.own + plane_v * (size_t)kv.own_cap * 128;
    const u16* k_par = (const u16*)kv.parent + plane_k * (size_t)kv.parent_cap * 128;
    const u16* v_par = (const u16*)kv.parent + plane_v * (size_t)kv.parent_cap * 128;
    unsigned gk[4];  // byte offset inside the tile of this lane's K chunk for loads j = t (mod 4)
#pragma unroll
    for (int t = 0; t < 4; ++t) gk[t] = lrow * 256 + (lp ^ (4 * t + lrow)) * 16;
    const unsigned gv = lrow * 256 + ((((lp >> 2) ^ lrow) << 2) | (lp & 3)) * 16;
    auto fill = [&](int tile, int slot) __attribute__((always_inline)) {
        unsigned char* kd = my + slot * kSlotBytes;
        unsigned char* vd = kd + kTileBytes;
        const int key0 = tile * kKT;
        if (key0 + kKT - 1 <= last_key && (key0 >= kv.n_shared || key0 + kKT <= kv.n_shared)) {
            const bool shared = key0 < kv.n_shared;
            const size_t row0 = (size_t)(shared ? key0 : key0 - kv.n_shared) * 128;
            const char* kb = uniform_ptr((const char*)((shared ? k_par : k_own) + row0));
            const char* vb = uniform_ptr((const char*)((shared ? v_par : v_own) + row0));
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + j * 1024 + gk[j & 3]),
                                                 (__attribute__((address_space(3))) void*)(kd + j * 1024), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(vb + j * 1024 + gv),
                                                 (__attribute__((address_space(3))) void*)(vd + j * 1024), 16, 0, 0);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const int r = 4 * j + lrow;
                const int key = min(key0 + r, last_key);
                const bool shared = key < kv.n_shared;
                const unsigned row_off = (unsigned)(shared ? key : key - kv.n_shared) * 128u;  // elements, < 2^31
                const u16* kr = (shared ? k_par : k_own) + row_off + (lp ^ (r & 15)) * 8;
                const u16* vr = (shared ? v_par : v_own) + row_off + ((((lp >> 2) ^ (r & 3)) << 2) | (lp & 3)) * 8;
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)kr,
                                                 (__attribute__((address_space(3))) void*)(kd + j * 1024), 16, 0, 0);
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)vr,
                                                 (__attribute__((address_space(3))) void*)(vd + j * 1024), 16, 0, 0);
            }
        }
    };

    // In the loop a refill is split: the K half of a slot is free once the tile's scores are done and is
    // reloaded under the P V products, the V half follows under the next tile's first LDS reads.  That form
    // exists for uniform tiles only (tile_is_uniform); the others are reloaded whole by fill().
    auto tile_is_uniform = [&](int tile) __attribute__((always_inline)) {
        const int key0 = tile * kKT;
        return key0 + kKT - 1 <= last_key && (key0 >= kv.n_shared || key0 + kKT <= kv.n_shared);
    };
    auto tile_base = [&](int tile, const u16* par, const u16* own) __attribute__((always_inline)) {
        const int key0 = tile * kKT;
        const bool shared = key0 < kv.n_shared;
        return uniform_ptr((const char*)((shared ? par : own) + (size_t)(shared ? key0 : key0 - kv.n_shared) * 128));
    };
    auto load_k_unit = [&](const char* kb, int slot, int j) __attribute__((always_inline)) {
        __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(kb + j * 1024 + gk[j & 3]),
                                         (__attribute__((address_space(3))) void*)(my + slot * kSlotBytes + j * 1024), 16,
                                         0, 0);
    };
    const char* pend_vb = nullptr;  // V half still to be reloaded (at the start of the next tile), or null
    int pend_slot = 0;
    auto load_pending_v = [&]() __attribute__((always_inline)) {
        unsigned char* vd = my + pend_slot * kSlotBytes + kTileBytes;
#pragma unroll
        for (int j = 0; j < 8; ++j)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(pend_vb + j * 1024 + gv),
                                             (__attribute__((address_space(3))) void*)(vd + j * 1024), 16, 0, 0);
        pend_vb = nullptr;
    };

    // Per-lane LDS read offsets.
    //   K fragment ks: row c, chunk 2ks + hh, stored at position (2ks + hh) ^ (c & 15): the ks term is an
    //   XOR with 32 ks on the byte offset.
    //   V^T fragment (db, ks, part): transposing read; lane = 16*G + s supplies the address of
    //   V[key = 16ks + 8*part + 4*(G>>1) + (s>>2)][dh = 32db + 16*(G&1) + 4*(s&3) .. +3]: the row's low two
    //   bits are s >> 2, so the db term is an XOR on the 64-byte group index and (ks, part) an immediate.
    const unsigned k_lane = c * 256 + ((hh ^ (c & 15)) * 16);
    const int G = lane >> 4, s = lane & 15;
    const int vt_row = 4 * (G >> 1) + (s >> 2);
    unsigned v_lane[4];
#pragma unroll
    for (int db = 0; db < 4; ++db)
        v_lane[db] = vt_row * 256 + ((db ^ (vt_row & 3)) << 6) + (2 * (G & 1) + ((s & 3) >> 1)) * 16 + 8 * (s & 1);

    // This wave's tiles are wave, wave + 4, ...; tile number i of them lives in slot i & 1.  Two tiles are
    // put in flight before the queries are fetched, and everything is waited for once: inside the loop the
    // only vector-memory operations outstanding are the refills.
    const int cnt = n_tiles > wave ? (n_tiles - wave + 3) / 4 : 0;
    if (cnt > 0) fill(wave, 0);
    if (cnt > 1) fill(wave + 4, 1);

    // The block's queries go to LDS in the K-tile layout (they are the B operand of S^T: lane = query
    // column, 8 consecutive dh per k-step); wave w fetches rows 16w .. 16w+15.  Keeping them in registers
    // instead costs 64 VGPRs per lane, which the softmax needs.
    unsigned char* q_lds = lds + kQOffset;
    if (wave < QB * 2) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int r = 16 * wave + 4 * j + lrow;
            const int qrow = min(q0 + r, n - 1);
            const u16* qp = q + (size_t)qrow * d_model + head * 128 + (lp ^ (r & 15)) * 8;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)qp,
                                             (__attribute__((address_space(3))) void*)(q_lds + (16 * wave + 4 * j) * 256),
                                             16, 0, 0);
        }
    }
    wait_vmcnt<0>();
    __syncthreads();

    // A tile is processed in two parts.  front: scores, softmax statistics, probabilities; it reports whether
    // any lane moved its reference maximum, in which case the accumulators must be rescaled before back:
    // P V products, slot refill.  The rescaling code is kept out of the loop that runs the common case (its
    // mere presence there makes the compiler copy 64 accumulator registers per tile ahead of the branch).
    bf16x8 pf[QB][2];
    float alpha[QB];
#if ATT_TIMELINE
    unsigned long long tl[6] = {0, 0, 0, 0, 0, 0};
    const unsigned long long tl_begin = __builtin_amdgcn_s_memtime();
#endif
    auto front = [&](auto masked, int i) __attribute__((always_inline)) -> bool {
        constexpr bool MASKED = decltype(masked)::value;
        const int tile = wave + 4 * i, slot = i & 1;
        const unsigned char* k_base = my + slot * kSlotBytes;

        // ---- S^T = K Q^T for the 32 keys of the tile ------------------------------------------------------------
        ATT_T(t0);
        // Fragment reads run two k-steps ahead of the MFMAs that use them; the scheduler is fenced so that it
        // keeps that distance (it otherwise sinks every read to just before its use and each k-step then
        // waits out a full LDS latency).
        bf16x8 kf[8], qf[QB][8];
        auto read_step = [&](int ks) __attribute__((always_inline)) {
            kf[ks] = *(const bf16x8*)(k_base + (k_lane ^ (32 * ks)));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
                qf[qb][ks] = (ATT_EXPERIMENT & 1) ? kf[ks] : *(const bf16x8*)(q_lds + qb * 8192 + (k_lane ^ (32 * ks)));
        };
        read_step(0);
        read_step(1);
        __builtin_amdgcn_sched_barrier(0);
        if (pend_vb) load_pending_v();
        f32x16 sacc[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks + 2 < 8) read_step(ks + 2);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[qb] = mfma32(kf[ks], qf[qb][ks], sacc[qb]);
            __builtin_amdgcn_sched_barrier(0);
        }

        // ---- online softmax; a lane owns one query column of each query block -------------------------------
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(sacc[0]), "+v"(sacc[1]));  // the scores are complete here
#endif
        ATT_T(t1);
        const int key0 = tile * kKT;
        bool any_rescale = false;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int q_abs = pos0 + q0 + qb * 32 + c;  // absolute position of this lane's query
            float sv[16];
            float mt = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sv[r] = sacc[qb][r];
                if (MASKED && key0 + acc_row(r, hh) > q_abs) sv[r] = -INFINITY;
                mt = fmaxf(mt, sv[r]);
            }
            mt = max_across_halves(mt) * scale_log2e;  // the scale is positive
            // The reference maximum follows the running maximum lazily: it moves only when a tile exceeds it
            // by more than 2^8, so the accumulators are rescaled a few times per query instead of at every
            // tile whose maximum creeps up.  Probabilities then reach 2^8 at most, which bf16 and the fp32
            // sums hold as well as values below 1; the final division by the sum removes the factor.
            const bool grow = mt > m_run[qb] + 8.0f;  // also the first finite maximum (m_run = -inf)
            const float m_new = grow ? mt : m_run[qb];
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            alpha[qb] = grow ? __builtin_amdgcn_exp2f(m_run[qb] - m_safe) : 1.0f;
            any_rescale |= grow && m_run[qb] != -INFINITY;  // nothing accumulated yet otherwise
            float ps = 0.f;
            float pv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pv[r] = (ATT_EXPERIMENT & 4) ? __builtin_fmaf(sv[r], scale_log2e, -m_safe)
                                             : __builtin_amdgcn_exp2f(__builtin_fmaf(sv[r], scale_log2e, -m_safe));
                ps += pv[r];
            }
            l_run[qb] = l_run[qb] * alpha[qb] + ps;
            m_run[qb] = m_new;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[qb][ks][e] = (__bf16)pv[8 * ks + e];
        }
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(pf[0][0]), "+v"(pf[0][1]), "+v"(pf[1][0]), "+v"(pf[1][1]));
        ATT_T(t2);
        tl[0] += t1 - t0; tl[1] += t2 - t1; tl[5] += 1;
#endif
        return __any(any_rescale);
    };
    auto rescale_all = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int db = 0; db < 4; ++db)
#pragma unroll
                for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha[qb];
    };
    auto back_impl = [&](auto split_refill, int i, const char* kb2) __attribute__((always_inline)) {
        constexpr bool SPLIT = decltype(split_refill)::value;  // reload the K half of the slot under the MFMAs
        const int slot = i & 1;
        const unsigned v_base = lds_addr(my + slot * kSlotBytes + kTileBytes);
        // ---- O^T += V^T P^T ----------------------------------------------------------------------------------------
        // All eight V^T fragments (two 8-byte transposing reads each) are requested at once and consumed in
        // order as they arrive.
        u32x4 vf[8];
        [&]<int... F>(std::integer_sequence<int, F...>) {
            (([&] {
                 constexpr int db = F / 2, ks = F % 2;
                 if (ATT_EXPERIMENT & 8) {
                     vf[F] = (u32x4){v_base, v_lane[db], (unsigned)ks, 0u};
                 } else {
                     const u32x2 lo = ds_read_tr16<(16 * ks) * 256>(v_base + v_lane[db]);
                     const u32x2 hi = ds_read_tr16<(16 * ks + 8) * 256>(v_base + v_lane[db]);
                     // the two 8-byte results are the low and high halves of the 16-byte operand
                     vf[F] = (u32x4){lo[0], lo[1], hi[0], hi[1]};
                 }
             }()),
             ...);
        }(std::make_integer_sequence<int, 8>{});
        [&]<int... F>(std::integer_sequence<int, F...>) {
            (([&] {
                 wait_tr_reads<14 - 2 * F>(vf[F]);
                 if (SPLIT && F < 4) {
                     load_k_unit(kb2, slot, 2 * F);
                     load_k_unit(kb2, slot, 2 * F + 1);
                 }
#pragma unroll
                 for (int qb = 0; qb < QB; ++qb)
                     oacc[qb][F / 2] = mfma32(__builtin_bit_cast(bf16x8, vf[F]), pf[qb][F % 2], oacc[qb][F / 2]);
             }()),
             ...);
        }(std::make_integer_sequence<int, 8>{});
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(oacc[0][3]), "+v"(oacc[1][3]));
#endif
    };
    auto back = [&](int i) __attribute__((always_inline)) {
        const int tile = wave + 4 * i, slot = i & 1;
        const bool refill = !(ATT_EXPERIMENT & 16) && i + 2 < cnt;
        ATT_T(t3);
        if (refill && tile_is_uniform(tile + 8)) {
            back_impl(std::true_type{}, i, tile_base(tile + 8, k_par, k_own));
            pend_vb = tile_base(tile + 8, v_par, v_own);
            pend_slot = slot;
            ATT_T(t4);
            wait_vmcnt<8>();  // the next tile has landed; the K half just requested may be in flight
#if ATT_TIMELINE
            ATT_T(t5);
            tl[2] += t4 - t3; tl[3] += t5 - t4;
#endif
        } else {
            back_impl(std::false_type{}, i, nullptr);
            if (refill) fill(tile + 8, slot);  // every V^T fragment has arrived: the slot is free
            ATT_T(t4);
            if (i + 1 < cnt) {
                if (refill) wait_vmcnt<16>();
                else wait_vmcnt<0>();
            }
#if ATT_TIMELINE
            ATT_T(t5);
            tl[2] += t4 - t3; tl[3] += t5 - t4;
#endif
        }
    };
    // Tiles below first_masked_tile lie under every query's diagonal and skip the mask arithmetic.
    const int cnt_plain = min(cnt, first_masked_tile > wave ? (first_masked_tile - wave + 3) / 4 : 0);
    int it = 0;
    auto run = [&](auto masked, int end) __attribute__((always_inline)) {
        while (it < end) {
            bool slow = false;
            for (; it < end; ++it) {
                if (front(masked, it)) {
                    slow = true;
                    break;
                }
                back(it);
            }
            if (slow) {
                rescale_all();
                back(it);
                ++it;
            }
        }
    };
    run(std::false_type{}, cnt_plain);
    run(std::true_type{}, cnt);
#if ATT_TIMELINE
    const unsigned long long tl_loop_end = __builtin_amdgcn_s_memtime();
#endif

    // ---- merge the four waves' partial results --------------------------------------------------------
    // Statistics live past the tile slots; the fp32 output regions (one per wave) overlap other waves' slots
    // and are written only after the barrier.
    constexpr int kORow = 132;                              // padded fp32 row
    constexpr int kRegion = QB * 32 * kORow;                // floats per wave
    float* obuf = (float*)lds;                              // [4][QB*32][132]
    float* stat_m = (float*)(lds + kStatOffset);            // [4][QB*32]
    float* stat_l = stat_m + 4 * QB * 32;                   // [4][QB*32]
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
        if (hh == 0) {
            stat_m[wave * QB * 32 + qb * 32 + c] = m_run[qb];
            stat_l[wave * QB * 32 + qb * 32 + c] = l_tot;
        }
    }
    __syncthreads();  // statistics visible; every wave is done with its tile slots
    float* mine = obuf + wave * kRegion;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        float m_all = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, stat_m[w * QB * 32 + qb * 32 + c]);
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = stat_m[w * QB * 32 + qb * 32 + c];
            l_all += mw == -INFINITY ? 0.f : stat_l[w * QB * 32 + qb * 32 + c] * exp2f(mw - m_all);
        }
        const float wscale = m_run[qb] == -INFINITY ? 0.f : exp2f(m_run[qb] - m_all) / l_all;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int g = 0; g < 4; ++g) {
                // registers 4g..4g+3 are dh = db*32 + 8g + 4hh + {0..3}: one 16-byte vector
                *(float4*)(mine + (qb * 32 + c) * kORow + db * 32 + 8 * g + 4 * hh) =
                    make_float4(oacc[qb][db][4 * g] * wscale, oacc[qb][db][4 * g + 1] * wscale,
                                oacc[qb][db][4 * g + 2] * wscale, oacc[qb][db][4 * g + 3] * wscale);
            }
    }
    __syncthreads();
    // Sum the four regions (fixed order) and write out in the GEMM operand layout: a thread handles 8
    // consecutive dh of one query per step.
    for (int idx = tid; idx < QB * 32 * 16; idx += 256) {
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        const float* src = obuf + qr * kORow + ch * 8;
        float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4 a2 = *(const float4*)(src + w * kRegion), b2 = *(const float4*)(src + w * kRegion + 4);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
        }
        u32x4 out;
        out[0] = pack_bf16x2(a.x, a.y); out[1] = pack_bf16x2(a.z, a.w);
        out[2] = pack_bf16x2(b.x, b.y); out[3] = pack_bf16x2(b.z, b.w);
        *(u32x4*)(o + tiled_offset(row0 + qrow, head * 16 + ch, d_model >> 5)) = out;
    }
#if ATT_TIMELINE
    __syncthreads();
    if (tid == 0) {
        unsigned long long* t = (unsigned long long*)o + (size_t)blockIdx.x * 8;
        t[0] = tl[0]; t[1] = tl[1]; t[2] = tl[2]; t[3] = tl[3]; t[4] = tl_loop_end - tl_begin; t[5] = tl[5];
        t[6] = __builtin_amdgcn_s_memtime() - tl_begin; t[7] = 0x1234;
    }
#endif
}


// ---------------------------------------------------------------------------------------------------------------
// Second kernel: the same work split over twice the waves, plus four waves that only fetch.  A workgroup is
// still NQ*32 queries of one head, but every computing wave owns ONE block of 32 queries and one quarter of the
// keys: wave = 4*qb + g handles query block qb against the tiles g, g+4, ...  The waves of a key quarter (one
// per query block) share that quarter's tiles in LDS; loader wave g keeps them one tile ahead, and all waves
// meet at one workgroup barrier per round.  With 64 accumulator registers per wave instead of 128, three waves
// fit a SIMD (two computing, one loading): while one waits for LDS or works through its softmax on the vector
// ALU, the other has the matrix pipe, and no computing wave is held by the issue of a global->LDS load.
template <int NQ>
__global__ __launch_bounds__(256 * NQ + 256) void chunk_attention2_bf16(const u16* __restrict__ q, u16* __restrict__ o,
                                                                  int n, int d_model, int n_heads, int pos0_arg,
                                                                  KvView kv_arg, int layer, float scale_log2e,
                                                                  const BranchTable* __restrict__ branches) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    // Waves 0 .. 4 NQ - 1 compute (key quarter g, query block qb); the last four waves only fetch tiles, one per
    // key quarter.  A global->LDS load holds the issuing wave for about a hundred cycles (the address path of a
    // CU takes 64 bytes per clock, and all quarters refill at the same moment): issued by the computing waves,
    // the loads of a round cost them as much as the round's arithmetic.
    const bool loader = wave >= 4 * NQ;
    const int g = wave & 3, qb = loader ? 0 : wave >> 2;
    const int c = lane & 31, hh = lane >> 5;
    const int head = blockIdx.x % n_heads;
    const int q_blocks = (n + NQ * 32 - 1) / (NQ * 32);
    const int bq = blockIdx.x / n_heads;
    const int branch = bq / q_blocks;  // 0 without a branch table
    const int q0 = (q_blocks - 1 - bq % q_blocks) * (NQ * 32);
    const int row0 = branch * n;
    const int pos0 = branches ? branches->pos0[branch] : pos0_arg;
    const KvView kv = branches ? branches->kv[branch] : kv_arg;
    q += (size_t)row0 * d_model;
    const int q_last = min(q0 + NQ * 32, n) - 1;  // last real query of this workgroup
    const int n_keys = pos0 + q_last + 1;
    const int n_tiles = (n_keys + kKT - 1) / kKT;
    const int last_key = n_keys - 1;
    const int first_masked_tile = (pos0 + q0 + 1) / kKT;

    unsigned char* grp = lds + g * kWaveLds;  // this key quarter's two slots (K tile + V tile each)
    const unsigned grp_addr = __builtin_amdgcn_readfirstlane(lds_byte_address(lds)) + g * kWaveLds;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + head;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + head;

    const int cnt = n_tiles > g ? (n_tiles - g + 3) / 4 : 0;  // tiles of this key quarter
    const int max_cnt = (n_tiles + 3) / 4;                    // of quarter 0: every wave runs that many rounds
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
            fill_part(tile, slot, false);
            fill_part(tile, slot, true);
        };
        if (cnt > 0) fill(g, 0);
        for (int it = 0; it < max_cnt; ++it) {
            asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // the tile of this round has landed
            __builtin_amdgcn_s_barrier();                     // ... and the other slot is free
            if (it + 1 < cnt) fill(g + 4 * (it + 1), (it + 1) & 1);
        }
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();  // the two barriers of the merge
        __syncthreads();
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

    const int q_abs = pos0 + q0 + qb * 32 + c;  // absolute position of this lane's query

#if ATT_TIMELINE
    unsigned long long tl[6] = {0, 0, 0, 0, 0, 0};
    const unsigned long long tl_begin = __builtin_amdgcn_s_memtime();
#endif
    for (int it = 0; it < max_cnt; ++it) {
        ATT_T(ta);
        // One barrier per round: the loader arrives when the tile of this round has landed, the computing waves
        // when they are done with the other slot, which the loader then refills.
        __builtin_amdgcn_s_barrier();
        ATT_T(tb);
        if (it >= cnt) continue;
        ATT_T(t0);
        const int tile = g + 4 * it, slot = it & 1;
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
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(sacc));
#endif
        ATT_T(t1);
        float sv[16];
#pragma unroll
        for (int r = 0; r < 16; ++r) sv[r] = sacc[r];
        if (tile >= first_masked_tile) {  // the tile reaches some query's diagonal (a few tiles per workgroup)
            asm volatile("");             // keeps this a branch: merged into selects it would run for every tile
            const int key0 = tile * kKT;
#pragma unroll
            for (int r = 0; r < 16; ++r)
                if (key0 + acc_row(r, hh) > q_abs) sv[r] = -INFINITY;
        }
        float mt = -INFINITY;
#pragma unroll
        for (int r = 0; r < 16; ++r) mt = fmaxf(mt, sv[r]);
        mt = max_across_halves(mt) * scale_log2e;  // the scale is positive
        const bool grow = mt > m_run + 8.0f;       // lazy reference maximum, see the first kernel
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
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(pf[0]), "+v"(pf[1]));
#endif
        ATT_T(t2);
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
#if ATT_TIMELINE
        asm volatile("s_nop 0" : "+v"(oacc[3]));
        ATT_T(t3);
        tl[0] += t1 - t0; tl[1] += t2 - t1; tl[2] += t3 - t2; tl[3] += tb - ta; tl[4] += t0 - tb; tl[5] += 1;
#endif
    }
#if ATT_TIMELINE
    const unsigned long long tl_loop_end = __builtin_amdgcn_s_memtime();
#endif

    // ---- merge the four key quarters of every query block ----------------------------------------------------------
    constexpr int kORow = 132;
    constexpr int kRegion = 64 * kORow;                     // floats per key quarter: [64 queries][132]
    float* obuf = (float*)lds;
    float* stat_m = (float*)(lds + kStatOffset);            // [4][64]
    float* stat_l = stat_m + 4 * 64;
    {
        const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
        if (hh == 0) {
            stat_m[g * 64 + qb * 32 + c] = m_run;
            stat_l[g * 64 + qb * 32 + c] = l_tot;
        }
    }
    __syncthreads();  // statistics visible; every wave is done with the tile slots
    {
        float m_all = -INFINITY;
#pragma unroll
        for (int w = 0; w < 4; ++w) m_all = fmaxf(m_all, stat_m[w * 64 + qb * 32 + c]);
        float l_all = 0.f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = stat_m[w * 64 + qb * 32 + c];
            l_all += mw == -INFINITY ? 0.f : stat_l[w * 64 + qb * 32 + c] * exp2f(mw - m_all);
        }
        const float wscale = m_run == -INFINITY ? 0.f : exp2f(m_run - m_all) / l_all;
        float* mine = obuf + g * kRegion + (qb * 32 + c) * kORow;
#pragma unroll
        for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int gg = 0; gg < 4; ++gg)
                *(float4*)(mine + db * 32 + 8 * gg + 4 * hh) =
                    make_float4(oacc[db][4 * gg] * wscale, oacc[db][4 * gg + 1] * wscale,
                                oacc[db][4 * gg + 2] * wscale, oacc[db][4 * gg + 3] * wscale);
    }
    __syncthreads();
    for (int idx = tid; idx < NQ * 32 * 16; idx += 256 * NQ) {
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        const float* src = obuf + qr * kORow + ch * 8;
        float4 a = *(const float4*)src, b = *(const float4*)(src + 4);
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float4 a2 = *(const float4*)(src + w * kRegion), b2 = *(const float4*)(src + w * kRegion + 4);
            a.x += a2.x; a.y += a2.y; a.z += a2.z; a.w += a2.w;
            b.x += b2.x; b.y += b2.y; b.z += b2.z; b.w += b2.w;
        }
        u32x4 out;
        out[0] = pack_bf16x2(a.x, a.y); out[1] = pack_bf16x2(a.z, a.w);
        out[2] = pack_bf16x2(b.x, b.y); out[3] = pack_bf16x2(b.z, b.w);
        *(u32x4*)(o + tiled_offset(row0 + qrow, head * 16 + ch, d_model >> 5)) = out;
    }
#if ATT_TIMELINE
    __syncthreads();
    if (tid == 0) {
        unsigned long long* t = (unsigned long long*)o + (size_t)blockIdx.x * 8;
        t[0] = tl[0]; t[1] = tl[1]; t[2] = tl[2]; t[3] = tl[3]; t[4] = tl_loop_end - tl_begin; t[5] = tl[5];
        t[6] = tl[4]; t[7] = 0x1234;
    }
#endif
}

}  // namespace

#ifndef JUP_ATTENTION_KERNEL
#define JUP_ATTENTION_KERNEL 2
#endif

hipError_t attention_configure() {
    hipError_t e2 = hipFuncSetAttribute((const void*)chunk_attention2_bf16<1>,
                                        hipFuncAttributeMaxDynamicSharedMemorySize, kAttLds);
    if (e2 == hipSuccess)
        e2 = hipFuncSetAttribute((const void*)chunk_attention2_bf16<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                 kAttLds);
    if (e2 != hipSuccess) return e2;
    hipError_t e = hipFuncSetAttribute((const void*)chunk_attention_bf16<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       kAttLds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)chunk_attention_bf16<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               kAttLds);
}

void launch_chunk_attention(const u16* q, u16* o, int n, int d_model, int n_heads, int pos0, const KvView& kv,
                            int layer, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    const BranchTable* none = nullptr;
#if JUP_ATTENTION_KERNEL == 2
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention2_bf16<1>, dim3((n + 31) / 32 * n_heads), dim3(512), kAttLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e, none);
    else
        hipLaunchKernelGGL(chunk_attention2_bf16<2>, dim3((n + 63) / 64 * n_heads), dim3(768), kAttLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e, none);
#else
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention_bf16<1>, dim3((n + 31) / 32 * n_heads), dim3(256), kAttLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e, none);
    else
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3((n + 63) / 64 * n_heads), dim3(256), kAttLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e, none);
#endif
}

void launch_branch_attention(const u16* q, u16* o, int n, int n_branches, int d_model, int n_heads,
                             const BranchTable* branches, int layer, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    const KvView none{};
#if JUP_ATTENTION_KERNEL == 2
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention2_bf16<1>, dim3(n_branches * ((n + 31) / 32) * n_heads), dim3(512), kAttLds,
                           s, q, o, n, d_model, n_heads, 0, none, layer, scale_log2e, branches);
    else
        hipLaunchKernelGGL(chunk_attention2_bf16<2>, dim3(n_branches * ((n + 63) / 64) * n_heads), dim3(768), kAttLds,
                           s, q, o, n, d_model, n_heads, 0, none, layer, scale_log2e, branches);
#else
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention_bf16<1>, dim3(n_branches * ((n + 31) / 32) * n_heads), dim3(256), kAttLds, s,
                           q, o, n, d_model, n_heads, 0, none, layer, scale_log2e, branches);
    else
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3(n_branches * ((n + 63) / 64) * n_heads), dim3(256), kAttLds, s,
                           q, o, n, d_model, n_heads, 0, none, layer, scale_log2e, branches);
#endif
}

}  // namespace jup
