// Chunk attention of the bf16 path: the chunk's queries against the cached prefix plus the causal
// triangle inside the chunk (Jupiter paper, Sec. IV-A.2, Fig. 4b), MFMA 32x32x16 with online softmax.
//
// One workgroup = QB*32 queries of one head, 4 waves.  The waves split the key range: wave w takes the
// 32-key tiles w, w+4, ... of the keys this query block can see.  Each wave runs a private two-slot
// LDS pipeline filled by direct global->LDS loads, so the main loop has no workgroup barrier.  Each
// wave computes the TRANSPOSED products
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

namespace jup {
namespace {

typedef short s16x4 __attribute__((ext_vector_type(4)));

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
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

// LDS tile layouts (rows of 256 bytes = 16 chunks of 16 bytes):
//   K: chunk ch of row r at position ch ^ (r & 15)            (16 consecutive rows, same chunk: 16 banksets)
//   V: chunk ch of row r at position (((ch >> 2) ^ (r & 3)) << 2) | (ch & 3)   (4 consecutive rows spread
//      their 64-byte groups over the four 64-byte bank groups for the transposing reads)
__device__ inline int k_pos(int r, int ch) { return ch ^ (r & 15); }
__device__ inline int v_pos(int r, int ch) { return (((ch >> 2) ^ (r & 3)) << 2) | (ch & 3); }

template <int QB>
__global__ __launch_bounds__(256) void chunk_attention_bf16(const u16* __restrict__ q, u16* __restrict__ o, int n,
                                                            int d_model, int n_heads, int pos0, KvView kv, int layer,
                                                            float scale_log2e) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int c = lane & 31, hh = lane >> 5;
    // Workgroup b runs on XCD b % 8: heads vary fastest so that every query block of a head reads that
    // head's keys and values through the same L2; the longest query blocks (most visible keys) start first.
    const int head = blockIdx.x % n_heads;
    const int q0 = ((int)(gridDim.x / n_heads) - 1 - (int)(blockIdx.x / n_heads)) * (QB * 32);
    const int q_last = min(q0 + QB * 32, n) - 1;  // last real query of this block
    const int n_keys = pos0 + q_last + 1;         // keys 0 .. n_keys-1 are visible to the block
    const int n_tiles = (n_keys + kKT - 1) / kKT;
    const int last_key = n_keys - 1;   // rows past it are loaded from it and masked
    const int first_masked_tile = (pos0 + q0 + 1) / kKT;  // tiles before it lie below every query's diagonal

    unsigned char* my = lds + wave * kWaveLds;
    const size_t plane_k = ((size_t)layer * 2 + 0) * n_heads + head;
    const size_t plane_v = ((size_t)layer * 2 + 1) * n_heads + head;

    // Q fragments (B operand of S^T): lane = query column, 8 consecutive dh per k-step.
    bf16x8 qf[QB][8];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int qrow = min(q0 + qb * 32 + c, n - 1);
        const u16* qp = q + (size_t)qrow * d_model + head * 128 + 8 * hh;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) qf[qb][ks] = *(const bf16x8*)(qp + 16 * ks);
    }

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
    // lands at row 4j + (i >> 4), position i & 15, and fetches the chunk that belongs there.
    const int lrow = lane >> 4, lp = lane & 15;
    // plane bases of the two cache segments (the parent's is never dereferenced when nothing is shared)
    const u16* k_own = (const u16*)kv.own + plane_k * (size_t)kv.own_cap * 128;
    const u16* v_own = (const u16*)kv.own + plane_v * (size_t)kv.own_cap * 128;
    const u16* k_par = (const u16*)kv.parent + plane_k * (size_t)kv.parent_cap * 128;
    const u16* v_par = (const u16*)kv.parent + plane_v * (size_t)kv.parent_cap * 128;
    auto fill = [&](int tile, int slot) {
        unsigned char* kd = my + slot * kSlotBytes;
        unsigned char* vd = kd + kTileBytes;
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int r = 4 * j + lrow;
            const int key = min(tile * kKT + r, last_key);
            const bool shared = key < kv.n_shared;
            const unsigned row_off = (unsigned)(shared ? key : key - kv.n_shared) * 128u;  // elements, < 2^31
            const u16* kr = (shared ? k_par : k_own) + row_off + (lp ^ (r & 15)) * 8;
            const u16* vr = (shared ? v_par : v_own) + row_off + ((((lp >> 2) ^ (r & 3)) << 2) | (lp & 3)) * 8;
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)kr,
                                             (__attribute__((address_space(3))) void*)(kd + j * 1024), 16, 0, 0);
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)vr,
                                             (__attribute__((address_space(3))) void*)(vd + j * 1024), 16, 0, 0);
        }
    };

    // Per-lane LDS read offsets.
    //   K fragment (ks): row c, chunk 2ks + hh.
    //   V^T fragment (db, ks, part): transposing read; lane = 16*G + s supplies the address of
    //   V[key = 16ks + 8*part + 4*(G>>1) + (s>>2)][dh = 32db + 16*(G&1) + 4*(s&3) .. +3].
    const int G = lane >> 4, s = lane & 15;
    const int vt_row = 4 * (G >> 1) + (s >> 2);         // + 16ks + 8part
    const int vt_dh = 16 * (G & 1) + 4 * (s & 3);       // + 32db   (in elements)

    int tile = wave;
    int slot = 0;
    if (tile < n_tiles) fill(tile, 0);
    for (; tile < n_tiles; tile += 4) {
        wait_vmcnt<0>();  // this tile has landed (only this wave reads it)
        if (tile + 4 < n_tiles) fill(tile + 4, slot ^ 1);
        const unsigned char* ks_base = my + slot * kSlotBytes;
        const unsigned char* vs_base = ks_base + kTileBytes;

        // S^T = K Q^T for the 32 keys of the tile.
        f32x16 sacc[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = *(const bf16x8*)(ks_base + c * 256 + k_pos(c, 2 * ks + hh) * 16);
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[qb] = mfma32(kf, qf[qb][ks], sacc[qb]);
        }

        const int key0 = tile * kKT;
        const bool need_mask = tile >= first_masked_tile;
        bf16x8 pf[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int q_abs = pos0 + q0 + qb * 32 + c;  // absolute position of this lane's query
            float sv[16];
            float mt = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                sv[r] = sacc[qb][r] * scale_log2e;
                if (need_mask && key0 + acc_row(r, hh) > q_abs) sv[r] = -INFINITY;
                mt = fmaxf(mt, sv[r]);
            }
            mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
            const float m_new = fmaxf(m_run[qb], mt);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_safe);
            float ps = 0.f;
            float pv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pv[r] = __builtin_amdgcn_exp2f(sv[r] - m_safe);
                ps += pv[r];
            }
            l_run[qb] = l_run[qb] * alpha + ps;
            m_run[qb] = m_new;
            if (__any(alpha != 1.0f)) {
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int r = 0; r < 16; ++r) oacc[qb][db][r] *= alpha;
            }
#pragma unroll
            for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                for (int e = 0; e < 8; ++e) pf[qb][ks][e] = (__bf16)pv[8 * ks + e];
        }

        // O^T += V^T P^T.
#pragma unroll
        for (int db = 0; db < 4; ++db) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                s16x4 part[2];
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const int r = 16 * ks + 8 * pt + vt_row;
                    const int el = 32 * db + vt_dh;  // element index in the row; chunk = el >> 3, +8 bytes if el & 4
                    const unsigned char* ap = vs_base + r * 256 + v_pos(r, el >> 3) * 16 + (el & 4) * 2;
                    part[pt] = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) s16x4*)ap);
                }
                // the two 8-byte results are the low and high halves of the 16-byte operand
                const u32x2 lo = __builtin_bit_cast(u32x2, part[0]), hi = __builtin_bit_cast(u32x2, part[1]);
                const bf16x8 vf = __builtin_bit_cast(bf16x8, (u32x4){lo[0], lo[1], hi[0], hi[1]});
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mfma32(vf, pf[qb][ks], oacc[qb][db]);
            }
        }
        slot ^= 1;
    }
    wait_vmcnt<0>();

    // ---- merge the four waves' partial results --------------------------------------------------------
    __syncthreads();  // every wave is done with its tile slots; LDS is reused below
    float* stat_m = (float*)lds;                  // [4][QB*32]
    float* stat_l = stat_m + 4 * QB * 32;         // [4][QB*32]
    float* obuf = stat_l + 4 * QB * 32;           // [QB*32][132] fp32 (padded rows)
    constexpr int kORow = 132;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32, 64);
        if (hh == 0) {
            stat_m[wave * QB * 32 + qb * 32 + c] = m_run[qb];
            stat_l[wave * QB * 32 + qb * 32 + c] = l_tot;
        }
    }
    __syncthreads();
    float wscale[QB];
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
        wscale[qb] = m_run[qb] == -INFINITY ? 0.f : exp2f(m_run[qb] - m_all) / l_all;
    }
    for (int w = 0; w < 4; ++w) {
        if (wave == w) {
#pragma unroll
            for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                for (int db = 0; db < 4; ++db)
#pragma unroll
                    for (int g = 0; g < 4; ++g) {
                        // registers 4g..4g+3 are dh = db*32 + 8g + 4hh + {0..3}: one 16-byte vector
                        float4* p = (float4*)(obuf + (qb * 32 + c) * kORow + db * 32 + 8 * g + 4 * hh);
                        float4 v = make_float4(oacc[qb][db][4 * g] * wscale[qb], oacc[qb][db][4 * g + 1] * wscale[qb],
                                               oacc[qb][db][4 * g + 2] * wscale[qb], oacc[qb][db][4 * g + 3] * wscale[qb]);
                        if (w > 0) {
                            const float4 old = *p;
                            v.x += old.x; v.y += old.y; v.z += old.z; v.w += old.w;
                        }
                        *p = v;
                    }
        }
        __syncthreads();
    }
    // Write out in the GEMM operand layout: thread handles 8 consecutive dh of one query per step.
    for (int idx = tid; idx < QB * 32 * 16; idx += 256) {
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        const float* src = obuf + qr * kORow + ch * 8;
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = pack_bf16x2(src[2 * e], src[2 * e + 1]);
        *(u32x4*)(o + tiled_offset(qrow, head * 16 + ch, d_model >> 5)) = out;
    }
}

}  // namespace

hipError_t attention_configure() {
    hipError_t e = hipFuncSetAttribute((const void*)chunk_attention_bf16<1>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                       4 * kWaveLds);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute((const void*)chunk_attention_bf16<2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                               4 * kWaveLds);
}

void launch_chunk_attention(const u16* q, u16* o, int n, int d_model, int n_heads, int pos0, const KvView& kv,
                            int layer, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention_bf16<1>, dim3((n + 31) / 32 * n_heads), dim3(256), 4 * kWaveLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e);
    else
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3((n + 63) / 64 * n_heads), dim3(256), 4 * kWaveLds, s, q, o, n,
                           d_model, n_heads, pos0, kv, layer, scale_log2e);
}

}  // namespace jup
