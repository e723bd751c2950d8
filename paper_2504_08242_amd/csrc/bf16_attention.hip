// Chunk attention of the bf16 path: the chunk's queries against the cached prefix plus the causal
// triangle inside the chunk (Jupiter paper, Sec. IV-A.2, Fig. 4b), MFMA 32x32x16 with online softmax.
//
// MFMA 32x32x16 bf16 operand layout (lane = 32*hh + c):
//   A: lane supplies A[m = c][k = 8*hh + e], e < 8;  B: lane supplies B[k = 8*hh + e][n = c];
//   D: lane holds D[m = 8*(i/4) + 4*hh + (i%4)][n = c] in register i < 16.
#include "bf16_common.h"

namespace jup {
namespace {

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}
// Row of D held in accumulator register i by a lane of half hh.
__device__ inline int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

// ------------------------------------------------------------------------------------------------
// Chunk attention: queries of the chunk against the cached prefix plus the causal triangle.
//
// One workgroup = QB*32 queries of one head, 4 waves.  The waves split the key range: wave w takes the
// 32-key tiles w, w+4, ... of the keys this query block can see, with a private LDS region, so the
// main loop needs no workgroup barrier.  Each wave computes the TRANSPOSED products
//     S^T[key][query] = K Q^T        (A = K tile rows, B = Q)
//     O^T[dh][query] += V^T P^T      (A = V^T tile, B = P^T taken straight from the S^T accumulators)
// so that a lane always owns one query column: softmax statistics are per-lane scalars.  The four
// partial results are merged at the end with the usual log-sum-exp weights.
//
// A lane (query column cq, half hh) holds S^T for keys  8*(i/4) + 4*hh + (i%4), i < 16.  The PV MFMA
// number ks (0/1) consumes registers 8ks..8ks+7, i.e. its contraction index 8*hh + e stands for key
// 16ks + 8*(e/4) + 4*hh + (e%4); V^T is written to LDS with the keys of a row in that order.
// ------------------------------------------------------------------------------------------------
constexpr int kKT = 32;                      // keys per tile
constexpr int kWaveLds = kKT * 128 * 2 * 2;  // K tile + V^T tile, bytes per wave

template <int QB>
__global__ __launch_bounds__(256) void chunk_attention_bf16(const u16* __restrict__ q, u16* __restrict__ o, int n,
                                                            int d_model, int n_heads, int pos0, KvView kv, int layer,
                                                            float scale_log2e) {
    __shared__ __attribute__((aligned(16))) unsigned char lds[4 * kWaveLds];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int c = lane & 31, hh = lane >> 5;
    const int head = blockIdx.y;
    const int q0 = blockIdx.x * (QB * 32);
    const int q_last = min(q0 + QB * 32, n) - 1;  // last real query of this block
    const int n_keys = pos0 + q_last + 1;         // keys 0 .. n_keys-1 are visible to the block
    const int n_tiles = (n_keys + kKT - 1) / kKT;
    const int last_key = n_keys - 1;  // rows past it are loaded from it and masked

    u16* Ks = (u16*)(lds + wave * kWaveLds);  // [32 keys][128], chunk ch of row r at ch ^ (r & 7)
    u16* Vt = Ks + kKT * 128;                 // [128 dh][32 keys], chunk ch of row r at ch ^ ((r >> 1) & 3)

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

    // Tile staging: lane loads 16-byte chunks lane + 64*j (j < 8) of the K tile and of the V tile;
    // chunk index = row * 16 + chunk_in_row (16 lanes cover one 256-byte row).
    u32x4 rk[8], rv[8];
    auto load_tile = [&](int tile) {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int idx = lane + 64 * j;
            const int r = idx >> 4, ch = idx & 15;
            const int key = min(tile * kKT + r, last_key);
            rk[j] = *(const u32x4*)(kv_row_bf16(kv, plane_k, key) + ch * 8);
            rv[j] = *(const u32x4*)(kv_row_bf16(kv, plane_v, key) + ch * 8);
        }
    };
    auto store_tile = [&]() {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int idx = lane + 64 * j;
            const int r = idx >> 4, ch = idx & 15;
            *(u32x4*)(Ks + r * 128 + ((ch ^ (r & 7)) << 3)) = rk[j];
            // V^T: key r goes to in-row position 16*ks + 8*hh' + 4*a + cc where r = 16*ks + 8*a + 4*hh' + cc
            const int kpos = (r & 16) | ((r & 4) << 1) | ((r & 8) >> 1) | (r & 3);
            const int kch = kpos >> 3, kin = kpos & 7;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int dh = ch * 8 + e;
                const unsigned word = rv[j][e >> 1];
                const u16 val = (e & 1) ? (u16)(word >> 16) : (u16)(word & 0xffff);
                Vt[dh * kKT + ((kch ^ ((dh >> 1) & 3)) << 3) + kin] = val;
            }
        }
    };

    int tile = wave;
    if (tile < n_tiles) load_tile(tile);
    for (; tile < n_tiles; tile += 4) {
        __builtin_amdgcn_wave_barrier();
        store_tile();
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        if (tile + 4 < n_tiles) load_tile(tile + 4);

        // S^T = K Q^T for the 32 keys of the tile.
        f32x16 sacc[QB];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb)
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[qb][r] = 0.f;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const bf16x8 kf = *(const bf16x8*)(Ks + c * 128 + (((2 * ks + hh) ^ (c & 7)) << 3));
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) sacc[qb] = mfma32(kf, qf[qb][ks], sacc[qb]);
        }

        const int key0 = tile * kKT;
        bf16x8 pf[QB][2];
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            const int q_abs = pos0 + q0 + qb * 32 + c;  // absolute position of this lane's query
            float sv[16];
            float mt = -INFINITY;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int key = key0 + acc_row(r, hh);
                sv[r] = key <= q_abs ? sacc[qb][r] * scale_log2e : -INFINITY;
                mt = fmaxf(mt, sv[r]);
            }
            mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
            const float m_new = fmaxf(m_run[qb], mt);
            const float m_safe = m_new == -INFINITY ? 0.f : m_new;
            const float alpha = exp2f(m_run[qb] - m_safe);
            float ps = 0.f;
            float pv[16];
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                pv[r] = exp2f(sv[r] - m_safe);
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
            const int dh = db * 32 + c;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const bf16x8 vf = *(const bf16x8*)(Vt + dh * kKT + (((2 * ks + hh) ^ ((dh >> 1) & 3)) << 3));
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) oacc[qb][db] = mfma32(vf, pf[qb][ks], oacc[qb][db]);
            }
        }
    }

    // ---- merge the four waves' partial results --------------------------------------------------------
    __syncthreads();  // every wave is done with its tile buffers; LDS is reused below
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
    // Write out: thread handles 8 consecutive dh of one query per step.
    for (int idx = tid; idx < QB * 32 * 16; idx += 256) {
        const int qr = idx >> 4, ch = idx & 15;
        const int qrow = q0 + qr;
        if (qrow >= n) continue;
        const float* src = obuf + qr * kORow + ch * 8;
        u32x4 out;
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (unsigned)f2bf(src[2 * e]) | ((unsigned)f2bf(src[2 * e + 1]) << 16);
        *(u32x4*)(o + (size_t)qrow * d_model + head * 128 + ch * 8) = out;
    }
}


}  // namespace

void launch_chunk_attention(const u16* q, u16* o, int n, int d_model, int n_heads, int pos0, const KvView& kv,
                            int layer, hipStream_t s) {
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);
    if (n <= 32)
        hipLaunchKernelGGL(chunk_attention_bf16<1>, dim3((n + 31) / 32, n_heads), dim3(256), 0, s, q, o, n, d_model,
                           n_heads, pos0, kv, layer, scale_log2e);
    else
        hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3((n + 63) / 64, n_heads), dim3(256), 0, s, q, o, n, d_model,
                           n_heads, pos0, kv, layer, scale_log2e);
}

}  // namespace jup
