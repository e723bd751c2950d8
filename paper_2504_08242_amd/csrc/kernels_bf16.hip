// Matrix-core (JUP_BF16) path for gfx950: bf16 storage, fp32 accumulation on MFMA 32x32x16, fp32
// residual stream inside a call.  One stage forward over one sub-sequence with its cached prefix
// (Jupiter paper, Sec. IV-A.2); the decoder layer of Sec. II-A in its Llama-2 form.
//
// Per layer:  rmsnorm -> [QKV GEMM + rotary + KV append] -> chunk attention -> [O GEMM + residual]
//             -> rmsnorm -> [gate/up GEMM + SwiGLU] -> [down GEMM + residual]
//
// MFMA 32x32x16 bf16 operand layout (wave of 64 lanes, lane = 32*hh + c):
//   A (M x K): lane supplies A[m = c][k = 8*hh + e], e = 0..7          (one 16-byte vector)
//   B (K x N): lane supplies B[k = 8*hh + e][n = c]
//   D (M x N): lane holds, in register i of 16, D[m = 8*(i/4) + 4*hh + (i%4)][n = c]
#include "jup_internal.h"

namespace jup {
namespace {

typedef unsigned short u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ inline u16 f2bf(float f) {
    __bf16 b = (__bf16)f;  // round to nearest even
    return __builtin_bit_cast(u16, b);
}
__device__ inline float bf2f(u16 b) { return __uint_as_float((unsigned)b << 16); }

__device__ inline f32x16 mfma32(bf16x8 a, bf16x8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
}

// Row of D held in accumulator register i by a lane of half hh.
__device__ inline int acc_row(int i, int hh) { return 8 * (i >> 2) + 4 * hh + (i & 3); }

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// ------------------------------------------------------------------------------------------------
// Weight packing (runs once, at jup_stage_create).
// ------------------------------------------------------------------------------------------------

// Within a head, packed row 64a + 32b + c holds original row 64b + 32a + c (a, b in {0,1}, c < 32):
// the rotary partners i and i + 64 then sit in adjacent 32-column blocks of one 64-column wave tile.
__device__ __host__ inline int rope_unpermute(int packed) {
    return (packed & 31) | ((packed & 32) << 1) | ((packed & 64) >> 1);
}

// dst: [3d, d].  Rows [0,d): Q heads (permuted inside each head), [d,2d): K heads (permuted), [2d,3d): V.
__global__ void pack_qkv(u16* __restrict__ dst, const u16* __restrict__ wq, const u16* __restrict__ wk,
                         const u16* __restrict__ wv, int d) {
    const int r = blockIdx.x;  // packed row
    const int which = r / d, rr = r % d;
    const int head = rr >> 7, in_head = rr & 127;
    const int src_row = head * 128 + (which == 2 ? in_head : rope_unpermute(in_head));
    const u16* src = (which == 0 ? wq : which == 1 ? wk : wv) + (size_t)src_row * d;
    const u32x4* s4 = (const u32x4*)src;
    u32x4* d4 = (u32x4*)(dst + (size_t)r * d);
    for (int i = threadIdx.x; i < d / 8; i += blockDim.x) d4[i] = s4[i];
}

// dst: [2f, d].  Packed rows come in groups of 64: 32 gate rows, then the 32 up rows of the same features.
__global__ void pack_gate_up(u16* __restrict__ dst, const u16* __restrict__ wg, const u16* __restrict__ wu, int d) {
    const int r = blockIdx.x;
    const int group = r >> 6, w = r & 63;
    const u16* src = (w < 32 ? wg : wu) + (size_t)(group * 32 + (w & 31)) * d;
    const u32x4* s4 = (const u32x4*)src;
    u32x4* d4 = (u32x4*)(dst + (size_t)r * d);
    for (int i = threadIdx.x; i < d / 8; i += blockDim.x) d4[i] = s4[i];
}

// ------------------------------------------------------------------------------------------------
// Rotary table of the chunk: tab[t][i] = (cos, sin)((pos0 + t) * theta^(-2i/dh)), angles in fp64.
// ------------------------------------------------------------------------------------------------
__global__ void rope_table(float2* __restrict__ tab, int n, int half, int pos0, float theta) {
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * half) return;
    const int i = gid % half, t = gid / half;
    const double ang = (double)(pos0 + t) * pow((double)theta, -(double)i / (double)half);
    tab[gid] = make_float2((float)cos(ang), (float)sin(ang));
}

// ------------------------------------------------------------------------------------------------
// RMSNorm.  One 256-thread block per row.  SRC_BF16: the row comes from hidden_in (bf16) and is also
// copied into the fp32 residual stream; otherwise it is read from the residual stream.
// ------------------------------------------------------------------------------------------------
template <bool SRC_BF16>
__global__ __launch_bounds__(256) void rmsnorm_bf16(const void* __restrict__ src, float* __restrict__ x32,
                                                    const u16* __restrict__ g, u16* __restrict__ xn, int d,
                                                    float eps) {
    __shared__ float part[4];
    const size_t row = blockIdx.x;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) {
        float v;
        if (SRC_BF16) {
            v = bf2f(((const u16*)src)[row * d + j]);
            x32[row * d + j] = v;
        } else {
            v = ((const float*)src)[row * d + j];
        }
        ss += v * v;
    }
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float inv = 1.0f / sqrtf((part[0] + part[1] + part[2] + part[3]) / (float)d + eps);
    for (int j = threadIdx.x; j < d; j += 256) {
        const float v = SRC_BF16 ? bf2f(((const u16*)src)[row * d + j]) : ((const float*)src)[row * d + j];
        xn[row * d + j] = f2bf(v * inv * bf2f(g[j]));
    }
}

// ------------------------------------------------------------------------------------------------
// GEMM  C[M, N] = A[M, K] * W[N, K]^T  with fused epilogues.
// 128 x 128 x 64 tiles, 256 threads = 2 x 2 waves of 64 x 64, LDS double buffer, register prefetch.
// LDS rows are 128 bytes (64 bf16); 16-byte chunk c of row r is stored at chunk c ^ (r & 7).
// ------------------------------------------------------------------------------------------------
enum { EPI_QKV = 0, EPI_RESID = 1, EPI_SWIGLU = 2 };

struct GemmArgs {
    const u16* A;  // [M, K]
    const u16* W;  // [N, K]
    int M, N, K;
    // EPI_QKV
    u16* q_out;          // [M, d]
    const float2* rope;  // [M, 64]
    KvView kv;
    int layer, n_heads, d_model, pos0;
    // EPI_RESID
    float* x32;      // [M, N] accumulated in place
    u16* final_out;  // optional bf16 copy of the updated rows (after the stage's last layer)
    // EPI_SWIGLU
    u16* act;  // [M, N/2]
};

constexpr int BM = 128, BN = 128, BK = 64;

__device__ inline u16* kv_slot_bf16(const KvView& kv, int layer, int which, int head, int n_heads, int pos) {
    const size_t plane = ((size_t)layer * 2 + which) * n_heads + head;
    return (u16*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * 128;
}

template <int EPI>
__global__ __launch_bounds__(256) void gemm_bf16_nt(const GemmArgs a) {
    __shared__ __attribute__((aligned(16))) u16 As[2][BM * BK];
    __shared__ __attribute__((aligned(16))) u16 Bs[2][BN * BK];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int c = lane & 31, hh = lane >> 5;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;

    // Global -> register staging: thread handles 16-byte chunks tid + 256*j (j < 4) of each tile;
    // chunk index = row * 8 + chunk_in_row.
    const u16* ga[4];
    const u16* gb[4];
    int lds_off[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int idx = tid + 256 * j;
        const int r = idx >> 3, ch = idx & 7;
        const int am = min(m0 + r, a.M - 1);  // rows past M are loaded from the last row and never stored
        ga[j] = a.A + (size_t)am * a.K + ch * 8;
        gb[j] = a.W + (size_t)(n0 + r) * a.K + ch * 8;
        lds_off[j] = r * BK + ((ch ^ (r & 7)) << 3);
    }
    u32x4 ra[4], rb[4];
    auto load_tile = [&](int kt) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            ra[j] = *(const u32x4*)(ga[j] + (size_t)kt * BK);
            rb[j] = *(const u32x4*)(gb[j] + (size_t)kt * BK);
        }
    };
    auto store_tile = [&](int buf) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            *(u32x4*)(&As[buf][lds_off[j]]) = ra[j];
            *(u32x4*)(&Bs[buf][lds_off[j]]) = rb[j];
        }
    };

    f32x16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

    const int KT = a.K / BK;
    load_tile(0);
    store_tile(0);
    __syncthreads();
    for (int kt = 0; kt < KT; ++kt) {
        const int buf = kt & 1;
        if (kt + 1 < KT) load_tile(kt + 1);
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            bf16x8 fa[2], fb[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                const int r = wm * 64 + i * 32 + c;
                fa[i] = *(const bf16x8*)(&As[buf][r * BK + (((2 * ks + hh) ^ (r & 7)) << 3)]);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int r = wn * 64 + j * 32 + c;
                fb[j] = *(const bf16x8*)(&Bs[buf][r * BK + (((2 * ks + hh) ^ (r & 7)) << 3)]);
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = mfma32(fa[i], fb[j], acc[i][j]);
        }
        if (kt + 1 < KT) store_tile(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogues: column block j = 0 / 1 of this wave are packed columns wn*64 + {0..31} / {32..63}.
    const int ncol0 = n0 + wn * 64;  // first packed column of this wave
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int m = m0 + wm * 64 + i * 32 + acc_row(r, hh);
            if (m >= a.M) continue;
            const float v0 = acc[i][0][r], v1 = acc[i][1][r];
            if (EPI == EPI_RESID) {
                float* p = a.x32 + (size_t)m * a.N + ncol0 + c;
                const float y0 = p[0] + v0, y1 = p[32] + v1;
                p[0] = y0;
                p[32] = y1;
                if (a.final_out) {
                    u16* o = a.final_out + (size_t)m * a.N + ncol0 + c;
                    o[0] = f2bf(y0);
                    o[32] = f2bf(y1);
                }
            } else if (EPI == EPI_SWIGLU) {
                // block 0 = gate, block 1 = up of features (ncol0/64)*32 + c
                const float s = v0 / (1.0f + __expf(-v0)) * v1;
                a.act[(size_t)m * (a.N >> 1) + (ncol0 >> 6) * 32 + c] = f2bf(s);
            } else {  // EPI_QKV
                const int which = ncol0 / a.d_model;
                const int in_model = ncol0 - which * a.d_model;
                const int head = in_model >> 7;
                const int wtile = (in_model & 127) >> 6;  // which 64-column half of the head (packed order)
                if (which == 2) {
                    u16* vs = kv_slot_bf16(a.kv, a.layer, 1, head, a.n_heads, a.pos0 + m) + wtile * 64 + c;
                    vs[0] = f2bf(v0);
                    vs[32] = f2bf(v1);
                } else {
                    // packed column 64*wtile + 32*b + c  <->  rotary index 64*b + 32*wtile + c
                    const int i_lo = 32 * wtile + c;
                    const float2 cs = a.rope[(size_t)m * 64 + i_lo];
                    const float lo = v0 * cs.x - v1 * cs.y;
                    const float hi = v1 * cs.x + v0 * cs.y;
                    u16* dst = which == 0 ? a.q_out + (size_t)m * a.d_model + head * 128
                                          : kv_slot_bf16(a.kv, a.layer, 0, head, a.n_heads, a.pos0 + m);
                    dst[i_lo] = f2bf(lo);
                    dst[i_lo + 64] = f2bf(hi);
                }
            }
        }
    }
}

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

__device__ inline const u16* kv_row_bf16(const KvView& kv, size_t plane, int pos) {
    if (pos < kv.n_shared) return (const u16*)kv.parent + (plane * kv.parent_cap + (size_t)pos) * 128;
    return (const u16*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * 128;
}

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

template <int EPI>
void launch_gemm(const GemmArgs& a, hipStream_t s) {
    dim3 grid(a.N / BN, (a.M + BM - 1) / BM);
    hipLaunchKernelGGL(gemm_bf16_nt<EPI>, grid, dim3(256), 0, s, a);
}

}  // namespace

hipError_t bf16_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s) {
    const jup_stage_config_t& c = st.cfg;
    const size_t d = c.d_model, f = c.d_ffn;
    for (int l = 0; l < c.n_layers; ++l) {
        char* base = (char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const jup_layer_weights_t& w = layers[l];
        hipLaunchKernelGGL(pack_qkv, dim3(3 * c.d_model), dim3(256), 0, s, (u16*)(base + st.pl.wqkv), (const u16*)w.wq,
                           (const u16*)w.wk, (const u16*)w.wv, c.d_model);
        hipLaunchKernelGGL(pack_gate_up, dim3(2 * c.d_ffn), dim3(256), 0, s, (u16*)(base + st.pl.wgu),
                           (const u16*)w.w_gate, (const u16*)w.w_up, c.d_model);
        hipError_t e = hipMemcpyAsync(base + st.pl.wo, w.wo, d * d * 2, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(base + st.pl.wdown, w.w_down, d * f * 2, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(base + st.pl.g_attn, w.g_attn, d * 2, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(base + st.pl.g_mlp, w.g_mlp, d * 2, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

hipError_t bf16_forward(const jup_stage& st, const void* hidden_in, int n, int pos, const KvView& kv,
                        void* hidden_out, hipStream_t s) {
    const jup_stage_config_t& c = st.cfg;
    const int d = c.d_model, f = c.d_ffn, H = c.n_heads;
    char* ws = (char*)st.workspace;
    float* x32 = (float*)(ws + st.wl.x32);
    u16* xn = (u16*)(ws + st.wl.xn);
    u16* q = (u16*)(ws + st.wl.q);
    u16* o = (u16*)(ws + st.wl.o);
    u16* act = (u16*)(ws + st.wl.act);
    float2* rope = (float2*)(ws + st.wl.rope);
    const float scale_log2e = 1.4426950408889634f / sqrtf(128.0f);

    hipLaunchKernelGGL(rope_table, dim3((n * 64 + 255) / 256), dim3(256), 0, s, rope, n, 64, pos, c.rope_theta);
    if (c.n_layers == 0) return hipMemcpyAsync(hidden_out, hidden_in, (size_t)n * d * 2, hipMemcpyDeviceToDevice, s);

    for (int l = 0; l < c.n_layers; ++l) {
        const char* wb = (const char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const u16* g1 = (const u16*)(wb + st.pl.g_attn);
        const u16* g2 = (const u16*)(wb + st.pl.g_mlp);

        {
        TraceScope ts(st, JUP_K_RMSNORM, s);
        if (l == 0)
            hipLaunchKernelGGL(rmsnorm_bf16<true>, dim3(n), dim3(256), 0, s, hidden_in, x32, g1, xn, d, c.rms_eps);
        else
            hipLaunchKernelGGL(rmsnorm_bf16<false>, dim3(n), dim3(256), 0, s, (const void*)x32, x32, g1, xn, d,
                               c.rms_eps);
        }

        GemmArgs a{};
        a.A = xn; a.W = (const u16*)(wb + st.pl.wqkv); a.M = n; a.N = 3 * d; a.K = d;
        a.q_out = q; a.rope = rope; a.kv = kv; a.layer = l; a.n_heads = H; a.d_model = d; a.pos0 = pos;
        {
            TraceScope ts(st, JUP_K_GEMM_QKV, s);
            launch_gemm<EPI_QKV>(a, s);
        }

        {
            TraceScope ts(st, JUP_K_ATTENTION, s);
            if (n <= 32)
                hipLaunchKernelGGL(chunk_attention_bf16<1>, dim3((n + 31) / 32, H), dim3(256), 0, s, q, o, n, d, H, pos,
                                   kv, l, scale_log2e);
            else
                hipLaunchKernelGGL(chunk_attention_bf16<2>, dim3((n + 63) / 64, H), dim3(256), 0, s, q, o, n, d, H, pos,
                                   kv, l, scale_log2e);
        }

        GemmArgs b{};
        b.A = o; b.W = (const u16*)(wb + st.pl.wo); b.M = n; b.N = d; b.K = d; b.x32 = x32;
        {
            TraceScope ts(st, JUP_K_GEMM_O, s);
            launch_gemm<EPI_RESID>(b, s);
        }
        {
            TraceScope ts(st, JUP_K_RMSNORM, s);
            hipLaunchKernelGGL(rmsnorm_bf16<false>, dim3(n), dim3(256), 0, s, (const void*)x32, x32, g2, xn, d,
                               c.rms_eps);
        }

        GemmArgs g{};
        g.A = xn; g.W = (const u16*)(wb + st.pl.wgu); g.M = n; g.N = 2 * f; g.K = d; g.act = act;
        {
            TraceScope ts(st, JUP_K_GEMM_GATE_UP, s);
            launch_gemm<EPI_SWIGLU>(g, s);
        }

        GemmArgs dn{};
        dn.A = act; dn.W = (const u16*)(wb + st.pl.wdown); dn.M = n; dn.N = d; dn.K = f; dn.x32 = x32;
        dn.final_out = (l == c.n_layers - 1) ? (u16*)hidden_out : nullptr;
        {
            TraceScope ts(st, JUP_K_GEMM_DOWN, s);
            launch_gemm<EPI_RESID>(dn, s);
        }
    }
    return hipGetLastError();
}

}  // namespace jup
