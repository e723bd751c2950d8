// Projections of a stage whose matrices are stored as 4-bit codes (JUP_BF16_W4): C[M, N] = A[M, K] * W[N, K]^T with
// W[n][k] = scale[n][k / 128] * (code[n][k] - 8), for decode-sized chunks (Jupiter paper, Sec. V: a decoding step
// feeds a handful of tokens per sequence, so a projection is bound by streaming its weights; Sec. VI-A: the paper
// runs its models with INT4 weights).  The kernel streams the codes, a quarter of the bf16 bytes, straight from
// global memory into registers and expands them there:
//
//   * A wave owns 16 RG rows x 64 columns (RG = 1, 2 or 4 row groups: one expansion of the codes serves up to 64
//     rows) and a range of K; the eight waves of a workgroup split the workgroup's K range, add their sums through
//     LDS in a fixed order and run the epilogue.  No barrier inside the K loop and no LDS traffic for the operands:
//     every wave streams on its own.
//   * v_mfma_f32_16x16x32_bf16.  Operand layout (lane = 16 q + r): A: lane supplies A[m = r][k = 8 q + e], e < 8;
//     B: lane supplies B[k = 8 q + e][n = r]; D: lane holds D[m = 4 q + i][n = r] in register i < 4, so a lane's
//     four results share one column and take one scale.
//   * Codes are stored per (64-column tile, 128-K group, 16-column block) as 1 KB: lane (r, q) owns 16 bytes, dword
//     ks holding the eight codes of column r for k = 128 g + 32 ks + 8 q + e.  Inside a dword, nibble p < 4 is
//     element 2 p and nibble p + 4 is element 2 p + 1: ((w >> 4 j) & 0x000F000F) | 0x43004300 is then the bf16 pair
//     (128 + code[2 j], 128 + code[2 j + 1]) -- two instructions per two weights, exact (a bf16 mantissa holds
//     128..255 in steps of one).
//   * The offset of 136 = 128 + 8 leaves through the row sums of A: sum_k A[m][k] (128 + c) - 136 sum_k A[m][k].
//     The row sums of a group come from one more MFMA per K step against a register of ones, and a group's
//     result enters the fp32 accumulator as scale * (t - 136 * rowsum): 4 FMAs per lane, group and column block.
//     Products of a bf16 value and an integer below 256 are exact in fp32, the sums round as any fp32 sum does.
//   * A (16 rows of the tiled activation layout per row group) is read from L2 with 16-byte loads, up to 1 KB per
//     wave and K step; lanes whose row lies past the chunk fetch nothing.
#include "bf16_common.h"

namespace jup {
namespace {

constexpr int W4_GROUP = 128;   // input features per scale
constexpr int W4_TILE_N = 64;   // columns per workgroup
constexpr int W4_WAVES = 8;

enum { W4_PACK_PLAIN = 0, W4_PACK_QKV = 1, W4_PACK_GATE_UP = 2 };

// Packed column -> (source matrix 0..2, source row).  QKV: a 16-column block of a Q or K head holds the rotary
// indices 8u..8u+7 in its lanes 0..7 and their partners 64 + 8u.. in lanes 8..15 (u = block within the head);
// V keeps the same order.  Gate/up: even packed columns are gate rows, odd ones up rows.
__device__ inline void w4_source(int mode, int pc, int rows_per, int& which, int& row) {
    if (mode == W4_PACK_QKV) {
        which = pc / rows_per;
        const int in = pc - which * rows_per;
        const int head = in >> 7, u = (in & 127) >> 4, r = in & 15;
        row = head * 128 + (r < 8 ? 8 * u + r : 64 + 8 * u + (r - 8));
    } else if (mode == W4_PACK_GATE_UP) {
        which = pc & 1;
        row = pc >> 1;
    } else {
        which = 0;
        row = pc;
    }
}

// One workgroup per (column tile, K group): 4 column blocks x 64 lanes.
__global__ __launch_bounds__(256) void pack_w4(unsigned char* __restrict__ dst, float* __restrict__ dst_scale,
                                               const unsigned char* __restrict__ c0, const unsigned char* __restrict__ c1,
                                               const unsigned char* __restrict__ c2, const float* __restrict__ s0,
                                               const float* __restrict__ s1, const float* __restrict__ s2, int K,
                                               int rows_per, int mode) {
    const int G = K / W4_GROUP;
    const int tile = blockIdx.x / G, g = blockIdx.x - tile * G;
    const int cg = threadIdx.x >> 6, lane = threadIdx.x & 63, r = lane & 15, q = lane >> 4;
    int which, row;
    w4_source(mode, tile * W4_TILE_N + cg * 16 + r, rows_per, which, row);
    const unsigned char* src = (which == 0 ? c0 : which == 1 ? c1 : c2) + (size_t)row * (K / 2);
    u32x4 out;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
        const int k = g * W4_GROUP + 32 * ks + 8 * q;  // eight codes = four bytes, low nibble first
        const unsigned w = *(const unsigned*)(src + k / 2);
        unsigned v = 0;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int e = p < 4 ? 2 * p : 2 * (p - 4) + 1;
            v |= ((w >> (4 * e)) & 0xFu) << (4 * p);
        }
        out[ks] = v;
    }
    *(u32x4*)(dst + (((size_t)tile * G + g) * 4 + cg) * 1024 + lane * 16) = out;
    if (q == 0) {
        const float* ss = which == 0 ? s0 : which == 1 ? s1 : s2;
        dst_scale[(((size_t)tile * G + g) * 16 + r) * 4 + cg] = ss[(size_t)row * G + g];
    }
}

__device__ inline bf16x8 w4_expand(unsigned w) {
    u32x4 v;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = ((w >> (4 * j)) & 0x000F000Fu) | 0x43004300u;
    return __builtin_bit_cast(bf16x8, v);
}

// What a wave fetches for one K group: the codes of its four column blocks and their scales, and four A fragments
// per row group.
struct W4Codes {
    u32x4 w[4];
    float4 sc;
};
template <int RG>
struct W4Rows {
    bf16x8 a[RG][4];
};

template <int EPI, int RG, int WAVES, bool STREAM_ONCE>
__global__ __launch_bounds__(64 * WAVES) void gemm_w4(const GemmArgs a) {
    __shared__ float red[WAVES][16][W4_TILE_N];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int r = lane & 15, q = lane >> 4;
    const int tile = blockIdx.x % a.n_tiles, split = blockIdx.x / a.n_tiles, rg0 = blockIdx.y * RG;
    const int G = a.K / W4_GROUP;
    // K groups of this workgroup, then of this wave (floor division: the shares differ by at most one group)
    const int ws0 = (int)((long)split * G / a.splits), ws1 = (int)((long)(split + 1) * G / a.splits);
    const int cnt = ws1 - ws0;
    const int g0 = ws0 + wave * cnt / WAVES, g1 = ws0 + (wave + 1) * cnt / WAVES;

    const int k_stages = a.K / 32;
    // Lanes whose row lies past the chunk fetch nothing (a 5-token chunk reads 5 of the 16 rows of its fragment) and
    // multiply zeros; their results are dropped.
    int a_row[RG];
    bool a_live[RG];
#pragma unroll
    for (int j = 0; j < RG; ++j) {
        a_row[j] = 16 * (rg0 + j) + r;
        a_live[j] = a_row[j] < a.M;
    }
    const unsigned char* wbase = (const unsigned char*)a.W + (size_t)tile * G * 4096 + lane * 16;
    const float* sbase = a.w_scale + ((size_t)tile * G * 16 + r) * 4;
    // STREAM_ONCE (one pass over the codes, up to 64 rows): every code is read exactly once, with the non-temporal hint,
    // so that the stream does not push the KV cache and the activations out of the caches (measured at 5 rows per call:
    // the attention launch behind the projections 15.0 -> 12.2 us, a step of 8 branches 3.96 -> 3.62 ms).  Longer chunks
    // take several passes, which find the codes in L2, and inside an overlapped call the other chunks' launches find them
    // in the caches (as for the bf16 kernels: not measured separately for the codes).
    auto fetch_codes = [&](W4Codes& d, int g) {
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
            const u32x4* src = (const u32x4*)(wbase + ((size_t)g * 4 + cg) * 1024);
            if constexpr (STREAM_ONCE) d.w[cg] = __builtin_nontemporal_load(src);
            else d.w[cg] = *src;
        }
        d.sc = *(const float4*)(sbase + (size_t)g * 64);
    };
    const u32x4 zero_bits = {0u, 0u, 0u, 0u};
    const bf16x8 zero_frag = __builtin_bit_cast(bf16x8, zero_bits);
    auto fetch_rows = [&](W4Rows<RG>& d, int g) {
#pragma unroll
        for (int j = 0; j < RG; ++j)
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) {
                d.a[j][ks] = zero_frag;
                if (a_live[j]) d.a[j][ks] = *(const bf16x8*)(a.A + tiled_offset(a_row[j], (4 * g + ks) * 4 + q, k_stages));
            }
    };

    f32x4 acc[RG][4];
#pragma unroll
    for (int j = 0; j < RG; ++j)
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) acc[j][cg] = f32x4{0.f, 0.f, 0.f, 0.f};
    const u32x4 ones_bits = {0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u};
    const bf16x8 ones = __builtin_bit_cast(bf16x8, ones_bits);

    auto compute = [&](const W4Codes& c, const W4Rows<RG>& d) {
        f32x4 rs[RG];
#pragma unroll
        for (int j = 0; j < RG; ++j) {
            rs[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) rs[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(d.a[j][ks], ones, rs[j], 0, 0, 0);
        }
        const float sc[4] = {c.sc.x, c.sc.y, c.sc.z, c.sc.w};
#pragma unroll
        for (int cg = 0; cg < 4; ++cg) {
            bf16x8 b[4];  // one expansion of the codes serves every row group
#pragma unroll
            for (int ks = 0; ks < 4; ++ks) b[ks] = w4_expand(c.w[cg][ks]);
#pragma unroll
            for (int j = 0; j < RG; ++j) {
                f32x4 t = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) t = __builtin_amdgcn_mfma_f32_16x16x32_bf16(d.a[j][ks], b[ks], t, 0, 0, 0);
#pragma unroll
                for (int i = 0; i < 4; ++i) acc[j][cg][i] += sc[cg] * (t[i] - 136.0f * rs[j][i]);
            }
        }
    };

    // Two groups of codes (from HBM) in flight per wave: the next one is fetched before the current one is used.
    // (Four in flight, a wave's whole share of K on the 7B shapes, measured no faster where the grid still fits one
    // round of workgroups -- QKV 13.3 vs 13.0 us, down 11.6 vs 11.8 us at 5 rows -- and slower for gate/up, 20.5 vs
    // 18.3 us: 216 registers per lane leave one workgroup per CU and its 344 workgroups then take two rounds.)  The
    // rows of A (from L2) travel with them while the registers allow it (up to 32 rows); with 64 rows they are
    // fetched when their group's turn comes, behind the prefetch of the next codes.
    constexpr bool ROWS_AHEAD = RG <= 2;
    W4Codes cur, nxt;
    W4Rows<RG> rows, rows_nxt;
    if (g0 < g1) {
        fetch_codes(cur, g0);
        if (ROWS_AHEAD) fetch_rows(rows, g0);
    }
    for (int g = g0; g < g1; ++g) {
        if (g + 1 < g1) {
            fetch_codes(nxt, g + 1);
            if (ROWS_AHEAD) fetch_rows(rows_nxt, g + 1);
        }
        if (!ROWS_AHEAD) fetch_rows(rows, g);
        compute(cur, rows);
        cur = nxt;
        if (ROWS_AHEAD) rows = rows_nxt;
    }

    // ---- per row group: sum over the waves (fixed order), then the epilogue, one output row per wave and pass ----
    static_assert(16 % WAVES == 0, "the epilogue deals the 16 rows of a row group to the waves");
    const int n = lane;                    // 64 lanes = the 64 columns of the tile
    const int col = tile * W4_TILE_N + n;  // packed column
#pragma unroll
    for (int j = 0; j < RG; ++j) {
        if (j > 0) __syncthreads();  // the sums of the row group before have been read
#pragma unroll
        for (int cg = 0; cg < 4; ++cg)
#pragma unroll
            for (int i = 0; i < 4; ++i) red[wave][4 * q + i][16 * cg + r] = acc[j][cg][i];
        __syncthreads();
#pragma unroll
        for (int pass = 0; pass < 16 / WAVES; ++pass) {
            const int m = wave + WAVES * pass;
            float v = 0.f;
#pragma unroll
            for (int w = 0; w < WAVES; ++w) v += red[w][m][n];
            const int row = 16 * (rg0 + j) + m;
            if (EPI == EPI_PARTIAL) {
                if (row < a.M) a.partial[((size_t)split * a.M + row) * a.N + col] = v;
            } else if (EPI == EPI_SWIGLU) {
                const float up = __shfl_xor(v, 1, 64);  // the odd neighbour holds the up projection of the same output
                if (!(n & 1) && row < a.M) {
                    const int oc = col >> 1;  // output feature
                    a.act[tiled_offset(row, oc >> 3, (a.N >> 1) >> 5) + (oc & 7)] =
                        f2bf(v * __builtin_amdgcn_rcpf(1.0f + __expf(-v)) * up);
                }
            } else {  // EPI_QKV
                const float other = __shfl_xor(v, 8, 64);  // rotary partner (lanes 0..7 <-> 8..15 of a 16-column block)
                const int which = col / a.d_model;
                const int in = col - which * a.d_model;
                const int head = in >> 7, u = (in & 127) >> 4, rr = in & 15;
                const int feature = rr < 8 ? 8 * u + rr : 64 + 8 * u + (rr - 8);
                float out = v;
                if (which != 2 && row < a.M) {
                    const float2 cs = a.rope[(size_t)row * 64 + (feature & 63)];
                    out = rr < 8 ? v * cs.x - other * cs.y : v * cs.x + other * cs.y;
                }
                if (row < a.M) {
                    u16* dst;
                    if (which == 0) {
                        dst = a.q_out + (size_t)row * a.d_model + head * 128;
                    } else if (!a.branches) {
                        dst = kv_slot_bf16(a.kv, a.layer, which - 1, head, a.n_heads, a.pos0 + row);
                    } else {
                        const int b = row / a.branches->n_tok, t = row - b * a.branches->n_tok;
                        dst = kv_slot_bf16(a.branches->kv[b], a.layer, which - 1, head, a.n_heads,
                                           a.branches->pos0[b] + t);
                    }
                    dst[feature] = f2bf(out);
                }
            }
        }
    }
}

template <int EPI, int RG>
hipError_t launch_rg(GemmArgs a, hipStream_t s) {
    // Eight waves per workgroup split its K range, whatever the row count: the order in which the K shares are summed
    // is then the same for a branch submitted alone and batched with others, and the two give the same bits.  Measured
    // on the 7B shapes at 64 rows per pass (246 registers per lane, so eight waves per CU either way): two workgroups of
    // four waves per CU run gate/up 4-5 % faster (its 344 workgroups then fit one round instead of two) and QKV 40 %
    // slower than one of eight; at 5 rows 4, 8 and 16 waves measured within 5 % of each other.
    constexpr int WAVES = W4_WAVES;
    a.n_tiles = a.N / W4_TILE_N;
    a.m_tiles = (a.M + 16 * RG - 1) / (16 * RG);
    const dim3 grid(a.n_tiles * a.splits, a.m_tiles);
    if (a.m_tiles == 1 && !a.shared_gpu) hipLaunchKernelGGL((gemm_w4<EPI, RG, WAVES, true>), grid, dim3(64 * WAVES), 0, s, a);
    else hipLaunchKernelGGL((gemm_w4<EPI, RG, WAVES, false>), grid, dim3(64 * WAVES), 0, s, a);
    return hipGetLastError();
}
// Rows per pass over the codes: 16, 32 or 64 (a longer chunk takes several passes of 64).
template <int EPI>
hipError_t launch_one(GemmArgs a, hipStream_t s) {
    if (a.M <= 16) return launch_rg<EPI, 1>(a, s);
    if (a.M <= 32) return launch_rg<EPI, 2>(a, s);
    return launch_rg<EPI, 4>(a, s);
}

}  // namespace

// Splits of K for the projections back to d_model (their N / 64 column tiles alone do not occupy the chip): as many
// as keep the grid within about one workgroup per CU, at most 8 (the reduce + norm pass sums up to 8 partial
// buffers), and no more than there are K groups.
int w4_plan_splits(int N, int K) {
    const int tiles = N / W4_TILE_N, G = K / W4_GROUP;
    int splits = 1;
    while (splits < 8 && tiles * splits * 2 <= 256 && splits * 2 <= G) splits *= 2;
    return splits;
}

hipError_t launch_gemm_w4(int epi, GemmArgs a, hipStream_t s) {
    if (a.M <= 0 || a.N % W4_TILE_N || a.K % W4_GROUP) return hipErrorInvalidValue;
    if (epi == EPI_PARTIAL) {
        a.splits = w4_plan_splits(a.N, a.K);
        return launch_one<EPI_PARTIAL>(a, s);
    }
    a.splits = 1;
    return epi == EPI_QKV ? launch_one<EPI_QKV>(a, s) : launch_one<EPI_SWIGLU>(a, s);
}

void launch_pack_w4_qkv(unsigned char* dst, float* dst_scale, const void* cq, const void* ck, const void* cv,
                        const float* sq, const float* sk, const float* sv, int d, hipStream_t s) {
    hipLaunchKernelGGL(pack_w4, dim3(3 * d / W4_TILE_N * (d / W4_GROUP)), dim3(256), 0, s, dst, dst_scale,
                       (const unsigned char*)cq, (const unsigned char*)ck, (const unsigned char*)cv, sq, sk, sv, d, d,
                       (int)W4_PACK_QKV);
}
void launch_pack_w4_gate_up(unsigned char* dst, float* dst_scale, const void* cg, const void* cu, const float* sg,
                            const float* su, int d, int f, hipStream_t s) {
    hipLaunchKernelGGL(pack_w4, dim3(2 * f / W4_TILE_N * (d / W4_GROUP)), dim3(256), 0, s, dst, dst_scale,
                       (const unsigned char*)cg, (const unsigned char*)cu, (const unsigned char*)nullptr, sg, su,
                       (const float*)nullptr, d, 0, (int)W4_PACK_GATE_UP);
}
void launch_pack_w4_plain(unsigned char* dst, float* dst_scale, const void* c, const float* sc, int n_rows, int k,
                          hipStream_t s) {
    hipLaunchKernelGGL(pack_w4, dim3(n_rows / W4_TILE_N * (k / W4_GROUP)), dim3(256), 0, s, dst, dst_scale,
                       (const unsigned char*)c, (const unsigned char*)nullptr, (const unsigned char*)nullptr, sc,
                       (const float*)nullptr, (const float*)nullptr, k, 0, (int)W4_PACK_PLAIN);
}

}  // namespace jup
