// Small memory-bound kernels of the bf16 path: weight packing (once, at stage creation), the rotary
// table of a chunk, and the fused "sum the K-split partials + residual + RMSNorm" pass.
#include "bf16_common.h"

namespace jup {
namespace {

// Row order inside the packed weights.  The QKV and gate/up projections compute the transposed product, after which
// lane (c, hh) of a wave holds, for a 32-row block of the weights, the rows 8*(i/4) + 4*hh + (i%4) in register i < 16
// and one token (c).  The rows of a block are ordered so that those 16 registers are what ONE lane needs:
//   Q and K heads: block j of a head = rotary indices 16 j .. 16 j + 15 and their partners 64 further on (Llama
//     half-split pairing); registers 0..7 of half hh = indices 16 j + 8 hh .. + 7, registers 8..15 = their partners.
//   V heads: block j = features 32 j .. 32 j + 31; registers 0..15 of half hh = features 32 j + 16 hh .. + 15.
//   gate/up: block B = output features 16 B .. 16 B + 15; registers 0..7 of half hh = gate rows of the features
//     16 B + 8 hh .. + 7, registers 8..15 = their up rows.
// Register i of half hh is packed row rho = 8*(i/4) + 4*hh + (i%4), i.e. i = 4*(rho>>3) + (rho&3), hh = (rho>>2)&1.
__device__ inline int packed_reg(int rho) { return 4 * (rho >> 3) + (rho & 3); }
__device__ inline int packed_half(int rho) { return (rho >> 2) & 1; }
// packed row p (0..127) of a Q or K head -> original row of the head
__device__ inline int rope_packed_to_orig(int p) {
    const int j = p >> 5, rho = p & 31, i = packed_reg(rho);
    return 16 * j + 8 * packed_half(rho) + (i & 7) + 64 * (i >> 3);
}
// packed row p (0..127) of a V head -> original row of the head
__device__ inline int v_packed_to_orig(int p) {
    const int j = p >> 5, rho = p & 31;
    return 32 * j + 16 * packed_half(rho) + packed_reg(rho);
}

enum { PACK_PLAIN = 0, PACK_QKV = 1, PACK_GATE_UP = 2 };

// One block per packed row n; copies that row's K/8 chunks into the tiled layout.
//   PACK_QKV:     rows [0,d) Q heads, [d,2d) K heads, [2d,3d) V heads (s0, s1, s2 = wq, wk, wv; rows_per = d)
//   PACK_GATE_UP: 32 packed rows per 16 output features, gate and up rows in the order described above (s0, s1 =
//                 w_gate, w_up)
//   PACK_PLAIN:   row n of s0
// W4: the sources are 4-bit codes ([rows, K/2] bytes, low nibble = even input feature) with fp32 scales
// ([rows, K/128]); the packed row holds bf16(scale * (code - 8)), the value the 4-bit kernels multiply by.
template <bool W4>
__global__ void pack_tiled(u16* __restrict__ dst, const void* __restrict__ s0, const void* __restrict__ s1,
                           const void* __restrict__ s2, const float* __restrict__ sc0, const float* __restrict__ sc1,
                           const float* __restrict__ sc2, int K, int rows_per, int mode) {
    const int n = blockIdx.x;
    int which = 0, src_row = n;
    if (mode == PACK_QKV) {
        which = n / rows_per;
        const int rr = n % rows_per;
        const int head = rr >> 7, in_head = rr & 127;
        src_row = head * 128 + (which == 2 ? v_packed_to_orig(in_head) : rope_packed_to_orig(in_head));
    } else if (mode == PACK_GATE_UP) {
        const int rho = n & 31, i = packed_reg(rho);
        which = i >> 3;
        src_row = 16 * (n >> 5) + 8 * packed_half(rho) + (i & 7);
    }
    const void* base = which == 0 ? s0 : which == 1 ? s1 : s2;
    const int k_stages = K / 32;
    if constexpr (W4) {
        const unsigned char* codes = (const unsigned char*)base + (size_t)src_row * (K / 2);
        const float* scales = (which == 0 ? sc0 : which == 1 ? sc1 : sc2) + (size_t)src_row * (K / 128);
        for (int ck = threadIdx.x; ck < K / 8; ck += blockDim.x) {
            const unsigned w = *(const unsigned*)(codes + ck * 4);  // eight codes, input features 8 ck .. 8 ck + 7
            const float sc = scales[ck >> 4];
            u32x4 out;
#pragma unroll
            for (int j = 0; j < 4; ++j)
                out[j] = pack_bf16x2(sc * (float)((int)((w >> (8 * j)) & 0xFu) - 8),
                                     sc * (float)((int)((w >> (8 * j + 4)) & 0xFu) - 8));
            *(u32x4*)(dst + tiled_offset(n, ck, k_stages)) = out;
        }
    } else {
        const u16* src = (const u16*)base + (size_t)src_row * K;
        for (int ck = threadIdx.x; ck < K / 8; ck += blockDim.x)
            *(u32x4*)(dst + tiled_offset(n, ck, k_stages)) = *(const u32x4*)(src + ck * 8);
    }
}

// The first kernel of a call also clears the arrival counters its later kernels count in (a fill by a kernel, not a
// memset: the call may be captured in a graph).
__device__ inline void clear_counters(int* zero, int n_zero) {
    for (int i = blockIdx.x * blockDim.x + threadIdx.x; i < n_zero; i += gridDim.x * blockDim.x) zero[i] = 0;
}

// tab[t][i] = (cos, sin)((pos0 + t) * theta^(-2i/128)); angles in fp64 so that large positions stay exact.
__global__ void rope_table(float2* __restrict__ tab, int n, int pos0, float theta, int* __restrict__ zero, int n_zero) {
    clear_counters(zero, n_zero);
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * 64) return;
    const int i = gid & 63, t = gid >> 6;
    const double ang = (double)(pos0 + t) * pow((double)theta, -(double)i / 64.0);
    tab[gid] = make_float2((float)cos(ang), (float)sin(ang));
}

// Token-tree call: token t sits tree->depth[t] positions behind the cached sequence.
__global__ void rope_table_tree(float2* __restrict__ tab, int n, int pos0, const TreeTable* __restrict__ tree,
                                float theta, int* __restrict__ zero, int n_zero) {
    clear_counters(zero, n_zero);
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n * 64) return;
    const int i = gid & 63, t = gid >> 6;
    const double ang = (double)(pos0 + tree->depth[t]) * pow((double)theta, -(double)i / 64.0);
    tab[gid] = make_float2((float)cos(ang), (float)sin(ang));
}

// Batched-branch call: row r is token r % n_tok of branch r / n_tok.
__global__ void rope_table_branches(float2* __restrict__ tab, int n_rows, const BranchTable* __restrict__ bt,
                                    float theta, int* __restrict__ zero, int n_zero) {
    clear_counters(zero, n_zero);
    const int gid = blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= n_rows * 64) return;
    const int i = gid & 63, r = gid >> 6;
    const int b = r / bt->n_tok, t = r - b * bt->n_tok;
    const double ang = (double)(bt->pos0[b] + t) * pow((double)theta, -(double)i / 64.0);
    tab[gid] = make_float2((float)cos(ang), (float)sin(ang));
}

// The table of a batched-branch call travels as a kernel argument and is parked in the workspace, where the
// kernels of the call find it (no host-to-device copy on the hot path).
__global__ void write_branch_table(const BranchTable t, BranchTable* __restrict__ dst) {
    if (threadIdx.x == 0) *dst = t;
}

// One block per row, IT float4 per thread (the row stays in registers between the two passes).  A row has
// few bytes and there are few rows, so the block is wide (d/8 threads when that is a whole number of waves):
// every load of a thread is independent and enough of them must be in flight per CU to cover HBM latency.
//   v    = (hidden_in ? bf16 row of hidden_in : x32 row) + sum over splits of the partial rows
//   x32 <- v                              (when anything was added or the row came from hidden_in)
//   xn  <- bf16(v * rsqrt(mean v^2 + eps) * g)   (when g != NULL)
//   out <- bf16(v)                        (when out != NULL)
template <int IT>
__global__ __launch_bounds__(1024) void reduce_norm(float* __restrict__ x32, const u16* __restrict__ hidden_in,
                                                    const float* __restrict__ partial, int splits, size_t split_stride,
                                                    const u16* __restrict__ g, u16* __restrict__ xn,
                                                    u16* __restrict__ out, int d, float eps) {
    __shared__ float part[16];
    const size_t row = blockIdx.x;
    const int nvec = d >> 2;  // float4 per row
    const int nthr = blockDim.x;
    float4 v[IT];
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int idx = threadIdx.x + it * nthr;
        if (idx < nvec) {
            float4 x;
            if (hidden_in) {
                const u32x2 h = *(const u32x2*)(hidden_in + row * d + idx * 4);
                x = make_float4(__uint_as_float(h[0] << 16), __uint_as_float(h[0] & 0xffff0000u),
                                __uint_as_float(h[1] << 16), __uint_as_float(h[1] & 0xffff0000u));
            } else {
                x = *(const float4*)(x32 + row * d + idx * 4);
            }
            float4 p[8];  // all loads first (at most 8 splits), then the sum in split order
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s < splits) p[s] = *(const float4*)(partial + s * split_stride + row * d + idx * 4);
#pragma unroll
            for (int s = 0; s < 8; ++s)
                if (s < splits) { x.x += p[s].x; x.y += p[s].y; x.z += p[s].z; x.w += p[s].w; }
            if (hidden_in || splits > 0) *(float4*)(x32 + row * d + idx * 4) = x;
            if (out) {
                u32x2 o;
                o[0] = pack_bf16x2(x.x, x.y);
                o[1] = pack_bf16x2(x.z, x.w);
                *(u32x2*)(out + row * d + idx * 4) = o;
            }
            v[it] = x;
            ss += x.x * x.x + x.y * x.y + x.z * x.z + x.w * x.w;
        }
    }
    if (!g) return;
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    float tot = 0.f;
    for (int w = 0; w < (nthr >> 6); ++w) tot += part[w];  // same order in every thread
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
#pragma unroll
    for (int it = 0; it < IT; ++it) {
        const int idx = threadIdx.x + it * nthr;
        if (idx < nvec) {
            const u32x2 gg = *(const u32x2*)(g + idx * 4);
            u32x2 o;
            o[0] = pack_bf16x2(v[it].x * inv * __uint_as_float(gg[0] << 16),
                               v[it].y * inv * __uint_as_float(gg[0] & 0xffff0000u));
            o[1] = pack_bf16x2(v[it].z * inv * __uint_as_float(gg[1] << 16),
                               v[it].w * inv * __uint_as_float(gg[1] & 0xffff0000u));
            *(u32x2*)(xn + tiled_offset((int)row, idx >> 1, d >> 5) + (idx & 1) * 4) = o;
        }
    }
}

}  // namespace

void launch_pack_qkv(u16* dst, const u16* wq, const u16* wk, const u16* wv, int d, hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<false>, dim3(3 * d), dim3(256), 0, s, dst, (const void*)wq, (const void*)wk,
                       (const void*)wv, (const float*)nullptr, (const float*)nullptr, (const float*)nullptr, d, d,
                       (int)PACK_QKV);
}
void launch_pack_gate_up(u16* dst, const u16* wg, const u16* wu, int d, int f, hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<false>, dim3(2 * f), dim3(256), 0, s, dst, (const void*)wg, (const void*)wu,
                       (const void*)nullptr, (const float*)nullptr, (const float*)nullptr, (const float*)nullptr, d, 0,
                       (int)PACK_GATE_UP);
}
void launch_pack_plain(u16* dst, const u16* w, int n_rows, int k, hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<false>, dim3(n_rows), dim3(256), 0, s, dst, (const void*)w, (const void*)nullptr,
                       (const void*)nullptr, (const float*)nullptr, (const float*)nullptr, (const float*)nullptr, k, 0,
                       (int)PACK_PLAIN);
}
// The same three layouts filled with the bf16 values of 4-bit matrices (codes + scales).
void launch_expand_qkv(u16* dst, const void* cq, const void* ck, const void* cv, const float* sq, const float* sk,
                       const float* sv, int d, hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<true>, dim3(3 * d), dim3(256), 0, s, dst, cq, ck, cv, sq, sk, sv, d, d, (int)PACK_QKV);
}
void launch_expand_gate_up(u16* dst, const void* cg, const void* cu, const float* sg, const float* su, int d, int f,
                           hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<true>, dim3(2 * f), dim3(256), 0, s, dst, cg, cu, (const void*)nullptr, sg, su,
                       (const float*)nullptr, d, 0, (int)PACK_GATE_UP);
}
void launch_expand_plain(u16* dst, const void* c, const float* sc, int n_rows, int k, hipStream_t s) {
    hipLaunchKernelGGL(pack_tiled<true>, dim3(n_rows), dim3(256), 0, s, dst, c, (const void*)nullptr,
                       (const void*)nullptr, sc, (const float*)nullptr, (const float*)nullptr, k, 0, (int)PACK_PLAIN);
}
void launch_rope_table(float2* tab, int n, int pos0, float theta, int* zero, int n_zero, hipStream_t s) {
    hipLaunchKernelGGL(rope_table, dim3((n * 64 + 255) / 256), dim3(256), 0, s, tab, n, pos0, theta, zero, n_zero);
}
void launch_rope_table_tree(float2* tab, int n, int pos0, const TreeTable* tree, float theta, int* zero, int n_zero,
                            hipStream_t s) {
    hipLaunchKernelGGL(rope_table_tree, dim3((n * 64 + 255) / 256), dim3(256), 0, s, tab, n, pos0, tree, theta, zero,
                       n_zero);
}
void launch_rope_table_branches(float2* tab, int n_rows, const BranchTable* branches, float theta, int* zero, int n_zero,
                                hipStream_t s) {
    hipLaunchKernelGGL(rope_table_branches, dim3((n_rows * 64 + 255) / 256), dim3(256), 0, s, tab, n_rows, branches,
                       theta, zero, n_zero);
}
void launch_write_branch_table(const BranchTable& host_table, BranchTable* dst, hipStream_t s) {
    hipLaunchKernelGGL(write_branch_table, dim3(1), dim3(64), 0, s, host_table, dst);
}
void launch_reduce_norm(float* x32, const u16* hidden_in, const float* partial, int splits, size_t split_stride,
                        const u16* g, u16* xn, u16* out, int n, int d, float eps, hipStream_t s) {
    if (d % 512 == 0 && d / 8 <= 1024)
        hipLaunchKernelGGL(reduce_norm<2>, dim3(n), dim3(d / 8), 0, s, x32, hidden_in, partial, splits, split_stride, g,
                           xn, out, d, eps);
    else
        hipLaunchKernelGGL(reduce_norm<8>, dim3(n), dim3(256), 0, s, x32, hidden_in, partial, splits, split_stride, g,
                           xn, out, d, eps);
}

}  // namespace jup
