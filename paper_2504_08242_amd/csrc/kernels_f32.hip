// Check-mode (JUP_F32) path: the stage forward with fp32 storage and fp32 arithmetic on plain
// vector-ALU kernels.  It exists to pin indexing and semantics (rotary pairs, head split, cache
// strides, mask boundary) against the CPU oracle at tight tolerances; speed is not a goal.
// Steps follow the decoder layer of Sec. II-A of the Jupiter paper in its Llama-2 form, applied to
// one sub-sequence with the cached prefix (Sec. IV-A.2).
#include "jup_internal.h"

namespace jup {
namespace {

constexpr int kWave = 64;

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
    return v;
}

// y[t][j] = x[t][j] * g[j] / sqrt(mean_j x^2 + eps); one 256-thread block per row.
__global__ __launch_bounds__(256) void f32_rmsnorm(const float* __restrict__ x, const float* __restrict__ g,
                                                   float* __restrict__ y, int d, float eps) {
    __shared__ float part[4];
    const float* xr = x + (size_t)blockIdx.x * d;
    float ss = 0.f;
    for (int j = threadIdx.x; j < d; j += 256) ss += xr[j] * xr[j];
    ss = wave_sum(ss);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = ss;
    __syncthreads();
    const float tot = part[0] + part[1] + part[2] + part[3];
    const float inv = 1.0f / sqrtf(tot / (float)d + eps);
    float* yr = y + (size_t)blockIdx.x * d;
    for (int j = threadIdx.x; j < d; j += 256) yr[j] = xr[j] * inv * g[j];
}

// C[m][n] = (R ? R[m][n] : 0) + sum_k A[m][k] * W[n][k].   A: [M, K] (lda), W: [N, K], C/R: [M, N] (ldc).
// R may be C itself: every element is read and then written by the one thread that owns it.
// 64x64 tile, 256 threads, 4x4 outputs per thread, K stepped by 16 through LDS.
__global__ __launch_bounds__(256) void f32_gemm_nt(const float* __restrict__ A, int lda, const float* __restrict__ W,
                                                   float* C, const float* R, int ldc, int M, int N, int K) {
    __shared__ float As[16][64 + 4];
    __shared__ float Ws[16][64 + 4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
    float acc[4][4] = {};
    for (int k0 = 0; k0 < K; k0 += 16) {
        for (int i = threadIdx.x; i < 64 * 16; i += 256) {
            const int r = i >> 4, kk = i & 15;
            const int m = m0 + r, n = n0 + r, k = k0 + kk;
            As[kk][r] = (m < M && k < K) ? A[(size_t)m * lda + k] : 0.f;
            Ws[kk][r] = (n < N && k < K) ? W[(size_t)n * K + k] : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int kk = 0; kk < 16; ++kk) {
            float a[4], w[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = As[kk][ty * 4 + i];
#pragma unroll
            for (int j = 0; j < 4; ++j) w[j] = Ws[kk][tx * 4 + j];
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], w[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int m = m0 + ty * 4 + i;
        if (m >= M) continue;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int n = n0 + tx * 4 + j;
            if (n >= N) continue;
            const size_t idx = (size_t)m * ldc + n;
            C[idx] = (R ? R[idx] : 0.f) + acc[i][j];
        }
    }
}

__device__ inline float* kv_slot(const KvView& kv, int layer, int which, int head, int n_heads, int dh, int pos) {
    // Writable slot of an absolute position (always >= n_shared: the host checked).
    const size_t plane = ((size_t)layer * 2 + which) * n_heads + head;
    return (float*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * dh;
}

__device__ inline const float* kv_row(const KvView& kv, int layer, int which, int head, int n_heads, int dh, int pos) {
    const size_t plane = ((size_t)layer * 2 + which) * n_heads + head;
    if (pos < kv.n_shared) return (const float*)kv.parent + (plane * kv.parent_cap + (size_t)pos) * dh;
    return (const float*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * dh;
}

// Rotates q and k of token t / head h in the fused [n, 3d] buffer at absolute position pos0 + t (token
// tree: pos0 + depth of t) and stores k (rotated) and v into cache entry pos0 + t.  One thread per
// (t, h, i < dh/2).
__global__ void f32_rope_append(float* __restrict__ qkv, int n, int d, int n_heads, int dh, int pos0, float theta,
                                KvView kv, int layer, const TreeTable* __restrict__ tree) {
    const int half = dh / 2;
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (long long)n * n_heads * half) return;
    const int i = (int)(gid % half);
    const int h = (int)((gid / half) % n_heads);
    const int t = (int)(gid / ((long long)half * n_heads));
    const int pos = pos0 + (tree ? tree->depth[t] : t), slot = pos0 + t;
    const double ang = (double)pos * pow((double)theta, -2.0 * (double)i / (double)dh);
    const float c = (float)cos(ang), s = (float)sin(ang);
    float* q = qkv + (size_t)t * 3 * d + (size_t)h * dh;
    float* k = q + d;
    const float* v = q + 2 * d;
    const float qa = q[i], qb = q[i + half];
    q[i] = qa * c - qb * s;
    q[i + half] = qb * c + qa * s;
    const float ka = k[i], kb = k[i + half];
    float* kc = kv_slot(kv, layer, 0, h, n_heads, dh, slot);
    float* vc = kv_slot(kv, layer, 1, h, n_heads, dh, slot);
    kc[i] = ka * c - kb * s;
    kc[i + half] = kb * c + ka * s;
    vc[i] = v[i];
    vc[i + half] = v[i + half];
}

// One wave per (query t, head h): softmax over the cached keys 0..pos0+t (running max / running sum),
// weighted sum of the cached values.  Lanes split head_dim (up to 256).  Token tree: of the chunk's own
// entries pos0.. only those of the query's ancestors and its own are visible.
__global__ __launch_bounds__(kWave) void f32_attention(const float* __restrict__ qkv, float* __restrict__ o, int d,
                                                       int n_heads, int dh, int pos0, KvView kv, int layer,
                                                       const TreeTable* __restrict__ tree) {
    const int t = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const float* q = qkv + (size_t)t * 3 * d + (size_t)h * dh;
    float qr[4], acc[4] = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int r = 0; r < 4; ++r) qr[r] = (lane + r * kWave < dh) ? q[lane + r * kWave] : 0.f;
    const float scale = 1.0f / sqrtf((float)dh);
    float m = -INFINITY, z = 0.f;
    const int n_keys = pos0 + t + 1;
    const unsigned long long sees = tree ? tree->sees[t] : ~0ull;
    for (int j = 0; j < n_keys; ++j) {
        if (j >= pos0 && !((sees >> ((j - pos0) & 63)) & 1)) continue;  // j - pos0 <= t < 64 in a tree call
        const float* kr = kv_row(kv, layer, 0, h, n_heads, dh, j);
        const float* vr = kv_row(kv, layer, 1, h, n_heads, dh, j);
        float part = 0.f;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (lane + r * kWave < dh) part = fmaf(qr[r], kr[lane + r * kWave], part);
        const float sc = wave_sum(part) * scale;
        const float m_new = fmaxf(m, sc);
        const float corr = expf(m - m_new);  // 0 on the first key (m = -inf)
        const float p = expf(sc - m_new);
        z = z * corr + p;
#pragma unroll
        for (int r = 0; r < 4; ++r)
            if (lane + r * kWave < dh) acc[r] = acc[r] * corr + p * vr[lane + r * kWave];
        m = m_new;
    }
    float* out = o + (size_t)t * d + (size_t)h * dh;
#pragma unroll
    for (int r = 0; r < 4; ++r)
        if (lane + r * kWave < dh) out[lane + r * kWave] = acc[r] / z;
}

// act[t][j] = silu(gate[t][j]) * up[t][j] with gate|up fused as [n, 2f].
__global__ void f32_swiglu(const float* __restrict__ gu, float* __restrict__ act, int n, int f) {
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (long long)n * f) return;
    const int j = (int)(gid % f);
    const long long t = gid / f;
    const float g = gu[t * 2 * f + j], u = gu[t * 2 * f + f + j];
    act[gid] = g / (1.0f + expf(-g)) * u;
}

void gemm(const float* A, int lda, const float* W, float* C, const float* R, int ldc, int M, int N, int K,
          hipStream_t s) {
    dim3 grid((N + 63) / 64, (M + 63) / 64);
    hipLaunchKernelGGL(f32_gemm_nt, grid, dim3(256), 0, s, A, lda, W, C, R, ldc, M, N, K);
}

}  // namespace

hipError_t f32_forward(const jup_stage& st, const float* hidden_in, int n, int pos, const KvView& kv,
                       float* hidden_out, hipStream_t s, const TreeTable* tree) {
    const jup_stage_config_t& c = st.cfg;
    const int d = c.d_model, f = c.d_ffn, H = c.n_heads, dh = c.head_dim;
    char* ws = (char*)st.workspace;
    float* x = (float*)(ws + st.wl.x32);
    float* xn = (float*)(ws + st.wl.xn);
    float* qkv = (float*)(ws + st.wl.q);
    float* o = (float*)(ws + st.wl.o);
    float* gu = (float*)(ws + st.wl.gu);
    float* act = (float*)(ws + st.wl.act);

    const TreeTable* tree_dev = nullptr;
    if (tree) {  // host table -> workspace
        tree_dev = (const TreeTable*)(ws + st.wl.tree);
        launch_write_tree_table(*tree, (TreeTable*)(ws + st.wl.tree), s);
    }
    hipError_t e = hipMemcpyAsync(x, hidden_in, (size_t)n * d * 4, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    for (int l = 0; l < c.n_layers; ++l) {
        const char* wb = (const char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const float* wqkv = (const float*)(wb + st.pl.wqkv);
        const float* wo = (const float*)(wb + st.pl.wo);
        const float* wgu = (const float*)(wb + st.pl.wgu);
        const float* wdown = (const float*)(wb + st.pl.wdown);
        const float* g1 = (const float*)(wb + st.pl.g_attn);
        const float* g2 = (const float*)(wb + st.pl.g_mlp);

        hipLaunchKernelGGL(f32_rmsnorm, dim3(n), dim3(256), 0, s, x, g1, xn, d, c.rms_eps);
        gemm(xn, d, wqkv, qkv, nullptr, 3 * d, n, 3 * d, d, s);
        {
            const long long work = (long long)n * H * (dh / 2);
            hipLaunchKernelGGL(f32_rope_append, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, qkv, n, d, H, dh,
                               pos, c.rope_theta, kv, l, tree_dev);
        }
        hipLaunchKernelGGL(f32_attention, dim3(n, H), dim3(kWave), 0, s, qkv, o, d, H, dh, pos, kv, l, tree_dev);
        gemm(o, d, wo, x, x, d, n, d, d, s);  // x <- x + o Wo^T (each element read and written by one thread)
        hipLaunchKernelGGL(f32_rmsnorm, dim3(n), dim3(256), 0, s, x, g2, xn, d, c.rms_eps);
        gemm(xn, d, wgu, gu, nullptr, 2 * f, n, 2 * f, d, s);
        {
            const long long work = (long long)n * f;
            hipLaunchKernelGGL(f32_swiglu, dim3((unsigned)((work + 255) / 256)), dim3(256), 0, s, gu, act, n, f);
        }
        gemm(act, f, wdown, x, x, d, n, d, f, s);
    }
    e = hipMemcpyAsync(hidden_out, x, (size_t)n * d * 4, hipMemcpyDeviceToDevice, s);
    if (e != hipSuccess) return e;
    return hipGetLastError();
}

}  // namespace jup
