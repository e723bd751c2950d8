// Calibration kernels for the benchmark: what the matrix cores of this chip sustain in a loop that does nothing
// else, and the shader clock the chip holds while other work runs.  They compute no part of the method.
#include "bf16_common.h"

namespace jup {
namespace {

// A bare MFMA loop: every wave keeps 8 independent 32x32x16 bf16 accumulations going (a 2 x 4 block of an outer
// product of two A and four B fragments, the register shape of the GEMM's wave tile), two waves per SIMD.  The
// fragments come from caller-provided (random) data, so the datapath toggles as it does on real operands; the
// four B fragments rotate every iteration.  Per workgroup, lane 0 of wave 0 reports the shader-clock and
// reference-clock ticks the loop took.
__global__ __launch_bounds__(512) void mfma_peak_loop(const u16* __restrict__ operands, long iters,
                                                     unsigned long long* __restrict__ ticks, float* __restrict__ sink) {
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const bf16x8* src = (const bf16x8*)operands + (size_t)((blockIdx.x * 8 + wave) % 64) * 64 * 8 + lane;
    bf16x8 a0 = src[0], a1 = src[64];
    bf16x8 b[4] = {src[128], src[192], src[256], src[320]};
    f32x16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc[i][r] = 0.f;
    const unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    for (long it = 0; it < iters; ++it) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            acc[2 * j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b[j], acc[2 * j], 0, 0, 0);
            acc[2 * j + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b[j], acc[2 * j + 1], 0, 0, 0);
        }
        const bf16x8 t = b[0];
        b[0] = b[1]; b[1] = b[2]; b[2] = b[3]; b[3] = t;
    }
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int r = 0; r < 16; ++r) s += acc[i][r];
    const unsigned long long t1 = __builtin_amdgcn_s_memtime(), r1 = __builtin_amdgcn_s_memrealtime();
    if (s == 12345.678f) sink[0] = s;  // keeps the accumulators alive; practically never true
    if (threadIdx.x == 0) {
        ticks[2 * blockIdx.x] = t1 - t0;
        ticks[2 * blockIdx.x + 1] = r1 - r0;
    }
}

// One wave that sleeps until `ref_ticks` ticks of the fixed-frequency reference clock have passed (bounded: it
// always ends) and reports how many shader-clock ticks went by meanwhile.
__global__ __launch_bounds__(64) void clock_probe(unsigned long long ref_ticks, unsigned long long* __restrict__ ticks) {
    const unsigned long long t0 = __builtin_amdgcn_s_memtime(), r0 = __builtin_amdgcn_s_memrealtime();
    unsigned long long r1 = r0;
    // at most 2^30 reference ticks (about 10 s) are ever asked for, validated on the host: the loop always ends
    while (r1 - r0 < ref_ticks) {
        __builtin_amdgcn_s_sleep(64);
        r1 = __builtin_amdgcn_s_memrealtime();
    }
    const unsigned long long t1 = __builtin_amdgcn_s_memtime();
    if (threadIdx.x == 0) {
        ticks[0] = t1 - t0;
        ticks[1] = r1 - r0;
    }
}

// Fill-path probe: 8 waves per workgroup copy 1 KB pieces of `buf` (a window every workgroup walks, so the pieces
// come from L2) into LDS with the direct global->LDS loads the GEMM ring uses, DEPTH pieces per wave in flight.
// What it moves per second is the ceiling of the GEMM's operand fill.
template <int DEPTH>
__global__ __launch_bounds__(512) void fill_probe(const char* __restrict__ buf, unsigned window, int pieces_per_wave) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char fill_lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = lds_byte_address(fill_lds);
    // (offsets in 32-bit arithmetic with a mask: a 64-bit remainder per piece costs a wave more time than the load)
    const unsigned mask = window - 1u;                              // the window is a power of two
    const unsigned wg_off = ((blockIdx.x >> 3) * 65536u) & mask;    // workgroups b, b + 8, ... share an XCD and its L2
    for (int i = 0; i < pieces_per_wave; i += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {
            const unsigned off = (wg_off + ((unsigned)(i + u) * 8u + wave) * 1024u) & mask;
            load_to_lds_16(uniform_ptr(buf + off), lane * 16, lds0 + (wave * 8 + (u & 7)) * 1024);
        }
        __builtin_amdgcn_s_waitcnt(0x0F70 | (DEPTH & 0xF) | ((DEPTH >> 4) << 14));  // vmcnt(DEPTH): one batch stays in flight
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing lands after the wave has gone
}

// Stream probe: the weight stream of a short-chunk projection with everything else taken away.  Every workgroup (8
// waves) copies its own contiguous region of `buf` into LDS with the same direct loads, DEPTH pieces of 1 KB per wave in
// flight; nothing is read twice, so the bytes come from HBM.  What it moves per second, and how long a launch of a
// projection's size takes, is the floor of a kernel that streams that many weight bytes once.
template <int DEPTH>
__global__ __launch_bounds__(512) void stream_probe(const char* __restrict__ buf, size_t region, int pieces_per_wave) {
    extern __shared__ __attribute__((aligned(1024))) unsigned char fill_lds[];
    const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const unsigned lds0 = lds_byte_address(fill_lds);
    const char* base = buf + (size_t)blockIdx.x * region + (size_t)wave * 1024;
    for (int i = 0; i < pieces_per_wave; i += DEPTH) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u)
            load_to_lds_16(uniform_ptr(base + (size_t)(i + u) * 8192), lane * 16, lds0 + (wave * 8 + (u & 7)) * 1024);
        __builtin_amdgcn_s_waitcnt(0x0F70 | (DEPTH & 0xF) | ((DEPTH >> 4) << 14));  // vmcnt(DEPTH): one batch stays in flight
    }
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0): nothing lands after the wave has gone
}

// LDS-read probe: every wave reads 1 KB per instruction (16 bytes per lane, consecutive: conflict-free), eight
// instructions in flight at a time (issued as text, one wait per batch: the rate of the LDS, not the latency of one
// read); lane 0 of the workgroup reports the shader-clock ticks of the loop.
__global__ void lds_read_probe(int trips, unsigned long long* __restrict__ ticks, unsigned* __restrict__ sink) {
    __shared__ __attribute__((aligned(1024))) unsigned char rd_lds[65536];
    for (int i = threadIdx.x; i < 16384; i += blockDim.x) ((unsigned*)rd_lds)[i] = i;
    __syncthreads();
    const unsigned addr = lds_byte_address(rd_lds) + (threadIdx.x & 63) * 16 + ((threadIdx.x >> 6) & 3) * 1024;
    u32x4 acc = {0u, 0u, 0u, 0u};
    const unsigned long long t0 = __builtin_amdgcn_s_memtime();
    for (int i = 0; i < trips; ++i) {
#pragma unroll
        for (int half = 0; half < 2; ++half) {
            u32x4 v[8];
            asm volatile(
                "ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:4096\n\tds_read_b128 %2, %8 offset:8192\n\t"
                "ds_read_b128 %3, %8 offset:12288\n\tds_read_b128 %4, %8 offset:16384\n\tds_read_b128 %5, %8 offset:20480\n\t"
                "ds_read_b128 %6, %8 offset:24576\n\tds_read_b128 %7, %8 offset:28672\n\ts_waitcnt lgkmcnt(0)"
                : "=v"(v[0]), "=v"(v[1]), "=v"(v[2]), "=v"(v[3]), "=v"(v[4]), "=v"(v[5]), "=v"(v[6]), "=v"(v[7])
                : "v"(addr + half * 32768)
                : "memory");
#pragma unroll
            for (int u = 0; u < 8; ++u) acc[u & 3] ^= v[u][u & 3];
        }
    }
    __syncthreads();  // the slowest wave ends the measurement: the first wave is served first and finishes early
    const unsigned long long t1 = __builtin_amdgcn_s_memtime();
    if (threadIdx.x == 0) ticks[blockIdx.x] = t1 - t0;
    if (acc[0] == 0x12345u && acc[1] == 7u) sink[0] = acc[2] ^ acc[3];  // keeps the reads alive; practically never true
}

}  // namespace
}  // namespace jup

extern "C" {

jup_status_t jup_diag_mfma_loop(const void* operands, size_t operand_bytes, int32_t n_workgroups, int64_t iters_per_wave,
                                void* ticks, float* sink, void* stream, double* flop) {
    const char* me = "jup_diag_mfma_loop";
    if (!operands || !ticks || !sink) return jup::set_error(JUP_EINVAL, "%s: NULL buffer", me);
    if (operand_bytes < 64 * 64 * 8 * 16 + 6 * 64 * 16)
        return jup::set_error(JUP_EINVAL, "%s: operands must hold at least %d bytes", me, 64 * 64 * 8 * 16 + 6 * 64 * 16);
    if (n_workgroups < 1 || n_workgroups > 65536 || iters_per_wave < 1 || iters_per_wave > (1ll << 32))
        return jup::set_error(JUP_EINVAL, "%s: n_workgroups or iters_per_wave out of range", me);
    hipLaunchKernelGGL(jup::mfma_peak_loop, dim3(n_workgroups), dim3(512), 0, (hipStream_t)stream,
                       (const jup::u16*)operands, (long)iters_per_wave, (unsigned long long*)ticks, sink);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return jup::set_error(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    if (flop) *flop = (double)n_workgroups * 8.0 * (double)iters_per_wave * 8.0 * 2.0 * 32 * 32 * 16;
    return JUP_OK;
}

jup_status_t jup_diag_fill_probe(const void* buf, size_t window_bytes, int32_t n_workgroups, int32_t depth,
                                 int32_t pieces_per_wave, void* stream, double* bytes) {
    const char* me = "jup_diag_fill_probe";
    if (!buf) return jup::set_error(JUP_EINVAL, "%s: NULL buffer", me);
    if (window_bytes < (1u << 20) || window_bytes > (1u << 31) || (window_bytes & (window_bytes - 1)))
        return jup::set_error(JUP_EINVAL, "%s: the window must be a power of two between 1 MiB and 2 GiB", me);
    if (n_workgroups < 1 || n_workgroups > 65536 || pieces_per_wave < 16 || pieces_per_wave % 16 || pieces_per_wave > (1 << 24))
        return jup::set_error(JUP_EINVAL, "%s: n_workgroups or pieces_per_wave (a multiple of 16) out of range", me);
    const hipStream_t s = (hipStream_t)stream;
    switch (depth) {
#define JUP_FILL_CASE(D)                                                                                              \
        case D:                                                                                                       \
            hipLaunchKernelGGL(jup::fill_probe<D>, dim3(n_workgroups), dim3(512), 65536, s, (const char*)buf, (unsigned)window_bytes, \
                               pieces_per_wave);                                                                      \
            break;
        JUP_FILL_CASE(1) JUP_FILL_CASE(2) JUP_FILL_CASE(4) JUP_FILL_CASE(8) JUP_FILL_CASE(16)
#undef JUP_FILL_CASE
        default: return jup::set_error(JUP_EINVAL, "%s: depth must be 1, 2, 4, 8 or 16", me);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return jup::set_error(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    if (bytes) *bytes = (double)n_workgroups * 8.0 * (double)pieces_per_wave * 1024.0;
    return JUP_OK;
}

jup_status_t jup_diag_stream_probe(const void* buf, size_t buf_bytes, int32_t n_workgroups, int32_t depth,
                                   int32_t pieces_per_wave, int32_t n_launches, void* stream, double* bytes) {
    const char* me = "jup_diag_stream_probe";
    if (!buf) return jup::set_error(JUP_EINVAL, "%s: NULL buffer", me);
    if (depth != 1 && depth != 2 && depth != 4 && depth != 8 && depth != 16)
        return jup::set_error(JUP_EINVAL, "%s: depth must be 1, 2, 4, 8 or 16", me);
    if (n_workgroups < 1 || n_workgroups > 65536 || pieces_per_wave < depth || pieces_per_wave % depth || pieces_per_wave > (1 << 24))
        return jup::set_error(JUP_EINVAL, "%s: n_workgroups or pieces_per_wave (a multiple of depth) out of range", me);
    const size_t region = (size_t)pieces_per_wave * 8192;  // 8 waves x 1 KB per piece
    if (n_launches < 1 || n_launches > 4096) return jup::set_error(JUP_EINVAL, "%s: n_launches out of range", me);
    const size_t per_launch = region * (size_t)n_workgroups;
    if (buf_bytes / region < (size_t)n_workgroups)
        return jup::set_error(JUP_EINVAL, "%s: the buffer holds %zu bytes, a launch reads %zu", me, buf_bytes, per_launch);
    const size_t slots = buf_bytes / per_launch;  // successive launches read successive parts of the buffer, round robin
    const hipStream_t s = (hipStream_t)stream;
    for (int32_t i = 0; i < n_launches; ++i) {
        const char* part = (const char*)buf + (size_t)(i % slots) * per_launch;
        switch (depth) {
#define JUP_STREAM_CASE(D)                                                                                            \
            case D:                                                                                                   \
                hipLaunchKernelGGL(jup::stream_probe<D>, dim3(n_workgroups), dim3(512), 65536, s, part, region,        \
                                   pieces_per_wave);                                                                  \
                break;
            JUP_STREAM_CASE(1) JUP_STREAM_CASE(2) JUP_STREAM_CASE(4) JUP_STREAM_CASE(8) JUP_STREAM_CASE(16)
#undef JUP_STREAM_CASE
            default: return jup::set_error(JUP_EINVAL, "%s: depth must be 1, 2, 4, 8 or 16", me);
        }
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return jup::set_error(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    if (bytes) *bytes = (double)n_launches * (double)per_launch;
    return JUP_OK;
}

jup_status_t jup_diag_lds_read_probe(int32_t n_workgroups, int32_t threads, int32_t trips, void* ticks, void* sink,
                                     void* stream, double* bytes_per_workgroup) {
    const char* me = "jup_diag_lds_read_probe";
    if (!ticks || !sink) return jup::set_error(JUP_EINVAL, "%s: NULL buffer", me);
    if (n_workgroups < 1 || n_workgroups > 65536 || trips < 1 || trips > (1 << 24) || threads < 64 || threads > 1024 ||
        threads % 64)
        return jup::set_error(JUP_EINVAL, "%s: n_workgroups, threads (a multiple of 64 up to 1024) or trips out of range", me);
    hipLaunchKernelGGL(jup::lds_read_probe, dim3(n_workgroups), dim3(threads), 0, (hipStream_t)stream, trips,
                       (unsigned long long*)ticks, (unsigned*)sink);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return jup::set_error(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    if (bytes_per_workgroup) *bytes_per_workgroup = (double)threads * 16.0 * 16.0 * (double)trips;
    return JUP_OK;
}

jup_status_t jup_diag_kernel_name(const jup_stage_t* stage, int32_t kernel_id, int32_t n_tokens, int32_t overlapped,
                                  char* buf, size_t size) {
    const char* me = "jup_diag_kernel_name";
    if (!stage || !buf || size == 0) return jup::set_error(JUP_EINVAL, "%s: NULL argument", me);
    if (n_tokens < 1) return jup::set_error(JUP_EINVAL, "%s: n_tokens must be positive", me);
    const jup_stage_config_t& c = stage->cfg;
    jup::GemmKind kind;
    switch (kernel_id) {
        case JUP_K_GEMM_QKV: kind = jup::GEMM_QKV; break;
        case JUP_K_GEMM_O: kind = jup::GEMM_O; break;
        case JUP_K_GEMM_GATE_UP: kind = jup::GEMM_GATE_UP; break;
        case JUP_K_GEMM_DOWN: kind = jup::GEMM_DOWN; break;
        default: return jup::set_error(JUP_EINVAL, "%s: kernel id %d is not a projection", me, kernel_id);
    }
    if (c.dtype != JUP_BF16 && !(c.dtype == JUP_BF16_W4 && c.w4_expanded && n_tokens > 64))
        return jup::set_error(JUP_EINVAL, "%s: only the bf16 projections pick among tilings", me);
    jup::gemm_kernel_name(kind, n_tokens, c.d_model, c.d_ffn, overlapped != 0, buf, size);
    return JUP_OK;
}

jup_status_t jup_diag_clock_probe(int64_t ref_ticks, void* ticks, void* stream) {
    const char* me = "jup_diag_clock_probe";
    if (!ticks) return jup::set_error(JUP_EINVAL, "%s: NULL buffer", me);
    if (ref_ticks < 1 || ref_ticks > (1ll << 30)) return jup::set_error(JUP_EINVAL, "%s: ref_ticks out of range", me);
    hipLaunchKernelGGL(jup::clock_probe, dim3(1), dim3(64), 0, (hipStream_t)stream, (unsigned long long)ref_ticks,
                       (unsigned long long*)ticks);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return jup::set_error(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    return JUP_OK;
}

}  // extern "C"
