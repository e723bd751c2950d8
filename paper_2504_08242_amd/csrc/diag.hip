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
