// Types and small device helpers shared by the bf16 (matrix-core) translation units.
#pragma once

#include "jup_internal.h"

namespace jup {

typedef unsigned short u16;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

__device__ inline u16 f2bf(float f) {
    __bf16 b = (__bf16)f;  // round to nearest even
    return __builtin_bit_cast(u16, b);
}
__device__ inline float bf2f(u16 b) { return __uint_as_float((unsigned)b << 16); }
__device__ inline unsigned pack_bf16x2(float lo, float hi) { return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16); }

// Tells the compiler that p is the same in every lane (it is: built from kernel arguments, the workgroup id
// and the wave number).  Kept opaque so that "uniform base + 32-bit lane offset" survives to instruction
// selection and the pointer arithmetic of a load stays on the scalar unit.
__device__ inline const char* uniform_ptr(const char* p) {
    const unsigned long long v = (unsigned long long)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v);
    const unsigned hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const char*)(((unsigned long long)hi << 32) | lo);
}

// 16 bytes per lane from global memory straight into LDS: lane i's piece lands at lds_base + 16 i, where
// lds_base (a wave-uniform LDS byte address) travels in M0.  Issued as text so that the caller controls every
// wait itself: the hardware counts these loads in vmcnt only, and the caller orders them against LDS reads of
// the same bytes with explicit vmcnt waits and barriers.  (The builtin form makes the compiler's wait-count
// pass drain every load in flight before LDS reads it cannot tell apart, which undoes prefetching.)  The
// "memory" clobber keeps the compiler from moving LDS accesses across the instruction.  First form: a 64-bit
// address per lane; second form: a wave-uniform base plus a 32-bit byte offset per lane.
__device__ inline void load_to_lds_16(const void* gptr, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(gptr), "s"(lds_base) : "memory", "m0");
}
__device__ inline void load_to_lds_16(const void* uniform_base, unsigned lane_offset, unsigned lds_base) {
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_offset), "s"(uniform_base), "s"(lds_base)
                 : "memory", "m0");
}
// LDS byte address of a pointer into the workgroup's dynamic LDS.
__device__ inline unsigned lds_byte_address(const void* p) {
    return (unsigned)(size_t)(const __attribute__((address_space(3))) void*)p;
}

// Exchange between workgroups inside one kernel (partial results merged by the workgroup that finishes last).  The
// chip has one L2 per XCD, and ordinary stores of one XCD are not seen by loads of another before the kernel ends;
// a device-scope fence would fix that by writing back and invalidating the WHOLE L2, once per wave that executes it,
// under the feet of every other workgroup of the XCD (measured: a decode-sized attention launch got 25-90 us slower).
// These accessors instead make each access coherent by itself: relaxed atomics at device scope, which the hardware
// performs as write-through stores and L2-bypassing loads, 8 bytes at a time.
__device__ inline void store_coherent2(float* p, float a, float b) {
    const unsigned long long bits = (unsigned long long)__float_as_uint(a) | ((unsigned long long)__float_as_uint(b) << 32);
    __hip_atomic_store((unsigned long long*)p, bits, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ inline float2 load_coherent2(const float* p) {
    const unsigned long long bits = __hip_atomic_load((const unsigned long long*)p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    return make_float2(__uint_as_float((unsigned)bits), __uint_as_float((unsigned)(bits >> 32)));
}
// Counts this workgroup in (call from ONE thread, after a workgroup barrier that follows every thread's coherent
// stores and a wait for their completion); returns how many were counted before it.
__device__ inline int arrive_coherent(int* counter) {
    return __hip_atomic_fetch_add(counter, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// Waits until this wave's stores have been performed (a coherent store is performed when it is visible chip-wide).
__device__ inline void wait_stores_performed() { __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup"); }

__device__ inline float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

// Cache plane (layer, K|V, head) -> row pointers.  Positions below n_shared live in the parent's buffer.
__device__ inline const u16* kv_row_bf16(const KvView& kv, size_t plane, int pos) {
    if (pos < kv.n_shared) return (const u16*)kv.parent + (plane * kv.parent_cap + (size_t)pos) * 128;
    return (const u16*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * 128;
}
__device__ inline u16* kv_slot_bf16(const KvView& kv, int layer, int which, int head, int n_heads, int pos) {
    const size_t plane = ((size_t)layer * 2 + which) * n_heads + head;
    return (u16*)kv.own + (plane * kv.own_cap + (size_t)(pos - kv.n_shared)) * 128;
}

// GEMM operand layout, used for the weights and for every activation matrix a GEMM reads:
// [rows/32 row blocks][K/32 stages][2 KB].  A 2 KB block is the LDS image of 32 rows x 32 columns: rows are
// 64 bytes, four rows form a 256-byte super-row, and the 16-byte chunk ch of row r sits at slot
// ((4*(r&3) + ch) ^ ((r>>2)&3)) of super-row r>>2.  Returns the bf16-element offset of chunk k_chunk = k/8
// of row `row`; element k sits at +(k % 8).  Row counts are padded up to a multiple of 32.
__device__ __host__ inline size_t tiled_offset(int row, int k_chunk, int k_stages) {
    const int r = row & 31, ch = k_chunk & 3;
    const size_t block = (size_t)(row >> 5) * k_stages + (k_chunk >> 2);
    return block * 1024 + (r >> 2) * 128 + ((((r & 3) << 2) + ch) ^ ((r >> 2) & 3)) * 8;
}

// ---- GEMM (bf16_gemm.hip) -----------------------------------------------------------------------
enum { EPI_QKV = 0, EPI_PARTIAL = 1, EPI_SWIGLU = 2 };

struct GemmArgs {
    const u16* A;  // [M, K] activations in the tiled layout (rows padded to a multiple of 32)
    const u16* W;  // [N, K] weights in the tiled layout written by the pack kernels ([N/32][K/32][2 KB]);
                   // 4-bit stages: the packed codes (w4_gemm.hip)
    const float* w_scale;  // 4-bit stages only: packed scales
    int M, N, K;
    int m_tiles, n_tiles, splits;  // grid = m_tiles * n_tiles * splits workgroups
    int n_stride;                  // columns between consecutive N tiles (tile width actually owned)
    int kt_per_split;              // K tiles of 32 per split
    // EPI_QKV
    u16* q_out;          // [M, d_model] rotated queries
    const float2* rope;  // [M, 64] (cos, sin)
    KvView kv;
    int layer, n_heads, d_model, pos0;
    const BranchTable* branches;  // non-null: row m belongs to branch m / n_tok (kv and pos0 above are unused)
    bool shared_gpu;     // another chunk's kernels run beside this launch (overlapped multi-chunk call)
    // EPI_PARTIAL
    float* partial;  // [splits][M][N] fp32
    // EPI_SWIGLU
    u16* act;  // [M, N/2] in the tiled layout (it is the down projection's A operand)
};

enum GemmKind { GEMM_QKV, GEMM_O, GEMM_GATE_UP, GEMM_DOWN };

// Fills the tiling fields of `a` for the given problem and launches.  Returns the number of K splits
// used (the caller sums that many partial buffers for EPI_PARTIAL).
int gemm_plan_splits(int M, int N, int K, bool shared);  // shared: see GemmArgs::shared_gpu
hipError_t launch_gemm_qkv(GemmArgs a, hipStream_t s);
hipError_t launch_gemm_swiglu(GemmArgs a, hipStream_t s);
hipError_t launch_gemm_partial(GemmArgs a, hipStream_t s);
// name of the instantiation a projection of M rows runs as (benchmarks: which tiling a counter reading belongs to)
void gemm_kernel_name(GemmKind kind, int M, int d_model, int d_ffn, bool shared_gpu, char* buf, size_t size);
hipError_t gemm_configure();  // raises the dynamic-LDS limit of every instantiation (once per process)

// ---- projections of a 4-bit stage (w4_gemm.hip) ----------------------------------------------------
// epi: EPI_QKV, EPI_SWIGLU or EPI_PARTIAL; the tiling fields of `a` are filled here.  EPI_PARTIAL writes
// w4_plan_splits(N, K) partial buffers.
int w4_plan_splits(int N, int K);
hipError_t launch_gemm_w4(int epi, GemmArgs a, hipStream_t s);
// dst / dst_scale: packed codes (N * K / 2 bytes) and packed scales (N * K / 128 floats) of one matrix
void launch_pack_w4_qkv(unsigned char* dst, float* dst_scale, const void* cq, const void* ck, const void* cv,
                        const float* sq, const float* sk, const float* sv, int d, hipStream_t s);
void launch_pack_w4_gate_up(unsigned char* dst, float* dst_scale, const void* cg, const void* cu, const float* sg,
                            const float* su, int d, int f, hipStream_t s);
void launch_pack_w4_plain(unsigned char* dst, float* dst_scale, const void* c, const float* sc, int n_rows, int k,
                          hipStream_t s);

// ---- attention (bf16_attention.hip) ---------------------------------------------------------------
// Key splits of a query block over workgroups.  A chunk of up to 256 tokens has few query blocks; behind a long
// cached sequence each of them gets several workgroups, every one with a contiguous range of at least 16 tiles of
// 32 keys.  The number of ranges is a function of the chunk's length and of the query
// block's own key count and of nothing else, so a result never depends on what else is in the launch (a branch
// computes the same bits alone and batched with others).  The same function sizes the grid on the host (with the
// longest key range of the launch) and tells every workgroup on the device how many ranges ITS query block has.
// Measured on the 8-layer 7B-shaped stage, 5-token chunk: 8192 cached positions 1.63 -> 1.02 ms per call, 2048
// positions 1.01 -> 0.88 ms, 512 positions unchanged (no split below 16 tiles per range); 64-token chunk behind 8192
// positions 1.70 -> 1.28 ms, 128-token 1.94 -> 1.57 ms.
constexpr int kAttSplitRow = 132;  // floats per query row in the scratch of a split launch: 128 outputs, max, sum, pad
// (257..512 tokens as 128-query workgroups against one of two key ranges: measured slower than 64-query workgroups
// against all keys, 35 vs 22 us per launch at 512 tokens: the exchange between the two workgroups goes through memory
// and costs more than the shared tile fills save)
__host__ __device__ constexpr int att_max_splits(int n) { return n <= 64 ? 8 : n <= 128 ? 4 : n <= 256 ? 2 : 1; }
__host__ __device__ inline int att_key_splits(int n, int n_tiles) {
    // a range is worth a workgroup from 16 tiles on (64-query workgroups, 65..256 tokens: 32, they already share
    // every tile among two query blocks)
    const int cap = att_max_splits(n), s = n_tiles / (n <= 64 ? 16 : 32);
    return s < 1 ? 1 : s > cap ? cap : s;
}
// Scratch of split launches (workspace): split_buf holds kAttSplitRow floats per (query row, range), split_count one
// arrival counter per (query block, head), zero between launches.  Upper bounds for chunks of up to T tokens, as one
// chunk or as up to kMaxBranches branches: padded query rows x ranges <= 512 for one chunk (64 x 8, 128 x 4, 256 x 2),
// <= 8 (T + 31 min(T, kMaxBranches)) for branches.
inline size_t att_split_rows(int T, int n_heads, bool branches) {
    const size_t b = T < kMaxBranches ? T : kMaxBranches;
    const size_t per_head = branches ? 8 * ((size_t)T + 31 * b) : 512;
    return (per_head < 512 ? 512 : per_head) * (size_t)n_heads;
}
inline size_t att_split_counters(int T, int n_heads, bool branches) {
    const size_t b = T < kMaxBranches ? T : kMaxBranches;
    return ((size_t)(T + 31) / 32 + (branches ? b : 0)) * (size_t)n_heads;
}
struct AttScratch {
    float* split_buf;
    int* split_count;
    size_t rows;      // capacity of split_buf in query rows x ranges
    size_t counters;  // capacity of split_count
};
// o is written in the tiled layout (it is the output projection's A operand)
hipError_t attention_configure();  // raises the dynamic-LDS limit (once per process)
// tree (device pointer, may be null): inside the chunk a query sees the tokens of its row of the table only
hipError_t launch_chunk_attention(const u16* q, u16* o, int n, int d_model, int n_heads, int pos0, const KvView& kv,
                            int layer, hipStream_t s, AttScratch scratch, const TreeTable* tree = nullptr,
                            bool shared_gpu = false);
// n_branches chunks of n tokens each (rows b*n .. b*n+n-1 of q and o), every one against its own cache;
// max_keys: the longest pos0 + n among the branches
hipError_t launch_branch_attention(const u16* q, u16* o, int n, int n_branches, int d_model, int n_heads,
                             const BranchTable* branches, int max_keys, int layer, hipStream_t s, AttScratch scratch);

// ---- packing, rotary table, reduce + norm (bf16_misc.hip) -------------------------------------------
void launch_pack_qkv(u16* dst, const u16* wq, const u16* wk, const u16* wv, int d, hipStream_t s);
void launch_pack_gate_up(u16* dst, const u16* wg, const u16* wu, int d, int f, hipStream_t s);
void launch_pack_plain(u16* dst, const u16* w, int n_rows, int k, hipStream_t s);
// the same layouts filled with bf16(scale * (code - 8)) of 4-bit matrices
void launch_expand_qkv(u16* dst, const void* cq, const void* ck, const void* cv, const float* sq, const float* sk,
                       const float* sv, int d, hipStream_t s);
void launch_expand_gate_up(u16* dst, const void* cg, const void* cu, const float* sg, const float* su, int d, int f,
                           hipStream_t s);
void launch_expand_plain(u16* dst, const void* c, const float* sc, int n_rows, int k, hipStream_t s);
// (the rotary-table kernel is the first of every call; it also clears the call's arrival counters: zero[0 .. n_zero))
void launch_rope_table(float2* tab, int n, int pos0, float theta, int* zero, int n_zero, hipStream_t s);
void launch_rope_table_tree(float2* tab, int n, int pos0, const TreeTable* tree, float theta, int* zero, int n_zero,
                            hipStream_t s);
void launch_rope_table_branches(float2* tab, int n_rows, const BranchTable* branches, float theta, int* zero, int n_zero,
                                hipStream_t s);
void launch_write_branch_table(const BranchTable& host_table, BranchTable* dst, hipStream_t s);
// x32 <- (hidden_in ? hidden_in : x32) + sum_s partial[s];  xn <- rmsnorm(x32) * g (if g), tiled layout;
// out <- bf16(x32) (if out), row-major
void launch_reduce_norm(float* x32, const u16* hidden_in, const float* partial, int splits, size_t split_stride,
                        const u16* g, u16* xn, u16* out, int n, int d, float eps, hipStream_t s);

}  // namespace jup
