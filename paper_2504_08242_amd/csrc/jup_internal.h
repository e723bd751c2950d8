// Internal declarations shared by the translation units of libjupiter_stage.so.
// Host structs behind the opaque handles, the workspace/packed-weight layouts, and the launchers
// of the check-mode (fp32) and matrix-core (bf16) kernels.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "jupiter_stage.h"

namespace jup {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

// Byte offsets of one layer's sections inside the packed weight buffer.
struct PackedLayout {
    size_t wqkv;   // [3d, d]   rows: all Q heads, all K heads, all V heads
    size_t wo;     // [d, d]
    size_t wgu;    // [2f, d]   fp32: gate rows then up rows; bf16: 32-row groups gate/up interleaved
    size_t wdown;  // [d, f]
    size_t g_attn; // [d]
    size_t g_mlp;  // [d]
    // 4-bit stages: the four sections above hold packed codes (half a byte per weight) and these the packed fp32
    // scales, one per 128 input features of an output row
    size_t sqkv, so, sgu, sdown;
    // 4-bit stages created with w4_expanded: bf16 copies of the four matrices in the bf16 path's tiled layout, read
    // by chunks too long for the 4-bit kernels
    size_t xqkv, xo, xgu, xdown;
    size_t layer_bytes;
};
PackedLayout packed_layout(const jup_stage_config_t& c);

// Byte offsets of the per-call scratch tensors inside the workspace, for chunks of up to T tokens.
struct WorkspaceLayout {
    size_t x32;   // [T, d] fp32 residual stream
    size_t xn;    // [T, d] normalised rows (stage dtype)
    size_t q;     // bf16: [T, d] rotated queries; fp32: [T, 3d] q|k|v
    size_t o;     // [T, d] attention output, heads concatenated
    size_t gu;    // fp32 only: [T, 2f] gate|up
    size_t act;   // [T, f] silu(gate) * up
    size_t rope;  // [T, head_dim/2] float2 (cos, sin) of the chunk's positions
    size_t partial;  // bf16 only: [8][T, d] fp32 K-split partial sums of the O / down projections
    size_t branches; // bf16 only: BranchTable of a batched-branch call
    size_t tree;     // TreeTable of a token-tree call
    // bf16 only: scratch of attention launches that split the keys of a query block over workgroups
    size_t att_split;      // [att_split_rows][132] fp32: un-normalised outputs and softmax statistics per key range
    size_t att_count;      // [att_count_n] int32 arrival counters, zero between launches
    size_t att_split_rows, att_count_n;
    size_t total;
};
// branches: the workspace also serves jup_stage_prefill_branches (more query blocks per launch: more scratch)
WorkspaceLayout workspace_layout(const jup_stage_config_t& c, int32_t T, bool branches = true);

// Where the attention and append kernels find a cache: positions < n_shared live in the parent's
// buffer (stride parent_cap), the rest in the own buffer at slot (position - n_shared).
struct KvView {
    void* own;
    const void* parent;
    int32_t n_shared;
    int32_t own_cap;    // slots in the own buffer
    int32_t parent_cap; // slots in the parent's buffer (0 if none)
};

// Batched-branch call: rows [b * n_tok, (b + 1) * n_tok) of the activation matrices belong to branch b,
// whose chunk starts at position pos0[b] of cache kv[b].
constexpr int kMaxBranches = JUP_MAX_BRANCHES;
struct BranchTable {
    int32_t n_branches, n_tok;
    int32_t pos0[kMaxBranches];
    KvView kv[kMaxBranches];
};

// Token-tree call: token t of the chunk is rotated at pos0 + depth[t], stored in slot pos0 + t, and attends,
// inside the chunk, to the tokens whose bit is set in sees[t] (its ancestors and itself; bit j = token j).
constexpr int kMaxTreeTokens = JUP_MAX_TREE_TOKENS;
static_assert(kMaxTreeTokens <= 64, "one 64-bit word of visibility per token");
struct TreeTable {
    int32_t n;
    int32_t depth[kMaxTreeTokens];
    unsigned long long sees[kMaxTreeTokens];
};

// jup_kv_keep(): entry base + slots[j] of every (layer, K|V, head) plane moves to entry base + j.
struct KeepList {
    int32_t n;
    int32_t slots[kMaxTreeTokens];
};

}  // namespace jup

struct jup_kv {
    jup_stage_config_t cfg;
    void* buf;
    int32_t max_positions; // absolute capacity
    int32_t len;
    jup_kv* parent;   // non-null for a fork
    int32_t n_shared; // 0 for a root cache
    int32_t n_children;
    int32_t max_child_shared; // largest n_shared among live children (recomputed lazily is overkill: kept as a bound)
};

// Optional per-kernel timing with HIP events on the caller's stream (benchmarks only).
struct jup_trace {
    int32_t kernel_id;  // jup_kernel_id_t being timed
    hipEvent_t* ev;     // pairs (start, stop)
    int32_t capacity;   // number of pairs
    int32_t used;
    int32_t dropped;    // launches not timed because the pool was full
};

// Lanes of jup_stage_prefill_chunks(): consecutive chunks go round the lanes; lane 0 is the caller's stream with
// the stage's workspace, every further lane a stream and a workspace of its own.  ev_qkv[lane][l] is recorded when
// the lane's current chunk has written its keys and values of layer l; a chunk waits, before its attention of
// layer l, for that event of every other lane (the chunks before it that its own stream does not order).
namespace jup { constexpr int kMaxLanes = JUP_MAX_LANES; }
struct jup_overlap {
    int32_t n_lanes;
    void* workspace[jup::kMaxLanes];     // [0] unused
    hipStream_t stream[jup::kMaxLanes];  // [0] unused
    hipEvent_t ev_fork;
    hipEvent_t ev_join[jup::kMaxLanes];  // [0] unused
    hipEvent_t* ev_qkv[jup::kMaxLanes];  // [n_layers] each
};

struct jup_stage {
    jup_stage_config_t cfg;
    void* packed;
    void* workspace;
    int32_t max_chunk_tokens;
    jup::PackedLayout pl;
    jup::WorkspaceLayout wl;
    jup_trace* trace;      // NULL when tracing is off
    jup_overlap* overlap;  // NULL until jup_stage_enable_overlap()
};

namespace jup {

// Brackets one kernel launch with a pair of events when the stage traces that kernel id.
struct TraceScope {
    jup_trace* t;
    hipStream_t s;
    int slot;
    TraceScope(const jup_stage& st, int kernel_id, hipStream_t stream) : t(st.trace), s(stream), slot(-1) {
        if (!t || t->kernel_id != kernel_id) { t = nullptr; return; }
        if (t->used >= t->capacity) { t->dropped++; t = nullptr; return; }
        slot = t->used++;
        (void)hipEventRecord(t->ev[2 * slot], s);
    }
    ~TraceScope() {
        if (t) (void)hipEventRecord(t->ev[2 * slot + 1], s);
    }
    TraceScope(const TraceScope&) = delete;
    TraceScope& operator=(const TraceScope&) = delete;
};

// Records the message jup_last_error() returns on this thread and hands the status code back (jup_api.hip).
jup_status_t set_error(jup_status_t code, const char* fmt, ...) __attribute__((format(printf, 2, 3)));

// ---- check-mode (fp32) path: kernels_f32.hip ------------------------------------------------------
hipError_t f32_forward(const jup_stage& st, const float* hidden_in, int n, int pos, const KvView& kv,
                       float* hidden_out, hipStream_t s, const TreeTable* tree = nullptr);

// ---- matrix-core (bf16) path: bf16_forward.hip (and bf16_gemm / bf16_attention / bf16_misc) ----------------------------------------------------
hipError_t bf16_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s);
hipError_t w4_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s);  // 4-bit stage
// How one forward is tied to the forwards of the neighbouring chunks (jup_stage_prefill_chunks): which scratch
// buffer it uses, the events it records after the cache append of every layer, and the events (of the chunk
// before it, running on the other stream) it waits for before the attention of every layer.
struct ChunkLink {
    void* workspace = nullptr;                 // nullptr: the stage's own
    const hipEvent_t* record_qkv = nullptr;    // [n_layers] or nullptr
    int n_wait = 0;                            // other lanes that hold an earlier chunk
    const hipEvent_t* wait_qkv[kMaxLanes] = {};  // [n_layers] each
};
hipError_t bf16_forward(const jup_stage& st, const void* hidden_in, int n, int pos, const KvView& kv,
                        void* hidden_out, hipStream_t s, const BranchTable* branches = nullptr,
                        const TreeTable* tree = nullptr, const ChunkLink* link = nullptr);

// ---- cache and table helpers: kv_ops.hip --------------------------------------------------------------
// The tables of a call travel as kernel arguments and are parked in the workspace, where the kernels of the
// call read them (no host-to-device copy on the hot path).
void launch_write_tree_table(const TreeTable& host_table, TreeTable* dst, hipStream_t s);
// own: the cache's own buffer; own_cap: its slots; base: first destination slot in that buffer
void launch_kv_keep(void* own, int own_cap, int n_planes, int row_bytes, int base, const KeepList& list, hipStream_t s);

}  // namespace jup
