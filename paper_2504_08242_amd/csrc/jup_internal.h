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
    size_t total;
};
WorkspaceLayout workspace_layout(const jup_stage_config_t& c, int32_t T);

// Where the attention and append kernels find a cache: positions < n_shared live in the parent's
// buffer (stride parent_cap), the rest in the own buffer at slot (position - n_shared).
struct KvView {
    void* own;
    const void* parent;
    int32_t n_shared;
    int32_t own_cap;    // slots in the own buffer
    int32_t parent_cap; // slots in the parent's buffer (0 if none)
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

struct jup_stage {
    jup_stage_config_t cfg;
    void* packed;
    void* workspace;
    int32_t max_chunk_tokens;
    jup::PackedLayout pl;
    jup::WorkspaceLayout wl;
};

namespace jup {

// ---- check-mode (fp32) path: kernels_f32.hip ------------------------------------------------------
hipError_t f32_forward(const jup_stage& st, const float* hidden_in, int n, int pos, const KvView& kv,
                       float* hidden_out, hipStream_t s);

// ---- matrix-core (bf16) path: kernels_bf16.hip ----------------------------------------------------
hipError_t bf16_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s);
hipError_t bf16_forward(const jup_stage& st, const void* hidden_in, int n, int pos, const KvView& kv,
                        void* hidden_out, hipStream_t s);

}  // namespace jup
