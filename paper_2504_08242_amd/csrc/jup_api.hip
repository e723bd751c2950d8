// Host side of the C ABI: argument validation, KV-cache bookkeeping, buffer layouts, dispatch to the
// fp32 check-mode path or the bf16 matrix-core path.  No device memory is allocated here.
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>

#include "bf16_common.h"

namespace {

thread_local char g_err[512] = "";

jup_status_t fail(jup_status_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

// bytes of an activation, gain or cache element (a 4-bit stage keeps all of those in bf16)
size_t elem_size(const jup_stage_config_t& c) { return c.dtype == JUP_F32 ? 4 : 2; }

}  // namespace

namespace jup {
// the same thread-local message for the entry points that live in other files
jup_status_t set_error(jup_status_t code, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}
}  // namespace jup

namespace {

// Empty string when the configuration is usable, otherwise the reason.
const char* check_cfg(const jup_stage_config_t* c) {
    if (!c) return "cfg is NULL";
    if (c->dtype != JUP_F32 && c->dtype != JUP_BF16 && c->dtype != JUP_BF16_W4)
        return "dtype must be JUP_F32, JUP_BF16 or JUP_BF16_W4";
    if (c->w4_expanded != 0 && !(c->w4_expanded == 1 && c->dtype == JUP_BF16_W4))
        return "w4_expanded must be 0, or 1 for a JUP_BF16_W4 stage";
    if (c->n_layers < 0 || c->n_layers > 4096) return "n_layers out of range";
    if (c->d_model <= 0 || c->n_heads <= 0 || c->head_dim <= 0 || c->d_ffn <= 0) return "sizes must be positive";
    if ((int64_t)c->n_heads * c->head_dim != c->d_model) return "d_model must equal n_heads * head_dim";
    if (c->head_dim & 1) return "head_dim must be even";
    if (c->head_dim > 256) return "head_dim above 256 is not supported";
    if (!(c->rms_eps >= 0.0f)) return "rms_eps must be >= 0";
    if (!(c->rope_theta > 0.0f)) return "rope_theta must be > 0";
    if (c->dtype != JUP_F32) {
        if (c->head_dim != 128) return "JUP_BF16 requires head_dim == 128";
        if (c->d_model % 256 || c->d_model > 8192) return "JUP_BF16 requires d_model % 256 == 0 and d_model <= 8192";
        if (c->d_ffn % 128) return "JUP_BF16 requires d_ffn % 128 == 0";
    }
    return "";
}

bool same_shape(const jup_stage_config_t& a, const jup_stage_config_t& b) {
    // a cache holds bf16 entries for JUP_BF16 and JUP_BF16_W4 stages alike: either kind of stage may use it
    return a.n_layers == b.n_layers && a.d_model == b.d_model && a.n_heads == b.n_heads &&
           a.head_dim == b.head_dim && elem_size(a) == elem_size(b);
}

size_t kv_bytes_for(const jup_stage_config_t& c, int64_t slots) {
    return (size_t)c.n_layers * 2 * (size_t)c.n_heads * (size_t)slots * (size_t)c.head_dim * elem_size(c);
}

bool misaligned(const void* p) { return ((uintptr_t)p % jup::kAlign) != 0; }
// the matrix-core kernels read and write rows of bf16 tensors 16 bytes at a time
bool misaligned16(const void* p) { return ((uintptr_t)p % 16) != 0; }

}  // namespace

namespace jup {

PackedLayout packed_layout(const jup_stage_config_t& c) {
    const size_t e = elem_size(c), d = c.d_model, f = c.d_ffn;
    PackedLayout p{};
    size_t off = 0;
    const bool w4 = c.dtype == JUP_BF16_W4;
    auto matrix = [&](size_t n_weights) { return align_up(w4 ? n_weights / 2 : n_weights * e); };
    p.wqkv = off;   off += matrix(3 * d * d);
    p.wo = off;     off += matrix(d * d);
    p.wgu = off;    off += matrix(2 * f * d);
    p.wdown = off;  off += matrix(d * f);
    p.g_attn = off; off += align_up(d * e);
    p.g_mlp = off;  off += align_up(d * e);
    if (w4) {
        p.sqkv = off;  off += align_up(3 * d * d / 128 * 4);
        p.so = off;    off += align_up(d * d / 128 * 4);
        p.sgu = off;   off += align_up(2 * f * d / 128 * 4);
        p.sdown = off; off += align_up(d * f / 128 * 4);
        if (c.w4_expanded) {
            p.xqkv = off;  off += align_up(3 * d * d * 2);
            p.xo = off;    off += align_up(d * d * 2);
            p.xgu = off;   off += align_up(2 * f * d * 2);
            p.xdown = off; off += align_up(d * f * 2);
        }
    }
    p.layer_bytes = off;
    return p;
}

WorkspaceLayout workspace_layout(const jup_stage_config_t& c, int32_t T, bool branches) {
    const size_t e = elem_size(c), d = c.d_model, f = c.d_ffn;
    const bool f32 = c.dtype == JUP_F32;
    // the matrix-core path stores GEMM operands in 32-row blocks
    const size_t t = f32 ? (size_t)T : ((size_t)T + 31) / 32 * 32;
    WorkspaceLayout w{};
    size_t off = 0;
    w.x32 = off;  off += align_up(t * d * 4);
    w.xn = off;   off += align_up(t * d * e);
    w.q = off;    off += align_up(t * d * e * (f32 ? 3 : 1));
    w.o = off;    off += align_up(t * d * e);
    w.gu = off;   off += f32 ? align_up(t * 2 * f * e) : 0;
    w.act = off;  off += align_up(t * f * e);
    w.rope = off; off += align_up(t * (size_t)(c.head_dim / 2) * 8);
    w.partial = off; off += f32 ? 0 : align_up(8 * t * d * 4);
    w.branches = off; off += f32 ? 0 : align_up(sizeof(BranchTable));
    w.tree = off; off += align_up(sizeof(TreeTable));
    w.att_split_rows = f32 ? 0 : att_split_rows(T, c.n_heads, branches);
    w.att_count_n = f32 ? 0 : att_split_counters(T, c.n_heads, branches);
    w.att_split = off; off += align_up(w.att_split_rows * kAttSplitRow * 4);
    w.att_count = off; off += align_up(w.att_count_n * 4);
    w.total = off;
    return w;
}

}  // namespace jup

extern "C" {

const char* jup_last_error(void) { return g_err; }

size_t jup_stage_packed_bytes(const jup_stage_config_t* cfg) {
    if (*check_cfg(cfg)) return 0;
    return jup::packed_layout(*cfg).layer_bytes * (size_t)cfg->n_layers + jup::kAlign;
}

size_t jup_stage_workspace_bytes(const jup_stage_config_t* cfg, int32_t max_chunk_tokens) {
    if (*check_cfg(cfg) || max_chunk_tokens <= 0) return 0;
    return jup::workspace_layout(*cfg, max_chunk_tokens).total + jup::kAlign;
}

jup_status_t jup_stage_create(const jup_stage_config_t* cfg, const jup_layer_weights_t* layers, void* packed,
                              size_t packed_bytes, void* workspace, size_t workspace_bytes,
                              int32_t max_chunk_tokens, void* stream, jup_stage_t** out) {
    if (out) *out = nullptr;
    const char* why = check_cfg(cfg);
    if (*why) return fail(JUP_EINVAL, "jup_stage_create: %s", why);
    if (!out) return fail(JUP_EINVAL, "jup_stage_create: out is NULL");
    if (cfg->n_layers > 0 && !layers) return fail(JUP_EINVAL, "jup_stage_create: layers is NULL");
    if (max_chunk_tokens <= 0) return fail(JUP_EINVAL, "jup_stage_create: max_chunk_tokens must be positive");
    if (!packed || !workspace) return fail(JUP_EINVAL, "jup_stage_create: packed and workspace must not be NULL");
    if (misaligned(packed) || misaligned(workspace))
        return fail(JUP_EINVAL, "jup_stage_create: packed and workspace must be 256-byte aligned");
    if (packed_bytes < jup_stage_packed_bytes(cfg))
        return fail(JUP_EINVAL, "jup_stage_create: packed buffer has %zu bytes, %zu needed", packed_bytes,
                    jup_stage_packed_bytes(cfg));
    if (workspace_bytes < jup_stage_workspace_bytes(cfg, max_chunk_tokens))
        return fail(JUP_EINVAL, "jup_stage_create: workspace has %zu bytes, %zu needed", workspace_bytes,
                    jup_stage_workspace_bytes(cfg, max_chunk_tokens));
    for (int l = 0; l < cfg->n_layers; ++l) {
        const jup_layer_weights_t& w = layers[l];
        if (!w.wq || !w.wk || !w.wv || !w.wo || !w.w_gate || !w.w_up || !w.w_down || !w.g_attn || !w.g_mlp)
            return fail(JUP_EINVAL, "jup_stage_create: layer %d has a NULL weight pointer", l);
        if (cfg->dtype == JUP_BF16_W4 && (!w.sq || !w.sk || !w.sv || !w.so || !w.s_gate || !w.s_up || !w.s_down))
            return fail(JUP_EINVAL, "jup_stage_create: layer %d has a NULL scale pointer", l);
        if (cfg->dtype != JUP_F32)
            for (const void* ptr : {w.wq, w.wk, w.wv, w.wo, w.w_gate, w.w_up, w.w_down, w.g_attn, w.g_mlp})
                if (misaligned16(ptr))
                    return fail(JUP_EINVAL, "jup_stage_create: layer %d has a weight pointer that is not 16-byte aligned", l);
    }

    jup_stage* st = new (std::nothrow) jup_stage();
    if (!st) return fail(JUP_ENOMEM, "jup_stage_create: out of host memory");
    st->cfg = *cfg;
    st->packed = packed;
    st->workspace = workspace;
    st->max_chunk_tokens = max_chunk_tokens;
    st->pl = jup::packed_layout(*cfg);
    st->wl = jup::workspace_layout(*cfg, max_chunk_tokens);
    st->trace = nullptr;
    st->overlap = nullptr;

    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (cfg->dtype == JUP_F32) {
        // Check mode reads the matrices as given: copy them section by section.
        const size_t d = cfg->d_model, f = cfg->d_ffn;
        for (int l = 0; l < cfg->n_layers && e == hipSuccess; ++l) {
            char* base = (char*)packed + (size_t)l * st->pl.layer_bytes;
            const jup_layer_weights_t& w = layers[l];
            struct { size_t off; const void* src; size_t bytes; } jobs[] = {
                {st->pl.wqkv, w.wq, d * d * 4},
                {st->pl.wqkv + d * d * 4, w.wk, d * d * 4},
                {st->pl.wqkv + 2 * d * d * 4, w.wv, d * d * 4},
                {st->pl.wo, w.wo, d * d * 4},
                {st->pl.wgu, w.w_gate, f * d * 4},
                {st->pl.wgu + f * d * 4, w.w_up, f * d * 4},
                {st->pl.wdown, w.w_down, d * f * 4},
                {st->pl.g_attn, w.g_attn, d * 4},
                {st->pl.g_mlp, w.g_mlp, d * 4},
            };
            for (auto& j : jobs) {
                e = hipMemcpyAsync(base + j.off, j.src, j.bytes, hipMemcpyDeviceToDevice, s);
                if (e != hipSuccess) break;
            }
        }
    } else if (cfg->dtype == JUP_BF16_W4) {
        e = jup::w4_pack_weights(*st, layers, s);
    } else {
        e = jup::bf16_pack_weights(*st, layers, s);
    }
    if (e != hipSuccess) {
        delete st;
        return fail(JUP_EDEVICE, "jup_stage_create: %s", hipGetErrorString(e));
    }
    *out = st;
    return JUP_OK;
}

static void trace_release(jup_stage* st) {
    if (!st->trace) return;
    for (int i = 0; i < 2 * st->trace->capacity; ++i)
        if (st->trace->ev[i]) (void)hipEventDestroy(st->trace->ev[i]);
    delete[] st->trace->ev;
    delete st->trace;
    st->trace = nullptr;
}

static void overlap_release(jup_stage* st) {
    jup_overlap* o = st->overlap;
    if (!o) return;
    for (int lane = 0; lane < jup::kMaxLanes; ++lane) {
        if (o->ev_qkv[lane]) {
            for (int l = 0; l < st->cfg.n_layers; ++l)
                if (o->ev_qkv[lane][l]) (void)hipEventDestroy(o->ev_qkv[lane][l]);
            delete[] o->ev_qkv[lane];
        }
        if (o->ev_join[lane]) (void)hipEventDestroy(o->ev_join[lane]);
        if (o->stream[lane]) (void)hipStreamDestroy(o->stream[lane]);
    }
    if (o->ev_fork) (void)hipEventDestroy(o->ev_fork);
    delete o;
    st->overlap = nullptr;
}

void jup_stage_destroy(jup_stage_t* stage) {
    if (!stage) return;
    trace_release(stage);
    overlap_release(stage);
    delete stage;
}

jup_status_t jup_stage_enable_overlap(jup_stage_t* stage, int32_t n_lanes, void* lane_workspaces,
                                      size_t lane_workspaces_bytes) {
    const char* me = "jup_stage_enable_overlap";
    if (!stage) return fail(JUP_EINVAL, "%s: stage is NULL", me);
    if (stage->overlap) return fail(JUP_EINVAL, "%s: already enabled", me);
    if (n_lanes < 2 || n_lanes > JUP_MAX_LANES) return fail(JUP_EINVAL, "%s: n_lanes=%d is outside 2..%d", me, n_lanes, JUP_MAX_LANES);
    if (!lane_workspaces || misaligned(lane_workspaces))
        return fail(JUP_EINVAL, "%s: lane_workspaces must be non-NULL and 256-byte aligned", me);
    const size_t each = jup_stage_workspace_bytes(&stage->cfg, stage->max_chunk_tokens);  // a multiple of 256
    const size_t need = each * (size_t)(n_lanes - 1);
    if (lane_workspaces_bytes < need) return fail(JUP_EINVAL, "%s: lane_workspaces has %zu bytes, %zu needed", me, lane_workspaces_bytes, need);
    const char* lo = (const char*)lane_workspaces;
    const char* ws = (const char*)stage->workspace;
    if (lo < ws + each && ws < lo + need) return fail(JUP_EINVAL, "%s: lane_workspaces overlaps the stage's workspace", me);
    jup_overlap* o = new (std::nothrow) jup_overlap();
    if (!o) return fail(JUP_ENOMEM, "%s: out of host memory", me);
    const int L = stage->cfg.n_layers;
    o->n_lanes = n_lanes;
    stage->overlap = o;  // from here on overlap_release() cleans up whatever exists
    hipError_t e = hipEventCreateWithFlags(&o->ev_fork, hipEventDisableTiming);
    for (int lane = 0; lane < n_lanes && e == hipSuccess; ++lane) {
        if (lane > 0) {
            o->workspace[lane] = (char*)lane_workspaces + each * (size_t)(lane - 1);
            e = hipStreamCreateWithFlags(&o->stream[lane], hipStreamNonBlocking);  // default priority
            if (e == hipSuccess) e = hipEventCreateWithFlags(&o->ev_join[lane], hipEventDisableTiming);
        }
        o->ev_qkv[lane] = new (std::nothrow) hipEvent_t[L > 0 ? L : 1]();
        if (!o->ev_qkv[lane]) {
            overlap_release(stage);
            return fail(JUP_ENOMEM, "%s: out of host memory", me);
        }
        for (int l = 0; l < L && e == hipSuccess; ++l) e = hipEventCreateWithFlags(&o->ev_qkv[lane][l], hipEventDisableTiming);
    }
    if (e != hipSuccess) {
        overlap_release(stage);
        return fail(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    }
    return JUP_OK;
}

jup_status_t jup_stage_trace(jup_stage_t* stage, int32_t kernel_id, int32_t max_launches) {
    if (!stage) return fail(JUP_EINVAL, "jup_stage_trace: stage is NULL");
    if (kernel_id == -1) {
        trace_release(stage);
        return JUP_OK;
    }
    if (kernel_id < 0 || kernel_id >= JUP_K_COUNT) return fail(JUP_EINVAL, "jup_stage_trace: bad kernel id %d", kernel_id);
    if (max_launches <= 0 || max_launches > (1 << 20))
        return fail(JUP_EINVAL, "jup_stage_trace: max_launches=%d out of range", max_launches);
    trace_release(stage);
    jup_trace* t = new (std::nothrow) jup_trace();
    if (!t) return fail(JUP_ENOMEM, "jup_stage_trace: out of host memory");
    t->kernel_id = kernel_id;
    t->capacity = max_launches;
    t->used = t->dropped = 0;
    t->ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_launches]();
    if (!t->ev) {
        delete t;
        return fail(JUP_ENOMEM, "jup_stage_trace: out of host memory");
    }
    stage->trace = t;
    for (int i = 0; i < 2 * max_launches; ++i) {
        hipError_t e = hipEventCreate(&t->ev[i]);
        if (e != hipSuccess) {
            t->ev[i] = nullptr;
            trace_release(stage);
            return fail(JUP_EDEVICE, "jup_stage_trace: %s", hipGetErrorString(e));
        }
    }
    return JUP_OK;
}

jup_status_t jup_stage_trace_read(jup_stage_t* stage, double* total_ms, int32_t* launches, int32_t* dropped) {
    if (!stage || !stage->trace) return fail(JUP_EINVAL, "jup_stage_trace_read: the stage is not tracing");
    jup_trace* t = stage->trace;
    double sum = 0.0;
    for (int i = 0; i < t->used; ++i) {
        hipError_t e = hipEventSynchronize(t->ev[2 * i + 1]);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t->ev[2 * i], t->ev[2 * i + 1]);
        if (e != hipSuccess) return fail(JUP_EDEVICE, "jup_stage_trace_read: %s", hipGetErrorString(e));
        sum += ms;
    }
    if (total_ms) *total_ms = sum;
    if (launches) *launches = t->used;
    if (dropped) *dropped = t->dropped;
    t->used = t->dropped = 0;
    return JUP_OK;
}

// ---- KV cache ---------------------------------------------------------------------------------

size_t jup_kv_bytes(const jup_stage_config_t* cfg, int32_t max_positions) {
    if (*check_cfg(cfg) || max_positions <= 0) return 0;
    return kv_bytes_for(*cfg, max_positions);
}

jup_status_t jup_kv_create(const jup_stage_config_t* cfg, int32_t max_positions, void* device_buf,
                           size_t device_bytes, jup_kv_t** out) {
    if (out) *out = nullptr;
    const char* why = check_cfg(cfg);
    if (*why) return fail(JUP_EINVAL, "jup_kv_create: %s", why);
    if (!out) return fail(JUP_EINVAL, "jup_kv_create: out is NULL");
    if (max_positions <= 0) return fail(JUP_EINVAL, "jup_kv_create: max_positions must be positive");
    if (!device_buf || misaligned(device_buf))
        return fail(JUP_EINVAL, "jup_kv_create: device_buf must be non-NULL and 256-byte aligned");
    if (device_bytes < kv_bytes_for(*cfg, max_positions))
        return fail(JUP_EINVAL, "jup_kv_create: buffer has %zu bytes, %zu needed", device_bytes,
                    kv_bytes_for(*cfg, max_positions));
    jup_kv* kv = new (std::nothrow) jup_kv();
    if (!kv) return fail(JUP_ENOMEM, "jup_kv_create: out of host memory");
    kv->cfg = *cfg;
    kv->buf = device_buf;
    kv->max_positions = max_positions;
    kv->len = 0;
    kv->parent = nullptr;
    kv->n_shared = 0;
    kv->n_children = 0;
    kv->max_child_shared = 0;
    *out = kv;
    return JUP_OK;
}

size_t jup_kv_fork_bytes(const jup_kv_t* parent, int32_t n_shared, int32_t max_positions) {
    if (!parent || n_shared < 0 || max_positions <= n_shared) return 0;
    return kv_bytes_for(parent->cfg, (int64_t)max_positions - n_shared);
}

jup_status_t jup_kv_fork(jup_kv_t* parent, int32_t n_shared, int32_t max_positions, void* device_buf,
                         size_t device_bytes, jup_kv_t** out) {
    if (out) *out = nullptr;
    if (!parent || !out) return fail(JUP_EINVAL, "jup_kv_fork: parent and out must not be NULL");
    if (parent->parent) return fail(JUP_EINVAL, "jup_kv_fork: the parent is itself a fork");
    if (n_shared < 0 || n_shared > parent->len)
        return fail(JUP_EPOS, "jup_kv_fork: n_shared=%d outside [0, parent length %d]", n_shared, parent->len);
    if (max_positions <= n_shared)
        return fail(JUP_EINVAL, "jup_kv_fork: max_positions=%d must exceed n_shared=%d", max_positions, n_shared);
    if (!device_buf || misaligned(device_buf))
        return fail(JUP_EINVAL, "jup_kv_fork: device_buf must be non-NULL and 256-byte aligned");
    const size_t need = kv_bytes_for(parent->cfg, (int64_t)max_positions - n_shared);
    if (device_bytes < need) return fail(JUP_EINVAL, "jup_kv_fork: buffer has %zu bytes, %zu needed", device_bytes, need);
    jup_kv* kv = new (std::nothrow) jup_kv();
    if (!kv) return fail(JUP_ENOMEM, "jup_kv_fork: out of host memory");
    kv->cfg = parent->cfg;
    kv->buf = device_buf;
    kv->max_positions = max_positions;
    kv->len = n_shared;
    kv->parent = parent;
    kv->n_shared = n_shared;
    kv->n_children = 0;
    kv->max_child_shared = 0;
    parent->n_children += 1;
    if (n_shared > parent->max_child_shared) parent->max_child_shared = n_shared;
    *out = kv;
    return JUP_OK;
}

jup_status_t jup_kv_reset(jup_kv_t* kv) {
    if (!kv) return fail(JUP_EINVAL, "jup_kv_reset: kv is NULL");
    if (kv->n_children > 0 && kv->max_child_shared > 0)
        return fail(JUP_EPOS, "jup_kv_reset: live forks share the first %d positions", kv->max_child_shared);
    kv->len = kv->n_shared;
    return JUP_OK;
}

jup_status_t jup_kv_truncate(jup_kv_t* kv, int32_t new_len) {
    if (!kv) return fail(JUP_EINVAL, "jup_kv_truncate: kv is NULL");
    if (new_len < 0 || new_len > kv->len)
        return fail(JUP_EPOS, "jup_kv_truncate: new_len=%d outside [0, %d]", new_len, kv->len);
    if (new_len < kv->n_shared)
        return fail(JUP_EPOS, "jup_kv_truncate: new_len=%d cuts into the shared prefix of %d", new_len, kv->n_shared);
    if (kv->n_children > 0 && new_len < kv->max_child_shared)
        return fail(JUP_EPOS, "jup_kv_truncate: live forks share the first %d positions", kv->max_child_shared);
    kv->len = new_len;
    return JUP_OK;
}

jup_status_t jup_kv_keep(jup_kv_t* kv, int32_t base_len, int32_t n_keep, const int32_t* slots, void* stream) {
    const char* me = "jup_kv_keep";
    if (!kv) return fail(JUP_EINVAL, "%s: kv is NULL", me);
    if (n_keep < 0 || n_keep > JUP_MAX_TREE_TOKENS)
        return fail(JUP_EINVAL, "%s: n_keep=%d is outside 0..%d", me, n_keep, JUP_MAX_TREE_TOKENS);
    if (n_keep > 0 && !slots) return fail(JUP_EINVAL, "%s: slots is NULL", me);
    if (base_len < 0 || base_len > kv->len)
        return fail(JUP_EPOS, "%s: base_len=%d outside [0, %d]", me, base_len, kv->len);
    if (base_len < kv->n_shared)
        return fail(JUP_EPOS, "%s: base_len=%d cuts into the shared prefix of %d", me, base_len, kv->n_shared);
    if (kv->n_children > 0 && base_len < kv->max_child_shared)
        return fail(JUP_EPOS, "%s: live forks share the first %d positions", me, kv->max_child_shared);
    jup::KeepList list{};
    list.n = n_keep;
    bool moves = false;
    for (int j = 0; j < n_keep; ++j) {
        if (slots[j] < 0 || (j > 0 && slots[j] <= slots[j - 1]))
            return fail(JUP_EINVAL, "%s: slots must be non-negative and strictly increasing (slots[%d]=%d)", me, j,
                        slots[j]);
        if ((int64_t)base_len + slots[j] >= kv->len)
            return fail(JUP_EPOS, "%s: slots[%d]=%d lies behind the %d cached positions", me, j, slots[j], kv->len);
        list.slots[j] = slots[j];
        moves |= slots[j] != j;
    }
    if (moves) {
        const jup_stage_config_t& c = kv->cfg;
        jup::launch_kv_keep(kv->buf, kv->max_positions - kv->n_shared, c.n_layers * 2 * c.n_heads,
                            c.head_dim * (int)elem_size(c), base_len - kv->n_shared, list, (hipStream_t)stream);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return fail(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    }
    kv->len = base_len + n_keep;
    return JUP_OK;
}

int32_t jup_kv_len(const jup_kv_t* kv) { return kv ? kv->len : -1; }
int32_t jup_kv_capacity(const jup_kv_t* kv) { return kv ? kv->max_positions : -1; }

jup_status_t jup_kv_check_append(const jup_kv_t* kv, int32_t n_tokens, int32_t pos_offset) {
    if (!kv) return fail(JUP_EINVAL, "kv is NULL");
    if (n_tokens < 0) return fail(JUP_EINVAL, "n_tokens=%d is negative", n_tokens);
    if (pos_offset < 0) return fail(JUP_EINVAL, "pos_offset=%d is negative", pos_offset);
    if (pos_offset > kv->len)
        return fail(JUP_EPOS, "pos_offset=%d leaves a hole after the %d cached positions", pos_offset, kv->len);
    if (pos_offset < kv->n_shared)
        return fail(JUP_EPOS, "pos_offset=%d lies inside the read-only shared prefix of %d", pos_offset, kv->n_shared);
    if (kv->n_children > 0 && pos_offset < kv->max_child_shared)
        return fail(JUP_EPOS, "pos_offset=%d would overwrite positions shared with live forks (%d)", pos_offset,
                    kv->max_child_shared);
    if ((int64_t)pos_offset + n_tokens > kv->max_positions)
        return fail(JUP_ECAP, "pos_offset=%d + n_tokens=%d exceeds max_positions=%d", pos_offset, n_tokens,
                    kv->max_positions);
    return JUP_OK;
}

jup_status_t jup_kv_destroy(jup_kv_t* kv) {
    if (!kv) return JUP_OK;
    if (kv->n_children > 0) return fail(JUP_EINVAL, "jup_kv_destroy: %d forks are still alive", kv->n_children);
    if (kv->parent) {
        kv->parent->n_children -= 1;
        if (kv->parent->n_children == 0) kv->parent->max_child_shared = 0;
    }
    delete kv;
    return JUP_OK;
}

// ---- the hot path -----------------------------------------------------------------------------
}  // extern "C"

namespace {
jup::KvView view_of(const jup_kv_t* kv) {
    jup::KvView view{};
    view.own = kv->buf;
    view.parent = kv->parent ? kv->parent->buf : nullptr;
    view.n_shared = kv->n_shared;
    view.own_cap = kv->max_positions - kv->n_shared;
    view.parent_cap = kv->parent ? kv->parent->max_positions : 0;
    return view;
}
}  // namespace

namespace {
// One chunk, ordinary (parents == NULL) or a token tree.
jup_status_t prefill_one(const char* me, jup_stage_t* stage, const void* hidden_in, int32_t n_tokens,
                         int32_t pos_offset, const int32_t* parents, bool is_tree, jup_kv_t* kv, void* hidden_out,
                         void* stream) {
    if (!stage) return fail(JUP_EINVAL, "%s: stage is NULL", me);
    if (!kv) return fail(JUP_EINVAL, "%s: kv is NULL", me);
    if (!same_shape(stage->cfg, kv->cfg)) return fail(JUP_EINVAL, "%s: the cache was made for another configuration", me);
    jup_status_t rc = jup_kv_check_append(kv, n_tokens, pos_offset);
    if (rc != JUP_OK) {
        char tmp[400];
        snprintf(tmp, sizeof(tmp), "%s", g_err);
        return fail(rc, "%s: %s", me, tmp);
    }
    if (n_tokens > stage->max_chunk_tokens)
        return fail(JUP_ECAP, "%s: n_tokens=%d exceeds the stage's max_chunk_tokens=%d", me, n_tokens,
                    stage->max_chunk_tokens);
    jup::TreeTable tree{};
    if (is_tree) {
        if (n_tokens > JUP_MAX_TREE_TOKENS)
            return fail(JUP_EINVAL, "%s: n_tokens=%d exceeds the %d tokens of a tree", me, n_tokens, JUP_MAX_TREE_TOKENS);
        if (n_tokens > 0 && !parents) return fail(JUP_EINVAL, "%s: parents is NULL", me);
        tree.n = n_tokens;
        for (int t = 0; t < n_tokens; ++t) {
            const int par = parents[t];
            if (par < -1 || par >= t)
                return fail(JUP_EINVAL, "%s: parents[%d]=%d is not -1 or an earlier token", me, t, par);
            tree.depth[t] = par < 0 ? 0 : tree.depth[par] + 1;
            tree.sees[t] = (par < 0 ? 0ull : tree.sees[par]) | (1ull << t);
        }
    }
    if (kv->parent && kv->parent->len < kv->n_shared)
        return fail(JUP_EPOS, "%s: the parent cache holds %d positions, fewer than the %d shared", me, kv->parent->len,
                    kv->n_shared);
    if (n_tokens == 0) {
        kv->len = pos_offset;
        return JUP_OK;
    }
    if (!hidden_in || !hidden_out) return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must not be NULL", me);
    if (stage->cfg.dtype != JUP_F32 && (misaligned16(hidden_in) || misaligned16(hidden_out)))
        return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must be 16-byte aligned", me);

    const jup::KvView view = view_of(kv);
    const jup::TreeTable* tt = is_tree ? &tree : nullptr;
    hipStream_t s = (hipStream_t)stream;
    hipError_t e;
    if (stage->cfg.dtype == JUP_F32)
        e = jup::f32_forward(*stage, (const float*)hidden_in, n_tokens, pos_offset, view, (float*)hidden_out, s, tt);
    else
        e = jup::bf16_forward(*stage, hidden_in, n_tokens, pos_offset, view, hidden_out, s, nullptr, tt);
    if (e != hipSuccess) return fail(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    kv->len = pos_offset + n_tokens;
    return JUP_OK;
}
}  // namespace

extern "C" {

jup_status_t jup_stage_prefill_chunk(jup_stage_t* stage, const void* hidden_in, int32_t n_tokens,
                                     int32_t pos_offset, jup_kv_t* kv, void* hidden_out, void* stream) {
    return prefill_one("jup_stage_prefill_chunk", stage, hidden_in, n_tokens, pos_offset, nullptr, false, kv,
                       hidden_out, stream);
}

}  // extern "C"

// ---- the entry point that allocates nothing ------------------------------------------------------------------
// Scratch of jup_stage_prefill_chunk_static(): lives in the code object, one copy per GPU the library runs on, held
// until the process ends.  In host code the name below is only a handle for hipGetSymbolAddress(); the device address
// it yields (per device) is what the kernels get.
static __device__ __align__(256) unsigned char scratch[JUP_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Device address of `scratch` on the current device; looked up once per device.
hipError_t static_scratch(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* ptr = nullptr;
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!ptr) return hipErrorInvalidSymbol;
        g_scratch_ptr[dev] = ptr;
    }
    *out = g_scratch_ptr[dev];
    return hipSuccess;
}
}  // namespace

extern "C" {

jup_status_t jup_stage_prefill_chunk_static(jup_stage_t* stage, const void* hidden_in, int32_t n_tokens,
                                            int32_t pos_offset, jup_kv_t* kv, void* hidden_out, void* stream) {
    const char* me = "jup_stage_prefill_chunk_static";
    if (!stage) return fail(JUP_EINVAL, "%s: stage is NULL", me);
    if (n_tokens < 0) return fail(JUP_EINVAL, "%s: n_tokens=%d is negative", me, n_tokens);
    // the same forward on a copy of the stage whose workspace is the static array, laid out for this chunk alone
    jup_stage view = *stage;
    view.overlap = nullptr;
    if (n_tokens > 0) {
        view.wl = jup::workspace_layout(stage->cfg, n_tokens, false);  // one chunk, no branches
        if (view.wl.total > (size_t)JUP_STATIC_SCRATCH_BYTES)
            return fail(JUP_ECAP, "%s: a chunk of %d tokens of this stage needs %zu bytes of scratch, the static buffer "
                        "holds %d (use jup_stage_prefill_chunk with a caller-provided workspace)", me, n_tokens,
                        view.wl.total, JUP_STATIC_SCRATCH_BYTES);
        void* ptr = nullptr;
        const hipError_t e = static_scratch(&ptr);
        if (e != hipSuccess) return fail(JUP_EDEVICE, "%s: address of the static scratch: %s", me, hipGetErrorString(e));
        view.workspace = ptr;
        view.max_chunk_tokens = n_tokens;
    }
    return prefill_one(me, &view, hidden_in, n_tokens, pos_offset, nullptr, false, kv, hidden_out, stream);
}

jup_status_t jup_stage_prefill_tree(jup_stage_t* stage, const void* hidden_in, int32_t n_tokens, int32_t pos_offset,
                                    const int32_t* parents, jup_kv_t* kv, void* hidden_out, void* stream) {
    return prefill_one("jup_stage_prefill_tree", stage, hidden_in, n_tokens, pos_offset, parents, true, kv,
                       hidden_out, stream);
}

jup_status_t jup_stage_prefill_chunks(jup_stage_t* stage, const void* hidden_in, int32_t n_chunks,
                                      const int32_t* chunk_tokens, int32_t pos_offset, jup_kv_t* kv, void* hidden_out,
                                      void* stream) {
    const char* me = "jup_stage_prefill_chunks";
    if (!stage) return fail(JUP_EINVAL, "%s: stage is NULL", me);
    if (!kv) return fail(JUP_EINVAL, "%s: kv is NULL", me);
    if (n_chunks < 0 || (n_chunks > 0 && !chunk_tokens)) return fail(JUP_EINVAL, "%s: bad chunk list", me);
    if (!same_shape(stage->cfg, kv->cfg)) return fail(JUP_EINVAL, "%s: the cache was made for another configuration", me);
    // everything is validated before anything is enqueued: the chunks are consecutive, so only the first position
    // and the total length matter beyond the per-chunk limits
    long total = 0;
    for (int c = 0; c < n_chunks; ++c) {
        if (chunk_tokens[c] < 0) return fail(JUP_EINVAL, "%s: chunk_tokens[%d]=%d is negative", me, c, chunk_tokens[c]);
        if (chunk_tokens[c] > stage->max_chunk_tokens)
            return fail(JUP_ECAP, "%s: chunk_tokens[%d]=%d exceeds the stage's max_chunk_tokens=%d", me, c, chunk_tokens[c],
                        stage->max_chunk_tokens);
        total += chunk_tokens[c];
    }
    if (total > INT32_MAX) return fail(JUP_ECAP, "%s: too many tokens", me);
    jup_status_t rc = jup_kv_check_append(kv, (int32_t)total, pos_offset);
    if (rc != JUP_OK) {
        char tmp[400];
        snprintf(tmp, sizeof(tmp), "%s", g_err);
        return fail(rc, "%s: %s", me, tmp);
    }
    if (kv->parent && kv->parent->len < kv->n_shared)
        return fail(JUP_EPOS, "%s: the parent cache holds %d positions, fewer than the %d shared", me, kv->parent->len,
                    kv->n_shared);
    if (total > 0 && (!hidden_in || !hidden_out)) return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must not be NULL", me);
    if (stage->cfg.dtype != JUP_F32 && (misaligned16(hidden_in) || misaligned16(hidden_out)))
        return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must be 16-byte aligned", me);

    const size_t row_bytes = (size_t)stage->cfg.d_model * elem_size(stage->cfg);
    // the bf16 projections overlap; those of a 4-bit stage do when every chunk is long enough to run on its bf16 copy
    bool bf16_gemms = stage->cfg.dtype == JUP_BF16 || (stage->cfg.dtype == JUP_BF16_W4 && stage->cfg.w4_expanded);
    int busy = 0;  // chunks with tokens so far
    for (int c = 0; c < n_chunks; ++c) {
        busy += chunk_tokens[c] > 0;
        if (stage->cfg.dtype == JUP_BF16_W4 && chunk_tokens[c] > 0 && chunk_tokens[c] <= 64) bf16_gemms = false;
    }
    jup_overlap* o = bf16_gemms && stage->cfg.n_layers > 0 ? stage->overlap : nullptr;
    if (!o || busy < 2) {  // one after the other on the caller's stream
        int32_t pos = pos_offset;
        const char* in = (const char*)hidden_in;
        char* out = (char*)hidden_out;
        for (int c = 0; c < n_chunks; ++c) {
            rc = prefill_one(me, stage, in, chunk_tokens[c], pos, nullptr, false, kv, out, stream);
            if (rc != JUP_OK) return rc;
            pos += chunk_tokens[c];
            in += (size_t)chunk_tokens[c] * row_bytes;
            out += (size_t)chunk_tokens[c] * row_bytes;
        }
        if (n_chunks == 0 || total == 0) kv->len = pos_offset;
        return JUP_OK;
    }

    // Chunk number i (among those with tokens) runs on lane i mod n_lanes.  A lane is a stream plus a scratch buffer,
    // so the chunks of one lane are ordered by their stream; against the chunks before it on the other lanes a chunk
    // waits, layer by layer, for their cache append before its attention.
    hipStream_t s0 = (hipStream_t)stream;
    // Short chunks gain from every lane they get (measured with 64-, 128- and 256-token chunks: each further lane hides
    // more launch gaps and lets more chunks share one pass of the weights through the last-level cache).  Longer
    // chunks take all four lanes when their number is a multiple of four and two otherwise: with 4 x 512 tokens
    // on three lanes the fourth chunk queues behind the first and ends up running alone (-6 %).
    int longest = 0;
    for (int c = 0; c < n_chunks; ++c) longest = chunk_tokens[c] > longest ? chunk_tokens[c] : longest;
    int n_lanes = longest > 256 && busy % 4 != 0 ? 2 : o->n_lanes;
    if (n_lanes > o->n_lanes) n_lanes = o->n_lanes;
    if (n_lanes > busy) n_lanes = busy;
    hipError_t e = hipEventRecord(o->ev_fork, s0);  // the other lanes start behind what the caller enqueued before
    for (int lane = 1; lane < n_lanes && e == hipSuccess; ++lane) e = hipStreamWaitEvent(o->stream[lane], o->ev_fork, 0);
    const jup::KvView view = view_of(kv);
    int32_t pos = pos_offset;
    const char* in = (const char*)hidden_in;
    char* out = (char*)hidden_out;
    int i = 0;
    for (int c = 0; c < n_chunks && e == hipSuccess; ++c) {
        const int n = chunk_tokens[c];
        if (n == 0) continue;
        const int lane = i % n_lanes;
        jup::ChunkLink link;
        link.workspace = lane ? o->workspace[lane] : stage->workspace;
        link.record_qkv = o->ev_qkv[lane];
        for (int other = 0; other < n_lanes; ++other)  // lanes that already hold a chunk of this call
            if (other != lane && other < i) link.wait_qkv[link.n_wait++] = o->ev_qkv[other];
        e = jup::bf16_forward(*stage, in, n, pos, view, out, lane ? o->stream[lane] : s0, nullptr, nullptr, &link);
        pos += n;
        in += (size_t)n * row_bytes;
        out += (size_t)n * row_bytes;
        ++i;
    }
    // The caller's stream continues when the other lanes are done.  Also when a launch failed half way: the lanes
    // that already run write cache entries and hidden_out, and whatever the caller enqueues next must be ordered
    // behind them.  The cache length then stays as it was: the entries past it are unspecified, as after any
    // failed call, and the next call at pos_offset <= length overwrites them.
    hipError_t ej = hipSuccess;
    for (int lane = 1; lane < n_lanes; ++lane) {
        hipError_t e1 = hipEventRecord(o->ev_join[lane], o->stream[lane]);
        if (e1 == hipSuccess) e1 = hipStreamWaitEvent(s0, o->ev_join[lane], 0);
        if (ej == hipSuccess) ej = e1;
    }
    if (e == hipSuccess) e = ej;
    if (e != hipSuccess) return fail(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    kv->len = pos;
    return JUP_OK;
}

jup_status_t jup_stage_prefill_branches(jup_stage_t* stage, int32_t n_branches, const void* hidden_in,
                                        int32_t n_tokens, const int32_t* pos_offsets, jup_kv_t* const* kvs,
                                        void* hidden_out, void* stream) {
    const char* me = "jup_stage_prefill_branches";
    if (!stage) return fail(JUP_EINVAL, "%s: stage is NULL", me);
    if (n_branches < 1 || n_branches > JUP_MAX_BRANCHES)
        return fail(JUP_EINVAL, "%s: n_branches=%d is outside 1..%d", me, n_branches, JUP_MAX_BRANCHES);
    if (!pos_offsets || !kvs) return fail(JUP_EINVAL, "%s: pos_offsets and kvs must not be NULL", me);
    if (n_tokens < 0) return fail(JUP_EINVAL, "%s: n_tokens=%d is negative", me, n_tokens);
    for (int b = 0; b < n_branches; ++b) {  // the list itself first, then every branch's positions
        jup_kv_t* kv = kvs[b];
        if (!kv) return fail(JUP_EINVAL, "%s: kvs[%d] is NULL", me, b);
        if (!same_shape(stage->cfg, kv->cfg))
            return fail(JUP_EINVAL, "%s: kvs[%d] was made for another configuration", me, b);
        for (int a = 0; a < b; ++a) {
            if (kvs[a] == kv) return fail(JUP_EINVAL, "%s: kvs[%d] and kvs[%d] are the same cache", me, a, b);
            if (kvs[a]->parent == kv || kv->parent == kvs[a])
                return fail(JUP_EINVAL, "%s: kvs[%d] and kvs[%d] are parent and fork: one call would write positions "
                            "the other reads", me, a, b);
        }
    }
    for (int b = 0; b < n_branches; ++b) {
        jup_kv_t* kv = kvs[b];
        jup_status_t rc = jup_kv_check_append(kv, n_tokens, pos_offsets[b]);
        if (rc != JUP_OK) {
            char tmp[400];
            snprintf(tmp, sizeof(tmp), "%s", g_err);
            return fail(rc, "%s: branch %d: %s", me, b, tmp);
        }
        if (kv->parent && kv->parent->len < kv->n_shared)
            return fail(JUP_EPOS, "%s: branch %d: the parent cache holds %d positions, fewer than the %d shared", me, b,
                        kv->parent->len, kv->n_shared);
    }
    const long rows = (long)n_branches * n_tokens;
    if (rows > stage->max_chunk_tokens)
        return fail(JUP_ECAP, "%s: %d branches x %d tokens exceed the stage's max_chunk_tokens=%d", me, n_branches,
                    n_tokens, stage->max_chunk_tokens);
    if (n_tokens == 0) {
        for (int b = 0; b < n_branches; ++b) kvs[b]->len = pos_offsets[b];
        return JUP_OK;
    }
    if (!hidden_in || !hidden_out) return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must not be NULL", me);
    if (stage->cfg.dtype != JUP_F32 && (misaligned16(hidden_in) || misaligned16(hidden_out)))
        return fail(JUP_EINVAL, "%s: hidden_in and hidden_out must be 16-byte aligned", me);

    hipStream_t s = (hipStream_t)stream;
    hipError_t e = hipSuccess;
    if (stage->cfg.dtype == JUP_F32) {
        // check mode: one branch after the other (it exists to be compared with, not to be fast)
        const size_t row_elems = (size_t)n_tokens * stage->cfg.d_model;
        for (int b = 0; b < n_branches && e == hipSuccess; ++b)
            e = jup::f32_forward(*stage, (const float*)hidden_in + b * row_elems, n_tokens, pos_offsets[b],
                                 view_of(kvs[b]), (float*)hidden_out + b * row_elems, s);
    } else {
        jup::BranchTable bt{};
        bt.n_branches = n_branches;
        bt.n_tok = n_tokens;
        for (int b = 0; b < n_branches; ++b) {
            bt.pos0[b] = pos_offsets[b];
            bt.kv[b] = view_of(kvs[b]);
        }
        e = jup::bf16_forward(*stage, hidden_in, (int)rows, 0, jup::KvView{}, hidden_out, s, &bt);
    }
    if (e != hipSuccess) return fail(JUP_EDEVICE, "%s: %s", me, hipGetErrorString(e));
    for (int b = 0; b < n_branches; ++b) kvs[b]->len = pos_offsets[b] + n_tokens;
    return JUP_OK;
}

}  // extern "C"
