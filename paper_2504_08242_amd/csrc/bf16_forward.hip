// Orchestration of the bf16 (matrix-core) path: one stage forward over one sub-sequence with its
// cached prefix (Jupiter paper, Sec. IV-A.2); decoder layer of Sec. II-A in its Llama-2 form.
//
// Per layer, seven launches on one stream (the caller's, or a lane's stream of the overlapped multi-chunk call):
//   reduce+norm  ->  QKV GEMM (+ rotary + KV append)  ->  chunk attention  ->  O GEMM (K-split partials)
//   ->  reduce+norm  ->  gate/up GEMM (+ SwiGLU)  ->  down GEMM (K-split partials)
// The projections back to d_model are too narrow to fill 256 CUs with tall tiles, so they split K and
// write fp32 partial tiles; the next reduce+norm pass adds them to the fp32 residual stream in a fixed
// order (bitwise reproducible) on its way to the normalised bf16 rows it has to produce anyway.
#include "bf16_common.h"

namespace jup {

hipError_t bf16_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s) {
    const jup_stage_config_t& c = st.cfg;
    const size_t d = c.d_model;
    hipError_t e = gemm_configure();
    if (e == hipSuccess) e = attention_configure();
    if (e != hipSuccess) return e;
    for (int l = 0; l < c.n_layers; ++l) {
        char* base = (char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const jup_layer_weights_t& w = layers[l];
        launch_pack_qkv((u16*)(base + st.pl.wqkv), (const u16*)w.wq, (const u16*)w.wk, (const u16*)w.wv, c.d_model, s);
        launch_pack_gate_up((u16*)(base + st.pl.wgu), (const u16*)w.w_gate, (const u16*)w.w_up, c.d_model, c.d_ffn, s);
        launch_pack_plain((u16*)(base + st.pl.wo), (const u16*)w.wo, c.d_model, c.d_model, s);
        launch_pack_plain((u16*)(base + st.pl.wdown), (const u16*)w.w_down, c.d_model, c.d_ffn, s);
        e = hipMemcpyAsync(base + st.pl.g_attn, w.g_attn, d * 2, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(base + st.pl.g_mlp, w.g_mlp, d * 2, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// 4-bit stage: codes and scales of the seven matrices go into their packed layouts (w4_gemm.hip); gains as above.
// A stage created with w4_expanded also gets their bf16 values in the layouts of the bf16 stage.
hipError_t w4_pack_weights(const jup_stage& st, const jup_layer_weights_t* layers, hipStream_t s) {
    const jup_stage_config_t& c = st.cfg;
    const size_t d = c.d_model;
    hipError_t e = attention_configure();
    if (e == hipSuccess && c.w4_expanded) e = gemm_configure();
    if (e != hipSuccess) return e;
    for (int l = 0; l < c.n_layers; ++l) {
        char* base = (char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const jup_layer_weights_t& w = layers[l];
        launch_pack_w4_qkv((unsigned char*)(base + st.pl.wqkv), (float*)(base + st.pl.sqkv), w.wq, w.wk, w.wv, w.sq, w.sk,
                           w.sv, c.d_model, s);
        launch_pack_w4_gate_up((unsigned char*)(base + st.pl.wgu), (float*)(base + st.pl.sgu), w.w_gate, w.w_up, w.s_gate,
                               w.s_up, c.d_model, c.d_ffn, s);
        launch_pack_w4_plain((unsigned char*)(base + st.pl.wo), (float*)(base + st.pl.so), w.wo, w.so, c.d_model,
                             c.d_model, s);
        launch_pack_w4_plain((unsigned char*)(base + st.pl.wdown), (float*)(base + st.pl.sdown), w.w_down, w.s_down,
                             c.d_model, c.d_ffn, s);
        if (c.w4_expanded) {
            launch_expand_qkv((u16*)(base + st.pl.xqkv), w.wq, w.wk, w.wv, w.sq, w.sk, w.sv, c.d_model, s);
            launch_expand_gate_up((u16*)(base + st.pl.xgu), w.w_gate, w.w_up, w.s_gate, w.s_up, c.d_model, c.d_ffn, s);
            launch_expand_plain((u16*)(base + st.pl.xo), w.wo, w.so, c.d_model, c.d_model, s);
            launch_expand_plain((u16*)(base + st.pl.xdown), w.w_down, w.s_down, c.d_model, c.d_ffn, s);
        }
        e = hipMemcpyAsync(base + st.pl.g_attn, w.g_attn, d * 2, hipMemcpyDeviceToDevice, s);
        if (e == hipSuccess) e = hipMemcpyAsync(base + st.pl.g_mlp, w.g_mlp, d * 2, hipMemcpyDeviceToDevice, s);
        if (e != hipSuccess) return e;
    }
    return hipGetLastError();
}

// bt == nullptr: one chunk of n tokens at position pos of cache kv.
// bt != nullptr: bt->n_branches chunks of bt->n_tok tokens each, n = their total number of rows; the rows of
// branch b are appended to and attend over cache bt->kv[b] from position bt->pos0[b] (pos and kv are unused).
// Everything that is not attention or cache traffic sees one [n, d] activation matrix either way, so the
// stage's weights are streamed once for all branches.
// link != nullptr: scratch buffer and cross-stream events of a chunk that overlaps with its neighbours.
// tree != nullptr (host table, bt == nullptr): the n tokens are a token tree; only the rotary positions
// (pos + depth) and the mask inside the chunk differ from an ordinary chunk.
hipError_t bf16_forward(const jup_stage& st, const void* hidden_in, int n, int pos, const KvView& kv,
                        void* hidden_out, hipStream_t s, const BranchTable* bt, const TreeTable* tree,
                        const ChunkLink* link) {
    const jup_stage_config_t& c = st.cfg;
    const int d = c.d_model, f = c.d_ffn, H = c.n_heads;
    char* ws = (char*)(link && link->workspace ? link->workspace : st.workspace);
    float* x32 = (float*)(ws + st.wl.x32);
    u16* xn = (u16*)(ws + st.wl.xn);
    u16* q = (u16*)(ws + st.wl.q);
    u16* o = (u16*)(ws + st.wl.o);
    u16* act = (u16*)(ws + st.wl.act);
    float* partial = (float*)(ws + st.wl.partial);
    float2* rope = (float2*)(ws + st.wl.rope);
    const size_t split_stride = (size_t)n * d;

    if (c.n_layers == 0) return hipMemcpyAsync(hidden_out, hidden_in, (size_t)n * d * 2, hipMemcpyDeviceToDevice, s);
    const BranchTable* bt_dev = nullptr;
    const TreeTable* tree_dev = nullptr;
    // the first kernel of the call builds the rotary table and clears the arrival counters of the call's split launches
    const AttScratch att{(float*)(ws + st.wl.att_split), (int*)(ws + st.wl.att_count), st.wl.att_split_rows,
                         st.wl.att_count_n};
    const int n_zero = (int)att.counters;
    int max_keys = 0;  // batched branches: the longest key range
    if (bt) {
        bt_dev = (const BranchTable*)(ws + st.wl.branches);
        launch_write_branch_table(*bt, (BranchTable*)(ws + st.wl.branches), s);
        launch_rope_table_branches(rope, n, bt_dev, c.rope_theta, att.split_count, n_zero, s);
        for (int b = 0; b < bt->n_branches; ++b) max_keys = bt->pos0[b] + bt->n_tok > max_keys ? bt->pos0[b] + bt->n_tok : max_keys;
    } else if (tree) {
        tree_dev = (const TreeTable*)(ws + st.wl.tree);
        launch_write_tree_table(*tree, (TreeTable*)(ws + st.wl.tree), s);
        launch_rope_table_tree(rope, n, pos, tree_dev, c.rope_theta, att.split_count, n_zero, s);
    } else {
        launch_rope_table(rope, n, pos, c.rope_theta, att.split_count, n_zero, s);
    }

    const bool shared = link != nullptr;  // other chunks' kernels run beside this chunk's
    // 4-bit stage: the projections read codes, everything else is the bf16 path.  With the expanded copy at hand,
    // chunks beyond one pass of the 4-bit kernels (64 rows) take the bf16 projections on it.
    const bool expanded = c.dtype == JUP_BF16_W4 && c.w4_expanded && n > 64;
    const bool w4 = c.dtype == JUP_BF16_W4 && !expanded;
    const size_t wqkv = expanded ? st.pl.xqkv : st.pl.wqkv, wo = expanded ? st.pl.xo : st.pl.wo;
    const size_t wgu = expanded ? st.pl.xgu : st.pl.wgu, wdown = expanded ? st.pl.xdown : st.pl.wdown;
    const int splits_o = w4 ? w4_plan_splits(d, d) : gemm_plan_splits(n, d, d, shared);
    const int splits_down = w4 ? w4_plan_splits(d, f) : gemm_plan_splits(n, d, f, shared);
    hipError_t e = hipSuccess;
    for (int l = 0; l < c.n_layers && e == hipSuccess; ++l) {
        const char* wb = (const char*)st.packed + (size_t)l * st.pl.layer_bytes;
        const u16* g1 = (const u16*)(wb + st.pl.g_attn);
        const u16* g2 = (const u16*)(wb + st.pl.g_mlp);
        {
            TraceScope ts(st, JUP_K_RMSNORM, s);
            if (l == 0)
                launch_reduce_norm(x32, (const u16*)hidden_in, nullptr, 0, 0, g1, xn, nullptr, n, d, c.rms_eps, s);
            else
                launch_reduce_norm(x32, nullptr, partial, splits_down, split_stride, g1, xn, nullptr, n, d, c.rms_eps,
                                   s);
        }
        {
            TraceScope ts(st, JUP_K_GEMM_QKV, s);
            GemmArgs a{};
            a.A = xn; a.W = (const u16*)(wb + wqkv); a.M = n; a.N = 3 * d; a.K = d;
            a.q_out = q; a.rope = rope; a.kv = kv; a.layer = l; a.n_heads = H; a.d_model = d; a.pos0 = pos;
            a.branches = bt_dev;
            a.shared_gpu = shared;
            a.w_scale = (const float*)(wb + st.pl.sqkv);
            e = w4 ? launch_gemm_w4(EPI_QKV, a, s) : launch_gemm_qkv(a, s);
        }
        // keys and values of this layer are in the cache: the next chunk may attend to them; this chunk needs
        // those of the chunk before it
        if (link && link->record_qkv && e == hipSuccess) e = hipEventRecord(link->record_qkv[l], s);
        for (int w = 0; link && w < link->n_wait && e == hipSuccess; ++w) e = hipStreamWaitEvent(s, link->wait_qkv[w][l], 0);
        {
            TraceScope ts(st, JUP_K_ATTENTION, s);
            if (e != hipSuccess) break;
            if (bt) e = launch_branch_attention(q, o, bt->n_tok, bt->n_branches, d, H, bt_dev, max_keys, l, s, att);
            else e = launch_chunk_attention(q, o, n, d, H, pos, kv, l, s, att, tree_dev, shared);
        }
        {
            TraceScope ts(st, JUP_K_GEMM_O, s);
            GemmArgs a{};
            a.A = o; a.W = (const u16*)(wb + wo); a.M = n; a.N = d; a.K = d; a.partial = partial; a.shared_gpu = shared;
            a.w_scale = (const float*)(wb + st.pl.so);
            if (e == hipSuccess) e = w4 ? launch_gemm_w4(EPI_PARTIAL, a, s) : launch_gemm_partial(a, s);
        }
        {
            TraceScope ts(st, JUP_K_RMSNORM, s);
            launch_reduce_norm(x32, nullptr, partial, splits_o, split_stride, g2, xn, nullptr, n, d, c.rms_eps, s);
        }
        {
            TraceScope ts(st, JUP_K_GEMM_GATE_UP, s);
            GemmArgs a{};
            a.A = xn; a.W = (const u16*)(wb + wgu); a.M = n; a.N = 2 * f; a.K = d; a.act = act; a.shared_gpu = shared;
            a.w_scale = (const float*)(wb + st.pl.sgu);
            if (e == hipSuccess) e = w4 ? launch_gemm_w4(EPI_SWIGLU, a, s) : launch_gemm_swiglu(a, s);
        }
        {
            TraceScope ts(st, JUP_K_GEMM_DOWN, s);
            GemmArgs a{};
            a.A = act; a.W = (const u16*)(wb + wdown); a.M = n; a.N = d; a.K = f; a.partial = partial; a.shared_gpu = shared;
            a.w_scale = (const float*)(wb + st.pl.sdown);
            if (e == hipSuccess) e = w4 ? launch_gemm_w4(EPI_PARTIAL, a, s) : launch_gemm_partial(a, s);
        }
    }
    if (e != hipSuccess) return e;
    // last layer's down-projection partials + residual -> hidden_out
    launch_reduce_norm(x32, nullptr, partial, splits_down, split_stride, nullptr, nullptr, (u16*)hidden_out, n, d,
                       c.rms_eps, s);
    return hipGetLastError();
}

}  // namespace jup
