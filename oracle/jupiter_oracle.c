/*
 * Jupiter stage oracle -- TEST INFRASTRUCTURE, not a product path.
 *
 * A plain, slow CPU statement of what one pipeline stage computes for one
 * prompt sub-sequence (Sec. IV-A.2 of the Jupiter paper: the prompt is split
 * into consecutive sub-sequences s_1..s_M that are injected one after the
 * other; when s_i is processed the stage reuses what it cached for
 * s_1..s_{i-1}).  The decoder layer is the one of Sec. II-A -- QKV project,
 * masked multi-head attention with its final linear layer, feed-forward
 * network, KVCache -- in the Llama-2 form the paper evaluates (Sec. V-A):
 * pre-norm RMSNorm, rotary position embedding with half-split pairing,
 * SwiGLU feed-forward, no biases, one KV head per query head.
 *
 * Only tests, the smoke check and the benchmark's cpu_baseline leg may call
 * this file.  It shares no code, header, table or helper with the HIP path.
 *
 * Precision: every tensor is stored as fp32; every reduction (dot products,
 * sums of squares, softmax sums, weighted value sums) accumulates in fp64 and
 * every transcendental (exp, sin, cos, pow, sqrt) is evaluated in fp64; a
 * result is rounded to fp32 once, when it is stored.
 *
 * Loop structure: textbook triple loops, two-pass softmax; no blocking, no
 * fusion.  OpenMP only distributes independent output elements over threads.
 *
 * KV cache layout (mirrors the contract of the library under test so that
 * positions can be compared slot by slot):
 *     kv[layer][which][head][position][i],  which: 0 = K (after RoPE), 1 = V
 *     element index = (((layer*2 + which)*n_heads + head)*max_positions
 *                      + position)*head_dim + i
 *
 * Token-tree variant (Sec. V-A: the candidate tokens of a speculative step are
 * verified in one forward pass; the paper evaluates with the token tree of
 * Medusa): the sub-sequence is a forest given by parents[t] in {-1, 0..t-1};
 * token t is stored at slot pos_offset + t, is rotated at position
 * pos_offset + depth(t) and sees the earlier sub-sequences, its ancestors and
 * itself.  A chain (parents[t] = t-1) is the ordinary sub-sequence.
 *
 * Pins (tests/test_oracle_*.py): an independent library decoder (Hugging Face
 * Llama layers with a DynamicCache, fp64, CPU), torch's scaled-dot-product
 * attention / rms_norm / silu, closed forms (uniform softmax -> running mean,
 * one-hot softmax, position-0 RoPE identity, constant-vector RMSNorm), the
 * relative-position invariance of RoPE scores, and brute force over every
 * composition of a short prompt against oracle/bruteforce.py.  Tree variant:
 * the same library decoder driven with an explicit ancestor mask and depth
 * positions, and the path property (a node's output is the last row of the
 * ordinary call on its root-to-node path).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { W_Q = 0, W_K, W_V, W_O, W_GATE, W_UP, W_DOWN, G_ATTN, G_MLP, W_PER_LAYER };

/* fp64-accumulated inner product of two fp32 vectors. */
static double dotd(const float *a, const float *b, int n)
{
    double acc = 0.0;
#pragma omp simd reduction(+ : acc)
    for (int i = 0; i < n; ++i)
        acc += (double)a[i] * (double)b[i];
    return acc;
}

/* y[t][j] = sum_k x[t][k] * w[j][k]   (x: [n,k_dim], w: [out,k_dim], y: [n,out]) */
static void linear_nt(const float *x, const float *w, float *y, int n, int out, int k_dim)
{
#pragma omp parallel for schedule(static)
    for (int j = 0; j < out; ++j)
        for (int t = 0; t < n; ++t)
            y[(size_t)t * out + j] = (float)dotd(x + (size_t)t * k_dim, w + (size_t)j * k_dim, k_dim);
}

/* RMSNorm of each row: y_j = x_j * g_j / sqrt(mean_i x_i^2 + eps). */
static void rmsnorm_rows(const float *x, const float *g, float *y, int n, int d, double eps)
{
#pragma omp parallel for schedule(static)
    for (int t = 0; t < n; ++t) {
        const float *xr = x + (size_t)t * d;
        double ss = 0.0;
        for (int i = 0; i < d; ++i)
            ss += (double)xr[i] * (double)xr[i];
        double inv = 1.0 / sqrt(ss / (double)d + eps);
        for (int j = 0; j < d; ++j)
            y[(size_t)t * d + j] = (float)((double)xr[j] * inv * (double)g[j]);
    }
}

/*
 * Rotary embedding of one head vector v[0..dh) at absolute position pos:
 * pair (i, i + dh/2) is rotated by the angle pos * theta^(-2i/dh).
 */
static void rope_head(float *v, int dh, int64_t pos, double theta)
{
    int half = dh / 2;
    for (int i = 0; i < half; ++i) {
        double ang = (double)pos * pow(theta, -2.0 * (double)i / (double)dh);
        double c = cos(ang), s = sin(ang);
        double a = (double)v[i], b = (double)v[i + half];
        v[i] = (float)(a * c - b * s);
        v[i + half] = (float)(b * c + a * s);
    }
}

static size_t kv_index(int layer, int which, int head, int pos, int n_heads, int max_positions, int dh)
{
    return ((((size_t)layer * 2 + (size_t)which) * (size_t)n_heads + (size_t)head) * (size_t)max_positions +
            (size_t)pos) *
           (size_t)dh;
}

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/*
 * One stage forward over one sub-sequence (Sec. IV-A.2); with parents != NULL over the token
 * tree of a speculative step (Sec. V-A), see oracle_stage_prefill_tree below.
 *
 *   weights     [n_layers * 9] host pointers, per layer in the order
 *               wq, wk, wv, wo ([d,d]), w_gate, w_up ([f,d]), w_down ([d,f]),
 *               g_attn, g_mlp ([d]); matrices row-major [out_features, in_features]
 *   hidden_in   [n_tokens, d] hidden states of the sub-sequence
 *   pos_offset  number of tokens of the earlier sub-sequences; their keys and
 *               values must already be in kv at positions 0..pos_offset-1
 *   kv          cache in the layout given at the top; slots
 *               [pos_offset, pos_offset+n_tokens) of every layer/head are written
 *   hidden_out  [n_tokens, d]
 *
 * Returns 0, or -1 for inconsistent sizes, -2 when the cache is too small,
 * -3 when memory for the intermediates cannot be obtained.
 */
static int stage_forward(int n_layers, int d, int n_heads, int dh, int f, double rms_eps, double rope_theta,
                         const float *const *weights, const float *hidden_in, int n_tokens, int pos_offset,
                         const int32_t *parents, float *kv, int max_positions, float *hidden_out)
{
    if (n_layers < 0 || d <= 0 || n_heads <= 0 || dh <= 0 || f <= 0 || d != n_heads * dh || (dh & 1) ||
        n_tokens < 0 || pos_offset < 0)
        return -1;
    if ((int64_t)pos_offset + n_tokens > max_positions)
        return -2;
    if (n_tokens == 0)
        return 0;
    if (parents)
        for (int t = 0; t < n_tokens; ++t)
            if (parents[t] < -1 || parents[t] >= t)
                return -1;

    const int n = n_tokens;
    const size_t nd = (size_t)n * d, nf = (size_t)n * f;
    float *x = malloc(nd * sizeof(float));    /* residual stream entering the layer */
    float *xn = malloc(nd * sizeof(float));   /* normalised rows */
    float *q = malloc(nd * sizeof(float));
    float *k = malloc(nd * sizeof(float));
    float *v = malloc(nd * sizeof(float));
    float *o = malloc(nd * sizeof(float));    /* attention output, heads concatenated */
    float *proj = malloc(nd * sizeof(float)); /* output of wo / w_down */
    float *h = malloc(nd * sizeof(float));    /* residual stream after attention */
    float *gate = malloc(nf * sizeof(float));
    float *up = malloc(nf * sizeof(float));
    /*
     * depth[t]: number of ancestors of token t inside this sub-sequence (t itself for a chain).
     * sees[t*n + j] = 1 when token t attends to token j of this sub-sequence: j is t or an ancestor of t.
     */
    int *depth = malloc((size_t)n * sizeof(int));
    unsigned char *sees = calloc((size_t)n * n, 1);
    int rc = 0;
    if (!x || !xn || !q || !k || !v || !o || !proj || !h || !gate || !up || !depth || !sees) {
        rc = -3;
        goto done;
    }
    memcpy(x, hidden_in, nd * sizeof(float));
    for (int t = 0; t < n; ++t) {
        const int par = parents ? parents[t] : t - 1;
        depth[t] = par < 0 ? 0 : depth[par] + 1;
        for (int a = t; a >= 0; a = parents ? parents[a] : a - 1)
            sees[(size_t)t * n + a] = 1;
    }

    for (int l = 0; l < n_layers; ++l) {
        const float *const *w = weights + (size_t)l * W_PER_LAYER;

        /* QKV project on the normalised sub-sequence (depends on this sub-sequence only). */
        rmsnorm_rows(x, w[G_ATTN], xn, n, d, rms_eps);
        linear_nt(xn, w[W_Q], q, n, d, d);
        linear_nt(xn, w[W_K], k, n, d, d);
        linear_nt(xn, w[W_V], v, n, d, d);

        /*
         * Rotary embedding at absolute positions (earlier tokens + own depth), then store K and V
         * in the cache slot of the token (earlier tokens + own index).
         */
#pragma omp parallel for collapse(2) schedule(static)
        for (int t = 0; t < n; ++t)
            for (int hh = 0; hh < n_heads; ++hh) {
                const int64_t pos = (int64_t)pos_offset + depth[t];
                const int slot = pos_offset + t;
                rope_head(q + (size_t)t * d + (size_t)hh * dh, dh, pos, rope_theta);
                rope_head(k + (size_t)t * d + (size_t)hh * dh, dh, pos, rope_theta);
                memcpy(kv + kv_index(l, 0, hh, slot, n_heads, max_positions, dh),
                       k + (size_t)t * d + (size_t)hh * dh, (size_t)dh * sizeof(float));
                memcpy(kv + kv_index(l, 1, hh, slot, n_heads, max_positions, dh),
                       v + (size_t)t * d + (size_t)hh * dh, (size_t)dh * sizeof(float));
            }

        /*
         * Masked attention: a query sees every cached slot of the earlier sub-sequences and, of
         * this sub-sequence, the slots of the tokens marked in `sees` (for a chain: slots 0..P of
         * the query at absolute position P).
         */
        const double scale = 1.0 / sqrt((double)dh);
#pragma omp parallel for collapse(2) schedule(dynamic, 4)
        for (int hh = 0; hh < n_heads; ++hh)
            for (int t = 0; t < n; ++t) {
                int *vis = malloc((size_t)(pos_offset + t + 1) * sizeof(int)); /* visible slots, ascending */
                int n_keys = 0;
                for (int j = 0; j < pos_offset; ++j)
                    vis[n_keys++] = j;
                for (int j = 0; j <= t; ++j)
                    if (sees[(size_t)t * n + j])
                        vis[n_keys++] = pos_offset + j;
                const float *qv = q + (size_t)t * d + (size_t)hh * dh;
                const float *kc = kv + kv_index(l, 0, hh, 0, n_heads, max_positions, dh);
                const float *vc = kv + kv_index(l, 1, hh, 0, n_heads, max_positions, dh);
                double *p = malloc((size_t)n_keys * sizeof(double));
                double *acc = calloc((size_t)dh, sizeof(double));
                double m = -INFINITY, z = 0.0;
                for (int j = 0; j < n_keys; ++j) {
                    p[j] = dotd(qv, kc + (size_t)vis[j] * dh, dh) * scale;
                    if (p[j] > m)
                        m = p[j];
                }
                for (int j = 0; j < n_keys; ++j) {
                    p[j] = exp(p[j] - m);
                    z += p[j];
                }
                for (int j = 0; j < n_keys; ++j) {
                    const double wj = p[j] / z;
                    const float *vj = vc + (size_t)vis[j] * dh;
                    for (int i = 0; i < dh; ++i)
                        acc[i] += wj * (double)vj[i];
                }
                for (int i = 0; i < dh; ++i)
                    o[(size_t)t * d + (size_t)hh * dh + i] = (float)acc[i];
                free(p);
                free(acc);
                free(vis);
            }

        /* Final linear layer of the attention block, residual. */
        linear_nt(o, w[W_O], proj, n, d, d);
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nd; ++i)
            h[i] = (float)((double)x[i] + (double)proj[i]);

        /* Feed-forward network (SwiGLU), residual. */
        rmsnorm_rows(h, w[G_MLP], xn, n, d, rms_eps);
        linear_nt(xn, w[W_GATE], gate, n, f, d);
        linear_nt(xn, w[W_UP], up, n, f, d);
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nf; ++i) {
            double g = (double)gate[i];
            gate[i] = (float)(g / (1.0 + exp(-g)) * (double)up[i]);
        }
        linear_nt(gate, w[W_DOWN], proj, n, d, f);
#pragma omp parallel for schedule(static)
        for (size_t i = 0; i < nd; ++i)
            x[i] = (float)((double)h[i] + (double)proj[i]);
    }
    memcpy(hidden_out, x, nd * sizeof(float));

done:
    free(x);
    free(xn);
    free(q);
    free(k);
    free(v);
    free(o);
    free(proj);
    free(h);
    free(gate);
    free(up);
    free(depth);
    free(sees);
    return rc;
}

int oracle_stage_prefill_chunk(int n_layers, int d, int n_heads, int dh, int f, double rms_eps, double rope_theta,
                               const float *const *weights, const float *hidden_in, int n_tokens, int pos_offset,
                               float *kv, int max_positions, float *hidden_out)
{
    return stage_forward(n_layers, d, n_heads, dh, f, rms_eps, rope_theta, weights, hidden_in, n_tokens, pos_offset,
                         NULL, kv, max_positions, hidden_out);
}

/*
 * One stage forward over the candidate tokens of a speculative step (Sec. V-A), arranged as a
 * token tree: parents[t] is the index of token t's parent inside this call, or -1 when t follows
 * the last earlier token directly; parents[t] < t.  Slots, positions and visibility as described
 * at the top of the file.  Returns as oracle_stage_prefill_chunk; -1 also for a parent index
 * outside [-1, t).
 */
int oracle_stage_prefill_tree(int n_layers, int d, int n_heads, int dh, int f, double rms_eps, double rope_theta,
                              const float *const *weights, const float *hidden_in, int n_tokens, int pos_offset,
                              const int32_t *parents, float *kv, int max_positions, float *hidden_out)
{
    if (!parents)
        return -1;
    return stage_forward(n_layers, d, n_heads, dh, f, rms_eps, rope_theta, weights, hidden_in, n_tokens, pos_offset,
                         parents, kv, max_positions, hidden_out);
}

/*
 * Single-step helpers, exported so that tests can pin each formula on its own
 * against closed forms and library routines.  They are the same static
 * functions the stage routine calls.
 */
void oracle_rmsnorm(const float *x, const float *g, float *y, int n, int d, double eps)
{
    rmsnorm_rows(x, g, y, n, d, eps);
}

void oracle_rope(float *v, int n_vec, int dh, const int64_t *pos, double theta)
{
    for (int r = 0; r < n_vec; ++r)
        rope_head(v + (size_t)r * dh, dh, pos[r], theta);
}

void oracle_linear_nt(const float *x, const float *w, float *y, int n, int out, int k_dim)
{
    linear_nt(x, w, y, n, out, k_dim);
}
