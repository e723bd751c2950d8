/*
 * jupiter_stage.h -- C ABI of the MI355X (gfx950) stage kernel of Jupiter's
 * intra-sequence pipeline parallelism.
 *
 * What the library computes.  A *stage* is a contiguous run of decoder layers
 * held by one device (Jupiter paper, Sec. IV-A.1).  A prompt is cut into
 * consecutive sub-sequences ("chunks") that are injected one after the other;
 * when chunk s_i is processed, the stage reuses what it cached for
 * s_1..s_{i-1}, which the causal mask makes sufficient (Sec. IV-A.2).  One call
 * of jup_stage_prefill_chunk() is one stage forward over one chunk, i.e. one
 * evaluation of the paper's latency function q(x, y) with x = n_tokens and
 * y = pos_offset (Sec. IV-B.2).  Per layer it does, in the order of the decoder
 * layer of Sec. II-A and in the Llama-2 form the paper evaluates (Sec. V-A):
 *
 *   1. RMSNorm of the chunk's hidden states, QKV projection (no bias)
 *   2. rotary embedding of Q and K at absolute positions pos_offset + t
 *      (pairs (i, i + head_dim/2), angle pos * theta^(-2i/head_dim))
 *   3. K (after the rotation) and V appended to the KV cache at slots
 *      [pos_offset, pos_offset + n_tokens)
 *   4. causal attention of the chunk's queries over the cached prefix
 *      0..pos_offset-1 plus the causal triangle inside the chunk (a token sees
 *      itself), scale 1/sqrt(head_dim)
 *   5. output projection, residual
 *   6. RMSNorm, SwiGLU feed-forward  silu(x Wg^T) * (x Wu^T) Wd^T, residual
 *
 * Decode-sized chunks (speculative verification, Sec. V-A; outline branches
 * that share the prompt's cache, Sec. V-B) are the same call with a small
 * n_tokens, on a cache made with jup_kv_fork() and rolled back with
 * jup_kv_truncate().
 *
 * Conventions
 *   - All tensor pointers are DEVICE pointers unless a comment says host.
 *     The library never allocates or frees device memory: every buffer,
 *     including its own packed weights and workspace, is provided by the caller
 *     (normally through PyTorch) and is borrowed until the handle is destroyed.
 *   - Matrices are row-major.  Weights are [out_features, in_features].  With the bfloat16 dtypes (JUP_BF16,
 *     JUP_BF16_W4) every weight, gain and hidden-state pointer must be 16-byte aligned (rows are read and
 *     written 16 bytes at a time); a misaligned one is JUP_EINVAL.
 *   - dtype JUP_BF16: hidden states, weights, gains and the KV cache are
 *     bfloat16; products accumulate in fp32 on the matrix cores and the residual
 *     stream is kept in fp32 inside a call.  dtype JUP_F32 ("check mode"): the
 *     same mathematics with fp32 storage and fp32 arithmetic throughout, on
 *     plain (non matrix-core) kernels; it exists to pin indexing and semantics.
 *   - dtype JUP_BF16_W4: as JUP_BF16, except that the seven projection matrices of a layer are given as
 *     4-bit codes with group-wise fp32 scales (the paper evaluates INT4 models, Sec. VI-A; it names no
 *     scheme, this is the library's): W[n][k] = scale[n][k / 128] * (code[n][k] - 8), codes 0..15 stored two
 *     per byte, row-major [out_features, in_features / 2], the low four bits of a byte holding the even k.
 *     Hidden states, gains and the KV cache stay bfloat16 (a cache made for a JUP_BF16 configuration of the
 *     same shape serves a JUP_BF16_W4 stage and vice versa).  The kernels behind it are built for decode-sized
 *     chunks (Sec. V), which are bound by streaming the weights: up to 16 tokens stream every matrix once;
 *     longer chunks are accepted and computed 16 rows at a time, re-reading the codes for every 16 rows.
 *   - Calls validate their arguments on the host before anything is enqueued;
 *     on error nothing is enqueued, no state changes, and jup_last_error()
 *     holds a message.  Kernel work is asynchronous on the given HIP stream.
 *   - A stage owns one workspace: calls on the same stage must not overlap
 *     (issue them on one stream, or synchronise between streams).
 *   - The handles are host objects (malloc/free); they are not thread-safe.
 */
#ifndef JUPITER_STAGE_H
#define JUPITER_STAGE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Marks the exported entry points (the library is built with hidden visibility otherwise). */
#define JUP_API __attribute__((visibility("default")))

typedef struct jup_stage jup_stage_t; /* opaque, host object */
typedef struct jup_kv jup_kv_t;       /* opaque, host object */

typedef enum { JUP_F32 = 0, JUP_BF16 = 1, JUP_BF16_W4 = 2 } jup_dtype_t;

typedef enum {
    JUP_OK = 0,
    JUP_EINVAL = -1,  /* null pointer, inconsistent or unsupported sizes, too-small buffer */
    JUP_EPOS = -2,    /* pos_offset would leave a hole, or touches a shared (read-only) prefix */
    JUP_ECAP = -3,    /* chunk does not fit the cache's max_positions or the stage's max_chunk_tokens */
    JUP_EDEVICE = -4, /* a HIP call failed (no device, launch error) */
    JUP_ENOMEM = -5   /* host allocation of a handle failed */
} jup_status_t;

/*
 * Shape of a stage.  Requirements: d_model == n_heads * head_dim; head_dim even.
 * JUP_BF16 and JUP_BF16_W4 additionally require head_dim == 128, d_model % 256 == 0, d_model <= 8192 and
 * d_ffn % 128 == 0 (the matrix-core tilings); JUP_F32 accepts any sizes.
 */
typedef struct {
    int32_t n_layers;
    int32_t d_model;
    int32_t n_heads;
    int32_t head_dim;
    int32_t d_ffn;
    float rms_eps;    /* inside the square root: x / sqrt(mean(x^2) + eps) */
    float rope_theta; /* rotary base, 1e4 for Llama-2 */
    int32_t dtype;    /* jup_dtype_t */
    /*
     * JUP_BF16_W4 only (must be 0 otherwise): 1 = the stage also keeps bf16(scale * (code - 8)) of its seven
     * matrices, 2 more bytes per weight in `packed`.  Chunks of more than 64 rows then run the bf16 kernels on that
     * copy (they are bound by arithmetic, where 4-bit weights save nothing) and shorter ones stream the codes (they
     * are bound by reading the weights, Sec. V); with 0 the stage holds codes only and a longer chunk takes one pass
     * over the codes per 64 rows.  The expanded weights carry one more rounding to bf16 than the codes.
     */
    int32_t w4_expanded;
} jup_stage_config_t;

/*
 * One decoder layer's parameters; device pointers of the stage dtype (JUP_BF16_W4: the seven matrices are
 * uint8 [out_features, in_features / 2] code pairs, the gains bfloat16).
 */
typedef struct {
    const void *wq, *wk, *wv, *wo; /* [d_model, d_model] */
    const void *w_gate, *w_up;     /* [d_ffn, d_model]   */
    const void *w_down;            /* [d_model, d_ffn]   */
    const void *g_attn, *g_mlp;    /* [d_model] RMSNorm gains before attention / before the FFN */
    /* JUP_BF16_W4 only (ignored otherwise): fp32 scales [out_features, in_features / 128] of the matrices above */
    const float *sq, *sk, *sv, *so, *s_gate, *s_up, *s_down;
} jup_layer_weights_t;

/* ---- stage ---------------------------------------------------------------------------------- */

/* Bytes of device memory jup_stage_create() needs for its packed copy of the weights. 0 on bad cfg. */
JUP_API size_t jup_stage_packed_bytes(const jup_stage_config_t *cfg);

/* Bytes of device workspace for chunks of up to max_chunk_tokens tokens. 0 on bad arguments. */
JUP_API size_t jup_stage_workspace_bytes(const jup_stage_config_t *cfg, int32_t max_chunk_tokens);

/*
 * Builds a stage (Sec. IV-A.1: a stage model made of consecutive decoder layers).
 *   cfg, layers     host structs; layers[n_layers] hold device pointers
 *   packed          device buffer of >= jup_stage_packed_bytes(cfg) bytes, 256-byte aligned.  The
 *                   weights are copied into it in the layout the kernels read (Q/K/V rows fused,
 *                   gate/up rows interleaved); the copy kernels are enqueued on `stream`, and once
 *                   they have run the caller's originals are no longer referenced.
 *   workspace       device buffer of >= jup_stage_workspace_bytes(cfg, max_chunk_tokens) bytes,
 *                   256-byte aligned; contents are scratch.
 *   stream          hipStream_t (NULL = the default stream)
 * Errors: JUP_EINVAL (null pointer, bad shape, small buffer), JUP_ENOMEM, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_stage_create(const jup_stage_config_t *cfg, const jup_layer_weights_t *layers, void *packed,
                              size_t packed_bytes, void *workspace, size_t workspace_bytes,
                              int32_t max_chunk_tokens, void *stream, jup_stage_t **out);

/* Frees the host object only. NULL is allowed. */
JUP_API void jup_stage_destroy(jup_stage_t *stage);

/* ---- KV cache ------------------------------------------------------------------------------- */

/*
 * KV cache contract (Sec. II-A item 4, Sec. II-B: keys and values of all previous tokens, stored
 * per decoder layer and reused without recomputation).  A cache of max_positions slots is one
 * device buffer of elements of the stage dtype laid out as
 *
 *     kv[layer][which][head][position][i]      which: 0 = K after the rotation, 1 = V
 *     element index = (((layer*2 + which)*n_heads + head)*max_positions + position)*head_dim + i
 *
 * A call for a chunk at pos_offset writes exactly the slots [pos_offset, pos_offset + n_tokens) of
 * every (layer, which, head) and nothing else.
 */
JUP_API size_t jup_kv_bytes(const jup_stage_config_t *cfg, int32_t max_positions);

/* Wraps a caller-provided device buffer (>= jup_kv_bytes, 256-byte aligned); length starts at 0. */
JUP_API jup_status_t jup_kv_create(const jup_stage_config_t *cfg, int32_t max_positions, void *device_buf,
                           size_t device_bytes, jup_kv_t **out);

/*
 * A cache that shares the first n_shared positions of `parent` read-only (Sec. V-B: the prompt's
 * KVCache is shared across all point-extending requests) and owns positions
 * [n_shared, max_positions).  Its buffer uses the layout above with max_positions replaced by
 * (max_positions - n_shared) and position replaced by (position - n_shared).
 * Requirements: parent is not itself a fork; 0 <= n_shared <= jup_kv_len(parent);
 * max_positions > n_shared.  The fork starts with length n_shared.  The parent must outlive the
 * fork, and while forks exist it must not be truncated below n_shared (calls that would do so
 * return JUP_EPOS).
 */
JUP_API size_t jup_kv_fork_bytes(const jup_kv_t *parent, int32_t n_shared, int32_t max_positions);
JUP_API jup_status_t jup_kv_fork(jup_kv_t *parent, int32_t n_shared, int32_t max_positions, void *device_buf,
                         size_t device_bytes, jup_kv_t **out);

/* Length back to 0 (to n_shared for a fork). Device memory is not touched.
 * JUP_EPOS if live forks share positions of this cache. */
JUP_API jup_status_t jup_kv_reset(jup_kv_t *kv);

/*
 * Drops positions >= new_len (Sec. V-A step 5: rejected candidate tokens are removed from the
 * KVCache).  JUP_EPOS if new_len > length, < 0, below a fork's shared prefix, or below the
 * n_shared of a live fork of this cache.
 */
JUP_API jup_status_t jup_kv_truncate(jup_kv_t *kv, int32_t new_len);

/*
 * Removal of rejected candidates after a token-tree step (Sec. V-A step 5; see jup_stage_prefill_tree()):
 * the cache keeps its first base_len entries and, behind them, the n_keep entries that sat at
 * base_len + slots[0], base_len + slots[1], ... (moved to base_len, base_len + 1, ...); all others are
 * dropped and the length becomes base_len + n_keep.  For the accepted root-to-node path of a tree
 * (slots = the path's token indices) the moved keys are already rotated for their new positions, so the
 * cache is then exactly the one an ordinary call on the accepted tokens would have left.
 *   slots   HOST array [n_keep], strictly increasing, 0 <= slots[j], base_len + slots[j] < length;
 *           0 <= n_keep <= JUP_MAX_TREE_TOKENS
 *   stream  hipStream_t the copies are enqueued on (they must follow the call that wrote the entries)
 * Errors: JUP_EINVAL (NULL, n_keep out of range, slots not increasing), JUP_EPOS (base_len or a slot outside
 * the cache, inside a fork's shared prefix, or below the n_shared of a live fork), JUP_EDEVICE.
 */
JUP_API jup_status_t jup_kv_keep(jup_kv_t *kv, int32_t base_len, int32_t n_keep, const int32_t *slots, void *stream);

JUP_API int32_t jup_kv_len(const jup_kv_t *kv);      /* positions currently valid; -1 for NULL */
JUP_API int32_t jup_kv_capacity(const jup_kv_t *kv); /* max_positions; -1 for NULL */

/*
 * Would a chunk of n_tokens at pos_offset be accepted?  Pure host logic, the same check
 * jup_stage_prefill_chunk() applies:
 *   n_tokens < 0 or pos_offset < 0            -> JUP_EINVAL
 *   pos_offset > length                       -> JUP_EPOS  (a hole: the prefix s_1..s_{i-1} would be incomplete)
 *   pos_offset < n_shared of a fork           -> JUP_EPOS  (shared prefix is read-only)
 *   pos_offset < n_shared of a live child     -> JUP_EPOS
 *   pos_offset + n_tokens > max_positions     -> JUP_ECAP
 * pos_offset < length is allowed and means "overwrite from here" (implicit truncate).
 */
JUP_API jup_status_t jup_kv_check_append(const jup_kv_t *kv, int32_t n_tokens, int32_t pos_offset);

/* Frees the host object.  JUP_EINVAL if forks of it are still alive. NULL is allowed. */
JUP_API jup_status_t jup_kv_destroy(jup_kv_t *kv);

/* ---- the hot path --------------------------------------------------------------------------- */

/*
 * One stage forward over one chunk (Sec. IV-A.2), steps 1-6 above for every layer of the stage.
 *   hidden_in   [n_tokens, d_model], stage dtype
 *   n_tokens    any value >= 0 (0 is a no-op); must be <= the stage's max_chunk_tokens
 *   pos_offset  number of tokens of the earlier chunks; see jup_kv_check_append()
 *   kv          cache made for the same configuration as the stage
 *   hidden_out  [n_tokens, d_model], stage dtype; may be the same buffer as hidden_in
 *   stream      hipStream_t (NULL = default stream); all kernels are enqueued there
 * On success the cache length becomes pos_offset + n_tokens.
 * Errors: JUP_EINVAL, JUP_EPOS, JUP_ECAP (nothing enqueued, length unchanged), JUP_EDEVICE.
 */
JUP_API jup_status_t jup_stage_prefill_chunk(jup_stage_t *stage, const void *hidden_in, int32_t n_tokens,
                                     int32_t pos_offset, jup_kv_t *kv, void *hidden_out, void *stream);

/*
 * jup_stage_prefill_chunk() for callers that cannot allocate device memory or hold a workspace for the call: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * results bit for bit; the scratch of the call (residual stream, normalised rows, queries, attention output, SwiGLU
 * output, rotary table, K-split partial sums, key-split attention partials) lies in a static device array of JUP_STATIC_SCRATCH_BYTES inside the
 * library instead of the workspace given to jup_stage_create(), which this call does not touch.  The call
 * allocates nothing (no hipMalloc, hipFree or allocating library routine).
 *   - Every GPU the library runs on holds one copy of the array until the process ends; its address is looked up
 *     once per device, on the first call with that device current.
 *   - The chunk's scratch must fit the array (the scratch of ONE chunk of n_tokens, without the share that batched
 *     branches add to a stage's workspace): a 7B-shaped stage runs up to 192 tokens, a 13B-shaped one 160, d_model
 *     8192 with FFN 28672 and 64 heads 64; beyond that JUP_ECAP (the message names the bytes needed) and nothing is
 *     enqueued.  The stage's max_chunk_tokens does not limit this call.
 *   - All calls on one GPU share the array, whatever their stage or stream: calls that overlap in time on one GPU
 *     race.  Issue them on one stream, or order them with events.  Nothing in the array has to survive between
 *     calls or start at zero.
 * Errors: as jup_stage_prefill_chunk(), plus JUP_ECAP as above and JUP_EDEVICE if the array's address cannot be found.
 */
#define JUP_STATIC_SCRATCH_BYTES (48 << 20)
JUP_API jup_status_t jup_stage_prefill_chunk_static(jup_stage_t *stage, const void *hidden_in, int32_t n_tokens,
                                                    int32_t pos_offset, jup_kv_t *kv, void *hidden_out, void *stream);

/*
 * Several consecutive chunks of one prompt in one call (Sec. IV-A.2: the sub-sequences s_1..s_M are injected one
 * after the other; sub-sequence s_i needs, layer by layer, what the stage cached for s_1..s_{i-1}, and nothing
 * else of them).  Computes what n_chunks calls of jup_stage_prefill_chunk() in order compute, the first at
 * pos_offset: the same cache entries are written, the final length is the same, and without
 * jup_stage_enable_overlap() outputs and cache values are equal bit for bit.  With it they are equal up to the
 * summation order of fp32 partial sums (the projections back to d_model split K into fewer pieces while other
 * chunks share the GPU), i.e. to the last bits of a bf16 value; the call is deterministic either way.
 *   hidden_in     [sum of chunk_tokens, d_model]; the chunks follow each other
 *   chunk_tokens  HOST array [n_chunks], each 0 .. the stage's max_chunk_tokens
 *   hidden_out    [sum of chunk_tokens, d_model]; may be the same buffer as hidden_in
 * After jup_stage_enable_overlap() a JUP_BF16 stage lets consecutive chunks overlap on the GPU: they go round
 * n_lanes lanes (a stream plus a scratch buffer each; lane 0 is `stream` with the stage's own workspace), and a
 * chunk waits, per layer, only for the cache appends of the chunks before it before its own attention.  The
 * ramp-up and the tail of one chunk's kernels are then filled with another chunk's work, and the weights of a
 * layer that one chunk streamed from HBM are still in the last-level cache when the next chunk asks for them
 * (the paper fills the stages of a pipeline with sub-sequences in the same way, across devices).  Chunks of up
 * to 256 tokens use all enabled lanes; longer ones all of them when their number is a multiple of four, else two.
 * On return all
 * work is ordered before whatever is enqueued on `stream` next.  Without jup_stage_enable_overlap(), and in check
 * mode, the chunks simply run one after the other on `stream`.
 * Errors: as jup_stage_prefill_chunk(); every chunk is validated before anything is enqueued.
 */
JUP_API jup_status_t jup_stage_prefill_chunks(jup_stage_t *stage, const void *hidden_in, int32_t n_chunks,
                                      const int32_t *chunk_tokens, int32_t pos_offset, jup_kv_t *kv,
                                      void *hidden_out, void *stream);

/*
 * Gives the stage what jup_stage_prefill_chunks() needs to overlap consecutive chunks on n_lanes lanes
 * (2 .. JUP_MAX_LANES): scratch for the further lanes, one DEVICE buffer, 256-byte aligned, of at least
 * (n_lanes - 1) * jup_stage_workspace_bytes(cfg, max_chunk_tokens) bytes, borrowed until jup_stage_destroy().
 * Creates n_lanes - 1 streams of default priority and n_lanes * (n_layers + 1) events, which
 * jup_stage_destroy() releases.  Call once, not on the hot path.
 * Errors: JUP_EINVAL (NULL, n_lanes out of range, misaligned, too small, overlapping the stage's workspace,
 * called twice), JUP_ENOMEM, JUP_EDEVICE.
 */
#define JUP_MAX_LANES 4
JUP_API jup_status_t jup_stage_enable_overlap(jup_stage_t *stage, int32_t n_lanes, void *lane_workspaces,
                                      size_t lane_workspaces_bytes);

/*
 * The same stage forward for several branches at once.  In outline-based pipeline parallel decoding the
 * branches of one request are independent sub-sequences over a shared prompt cache (Sec. V-B, Fig. 11),
 * each advanced by a few tokens per step (Sec. V-A: one token plus speculative candidates).  The paper
 * staggers the branches over the stages of the pipeline; inside ONE stage this call goes further and pushes
 * the chunks of all branches through the layers together, so that the stage's weights, whose streaming from
 * HBM bounds a decode-sized chunk, are read once per step instead of once per branch.  This batching is an
 * optimisation of this library, not a mechanism of the paper.
 *   n_branches   1 .. JUP_MAX_BRANCHES
 *   hidden_in    [n_branches * n_tokens, d_model], stage dtype: rows b*n_tokens .. (b+1)*n_tokens-1 are
 *                the chunk of branch b
 *   n_tokens     tokens per branch (the same for all); n_branches * n_tokens <= the stage's max_chunk_tokens
 *   pos_offsets  HOST array [n_branches]: pos_offset of every branch's chunk (rules of jup_kv_check_append)
 *   kvs          HOST array [n_branches] of caches, all different, none the parent of another in the list
 *   hidden_out   [n_branches * n_tokens, d_model]; may be the same buffer as hidden_in
 * The result equals n_branches calls of jup_stage_prefill_chunk(), one per branch, bit for bit in the
 * JUP_BF16 path's caches and outputs (rows do not interact outside attention, and every row meets the same
 * arithmetic in the same order either way).  On success every cache b has length pos_offsets[b] + n_tokens.
 * Errors: as jup_stage_prefill_chunk(); all branches are validated before anything is enqueued, and on error
 * no cache changes.
 */
#define JUP_MAX_BRANCHES 16
JUP_API jup_status_t jup_stage_prefill_branches(jup_stage_t *stage, int32_t n_branches, const void *hidden_in,
                                        int32_t n_tokens, const int32_t *pos_offsets, jup_kv_t *const *kvs,
                                        void *hidden_out, void *stream);

/*
 * The same stage forward over the candidate tokens of one speculative decoding step (Sec. V-A, steps 3-5:
 * all candidates go through the model in one forward pass, their intermediate results are stored in the
 * KVCache, and the rejected ones are removed afterwards).  The candidates form a token tree, the drafting
 * scheme the paper evaluates with (Medusa's): token t continues token parents[t] of the same call, or the
 * cached sequence itself when parents[t] is -1.
 *   parents     HOST array [n_tokens], parents[t] in {-1, 0 .. t-1}
 *   n_tokens    0 .. JUP_MAX_TREE_TOKENS (and <= the stage's max_chunk_tokens)
 *   others      as jup_stage_prefill_chunk()
 * Token t
 *   - is rotated at position pos_offset + depth(t)   (depth = number of ancestors inside the call),
 *   - is stored in cache entry pos_offset + t,
 *   - attends to the entries 0 .. pos_offset-1, to its ancestors' entries and to its own.
 * Row t of hidden_out is therefore what an ordinary call on the tokens of t's root-to-node path would give
 * for its last token; a chain (parents[t] = t-1) is exactly jup_stage_prefill_chunk().  On success the cache
 * length is pos_offset + n_tokens; the caller then verifies the candidates and calls jup_kv_keep() with the
 * accepted path (or jup_kv_truncate() to drop them all).
 * Errors: as jup_stage_prefill_chunk(), plus JUP_EINVAL for n_tokens > JUP_MAX_TREE_TOKENS, parents == NULL
 * or a parent index outside [-1, t).
 */
#define JUP_MAX_TREE_TOKENS 64
JUP_API jup_status_t jup_stage_prefill_tree(jup_stage_t *stage, const void *hidden_in, int32_t n_tokens,
                                    int32_t pos_offset, const int32_t *parents, jup_kv_t *kv, void *hidden_out,
                                    void *stream);

/* ---- per-kernel timing (benchmarks) ----------------------------------------------------------- */

/*
 * Kernels of one layer of the JUP_BF16 path, in launch order.  The profiler of the paper records
 * per-layer run-time traces of the prefill (Sec. III, step 1); these ids let a benchmark time one
 * kernel class in place, with HIP events recorded on the stream the kernel is launched on.
 */
typedef enum {
    JUP_K_RMSNORM = 0,
    JUP_K_GEMM_QKV = 1,    /* QKV projection + rotary + KV append */
    JUP_K_ATTENTION = 2,   /* prefix + causal chunk attention */
    JUP_K_GEMM_O = 3,      /* output projection + residual */
    JUP_K_GEMM_GATE_UP = 4, /* gate/up projection + SwiGLU */
    JUP_K_GEMM_DOWN = 5,   /* down projection + residual */
    JUP_K_COUNT = 6
} jup_kernel_id_t;

/*
 * Starts timing every launch of kernel class `kernel_id` made by later jup_stage_prefill_chunk()
 * calls on this stage: an event pair brackets each launch (at most max_launches pairs; further
 * launches run untimed and are counted as dropped).  kernel_id = -1 stops tracing and releases the
 * events.  Tracing perturbs the stream slightly: time whole calls with tracing off.
 * Errors: JUP_EINVAL (NULL stage, bad id, max_launches <= 0), JUP_ENOMEM, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_stage_trace(jup_stage_t *stage, int32_t kernel_id, int32_t max_launches);

/*
 * Waits for the recorded events, returns the summed duration in milliseconds and the number of
 * launches timed / dropped (host pointers, each may be NULL), and rewinds the event pool.
 * JUP_EINVAL if the stage is not tracing.
 */
JUP_API jup_status_t jup_stage_trace_read(jup_stage_t *stage, double *total_ms, int32_t *launches, int32_t *dropped);

/* ---- calibration of the chip (benchmarks) ------------------------------------------------------- */

/*
 * What the matrix cores sustain when they do nothing else: the yardstick the measured GEMMs are held against
 * beside the published peak (Sec. III step 1 profiles the devices the model runs on; this is the part of such a
 * profile that the roofline needs).  Launches n_workgroups workgroups of 8 waves (two per SIMD); every wave runs
 * iters_per_wave rounds of 8 independent 32x32x16 bf16 MFMAs on fragments taken from `operands`.
 *   operands        DEVICE, >= 530432 bytes of bf16 values (random data gives the power draw of real operands)
 *   ticks           DEVICE, uint64 [n_workgroups][2]: shader-clock ticks and 100 MHz reference-clock ticks the
 *                   loop of each workgroup took (their ratio x 100 MHz is the clock the chip held)
 *   sink            DEVICE, one float (never written in practice; keeps the arithmetic alive)
 *   flop            HOST out, may be NULL: floating-point operations of the launch
 * The caller times the launch (events on `stream`).  Errors: JUP_EINVAL, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_diag_mfma_loop(const void *operands, size_t operand_bytes, int32_t n_workgroups,
                                        int64_t iters_per_wave, void *ticks, float *sink, void *stream, double *flop);

/*
 * Which instantiation of the projection kernel a chunk of n_tokens runs as: "gemm_bf16<row blocks,column blocks,
 * waves along M,waves along N,epilogue>" written to buf (HOST, size bytes, always terminated).  overlapped != 0:
 * inside an overlapped jup_stage_prefill_chunks() call.  A benchmark uses it to tell whether a hardware-counter
 * reading kept on file was taken for the tiling that runs today.  kernel_id: one of the four JUP_K_GEMM_* ids.
 * Errors: JUP_EINVAL (NULL, not a projection id, not a JUP_BF16 stage).
 */
JUP_API jup_status_t jup_diag_kernel_name(const jup_stage_t *stage, int32_t kernel_id, int32_t n_tokens,
                                          int32_t overlapped, char *buf, size_t size);

/*
 * The shader clock held while other work runs: one wave that sleeps until ref_ticks ticks of the 100 MHz
 * reference clock have passed (it always ends) and then writes {shader-clock ticks, reference ticks} (uint64
 * [2], DEVICE) .  Launch it on a stream of its own beside the work to be observed.
 * 1 <= ref_ticks <= 2^30 (about 10 s).  Errors: JUP_EINVAL, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_diag_clock_probe(int64_t ref_ticks, void *ticks, void *stream);

/*
 * What the operand-fill path of the projection kernels can move: n_workgroups x 8 waves copy 1 KB pieces of buf
 * (DEVICE; every workgroup walks the same window of window_bytes, a power of two between 1 MiB and 2 GiB that the
 * buffer holds, so the pieces come from L2 when the window fits there) into LDS with
 * direct global->LDS loads, `depth` (1, 2, 4, 8 or 16) pieces per wave in flight, pieces_per_wave (a multiple of 16)
 * pieces each.  bytes (HOST out, may be NULL): bytes the launch moves.  The caller times the launch.
 * Errors: JUP_EINVAL, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_diag_fill_probe(const void *buf, size_t window_bytes, int32_t n_workgroups, int32_t depth,
                                         int32_t pieces_per_wave, void *stream, double *bytes);

/*
 * Floor of a projection that streams its weights once: n_workgroups x 8 waves copy disjoint contiguous regions of buf
 * (DEVICE, buf_bytes long; pieces_per_wave x 8 KiB per workgroup) into LDS with direct global->LDS loads, `depth`
 * (1, 2, 4, 8 or 16; pieces_per_wave is a multiple of it) pieces of 1 KiB per wave in flight; nothing is read twice
 * inside a launch.  n_launches (1..4096) launches are enqueued back to back, like the kernels of a call; successive
 * launches read successive parts of the buffer, round robin (a buffer several times the last-level cache keeps every
 * launch cold).  bytes (HOST out, may be NULL): bytes all launches move.  The caller times them.  Errors: JUP_EINVAL
 * (also when the buffer is too short for one launch), JUP_EDEVICE.
 */
JUP_API jup_status_t jup_diag_stream_probe(const void *buf, size_t buf_bytes, int32_t n_workgroups, int32_t depth,
                                           int32_t pieces_per_wave, int32_t n_launches, void *stream, double *bytes);

/*
 * LDS read rate of a CU: n_workgroups workgroups of `threads` lanes (a multiple of 64, up to 1024) read 16 KB per
 * wave and trip from LDS, 16 bytes per lane and instruction without bank conflicts.  ticks (DEVICE, uint64
 * [n_workgroups]): shader-clock ticks of each workgroup's loop; sink (DEVICE, one uint32, never written in practice);
 * bytes_per_workgroup (HOST out, may be NULL).  Errors: JUP_EINVAL, JUP_EDEVICE.
 */
JUP_API jup_status_t jup_diag_lds_read_probe(int32_t n_workgroups, int32_t threads, int32_t trips, void *ticks,
                                             void *sink, void *stream, double *bytes_per_workgroup);

/* Message of the last error on this thread ("" if none). Never NULL. */
JUP_API const char *jup_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* JUPITER_STAGE_H */
