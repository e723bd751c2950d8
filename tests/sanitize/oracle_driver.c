/*
 * Drives every entry point of oracle/jupiter_oracle.c on a tiny stage with buffers of exactly the documented sizes,
 * for a build with -fsanitize=address,undefined: an index that leaves its range or an undefined operation aborts.
 * Inputs come from a file written by the test (so that the same numbers can be fed to the ordinary build);
 * outputs go to a file the test compares with the ordinary build's.
 *
 *   oracle_driver <inputs.bin> <outputs.bin>
 * inputs.bin:  int32 header {n_layers, d, n_heads, dh, f, n_total, max_positions, n_chunks, chunk sizes[8],
 *              n_tree, parents[16]} followed by float32 data: per layer wq wk wv wo w_gate w_up w_down g_attn g_mlp,
 *              then hidden [n_total + n_tree, d].
 */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int oracle_stage_prefill_chunk(int n_layers, int d, int n_heads, int dh, int f, double rms_eps, double rope_theta,
                               const float *const *weights, const float *hidden_in, int n_tokens, int pos_offset,
                               float *kv, int max_positions, float *hidden_out);
int oracle_stage_prefill_tree(int n_layers, int d, int n_heads, int dh, int f, double rms_eps, double rope_theta,
                              const float *const *weights, const float *hidden_in, int n_tokens, int pos_offset,
                              const int32_t *parents, float *kv, int max_positions, float *hidden_out);
void oracle_rmsnorm(const float *x, const float *g, float *y, int n, int d, double eps);
void oracle_rope(float *v, int n_vec, int dh, const int64_t *pos, double theta);
void oracle_linear_nt(const float *x, const float *w, float *y, int n, int out, int k_dim);
int oracle_num_threads(void);

static float *read_floats(FILE *fp, size_t n)
{
    float *p = (float *)malloc(n * sizeof(float)); /* exactly n: one element past it is an error ASan reports */
    if (!p || fread(p, sizeof(float), n, fp) != n) {
        fprintf(stderr, "short read of %zu floats\n", n);
        exit(2);
    }
    return p;
}

int main(int argc, char **argv)
{
    if (argc != 3)
        return 2;
    FILE *fp = fopen(argv[1], "rb");
    if (!fp)
        return 2;
    int32_t h[33];
    if (fread(h, sizeof(int32_t), 33, fp) != 33)
        return 2;
    const int L = h[0], d = h[1], H = h[2], dh = h[3], f = h[4], n_total = h[5], cap = h[6], n_chunks = h[7];
    const int32_t *chunks = h + 8, *parents = h + 17;
    const int n_tree = h[16];
    const size_t sizes[9] = {(size_t)d * d, (size_t)d * d, (size_t)d * d, (size_t)d * d, (size_t)f * d,
                             (size_t)f * d, (size_t)d * f, (size_t)d,     (size_t)d};
    const float **w = (const float **)malloc(sizeof(float *) * 9 * (size_t)L);
    for (int l = 0; l < L; ++l)
        for (int k = 0; k < 9; ++k)
            w[9 * l + k] = read_floats(fp, sizes[k]);
    float *hidden = read_floats(fp, (size_t)(n_total + n_tree) * d);
    fclose(fp);

    const size_t kv_n = (size_t)L * 2 * H * cap * dh;
    float *kv = (float *)calloc(kv_n, sizeof(float));
    float *out = (float *)malloc((size_t)(n_total + n_tree) * d * sizeof(float));
    int pos = 0;
    for (int c = 0; c < n_chunks; ++c) {
        const int rc = oracle_stage_prefill_chunk(L, d, H, dh, f, 1e-5, 1e4, w, hidden + (size_t)pos * d, chunks[c], pos,
                                                  kv, cap, out + (size_t)pos * d);
        if (rc != 0) {
            fprintf(stderr, "chunk %d: rc %d\n", c, rc);
            return 1;
        }
        pos += chunks[c];
    }
    if (pos != n_total)
        return 2;
    if (n_tree > 0 &&
        oracle_stage_prefill_tree(L, d, H, dh, f, 1e-5, 1e4, w, hidden + (size_t)pos * d, n_tree, pos, parents, kv, cap,
                                  out + (size_t)pos * d) != 0) {
        fprintf(stderr, "tree failed\n");
        return 1;
    }
    /* the calls a caller gets wrong must come back as errors, not as out-of-range accesses */
    if (oracle_stage_prefill_chunk(L, d, H, dh, f, 1e-5, 1e4, w, hidden, 2, cap - 1, kv, cap, out) == 0) {
        fprintf(stderr, "a chunk past the capacity was accepted\n");
        return 1;
    }
    const int32_t bad_parents[3] = {-1, 1, 0};
    if (oracle_stage_prefill_tree(L, d, H, dh, f, 1e-5, 1e4, w, hidden, 3, 0, bad_parents, kv, cap, out) == 0) {
        fprintf(stderr, "a parent that is not an earlier token was accepted\n");
        return 1;
    }

    /* single-step helpers on exact-size buffers */
    float *y = (float *)malloc((size_t)n_total * d * sizeof(float));
    oracle_rmsnorm(hidden, w[7], y, n_total, d, 1e-5);
    float *proj = (float *)malloc((size_t)n_total * f * sizeof(float));
    oracle_linear_nt(hidden, w[4], proj, n_total, f, d);
    int64_t *p64 = (int64_t *)malloc(sizeof(int64_t) * (size_t)n_total * H);
    for (int i = 0; i < n_total * H; ++i)
        p64[i] = (int64_t)1 << (i % 40); /* large positions: angle arithmetic must not overflow an int */
    oracle_rope(y, n_total * H, dh, p64, 1e4);

    fp = fopen(argv[2], "wb");
    if (!fp)
        return 2;
    fwrite(out, sizeof(float), (size_t)(n_total + n_tree) * d, fp);
    fwrite(kv, sizeof(float), kv_n, fp);
    fwrite(y, sizeof(float), (size_t)n_total * d, fp);
    fwrite(proj, sizeof(float), (size_t)n_total * f, fp);
    fclose(fp);
    printf("oracle_driver ok, %d threads\n", oracle_num_threads());
    for (int i = 0; i < 9 * L; ++i)
        free((void *)w[i]);
    free(w); free(hidden); free(kv); free(out); free(y); free(proj); free(p64);
    return 0;
}
