// The parallelism planner of the Jupiter paper (Sec. IV-B) as host code: the two dynamic programs (Eq. 1 for
// the layers, Eq. 2 and 3 for the tokens) and the choice of the number of sub-sequences (Eq. 4).  No device
// code; the file is built with the rest of the library so that one shared object carries the whole C ABI.
#include <cmath>
#include <limits>
#include <new>
#include <vector>

#include "jup_internal.h"
#include "jupiter_plan.h"

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();
using jup::set_error;

// Position of v on a strictly increasing grid: value(v) = (1 - w) f[i] + w f[i + 1].  Above the grid the
// outermost segment is continued (w > 1); below it the first grid point's value is held (a segment continued
// downwards can cross zero, and a latency that is not positive makes Eq. 2-4 meaningless).
struct Seg {
    int32_t i;
    double w;
};
Seg locate(const std::vector<int32_t>& grid, int32_t v) {
    const int n = (int)grid.size();
    if (n == 1 || v <= grid[0]) return {0, 0.0};
    int i = 0;
    while (i < n - 2 && grid[i + 1] <= v) ++i;
    return {i, (double)(v - grid[i]) / (double)(grid[i + 1] - grid[i])};
}

}  // namespace

struct jup_seq_plan {
    int32_t b, n_devices, s_max, k_max;
    std::vector<int32_t> xs, ys;
    std::vector<double> q;      // [nx][ny]
    double q_floor;             // smallest profiled latency: a value continued beyond the grid never falls below it
    std::vector<Seg> seg_x;     // for x = 0..s_max (entry 0 unused)
    std::vector<Seg> seg_y;     // for y = 0..s_max
    std::vector<double> W;      // [k_max + 1][s_max + 1], W[k][y]
    std::vector<int32_t> cut;   // [k_max + 1][s_max + 1]: the l of Eq. 2 that attains W[k][y] (0 for k = 1)

    double q_at(int32_t x, int32_t y) const { return q_on(seg_x[x], seg_y[y]); }
    double q_on(const Seg sx, const Seg sy) const {
        const int ny = (int)ys.size();
        const int i2 = sx.i + 1 < (int)xs.size() ? sx.i + 1 : sx.i;
        const int j2 = sy.i + 1 < ny ? sy.i + 1 : sy.i;
        const double lo = (1.0 - sy.w) * q[(size_t)sx.i * ny + sy.i] + sy.w * q[(size_t)sx.i * ny + j2];
        const double hi = (1.0 - sy.w) * q[(size_t)i2 * ny + sy.i] + sy.w * q[(size_t)i2 * ny + j2];
        return std::fmax((1.0 - sx.w) * lo + sx.w * hi, q_floor);
    }
    double t_star(int32_t x, int32_t l) const { return x < b ? kInf : q_at(x, l); }
    size_t at(int32_t k, int32_t y) const { return (size_t)k * (s_max + 1) + y; }
};

extern "C" {

jup_status_t jup_plan_layers(int32_t n_layers, int32_t n_devices, const double* layer_time, const double* layer_mem,
                             const double* mem_budget, int32_t* last_layer, double* slowest) {
    const char* me = "jup_plan_layers";
    if (n_layers < 1 || n_devices < 1) return set_error(JUP_EINVAL, "%s: n_layers and n_devices must be at least 1", me);
    if (!layer_time || !layer_mem || !mem_budget || !last_layer || !slowest)
        return set_error(JUP_EINVAL, "%s: NULL argument", me);
    for (long i = 0; i < (long)n_layers * n_devices; ++i)
        if (!(layer_time[i] >= 0.0)) return set_error(JUP_EINVAL, "%s: layer_time[%ld] is negative or NaN", me, i);
    for (int l = 0; l < n_layers; ++l)
        if (!(layer_mem[l] >= 0.0)) return set_error(JUP_EINVAL, "%s: layer_mem[%d] is negative or NaN", me, l);
    for (int n = 0; n < n_devices; ++n)
        if (std::isnan(mem_budget[n])) return set_error(JUP_EINVAL, "%s: mem_budget[%d] is NaN", me, n);
    if (n_layers < n_devices)
        return set_error(JUP_ECAP, "%s: %d layers cannot give each of %d devices one", me, n_layers, n_devices);

    try {
        const int L = n_layers, D = n_devices;
        // T(i..j, n) from prefix sums: time_to[n][j] = t_1 + .. + t_j on device n, mem_to[j] likewise
        std::vector<double> time_to((size_t)D * (L + 1), 0.0), mem_to(L + 1, 0.0);
        for (int n = 0; n < D; ++n)
            for (int j = 1; j <= L; ++j)
                time_to[(size_t)n * (L + 1) + j] = time_to[(size_t)n * (L + 1) + j - 1] + layer_time[(size_t)n * L + j - 1];
        for (int j = 1; j <= L; ++j) mem_to[j] = mem_to[j - 1] + layer_mem[j - 1];
        auto T = [&](int i, int j, int n) {  // layers i..j (1-based) on device n (0-based)
            if (mem_to[j] - mem_to[i - 1] > mem_budget[n]) return kInf;
            return time_to[(size_t)n * (L + 1) + j] - time_to[(size_t)n * (L + 1) + i - 1];
        };
        // A[n][y] for the first n devices (1-based) and the first y layers; cut[n][y] = the l that attains it
        std::vector<double> A((size_t)(D + 1) * (L + 1), kInf);
        std::vector<int32_t> cut((size_t)(D + 1) * (L + 1), 0);
        auto at = [&](int n, int y) { return (size_t)n * (L + 1) + y; };
        for (int y = 1; y <= L; ++y) A[at(1, y)] = T(1, y, 0);
        for (int n = 2; n <= D; ++n)
            for (int y = n; y <= L; ++y) {
                double best = kInf;
                int best_l = 0;
                for (int l = n - 1; l < y; ++l) {
                    const double v = std::fmax(A[at(n - 1, l)], T(l + 1, y, n - 1));
                    if (v < best) { best = v; best_l = l; }
                }
                A[at(n, y)] = best;
                cut[at(n, y)] = best_l;
            }
        if (A[at(D, L)] == kInf) return set_error(JUP_ECAP, "%s: no partition fits the memory budgets", me);
        *slowest = A[at(D, L)];
        for (int n = D, y = L; n >= 1; --n) {
            last_layer[n - 1] = y;
            y = cut[at(n, y)];
        }
    } catch (const std::bad_alloc&) {
        return set_error(JUP_ENOMEM, "%s: out of host memory", me);
    }
    return JUP_OK;
}

jup_status_t jup_seq_plan_create(const int32_t* xs, int32_t nx, const int32_t* ys, int32_t ny, const double* q,
                                 int32_t b, int32_t n_devices, int32_t s_max, jup_seq_plan_t** out) {
    return jup_seq_plan_create_aligned(xs, nx, ys, ny, q, b, 1, n_devices, s_max, out);
}

jup_status_t jup_seq_plan_create_aligned(const int32_t* xs, int32_t nx, const int32_t* ys, int32_t ny, const double* q,
                                         int32_t b, int32_t granule, int32_t n_devices, int32_t s_max,
                                         jup_seq_plan_t** out) {
    const char* me = "jup_seq_plan_create";
    if (out) *out = nullptr;
    if (!xs || !ys || !q || !out) return set_error(JUP_EINVAL, "%s: NULL argument", me);
    if (nx < 1 || ny < 1 || nx > 4096 || ny > 4096) return set_error(JUP_EINVAL, "%s: grid sizes must be in 1..4096", me);
    if (b < 1) return set_error(JUP_EINVAL, "%s: the minimum sub-sequence length b=%d must be at least 1", me, b);
    if (granule < 1 || granule > 16384) return set_error(JUP_EINVAL, "%s: granule=%d is outside 1..16384", me, granule);
    if (n_devices < 1 || n_devices > 64) return set_error(JUP_EINVAL, "%s: n_devices=%d is outside 1..64", me, n_devices);
    if (s_max < 1 || s_max > 16384) return set_error(JUP_EINVAL, "%s: s_max=%d is outside 1..16384", me, s_max);
    if (xs[0] < 1 || ys[0] < 0) return set_error(JUP_EINVAL, "%s: xs must start at 1 or more, ys at 0 or more", me);
    for (int i = 1; i < nx; ++i)
        if (xs[i] <= xs[i - 1]) return set_error(JUP_EINVAL, "%s: xs is not strictly increasing at %d", me, i);
    for (int j = 1; j < ny; ++j)
        if (ys[j] <= ys[j - 1]) return set_error(JUP_EINVAL, "%s: ys is not strictly increasing at %d", me, j);
    for (long i = 0; i < (long)nx * ny; ++i)
        if (!(q[i] > 0.0) || std::isinf(q[i])) return set_error(JUP_EINVAL, "%s: q[%ld] is not a positive finite latency", me, i);

    jup_seq_plan* p = nullptr;
    try {
        p = new jup_seq_plan();
        p->b = b;
        p->n_devices = n_devices;
        p->s_max = s_max;
        p->k_max = 4 * n_devices;
        p->xs.assign(xs, xs + nx);
        p->ys.assign(ys, ys + ny);
        p->q.assign(q, q + (size_t)nx * ny);
        p->q_floor = q[0];
        for (long i = 1; i < (long)nx * ny; ++i) p->q_floor = std::fmin(p->q_floor, q[i]);
        p->seg_x.resize(s_max + 1);
        p->seg_y.resize(s_max + 1);
        for (int v = 0; v <= s_max; ++v) {
            p->seg_x[v] = locate(p->xs, v);
            p->seg_y[v] = locate(p->ys, v);
        }
        const int K = p->k_max, S = s_max;
        p->W.assign((size_t)(K + 1) * (S + 1), kInf);
        p->cut.assign((size_t)(K + 1) * (S + 1), 0);
        for (int y = 1; y <= S; ++y) p->W[p->at(1, y)] = p->t_star(y, 0);
        for (int k = 2; k <= K; ++k) {
            const double* prev = &p->W[p->at(k - 1, 0)];
            // W(1..l, k-1) is infinite below (k-1) b tokens and T*(y-l, l) above y - b: only the l between count
            // (cut points are multiples of the granule: every sub-sequence but the last a whole number of granules)
            const long l_lo = ((long)(k - 1) * b + granule - 1) / granule * granule;
            for (int y = 1; y <= S; ++y) {
                double best = kInf;
                int best_l = 0;
                for (long l = l_lo; l <= (long)y - b; l += granule) {
                    const double v = std::fmax(prev[l], p->q_at(y - (int)l, (int)l));
                    if (v < best) { best = v; best_l = (int)l; }
                }
                p->W[p->at(k, y)] = best;
                p->cut[p->at(k, y)] = best_l;
            }
        }
    } catch (const std::bad_alloc&) {
        delete p;
        return set_error(JUP_ENOMEM, "%s: out of host memory", me);
    }
    *out = p;
    return JUP_OK;
}

void jup_seq_plan_destroy(jup_seq_plan_t* plan) { delete plan; }

double jup_seq_plan_q(const jup_seq_plan_t* plan, int32_t x, int32_t y) {
    if (!plan || x < 1 || y < 0) return std::numeric_limits<double>::quiet_NaN();
    // lengths beyond s_max are located on the spot
    if (x <= plan->s_max && y <= plan->s_max) return plan->q_at(x, y);
    return plan->q_on(locate(plan->xs, x), locate(plan->ys, y));
}

jup_status_t jup_seq_plan_partition(const jup_seq_plan_t* plan, int32_t y, int32_t k, int32_t* lengths, double* slowest,
                                    double* total) {
    const char* me = "jup_seq_plan_partition";
    if (!plan) return set_error(JUP_EINVAL, "%s: plan is NULL", me);
    if (y < 1 || y > plan->s_max) return set_error(JUP_EINVAL, "%s: y=%d is outside 1..%d", me, y, plan->s_max);
    if (k < 1 || k > plan->k_max) return set_error(JUP_EINVAL, "%s: k=%d is outside 1..%d", me, k, plan->k_max);
    const double w = plan->W[plan->at(k, y)];
    if (w == kInf)
        return set_error(JUP_ECAP, "%s: %d tokens cannot be cut into %d sub-sequences of at least %d", me, y, k, plan->b);
    double sum = 0.0;
    for (int kk = k, yy = y; kk >= 1; --kk) {  // the last sub-sequence first
        const int l = plan->cut[plan->at(kk, yy)];
        if (lengths) lengths[kk - 1] = yy - l;
        sum += plan->q_at(yy - l, l);
        yy = l;
    }
    if (slowest) *slowest = w;
    if (total) *total = sum;
    return JUP_OK;
}

jup_status_t jup_seq_plan_best(const jup_seq_plan_t* plan, int32_t y, int32_t* k_out, int32_t* lengths, double* latency) {
    const char* me = "jup_seq_plan_best";
    if (!plan || !k_out) return set_error(JUP_EINVAL, "%s: plan and k_out must not be NULL", me);
    if (y < 1 || y > plan->s_max) return set_error(JUP_EINVAL, "%s: y=%d is outside 1..%d", me, y, plan->s_max);
    int best_k = 0;
    double best = kInf;
    for (int k = 1; k <= plan->k_max; ++k) {
        const double w = plan->W[plan->at(k, y)];
        if (w == kInf) continue;
        double sum = 0.0;
        for (int kk = k, yy = y; kk >= 1; --kk) {
            const int l = plan->cut[plan->at(kk, yy)];
            sum += plan->q_at(yy - l, l);
            yy = l;
        }
        const double lat = sum + (plan->n_devices - 1) * w;  // Eq. 4
        if (lat < best) { best = lat; best_k = k; }
    }
    if (best_k == 0) return set_error(JUP_ECAP, "%s: %d tokens are fewer than the minimum sub-sequence length %d", me, y, plan->b);
    *k_out = best_k;
    if (latency) *latency = best;
    if (lengths) return jup_seq_plan_partition(plan, y, best_k, lengths, nullptr, nullptr);
    return JUP_OK;
}

}  // extern "C"
