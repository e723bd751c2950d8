// Small kernels around the cache that both the check-mode and the matrix-core path use: parking the table of a
// token-tree call in the workspace, and compacting the cache after the verification of such a call.
#include "jup_internal.h"

namespace jup {
namespace {

__global__ void write_tree_table(const TreeTable t, TreeTable* __restrict__ dst) {
    if (threadIdx.x == 0) dst->n = t.n;
    if ((int)threadIdx.x < kMaxTreeTokens) {
        dst->depth[threadIdx.x] = t.depth[threadIdx.x];
        dst->sees[threadIdx.x] = t.sees[threadIdx.x];
    }
}

// Removal of the rejected candidates (Sec. V-A step 5).  A thread owns one column (a piece of 16 bytes, of 8
// when the rows are no multiple of 16) of one plane and moves it row by row, in list order: destination
// base + j never lies behind a source still to be read (slots[j'] >= j' > j for every later j'), and nobody
// else touches the column, so the move is done in place.
template <typename Piece>
__global__ __launch_bounds__(256) void kv_keep(Piece* own, int own_cap, int n_planes, int pieces, int base,
                                               const KeepList list) {
    const long long gid = (long long)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= (long long)n_planes * pieces) return;
    const int plane = (int)(gid / pieces), piece = (int)(gid % pieces);
    Piece* col = own + ((size_t)plane * own_cap + base) * pieces + piece;
    for (int j = 0; j < list.n; ++j)
        if (list.slots[j] != j) col[(size_t)j * pieces] = col[(size_t)list.slots[j] * pieces];
}

}  // namespace

void launch_write_tree_table(const TreeTable& host_table, TreeTable* dst, hipStream_t s) {
    hipLaunchKernelGGL(write_tree_table, dim3(1), dim3(64), 0, s, host_table, dst);
}

void launch_kv_keep(void* own, int own_cap, int n_planes, int row_bytes, int base, const KeepList& list,
                    hipStream_t s) {
    const bool wide = row_bytes % 16 == 0;  // rows are a multiple of 8 bytes: head_dim is even
    const int pieces = row_bytes / (wide ? 16 : 8);
    const dim3 grid((unsigned)(((long long)n_planes * pieces + 255) / 256));
    if (wide)
        hipLaunchKernelGGL(kv_keep<uint4>, grid, dim3(256), 0, s, (uint4*)own, own_cap, n_planes, pieces, base, list);
    else
        hipLaunchKernelGGL(kv_keep<uint2>, grid, dim3(256), 0, s, (uint2*)own, own_cap, n_planes, pieces, base, list);
}

}  // namespace jup
