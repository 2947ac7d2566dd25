// stree_tree_index: depth, ancestor bit mask (tree mask L) and k-th ancestor
// table of every sequence, written to global memory.  Integer work, exact.
#include "common.hpp"
#include "launch.hpp"

namespace stree {

__global__ __launch_bounds__(kThreads) void tree_index_kernel(
    const int32_t *__restrict__ parent, int n, int words, int W, int32_t *__restrict__ depth_out,
    uint32_t *__restrict__ mask_out, int32_t *__restrict__ anc_out, int32_t *__restrict__ status) {
    __shared__ TreeLds T;
    __shared__ uint32_t mask[kMaxNodes * kMaxWords];
    __shared__ int par[kMaxNodes];
    const int b = blockIdx.x;
    const int i = threadIdx.x;
    const int32_t *par_g = parent + (size_t)b * n;
    const int bad = build_tree_index(T, mask, par_g, n, n, words, 0.f, 0.f);
    if (status && i == 0) status[b] = bad;
    if (bad) {
        if (i < n) {
            if (depth_out) depth_out[(size_t)b * n + i] = 0;
            if (mask_out)
                for (int w = 0; w < words; ++w) mask_out[((size_t)b * n + i) * words + w] = 0u;
            if (anc_out)
                for (int k = 0; k < W; ++k) anc_out[((size_t)b * n + i) * W + k] = 0;
        }
        return;
    }
    if (i < n) par[i] = par_g[i];
    __syncthreads();
    if (i < n) {
        const int d = T.cnt[i] - 1;
        if (depth_out) depth_out[(size_t)b * n + i] = d;
        if (mask_out)
            for (int w = 0; w < words; ++w) mask_out[((size_t)b * n + i) * words + w] = mask[i * words + w];
        if (anc_out) {
            int v = i;
            for (int k = 0; k < W; ++k) {
                int e;
                if (k <= d) {
                    e = v;
                    v = par[v];
                } else {
                    e = -(k - d);
                }
                anc_out[((size_t)b * n + i) * W + k] = e;
            }
        }
    }
}

hipError_t launch_tree_index(const stree_dims &d, const int32_t *parent, int32_t *depth_out,
                             uint32_t *mask_out, int32_t *anc_out, int32_t *status, hipStream_t st) {
    const int words = (d.nnodes + 31) / 32;
    hipLaunchKernelGGL(tree_index_kernel, dim3(d.batch), dim3(kThreads), 0, st, parent, d.nnodes, words,
                       d.conv_width, depth_out, mask_out, anc_out, status);
    return hipGetLastError();
}

}  // namespace stree
