// stree_tree_conv: depthwise causal conv1d along each node's ancestor chain.
// Pure streaming: one 16-byte channel vector per thread, W gathered rows
// (ancestors hit L2, the tree's rows are a few hundred KB per sequence).
#include "common.hpp"
#include "launch.hpp"

namespace stree {

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void load(const float *p, float (&o)[4]) {
        const float4 v = *reinterpret_cast<const float4 *>(p);
        o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
    }
    static __device__ __forceinline__ void store(float *p, const float (&o)[4]) {
        *reinterpret_cast<float4 *>(p) = make_float4(o[0], o[1], o[2], o[3]);
    }
};
template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void load(const bf16_t *p, float (&o)[8]) {
        const uint4 v = *reinterpret_cast<const uint4 *>(p);
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
    static __device__ __forceinline__ void store(bf16_t *p, const float (&o)[8]) {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)o[e];
        *reinterpret_cast<bf16x8 *>(p) = v;
    }
};

constexpr int kConvNodes = 4;   // nodes per workgroup: weights and the tree check are shared

// 1-D grid of ceil8(B * cblocks * nblocks) workgroups.  Workgroup ids are dealt to the 8 XCDs
// round-robin by the hardware; the id is remapped so that each XCD gets a contiguous range of
// (sequence, channel block, node block) with the node block fastest: the ancestors' rows that the
// node blocks of one (sequence, channel block) share are then fetched into one L2 only.
template <typename T, int W>
__global__ __launch_bounds__(kThreads) void tree_conv_kernel(
    const int32_t *__restrict__ parent, int nbatch, int n, int Cc, int silu, const T *__restrict__ xbc_pre,
    const T *__restrict__ conv_state, const T *__restrict__ w, const T *__restrict__ bias,
    T *__restrict__ out, int32_t *__restrict__ status) {
    constexpr int VEC = Vec16<T>::N;
    __shared__ int par[kMaxNodes];
    __shared__ int bad_s;
    const int tid = threadIdx.x;
    const int cblocks = (Cc / VEC + kThreads - 1) / kThreads, nblocks = (n + kConvNodes - 1) / kConvNodes;
    const int logical = (blockIdx.x & 7) * (gridDim.x >> 3) + (blockIdx.x >> 3);
    if (logical >= nbatch * cblocks * nblocks) return;
    const int nb = logical % nblocks, cblk = (logical / nblocks) % cblocks, b = logical / (nblocks * cblocks);
    const int i0 = nb * kConvNodes;
    if (tid == 0) bad_s = 0x7fffffff;
    __syncthreads();
    if (tid < n) {
        const int p = parent[(size_t)b * n + tid];
        const bool ok = (tid == 0) ? (p == -1) : (p >= 0 && p < tid);
        if (!ok) atomicMin(&bad_s, tid + 1);
        par[tid] = ok ? p : -1;
    }
    __syncthreads();
    const int bad = bad_s == 0x7fffffff ? 0 : bad_s;
    if (status && cblk == 0 && nb == 0 && tid == 0) status[b] = bad;
    const int c0 = (cblk * kThreads + tid) * VEC;
    if (c0 >= Cc) return;
    if (bad) {
        float z[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) z[e] = 0.f;
        for (int i = i0; i < min(i0 + kConvNodes, n); ++i) Vec16<T>::store(out + ((size_t)b * n + i) * Cc + c0, z);
        return;
    }
    float wv[W][VEC];  // flat [e*W + j] = w[c0+e][j]
#pragma unroll
    for (int q = 0; q < W; ++q) Vec16<T>::load(w + (size_t)c0 * W + q * VEC, wv[q]);
    float bv[VEC];
    if (bias) Vec16<T>::load(bias + c0, bv);
    else {
#pragma unroll
        for (int e = 0; e < VEC; ++e) bv[e] = 0.f;
    }
    // all gathered rows of the workgroup's nodes are requested before any is used
    float r[kConvNodes][W][VEC];
#pragma unroll
    for (int m = 0; m < kConvNodes; ++m) {
        const int i = min(i0 + m, n - 1);
        int v = i, above = 0;
#pragma unroll
        for (int k = 0; k < W; ++k) {   // k-th ancestor, or conv_state once above the root
            const T *src;
            if (v >= 0) {
                src = xbc_pre + ((size_t)b * n + v) * Cc + c0;
                v = par[v];
            } else {
                ++above;  // `above` rows over the root: state row (W-1) - above
                src = conv_state + ((size_t)b * (W - 1) + (W - 1 - above)) * Cc + c0;
            }
            Vec16<T>::load(src, r[m][k]);
        }
    }
#pragma unroll
    for (int m = 0; m < kConvNodes; ++m) {
        if (i0 + m < n) {
            float acc[VEC];
#pragma unroll
            for (int e = 0; e < VEC; ++e) acc[e] = bv[e];
#pragma unroll
            for (int k = 0; k < W; ++k)
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fmaf((&wv[0][0])[e * W + (W - 1 - k)], r[m][k][e], acc[e]);
            if (silu) {
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = acc[e] / (1.f + __expf(-acc[e]));
            }
            Vec16<T>::store(out + ((size_t)b * n + i0 + m) * Cc + c0, acc);
        }
    }
}

template <typename T>
static hipError_t launch_conv_t(const stree_dims &d, const int32_t *parent, const void *xbc_pre,
                                const void *conv_state, const void *conv_w, const void *conv_b,
                                void *xbc_out, int32_t *status, hipStream_t st) {
    constexpr int VEC = Vec16<T>::N;
    const int Cc = d.nheads * d.headdim + 2 * d.ngroups * d.dstate;
    const int total = ((Cc / VEC + kThreads - 1) / kThreads) * ((d.nnodes + kConvNodes - 1) / kConvNodes) * d.batch;
    const dim3 grid((total + 7) / 8 * 8);
    const int silu = (d.flags & STREE_FLAG_CONV_SILU) ? 1 : 0;
#define STREE_CONV_CASE(WW)                                                                             \
    case WW:                                                                                            \
        hipLaunchKernelGGL((tree_conv_kernel<T, WW>), grid, dim3(kThreads), 0, st, parent, d.batch, d.nnodes, Cc, \
                           silu, (const T *)xbc_pre, (const T *)conv_state, (const T *)conv_w,          \
                           (const T *)conv_b, (T *)xbc_out, status);                                    \
        break;
    switch (d.conv_width) {
        STREE_CONV_CASE(2)
        STREE_CONV_CASE(3)
        STREE_CONV_CASE(4)
        default: return hipErrorInvalidValue;
    }
#undef STREE_CONV_CASE
    return hipGetLastError();
}

hipError_t launch_tree_conv(const stree_dims &d, const int32_t *parent, const void *xbc_pre,
                            const void *conv_state, const void *conv_w, const void *conv_b, void *xbc_out,
                            int32_t *status, hipStream_t st) {
    if (d.io_dtype == STREE_BF16)
        return launch_conv_t<bf16_t>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, st);
    return launch_conv_t<float>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, st);
}

}  // namespace stree
