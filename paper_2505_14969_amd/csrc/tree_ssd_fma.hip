// Plain fp32-FMA tree scan: covers every shape in the library's envelope (any
// headdim/dstate <= 256, fp32 or bf16 storage).  One workgroup per
// (batch, head); all arithmetic in fp32.  This is the fp32 path (1e-4 parity)
// and the fallback for shapes the MFMA kernel does not take.
//
// Per block of IB rows i:   Wt[ii][j] = L_ij * <C_i,B_j> * exp(s_i - s_j) * dt_j
//                           y_i = exp(s_i) * h0 C_i + sum_j Wt[ii][j] x_j + D x_i
#include "common.hpp"
#include "launch.hpp"

namespace stree {

constexpr int kFmaRows = 16;

template <typename T>
__global__ __launch_bounds__(kThreads) void tree_ssd_fma_kernel(
    const int32_t *__restrict__ parent, int n, int H, int P, int S, int G, const T *__restrict__ x,
    long x_sn, const float *__restrict__ dt, const float *__restrict__ A, const T *__restrict__ Bm,
    long b_sn, const T *__restrict__ Cm, long c_sn, const float *__restrict__ D,
    const float *__restrict__ h0, T *__restrict__ y, int32_t *__restrict__ status) {
    __shared__ TreeLds tree;
    __shared__ uint32_t mask[kMaxNodes * kMaxWords];
    __shared__ float Wt[kFmaRows][kMaxNodes];
    const int tid = threadIdx.x, h = blockIdx.x, b = blockIdx.y;
    const int g = h / (H / G);
    const int words = (n + 31) / 32;
    const float A_h = A[h];
    const float dt_i = tid < n ? dt[((size_t)b * n + tid) * H + h] : 0.f;
    const int bad = build_tree_index(tree, mask, parent + (size_t)b * n, n, n, words, dt_i, A_h);
    if (status && h == 0 && tid == 0) status[b] = bad;
    T *yb = y + (size_t)b * n * H * P + (size_t)h * P;
    if (bad) {
        for (int idx = tid; idx < n * P; idx += kThreads) {
            T z;
            from_f32(0.f, z);
            yb[(size_t)(idx / P) * H * P + idx % P] = z;
        }
        return;
    }
    const T *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
    const T *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
    const T *Cb = Cm + (size_t)b * n * c_sn + (size_t)g * S;
    const float *hb = h0 ? h0 + ((size_t)b * H + h) * P * S : nullptr;
    const float D_h = D ? D[h] : 0.f;

    for (int i0 = 0; i0 < n; i0 += kFmaRows) {
        const int rows = min(kFmaRows, n - i0);
        // decay-weighted masked scores for rows i0..i0+rows-1, columns 0..i0+rows-1
        const int ncol = i0 + rows;
        for (int idx = tid; idx < rows * ncol; idx += kThreads) {
            const int ii = idx / ncol, j = idx % ncol, i = i0 + ii;
            float wv = 0.f;
            if (mask_bit(mask, words, i, j)) {
                const T *ci = Cb + (size_t)i * c_sn;
                const T *bj = Bb + (size_t)j * b_sn;
                float dot = 0.f;
                for (int s = 0; s < S; ++s) dot = fmaf(to_f32(ci[s]), to_f32(bj[s]), dot);
                wv = dot * expf(tree.s[i] - tree.s[j]) * tree.dt[j];
            }
            Wt[ii][j] = wv;
        }
        __syncthreads();
        for (int idx = tid; idx < rows * P; idx += kThreads) {
            const int ii = idx / P, p = idx % P, i = i0 + ii;
            float acc = 0.f;
            if (hb) {
                const T *ci = Cb + (size_t)i * c_sn;
                const float *hp = hb + (size_t)p * S;
                for (int s = 0; s < S; ++s) acc = fmaf(hp[s], to_f32(ci[s]), acc);
                acc *= expf(tree.s[i]);
            }
            for (int j = 0; j <= i; ++j) {
                const float wv = Wt[ii][j];
                if (wv != 0.f) acc = fmaf(wv, to_f32(xb[(size_t)j * x_sn + p]), acc);
            }
            acc = fmaf(D_h, to_f32(xb[(size_t)i * x_sn + p]), acc);
            T o;
            from_f32(acc, o);
            yb[(size_t)i * H * P + p] = o;
        }
        __syncthreads();
    }
}

hipError_t launch_tree_ssd_fma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                               const float *A, const void *Bm, const void *Cm, const float *D,
                               const float *h0, void *y, int32_t *status, hipStream_t st) {
    const dim3 grid(d.nheads, d.batch);
    if (d.io_dtype == STREE_BF16)
        hipLaunchKernelGGL(tree_ssd_fma_kernel<bf16_t>, grid, dim3(kThreads), 0, st, parent, d.nnodes, d.nheads,
                           d.headdim, d.dstate, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, A,
                           (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D, h0,
                           (bf16_t *)y, status);
    else
        hipLaunchKernelGGL(tree_ssd_fma_kernel<float>, grid, dim3(kThreads), 0, st, parent, d.nnodes, d.nheads,
                           d.headdim, d.dstate, d.ngroups, (const float *)x, (long)d.x_stride_n, dt, A,
                           (const float *)Bm, (long)d.b_stride_n, (const float *)Cm, (long)d.c_stride_n, D, h0,
                           (float *)y, status);
    return hipGetLastError();
}

}  // namespace stree
