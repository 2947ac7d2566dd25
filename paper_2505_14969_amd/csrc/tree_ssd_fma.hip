// Plain fp32-FMA tree scan: covers every shape in the library's envelope (any
// headdim/dstate <= 256, fp32 or bf16 storage, any alignment).  One workgroup per
// (batch, head); all arithmetic in fp32.  This is the fp32 path (1e-4 parity)
// and the fallback for shapes the MFMA kernels do not take.
//
// Per block of 16 rows i:   Wt[ii][j] = L_ij * <C_i,B_j> * exp(s_i - s_j) * dt_j
//                           y_i = exp(s_i) * h0 C_i + sum_j Wt[ii][j] x_j + D x_i
// Operands pass through LDS as fp32 tiles so that global memory is read with the lanes of a wave
// on consecutive elements and the inner products run from LDS: the C rows of the block, the B
// rows 16 at a time (the scores), the state 32 columns of the state index at a time (the h0
// term, accumulated per output element in an LDS tile between those pieces).
#include "common.hpp"
#include "launch.hpp"

namespace stree {

constexpr int kFmaRows = 16;
constexpr int kFmaSC = 32;     // state-index columns of h0 per piece

// dynamic LDS, in floats: C rows [16][S+1] | B rows [16][S+1] or h0 piece [P][33] | y tile [16][P]
__host__ __device__ constexpr size_t fma_lds_floats(int P, int S) {
    const size_t rows = (size_t)kFmaRows * (S + 1), piece = (size_t)P * (kFmaSC + 1);
    return rows + (rows > piece ? rows : piece) + (size_t)kFmaRows * P;
}

template <typename T, typename HT>
__global__ __launch_bounds__(kThreads) void tree_ssd_fma_kernel(
    const int32_t *__restrict__ parent, int n, int H, int P, int S, int G, const T *__restrict__ x,
    long x_sn, const float *__restrict__ dt, const float *__restrict__ dt_bias, const float *__restrict__ A,
    const T *__restrict__ Bm,
    long b_sn, const T *__restrict__ Cm, long c_sn, const float *__restrict__ D,
    const HT *__restrict__ h0, T *__restrict__ y, int32_t *__restrict__ status) {
    extern __shared__ __align__(16) float dyn[];
    __shared__ TreeLds tree;
    __shared__ uint32_t mask[kMaxNodes * kMaxWords];
    __shared__ float Wt[kFmaRows][kMaxNodes];
    const int tid = threadIdx.x, h = blockIdx.x, b = blockIdx.y;
    const int g = h / (H / G);
    const int words = (n + 31) / 32;
    const float A_h = A[h];
    const float dt_i = tid < n ? step_size(dt[((size_t)b * n + tid) * H + h], dt_bias, h) : 0.f;
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
    const HT *hb = h0 ? h0 + ((size_t)b * H + h) * P * S : nullptr;
    const float D_h = D ? D[h] : 0.f;
    const int SP1 = S + 1, HP1 = kFmaSC + 1;
    float *sCt = dyn, *sBH = dyn + kFmaRows * SP1;
    float *sY = sBH + max(kFmaRows * SP1, P * HP1);

    for (int i0 = 0; i0 < n; i0 += kFmaRows) {
        const int rows = min(kFmaRows, n - i0);
        const int ncol = i0 + rows;                       // columns 0 .. ncol-1 can hold ancestors
        __syncthreads();                                  // the previous block is done with every tile
        for (int idx = tid; idx < rows * S; idx += kThreads) {
            const int ii = idx / S, sidx = idx - ii * S;
            sCt[ii * SP1 + sidx] = to_f32(Cb[(size_t)(i0 + ii) * c_sn + sidx]);
        }
        // ---- decay-weighted masked scores, 16 columns at a time ------------------------------------
        for (int j0 = 0; j0 < ncol; j0 += kFmaRows) {
            const int cols = min(kFmaRows, ncol - j0);
            __syncthreads();                              // C rows staged / the last B rows consumed
            for (int idx = tid; idx < cols * S; idx += kThreads) {
                const int jj = idx / S, sidx = idx - jj * S;
                sBH[jj * SP1 + sidx] = to_f32(Bb[(size_t)(j0 + jj) * b_sn + sidx]);
            }
            __syncthreads();
            const int ii = tid >> 4, jj = tid & 15, i = i0 + ii, j = j0 + jj;
            if (ii < rows && jj < cols) {
                float wv = 0.f;
                if (mask_bit(mask, words, i, j)) {
                    const float *ci = sCt + ii * SP1, *bj = sBH + jj * SP1;
                    float dot = 0.f;
                    for (int sidx = 0; sidx < S; ++sidx) dot = fmaf(ci[sidx], bj[sidx], dot);
                    wv = dot * expf(tree.s[i] - tree.s[j]) * tree.dt[j];
                }
                Wt[ii][j] = wv;
            }
        }
        // ---- h0 term: y[ii][p] = sum_s h0[p][s] C[ii][s], a piece of the state index at a time ----------
        for (int idx = tid; idx < rows * P; idx += kThreads) sY[idx] = 0.f;
        if (hb) {
            for (int sc0 = 0; sc0 < S; sc0 += kFmaSC) {
                const int sc = min(kFmaSC, S - sc0);
                __syncthreads();                          // the B rows / the last piece consumed
                for (int idx = tid; idx < P * kFmaSC; idx += kThreads) {
                    const int p = idx / kFmaSC, sidx = idx - p * kFmaSC;
                    if (sidx < sc) sBH[p * HP1 + sidx] = to_f32(hb[(size_t)p * S + sc0 + sidx]);
                }
                __syncthreads();
                for (int idx = tid; idx < rows * P; idx += kThreads) {
                    const int ii = idx / P, p = idx - ii * P;
                    const float *ci = sCt + ii * SP1 + sc0, *hp = sBH + p * HP1;
                    float acc = sY[idx];
                    for (int sidx = 0; sidx < sc; ++sidx) acc = fmaf(hp[sidx], ci[sidx], acc);
                    sY[idx] = acc;                        // (element idx belongs to this thread in every piece)
                }
            }
        }
        __syncthreads();                                  // the scores of the block are complete
        // ---- y_i = exp(s_i) (h0 term) + sum_j Wt x_j + D x_i: lanes along p ----------------------------
        for (int idx = tid; idx < rows * P; idx += kThreads) {
            const int ii = idx / P, p = idx - ii * P, i = i0 + ii;
            float acc = hb ? sY[idx] * expf(tree.s[i]) : 0.f;
            for (int j = 0; j <= i; ++j) {
                const float wv = Wt[ii][j];
                if (wv != 0.f) acc = fmaf(wv, to_f32(xb[(size_t)j * x_sn + p]), acc);
            }
            acc = fmaf(D_h, to_f32(xb[(size_t)i * x_sn + p]), acc);
            T o;
            from_f32(acc, o);
            yb[(size_t)i * H * P + p] = o;
        }
    }
}

template <typename T, typename HT>
static LdsLimit &fma_lds_limit() {
    static LdsLimit lim;
    return lim;
}

template <typename T, typename HT>
static hipError_t prepare_fma_t() {
    return fma_lds_limit<T, HT>().raise(reinterpret_cast<const void *>(&tree_ssd_fma_kernel<T, HT>),
                                        fma_lds_floats(256, 256) * sizeof(float));
}

template <typename T, typename HT>
static hipError_t launch_fma_t(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                               const float *A, const void *Bm, const void *Cm, const float *D, const void *h0,
                               void *y, int32_t *status, hipStream_t st) {
    const size_t lds = fma_lds_floats(d.headdim, d.dstate) * sizeof(float);
    if (lds > 48 * 1024) {   // beyond the default cap on dynamic LDS: raised once, to what headdim = dstate = 256 need
        const hipError_t e = fma_lds_limit<T, HT>().raise(reinterpret_cast<const void *>(&tree_ssd_fma_kernel<T, HT>),
                                                          fma_lds_floats(256, 256) * sizeof(float));
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL((tree_ssd_fma_kernel<T, HT>), dim3(d.nheads, d.batch), dim3(kThreads), lds, st, parent, d.nnodes,
                       d.nheads, d.headdim, d.dstate, d.ngroups, (const T *)x, (long)d.x_stride_n, dt, step_bias(d),
                       A, (const T *)Bm, (long)d.b_stride_n, (const T *)Cm, (long)d.c_stride_n, D,
                       (const HT *)h0, (T *)y, status);
    return hipGetLastError();
}

hipError_t prepare_tree_ssd_fma() {
    hipError_t e = prepare_fma_t<bf16_t, bf16_t>();
    if (e == hipSuccess) e = prepare_fma_t<bf16_t, float>();
    if (e == hipSuccess) e = prepare_fma_t<float, float>();
    return e;
}

hipError_t launch_tree_ssd_fma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                               const float *A, const void *Bm, const void *Cm, const float *D,
                               const void *h0, void *y, int32_t *status, hipStream_t st) {
    if (d.io_dtype == STREE_BF16) {                 // (a bf16 state goes with bf16 io only)
        if (d.state_dtype == STREE_BF16)
            return launch_fma_t<bf16_t, bf16_t>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
        return launch_fma_t<bf16_t, float>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    }
    return launch_fma_t<float, float>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
}

}  // namespace stree
