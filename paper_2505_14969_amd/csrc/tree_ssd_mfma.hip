// Tree scan on the bf16 MFMA units (gfx950, v_mfma_f32_32x32x16_bf16).
//
// One workgroup (4 waves) per (batch, head).  Nodes are processed in blocks of
// 64 rows I and 64 columns J <= I (labels are topological, so L_ij = 0 for
// j > i).  Every product is formed transposed, so that in all accumulators a
// lane owns one node i (n index of the MFMA) and the registers run over the
// other index; row scalings by exp(s_i) and the mask row of node i are then
// per-lane values:
//
//   phase 1   Yt[p][i]  = sum_s  h0b[p][s] * C[i][s]          then *= exp(s_i)
//   phase 2   Gt[j][i]  = sum_s  B[j][s]  * C[i][s]
//             M[i][j]   = L_ij ? Gt[j][i] * exp(s_i - s_j) * dt_j : 0   (select, never 0*inf)
//   phase 3   Yt[p][i] += sum_j  Xt[p][j] * M[i][j]
//   epilogue  y[i][p]   = Yt[p][i] + D * x[i][p]
//
// All MFMA operands are read from LDS rows that are contiguous in the
// contraction index, padded by 16 bytes per row against bank conflicts.
// MFMA operand layout (32x32x16): lane l holds row (l % 32) of its operand and
// the 8 contraction indices 8*(l/32)..+7; accumulator register r of lane l is
// element [8*(r/4) + 4*(l/32) + r%4][l % 32].
#include "common.hpp"
#include "launch.hpp"

#ifndef STREE_PHASE_CLOCK
#define STREE_PHASE_CLOCK(k)
#endif

namespace stree {

constexpr int kBlk = 64;         // node block
constexpr int kNP = kBlk + 8;    // padded row of a [.. x 64] bf16 LDS tile

struct MfmaLdsPlan {
    int sp;                      // padded state row, elements
    size_t off_c, off_b, off_h, off_xt, off_m, off_mask, total;
};

__host__ __device__ inline MfmaLdsPlan mfma_lds_plan(int P, int S, int npad, int words) {
    MfmaLdsPlan pl;
    pl.sp = S + 8;
    const size_t c_bytes = (size_t)kBlk * pl.sp * 2;
    const size_t y_bytes = (size_t)kBlk * (P + 4) * 4;  // fp32 output staging shares the B tile
    size_t o = 0;
    pl.off_c = o; o += c_bytes;
    pl.off_b = o; o += (c_bytes > y_bytes ? c_bytes : y_bytes);
    pl.off_h = o; o += (size_t)P * pl.sp * 2;
    pl.off_xt = o; o += (size_t)P * kNP * 2;
    pl.off_m = o; o += (size_t)kBlk * kNP * 2;
    pl.off_mask = o; o += (size_t)npad * words * 4;
    pl.total = o;
    return pl;
}

template <int P>
__global__ __launch_bounds__(kThreads) void tree_ssd_mfma_kernel(
    const int32_t *__restrict__ parent, int n, int H, int S, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ A, const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const float *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status) {
    constexpr int YT = (P / 32) * 2;          // 32x32 tiles of Yt[p][i] per node block
    constexpr int YQ = (YT + 3) / 4;          // tiles per wave
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ TreeLds tree;

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    const int h = blockIdx.x, b = blockIdx.y;
    const int g = h / (H / G);
    const int npad = (n + kBlk - 1) / kBlk * kBlk;
    const int words = (n + 31) / 32;
    const MfmaLdsPlan pl = mfma_lds_plan(P, S, npad, words);
    const int SP = pl.sp;
    bf16_t *sC = reinterpret_cast<bf16_t *>(lds + pl.off_c);
    bf16_t *sB = reinterpret_cast<bf16_t *>(lds + pl.off_b);
    float *sY = reinterpret_cast<float *>(lds + pl.off_b);
    bf16_t *sH = reinterpret_cast<bf16_t *>(lds + pl.off_h);
    bf16_t *sXT = reinterpret_cast<bf16_t *>(lds + pl.off_xt);
    bf16_t *sM = reinterpret_cast<bf16_t *>(lds + pl.off_m);
    uint32_t *mask = reinterpret_cast<uint32_t *>(lds + pl.off_mask);

    STREE_PHASE_CLOCK(0);
    // ---- initial state -> bf16 MFMA operand rows sH[p][s] -------------------------------
    if (h0) {
        const float *hb = h0 + ((size_t)b * H + h) * P * S;
        for (int idx = tid; idx < P * S / 4; idx += kThreads) {
            const int e = idx * 4, p = e / S, s = e % S;
            const float4 v = *reinterpret_cast<const float4 *>(hb + e);
            bf16x4 o;
            o[0] = (bf16_t)v.x; o[1] = (bf16_t)v.y; o[2] = (bf16_t)v.z; o[3] = (bf16_t)v.w;
            *reinterpret_cast<bf16x4 *>(&sH[p * SP + s]) = o;
        }
    }
    STREE_PHASE_CLOCK(1);
    // ---- tree index: depth, mask rows L_i, s_i = (A_tree)_i ---------------------------
    const float A_h = A[h];
    const float dt_i = tid < n ? dt[((size_t)b * n + tid) * H + h] : 0.f;
    const int bad = build_tree_index(tree, mask, parent + (size_t)b * n, n, npad, words, dt_i, A_h);
    if (status && h == 0 && tid == 0) status[b] = bad;
    STREE_PHASE_CLOCK(2);
    bf16_t *yb = y + (size_t)b * n * H * P + (size_t)h * P;
    if (bad) {
        for (int idx = tid; idx < n * (P / 8); idx += kThreads) {
            const int r = idx / (P / 8), c = idx % (P / 8);
            *reinterpret_cast<uint4 *>(yb + (size_t)r * H * P + c * 8) = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    const bf16_t *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
    const bf16_t *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
    const bf16_t *Cb = Cm + (size_t)b * n * c_sn + (size_t)g * S;
    const float D_h = D ? D[h] : 0.f;
    const int s8 = S / 8;

    for (int i0 = 0; i0 < npad; i0 += kBlk) {
        // ---- C rows of this block -------------------------------------------------------
        for (int idx = tid; idx < kBlk * s8; idx += kThreads) {
            const int r = idx / s8, c = idx % s8, i = i0 + r;
            uint4 v = make_uint4(0, 0, 0, 0);
            if (i < n) v = *reinterpret_cast<const uint4 *>(Cb + (size_t)i * c_sn + c * 8);
            *reinterpret_cast<uint4 *>(&sC[r * SP + c * 8]) = v;
        }
        __syncthreads();
        STREE_PHASE_CLOCK(3);

        floatx16 acc[YQ];
#pragma unroll
        for (int q = 0; q < YQ; ++q)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;

        // ---- phase 1: Yt = h0b * C^T, scaled by exp(s_i) -------------------------------
        if (h0) {
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int t = wave + 4 * q;
                if (t < YT) {
                    const int it = t & 1, pt = t >> 1;
                    const bf16_t *ap = &sH[(pt * 32 + l32) * SP + 8 * lh];
                    const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
                    for (int k0 = 0; k0 < S; k0 += 16) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ap + k0);
                        const bf16x8 bb = *reinterpret_cast<const bf16x8 *>(bp + k0);
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[q], 0, 0, 0);
                    }
                    const float e = __expf(tree.s[i0 + it * 32 + l32]);
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[q][r] *= e;
                }
            }
        }

        STREE_PHASE_CLOCK(4);
        for (int j0 = 0; j0 <= i0; j0 += kBlk) {
            // ---- skip column blocks that hold no ancestor of this row block ------------
            if (j0 < i0) {
                int any = 0;
                if (tid < kBlk && i0 + tid < n) {
                    const int wj = j0 >> 5;
                    any = (mask[(i0 + tid) * words + wj] | mask[(i0 + tid) * words + wj + 1]) != 0u;
                }
                if (!__syncthreads_or(any)) continue;
            }
            // ---- B rows and X^T of the column block ---------------------------------------
            for (int idx = tid; idx < kBlk * s8; idx += kThreads) {
                const int r = idx / s8, c = idx % s8, j = j0 + r;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (j < n) v = *reinterpret_cast<const uint4 *>(Bb + (size_t)j * b_sn + c * 8);
                *reinterpret_cast<uint4 *>(&sB[r * SP + c * 8]) = v;
            }
            for (int idx = tid; idx < kBlk * (P / 8); idx += kThreads) {
                const int r = idx / (P / 8), c = idx % (P / 8), j = j0 + r;
                uint4 v = make_uint4(0, 0, 0, 0);
                if (j < n) v = *reinterpret_cast<const uint4 *>(xb + (size_t)j * x_sn + c * 8);
                // (every lane of the wave is here: kBlk * P/8 is a multiple of the workgroup size)
                store_transposed_pair<P / 8>(reinterpret_cast<unsigned short *>(sXT), kNP, r, c * 8, v, lane);
            }
            __syncthreads();
            STREE_PHASE_CLOCK(5);

            // ---- phase 2: Gt = B * C^T; mask and decay -> M[i][j] as bf16 ----------------
            {
                const int it = wave & 1, jt = wave >> 1;
                floatx16 gt;
#pragma unroll
                for (int r = 0; r < 16; ++r) gt[r] = 0.f;
                const bf16_t *ap = &sB[(jt * 32 + l32) * SP + 8 * lh];
                const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
                for (int k0 = 0; k0 < S; k0 += 16) {
                    const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ap + k0);
                    const bf16x8 bb = *reinterpret_cast<const bf16x8 *>(bp + k0);
                    gt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, gt, 0, 0, 0);
                }
                const int il = it * 32 + l32, i = i0 + il;
                const int wj = (j0 >> 5) + jt;
                const uint32_t mrow = (i < n && wj < words) ? mask[i * words + wj] : 0u;
                const float s_i = tree.s[i];
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int jl = jt * 32 + 8 * rg + 4 * lh;      // first of 4 consecutive j
                    const float4 sj = *reinterpret_cast<const float4 *>(&tree.s[j0 + jl]);
                    const float4 dj = *reinterpret_cast<const float4 *>(&tree.dt[j0 + jl]);
                    const float sjv[4] = {sj.x, sj.y, sj.z, sj.w};
                    const float djv[4] = {dj.x, dj.y, dj.z, dj.w};
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const bool on = (mrow >> (8 * rg + 4 * lh + e)) & 1u;
                        const float v = on ? gt[4 * rg + e] * __expf(s_i - sjv[e]) * djv[e] : 0.f;
                        o[e] = (bf16_t)v;
                    }
                    *reinterpret_cast<bf16x4 *>(&sM[il * kNP + jl]) = o;
                }
            }
            __syncthreads();
            STREE_PHASE_CLOCK(6);

            // ---- phase 3: Yt += Xt * M^T ---------------------------------------------------
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int t = wave + 4 * q;
                if (t < YT) {
                    const int it = t & 1, pt = t >> 1;
                    const bf16_t *ap = &sXT[(pt * 32 + l32) * kNP + 8 * lh];
                    const bf16_t *bp = &sM[(it * 32 + l32) * kNP + 8 * lh];
#pragma unroll
                    for (int k0 = 0; k0 < kBlk; k0 += 16) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ap + k0);
                        const bf16x8 bb = *reinterpret_cast<const bf16x8 *>(bp + k0);
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[q], 0, 0, 0);
                    }
                }
            }
            __syncthreads();
        }
        STREE_PHASE_CLOCK(7);

        // ---- epilogue: stage fp32 Y rows (over the dead B tile), add D*x, store bf16 -----
#pragma unroll
        for (int q = 0; q < YQ; ++q) {
            const int t = wave + 4 * q;
            if (t < YT) {
                const int it = t & 1, pt = t >> 1;
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const float4 v = make_float4(acc[q][4 * rg], acc[q][4 * rg + 1], acc[q][4 * rg + 2], acc[q][4 * rg + 3]);
                    *reinterpret_cast<float4 *>(&sY[(it * 32 + l32) * (P + 4) + pt * 32 + 8 * rg + 4 * lh]) = v;
                }
            }
        }
        __syncthreads();
        for (int idx = tid; idx < kBlk * (P / 8); idx += kThreads) {
            const int r = idx / (P / 8), c = idx % (P / 8), i = i0 + r;
            if (i < n) {
                const float4 a0 = *reinterpret_cast<const float4 *>(&sY[r * (P + 4) + c * 8]);
                const float4 a1 = *reinterpret_cast<const float4 *>(&sY[r * (P + 4) + c * 8 + 4]);
                const uint4 xv = *reinterpret_cast<const uint4 *>(xb + (size_t)i * x_sn + c * 8);
                bf16x8 o;
                o[0] = (bf16_t)fmaf(D_h, bf16_lo(xv.x), a0.x);
                o[1] = (bf16_t)fmaf(D_h, bf16_hi(xv.x), a0.y);
                o[2] = (bf16_t)fmaf(D_h, bf16_lo(xv.y), a0.z);
                o[3] = (bf16_t)fmaf(D_h, bf16_hi(xv.y), a0.w);
                o[4] = (bf16_t)fmaf(D_h, bf16_lo(xv.z), a1.x);
                o[5] = (bf16_t)fmaf(D_h, bf16_hi(xv.z), a1.y);
                o[6] = (bf16_t)fmaf(D_h, bf16_lo(xv.w), a1.z);
                o[7] = (bf16_t)fmaf(D_h, bf16_hi(xv.w), a1.w);
                *reinterpret_cast<bf16x8 *>(yb + (size_t)i * H * P + c * 8) = o;
            }
        }
        // the next block's C load and its barrier separate these sY reads from the next B load
    }
    STREE_PHASE_CLOCK(8);
}

bool tree_ssd_mfma_supported(const stree_dims &d, const void *x, const void *Bm, const void *Cm,
                             const float *h0, const void *y) {
    if (d.io_dtype != STREE_BF16) return false;
    if (!(d.headdim == 32 || d.headdim == 64 || d.headdim == 128)) return false;
    if (d.dstate % 16 != 0 || d.dstate < 16) return false;
    if ((d.x_stride_n | d.b_stride_n | d.c_stride_n) % 8 != 0) return false;
    const uintptr_t bits = (uintptr_t)x | (uintptr_t)Bm | (uintptr_t)Cm | (uintptr_t)h0 | (uintptr_t)y;
    if (bits % 16 != 0) return false;
    const int npad = (d.nnodes + kBlk - 1) / kBlk * kBlk;
    return mfma_lds_plan(d.headdim, d.dstate, npad, (d.nnodes + 31) / 32).total + sizeof(TreeLds) <= 160 * 1024;
}

template <int P>
static hipError_t launch_p(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                           const float *A, const void *Bm, const void *Cm, const float *D, const float *h0,
                           void *y, int32_t *status, hipStream_t st) {
    const int npad = (d.nnodes + kBlk - 1) / kBlk * kBlk;
    const size_t lds = mfma_lds_plan(P, d.dstate, npad, (d.nnodes + 31) / 32).total;
    static size_t lds_set = 0;  // raise the dynamic-LDS limit once per size (64 KB is the default cap)
    if (lds > lds_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_ssd_mfma_kernel<P>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        lds_set = lds;
    }
    hipLaunchKernelGGL(tree_ssd_mfma_kernel<P>, dim3(d.nheads, d.batch), dim3(kThreads), lds, st, parent, d.nnodes,
                       d.nheads, d.dstate, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, A,
                       (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D, h0,
                       (bf16_t *)y, status);
    return hipGetLastError();
}

hipError_t launch_tree_ssd_mfma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                const float *A, const void *Bm, const void *Cm, const float *D,
                                const float *h0, void *y, int32_t *status, hipStream_t st) {
    if (tree_ssd_mfma64_supported(d))
        return launch_tree_ssd_mfma64(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    switch (d.headdim) {
        case 32: return launch_p<32>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
        case 64: return launch_p<64>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
        case 128: return launch_p<128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace stree
