// Tree scan for trees of at most 64 nodes (one node block), the shape of a
// speculative-decoding step: persistent, software-pipelined variant of the MFMA
// kernel in tree_ssd_mfma.hip (same products, same accumulator layouts).
//
// A workgroup walks a list of (batch, head) units.  While it computes unit u
// from LDS, the global loads of its next unit (h0 32 KB, x, B, C, parent, dt)
// are already in flight into registers, so HBM latency is paid once per
// workgroup, not once per unit.  Units are dealt out so that all heads of one
// sequence land on the same XCD (workgroup id % 8), whose L2 then serves the
// B / C rows that the heads of a group share.
//
// Per unit:   regs -> LDS (C, B, X^T, h0 as bf16), wave 0 builds the tree index
//             barrier; issue next unit's loads; store the previous unit's y rows from LDS
//             phases 1+2 in one sweep over the state index (shared C fragment):
//                      Yt = h0b C^T, *= exp(s_i);  Gt = B C^T -> M (mask, decay) -> LDS
//             barrier
//             phase 3  Yt += Xt M^T ;  y = Yt + D x -> bf16 rows in LDS
//             barrier
#include "common.hpp"
#include "launch.hpp"

#ifndef STREE_PHASE_CLOCK
#define STREE_PHASE_CLOCK(k)
#endif

namespace stree {

namespace {

constexpr int kB64 = 64;
constexpr int kNP64 = kB64 + 8;

template <int P, int S>
struct Lds64 {
    static constexpr int SP = S + 8;
    static constexpr int YOP = P + 8;   // padded bf16 output row
    static constexpr size_t c_bytes = (size_t)kB64 * SP * 2;
    static constexpr size_t off_c = 0;
    static constexpr size_t off_b = off_c + c_bytes;
    static constexpr size_t off_h = off_b + c_bytes;
    static constexpr size_t off_xt = off_h + (size_t)P * SP * 2;
    static constexpr size_t off_m = off_xt + (size_t)P * kNP64 * 2;
    static constexpr size_t off_yo = off_m + (size_t)kB64 * kNP64 * 2;
    static constexpr size_t off_s = off_yo + (size_t)kB64 * YOP * 2;     // float s[64]
    static constexpr size_t off_dt = off_s + 256;                       // float dt[64]
    static constexpr size_t off_mask = off_dt + 256;                    // uint32 mask[64][2]
    static constexpr size_t off_bad = off_mask + 512;                   // int
    static constexpr size_t total = off_bad + 16;
};

// Wave-level tree index for n <= 64: lane i owns node i; pointer doubling with
// cross-lane reads (ds_bpermute), no barriers.  Returns the status (uniform).
__device__ __forceinline__ int wave_tree_index(int lane, int n, int parent_i, float dt_i, float A_h, float *s_out,
                                               float *dt_out, uint32_t *mask_out) {
    int p = -1;
    bool ok = true;
    if (lane < n) {
        p = parent_i;
        ok = (lane == 0) ? (p == -1) : (p >= 0 && p < lane);
        if (!ok) p = -1;
    }
    const unsigned long long badmask = __ballot(!ok);
    if (badmask) return __ffsll((long long)badmask);  // first bad lane + 1
    float s = lane < n ? dt_i * A_h : 0.f;
    uint32_t mlo = (lane < 32) ? (1u << lane) : 0u, mhi = (lane >= 32) ? (1u << (lane - 32)) : 0u;
    if (lane >= n) mlo = mhi = 0u;
    for (int round = 0; round < 6; ++round) {
        if (!__any(p >= 0)) break;
        const int q = p >= 0 ? p : lane;
        const float rs = __shfl(s, q);
        const int rp = __shfl(p, q);
        const uint32_t rlo = __shfl(mlo, q), rhi = __shfl(mhi, q);
        if (p >= 0) {
            s += rs;
            mlo |= rlo;
            mhi |= rhi;
            p = rp;
        }
    }
    s_out[lane] = s;
    dt_out[lane] = lane < n ? dt_i : 0.f;
    mask_out[lane * 2] = mlo;
    mask_out[lane * 2 + 1] = mhi;
    return 0;
}

template <int P, int S>
__global__ __launch_bounds__(kThreads) void tree_ssd_mfma64_kernel(
    const int32_t *__restrict__ parent, int n, int nbatch, int H, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ A, const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const float *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status) {
    using L = Lds64<P, S>;
    constexpr int SP = L::SP, YOP = L::YOP;
    constexpr int NC = kB64 * (S / 8) / kThreads;   // 16-byte chunks of C (and B) per thread
    constexpr int NX = kB64 * (P / 8) / kThreads;   // of x
    constexpr int NH = P * S / 4 / kThreads;        // float4 chunks of h0 per thread
    constexpr int YT = (P / 32) * 2, YQ = (YT + 3) / 4;
    static_assert(NC >= 1 && NX >= 1 && NH >= 1, "tile too small for 256 threads");
    extern __shared__ __align__(16) unsigned char lds[];
    bf16_t *sC = reinterpret_cast<bf16_t *>(lds + L::off_c);
    bf16_t *sB = reinterpret_cast<bf16_t *>(lds + L::off_b);
    bf16_t *sYo = reinterpret_cast<bf16_t *>(lds + L::off_yo);
    bf16_t *sH = reinterpret_cast<bf16_t *>(lds + L::off_h);
    unsigned short *sXT = reinterpret_cast<unsigned short *>(lds + L::off_xt);
    bf16_t *sM = reinterpret_cast<bf16_t *>(lds + L::off_m);
    float *sS = reinterpret_cast<float *>(lds + L::off_s);
    float *sDt = reinterpret_cast<float *>(lds + L::off_dt);
    uint32_t *sMask = reinterpret_cast<uint32_t *>(lds + L::off_mask);
    int *sBad = reinterpret_cast<int *>(lds + L::off_bad);

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    const int n_units = nbatch * H;
    const int per_xcd = (n_units + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int rstep = gridDim.x >> 3;
    const int hpg = H / G;

    // unit r of this XCD -> (b, h); false when past the end
    auto decode = [&](int r, int &b, int &h) -> bool {
        const int logical = xcd * per_xcd + r;
        if (r >= per_xcd || logical >= n_units) return false;
        b = logical / H;
        h = logical - b * H;
        return true;
    };

    uint4 rC[NC], rB[NC], rX[NX];
    float4 rH[NH];
    int rpar = -1;
    float rdt = 0.f, rA = 0.f, rD = 0.f;

    auto issue_loads = [&](int b, int h) {
        const int g = h / hpg;
        const bf16_t *Cb = Cm + (size_t)b * n * c_sn + (size_t)g * S;
        const bf16_t *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
        const bf16_t *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
        if (tid < n) {
            rpar = parent[(size_t)b * n + tid];
            rdt = dt[((size_t)b * n + tid) * H + h];
        }
        rA = A[h];
        rD = D ? D[h] : 0.f;
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int idx = tid + q * kThreads, r = idx / (S / 8), c = idx % (S / 8);
            rC[q] = make_uint4(0, 0, 0, 0);
            rB[q] = make_uint4(0, 0, 0, 0);
            if (r < n) {
                rC[q] = *reinterpret_cast<const uint4 *>(Cb + (size_t)r * c_sn + c * 8);
                rB[q] = *reinterpret_cast<const uint4 *>(Bb + (size_t)r * b_sn + c * 8);
            }
        }
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int idx = tid + q * kThreads, r = idx / (P / 8), c = idx % (P / 8);
            rX[q] = make_uint4(0, 0, 0, 0);
            if (r < n) rX[q] = *reinterpret_cast<const uint4 *>(xb + (size_t)r * x_sn + c * 8);
        }
        if (h0) {
            const float *hb = h0 + ((size_t)b * H + h) * P * S;
#pragma unroll
            for (int q = 0; q < NH; ++q) rH[q] = *reinterpret_cast<const float4 *>(hb + (size_t)(tid + q * kThreads) * 4);
        }
    };

    int r = blockIdx.x >> 3, b = 0, h = 0;
    bool have = decode(r, b, h);
    if (have) issue_loads(b, h);

    // y rows of the previous unit wait in sYo and are stored while the next unit computes, so
    // that no store is outstanding when the loop top waits for its loads (on gfx9 loads and
    // stores share one counter and complete out of order with respect to each other)
    bf16_t *y_pending = nullptr;
    auto flush_y = [&]() {
        if (y_pending) {
#pragma unroll
            for (int q = 0; q < NX; ++q) {
                const int idx = tid + q * kThreads, rr = idx / (P / 8), c = idx % (P / 8);
                if (rr < n)
                    *reinterpret_cast<uint4 *>(y_pending + (size_t)rr * H * P + c * 8) =
                        *reinterpret_cast<const uint4 *>(&sYo[rr * YOP + c * 8]);
            }
        }
    };

    while (have) {
        [[maybe_unused]] const int prof_unit = b * H + h;  // only read by probe builds
        STREE_PHASE_CLOCK(0);
        const float A_h = rA, D_h = rD;
        // ---- registers -> LDS -----------------------------------------------------------------
        if (wave == 0) {
            const int bad = wave_tree_index(lane, n, rpar, rdt, A_h, sS, sDt, sMask);
            if (lane == 0) *sBad = bad;
        }
        STREE_PHASE_CLOCK(1);
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int idx = tid + q * kThreads, rr = idx / (S / 8), c = idx % (S / 8);
            *reinterpret_cast<uint4 *>(&sC[rr * SP + c * 8]) = rC[q];
            *reinterpret_cast<uint4 *>(&sB[rr * SP + c * 8]) = rB[q];
        }
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int idx = tid + q * kThreads, rr = idx / (P / 8), c = idx % (P / 8);
            const uint32_t wv[4] = {rX[q].x, rX[q].y, rX[q].z, rX[q].w};
            unsigned short *dst = sXT + (c * 8) * kNP64 + rr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[(2 * e) * kNP64] = (unsigned short)(wv[e] & 0xffffu);
                dst[(2 * e + 1) * kNP64] = (unsigned short)(wv[e] >> 16);
            }
        }
        if (h0) {
#pragma unroll
            for (int q = 0; q < NH; ++q) {
                const int e = (tid + q * kThreads) * 4, p = e / S, s = e % S;
                bf16x4 o;
                o[0] = (bf16_t)rH[q].x; o[1] = (bf16_t)rH[q].y; o[2] = (bf16_t)rH[q].z; o[3] = (bf16_t)rH[q].w;
                *reinterpret_cast<bf16x4 *>(&sH[p * SP + s]) = o;
            }
        }
        STREE_PHASE_CLOCK(2);
        __syncthreads();
        STREE_PHASE_CLOCK(3);

        // ---- next unit's loads go out now and fly during the compute below; so do the
        //      previous unit's y rows ---------------------------------------------------------
        const int cb = b, ch = h;
        r += rstep;
        have = decode(r, b, h);
        if (have) issue_loads(b, h);
        flush_y();
        y_pending = y + (size_t)cb * n * H * P + (size_t)ch * P;
        STREE_PHASE_CLOCK(4);

        const int bad = *sBad;
        if (status && ch == 0 && tid == 0) status[cb] = bad;

        floatx16 acc[YQ];
#pragma unroll
        for (int q = 0; q < YQ; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
        const int it = wave & 1;            // node half of every tile this wave owns
        const int il = it * 32 + l32;       // this lane's node

        if (!bad) {
            // ---- phases 1 and 2 in one sweep over the state index: the C fragment feeds both
            //      Yt = h0b C^T and Gt = B C^T -----------------------------------------------------
            const int jt = wave >> 1;
            const bool gt_live = !(jt == 1 && it == 0);   // j > i everywhere in that tile
            floatx16 gt;
#pragma unroll
            for (int e = 0; e < 16; ++e) gt[e] = 0.f;
            const bf16_t *cp = &sC[il * SP + 8 * lh];
            const bf16_t *bp = &sB[(jt * 32 + l32) * SP + 8 * lh];
#pragma unroll
            for (int k0 = 0; k0 < S; k0 += 16) {
                const bf16x8 cf = *reinterpret_cast<const bf16x8 *>(cp + k0);
                if (h0) {
#pragma unroll
                    for (int q = 0; q < YQ; ++q) {
                        const int t = wave + 4 * q;
                        if (t < YT) {
                            const bf16x8 hf = *reinterpret_cast<const bf16x8 *>(&sH[((t >> 1) * 32 + l32) * SP + 8 * lh + k0]);
                            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hf, cf, acc[q], 0, 0, 0);
                        }
                    }
                }
                if (gt_live) {
                    const bf16x8 bf = *reinterpret_cast<const bf16x8 *>(bp + k0);
                    gt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf, cf, gt, 0, 0, 0);
                }
            }
            STREE_PHASE_CLOCK(5);
            const float s_i = sS[il];
            if (h0) {
                const float e = __expf(s_i);
#pragma unroll
                for (int q = 0; q < YQ; ++q)
#pragma unroll
                    for (int rg = 0; rg < 16; ++rg) acc[q][rg] *= e;
            }
            STREE_PHASE_CLOCK(6);
            // ---- mask and decay: M[i][j] = L_ij ? Gt[j][i] exp(s_i - s_j) dt_j : 0 (select) -----
            const uint32_t mrow = sMask[il * 2 + jt];
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int jl = jt * 32 + 8 * rg + 4 * lh;
                const float4 sj = *reinterpret_cast<const float4 *>(&sS[jl]);
                const float4 dj = *reinterpret_cast<const float4 *>(&sDt[jl]);
                const float sjv[4] = {sj.x, sj.y, sj.z, sj.w};
                const float djv[4] = {dj.x, dj.y, dj.z, dj.w};
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const bool on = (mrow >> (8 * rg + 4 * lh + e)) & 1u;
                    const float v = on ? gt[4 * rg + e] * __expf(s_i - sjv[e]) * djv[e] : 0.f;
                    o[e] = (bf16_t)v;
                }
                *reinterpret_cast<bf16x4 *>(&sM[il * kNP64 + jl]) = o;
            }
        }
        STREE_PHASE_CLOCK(7);
        __syncthreads();
        STREE_PHASE_CLOCK(8);

        // ---- phase 3: Yt += Xt M^T; y = Yt + D x as bf16 into the output staging rows -----------
#pragma unroll
        for (int q = 0; q < YQ; ++q) {
            const int t = wave + 4 * q;
            if (t < YT) {
                const int pt = t >> 1;
                if (!bad) {
                    const bf16_t *ap = reinterpret_cast<const bf16_t *>(sXT) + (pt * 32 + l32) * kNP64 + 8 * lh;
                    const bf16_t *bp = &sM[il * kNP64 + 8 * lh];
#pragma unroll
                    for (int k0 = 0; k0 < kB64; k0 += 16) {
                        const bf16x8 a = *reinterpret_cast<const bf16x8 *>(ap + k0);
                        const bf16x8 bb = *reinterpret_cast<const bf16x8 *>(bp + k0);
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bb, acc[q], 0, 0, 0);
                    }
                }
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int p0 = pt * 32 + 8 * rg + 4 * lh;
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const float xv = __uint_as_float((uint32_t)sXT[(p0 + e) * kNP64 + il] << 16);
                        o[e] = bad ? (bf16_t)0.f : (bf16_t)fmaf(D_h, xv, acc[q][4 * rg + e]);
                    }
                    *reinterpret_cast<bf16x4 *>(&sYo[il * YOP + p0]) = o;
                }
            }
        }
        STREE_PHASE_CLOCK(9);
        __syncthreads();
        STREE_PHASE_CLOCK(10);
    }
    flush_y();
}

template <int P, int S>
hipError_t launch64_ps(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                       const void *Bm, const void *Cm, const float *D, const float *h0, void *y,
                       int32_t *status, hipStream_t st) {
    constexpr size_t lds = Lds64<P, S>::total;
    static bool attr_set = false;  // dynamic LDS above 64 KB needs the attribute once
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_ssd_mfma64_kernel<P, S>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_units = d.batch * d.nheads;
    const int per_cu = (int)((160 * 1024) / (lds + 64));      // resident workgroups per CU by LDS
    int grid = (n_units + 7) / 8 * 8;
    const int cap = 256 * (per_cu < 1 ? 1 : per_cu);
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((tree_ssd_mfma64_kernel<P, S>), dim3(grid), dim3(kThreads), lds, st, parent, d.nnodes,
                       d.batch, d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, A,
                       (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D, h0,
                       (bf16_t *)y, status);
    return hipGetLastError();
}

}  // namespace

bool tree_ssd_mfma64_supported(const stree_dims &d) {
    if (d.nnodes > kB64) return false;
    const int P = d.headdim, S = d.dstate;
    return (P == 64 && (S == 128 || S == 64)) || (P == 128 && S == 128) || (P == 32 && S == 128);
}

hipError_t launch_tree_ssd_mfma64(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D,
                                  const float *h0, void *y, int32_t *status, hipStream_t st) {
    const int P = d.headdim, S = d.dstate;
    if (P == 64 && S == 128) return launch64_ps<64, 128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (P == 64 && S == 64) return launch64_ps<64, 64>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (P == 128 && S == 128) return launch64_ps<128, 128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (P == 32 && S == 128) return launch64_ps<32, 128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    return hipErrorInvalidValue;
}

}  // namespace stree
