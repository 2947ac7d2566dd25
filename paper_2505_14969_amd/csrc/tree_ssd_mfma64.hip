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
//             waves 0-3: phase 1  Yt = h0b C^T, *= exp(s_i)
//             waves 4-7: phase 2  Gt = B C^T -> M (mask, decay) -> LDS      (concurrently)
//             barrier
//             waves 0-3: phase 3  Yt += Xt M^T ;  y = Yt + D x -> bf16 rows in LDS
//             barrier
#include "common.hpp"
#include "launch.hpp"

#ifndef STREE_PHASE_CLOCK
#define STREE_PHASE_CLOCK(k)
#endif
#ifndef STREE_PHASE_CLOCK_G
#define STREE_PHASE_CLOCK_G(k)
#endif

namespace stree {

namespace {

constexpr int kB64 = 64;
constexpr int kNP64 = kB64 + 8;
constexpr int kT64 = 512;   // 8 waves: 4 own Yt tiles, 3 own Gt tiles, 1 builds the tree index

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

// WPE = waves per SIMD the register budget is sized for: 4 when two workgroups fit a CU's LDS
template <int P, int S, int WPE>
__global__ __launch_bounds__(kT64) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void tree_ssd_mfma64_kernel(
    const int32_t *__restrict__ parent, int n, int nbatch, int H, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ A, const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const float *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status) {
    using L = Lds64<P, S>;
    constexpr int SP = L::SP, YOP = L::YOP;
    constexpr int NC = kB64 * (S / 8) / kT64;   // 16-byte chunks of C (and B) per thread
    constexpr int NX = kB64 * (P / 8) / kT64;   // of x
    constexpr int NH = P * S / 4 / kT64;        // float4 chunks of h0 per thread
    constexpr int YT = (P / 32) * 2, YQ = YT / 4;   // Yt tiles, tiles per Y wave
    static_assert(NC >= 1 && NX >= 1 && NH >= 1 && YQ >= 1, "tile too small for 512 threads");
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

    // Waves 0-3 own the Yt tiles (phases 1 and 3), waves 4-7 the Gt tiles (phase 2).  The
    // Gt tile of wave 6 is (j >= 32, i < 32): all zero since j > i, so wave 6 builds the
    // tree index instead and its lanes carry parent[] and dt[].
    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    constexpr int kTreeWave = 6;
    const int it = wave & 1;             // node half of the tiles this wave owns
    const int il = it * 32 + l32;        // this lane's node in accumulators
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

    // per-thread offsets of the 16-byte chunks never change from unit to unit: one 32-bit
    // offset per tensor, the unit's base pointer and the per-chunk row step are uniform.
    // Rows >= n are read from row n-1 (valid memory) and zeroed afterwards: no branches.
    constexpr int kRowsC = kT64 / (S / 8), kRowsX = kT64 / (P / 8);
    const int rc0 = tid / (S / 8), cc0 = tid % (S / 8), rx0 = tid / (P / 8), cx0 = tid % (P / 8);
    uint32_t offC[NC], offB[NC], offX[NX];
#pragma unroll
    for (int q = 0; q < NC; ++q) {
        const int rr = min(rc0 + q * kRowsC, n - 1);
        offC[q] = (uint32_t)(rr * (int)c_sn + cc0 * 8) * 2u;
        offB[q] = (uint32_t)(rr * (int)b_sn + cc0 * 8) * 2u;
    }
#pragma unroll
    for (int q = 0; q < NX; ++q) offX[q] = (uint32_t)(min(rx0 + q * kRowsX, n - 1) * (int)x_sn + cx0 * 8) * 2u;

    auto issue_loads = [&](int b, int h) {
        const int g = h / hpg;
        const char *Cb = reinterpret_cast<const char *>(Cm + (size_t)b * n * c_sn + (size_t)g * S);
        const char *Bb = reinterpret_cast<const char *>(Bm + (size_t)b * n * b_sn + (size_t)g * S);
        const char *xb = reinterpret_cast<const char *>(x + (size_t)b * n * x_sn + (size_t)h * P);
        if (wave == kTreeWave) {
            const int node = min(lane, n - 1);
            rpar = parent[(size_t)b * n + node];
            rdt = dt[((size_t)b * n + node) * H + h];
        }
        rA = A[h];
        rD = D ? D[h] : 0.f;
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            rC[q] = *reinterpret_cast<const uint4 *>(Cb + offC[q]);
            rB[q] = *reinterpret_cast<const uint4 *>(Bb + offB[q]);
        }
#pragma unroll
        for (int q = 0; q < NX; ++q) rX[q] = *reinterpret_cast<const uint4 *>(xb + offX[q]);
        if (h0) {
            const char *hb = reinterpret_cast<const char *>(h0 + ((size_t)b * H + h) * P * S);
#pragma unroll
            for (int q = 0; q < NH; ++q)
                rH[q] = *reinterpret_cast<const float4 *>(hb + (uint32_t)(tid + q * kT64) * 16u);
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
                const int idx = tid + q * kT64, rr = idx / (P / 8), c = idx % (P / 8);
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
        // ---- registers -> LDS; the tree wave builds the index first ------------------------------
        if (wave == kTreeWave) {
            const int bad = wave_tree_index(lane, n, rpar, rdt, A_h, sS, sDt, sMask);
            if (lane == 0) *sBad = bad;
        }
        STREE_PHASE_CLOCK(1);
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int rr = rc0 + q * kRowsC;
            const uint32_t keep = rr < n ? 0xffffffffu : 0u;   // zero the rows beyond the tree
            *reinterpret_cast<uint4 *>(&sC[rr * SP + cc0 * 8]) =
                make_uint4(rC[q].x & keep, rC[q].y & keep, rC[q].z & keep, rC[q].w & keep);
            *reinterpret_cast<uint4 *>(&sB[rr * SP + cc0 * 8]) =
                make_uint4(rB[q].x & keep, rB[q].y & keep, rB[q].z & keep, rB[q].w & keep);
        }
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int rr = rx0 + q * kRowsX, c = cx0;
            const uint32_t keep = rr < n ? 0xffffffffu : 0u;
            const uint32_t wv[4] = {rX[q].x & keep, rX[q].y & keep, rX[q].z & keep, rX[q].w & keep};
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
                const int e = (tid + q * kT64) * 4, p = e / S, s = e % S;
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

        if (!bad) {
            const bf16_t *cp = &sC[il * SP + 8 * lh];
            if (wave < 4) {
                // ---- phase 1 (Y waves): Yt = h0b C^T, then *= exp(s_i) ----------------------------
                if (h0) {
                    // fragments of half the state index are read in one batch, then consumed
#pragma unroll
                    for (int kb = 0; kb < S; kb += S / 2) {
                        bf16x8 cf[S / 32], hf[YQ][S / 32];
#pragma unroll
                        for (int j = 0; j < S / 32; ++j) {
                            cf[j] = *reinterpret_cast<const bf16x8 *>(cp + kb + 16 * j);
#pragma unroll
                            for (int q = 0; q < YQ; ++q)
                                hf[q][j] = *reinterpret_cast<const bf16x8 *>(
                                    &sH[(((wave + 4 * q) >> 1) * 32 + l32) * SP + 8 * lh + kb + 16 * j]);
                        }
#pragma unroll
                        for (int j = 0; j < S / 32; ++j)
#pragma unroll
                            for (int q = 0; q < YQ; ++q)
                                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hf[q][j], cf[j], acc[q], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);   // keep the two batches apart: register budget
                    }
                    const float e = __expf(sS[il]);
#pragma unroll
                    for (int q = 0; q < YQ; ++q)
#pragma unroll
                        for (int rg = 0; rg < 16; ++rg) acc[q][rg] *= e;
                }
            } else if (wave != kTreeWave) {
                // ---- phase 2 (G waves): Gt = B C^T, mask and decay -> M[i][j] as bf16 --------------
                const int jt = (wave - 4) >> 1;
                STREE_PHASE_CLOCK_G(9);
                floatx16 gt;
#pragma unroll
                for (int e = 0; e < 16; ++e) gt[e] = 0.f;
                const bf16_t *bp = &sB[(jt * 32 + l32) * SP + 8 * lh];
#pragma unroll
                for (int kb = 0; kb < S; kb += S / 2) {
                    bf16x8 cf[S / 32], bf[S / 32];
#pragma unroll
                    for (int j = 0; j < S / 32; ++j) {
                        cf[j] = *reinterpret_cast<const bf16x8 *>(cp + kb + 16 * j);
                        bf[j] = *reinterpret_cast<const bf16x8 *>(bp + kb + 16 * j);
                    }
#pragma unroll
                    for (int j = 0; j < S / 32; ++j)
                        gt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bf[j], cf[j], gt, 0, 0, 0);
                    __builtin_amdgcn_sched_barrier(0);
                }
                STREE_PHASE_CLOCK_G(10);
                const float s_i = sS[il];
                const uint32_t mrow = sMask[il * 2 + jt] >> (4 * lh);   // bit 8*rg + e <-> j = jl + e
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
                        const bool on = (mrow >> (8 * rg + e)) & 1u;
                        const float v = on ? gt[4 * rg + e] * __expf(s_i - sjv[e]) * djv[e] : 0.f;
                        o[e] = (bf16_t)v;
                    }
                    *reinterpret_cast<bf16x4 *>(&sM[il * kNP64 + jl]) = o;
                }
                STREE_PHASE_CLOCK_G(11);
            }
        }
        STREE_PHASE_CLOCK(5);
        __syncthreads();
        STREE_PHASE_CLOCK(6);

        // ---- phase 3 (Y waves): Yt += Xt M^T over j <= i only (nodes i < 32 have no ancestor
        //      j >= 32, that quadrant of M is never written or read); y = Yt + D x -> bf16 rows ---
        if (wave < 4) {
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int pt = (wave + 4 * q) >> 1;
                if (!bad) {
                    const bf16_t *ap = reinterpret_cast<const bf16_t *>(sXT) + (pt * 32 + l32) * kNP64 + 8 * lh;
                    const bf16_t *bp = &sM[il * kNP64 + 8 * lh];
                    const int kend = it ? kB64 : 32;
                    for (int k0 = 0; k0 < kend; k0 += 16) {
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
        STREE_PHASE_CLOCK(7);
        __syncthreads();
        STREE_PHASE_CLOCK(8);
    }
    flush_y();
}

template <int P, int S>
hipError_t launch64_ps(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                       const void *Bm, const void *Cm, const float *D, const float *h0, void *y,
                       int32_t *status, hipStream_t st) {
    constexpr size_t lds = Lds64<P, S>::total;
    constexpr int WPE = (2 * (lds + 64) <= 160 * 1024) ? 4 : 2;
    static bool attr_set = false;  // dynamic LDS above 64 KB needs the attribute once
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(&tree_ssd_mfma64_kernel<P, S, WPE>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    const int n_units = d.batch * d.nheads;
    const int per_cu = (int)((160 * 1024) / (lds + 64));      // resident workgroups per CU by LDS
    int grid = (n_units + 7) / 8 * 8;
    const int cap = 256 * (per_cu < 1 ? 1 : per_cu);
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((tree_ssd_mfma64_kernel<P, S, WPE>), dim3(grid), dim3(kT64), lds, st, parent, d.nnodes,
                       d.batch, d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, A,
                       (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D, h0,
                       (bf16_t *)y, status);
    return hipGetLastError();
}

}  // namespace

bool tree_ssd_mfma64_supported(const stree_dims &d) {
    if (d.nnodes > kB64) return false;
    const int P = d.headdim, S = d.dstate;
    return (P == 64 && (S == 128 || S == 64)) || (P == 128 && S == 128);
}

hipError_t launch_tree_ssd_mfma64(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D,
                                  const float *h0, void *y, int32_t *status, hipStream_t st) {
    const int P = d.headdim, S = d.dstate;
    if (P == 64 && S == 128) return launch64_ps<64, 128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (P == 64 && S == 64) return launch64_ps<64, 64>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (P == 128 && S == 128) return launch64_ps<128, 128>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    return hipErrorInvalidValue;
}

}  // namespace stree
