// Tree scan for trees of at most 64 nodes (one node block), the shape of a
// speculative-decoding step: persistent, software-pipelined, wave-specialised
// variant of the MFMA kernel in tree_ssd_mfma.hip (same products, same
// accumulator layouts).
//
// A workgroup of 8 waves walks a list of (batch, head) units.  Units are dealt
// out so that all heads of one sequence land on the same XCD (workgroup id % 8),
// whose L2 then serves the B / C rows that the heads of a group share.
//
//   Y waves 0-3   own the four 32x32 tiles of Yt[p][i]; carry the h0 prefetch of even units
//   G waves 4,5,7 own the three live tiles of Gt[j][i]; carry the x prefetch and, with the
//   T wave  6     (its Gt tile has j > i everywhere; builds the tree index), the h0 prefetch
//                 of odd units: the h0 tiles of two future units are always in flight
//
// A workgroup's units are consecutive, so mostly heads of one sequence and
// group: C, B and Gt = B C^T are staged / computed once per run of such heads
// (CB^T once per group), only the decay weighting is redone per head.
//
// Steady state for unit k, with the registers already holding unit k+1:
//   barrier 1
//     Y: phase 1  Yt = h0b C^T, *= exp(s_i)
//     G: phase 2  (Gt = B C^T if the tiles are new) M = L ? Gt exp(s_i - s_j) dt_j : 0 -> LDS
//   barrier 2   (h0b tile and the tree arrays are dead from here on)
//     Y: phase 3  Yt += Xt M^T; y = Yt + D x -> bf16, stored straight from the accumulators
//     Y or G (whoever carries unit k+1): h0(k+1) regs -> LDS as bf16; issue h0(k+3) loads
//     G: new C tile if unit k+1 starts another sequence or group
//     T: tree index of unit k+1, issue parent/dt (k+2) loads
//     G: x(k+1) regs -> the other X^T tile in LDS, issue x(k+2) loads
// so the big global loads (h0, x) are in flight for a whole unit period.
#include "common.hpp"
#include "launch.hpp"

#ifndef STREE_PHASE_CLOCK
#define STREE_PHASE_CLOCK(k)
#endif
#ifndef STREE_PHASE_CLOCK_G
#define STREE_PHASE_CLOCK_G(k)
#endif
#ifndef STREE_PHASE_ENTRY
#define STREE_PHASE_ENTRY(u)
#define STREE_PHASE_PRO(slot, t)
#endif
#ifndef STREE_EXIT_POINT
#define STREE_EXIT_INIT
#define STREE_EXIT_POINT(n)
#endif


namespace stree {

namespace {

constexpr int kB64 = 64;
constexpr int kNP64 = kB64 + 8;
constexpr int kT64 = 512;   // 8 waves: 4 Y waves, 3 G waves, 1 tree wave

// static LDS of the kernel below (C, B, h0b tiles, two X^T tiles, M, tree arrays)
template <int P, int S>
struct Lds64 {
    static constexpr int SP = S + 8;
    static constexpr size_t total = (size_t)2 * kB64 * SP * 2 + (size_t)P * SP * 2 + (size_t)2 * P * kNP64 * 2 +
                                    (size_t)kB64 * kNP64 * 2 + 1040;
};

// Output stores that write through L2 (system scope): y is never read again by this kernel, and
// lines left dirty in the eight L2s would all be written back at once when the kernel ends.
__device__ __forceinline__ void store_through16(void *p, uint4 v) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 vv = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1" ::"v"(p), "v"(vv) : "memory");
}

// Wave-level tree index for n <= 64: lane i owns node i; pointer doubling with
// cross-lane reads (ds_bpermute), no barriers.  Returns the status (uniform).
// Outputs are in log2 units so that the decay is one v_exp_f32 per element:
//   s2[i] = log2(e) * s_i          u[j] = s2[j] - log2(dt_j)
//   exp(s_i - s_j) * dt_j = exp2(s2[i] - u[j])      (dt_j = 0 -> u = +inf -> 0)
__device__ __forceinline__ int wave_tree_index(int lane, int n, int parent_i, float dt_i, float A_h, float *s2_out,
                                               float *u_out, uint32_t *mask_out) {
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
    const float s2 = s * 1.44269504088896340736f;
    s2_out[lane] = s2;
    u_out[lane] = s2 - __log2f(lane < n ? dt_i : 0.f);
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
    constexpr int SP = L::SP;
    constexpr int kHalf = kT64 / 2;                 // threads per role group
    constexpr int NC = kB64 * (S / 8) / kHalf;      // 16-byte chunks of C (and of B) per G thread
    constexpr int NX = kB64 * (P / 8) / kHalf;      // of x per G thread; of y per Y thread
    constexpr int NH = P * S / 4 / kHalf;           // float4 chunks of h0 per Y thread
    constexpr int YT = (P / 32) * 2, YQ = YT / 4;   // Yt tiles, tiles per Y wave
    constexpr int kRowsC = kHalf / (S / 8), kRowsX = kHalf / (P / 8);
    static_assert(NC >= 1 && NX >= 1 && NH >= 1 && YQ >= 1, "tile too small for this thread count");
    // separate LDS objects (not slices of one array), so that the compiler knows that a write to
    // one tile cannot alias a read of another and does not serialise them
    __shared__ __align__(16) bf16_t sC[kB64 * SP];
    __shared__ __align__(16) bf16_t sB[kB64 * SP];
    __shared__ __align__(16) bf16_t sH[P * SP];
    __shared__ __align__(16) unsigned short sXT2[2][P * kNP64];   // X^T of units k and k+1
    __shared__ __align__(16) bf16_t sM[kB64 * kNP64];
    __shared__ __align__(16) float sS2[kB64];
    __shared__ __align__(16) float sU[kB64];
    __shared__ uint32_t sMask[kB64 * 2];
    __shared__ int sBad[1];
    __shared__ float sDh[1];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    constexpr int kTreeWave = 6;
    const bool isY = wave < 4;
    const int rt = tid & (kHalf - 1);    // thread index within its role group
    const int it = wave & 1;             // node half of the tiles this wave owns
    const int il = it * 32 + l32;        // this lane's node in accumulators
    const int n_units = nbatch * H;
    const int per_xcd = (n_units + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int wg = blockIdx.x >> 3, nwg = gridDim.x >> 3;   // this workgroup among its XCD's
    const int hpg = H / G;
    // XCD x owns the contiguous unit range [x*per_xcd, ...); its workgroups split that range
    // into contiguous runs, so a workgroup mostly sees consecutive heads of one sequence and
    // group: their C, B tiles, the tree mask and Gt = B C^T are then reused, not redone.
    const int cnt = max(0, min(per_xcd, n_units - xcd * per_xcd));
    const int u0 = xcd * per_xcd + (int)((long)wg * cnt / nwg);
    const int nU = xcd * per_xcd + (int)((long)(wg + 1) * cnt / nwg) - u0;
    // (b, h) of unit k by stepping from unit 0 (k is 0, 1 or 2 units ahead of a known one):
    // scalar adds and compares only, no division inside the unit loop
    const int ub0 = __builtin_amdgcn_readfirstlane(u0 / H), uh0 = __builtin_amdgcn_readfirstlane(u0 % H);
    auto step = [&](int &b, int &h) {
        if (++h == H) {
            h = 0;
            ++b;
        }
    };
    // a unit needs new C/B tiles when it is the first one or starts another sequence or group
    auto fresh_at = [&](int k, int h) -> bool { return k == 0 || h % hpg == 0; };

    // ---- prefetch registers and their loaders ---------------------------------------------------
    // per-thread chunk offsets never change from unit to unit; the unit's base pointer is uniform.
    // Rows >= n are read from row n-1 (valid memory) and zeroed when staged: no branches.
    // one register array serves both roles (a thread is either Y or G for its whole life):
    //   pre[0..NH)  h0 chunks (fp32 bits) of a future unit: the Y threads carry the even units
    //               of the run, the G threads the odd ones, so two units' h0 are in flight
    //   pre[NH..)   x chunks of the next unit (G threads)
    constexpr int NPRE = NH + NX;
    uint4 pre[NPRE];
    int rpar = -1;
    float rdt = 0.f, rA = 0.f;
    // The chunk coordinates of a thread are loop invariants; keeping them all in registers
    // across the unit loop would cost more registers than the budget of 128 allows, so every
    // helper below re-derives them from an opaque copy of the thread index (a few VALU ops).
    auto opaque = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };

    float rD = 0.f;                  // D[h] of the unit whose h0 is in pre[]
    auto load_H = [&](int b, int h) {       // the role group that carries this unit
        // the lane-dependent zero keeps this a vector load: it then sits in the same in-order
        // queue as the h0 chunks instead of forcing a scalar-cache wait in the hot window
        if (D) rD = D[h + (opaque(lane) & 0)];
        const char *hb = reinterpret_cast<const char *>(h0 + ((size_t)b * H + h) * P * S);
        const uint32_t off = (uint32_t)opaque(rt) * 16u;
#pragma unroll
        for (int q = 0; q < NH; ++q) pre[q] = *reinterpret_cast<const uint4 *>(hb + q * (kHalf * 16) + off);
    };
    // C and B tiles of a unit: global -> registers -> LDS in one go (G threads).  Runs only when
    // the (sequence, group) changes, i.e. about once per workgroup.
    auto restage_CB = [&](int b, int h) {
        const int g = h / hpg;
        const char *Cb = reinterpret_cast<const char *>(Cm + (size_t)b * n * c_sn + (size_t)g * S);
        const char *Bb = reinterpret_cast<const char *>(Bm + (size_t)b * n * b_sn + (size_t)g * S);
        const int t = opaque(rt), rc0 = t / (S / 8), cc0 = t % (S / 8);
        uint4 c[NC], bq[NC];
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int rr = min(rc0 + q * kRowsC, n - 1);
            c[q] = *reinterpret_cast<const uint4 *>(Cb + (uint32_t)(rr * (int)c_sn + cc0 * 8) * 2u);
            bq[q] = *reinterpret_cast<const uint4 *>(Bb + (uint32_t)(rr * (int)b_sn + cc0 * 8) * 2u);
        }
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int rr = rc0 + q * kRowsC;
            const uint32_t keep = rr < n ? 0xffffffffu : 0u;   // zero the rows beyond the tree
            *reinterpret_cast<uint4 *>(&sC[rr * SP + cc0 * 8]) =
                make_uint4(c[q].x & keep, c[q].y & keep, c[q].z & keep, c[q].w & keep);
            *reinterpret_cast<uint4 *>(&sB[rr * SP + cc0 * 8]) =
                make_uint4(bq[q].x & keep, bq[q].y & keep, bq[q].z & keep, bq[q].w & keep);
        }
    };
    auto load_X = [&](int b, int h) {       // G threads
        const char *xb = reinterpret_cast<const char *>(x + (size_t)b * n * x_sn + (size_t)h * P);
        const int t = opaque(rt), rx0 = t / (P / 8), cx0 = t % (P / 8);
#pragma unroll
        for (int q = 0; q < NX; ++q)
            pre[NH + q] = *reinterpret_cast<const uint4 *>(
                xb + (uint32_t)(min(rx0 + q * kRowsX, n - 1) * (int)x_sn + cx0 * 8) * 2u);
    };
    auto load_T = [&](int b, int h) {       // tree wave
        const int node = min(opaque(lane), n - 1);
        rpar = parent[(uint32_t)(b * n + node)];
        rdt = dt[(uint32_t)((b * n + node) * H + h)];
        rA = A[h];
    };
    // ---- registers -> LDS -------------------------------------------------------------------------
    auto stage_H = [&]() {
        const int t = opaque(rt);
#pragma unroll
        for (int q = 0; q < NH; ++q) {
            const int e = (t + q * kHalf) * 4, p = e / S, sidx = e % S;
            bf16x4 o;
            o[0] = (bf16_t)__uint_as_float(pre[q].x); o[1] = (bf16_t)__uint_as_float(pre[q].y);
            o[2] = (bf16_t)__uint_as_float(pre[q].z); o[3] = (bf16_t)__uint_as_float(pre[q].w);
            *reinterpret_cast<bf16x4 *>(&sH[p * SP + sidx]) = o;
        }
        if (rt == 0) *sDh = rD;      // D of that unit, for the Y waves
    };
    auto stage_X = [&](int buf) {
        unsigned short *sXT = sXT2[buf];
        const int t = opaque(rt), rx0 = t / (P / 8), cx0 = t % (P / 8);
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int rr = rx0 + q * kRowsX;
            const uint32_t keep = rr < n ? 0xffffffffu : 0u;
            const uint4 xq = pre[NH + q];
            const uint32_t wv[4] = {xq.x & keep, xq.y & keep, xq.z & keep, xq.w & keep};
            unsigned short *dst = sXT + (cx0 * 8) * kNP64 + rr;
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                dst[(2 * e) * kNP64] = (unsigned short)(wv[e] & 0xffffu);
                dst[(2 * e + 1) * kNP64] = (unsigned short)(wv[e] >> 16);
            }
        }
    };
    auto stage_T = [&]() {
        const int ln = opaque(lane);   // LDS addresses re-derived here, not carried across the loop
        const int bad = wave_tree_index(ln, n, rpar, rdt, rA, sS2, sU, sMask);
        if (ln == 0) *sBad = bad;
    };

    if (nU <= 0) return;
    STREE_EXIT_INIT;
    STREE_EXIT_POINT(1);
    STREE_PHASE_PRO(23, 0);
    STREE_PHASE_ENTRY(u0);
    // (b, h) of the current unit and of the next three.  The loop starts one unit early (k = -1):
    // that pass has no unit to compute and only runs the staging half, which brings unit 0 into
    // LDS and issues the loads of units 1 and 2 -- the same code as in the steady state, so the
    // instruction cache sees each part of the loop body once.
    int cb = ub0, ch = uh0, b1 = ub0, h1 = uh0;
    int b2 = b1, h2 = h1;
    step(b2, h2);
    int b3 = b2, h3 = h2;
    step(b3, h3);
    // the first loads of every role, before anything is waited for
    if (isY) {
        if (h0) load_H(b1, h1);
        STREE_PHASE_PRO(16, 0);
    } else {
        load_X(b1, h1);
        if (wave == kTreeWave) load_T(b1, h1);
        STREE_PHASE_PRO(18, 256);
    }
    STREE_EXIT_POINT(2);

    // One accumulator set serves both roles: the Y waves' Yt tiles of the current unit, or
    // (acc[0]) the G waves' Gt tile of the current (sequence, group), kept across its heads.
    floatx16 acc[YQ];
#pragma unroll
    for (int q = 0; q < YQ; ++q)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;

    for (int k = -1; k < nU; ++k) {
        [[maybe_unused]] const int prof_unit = cb * H + ch;  // only read by probe builds
        const bool live = k >= 0;                             // false in the staging-only first pass
        int bad = 0;
        float D_h = 0.f;
        if (live) {
            __syncthreads();                                  // barrier 1: unit k is staged
            STREE_PHASE_CLOCK(0);
            bad = *sBad;
            D_h = *sDh;
            if (status && ch == 0 && tid == 0) status[cb] = bad;
            STREE_EXIT_POINT(10 + 10 * k);
        }
        const unsigned short *sXT = sXT2[k & 1];

        if (!live) {
        } else if (isY) {
#pragma unroll
            for (int q = 0; q < YQ; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
            // ---- phase 1: Yt = h0b C^T, then *= exp(s_i) -------------------------------------------
            if (h0 && !bad) {
                const bf16_t *cp = &sC[il * SP + 8 * lh];
#pragma unroll
                for (int kb = 0; kb < S; kb += S / 2) {   // fragments of half the state index per batch
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
                    __builtin_amdgcn_sched_barrier(0);   // keep the batches apart: register budget
                }
                const float e = __builtin_amdgcn_exp2f(sS2[il]);
#pragma unroll
                for (int q = 0; q < YQ; ++q)
#pragma unroll
                    for (int rg = 0; rg < 16; ++rg) acc[q][rg] *= e;
            }
            STREE_PHASE_CLOCK(1);
        } else if (wave != kTreeWave && !bad) {
            // ---- phase 2: Gt = B C^T (only when the C/B tiles are new), mask and decay -> M ----------
            const int jt = (wave - 4) >> 1;
            STREE_PHASE_CLOCK_G(9);
            floatx16 &gt = acc[0];
            if (fresh_at(k, ch)) {
#pragma unroll
                for (int e = 0; e < 16; ++e) gt[e] = 0.f;
                const bf16_t *cp = &sC[il * SP + 8 * lh];
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
                }
            }
            STREE_PHASE_CLOCK_G(10);
            const float s2_i = sS2[il];
            const uint32_t mrow = sMask[il * 2 + jt] >> (4 * lh);   // bit 8*rg + e <-> j = jl + e
            float4 uj[4];
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) uj[rg] = *reinterpret_cast<const float4 *>(&sU[jt * 32 + 8 * rg + 4 * lh]);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int jl = jt * 32 + 8 * rg + 4 * lh;
                const float ujv[4] = {uj[rg].x, uj[rg].y, uj[rg].z, uj[rg].w};
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    // bitwise select: an overflowed exp2 under a cleared mask bit never reaches M
                    const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)mrow, 8 * rg + e, 1);
                    const float v = gt[4 * rg + e] * __builtin_amdgcn_exp2f(s2_i - ujv[e]);
                    o[e] = (bf16_t)__uint_as_float(__float_as_uint(v) & keep);
                }
                *reinterpret_cast<bf16x4 *>(&sM[il * kNP64 + jl]) = o;
            }
            STREE_PHASE_CLOCK_G(11);
        }
        if (live) STREE_EXIT_POINT(11 + 10 * k);
        if (live) __syncthreads();                            // barrier 2: M is ready; h0b, C and the tree arrays are dead
        if (live) STREE_EXIT_POINT(12 + 10 * k);
        STREE_PHASE_CLOCK(2);

        const bool more = k + 1 < nU, more2 = k + 2 < nU, more3 = k + 3 < nU;
        const bool y_stages = (k & 1) != 0;    // unit k+1 is even: its h0 sits in the Y threads
        if (isY) {
            // ---- phase 3: Yt += Xt M^T over j <= i only (nodes i < 32 have no ancestor j >= 32:
            //      that quadrant of M is never written or read); y = Yt + D x -> own 32x32 block
            //      of the bf16 staging rows ------------------------------------------------------------
            bf16x4 yreg[YQ][4];
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                if (!live) break;
                const int pt = (wave + 4 * q) >> 1;
                float xv[16];   // x[i][p] of this lane's node for the 16 p of its accumulator
#pragma unroll
                for (int rg = 0; rg < 4; ++rg)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        xv[4 * rg + e] =
                            __uint_as_float((uint32_t)sXT[(pt * 32 + 8 * rg + 4 * lh + e) * kNP64 + il] << 16);
                if (!bad) {
                    const bf16_t *ap = reinterpret_cast<const bf16_t *>(sXT) + (pt * 32 + l32) * kNP64 + 8 * lh;
                    const bf16_t *bp = &sM[il * kNP64 + 8 * lh];
                    if (it) {
                        bf16x8 a[4], bb[4];
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            a[j] = *reinterpret_cast<const bf16x8 *>(ap + 16 * j);
                            bb[j] = *reinterpret_cast<const bf16x8 *>(bp + 16 * j);
                        }
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], bb[j], acc[q], 0, 0, 0);
                    } else {
                        bf16x8 a[2], bb[2];
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            a[j] = *reinterpret_cast<const bf16x8 *>(ap + 16 * j);
                            bb[j] = *reinterpret_cast<const bf16x8 *>(bp + 16 * j);
                        }
#pragma unroll
                        for (int j = 0; j < 2; ++j)
                            acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], bb[j], acc[q], 0, 0, 0);
                    }
                }
                // y = Yt + D x; kept in registers as bf16 until the stores further down
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        o[e] = bad ? (bf16_t)0.f : (bf16_t)fmaf(D_h, xv[4 * rg + e], acc[q][4 * rg + e]);
                    yreg[q][rg] = o;
                }
            }
            STREE_PHASE_CLOCK(3);
            if (live) STREE_EXIT_POINT(13 + 10 * k);
            // next unit's state tile (its loads have been in flight for a whole unit period)
            if (more) {
                if (h0) {
                    if (y_stages) stage_H();
                    if (!live) STREE_PHASE_PRO(17, 0);
                } else if (rt == 0) {
                    *sDh = D ? D[h1] : 0.f;
                }
            }
            STREE_PHASE_CLOCK(4);
            // y leaves as 64-byte row pieces: the accumulators give a lane 4 consecutive p of one
            // node, which as direct stores would be 16-byte pieces of 32 different lines per
            // instruction.  Each wave therefore turns its 32x32 tile around in a private 2 KB of LDS
            // (a wave's LDS operations complete in order: no barrier) and stores 16 bytes per lane,
            // four lanes to a row.  The LDS used is the B tile's, idle except while the next unit
            // brings new C / B tiles; that pass stores straight from the accumulators instead.
            // The stores go out after the wait for the h0 loads above and are long complete at
            // the next such wait: on gfx9 loads and stores share one counter and complete out of
            // order with respect to each other, so a store in flight would turn that wait into a
            // wait for everything.
            if (live) {
                char *yb = reinterpret_cast<char *>(y + (size_t)cb * n * H * P + (size_t)ch * P);
                if (!(more && fresh_at(k + 1, h1))) {
                    char *ys = reinterpret_cast<char *>(sB) + opaque(wave) * 2048;
                    const int ln = opaque(lane), wr = ln & 31, wh = ln >> 5;
                    const int rr = ln >> 2, rc = ln & 3;
#pragma unroll
                    for (int q = 0; q < YQ; ++q) {
                        const int pt = (wave + 4 * q) >> 1;
                        // row r keeps its 16-byte chunk c at slot c ^ ((r >> 2) & 3)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            *reinterpret_cast<bf16x4 *>(ys + wr * 64 + ((rg ^ ((wr >> 2) & 3)) * 16) + wh * 8) =
                                yreg[q][rg];
#pragma unroll
                        for (int half = 0; half < 2; ++half) {
                            const int row = half * 16 + rr;
                            const uint4 v =
                                *reinterpret_cast<const uint4 *>(ys + row * 64 + ((rc ^ ((row >> 2) & 3)) * 16));
                            const int node = it * 32 + row;
                            if (node < n)
                                store_through16(yb + (uint32_t)(node * H * P + pt * 32 + rc * 8) * 2u, v);
                        }
                    }
                } else if (il < n) {
                    const int row = opaque(il), lh = opaque(lane) >> 5;   // re-derived: not carried across the loop
#pragma unroll
                    for (int q = 0; q < YQ; ++q) {
                        const int pt = (wave + 4 * q) >> 1;
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            *reinterpret_cast<bf16x4 *>(yb + (uint32_t)(row * H * P + pt * 32 + 8 * rg + 4 * lh) * 2u) =
                                yreg[q][rg];   // 8-byte pieces: left to L2 to merge, not written through
                    }
                }
            }
            if (h0 && more3 && y_stages) load_H(b3, h3);
            STREE_PHASE_CLOCK(5);
        } else if (more) {
            if (h0 && !y_stages) {
                stage_H();
                if (more3) load_H(b3, h3);
            }
            if (wave == kTreeWave) {
                stage_T();
                if (!live) STREE_PHASE_PRO(20, 384);
                if (more2) load_T(b2, h2);
            }
            if (fresh_at(k + 1, h1)) restage_CB(b1, h1);
            if (!live) STREE_PHASE_PRO(19, 256);
            stage_X((k + 1) & 1);                          // the other X^T tile: unit k still reads its own
            if (!live) STREE_PHASE_PRO(21, 256);
            if (more2) {
                load_X(b2, h2);
                if (!live && h0) load_H(b2, h2);           // unit 1: the first odd unit
            }
            if (!live) STREE_PHASE_PRO(22, 256);
        }
        STREE_PHASE_CLOCK(6);
        STREE_PHASE_CLOCK(7);
        STREE_EXIT_POINT(4 + k);
        cb = b1; ch = h1;
        b1 = b2; h1 = h2;
        b2 = b3; h2 = h3;
        step(b3, h3);
    }
}

template <int P, int S>
hipError_t launch64_ps(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                       const void *Bm, const void *Cm, const float *D, const float *h0, void *y,
                       int32_t *status, hipStream_t st) {
    constexpr size_t lds = Lds64<P, S>::total;   // static LDS of the kernel (upper bound)
    constexpr int WPE = (2 * (lds + 64) <= 160 * 1024) ? 4 : 2;
    const int n_units = d.batch * d.nheads;
    const int per_cu = (int)((160 * 1024) / (lds + 64));      // resident workgroups per CU by LDS
    int grid = (n_units + 7) / 8 * 8;
    const int cap = 256 * (per_cu < 1 ? 1 : per_cu);
    if (grid > cap) grid = cap;
    hipLaunchKernelGGL((tree_ssd_mfma64_kernel<P, S, WPE>), dim3(grid), dim3(kT64), 0, st, parent, d.nnodes,
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

bool tree_ssd_replay_fused_supported(const stree_dims &, const stree_dims &, const void *, const void *, const void *,
                                     const void *, const void *, const void *) {
    return false;
}
hipError_t launch_tree_ssd_replay_fused(const stree_dims &, const stree_dims &, const int32_t *, const int32_t *,
                                        const void *, const float *, const void *, const int32_t *, const void *,
                                        const float *, const float *, const void *, const void *, const float *,
                                        const float *, float *, void *, int32_t *, int32_t *, hipStream_t) {
    return hipErrorInvalidValue;
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
