// stree_linear_ssd: the ordinary causal scan of a long token sequence (the lower-triangular case of
// the tree mask: the paper's remark in Sec. 3 that a chain reduces the method to Mamba2 with an
// initial state), as one chunked kernel with the state passed from chunk to chunk in registers.
// This is the prefix pass in front of tree decoding: y for every prefix token and the state after
// the last one, which then seeds stree_tree_ssd.
//
// One workgroup (4 waves) per (batch, head) walks the sequence in chunks of 64 tokens.  With s_i the
// inclusive cumulative log-decay inside the chunk and h the state before it,
//
//   y_i   = exp(s_i) h C_i + sum_{j <= i} exp(s_i - s_j) dt_j <C_i, B_j> x_j + D x_i
//   h_new = exp(s_last) h + sum_j dt_j exp(s_last - s_j) x_j (outer) B_j
//
// The first line is the tree kernel's three products with the causal mask j <= i in place of the
// ancestor mask (same transposed MFMA tiles, same accumulator layouts).  The state lives in MFMA
// accumulators as h^T[s][p] for the whole sequence; its update is one more MFMA product
// B^T (S x 64) times the weighted x (64 x P).  The weights are fp32 and the state must stay fp32
// accurate over thousands of tokens, so the weighted x is fed as two bf16 terms (value and rounding
// remainder): each product is then exact to about 2^-17, and because those errors are independent
// and every chunk's increment is damped by the later decay, the state after 4096 tokens stays
// within 5e-6 of the fp64 scan (a third term bought nothing measurable against the 1e-4 bound and
// cost a third more MFMA and conversion work).  Only h as the operand of the y product is rounded
// to bf16.
#include "common.hpp"
#include "launch.hpp"

namespace stree {

namespace {

constexpr int kChunk = 64;
constexpr int kCP = kChunk + 8;    // padded row of a [.. x 64] bf16 LDS tile

// WY = false: state only (no y, no C): a third of the LDS, so more workgroups per CU
template <int P, int S, bool WY, typename HT>
__global__ __launch_bounds__(kThreads) void linear_ssd_kernel(
    int T, int H, int G, const bf16_t *__restrict__ x, long x_sn, const float *__restrict__ dt,
    const float *__restrict__ dt_bias, const float *__restrict__ A, const bf16_t *__restrict__ Bm, long b_sn, const bf16_t *__restrict__ Cm,
    long c_sn, const float *__restrict__ D, const HT *__restrict__ h0, bf16_t *__restrict__ y,
    HT *__restrict__ h_out) {
    constexpr int SP = S + 8;
    constexpr int YT = (P / 32) * 2, YQ = YT / 4;            // Yt tiles [p][i], per wave
    // state tiles h^T[s][p]: a wave owns one p tile and TQ consecutive s tiles, so that the weighted
    // x fragments (which depend on the p tile only) are formed once per wave
    constexpr int ST = S / 32, PT = P / 32, WPP = 4 / PT, TQ = ST / WPP;
    static_assert(PT == 2 || PT == 4, "four waves share 2 or 4 p tiles");
    constexpr int NC = kChunk * (S / 8) / kThreads;          // 16-byte chunks of C (and B) per thread
    constexpr int NX = kChunk * (P / 8) / kThreads;          // of x per thread
    constexpr int kRowsC = kThreads / (S / 8), kRowsX = kThreads / (P / 8);
    static_assert(YQ >= 1 && TQ >= 1 && NC >= 1 && NX >= 1, "tile too small for 256 threads");
    __shared__ __align__(16) bf16_t sC[WY ? kChunk * SP : 8]; // C rows; after phase 2 the y staging area
    __shared__ __align__(16) bf16_t sB[(WY && kChunk * SP > S * kCP) ? kChunk * SP : S * kCP];   // B rows, then B^T
    __shared__ __align__(16) bf16_t sH[WY ? P * SP : 8];      // state as bf16 operand rows [p][s]
    __shared__ __align__(16) unsigned short sXT[P * kCP];     // x^T [p][j]
    __shared__ __align__(16) bf16_t sM[WY ? kChunk * kCP : 8];
    __shared__ __align__(16) float sS2[kChunk], sU[kChunk], sW[kChunk];
    __shared__ float sDecay[1];

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    const int h = blockIdx.x, b = blockIdx.y, g = h / (H / G);
    const float A2 = A[h] * 1.44269504088896340736f;          // log2 domain
    const float bias_h = dt_bias ? dt_bias[h] : 0.f;
    const float D_h = D ? D[h] : 0.f;
    const char *xb = reinterpret_cast<const char *>(x + (size_t)b * T * x_sn + (size_t)h * P);
    const char *Bb = reinterpret_cast<const char *>(Bm + (size_t)b * T * b_sn + (size_t)g * S);
    const char *Cb = reinterpret_cast<const char *>(Cm + (size_t)b * T * c_sn + (size_t)g * S);
    const float *dtb = dt + (size_t)b * T * H + h;

    // register r of lane l of tile (st, pt) is h[p = pt*32 + l%32][s = st*32 + 8(r/4) + 4(l/32) + r%4]
    floatx16 hacc[TQ];
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
        const int st = (wave % WPP) * TQ + q, pt = wave / WPP;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (h0) {
                const HT *src = h0 + ((size_t)b * H + h) * P * S + (size_t)(pt * 32 + l32) * S + st * 32 + 8 * rg + 4 * lh;
                if constexpr (sizeof(HT) == 4) {
                    v = *reinterpret_cast<const float4 *>(src);
                } else {                                  // a bf16 state: widened exactly
                    const uint2 w = *reinterpret_cast<const uint2 *>(src);
                    v = make_float4(bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y));
                }
            }
            hacc[q][4 * rg] = v.x; hacc[q][4 * rg + 1] = v.y; hacc[q][4 * rg + 2] = v.z; hacc[q][4 * rg + 3] = v.w;
        }
    }
    auto state_to_lds = [&]() {
#pragma unroll
        for (int q = 0; q < TQ; ++q) {
            const int st = (wave % WPP) * TQ + q, pt = wave / WPP;
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                bf16x4 o;
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = (bf16_t)hacc[q][4 * rg + e];
                *reinterpret_cast<bf16x4 *>(&sH[(pt * 32 + l32) * SP + st * 32 + 8 * rg + 4 * lh]) = o;
            }
        }
    };
    if constexpr (WY) state_to_lds();

    // chunk inputs in registers: rows beyond T are read from the last token and zeroed when staged
    uint4 rc[NC], rb[NC], rx[NX];
    float rdt = 0.f;
    const int rc0 = tid / (S / 8), cc0 = tid % (S / 8), rx0 = tid / (P / 8), cx0 = tid % (P / 8);
    // loaders of the three operand groups: each is issued as soon as its registers have been staged,
    // so that the loads of the next chunk fly for (nearly) a whole chunk period
    auto load_xc = [&](int c0) {
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int tok = min(c0 + rx0 + q * kRowsX, T - 1);
            rx[q] = load_stream16(xb + ((size_t)tok * x_sn + cx0 * 8) * 2);   // x and y: touched once
        }
        if constexpr (WY) {
#pragma unroll
            for (int q = 0; q < NC; ++q) {
                const int tok = min(c0 + rc0 + q * kRowsC, T - 1);
                rc[q] = *reinterpret_cast<const uint4 *>(Cb + ((size_t)tok * c_sn + cc0 * 8) * 2);
            }
        }
        if (tid < kChunk) rdt = (c0 + tid < T) ? dtb[(size_t)(c0 + tid) * H] : 0.f;
    };
    auto load_b = [&](int c0) {
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int tok = min(c0 + rc0 + q * kRowsC, T - 1);
            rb[q] = *reinterpret_cast<const uint4 *>(Bb + ((size_t)tok * b_sn + cc0 * 8) * 2);
        }
    };
    auto write_bt = [&](int c0) {   // B^T [s][j] from the registers
        unsigned short *sBT = reinterpret_cast<unsigned short *>(sB);
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int r = rc0 + q * kRowsC;
            const uint32_t keep = (c0 + r < T) ? 0xffffffffu : 0u;
            store_transposed_pair<S / 8, true>(sBT, kCP, r, cc0 * 8,
                                         make_uint4(rb[q].x & keep, rb[q].y & keep, rb[q].z & keep, rb[q].w & keep), lane);
        }
    };
    load_xc(0);
    load_b(0);

    for (int c0 = 0; c0 < T; c0 += kChunk) {
        // ---- S1: stage C, B (rows), x^T; cumulative log-decay of the chunk --------------------------
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int r = rc0 + q * kRowsC;
            const uint32_t keep = (c0 + r < T) ? 0xffffffffu : 0u;
            if constexpr (WY) {
                *reinterpret_cast<uint4 *>(&sC[r * SP + cc0 * 8]) =
                    make_uint4(rc[q].x & keep, rc[q].y & keep, rc[q].z & keep, rc[q].w & keep);
                *reinterpret_cast<uint4 *>(&sB[r * SP + cc0 * 8]) =
                    make_uint4(rb[q].x & keep, rb[q].y & keep, rb[q].z & keep, rb[q].w & keep);
            }
        }
#pragma unroll
        for (int q = 0; q < NX; ++q) {
            const int r = rx0 + q * kRowsX;
            const uint32_t keep = (c0 + r < T) ? 0xffffffffu : 0u;
            store_transposed_pair<P / 8, true>(sXT, kCP, r, cx0 * 8,
                                         make_uint4(rx[q].x & keep, rx[q].y & keep, rx[q].z & keep, rx[q].w & keep), lane);
        }
        if (tid < kChunk) {   // wave 0: inclusive scan of dt * A over the chunk's tokens (on the
            // chunk's critical path: every other wave waits for it at the barrier below)
            if (dt_bias) rdt = (c0 + lane < T) ? softplus_step(rdt + bias_h) : 0.f;   // raw projection -> step size
            const float s2 = wave_inclusive_sum(rdt * A2);
            // The state's weights dt_j exp(s_last - s_j) from the sum of the steps BEHIND token j, taken
            // on its own: its rounding error is relative to that sum -- small wherever the weight is
            // not negligible -- while s_last - s_j as a difference of prefix sums carries the error of
            // |s_last| (a strong decay over 64 tokens: 1e-4 in the weight, the whole error budget of
            // the state).
            float whole;
            const float behind = wave_exclusive_suffix_sum(rdt * A2, whole);
            sS2[lane] = s2;
            sU[lane] = s2 - __log2f(rdt);                      // dt = 0 -> +inf -> weight 0
            sW[lane] = rdt * __builtin_amdgcn_exp2f(behind);
            if (lane == 0) *sDecay = __builtin_amdgcn_exp2f(whole);
        }
        if constexpr (!WY) write_bt(c0);                      // no B rows needed: B^T at once
        if (c0 + kChunk < T) {
            load_xc(c0 + kChunk);
            if constexpr (!WY) load_b(c0 + kChunk);
        }
        __syncthreads();

        floatx16 acc[YQ];
        if constexpr (WY) {
            // ---- phase 1: Yt = h C^T, *= exp(s_i) ------------------------------------------------
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int t = wave + 4 * q, it = t & 1, pt = t >> 1;
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
                const bf16_t *ap = &sH[(pt * 32 + l32) * SP + 8 * lh];
                const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
#pragma unroll
                for (int k0 = 0; k0 < S; k0 += 16)
                    acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(ap + k0),
                                                                     *reinterpret_cast<const bf16x8 *>(bp + k0), acc[q], 0, 0, 0);
                const float e2 = __builtin_amdgcn_exp2f(sS2[it * 32 + l32]);
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[q][e] *= e2;
            }
            // ---- phase 2: Gt = B C^T, causal mask and decay -> M (tile jt = 1, it = 0 has j > i) ----
            {
                const int it = wave & 1, jt = wave >> 1;
                if (!(jt == 1 && it == 0)) {
                    floatx16 gt;
#pragma unroll
                    for (int e = 0; e < 16; ++e) gt[e] = 0.f;
                    const bf16_t *ap = &sB[(jt * 32 + l32) * SP + 8 * lh];
                    const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
#pragma unroll
                    for (int k0 = 0; k0 < S; k0 += 16)
                        gt = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*reinterpret_cast<const bf16x8 *>(ap + k0),
                                                                     *reinterpret_cast<const bf16x8 *>(bp + k0), gt, 0, 0, 0);
                    const int il = it * 32 + l32;
                    const float s2_i = sS2[il];
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int jl = jt * 32 + 8 * rg + 4 * lh;
                        const float4 uj = *reinterpret_cast<const float4 *>(&sU[jl]);
                        const float ujv[4] = {uj.x, uj.y, uj.z, uj.w};
                        bf16x4 o;
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            // select, never 0 * inf: an overflowed weight above the diagonal is dropped
                            const uint32_t keep = (jl + e <= il) ? 0xffffffffu : 0u;
                            const float v = gt[4 * rg + e] * __builtin_amdgcn_exp2f(s2_i - ujv[e]);
                            o[e] = (bf16_t)__uint_as_float(__float_as_uint(v) & keep);
                        }
                        *reinterpret_cast<bf16x4 *>(&sM[il * kCP + jl]) = o;
                    }
                }
            }
        }

        // ---- B^T over the dead B rows (from the registers), then the next chunk's B loads ------------
        if constexpr (WY) {
            __syncthreads();
            write_bt(c0);
            if (c0 + kChunk < T) load_b(c0 + kChunk);
        }

        if constexpr (WY) {
            // ---- phase 3: Yt += Xt M^T over j <= i; y = Yt + D x; 64-byte row pieces via a per-wave
            //      turn in LDS (the C rows are dead) ------------------------------------------------
            char *ys = reinterpret_cast<char *>(sC) + wave * 2048;
            char *yb = reinterpret_cast<char *>(y + ((size_t)b * T + c0) * H * P + (size_t)h * P);
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int t = wave + 4 * q, it = t & 1, pt = t >> 1, il = it * 32 + l32;
                float xv[16];
#pragma unroll
                for (int rg = 0; rg < 4; ++rg)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        xv[4 * rg + e] = __uint_as_float((uint32_t)sXT[transposed_at<true>(kCP, pt * 32 + 8 * rg + 4 * lh + e, il)] << 16);
                const bf16_t *xt = reinterpret_cast<const bf16_t *>(sXT);
                const bf16_t *bp = &sM[il * kCP + 8 * lh];
                const int ksteps = it ? 4 : 2;
                for (int j = 0; j < ksteps; ++j)
                    acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        *reinterpret_cast<const bf16x8 *>(xt + transposed_at<true>(kCP, pt * 32 + l32, 8 * lh + 16 * j)),
                        *reinterpret_cast<const bf16x8 *>(bp + 16 * j), acc[q], 0, 0, 0);
                // row r of the wave's tile keeps its 16-byte chunk c at slot c ^ ((r >> 2) & 3)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    bf16x4 o;
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[e] = (bf16_t)fmaf(D_h, xv[4 * rg + e], acc[q][4 * rg + e]);
                    *reinterpret_cast<bf16x4 *>(ys + l32 * 64 + ((rg ^ ((l32 >> 2) & 3)) * 16) + lh * 8) = o;
                }
#pragma unroll
                for (int half = 0; half < 2; ++half) {
                    const int row = half * 16 + (lane >> 2), rcc = lane & 3;
                    const uint4 v = *reinterpret_cast<const uint4 *>(ys + row * 64 + ((rcc ^ ((row >> 2) & 3)) * 16));
                    const int tok = it * 32 + row;
                    if (c0 + tok < T)
                        store_stream16(yb + ((size_t)tok * H * P + pt * 32 + rcc * 8) * 2, v);
                }
            }
            __syncthreads();   // B^T is complete
        }

        // ---- state: h^T = exp(s_last) h^T + B^T (w x), the weighted x as two bf16 terms --------------
        {
            const float decay = *sDecay;
            const bf16_t *sBT = sB;
#pragma unroll
            for (int q = 0; q < TQ; ++q)
#pragma unroll
                for (int e = 0; e < 16; ++e) hacc[q][e] *= decay;
            const int pt = wave / WPP;
#pragma unroll
            for (int k0 = 0; k0 < kChunk; k0 += 16) {
                const float4 w0 = *reinterpret_cast<const float4 *>(&sW[k0 + 8 * lh]);
                const float4 w1 = *reinterpret_cast<const float4 *>(&sW[k0 + 8 * lh + 4]);
                const float wv[8] = {w0.x, w0.y, w0.z, w0.w, w1.x, w1.y, w1.z, w1.w};
                const uint4 xr = *reinterpret_cast<const uint4 *>(&sXT[transposed_at<true>(kCP, pt * 32 + l32, 8 * lh + k0)]);
                const float xf[8] = {bf16_lo(xr.x), bf16_hi(xr.x), bf16_lo(xr.y), bf16_hi(xr.y),
                                     bf16_lo(xr.z), bf16_hi(xr.z), bf16_lo(xr.w), bf16_hi(xr.w)};
                bf16x8 t0, t1;
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const float v = wv[e] * xf[e];
                    t0[e] = (bf16_t)v;
                    t1[e] = (bf16_t)(v - (float)t0[e]);
                }
#pragma unroll
                for (int q = 0; q < TQ; ++q) {
                    const int st = (wave % WPP) * TQ + q;
                    const bf16x8 bt = *reinterpret_cast<const bf16x8 *>(&sBT[transposed_at<true>(kCP, st * 32 + l32, 8 * lh + k0)]);
                    hacc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bt, t0, hacc[q], 0, 0, 0);
                    hacc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bt, t1, hacc[q], 0, 0, 0);
                }
            }
        }
        if (WY && c0 + kChunk < T) state_to_lds();   // the next chunk's phase 1 operand
        __syncthreads();
    }
    // ---- final state ------------------------------------------------------------------------------
#pragma unroll
    for (int q = 0; q < TQ; ++q) {
        const int st = (wave % WPP) * TQ + q, pt = wave / WPP;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            HT *dst = h_out + ((size_t)b * H + h) * P * S + (size_t)(pt * 32 + l32) * S + st * 32 + 8 * rg + 4 * lh;
            if constexpr (sizeof(HT) == 4)
                *reinterpret_cast<float4 *>(dst) =
                    make_float4(hacc[q][4 * rg], hacc[q][4 * rg + 1], hacc[q][4 * rg + 2], hacc[q][4 * rg + 3]);
            else                                          // a bf16 state: rounded to nearest even once, here
                *reinterpret_cast<uint2 *>(dst) =
                    pack_bf16x4(hacc[q][4 * rg], hacc[q][4 * rg + 1], hacc[q][4 * rg + 2], hacc[q][4 * rg + 3]);
        }
    }
}

template <int P, int S, typename HT>
hipError_t launch_ps(const stree_dims &d, const void *x, const float *dt, const float *A, const void *Bm,
                     const void *Cm, const float *D, const void *h0, void *y, void *h_out, hipStream_t st) {
    if (y)
        hipLaunchKernelGGL((linear_ssd_kernel<P, S, true, HT>), dim3(d.nheads, d.batch), dim3(kThreads), 0, st, d.nnodes,
                           d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, step_bias(d), A,
                           (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D,
                           (const HT *)h0, (bf16_t *)y, (HT *)h_out);
    else
        hipLaunchKernelGGL((linear_ssd_kernel<P, S, false, HT>), dim3(d.nheads, d.batch), dim3(kThreads), 0, st, d.nnodes,
                           d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, step_bias(d), A,
                           (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D,
                           (const HT *)h0, (bf16_t *)y, (HT *)h_out);
    return hipGetLastError();
}

template <int P, int S>
hipError_t launch_p(const stree_dims &d, const void *x, const float *dt, const float *A, const void *Bm,
                    const void *Cm, const float *D, const void *h0, void *y, void *h_out, hipStream_t st) {
    if (d.state_dtype == STREE_BF16) return launch_ps<P, S, bf16_t>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
    return launch_ps<P, S, float>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
}

}  // namespace

bool linear_ssd_supported(const stree_dims &d, const void *x, const void *Bm, const void *Cm, const void *y,
                          const void *h0, const void *h_out) {
    if (d.io_dtype != STREE_BF16) return false;
    const int P = d.headdim, S = d.dstate;
    if (!((P == 64 && (S == 128 || S == 64 || S == 256)) || (P == 128 && S == 128))) return false;
    if ((d.x_stride_n | d.b_stride_n | d.c_stride_n) % 8 != 0) return false;
    // (the state is read and written 16 bytes at a time, like the rows)
    return (((uintptr_t)x | (uintptr_t)Bm | (uintptr_t)Cm | (uintptr_t)y | (uintptr_t)h0 | (uintptr_t)h_out) % 16) == 0;
}

hipError_t launch_linear_ssd(const stree_dims &d, const void *x, const float *dt, const float *A, const void *Bm,
                             const void *Cm, const float *D, const void *h0, void *y, void *h_out, hipStream_t st) {
    const int P = d.headdim, S = d.dstate;
    if (P == 64 && S == 128) return launch_p<64, 128>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
    if (P == 64 && S == 64) return launch_p<64, 64>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
    if (P == 64 && S == 256) return launch_p<64, 256>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
    if (P == 128 && S == 128) return launch_p<128, 128>(d, x, dt, A, Bm, Cm, D, h0, y, h_out, st);
    return hipErrorInvalidValue;
}

}  // namespace stree
