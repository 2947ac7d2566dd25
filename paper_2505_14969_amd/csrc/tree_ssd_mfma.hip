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
#include <mutex>

#include "common.hpp"
#include "launch.hpp"

namespace stree {

constexpr int kBlk = 64;         // node block
constexpr int kNP = kBlk + 8;    // padded row of a [.. x 64] bf16 LDS tile

struct MfmaLdsPlan {
    int sp;                      // padded state row, elements
    size_t off_c, off_b, off_h, off_xt, off_m, off_mask, total;
};

// share_h: the bf16 state tile (needed in phase 1 only) lives in the B tile's LDS instead of its
// own: taken for trees of more than 128 nodes, where it is the difference between one and two
// workgroups per CU
__host__ __device__ inline bool mfma_share_h(int npad) { return npad > 128; }
__host__ __device__ inline MfmaLdsPlan mfma_lds_plan(int P, int S, int npad, int words) {
    MfmaLdsPlan pl;
    pl.sp = S + 8;
    const size_t c_bytes = (size_t)kBlk * pl.sp * 2;
    const size_t y_bytes = (size_t)kBlk * (P + 4) * 4;  // fp32 output staging shares the B tile
    const size_t h_bytes = (size_t)P * pl.sp * 2;       // and so does the bf16 state tile (phase 1 only)
    const bool share = mfma_share_h(npad);
    size_t b_bytes = c_bytes > y_bytes ? c_bytes : y_bytes;
    if (share && h_bytes > b_bytes) b_bytes = h_bytes;
    size_t o = 0;
    pl.off_c = o; o += c_bytes;
    pl.off_b = o; o += b_bytes;
    pl.off_h = pl.off_b;
    if (!share) { pl.off_h = o; o += h_bytes; }
    pl.off_xt = o; o += (size_t)P * kNP * 2;
    pl.off_m = o; o += (size_t)kBlk * kNP * 2;
    pl.off_mask = o; o += (size_t)npad * words * 4;
    pl.total = o;
    return pl;
}

// Tile loads travel through registers: the loads of the next (row block, column block) pair are
// issued before the current pair is computed and written to LDS after it, so that their latency
// is hidden by the MFMA phases; the first tiles and the initial state are requested before the
// tree index is built.
constexpr int kMaxS32 = 8;       // dstate <= 256: at most 8 16-byte pieces of a C or B tile per thread
constexpr int kH0Batch = 8;      // float4 pieces of h0 per thread requested ahead of the tree index

// (for headdim <= 64 two workgroups fit the LDS of a CU: the register budget is held to that)
template <int P, bool SH, typename HT>
__global__ __launch_bounds__(kThreads, P <= 64 ? 2 : 1) void tree_ssd_mfma_kernel(
    const int32_t *__restrict__ parent, int n, int H, int S, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ dt_bias, const float *__restrict__ A,
    const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const HT *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status) {
    constexpr int YT = (P / 32) * 2;          // 32x32 tiles of Yt[p][i] per node block
    constexpr int YQ = (YT + 3) / 4;          // tiles per wave
    constexpr int XQ = P / 32;                // 16-byte pieces of an x tile per thread
    extern __shared__ __align__(16) unsigned char lds[];
    __shared__ TreeLds tree;
    __shared__ uint32_t nz_bits;              // bit 4*ib+jb: row block ib has an ancestor in column block jb < ib

    const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, l32 = lane & 31, lh = lane >> 5;
    const int h = blockIdx.x, b = blockIdx.y;
    const int g = h / (H / G);
    const int npad = (n + kBlk - 1) / kBlk * kBlk;
    const int nblk = npad / kBlk;
    const int words = (n + 31) / 32;
    const MfmaLdsPlan pl = mfma_lds_plan(P, S, npad, words);
    const int SP = pl.sp;
    bf16_t *sC = reinterpret_cast<bf16_t *>(lds + pl.off_c);
    bf16_t *sB = reinterpret_cast<bf16_t *>(lds + pl.off_b);
    float *sY = reinterpret_cast<float *>(lds + pl.off_b);
    bf16_t *sH = reinterpret_cast<bf16_t *>(lds + pl.off_h);   // SH: the B tile's LDS, between a row block's start and its first B tile
    bf16_t *sXT = reinterpret_cast<bf16_t *>(lds + pl.off_xt);
    bf16_t *sM = reinterpret_cast<bf16_t *>(lds + pl.off_m);
    uint32_t *mask = reinterpret_cast<uint32_t *>(lds + pl.off_mask);

    const bf16_t *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
    const bf16_t *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
    const bf16_t *Cb = Cm + (size_t)b * n * c_sn + (size_t)g * S;
    const HT *hb = h0 ? h0 + ((size_t)b * H + h) * P * S : nullptr;
    // four consecutive state values, widened exactly when the state is kept in bf16
    auto load_h4 = [&](int idx) -> float4 {
        if constexpr (sizeof(HT) == 4) {
            return *reinterpret_cast<const float4 *>(hb + (size_t)idx * 4);
        } else {
            const uint2 w = *reinterpret_cast<const uint2 *>(hb + (size_t)idx * 4);
            return make_float4(bf16_lo(w.x), bf16_hi(w.x), bf16_lo(w.y), bf16_hi(w.y));
        }
    };
    const int s8 = S / 8;
    const int cb_items = kBlk * s8;           // 16-byte pieces of a C or B tile
    const int h_items = P * S / 4;            // float4 pieces of h0

    // ---- tile movers: global -> registers, registers -> LDS ---------------------------------
    // Loads are unconditional (rows past the tree and pieces past the tile are clamped to valid
    // addresses), so that they are issued back to back with no wait between them; what must be
    // zero is zeroed when the registers are written to LDS.
    uint4 creg[kMaxS32], breg[kMaxS32], xreg[XQ];
    float4 hreg[kH0Batch];
    int rc[kMaxS32];                          // piece q of a C or B tile: (row << 8) | 16-byte column
#pragma unroll
    for (int q = 0; q < kMaxS32; ++q) {
        const int idx = min(q * kThreads + tid, cb_items - 1);
        rc[q] = ((idx / s8) << 8) | (idx % s8);
    }
    // Per-thread tile coordinates are loop invariants: left alone, the compiler hoists every LDS and
    // global address derived from them out of the pair loop, runs out of registers and spills them,
    // and each reload is followed by a wait for everything in flight (some thirty serial round trips
    // per row block in the 256-node configuration).  The movers below therefore derive their
    // addresses from a copy of the coordinates that the compiler cannot see through.
    auto opaque = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };
    auto load_rows = [&](uint4 (&r)[kMaxS32], const bf16_t *base, long sn, int row0) {
#pragma unroll
        for (int q = 0; q < kMaxS32; ++q) {
            const int i = min(row0 + (rc[q] >> 8), n - 1);
            r[q] = *reinterpret_cast<const uint4 *>(base + (size_t)i * sn + (rc[q] & 0xff) * 8);
        }
    };
    auto store_rows = [&](const uint4 (&r)[kMaxS32], bf16_t *tile, int row0) {
#pragma unroll
        for (int q = 0; q < kMaxS32; ++q) {
            if (q * kThreads + tid < cb_items) {
                const int rcq = opaque(rc[q]);
                uint4 v = r[q];
                if (row0 + (rcq >> 8) >= n) v = make_uint4(0, 0, 0, 0);
                *reinterpret_cast<uint4 *>(&tile[(rcq >> 8) * SP + (rcq & 0xff) * 8]) = v;
            }
        }
    };
    auto load_x = [&](int row0) {
#pragma unroll
        for (int q = 0; q < XQ; ++q) {
            const int idx = q * kThreads + tid;
            const int j = min(row0 + idx / (P / 8), n - 1);
            xreg[q] = *reinterpret_cast<const uint4 *>(xb + (size_t)j * x_sn + (idx % (P / 8)) * 8);
        }
    };
    auto store_x = [&](int row0) {
#pragma unroll
        for (int q = 0; q < XQ; ++q) {
            const int idx = q * kThreads + opaque(tid);
            uint4 v = xreg[q];
            if (row0 + idx / (P / 8) >= n) v = make_uint4(0, 0, 0, 0);
            // (every lane of the wave is here: kBlk * P/8 is a multiple of the workgroup size)
            store_transposed_pair<P / 8>(reinterpret_cast<unsigned short *>(sXT), kNP, idx / (P / 8),
                                         (idx % (P / 8)) * 8, v, lane);
        }
    };
    // `one` is 1.0f that the compiler cannot see through, defined after the tree index: the
    // conversion of the prefetched h0 pieces (and the wait for them) cannot move above that point.
    auto store_h = [&](int idx, const float4 &v, float one) {
        const int e = idx * 4, p = e / S, s = e % S;
        bf16x4 o;
        o[0] = (bf16_t)(v.x * one); o[1] = (bf16_t)(v.y * one); o[2] = (bf16_t)(v.z * one); o[3] = (bf16_t)(v.w * one);
        *reinterpret_cast<bf16x4 *>(&sH[p * SP + s]) = o;
    };

    // ---- requests that do not depend on the tree: the small per-node values first (loads return
    //      in order, and the tree index needs only these), then h0 and the tiles of pair (0, 0) ----
    const float A_h = A[h];
    const float D_h = D ? D[h] : 0.f;          // (asked for here: after the tree index its latency is exposed)
    const float bias_h = dt_bias ? dt_bias[h] : 0.f;
    const float dt_raw = tid < n ? dt[((size_t)b * n + tid) * H + h] : 0.f;
    const int parent_i = tid < n ? parent[(size_t)b * n + tid] : -1;
    if (h0) {
#pragma unroll
        for (int q = 0; q < kH0Batch; ++q) {
            const int idx = min(q * kThreads + tid, h_items - 1);
            hreg[q] = load_h4(idx);
        }
    }
    load_rows(creg, Cb, c_sn, 0);
    load_rows(breg, Bb, b_sn, 0);
    load_x(0);

    // ---- tree index: depth, mask rows L_i, s_i = (A_tree)_i ---------------------------------
    if (tid == 0) nz_bits = 0u;
    const float dt_i = (dt_bias && tid < n) ? softplus_step(dt_raw + bias_h) : dt_raw;
    const int bad = build_tree_index(tree, mask, parent_i, n, npad, words, dt_i, A_h);
    if (status && h == 0 && tid == 0) status[b] = bad;
    bf16_t *yb = y + (size_t)b * n * H * P + (size_t)h * P;
    if (bad) {
        for (int idx = tid; idx < n * (P / 8); idx += kThreads) {
            const int r = idx / (P / 8), c = idx % (P / 8);
            *reinterpret_cast<uint4 *>(yb + (size_t)r * H * P + c * 8) = make_uint4(0, 0, 0, 0);
        }
        return;
    }
    // column blocks that hold an ancestor of some node of a row block (the others are skipped)
    if (tid < n) {
        const int ib = tid >> 6;
        uint32_t bits = 0u;
        for (int jb = 0; jb < ib; ++jb)
            if ((mask[tid * words + 2 * jb] | mask[tid * words + 2 * jb + 1]) != 0u) bits |= 1u << (4 * ib + jb);
        if (bits) atomicOr(&nz_bits, bits);
    }
    float one = 1.0f;                        // (see store_h)
    asm volatile("" : "+v"(one));
    __syncthreads();
    const uint32_t nz = __builtin_amdgcn_readfirstlane(nz_bits);

    // first column block of row block ib, and the one after jb (the diagonal block is always taken)
    auto next_col = [&](int ib, int after) {
        const uint32_t row = ((nz >> (4 * ib)) & 0xfu) | (1u << ib);
        const uint32_t rest = row & ~((1u << (after + 1)) - 1u);
        return __builtin_ctz(rest);
    };

    // acc += sum over the S state indices of a-row * b-row, four 16-wide steps per round so that
    // the LDS reads of a round are in flight together (S is a multiple of 16, not always of 64)
    auto contract_s = [&](floatx16 &c, const bf16_t *ap, const bf16_t *bp) {
        for (int k0 = 0; k0 < S; k0 += 64) {
            bf16x8 a[4], bb[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int kk = min(k0 + 16 * u, S - 16);
                a[u] = *reinterpret_cast<const bf16x8 *>(ap + kk);
                bb[u] = *reinterpret_cast<const bf16x8 *>(bp + kk);
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (k0 + 16 * u < S) c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[u], bb[u], c, 0, 0, 0);
        }
    };

    floatx16 acc[YQ];
    int ib = 0, jb = 0;
    bool new_rows = true;
    while (true) {
        const int i0 = ib * kBlk, j0 = jb * kBlk;
        // ---- this pair's tiles: registers -> LDS; the next pair's: global -> registers ------
        if (new_rows) {
            // ---- a row block starts: C rows, and the state tile in the B tile's LDS for phase 1 -----
            store_rows(creg, sC, i0);
            if (h0 && (SH || ib == 0)) {
                if (SH && ib > 0) {    // the state tile again (from L2)
#pragma unroll
                    for (int q = 0; q < kH0Batch; ++q) {
                        const int idx = min(q * kThreads + opaque(tid), h_items - 1);
                        hreg[q] = load_h4(idx);
                    }
                }
#pragma unroll
                for (int q = 0; q < kH0Batch; ++q) {
                    const int idx = q * kThreads + opaque(tid);
                    if (idx < h_items) store_h(idx, hreg[q], one);
                }
                for (int idx = kH0Batch * kThreads + tid; idx < h_items; idx += kThreads)
                    store_h(idx, load_h4(idx), one);
            }
            __syncthreads();
#pragma unroll
            for (int q = 0; q < YQ; ++q)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[q][r] = 0.f;
            // ---- phase 1 (once per row block): Yt = h0b * C^T, scaled by exp(s_i) -------------------
            if (h0) {
#pragma unroll
                for (int q = 0; q < YQ; ++q) {
                    const int t = wave + 4 * q;
                    if (t < YT) {
                        const int it = t & 1, pt = t >> 1;
                        const bf16_t *ap = &sH[(pt * 32 + l32) * SP + 8 * lh];
                        const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
                        contract_s(acc[q], ap, bp);
                        const float e = __expf(tree.s[i0 + it * 32 + l32]);
#pragma unroll
                        for (int r = 0; r < 16; ++r) acc[q][r] *= e;
                    }
                }
                if constexpr (SH) __syncthreads();   // the state tile's readers are done before the B tile takes its place
            }
        }
        store_rows(breg, sB, j0);
        store_x(j0);
        int nib = ib, njb;
        if (jb == ib) {
            nib = ib + 1;
            njb = nib < nblk ? next_col(nib, -1) : 0;
        } else {
            njb = next_col(ib, jb);
        }
        const bool more = nib < nblk;
        if (more) {
            if (nib != ib) {
                load_rows(creg, Cb, c_sn, nib * kBlk);
            }
            load_rows(breg, Bb, b_sn, njb * kBlk);
            load_x(njb * kBlk);
        }
        __syncthreads();

        // ---- phase 2: Gt = B * C^T; mask and decay -> M[i][j] as bf16 ------------------------
        {
            const int it = wave & 1, jt = wave >> 1;
            floatx16 gt;
#pragma unroll
            for (int r = 0; r < 16; ++r) gt[r] = 0.f;
            const bf16_t *ap = &sB[(jt * 32 + l32) * SP + 8 * lh];
            const bf16_t *bp = &sC[(it * 32 + l32) * SP + 8 * lh];
            contract_s(gt, ap, bp);
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

        // ---- phase 3: Yt += Xt * M^T ------------------------------------------------------------
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

        // ---- after the diagonal block: fp32 Y rows staged over the B tile (its last reader was
        //      phase 2), D * x added from the X^T tile of this same block, bf16 rows stored -----
        if (jb == ib) {
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                const int t = wave + 4 * q;
                if (t < YT) {
                    const int it = t & 1, pt = t >> 1;
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const float4 v =
                            make_float4(acc[q][4 * rg], acc[q][4 * rg + 1], acc[q][4 * rg + 2], acc[q][4 * rg + 3]);
                        *reinterpret_cast<float4 *>(&sY[(it * 32 + l32) * (P + 4) + pt * 32 + 8 * rg + 4 * lh]) = v;
                    }
                }
            }
            __syncthreads();
            const unsigned short *xt = reinterpret_cast<const unsigned short *>(sXT);
#pragma unroll
            for (int q = 0; q < XQ; ++q) {
                const int idx = q * kThreads + tid;
                const int r = idx / (P / 8), c = idx % (P / 8), i = i0 + r;
                if (i < n) {
                    const float4 a0 = *reinterpret_cast<const float4 *>(&sY[r * (P + 4) + c * 8]);
                    const float4 a1 = *reinterpret_cast<const float4 *>(&sY[r * (P + 4) + c * 8 + 4]);
                    const float av[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
                    bf16x8 o;
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const float xv = __uint_as_float((uint32_t)xt[(c * 8 + e) * kNP + r] << 16);
                        o[e] = (bf16_t)fmaf(D_h, xv, av[e]);
                    }
                    uint4 ov;
                    __builtin_memcpy(&ov, &o, 16);
                    store_stream16(yb + (size_t)i * H * P + c * 8, ov);
                }
            }
        }
        if (!more) break;
        __syncthreads();   // every reader of the tiles is done before the next pair overwrites them
        new_rows = nib != ib;
        ib = nib;
        jb = njb;
    }
}

bool tree_ssd_mfma_supported(const stree_dims &d, const void *x, const void *Bm, const void *Cm,
                             const void *h0, const void *y) {
    if (d.io_dtype != STREE_BF16) return false;
    if (!(d.headdim == 32 || d.headdim == 64 || d.headdim == 128)) return false;
    if (d.dstate % 16 != 0 || d.dstate < 16) return false;
    if ((d.x_stride_n | d.b_stride_n | d.c_stride_n) % 8 != 0) return false;
    const uintptr_t bits = (uintptr_t)x | (uintptr_t)Bm | (uintptr_t)Cm | (uintptr_t)h0 | (uintptr_t)y;
    if (bits % 16 != 0) return false;
    const int npad = (d.nnodes + kBlk - 1) / kBlk * kBlk;
    return mfma_lds_plan(d.headdim, d.dstate, npad, (d.nnodes + 31) / 32).total + sizeof(TreeLds) <= 160 * 1024;
}

template <int P, bool SH, typename HT>
static LdsLimit &mfma_lds_limit() {
    static LdsLimit lim;
    return lim;
}

// the most dynamic LDS this instantiation can be launched with: what the CU has less the kernel's static part
template <int P, bool SH, typename HT>
static hipError_t prepare_pt() {
    hipFuncAttributes attr;
    const void *k = reinterpret_cast<const void *>(&tree_ssd_mfma_kernel<P, SH, HT>);
    hipError_t e = hipFuncGetAttributes(&attr, k);
    if (e != hipSuccess) return e;
    return mfma_lds_limit<P, SH, HT>().raise(k, 160 * 1024 - attr.sharedSizeBytes);
}

template <int P, bool SH, typename HT>
static hipError_t launch_pt(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                           const float *A, const void *Bm, const void *Cm, const float *D, const void *h0,
                            void *y, int32_t *status, hipStream_t st) {
    const int npad = (d.nnodes + kBlk - 1) / kBlk * kBlk;
    const size_t lds = mfma_lds_plan(P, d.dstate, npad, (d.nnodes + 31) / 32).total;
    // the dynamic-LDS limit of this instantiation (64 KB by default)
    const hipError_t e = mfma_lds_limit<P, SH, HT>().raise(
        reinterpret_cast<const void *>(&tree_ssd_mfma_kernel<P, SH, HT>), lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((tree_ssd_mfma_kernel<P, SH, HT>), dim3(d.nheads, d.batch), dim3(kThreads), lds, st, parent, d.nnodes,
                       d.nheads, d.dstate, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, step_bias(d),
                       A, (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D,
                       (const HT *)h0, (bf16_t *)y, status);
    return hipGetLastError();
}

template <int P, bool SH>
static hipError_t launch_p(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                           const float *A, const void *Bm, const void *Cm, const float *D, const void *h0,
                           void *y, int32_t *status, hipStream_t st) {
    if (d.state_dtype == STREE_BF16) return launch_pt<P, SH, bf16_t>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    return launch_pt<P, SH, float>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
}

hipError_t prepare_tree_ssd_mfma() {
    hipError_t e = hipSuccess;
#define STREE_PREP(P, SH)                                            \
    if (e == hipSuccess) e = prepare_pt<P, SH, float>();             \
    if (e == hipSuccess) e = prepare_pt<P, SH, bf16_t>()
    STREE_PREP(32, true);
    STREE_PREP(32, false);
    STREE_PREP(64, true);
    STREE_PREP(64, false);
    STREE_PREP(128, true);
    STREE_PREP(128, false);
#undef STREE_PREP
    return e;
}

hipError_t launch_tree_ssd_mfma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                const float *A, const void *Bm, const void *Cm, const float *D,
                                const void *h0, void *y, int32_t *status, hipStream_t st) {
    if (tree_ssd_mfma64_supported(d))
        return launch_tree_ssd_mfma64(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (tree_ssd_blocks_supported(d) && !(d.flags & STREE_FLAG_GENERAL_MFMA))
        return launch_tree_ssd_blocks(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    const bool sh = mfma_share_h((d.nnodes + kBlk - 1) / kBlk * kBlk);
    switch (d.headdim) {
        case 32:
            return sh ? launch_p<32, true>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                      : launch_p<32, false>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
        case 64:
            return sh ? launch_p<64, true>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                      : launch_p<64, false>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
        case 128:
            return sh ? launch_p<128, true>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                      : launch_p<128, false>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    }
    return hipErrorInvalidValue;
}

}  // namespace stree
