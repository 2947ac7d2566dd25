// Tree scan for trees of 65 .. 256 nodes: the persistent, wave-specialised kernel of
// tree_ssd_mfma64.hip carried over to several node blocks.
//
// Nodes are taken in blocks of 64 rows I and 64 columns J <= I (labels are topological, so the
// tree mask L_ij of Sec. 3 "Formalization" is zero for j > i).  A workgroup of 8 waves walks a
// contiguous run of (batch, head) units; within a unit it walks the (row block, column block)
// pairs, row block by row block, the diagonal pair last.  One such pair is a PASS:
//
//   barrier 1
//     Y waves 0-3:  first pass of a row block: phase 1  Yt[p][i] = h0b C_I^T, *= exp(s_i)
//     G waves 4-7:  X_J registers -> X^T tile; request X of the next pass;
//                   phase 2  Gt = B_J C_I^T, M = L ? Gt exp(s_i - s_j) dt_j : 0 -> LDS
//   barrier 2
//     Y waves:      phase 3  Yt += Xt M^T; on the diagonal pass y = Yt + D x, turned around per wave
//                   in LDS and stored as row pieces; on a unit's last pass the next unit's state
//                   tile registers -> LDS (bf16), request the state tile of the unit after that
//     G waves:      the next pass's B_J (and C_I when it starts a row block) registers -> LDS,
//                   request the tiles of the pass after that; wave 6 builds the tree index of the
//                   next block of 64 nodes of this unit (in the unit's last pass: of the first
//                   block of the next unit)
//
// so that every tile is in flight for a whole pass and the fp32 state tile for a whole unit.  The
// bf16 state tile stays in LDS for all row blocks of its unit (read from memory once), the tree
// index is built block by block, each before the first pass that needs it (the ancestor bit rows
// once per sequence), by one wave, with pointer doubling through LDS: lane l owns nodes l, l + 64, ...
//
// Same products, operand layouts and accumulator layouts as tree_ssd_mfma64.hip: every product is
// formed transposed, so that a lane owns one node i in all accumulators.
#include <type_traits>

#include "common.hpp"
#include "launch.hpp"

namespace stree {

namespace {

constexpr int kBk = 64;            // node block
constexpr int kNPk = kBk + 8;      // padded row of a [.. x 64] bf16 LDS tile
constexpr int kTk = 512;           // 8 waves: 4 Y waves, 4 G waves (wave 6 also builds the tree index)
constexpr int kTreeWaveK = 6;

// LDS words of the ancestor bit rows: a node of row block I has ancestors in column blocks 0..I only,
// so its row keeps 2 (I + 1) words; block I starts at word 64 I (I + 1)
__host__ __device__ constexpr int mask_words(int nb) { return kBk * nb * (nb + 1); }

template <int P, int S, int NB>
struct LdsBlocks {
    static constexpr int SP = S + 8;
    static constexpr size_t total = (size_t)2 * kBk * SP * 2 + (size_t)P * SP * 2 + (size_t)P * kNPk * 2 +
                                    (size_t)kBk * kNPk * 2 + (size_t)2 * NB * kBk * 4 + (size_t)mask_words(NB) * 4 + 16;
};

struct PassId {                    // unit k of the workgroup's run = (b, h); pair (ib, jb), jb <= ib
    int b, h, ib, jb, k;
};

// NB = node blocks the LDS tree arrays are sized for (2: trees of at most 128 nodes, 4: 256).
// WPE = waves per SIMD the register budget is sized for: 4 when two workgroups fit a CU's LDS.
// HT = type the state is kept in (fp32, or bf16: then h0 is the MFMA operand as it comes).
template <int P, int S, int NB, int WPE, typename HT>
__global__ __launch_bounds__(kTk) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void tree_ssd_blocks_kernel(
    const int32_t *__restrict__ parent, int n, int nbatch, int H, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ dt_bias, const float *__restrict__ A,
    const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const HT *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status) {
    constexpr int SP = S + 8;
    constexpr int kHalf = kTk / 2;                  // threads per role group
    constexpr int NC = kBk * (S / 8) / kHalf;       // 16-byte chunks of a C (or B) tile per G thread
    constexpr int NX = kBk * (P / 8) / kHalf;       // of an x tile per G thread
    constexpr int NH = P * S / 4 / kHalf;           // float4 chunks of h0 per Y thread
    constexpr int YT = (P / 32) * 2, YQ = YT / 4;   // Yt tiles per row block, tiles per Y wave
    constexpr int kRowsC = kHalf / (S / 8), kRowsX = kHalf / (P / 8);
    static_assert(NC >= 1 && NX >= 1 && NH >= 1 && YQ >= 1, "tile too small for this thread count");
    // separate LDS objects, so that the compiler knows that a write to one tile cannot alias a
    // read of another
    __shared__ __align__(16) bf16_t sC[kBk * SP];
    __shared__ __align__(16) bf16_t sB[kBk * SP];
    __shared__ __align__(16) bf16_t sH[P * SP];
    __shared__ __align__(16) unsigned short sXT[P * kNPk];
    __shared__ __align__(16) bf16_t sM[kBk * kNPk];
    __shared__ __align__(16) float sS2[NB * kBk];   // log2(e) s_i
    __shared__ __align__(16) float sU[NB * kBk];    // s2_j - log2(dt_j); the jump pointers while the index is built
    __shared__ __align__(16) uint32_t sMask[mask_words(NB)];
    __shared__ int sBad[1];
    __shared__ float sDh[1];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = tid >> 6;
    // the role as a scalar: the two roles are then two arms of a uniform branch, not one stretch of code
    // run under two execution masks, and neither arm inherits the other's loads in flight
    const bool isY = __builtin_amdgcn_readfirstlane(wave) < 4;
    const int rt = tid & (kHalf - 1);    // thread index within its role group
    const int nblk = (n + kBk - 1) / kBk;
    const int n_units = nbatch * H;
    const int per_xcd = (n_units + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int wg = blockIdx.x >> 3, nwg = gridDim.x >> 3;   // this workgroup among its XCD's
    const int hpg = H / G;
    // XCD x owns the contiguous unit range [x * per_xcd, ...); its workgroups split it into
    // contiguous runs (the heads of a group share their B / C rows through that XCD's L2)
    const int cnt = max(0, min(per_xcd, n_units - xcd * per_xcd));
    const int ubase = cnt / nwg, urem = cnt % nwg;
    const int u0 = xcd * per_xcd + wg * ubase + min(wg, urem);
    const int nU = ubase + (wg < urem ? 1 : 0);
    if (nU <= 0) return;

    auto opaque = [](int v) {            // a copy the compiler cannot see through: what is derived from
        asm volatile("" : "+v"(v));      // it is recomputed where used instead of kept in registers
        return v;
    };
    auto next_pass = [&](PassId p) {
        if (p.jb < p.ib) {
            ++p.jb;
        } else if (p.ib + 1 < nblk) {
            ++p.ib;
            p.jb = 0;
        } else {
            p.ib = p.jb = 0;
            ++p.k;
            if (++p.h == H) {
                p.h = 0;
                ++p.b;
            }
        }
        return p;
    };

    // ---- prefetch registers and their loaders ---------------------------------------------------
    // Rows past the tree are read from row n-1 (valid memory): no branches, and nothing to zero when
    // they are staged -- as columns j >= n they have no ancestor bit and u_j = +inf (weight 0, removed
    // by the select), as rows i >= n they only reach outputs that are never stored.
    // One register array serves both roles (a thread is either Y or G for its whole life):
    //   Y threads  pre[0 .. NH)          state tile of the next unit (fp32 bits)
    //   G threads  pre[0 .. NC)          B tile of the next pass        pre[NC .. 2 NC)   C tile of the next row block
    //              pre[2 NC .. 2 NC+NX)  x tile of the next pass
    constexpr int kPreB = 0, kPreC = NC, kPreX = 2 * NC;
    constexpr int NPRE = (NH > 2 * NC + NX) ? NH : 2 * NC + NX;
    uint4 pre[NPRE];
    int rpar[NB];                        // tree wave: parents and steps of the next unit, node lane + 64 slot
    float rdt[NB];
    float rD = 0.f;
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        rpar[s] = -1;
        rdt[s] = 0.f;
    }
    auto load_H = [&](int b, int h) {
        if (D) rD = D[h + (opaque(lane) & 0)];   // (a vector load: it queues with the state chunks)
        const char *hb = reinterpret_cast<const char *>(h0 + ((size_t)b * H + h) * P * S);
        if constexpr (sizeof(HT) == 4) {
            const uint32_t off = (uint32_t)opaque(rt) * 16u;
#pragma unroll
            for (int q = 0; q < NH; ++q) pre[q] = load_stream16(hb + q * (kHalf * 16) + off);
        } else {                                   // a bf16 state: eight values per 16-byte chunk, half as many chunks
            const uint32_t off = (uint32_t)opaque(rt) * 16u;
#pragma unroll
            for (int q = 0; q < NH / 2; ++q) pre[q] = load_stream16(hb + q * (kHalf * 16) + off);
        }
    };
    auto load_rows = [&](int r0, const bf16_t *base, long sn, int b, int g, int blk) {
        const char *rb = reinterpret_cast<const char *>(base + (size_t)b * n * sn + (size_t)g * S);
        const uint32_t t = (uint32_t)opaque(rt);
        const int rc0 = (int)(t / (S / 8)), cc0 = (int)(t % (S / 8));
#pragma unroll
        for (int q = 0; q < NC; ++q) {
            const int rr = min(blk * kBk + rc0 + q * kRowsC, n - 1);
            pre[r0 + q] = *reinterpret_cast<const uint4 *>(rb + (uint32_t)(rr * (int)sn + cc0 * 8) * 2u);
        }
    };
    auto load_B = [&](const PassId &p) { load_rows(kPreB, Bm, b_sn, p.b, p.h / hpg, p.jb); };
    auto load_C = [&](const PassId &p) { load_rows(kPreC, Cm, c_sn, p.b, p.h / hpg, p.ib); };
    auto load_X = [&](const PassId &p) {
        const char *xb = reinterpret_cast<const char *>(x + (size_t)p.b * n * x_sn + (size_t)p.h * P);
        const uint32_t t = (uint32_t)opaque(rt);
        const int rx0 = (int)(t / (P / 8)), cx0 = (int)(t % (P / 8));
#pragma unroll
        for (int q = 0; q < NX; ++q)
            pre[kPreX + q] = *reinterpret_cast<const uint4 *>(
                xb + (uint32_t)(min(p.jb * kBk + rx0 + q * kRowsX, n - 1) * (int)x_sn + cx0 * 8) * 2u);
    };
    auto load_T = [&](int b, int h) {       // tree wave
        const int ln = opaque(lane);
#pragma unroll
        for (int s = 0; s < NB; ++s) {
            const int node = min(ln + 64 * s, n - 1);
            rpar[s] = parent[(uint32_t)(b * n + node)];
            rdt[s] = dt[(uint32_t)((b * n + node) * H + h)];
        }
    };
    // ---- registers -> LDS -------------------------------------------------------------------------
    auto stage_rows = [&](int r0, bf16_t *tile) {
        const uint32_t t = (uint32_t)opaque(rt);
        const int rc0 = (int)(t / (S / 8)), cc0 = (int)(t % (S / 8));
#pragma unroll
        for (int q = 0; q < NC; ++q)
            *reinterpret_cast<uint4 *>(&tile[(rc0 + q * kRowsC) * SP + cc0 * 8]) = pre[r0 + q];
    };
    auto stage_X = [&]() {
        const uint32_t t = (uint32_t)opaque(rt);
        const int rx0 = (int)(t / (P / 8)), cx0 = (int)(t % (P / 8));
#pragma unroll
        for (int q = 0; q < NX; ++q)
            store_transposed_pair<P / 8, true>(sXT, kNPk, rx0 + q * kRowsX, cx0 * 8, pre[kPreX + q], opaque(lane));
    };
    auto stage_H = [&]() {
        const uint32_t t = (uint32_t)opaque(rt);
#pragma unroll
        for (int q = 0; q < (sizeof(HT) == 4 ? NH : NH / 2); ++q) {
            if constexpr (sizeof(HT) == 4) {
                const uint32_t e = (t + q * kHalf) * 4u, p = e / S, sidx = e % S;
                bf16x4 o;
                o[0] = (bf16_t)__uint_as_float(pre[q].x); o[1] = (bf16_t)__uint_as_float(pre[q].y);
                o[2] = (bf16_t)__uint_as_float(pre[q].z); o[3] = (bf16_t)__uint_as_float(pre[q].w);
                *reinterpret_cast<bf16x4 *>(&sH[p * SP + sidx]) = o;
            } else {                               // already the MFMA operand: copied as it came
                const uint32_t e = (t + q * kHalf) * 8u, p = e / S, sidx = e % S;
                *reinterpret_cast<uint4 *>(&sH[p * SP + sidx]) = pre[q];
            }
        }
        if (rt == 0) *sDh = rD;      // D of that unit, for the Y waves
    };

    // ---- tree index of a unit, by one wave (Sec. 3: depth-ordered packing, Eq. a_tree) --------------
    // Lane l owns nodes l + 64 slot.  The index is built one block of 64 nodes (slot) at a time, each
    // just before the first pass that needs it -- block 0 in front of the unit, block s while the Y
    // waves are in phase 3 of the unit's pass number s - 1 -- so that a unit does not wait for the
    // whole tree's index before its first pass.  Within a slot: pointer doubling in place through
    // LDS over the parents that lie in the same slot -- every node keeps a jump pointer (in sU, as
    // integer bits) and the aggregate (log-decay sum in sS2, ancestor bits in its mask row) of the
    // path segment from itself up to, not including, the jump target; a round merges the target's
    // segment and takes over its pointer -- and then one merge with the first ancestor in a lower
    // slot, whose own aggregate is complete.  A wave's LDS operations complete in order and a round
    // reads before it writes, so no barrier is needed.  The bit rows depend on the sequence only:
    // rebuilt when it changes.  In log2 units so that the decay is one v_exp_f32 per element:
    //   s2[i] = log2(e) s_i      u[j] = s2[j] - log2(dt_j)      exp(s_i - s_j) dt_j = exp2(s2[i] - u[j])
    int cpar[NB];                        // the unit's parents and steps, copied out of the load registers
    float cdt[NB];                       // (reading those again later would wait for whatever is in flight)
    bool unit_newb = true;
    float unit_A2 = 0.f;                 // log2(e) A_h of the unit (fetched once, in front of slot 0)
#pragma unroll
    for (int s = 0; s < NB; ++s) {
        cpar[s] = -1;
        cdt[s] = 0.f;
    }
    auto build_slot = [&](auto slc, bool newb) {
        constexpr int sl = decltype(slc)::value;
        const int ln = opaque(lane), node = ln + 64 * sl, lo = 64 * sl;
        const float A2 = unit_A2;
        int j = node < n ? cpar[sl] : -1;
        float s = node < n ? cdt[sl] * A2 : 0.f;
        uint2 *own = reinterpret_cast<uint2 *>(&sMask[kBk * sl * (sl + 1) + ln * 2 * (sl + 1)]);
        if (newb) {
#pragma unroll
            for (int w = 0; w <= sl; ++w)
                own[w] = make_uint2((node < n && 2 * w == (node >> 5)) ? (1u << (node & 31)) : 0u,
                                    (node < n && 2 * w + 1 == (node >> 5)) ? (1u << (node & 31)) : 0u);
        }
        sS2[node] = s;
        sU[node] = __int_as_float(j);
        for (int round = 0; round < 6; ++round) {   // chains inside a slot are at most 64 long
            const bool in = j >= lo;
            if (!__any(in)) break;
            const int q = in ? j : node;            // (a lane with nothing to merge reads its own entry)
            const float rs = sS2[q];
            const int rj = __float_as_int(sU[q]);
            if (newb) {
                const uint2 *tgt = reinterpret_cast<const uint2 *>(&sMask[kBk * sl * (sl + 1) + (q & 63) * 2 * (sl + 1)]);
                uint2 add[sl + 1];
#pragma unroll
                for (int w = 0; w <= sl; ++w) add[w] = tgt[w];
                // (another lane may read this row already merged while the owner's jump pointer in LDS is
                // still the old one: the extra bits are ancestors all the same, OR-ing them again in a
                // later round changes nothing)
#pragma unroll
                for (int w = 0; w <= sl; ++w) {
                    const uint2 o = own[w];
                    own[w] = in ? make_uint2(o.x | add[w].x, o.y | add[w].y) : o;
                }
            }
            if (in) {
                s += rs;
                j = rj;
            }
            sS2[node] = s;
            sU[node] = __int_as_float(j);
        }
        if constexpr (sl > 0) {                     // the first ancestor below this slot: its aggregate is final
            const bool has = j >= 0;
            const int q = has ? j : 0, qb = q >> 6;
            const float rs = sS2[q];
            if (newb) {
                const uint2 *tgt = reinterpret_cast<const uint2 *>(&sMask[kBk * qb * (qb + 1) + (q & 63) * 2 * (qb + 1)]);
#pragma unroll
                for (int w = 0; w < sl; ++w) {      // (the target's row has qb + 1 <= sl pairs of words)
                    const uint2 t = tgt[min(w, qb)];
                    const uint2 o = own[w];
                    own[w] = (has && w <= qb) ? make_uint2(o.x | t.x, o.y | t.y) : o;
                }
            }
            if (has) s += rs;
        }
        sS2[node] = s;
        sU[node] = s - __log2f(node < n ? cdt[sl] : 0.f);   // dt = 0 (and nodes past the tree): u = +inf, weight 0
    };
    // validation of the whole tree, the copies of its parents and steps, and slot 0
    auto build_first = [&](int b, int h, bool newb) {
        const int ln = opaque(lane);
        const float bias_h = dt_bias ? dt_bias[__builtin_amdgcn_readfirstlane(h)] : 0.f;
        int bad = 0;
#pragma unroll
        for (int sl = NB - 1; sl >= 0; --sl) {      // (descending: the smallest bad label wins)
            const int node = ln + 64 * sl;
            const int p = rpar[sl];
            const bool ok = node >= n || ((node == 0) ? (p == -1) : (p >= 0 && p < node));
            const unsigned long long bm = __ballot(!ok);
            if (bm) bad = (int)__ffsll((long long)bm) + 64 * sl;
            cpar[sl] = p;
            cdt[sl] = rdt[sl];
            if (dt_bias) cdt[sl] = node < n ? softplus_step(rdt[sl] + bias_h) : 0.f;   // raw projection -> step size
        }
        if (ln == 0) {
            *sBad = bad;
            if (status && h == 0) status[b] = bad;
        }
        unit_newb = newb;
        unit_A2 = A[__builtin_amdgcn_readfirstlane(h)] * 1.44269504088896340736f;
        if (bad) return;
        build_slot(std::integral_constant<int, 0>{}, newb);
    };
    auto build_later = [&](int sl) {                 // slot sl >= 1 of the current unit
        if (*sBad) return;
        if (sl == 1) build_slot(std::integral_constant<int, 1>{}, unit_newb);
        if constexpr (NB > 2) {
            if (sl == 2) build_slot(std::integral_constant<int, 2>{}, unit_newb);
            if (sl == 3) build_slot(std::integral_constant<int, 3>{}, unit_newb);
        }
    };

    // ---- the two roles run their own loops (same barrier sequence in both) ---------------------------
    // A role requests its loads at the TOP of a loop iteration and has ONE point, at the bottom, at
    // which it waits for them, stages what arrived: no load is pending where control flow merges (the
    // loop entry, the back edge).  The compiler's wait-count bookkeeping does not survive such a merge
    // of paths with different loads in flight -- it falls back to waiting for everything wherever a
    // register that MAY have a load pending is touched, which turns every use of a reused register
    // into a wait for requests issued a moment ago.  For the same reason the roles share no code inside
    // the loop: registers with a load pending in one role would be temporaries of the other.  (The
    // state tile and the tree wave's parents / steps are the exception: requested at a unit's first
    // pass, used at its last; their registers hold nothing else in between.)
    const int ub0 = __builtin_amdgcn_readfirstlane(u0 / H), uh0 = __builtin_amdgcn_readfirstlane(u0 % H);
    PassId cur = {ub0, uh0, 0, 0, 0};
    PassId n1 = next_pass(cur);

    if (isY) {
        floatx16 acc[YQ];                // Yt tiles of the current row block
        if (h0) {
            load_H(cur.b, cur.h);
            stage_H();
        } else if (rt == 0) {
            *sDh = D ? D[cur.h] : 0.f;
        }
        while (true) {
            // a unit's last pass: the next unit's state tile, in flight for this pass
            if (h0 && cur.ib == nblk - 1 && cur.jb == cur.ib && cur.k + 1 < nU) load_H(n1.b, n1.h);
            __syncthreads();                                  // barrier 1: the tiles of this pass are staged
            const int bad = *sBad;
            const float D_h = *sDh;
            const bool diag = cur.ib == cur.jb;
            const int i0 = cur.ib * kBk;
            if (cur.jb == 0) {
                // ---- phase 1 (once per row block): Yt = h0b C^T, then *= exp(s_i) ----------------------
#pragma unroll
                for (int q = 0; q < YQ; ++q)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
                if (h0 && !bad) {
                    const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, il = (opaque(wave) & 1) * 32 + l32;
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
                                    &sH[(((opaque(wave) + 4 * q) >> 1) * 32 + l32) * SP + 8 * lh + kb + 16 * j]);
                        }
#pragma unroll
                        for (int j = 0; j < S / 32; ++j)
#pragma unroll
                            for (int q = 0; q < YQ; ++q)
                                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(hf[q][j], cf[j], acc[q], 0, 0, 0);
                        __builtin_amdgcn_sched_barrier(0);
                    }
                    const float e = __builtin_amdgcn_exp2f(sS2[i0 + il]);
#pragma unroll
                    for (int q = 0; q < YQ; ++q)
#pragma unroll
                        for (int rg = 0; rg < 16; ++rg) acc[q][rg] *= e;
                }
            }
            __syncthreads();                                  // barrier 2: M is ready
            const bool last_of_unit = diag && cur.ib == nblk - 1;
            const bool more_units = cur.k + 1 < nU;
            // ---- phase 3: Yt += Xt M^T (diagonal pair: nodes i < 32 have no ancestor j >= 32) ----------
            bf16x4 yreg[YQ][4];
            {
                const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, it = opaque(wave) & 1, il = it * 32 + l32;
#pragma unroll
                for (int q = 0; q < YQ; ++q) {
                    const int pt = (opaque(wave) + 4 * q) >> 1;
                    if (!bad) {
                        const bf16_t *xt = reinterpret_cast<const bf16_t *>(sXT);   // (swizzled: transposed_at)
                        const bf16_t *bp = &sM[il * kNPk + 8 * lh];
                        if (it || !diag) {
                            bf16x8 a[4], bb[4];
#pragma unroll
                            for (int j = 0; j < 4; ++j) {
                                a[j] = *reinterpret_cast<const bf16x8 *>(
                                    xt + transposed_at<true>(kNPk, pt * 32 + l32, 8 * lh + 16 * j));
                                bb[j] = *reinterpret_cast<const bf16x8 *>(bp + 16 * j);
                            }
#pragma unroll
                            for (int j = 0; j < 4; ++j)
                                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], bb[j], acc[q], 0, 0, 0);
                        } else {
                            bf16x8 a[2], bb[2];
#pragma unroll
                            for (int j = 0; j < 2; ++j) {
                                a[j] = *reinterpret_cast<const bf16x8 *>(
                                    xt + transposed_at<true>(kNPk, pt * 32 + l32, 8 * lh + 16 * j));
                                bb[j] = *reinterpret_cast<const bf16x8 *>(bp + 16 * j);
                            }
#pragma unroll
                            for (int j = 0; j < 2; ++j)
                                acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j], bb[j], acc[q], 0, 0, 0);
                        }
                    }
                    if (diag) {
                        // y = Yt + D x (x_i from the X^T tile: on the diagonal pair J = I); bf16 in
                        // registers until stored
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {
                            bf16x4 o;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const float xv =
                                    __uint_as_float((uint32_t)sXT[transposed_at<true>(kNPk, pt * 32 + 8 * rg + 4 * lh + e, il)] << 16);
                                o[e] = bad ? (bf16_t)0.f : (bf16_t)fmaf(D_h, xv, acc[q][4 * rg + e]);
                            }
                            yreg[q][rg] = o;
                        }
                    }
                }
            }
            // the next unit's state tile registers -> LDS: the one wait for loads of this role; before the
            // y stores below, so that it is not a wait for those stores as well
            if (last_of_unit && more_units) {
                if (h0) stage_H();
                else if (rt == 0) *sDh = D ? D[n1.h] : 0.f;
            }
            // y leaves as 64-byte row pieces: each wave turns its 32x32 tile around in a private 2 KB
            // of the B tile's LDS (idle until barrier (a)) and stores 16 bytes per lane, four lanes to
            // a row; through L2 with the streaming hint
            if (diag) {
                // (the rest of this sequence's y from this head's first column: the bound of the buffer stores)
                const __amdgpu_buffer_rsrc_t yb = make_store_rsrc(y + (size_t)cur.b * n * H * P + (size_t)cur.h * P,
                                                                  (uint32_t)(n * H * P - cur.h * P) * 2u);
                char *ys = reinterpret_cast<char *>(sB) + opaque(wave) * 2048;
                const int ln = opaque(lane), wr = ln & 31, wh = ln >> 5;
                const int rr = ln >> 2, rc = ln & 3;
#pragma unroll
                for (int q = 0; q < YQ; ++q) {
                    const int pt = (opaque(wave) + 4 * q) >> 1;
                    // row r keeps its 16-byte chunk c at slot c ^ ((r >> 2) & 3)
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg)
                        *reinterpret_cast<bf16x4 *>(ys + wr * 64 + ((rg ^ ((wr >> 2) & 3)) * 16) + wh * 8) = yreg[q][rg];
#pragma unroll
                    for (int half = 0; half < 2; ++half) {
                        const int row = half * 16 + rr;
                        const uint4 v = *reinterpret_cast<const uint4 *>(ys + row * 64 + ((rc ^ ((row >> 2) & 3)) * 16));
                        const int node = i0 + (opaque(wave) & 1) * 32 + row;
                        if (node < n) buffer_store_through16(yb, (uint32_t)(node * H * P + pt * 32 + rc * 8) * 2u, v);
                    }
                }
            }
            __syncthreads();                                  // barrier (a): X^T, M and the y scratch are dead
            if (n1.k >= nU) break;
            cur = n1;
            n1 = next_pass(n1);
        }
    } else {
        floatx16 gt;                     // this wave's Gt tile
        const bool isT = __builtin_amdgcn_readfirstlane(wave) == kTreeWaveK;
        if (isT) load_T(cur.b, cur.h);                       // (first: the index waits for these alone)
        load_C(cur);
        load_B(cur);
        load_X(cur);
        if (isT) build_first(cur.b, cur.h, true);
        stage_rows(kPreC, sC);
        stage_rows(kPreB, sB);
        stage_X();
        while (true) {
            // the next pass's tiles: in flight for this whole pass
            // the next unit's parents and steps (tree wave): in flight for this whole unit
            if (isT && cur.ib == 0 && cur.jb == 0 && cur.k + 1 < nU) {
                int b1 = cur.b, h1 = cur.h;
                if (++h1 == H) {
                    h1 = 0;
                    ++b1;
                }
                load_T(b1, h1);
            }
            const bool v1 = n1.k < nU;
            if (v1) {
                load_B(n1);
                load_X(n1);
                if (n1.jb == 0) load_C(n1);
            }
            __syncthreads();                                  // barrier 1
            const int bad = *sBad;
            const bool diag = cur.ib == cur.jb;
            const int i0 = cur.ib * kBk, j0 = cur.jb * kBk;
            // ---- phase 2: Gt = B_J C_I^T, mask and decay -> M.  On the diagonal pair the tile with
            //      j >= 32 > i is all zero: neither computed nor read ---------------------------------
            const int jt = (opaque(wave) - 4) >> 1, it = opaque(wave) & 1;
            if (!bad && !(diag && it == 0 && jt == 1)) {
                const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, il = it * 32 + l32;
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
                const float s2_i = sS2[i0 + il];
                // bit 8*rg + e of mrow <-> j = j0 + jt*32 + 8*rg + 4*lh + e
                const uint32_t mrow =
                    sMask[kBk * cur.ib * (cur.ib + 1) + il * 2 * (cur.ib + 1) + cur.jb * 2 + jt] >> (4 * lh);
                float4 uj[4];
#pragma unroll
                for (int rg = 0; rg < 4; ++rg)
                    uj[rg] = *reinterpret_cast<const float4 *>(&sU[j0 + jt * 32 + 8 * rg + 4 * lh]);
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
                    *reinterpret_cast<bf16x4 *>(&sM[il * kNPk + jl]) = o;
                }
            }
            __syncthreads();                                  // barrier 2: M is ready; B, C and the tree arrays are dead
            const bool last_of_unit = diag && cur.ib == nblk - 1;
            const bool more_units = cur.k + 1 < nU;
            // the tree index while the Y waves are in phase 3: the current unit's next block of nodes, or,
            // in its last pass, the next unit's first
            if (isT) {
                const int pidx = cur.ib * (cur.ib + 1) / 2 + cur.jb;      // number of this pass within its unit
                if (pidx + 1 < nblk) build_later(pidx + 1);
                else if (last_of_unit && more_units) build_first(n1.b, n1.h, n1.b != cur.b);
            }
            __syncthreads();                                  // barrier (a): X^T and the y scratch in the B tile are dead
            // ---- the one wait of this role: the next pass's tiles registers -> LDS ----------------------
            if (!v1) break;
            stage_rows(kPreB, sB);
            stage_X();
            if (n1.jb == 0) stage_rows(kPreC, sC);
            cur = n1;
            n1 = next_pass(n1);
        }
    }
}

template <int P, int S, int NB>
hipError_t launch_blocks_ps(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                            const void *Bm, const void *Cm, const float *D, const void *h0, void *y,
                            int32_t *status, hipStream_t st) {
    constexpr size_t lds = LdsBlocks<P, S, NB>::total;        // static LDS (upper bound)
    constexpr int WPE = (2 * (lds + 64) <= 160 * 1024) ? 4 : 2;
    const int n_units = d.batch * d.nheads;
    int grid = (n_units + 7) / 8 * 8;
    const int cap = 256 * (WPE == 4 ? 2 : 1);
    if (grid > cap) grid = cap;
#define STREE_LAUNCH_BLOCKS(HT)                                                                                       \
    hipLaunchKernelGGL((tree_ssd_blocks_kernel<P, S, NB, WPE, HT>), dim3(grid), dim3(kTk), 0, st, parent, d.nnodes,   \
                       d.batch, d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt, step_bias(d), A,      \
                       (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm, (long)d.c_stride_n, D,             \
                       (const HT *)h0, (bf16_t *)y, status)
    if (d.state_dtype == STREE_BF16) STREE_LAUNCH_BLOCKS(bf16_t);
    else STREE_LAUNCH_BLOCKS(float);
#undef STREE_LAUNCH_BLOCKS
    return hipGetLastError();
}

}  // namespace

// bf16, 65 .. 256 nodes, the head shapes below; alignment is checked by the caller (tree_ssd_mfma_supported)
bool tree_ssd_blocks_supported(const stree_dims &d) {
    if (d.nnodes <= kBk || d.nnodes > 4 * kBk) return false;
    return (d.headdim == 64 && (d.dstate == 128 || d.dstate == 64 || d.dstate == 256)) ||
           (d.headdim == 128 && d.dstate == 128);
}

hipError_t launch_tree_ssd_blocks(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D, const void *h0,
                                  void *y, int32_t *status, hipStream_t st) {
    const bool small = d.nnodes <= 2 * kBk;
    if (d.headdim == 128)
        return small ? launch_blocks_ps<128, 128, 2>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                     : launch_blocks_ps<128, 128, 4>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (d.dstate == 128)
        return small ? launch_blocks_ps<64, 128, 2>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                     : launch_blocks_ps<64, 128, 4>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    if (d.dstate == 256)
        return small ? launch_blocks_ps<64, 256, 2>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                     : launch_blocks_ps<64, 256, 4>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
    return small ? launch_blocks_ps<64, 64, 2>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st)
                 : launch_blocks_ps<64, 64, 4>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, st);
}

}  // namespace stree
