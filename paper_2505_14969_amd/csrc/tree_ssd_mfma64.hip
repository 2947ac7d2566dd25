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
//     Y: phase 3  Yt += Xt M^T; y = Yt + D x -> bf16, turned around per wave in LDS, stored as row pieces
//     Y or G (whoever carries unit k+1): h0(k+1) regs -> LDS as bf16; issue h0(k+3) loads
//     G: new C tile if unit k+1 starts another sequence or group
//     T: tree index of unit k+1, issue parent/dt (k+2) loads
//     G: x(k+1) regs -> the other X^T tile in LDS, issue x(k+2) loads
// so the big global loads (h0, x) are in flight for a whole unit period.
//
// Template flag RP folds the commit of the previous tree into the state as it is loaded
// (Alg. 1: replay at the start of the next iteration).
#include "common.hpp"
#include "launch.hpp"

namespace stree {

namespace {

constexpr int kB64 = 64;
constexpr int kNP64 = kB64 + 8;
constexpr int kT64 = 512;   // 8 waves: 4 Y waves, 3 G waves, 1 tree wave

constexpr int kRC = 8;      // path nodes of the previous tree whose x / B rows are staged in LDS per unit
constexpr int kYStage = 4 * 2048;   // bytes at the start of the B tile's LDS that the Y waves turn y around in

// static LDS of the kernel below (C, B, h0b tiles, two X^T tiles, M, tree arrays; with replay
// the path arrays and, where the B tile has no room behind the y staging area, the path rows)
template <int P, int S>
struct Lds64 {
    static constexpr int SP = S + 8;
    static constexpr size_t replay_rows = (size_t)kRC * (P + S) * 2;
    static constexpr bool rows_in_b = (size_t)kB64 * SP * 2 >= kYStage + replay_rows;
    static constexpr size_t total = (size_t)2 * kB64 * SP * 2 + (size_t)P * SP * 2 + (size_t)2 * P * kNP64 * 2 +
                                    (size_t)kB64 * kNP64 * 2 + 1040;
    static constexpr size_t total_replay = total + 336 + (rows_in_b ? 0 : replay_rows);
};

// The previous iteration's tree and cached activations (fused replay variant only).
struct ReplayArgs {
    const int32_t *parent, *accepted;   // [B, pn], [B]
    const bf16_t *x, *Bm;               // [B, pn, H, P], [B, pn, G, S] with token strides x_sn, b_sn
    const float *dt;                    // [B, pn, H]
    long x_sn, b_sn;
    int pn;
    void *h_out;                        // [B, H, P, S]: the replayed state, in the type the state is kept in
    int32_t *status;                    // [B] or null
};

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
        const float rs = wave_read(s, q);
        const int rp = wave_read(p, q);
        const uint32_t rlo = wave_read(mlo, q), rhi = wave_read(mhi, q);
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

// WPE = waves per SIMD the register budget is sized for: 4 when two workgroups fit a CU's LDS.
//
// RP = fused activation replay (Alg. 1): the state loaded for a unit is first advanced along the
// accepted path of the previous tree,
//   h* = exp(s_k) h0 + sum_{j on path(k)} dt_j exp(s_k - s_j) x_j (outer) B_j,
// in the fp32 registers it arrives in, written back once to h_out, and only then rounded to the
// bf16 MFMA operand.  The tree wave works the path of the next unit out in the scan half, in which
// it has nothing else to do (same pointer doubling as the tree index, on the previous tree), and
// asks for the x / B rows of its first kRC nodes; they are in flight until the staging half,
// where it puts them into LDS; one more barrier per unit (c) separates that from the FMAs of the
// threads that carry the unit.  Longer paths read the remaining rows from
// global memory.  Each thread owns one 4-wide piece of the state index and NH consecutive rows.
// HT = type the state is kept in: fp32, or bf16 (then h0 is the MFMA operand as it comes, and the replayed
// state is rounded once, to the value that is both written back and scanned from).
template <int P, int S, int WPE, bool RP, bool SPL, typename HT>
__global__ __launch_bounds__(kT64) __attribute__((amdgpu_waves_per_eu(WPE, WPE))) void tree_ssd_mfma64_kernel(
    const int32_t *__restrict__ parent, int n, int nbatch, int H, int G, const bf16_t *__restrict__ x, long x_sn,
    const float *__restrict__ dt, const float *__restrict__ dt_bias, const float *__restrict__ A,
    const bf16_t *__restrict__ Bm, long b_sn,
    const bf16_t *__restrict__ Cm, long c_sn, const float *__restrict__ D, const HT *__restrict__ h0,
    bf16_t *__restrict__ y, int32_t *__restrict__ status, ReplayArgs R) {
    using L = Lds64<P, S>;
    constexpr int SP = L::SP;
    constexpr int kHalf = kT64 / 2;                 // threads per role group
    constexpr int NC = kB64 * (S / 8) / kHalf;      // 16-byte chunks of C (and of B) per G thread
    constexpr int NX = kB64 * (P / 8) / kHalf;      // of x per G thread; of y per Y thread
    constexpr int NH = P * S / 4 / kHalf;           // float4 chunks of h0 per Y thread
    constexpr int YT = (P / 32) * 2, YQ = YT / 4;   // Yt tiles, tiles per Y wave
    constexpr int kRowsC = kHalf / (S / 8), kRowsX = kHalf / (P / 8);
    static_assert(NC >= 1 && NX >= 1 && NH >= 1 && YQ >= 1, "tile too small for this thread count");
    static_assert(!RP || NH % 4 == 0, "replay reads a thread's x values four at a time");
    static_assert(NH % 2 == 0 && S % 8 == 0, "a bf16 state is moved eight values at a time");
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
    // replay: path of the accepted node (position -> node, weight), its length and exp(s_k)
    __shared__ float sRcoef[RP ? kB64 : 1];
    __shared__ unsigned char sRnode[RP ? kB64 : 4];
    __shared__ int sRlen[1];
    __shared__ float sRdec[1];
    __shared__ __align__(16) bf16_t sRrows[(RP && !L::rows_in_b) ? kRC * (P + S) : 8];

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = tid >> 6;
    constexpr int kTreeWave = 6;
    const bool isY = wave < 4;
    const int rt = tid & (kHalf - 1);    // thread index within its role group
    const int n_units = nbatch * H;
    const int per_xcd = (n_units + 7) >> 3;
    const int xcd = blockIdx.x & 7;
    const int wg = blockIdx.x >> 3, nwg = gridDim.x >> 3;   // this workgroup among its XCD's
    const int hpg = H / G;
    // XCD x owns the contiguous unit range [x*per_xcd, ...); its workgroups split that range
    // into contiguous runs, so a workgroup mostly sees consecutive heads of one sequence and
    // group: their C, B tiles, the tree mask and Gt = B C^T are then reused, not redone.
    const int cnt = max(0, min(per_xcd, n_units - xcd * per_xcd));
    // the first cnt % nwg workgroups take one unit more.  (Workgroups are placed one per CU first and
    // the second one per CU later: a CU then holds workgroup w and w + nwg/2, a long and a short run.)
    const int ubase = cnt / nwg, urem = cnt % nwg;
    const int u0 = xcd * per_xcd + wg * ubase + min(wg, urem);
    const int nU = ubase + (wg < urem ? 1 : 0);
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
    float rdt = 0.f;
    // The chunk coordinates of a thread are loop invariants; keeping them all in registers
    // across the unit loop would cost more registers than the budget of 128 allows, so every
    // helper below re-derives them from an opaque copy of the thread index (a few VALU ops).
    auto opaque = [](int v) {
        asm volatile("" : "+v"(v));
        return v;
    };
    // the node half of the tiles a wave owns.  With the replay the register budget has no room for
    // it (nor for anything else the compiler would hoist out of the unit loop): kept live it is
    // spilled, and a reload waits for every load in flight, so there it is re-derived where used
    // from a copy of the wave index that the compiler cannot see through.
    const int it0 = wave & 1;

    float rD = 0.f;                  // D[h] of the unit whose h0 is in pre[]
    // chunk q of a thread: without replay element (t + q*kHalf)*4 of the P x S tile; with replay
    // row (t / S4) * NH + q, piece t % S4, so that a thread's rows are consecutive
    constexpr int S4 = S / 4;
    // replay on a state kept in bf16: a thread owns NH/2 rows of EIGHT columns, so that the state moves in
    // 16-byte pieces as the fp32 one does (where its x values still come four at a time; otherwise the
    // fp32 map with 8-byte pieces)
    constexpr bool kWide = RP && sizeof(HT) == 2 && (NH / 2) % 4 == 0;
    auto load_H = [&](int b, int h) {       // the role group that carries this unit
        // the lane-dependent zero keeps this a vector load: it then sits in the same in-order
        // queue as the h0 chunks instead of forcing a scalar-cache wait in the hot window
        if (D) rD = D[h + (opaque(lane) & 0)];
        const char *hb = reinterpret_cast<const char *>(h0 + ((size_t)b * H + h) * P * S);
        constexpr uint32_t HB = sizeof(HT);    // a bf16 state: the same four values per chunk, in 8 bytes
        auto chunk = [&](int q, const char *src) {
            if constexpr (HB == 4) {
                pre[q] = load_stream16(src);
            } else {
                const uint2 v = load_stream8(src);
                pre[q].x = v.x;
                pre[q].y = v.y;
            }
        };
        if constexpr (kWide) {                 // replay on a bf16 state: NH/2 rows of eight columns per thread
            const int t = opaque(rt);
            const uint32_t off = (uint32_t)(((t / (S / 8)) * (NH / 2)) * S + (t % (S / 8)) * 8) * 2u;
#pragma unroll
            for (int q = 0; q < NH / 2; ++q) pre[q] = load_stream16(hb + off + q * (S * 2));
        } else if constexpr (RP) {
            const int t = opaque(rt);
            const uint32_t off = (uint32_t)(((t / S4) * NH) * S + (t % S4) * 4) * HB;
#pragma unroll
            for (int q = 0; q < NH; ++q) chunk(q, hb + off + q * (S * HB));
        } else if constexpr (HB == 4) {
            const uint32_t off = (uint32_t)opaque(rt) * 16u;
#pragma unroll
            for (int q = 0; q < NH; ++q) pre[q] = load_stream16(hb + q * (kHalf * 16) + off);
        } else {                               // no replay, bf16 state: eight values per 16-byte chunk, half as many chunks
            const uint32_t off = (uint32_t)opaque(rt) * 16u;
#pragma unroll
            for (int q = 0; q < NH / 2; ++q) pre[q] = load_stream16(hb + q * (kHalf * 16) + off);
        }
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
    };
    // ---- registers -> LDS -------------------------------------------------------------------------
    // rbuf: the LDS rows of the replayed path (x rows [kRC][P], then B rows [kRC][S]); b, h: the unit
    auto stage_H = [&]([[maybe_unused]] const char *rbuf, [[maybe_unused]] int b, [[maybe_unused]] int h) {
        const int t = opaque(rt);
        if constexpr (kWide) {
            constexpr int S8 = S / 8, NR = NH / 2;
            const int prow = (t / S8) * NR, s8 = t % S8;
            const int len = *sRlen;
            const float dec = *sRdec;
            float hv[NR][8];
#pragma unroll
            for (int q = 0; q < NR; ++q) {
                const uint32_t w4[4] = {pre[q].x, pre[q].y, pre[q].z, pre[q].w};
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    hv[q][2 * e] = dec * bf16_lo(w4[e]);
                    hv[q][2 * e + 1] = dec * bf16_hi(w4[e]);
                }
            }
            auto rank1 = [&](float cf, uint4 b8, const uint32_t (&xw)[NR / 2]) {
                const float bv[8] = {cf * bf16_lo(b8.x), cf * bf16_hi(b8.x), cf * bf16_lo(b8.y), cf * bf16_hi(b8.y),
                                     cf * bf16_lo(b8.z), cf * bf16_hi(b8.z), cf * bf16_lo(b8.w), cf * bf16_hi(b8.w)};
#pragma unroll
                for (int q = 0; q < NR; ++q) {
                    const float xv = (q & 1) ? bf16_hi(xw[q >> 1]) : bf16_lo(xw[q >> 1]);
#pragma unroll
                    for (int e = 0; e < 8; ++e) hv[q][e] = fmaf(xv, bv[e], hv[q][e]);
                }
            };
            const int nl = min(len, kRC);
            for (int j = 0; j < nl; ++j) {
                const uint4 b8 = *reinterpret_cast<const uint4 *>(rbuf + (kRC * P + j * S + s8 * 8) * 2);
                uint32_t xw[NR / 2];
#pragma unroll
                for (int w = 0; w < NR / 2; w += 2) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(rbuf + (j * P + prow + 2 * w) * 2);
                    xw[w] = v.x;
                    xw[w + 1] = v.y;
                }
                rank1(sRcoef[j], b8, xw);
            }
            if (len > kRC) {   // the rest of a long path: rows straight from global memory
                const int g = h / hpg;
                const char *xb = reinterpret_cast<const char *>(R.x + (size_t)b * R.pn * R.x_sn + (size_t)h * P + prow);
                const char *Bb = reinterpret_cast<const char *>(R.Bm + (size_t)b * R.pn * R.b_sn + (size_t)g * S + s8 * 8);
                for (int j = kRC; j < len; ++j) {
                    const int node = sRnode[j];
                    const uint4 b8 = *reinterpret_cast<const uint4 *>(Bb + (size_t)node * R.b_sn * 2);
                    uint32_t xw[NR / 2];
#pragma unroll
                    for (int w = 0; w < NR / 2; w += 2) {
                        const uint2 v = *reinterpret_cast<const uint2 *>(xb + ((size_t)node * R.x_sn + 2 * w) * 2);
                        xw[w] = v.x;
                        xw[w + 1] = v.y;
                    }
                    rank1(sRcoef[j], b8, xw);
                }
            }
            // the replayed state, rounded once: the value written back (through L2) is the MFMA operand
            char *ob = reinterpret_cast<char *>(reinterpret_cast<HT *>(R.h_out) + ((size_t)b * H + h) * P * S);
#pragma unroll
            for (int q = 0; q < NR; ++q) {
                const uint2 lo = pack_bf16x4(hv[q][0], hv[q][1], hv[q][2], hv[q][3]);
                const uint2 hi = pack_bf16x4(hv[q][4], hv[q][5], hv[q][6], hv[q][7]);
                const uint4 o = make_uint4(lo.x, lo.y, hi.x, hi.y);
                store_through16(ob + (uint32_t)((prow + q) * S + s8 * 8) * 2u, o);
                *reinterpret_cast<uint4 *>(&sH[(prow + q) * SP + s8 * 8]) = o;
            }
        } else if constexpr (RP) {
            const int prow = (t / S4) * NH, s4 = t % S4;
            const int len = *sRlen;
            const float dec = *sRdec;
            float hv[NH][4];
#pragma unroll
            for (int q = 0; q < NH; ++q) {
                if constexpr (sizeof(HT) == 4) {
                    hv[q][0] = dec * __uint_as_float(pre[q].x); hv[q][1] = dec * __uint_as_float(pre[q].y);
                    hv[q][2] = dec * __uint_as_float(pre[q].z); hv[q][3] = dec * __uint_as_float(pre[q].w);
                } else {
                    hv[q][0] = dec * bf16_lo(pre[q].x); hv[q][1] = dec * bf16_hi(pre[q].x);
                    hv[q][2] = dec * bf16_lo(pre[q].y); hv[q][3] = dec * bf16_hi(pre[q].y);
                }
            }
            auto rank1 = [&](float cf, uint2 b4, const uint32_t (&xw)[NH / 2]) {
                const float bv[4] = {cf * bf16_lo(b4.x), cf * bf16_hi(b4.x), cf * bf16_lo(b4.y), cf * bf16_hi(b4.y)};
#pragma unroll
                for (int q = 0; q < NH; ++q) {
                    const float xv = (q & 1) ? bf16_hi(xw[q >> 1]) : bf16_lo(xw[q >> 1]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) hv[q][e] = fmaf(xv, bv[e], hv[q][e]);
                }
            };
            const int nl = min(len, kRC);
            for (int j = 0; j < nl; ++j) {
                const uint2 b4 = *reinterpret_cast<const uint2 *>(rbuf + (kRC * P + j * S + s4 * 4) * 2);
                uint32_t xw[NH / 2];
#pragma unroll
                for (int w = 0; w < NH / 2; w += 2) {
                    const uint2 v = *reinterpret_cast<const uint2 *>(rbuf + (j * P + prow + 2 * w) * 2);
                    xw[w] = v.x;
                    xw[w + 1] = v.y;
                }
                rank1(sRcoef[j], b4, xw);
            }
            if (len > kRC) {   // the rest of a long path: rows straight from global memory
                const int g = h / hpg;
                const char *xb = reinterpret_cast<const char *>(R.x + (size_t)b * R.pn * R.x_sn + (size_t)h * P + prow);
                const char *Bb = reinterpret_cast<const char *>(R.Bm + (size_t)b * R.pn * R.b_sn + (size_t)g * S + s4 * 4);
                for (int j = kRC; j < len; ++j) {
                    const int node = sRnode[j];
                    const uint2 b4 = *reinterpret_cast<const uint2 *>(Bb + (size_t)node * R.b_sn * 2);
                    uint32_t xw[NH / 2];
#pragma unroll
                    for (int w = 0; w < NH / 2; w += 2) {
                        const uint2 v = *reinterpret_cast<const uint2 *>(xb + ((size_t)node * R.x_sn + 2 * w) * 2);
                        xw[w] = v.x;
                        xw[w + 1] = v.y;
                    }
                    rank1(sRcoef[j], b4, xw);
                }
            }
            // the replayed state: written once, through L2 (never read again by this kernel)
            char *ob = reinterpret_cast<char *>(reinterpret_cast<HT *>(R.h_out) + ((size_t)b * H + h) * P * S);
#pragma unroll
            for (int q = 0; q < NH; ++q) {
                bf16x4 o;
                o[0] = (bf16_t)hv[q][0]; o[1] = (bf16_t)hv[q][1]; o[2] = (bf16_t)hv[q][2]; o[3] = (bf16_t)hv[q][3];
                if constexpr (sizeof(HT) == 4)
                    store_through16(ob + (uint32_t)((prow + q) * S + s4 * 4) * 4u,
                                    make_uint4(__float_as_uint(hv[q][0]), __float_as_uint(hv[q][1]),
                                               __float_as_uint(hv[q][2]), __float_as_uint(hv[q][3])));
                else
                    store_through8(ob + (uint32_t)((prow + q) * S + s4 * 4) * 2u, __builtin_bit_cast(uint2, o));
                *reinterpret_cast<bf16x4 *>(&sH[(prow + q) * SP + s4 * 4]) = o;
            }
        } else if constexpr (sizeof(HT) == 4) {
#pragma unroll
            for (int q = 0; q < NH; ++q) {
                const int e = (t + q * kHalf) * 4, p = e / S, sidx = e % S;
                bf16x4 o;
                o[0] = (bf16_t)__uint_as_float(pre[q].x); o[1] = (bf16_t)__uint_as_float(pre[q].y);
                o[2] = (bf16_t)__uint_as_float(pre[q].z); o[3] = (bf16_t)__uint_as_float(pre[q].w);
                *reinterpret_cast<bf16x4 *>(&sH[p * SP + sidx]) = o;
            }
        } else {                                   // already the MFMA operand: copied as it came
#pragma unroll
            for (int q = 0; q < NH / 2; ++q) {
                const int e = (t + q * kHalf) * 8, p = e / S, sidx = e % S;
                *reinterpret_cast<uint4 *>(&sH[p * SP + sidx]) = pre[q];
            }
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
            store_transposed_pair<P / 8>(sXT, kNP64, rr, cx0 * 8,
                                         make_uint4(xq.x & keep, xq.y & keep, xq.z & keep, xq.w & keep), opaque(lane));
        }
    };
    auto stage_T = [&](int h) {
        const int ln = opaque(lane);   // LDS addresses re-derived here, not carried across the loop
        float dt_i = rdt;
        if constexpr (SPL) dt_i = softplus_step(rdt + dt_bias[h]);               // raw projection -> step size
        const int bad = wave_tree_index(ln, n, rpar, dt_i, A[h], sS2, sU, sMask);
        if (ln == 0) *sBad = bad;
    };

    // ---- replay (tree wave): previous tree's path one unit ahead ----------------------------------
    // Registers that only the tree wave needs live in its copy of acc[0], which it never uses
    // as an accumulator: 0-3 x row pieces, 4-11 B row pieces, 12 position on the path, 13 weight,
    // 14 path length, 15 exp(s_k).
    constexpr int PX = P / 8, PB = S / 8;                     // 16-byte pieces per x row, per B row
    constexpr int NXG = (kRC * PX + 63) / 64, NBG = (kRC * PB + 63) / 64;   // pieces per lane
    static_assert(!RP || (NXG <= 1 && NBG <= 2) || WPE < 4, "tree-wave registers exceed its accumulator copy");
    int rpp = -1;
    float rpdt = 0.f;
    uint4 gxw[(RP && WPE < 4) ? NXG : 1], gbw[(RP && WPE < 4) ? NBG : 1];   // roomy variants: plain registers
    int wpos = -1, wlen = 0;
    float wcf = 0.f, wdec = 1.f;
    auto load_R = [&](int b, int h) {
        const int node = min(opaque(lane), R.pn - 1);
        rpp = R.parent[(uint32_t)(b * R.pn + node)];
        rpdt = R.dt[(uint32_t)((b * R.pn + node) * H + h)];
    };
    auto path_R = [&](floatx16 &tw, int b, int h) {
        const int ln = opaque(lane);
        const int pn = R.pn;
        // uniform values by scalar loads (a vector load here would be the newest one in flight, and
        // waiting for it would wait for the whole h0 prefetch)
        const int rk = R.accepted[__builtin_amdgcn_readfirstlane(b)];
        const float rRA = A[__builtin_amdgcn_readfirstlane(h)];
        float pdt_i = rpdt;
        if constexpr (SPL) pdt_i = softplus_step(rpdt + dt_bias[__builtin_amdgcn_readfirstlane(h)]);
        const bool kbad = rk < -1 || rk >= pn;
        int pos = -1, len = 0;
        float cf = 0.f, dc = 1.f;
        const int st = wave_path(ln, pn, (rk >= 0 && !kbad) ? rk : 0, rpp, pdt_i, rRA, pos, cf, len, dc);
        if (st != 0 || rk < 0 || kbad) {   // nothing to replay: the state passes through
            pos = -1;
            len = 0;
            cf = 0.f;
            dc = 1.f;
        }
        if (R.status && h == 0 && ln == 0) R.status[b] = st ? st : (kbad ? -1 : 0);
        // x / B rows of the first kRC path nodes: 16-byte pieces dealt over the lanes
        const int g = h / hpg;
        const char *xb = reinterpret_cast<const char *>(R.x + (size_t)b * pn * R.x_sn + (size_t)h * P);
        const char *Bb = reinterpret_cast<const char *>(R.Bm + (size_t)b * pn * R.b_sn + (size_t)g * S);
        int nx[NXG], nb[NBG];      // node of the path position each of this lane's pieces belongs to
#pragma unroll
        for (int i = 0; i < NXG; ++i) nx[i] = 0;
#pragma unroll
        for (int i = 0; i < NBG; ++i) nb[i] = 0;
#pragma unroll
        for (int sl = 0; sl < kRC; ++sl) {
            const unsigned long long m = __ballot(pos == sl);
            const int nd = m ? (int)__ffsll((long long)m) - 1 : 0;
#pragma unroll
            for (int i = 0; i < NXG; ++i) nx[i] = ((ln + 64 * i) / PX == sl) ? nd : nx[i];
#pragma unroll
            for (int i = 0; i < NBG; ++i) nb[i] = ((ln + 64 * i) / PB == sl) ? nd : nb[i];
        }
        uint4 gx[NXG], gb[NBG];
#pragma unroll
        for (int i = 0; i < NXG; ++i)
            gx[i] = *reinterpret_cast<const uint4 *>(xb + (uint32_t)(nx[i] * (int)R.x_sn + ((ln + 64 * i) % PX) * 8) * 2u);
#pragma unroll
        for (int i = 0; i < NBG; ++i)
            gb[i] = *reinterpret_cast<const uint4 *>(Bb + (uint32_t)(nb[i] * (int)R.b_sn + ((ln + 64 * i) % PB) * 8) * 2u);
        if constexpr (WPE < 4) {
#pragma unroll
            for (int i = 0; i < NXG; ++i) gxw[i] = gx[i];
#pragma unroll
            for (int i = 0; i < NBG; ++i) gbw[i] = gb[i];
            wpos = pos; wcf = cf; wlen = len; wdec = dc;
        } else {
            tw[0] = __uint_as_float(gx[0].x); tw[1] = __uint_as_float(gx[0].y);
            tw[2] = __uint_as_float(gx[0].z); tw[3] = __uint_as_float(gx[0].w);
#pragma unroll
            for (int i = 0; i < NBG; ++i) {
                tw[4 + 4 * i] = __uint_as_float(gb[i].x); tw[5 + 4 * i] = __uint_as_float(gb[i].y);
                tw[6 + 4 * i] = __uint_as_float(gb[i].z); tw[7 + 4 * i] = __uint_as_float(gb[i].w);
            }
            tw[12] = __int_as_float(pos); tw[13] = cf; tw[14] = __int_as_float(len); tw[15] = dc;
        }
    };
    auto write_R = [&](const floatx16 &tw, char *rbuf) {
        const int ln = opaque(lane);
        uint4 gx[NXG], gb[NBG];
        int pos, len;
        float cf, dc;
        if constexpr (WPE < 4) {
#pragma unroll
            for (int i = 0; i < NXG; ++i) gx[i] = gxw[i];
#pragma unroll
            for (int i = 0; i < NBG; ++i) gb[i] = gbw[i];
            pos = wpos; cf = wcf; len = wlen; dc = wdec;
        } else {
            gx[0] = make_uint4(__float_as_uint(tw[0]), __float_as_uint(tw[1]), __float_as_uint(tw[2]), __float_as_uint(tw[3]));
#pragma unroll
            for (int i = 0; i < NBG; ++i)
                gb[i] = make_uint4(__float_as_uint(tw[4 + 4 * i]), __float_as_uint(tw[5 + 4 * i]),
                                   __float_as_uint(tw[6 + 4 * i]), __float_as_uint(tw[7 + 4 * i]));
            pos = __float_as_int(tw[12]); cf = tw[13]; len = __float_as_int(tw[14]); dc = tw[15];
        }
#pragma unroll
        for (int i = 0; i < NXG; ++i) {
            const int idx = ln + 64 * i;
            if (idx < kRC * PX) *reinterpret_cast<uint4 *>(rbuf + ((idx / PX) * P + (idx % PX) * 8) * 2) = gx[i];
        }
#pragma unroll
        for (int i = 0; i < NBG; ++i) {
            const int idx = ln + 64 * i;
            if (idx < kRC * PB)
                *reinterpret_cast<uint4 *>(rbuf + (kRC * P + (idx / PB) * S + (idx % PB) * 8) * 2) = gb[i];
        }
        if (pos >= 0) {
            sRnode[pos] = (unsigned char)ln;
            sRcoef[pos] = cf;
        }
        if (ln == 0) {
            *sRlen = len;
            *sRdec = dc;
        }
    };
    // LDS rows of the replayed path: behind the y staging area of the idle B tile, or their own array
    char *const rrows = L::rows_in_b ? reinterpret_cast<char *>(sB) + kYStage : reinterpret_cast<char *>(sRrows);

    if (nU <= 0) return;
    // (b, h) of the current unit and of the next three.  The loop starts one unit early (k = -1):
    // that pass has no unit to compute and only runs the staging half, which brings unit 0 into
    // LDS and issues the loads of units 1 and 2 -- the same code as in the steady state, so the
    // instruction cache sees each part of the loop body once.
    int cb = ub0, ch = uh0, b1 = ub0, h1 = uh0;
    int b2 = b1, h2 = h1;
    step(b2, h2);
    int b3 = b2, h3 = h2;
    step(b3, h3);
    // One accumulator set serves both roles: the Y waves' Yt tiles of the current unit, or
    // (acc[0]) the G waves' Gt tile of the current (sequence, group), kept across its heads.
    floatx16 acc[YQ];

    // the first loads of every role, before anything is waited for.  With the replay the first
    // state tile is the exception (kLateH0): it is asked for once the tree wave has requested the
    // path rows of unit 0.  The replay of unit 0 is two dependent round trips (the previous tree's
    // parents and step sizes, then the rows of the path), and behind 16 KB of state per thread
    // group and workgroup each of them takes several times as long, while the first scan waits for
    // them all the same.
    constexpr bool kLateH0 = RP;
    if constexpr (kLateH0) {
#pragma unroll
        for (int q = 0; q < YQ; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
        if (!isY) {
            load_X(b1, h1);
            if (wave == kTreeWave) {
                load_T(b1, h1);
                load_R(b1, h1);
            }
        }
        if (wave == kTreeWave) path_R(acc[0], b1, h1);
        // the state of unit 1 (carried by the G threads) goes out now, while nothing else uses the
        // memory system; the tree wave asks for its share after its path rows
        if (!isY && h0 && nU > 1) load_H(b2, h2);
        __syncthreads();                                      // the path rows of unit 0 are requested
        if (isY) {
            if (h0) load_H(b1, h1);
        }
    } else {
        if (isY) {
            if (h0) load_H(b1, h1);
        } else {
            load_X(b1, h1);
            if (wave == kTreeWave) load_T(b1, h1);
        }
#pragma unroll
        for (int q = 0; q < YQ; ++q)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[q][e] = 0.f;
    }

    for (int k = -1; k < nU; ++k) {
        const bool live = k >= 0;                             // false in the staging-only first pass
        int bad = 0;
        float D_h = 0.f;
        if (live) {
            __syncthreads();                                  // barrier 1: unit k is staged
            bad = *sBad;
            D_h = *sDh;
            if (status && ch == 0 && tid == 0) status[cb] = bad;
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
                const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, it = RP ? (opaque(wave) & 1) : it0, il = it * 32 + l32;   // re-derived per phase
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
        } else if (wave != kTreeWave && !bad) {
            // ---- phase 2: Gt = B C^T (only when the C/B tiles are new), mask and decay -> M ----------
            const int jt = ((RP ? opaque(wave) : wave) - 4) >> 1;   // (see it0)
            const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, it = RP ? (opaque(wave) & 1) : it0, il = it * 32 + l32;   // re-derived per phase
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
        } else if (RP && wave == kTreeWave) {
            // ---- replay: path of unit k+1 on the previous tree and the loads of its x / B rows, in the
            //      half in which this wave has nothing else to do; they are written to LDS at the start
            //      of the staging half.  Then the parent / dt loads for the path of unit k+2.
            if (k + 1 < nU) {
                path_R(acc[0], b1, h1);
                if (k + 2 < nU) load_R(b2, h2);
            }
        }
        if (live) __syncthreads();                            // barrier 2: M is ready; h0b, C and the tree arrays are dead

        const bool more = k + 1 < nU, more2 = k + 2 < nU, more3 = k + 3 < nU;
        const bool y_stages = (k & 1) != 0;    // unit k+1 is even: its h0 sits in the Y threads
        // new C / B tiles for unit k+1 overwrite the B tile's LDS, which this half uses as scratch
        // (y staging, replayed path rows): they wait for one more barrier (a).  Not in the first
        // pass, which has no such use and wants the tiles early.
        const bool fresh_next = more && fresh_at(k + 1, h1);
        const bool late_tiles = live && fresh_next;
        // replayed path rows of unit k+1: in the first pass the M tile's LDS (the B tile is being
        // written), later the B tile's
        [[maybe_unused]] char *rbuf = (L::rows_in_b && !live) ? reinterpret_cast<char *>(sM) : rrows;
        if (isY) {
            // ---- phase 3: Yt += Xt M^T over j <= i only (nodes i < 32 have no ancestor j >= 32:
            //      that quadrant of M is never written or read); y = Yt + D x ---------------------------
            bf16x4 yreg[YQ][4];
            const int lnp = opaque(lane), l32 = lnp & 31, lh = lnp >> 5, it = RP ? (opaque(wave) & 1) : it0, il = it * 32 + l32;   // re-derived per phase
#pragma unroll
            for (int q = 0; q < YQ; ++q) {
                if (!live) break;
                const int pt = ((RP ? opaque(wave) : wave) + 4 * q) >> 1;   // (see it0)
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
            // first pass: the Y threads have nothing to scan and stage the first C / B tiles (later
            // tiles come from the G threads, after barrier (a))
            if (!live && fresh_next) restage_CB(b1, h1);
            if (RP && more) __syncthreads();                  // barrier (c): path rows of unit k+1 are in LDS
            // next unit's state tile (its loads have been in flight for a whole unit period)
            if (more) {
                if (h0) {
                    if (y_stages) stage_H(rbuf, b1, h1);
                } else if (rt == 0) {
                    *sDh = D ? D[h1] : 0.f;
                }
            }
            // y leaves as 64-byte row pieces: the accumulators give a lane 4 consecutive p of one
            // node, which as direct stores would be 16-byte pieces of 32 different lines per
            // instruction.  Each wave therefore turns its 32x32 tile around in a private 2 KB of LDS
            // (a wave's LDS operations complete in order: no barrier) and stores 16 bytes per lane,
            // four lanes to a row.  The LDS used is the B tile's, which is idle in this half.
            // The stores go out after the wait for the h0 loads above and are long complete at
            // the next such wait: on gfx9 loads and stores share one counter and complete out of
            // order with respect to each other, so a store in flight would turn that wait into a
            // wait for everything.
            if (live) {
                char *yb = reinterpret_cast<char *>(y + (size_t)cb * n * H * P + (size_t)ch * P);
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
                        const int node = (RP ? (opaque(wave) & 1) : it0) * 32 + row;
                        if (node < n)
                            store_through16(yb + (uint32_t)(node * H * P + pt * 32 + rc * 8) * 2u, v);
                    }
                }
            }
            // h0 of unit k+3 after staging unit k+1.  Unit 2 is the exception: asked for in the
            // first pass it would sit in the memory queues in front of the small x / parent / dt
            // loads of units 1 and 2 and make the last scan wait for them; asked for one pass
            // later, the state of the last unit of a short run is the last thing to arrive.
            if (h0 && more3 && y_stages && live) load_H(b3, h3);
            if (h0 && more2 && k == 0) load_H(b2, h2);
            if (late_tiles) __syncthreads();                  // barrier (a): scratch use of the B tile is over
        } else if (more) {
            if constexpr (RP) {
                if (wave == kTreeWave) {
                    if (!live) {                           // unit 0: path and rows within this pass
                        if constexpr (!kLateH0) path_R(acc[0], b1, h1);   // (else: done before the loop)
                        if (more2) load_R(b2, h2);
                    }
                    write_R(acc[0], rbuf);                 // (waits for the row loads issued in the scan half)
                }
                __syncthreads();                           // barrier (c)
            }
            if (wave == kTreeWave) {
                stage_T(h1);
            }
            stage_X((k + 1) & 1);                          // the other X^T tile: unit k still reads its own
            // the registers just staged are free: x and parent / dt of unit k+2 go out at once (a
            // pass is short when HBM is idle, and they are needed at this point of the next one)
            if (more2) {
                load_X(b2, h2);
                if (wave == kTreeWave) load_T(b2, h2);
            }
            if (h0 && !y_stages) {
                stage_H(rbuf, b1, h1);
                if (more3) load_H(b3, h3);
            }
            if (!kLateH0 && more2 && !live && h0) load_H(b2, h2);      // unit 1: the first odd unit (kLateH0: before the loop)
            if (late_tiles) {
                __syncthreads();                           // barrier (a)
                restage_CB(b1, h1);
            }
        }
        cb = b1; ch = h1;
        b1 = b2; h1 = h2;
        b2 = b3; h2 = h3;
        step(b3, h3);
    }
}

template <int P, int S, bool RP>
hipError_t launch64_ps(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                       const void *Bm, const void *Cm, const float *D, const void *h0, void *y,
                       int32_t *status, const ReplayArgs &R, hipStream_t st) {
    constexpr size_t lds = RP ? Lds64<P, S>::total_replay : Lds64<P, S>::total;   // static LDS (upper bound)
    constexpr int WPE = (2 * (lds + 64) <= 160 * 1024) ? 4 : 2;
    const int n_units = d.batch * d.nheads;
    const int per_cu = (int)((160 * 1024) / (lds + 64));      // resident workgroups per CU by LDS
    int grid = (n_units + 7) / 8 * 8;
    const int cap = 256 * (per_cu < 1 ? 1 : (per_cu > 2 ? 2 : per_cu));
    if (grid > cap) grid = cap;
    // (the in-kernel softplus is a variant of its own: compiled into the common one, even unused, it costs time)
#define STREE_LAUNCH64(SPL, HT)                                                                                     \
    hipLaunchKernelGGL((tree_ssd_mfma64_kernel<P, S, WPE, RP, SPL, HT>), dim3(grid), dim3(kT64), 0, st, parent,     \
                       d.nnodes, d.batch, d.nheads, d.ngroups, (const bf16_t *)x, (long)d.x_stride_n, dt,           \
                       step_bias(d), A, (const bf16_t *)Bm, (long)d.b_stride_n, (const bf16_t *)Cm,                 \
                       (long)d.c_stride_n, D, (const HT *)h0, (bf16_t *)y, status, R)
    const bool hb = d.state_dtype == STREE_BF16;
    if (step_bias(d)) {
        if (hb) STREE_LAUNCH64(true, bf16_t);
        else STREE_LAUNCH64(true, float);
    } else {
        if (hb) STREE_LAUNCH64(false, bf16_t);
        else STREE_LAUNCH64(false, float);
    }
#undef STREE_LAUNCH64
    return hipGetLastError();
}

template <bool RP>
hipError_t launch64(const stree_dims &d, const int32_t *parent, const void *x, const float *dt, const float *A,
                    const void *Bm, const void *Cm, const float *D, const void *h0, void *y, int32_t *status,
                    const ReplayArgs &R, hipStream_t st) {
    const int P = d.headdim, S = d.dstate;
    if (P == 64 && S == 128) return launch64_ps<64, 128, RP>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, R, st);
    if (P == 64 && S == 64) return launch64_ps<64, 64, RP>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, R, st);
    if (P == 64 && S == 256) return launch64_ps<64, 256, RP>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, R, st);
    if (P == 128 && S == 128) return launch64_ps<128, 128, RP>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, R, st);
    return hipErrorInvalidValue;
}

}  // namespace

bool tree_ssd_mfma64_supported(const stree_dims &d) {
    if (d.nnodes > kB64) return false;
    const int P = d.headdim, S = d.dstate;
    return (P == 64 && (S == 128 || S == 64 || S == 256)) || (P == 128 && S == 128);
}

bool tree_ssd_replay_fused_supported(const stree_dims &d, const stree_dims &dp, const void *px, const void *pB,
                                     const void *x, const void *Bm, const void *Cm, const void *y, const void *h0,
                                     const void *h_out) {
    if (d.io_dtype != STREE_BF16 || !tree_ssd_mfma64_supported(d) || dp.nnodes > kB64) return false;
    if ((d.x_stride_n | d.b_stride_n | d.c_stride_n | dp.x_stride_n | dp.b_stride_n) % 8 != 0) return false;
    const uintptr_t bits = (uintptr_t)x | (uintptr_t)Bm | (uintptr_t)Cm | (uintptr_t)y | (uintptr_t)px | (uintptr_t)pB |
                           (uintptr_t)h0 | (uintptr_t)h_out;   // (the state is read and written 16 bytes at a time)
    return bits % 16 == 0;
}

hipError_t launch_tree_ssd_replay_fused(const stree_dims &d, const stree_dims &dp, const int32_t *pparent,
                                        const int32_t *paccepted, const void *px, const float *pdt, const void *pB,
                                        const int32_t *parent, const void *x, const float *dt, const float *A,
                                        const void *Bm, const void *Cm, const float *D, const void *h0,
                                        void *h_out, void *y, int32_t *status, int32_t *rstatus, hipStream_t st) {
    const ReplayArgs R = {pparent, paccepted, (const bf16_t *)px, (const bf16_t *)pB, pdt,
                          (long)dp.x_stride_n, (long)dp.b_stride_n, dp.nnodes, h_out, rstatus};
    return launch64<true>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, R, st);
}

hipError_t launch_tree_ssd_mfma64(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D,
                                  const void *h0, void *y, int32_t *status, hipStream_t st) {
    return launch64<false>(d, parent, x, dt, A, Bm, Cm, D, h0, y, status, ReplayArgs{}, st);
}

}  // namespace stree
