// stree_tree_conv: depthwise causal conv1d along each node's ancestor chain.
//
// A workgroup owns 8 channel vectors (16 bytes each) of one sequence and brings every row of
// that channel block into LDS once: the N pre-conv rows of the tree and, behind them, the W-1
// rows "above the root".  Each thread then walks the ancestor chains of its nodes in LDS, so a
// pre-conv element is fetched from memory exactly once however many descendants read it.
//
// The rows above the root are the conv state.  In the replay variant they are the conv state
// AFTER the previous iteration's accepted path,
//   last W-1 rows of [conv_state ; prev_xbc_pre[path(k)]],
// taken on the fly from the previous tree's rows (and written out as the new conv state), so
// that the conv-tail update of the state commit needs no launch of its own.
#include "common.hpp"
#include "launch.hpp"

namespace stree {

template <typename T>
struct Vec16;
template <>
struct Vec16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4 &v, float (&o)[4]) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&o)[4]) {
        return make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
    }
};
template <>
struct Vec16<bf16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4 &v, float (&o)[8]) {
        o[0] = bf16_lo(v.x); o[1] = bf16_hi(v.x); o[2] = bf16_lo(v.y); o[3] = bf16_hi(v.y);
        o[4] = bf16_lo(v.z); o[5] = bf16_hi(v.z); o[6] = bf16_lo(v.w); o[7] = bf16_hi(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&o)[8]) {
        bf16x8 v;
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = (bf16_t)o[e];
        return __builtin_bit_cast(uint4, v);
    }
};

constexpr int kConvVecs = 8;                        // channel vectors per workgroup
constexpr int kConvLanes = kThreads / kConvVecs;    // node lanes: thread (g, v) does nodes g, g+16, ...

struct ConvReplay {          // previous tree (replay variant); parent == nullptr: plain conv
    const int32_t *parent, *accepted;
    const void *xbc_pre;     // [B, pn, Cc]
    void *conv_state_out;    // [B, W-1, Cc]
    int32_t *status;         // [B] or null
    int pn;
};

// grid: B * ceil(Cc / (8 vectors)); dynamic LDS: (N + W - 1) rows of 128 bytes
template <typename T, int W, bool RP>
__global__ __launch_bounds__(kThreads) void tree_conv_kernel(
    const int32_t *__restrict__ parent, int n, int Cc, int silu, const T *__restrict__ xbc_pre,
    const T *__restrict__ conv_state, const T *__restrict__ w, const T *__restrict__ bias, T *__restrict__ out,
    int32_t *__restrict__ status, ConvReplay R) {
    constexpr int VEC = Vec16<T>::N;
    extern __shared__ __align__(16) uint4 rows[];      // [n + W - 1][kConvVecs]; row n + m - 1 = m rows above the root
    __shared__ int par[kMaxNodes];
    __shared__ __align__(16) uint4 wsh[(4 + 1) * kConvVecs];   // weight pieces 0 .. W-1 and the bias of each channel vector
    __shared__ int bad_w[kThreads / 64], pbad_w[kThreads / 64];   // first bad node + 1 per wave, or INT_MAX
    const int tid = threadIdx.x, v = tid % kConvVecs, g = tid / kConvVecs;
    const int cblocks = (Cc / VEC + kConvVecs - 1) / kConvVecs;
    const int cblk = blockIdx.x % cblocks, b = blockIdx.x / cblocks;
    const int c0 = (cblk * kConvVecs + v) * VEC;
    const bool has_c = c0 < Cc;

    // Every global load of the kernel is issued up front, before anything is waited for: both trees'
    // parents, the tree's rows, weights and bias, the old conv state rows and (replay) the path rows
    // -- and no more requests than can be used: the kernel's phases run in step across the chip, and
    // every request a wave issues, also one whose lanes all read nothing, showed in its duration.
    // They are raw buffer loads: a uniform descriptor of the array (this sequence's part of it) plus a
    // 32-bit byte offset per lane, and a lane that has nothing to fetch -- a row past the tree, a
    // channel past the last one, a node lane without a state row -- passes an offset past the end and
    // reads zeros: no branch around any load, so the compiler knows how many requests are behind the
    // one it waits for and a wait for an early one (the previous tree's parents, below) is not a
    // wait for them all.
    const uint4 zero4 = make_uint4(0u, 0u, 0u, 0u);
    constexpr uint32_t kNone = 0xffffffffu, kE = (uint32_t)sizeof(T);
    auto ld16 = [&](__amdgpu_buffer_rsrc_t rsrc, uint32_t off, bool on) { return buffer_load16(rsrc, on ? off : kNone); };
    const __amdgpu_buffer_rsrc_t r_pre = make_buffer(xbc_pre + (size_t)b * n * Cc, (size_t)n * Cc * kE);
    const __amdgpu_buffer_rsrc_t r_w = make_buffer(w, (size_t)Cc * W * kE);
    const __amdgpu_buffer_rsrc_t r_b = make_buffer(bias, bias ? (size_t)Cc * kE : 0);
    const __amdgpu_buffer_rsrc_t r_cs = make_buffer(conv_state + (size_t)b * (W - 1) * Cc, (size_t)(W - 1) * Cc * kE);
    auto ld_row = [&](int i) { return ld16(r_pre, ((uint32_t)i * (uint32_t)Cc + (uint32_t)c0) * kE, has_c); };
    // replay, previous trees of at most 64 nodes: every wave holds that tree's parents, one per lane
    // (requested first: the walk below needs them before anything else is needed)
    int pparent_lane = -1, pparent_mine = -1;
    if constexpr (RP)
        pparent_lane = buffer_load4(make_buffer(R.parent + (size_t)b * R.pn, (size_t)R.pn * 4), (uint32_t)(tid & 63) * 4u);
    // both trees' parents, one entry per thread (the envelope has at most kThreads nodes): requested
    // with everything else, so that validating them costs no round trip of its own later
    static_assert(kMaxNodes <= kThreads, "one parent entry per thread");
    const int parent_mine = buffer_load4(make_buffer(parent + (size_t)b * n, (size_t)n * 4), (uint32_t)tid * 4u);
    if constexpr (RP) {
        if (R.pn > 64)      // (smaller previous trees are validated on the per-wave copy above)
            pparent_mine = buffer_load4(make_buffer(R.parent + (size_t)b * R.pn, (size_t)R.pn * 4), (uint32_t)tid * 4u);
    }
    // the first four rows of this thread (all of them for trees of up to 4 * kConvLanes nodes)
    const uint4 t0 = ld_row(g), t1 = ld_row(g + kConvLanes);
    uint4 t2 = zero4, t3 = zero4;
    if (n > 2 * kConvLanes) {                 // (uniform: a request that reads nothing still costs its issue)
        t2 = ld_row(g + 2 * kConvLanes);
        t3 = ld_row(g + 3 * kConvLanes);
    }
    // weights and bias of this thread's channel vector: W + 1 sixteen-byte pieces that all node lanes
    // need -- node lane q fetches piece q (lane W the bias) in ONE request and they are handed out
    // through LDS behind the barrier below, instead of W + 1 requests by every lane
    const uint4 wpc = ld16(r_w, (uint32_t)(c0 * W + min(g, W - 1) * VEC) * kE, has_c && g < W);
    const uint4 bpc = ld16(r_b, (uint32_t)c0 * kE, has_c && g == W);
    // rows above the root, m = 1 (newest) .. W-1, one per node lane g = m - 1
    const int m = g + 1;
    const bool is_state_lane = g < W - 1 && has_c;
    // lane m's candidates (no arrays, no select between loaded values: a lane that does not need a
    // candidate reads zeros, and the two it can need after a valid walk are OR-ed):
    //   keep_row  conv_state row W-1-m: nothing accepted, or the previous tree is invalid
    //   old_row   conv_state row W-1-(m-L), L = nodes found on the walk, if the path is shorter than m
    //   prow      the pre-conv row of the (m-1)-th node of the walk otherwise
    // (each is requested only where the walk's outcome -- uniform -- can make some lane use it: a
    // request that reads nothing still costs its issue in every wave)
    const uint32_t keep_off = (uint32_t)((W - 1 - min(m, W - 1)) * Cc + c0) * kE;
    uint4 keep_row = zero4, old_row = zero4, prow = zero4;
    if constexpr (!RP) keep_row = ld16(r_cs, keep_off, is_state_lane);
    // Replay: walk up from the accepted node of the previous tree (uniform; each step checked on its
    // own so that a corrupt parent array cannot send the walk out of bounds): through the parents
    // held in the lanes where that tree has at most 64 nodes -- one round trip for the whole walk --
    // else by scalar loads, one dependent round trip per step.
    // anc_ok = nodes found on the walk, at most W-1; lane m needs the (m-1)-th of them.
    int k_prev = -1, anc_ok = 0;
    bool k_bad = false;
    if constexpr (RP) {
        k_prev = R.accepted[b];
        k_bad = k_prev < -1 || k_prev >= R.pn;
        int cur = k_bad ? -1 : k_prev, mine = -1;
#pragma unroll
        for (int sstep = 0; sstep < W - 1; ++sstep) {
            if (cur >= 0) {
                ++anc_ok;
                if (sstep == m - 1) mine = cur;
                const int pz = R.pn <= 64 ? __builtin_amdgcn_readlane(pparent_lane, cur)
                                          : R.parent[(size_t)b * R.pn + cur];
                cur = (cur > 0 && pz >= 0 && pz < cur) ? pz : -1;
            }
        }
        const __amdgpu_buffer_rsrc_t r_pp =
            make_buffer(reinterpret_cast<const T *>(R.xbc_pre) + (size_t)b * R.pn * Cc, (size_t)R.pn * Cc * kE);
        if (anc_ok > 0)
            prow = ld16(r_pp, ((uint32_t)max(mine, 0) * (uint32_t)Cc + (uint32_t)c0) * kE, is_state_lane && mine >= 0);
        if (anc_ok > 0 && anc_ok < W - 1)
            old_row = ld16(r_cs, (uint32_t)(max((W - 1) - (m - anc_ok), 0) * Cc + c0) * kE, is_state_lane && m > anc_ok);
        if (anc_ok == 0) keep_row = ld16(r_cs, keep_off, is_state_lane);
    }
    // Tree validity: every thread checks its own node, a wave reports its first bad one (no LDS
    // atomics, nothing to initialise: no barrier in front of this).  A previous tree of at most 64
    // nodes is also checked by every wave on its own copy, so that the rows above the root can be
    // placed before the one barrier below instead of behind a second one.
    auto node_ok = [](int node, int pz) { return (node == 0) ? (pz == -1) : (pz >= 0 && pz < node); };
    auto first_bad = [&](bool ok, int base) {       // (uniform per wave) base + lane + 1 of the first bad lane
        const unsigned long long bm = __ballot(!ok);
        return bm ? base + (int)__ffsll((long long)bm) : 0x7fffffff;
    };
    {
        const bool ok = tid >= n || node_ok(tid, parent_mine);
        const int fb = first_bad(ok, tid & ~63);
        if ((tid & 63) == 0) bad_w[tid >> 6] = fb;
        if (tid < n) par[tid] = ok ? parent_mine : -1;
    }
    int pbad_own = 0;
    const bool early_state = !RP;
    if constexpr (RP) {
        if (R.pn <= 64) {
            const int ln = tid & 63, f = first_bad(ln >= R.pn || node_ok(ln, pparent_lane), 0);
            pbad_own = f == 0x7fffffff ? 0 : f;
        } else {
            const int fb = first_bad(tid >= R.pn || node_ok(tid, pparent_mine), tid & ~63);
            if ((tid & 63) == 0) pbad_w[tid >> 6] = fb;
        }
    }
    if (g <= W) wsh[g * kConvVecs + v] = make_uint4(wpc.x | bpc.x, wpc.y | bpc.y, wpc.z | bpc.z, wpc.w | bpc.w);
    if (g < n) rows[g * kConvVecs + v] = t0;
    if (g + kConvLanes < n) rows[(g + kConvLanes) * kConvVecs + v] = t1;
    if (g + 2 * kConvLanes < n) rows[(g + 2 * kConvLanes) * kConvVecs + v] = t2;
    if (g + 3 * kConvLanes < n) rows[(g + 3 * kConvLanes) * kConvVecs + v] = t3;
    for (int i0 = g + 4 * kConvLanes; i0 < n; i0 += 4 * kConvLanes) {   // larger trees: four rows at a time
        const uint4 u0 = ld_row(i0), u1 = ld_row(i0 + kConvLanes), u2 = ld_row(i0 + 2 * kConvLanes),
                    u3 = ld_row(i0 + 3 * kConvLanes);
        rows[i0 * kConvVecs + v] = u0;
        if (i0 + kConvLanes < n) rows[(i0 + kConvLanes) * kConvVecs + v] = u1;
        if (i0 + 2 * kConvLanes < n) rows[(i0 + 2 * kConvLanes) * kConvVecs + v] = u2;
        if (i0 + 3 * kConvLanes < n) rows[(i0 + 3 * kConvLanes) * kConvVecs + v] = u3;
    }
    // the m-th newest row of [conv_state ; path rows]: a path row if the path has at least m nodes,
    // else the (m - L)-th newest old row, L = nodes on the path (0: nothing accepted, or the previous
    // tree / the accepted index is invalid)
    auto place_state_rows = [&](int pbad) {
        if (g >= W - 1) return;
        if constexpr (RP) {
            if (R.status && cblk == 0 && tid == 0) R.status[b] = pbad ? pbad : (k_bad ? -1 : 0);
        }
        uint4 r = make_uint4(keep_row.x | old_row.x | prow.x, keep_row.y | old_row.y | prow.y,
                             keep_row.z | old_row.z | prow.z, keep_row.w | old_row.w | prow.w);   // (one of them was read)
        if constexpr (RP) {
            // an invalid previous tree accepts nothing after all: the old row, fetched only now
            if (pbad && anc_ok > 0 && has_c)
                r = *reinterpret_cast<const uint4 *>(conv_state + ((size_t)b * (W - 1) + (W - 1 - m)) * Cc + c0);
        }
        rows[(n + m - 1) * kConvVecs + v] = r;
        if constexpr (RP) {   // the new conv state, oldest first: row W-1-m
            if (has_c)
                store_written_through16(reinterpret_cast<T *>(R.conv_state_out) +
                                            ((size_t)b * (W - 1) + (W - 1 - m)) * Cc + c0, r);
        }
    };
    if (early_state) place_state_rows(pbad_own);
    __syncthreads();
    int bad = 0x7fffffff;
#pragma unroll
    for (int q = 0; q < kThreads / 64; ++q) bad = min(bad, bad_w[q]);
    bad = bad == 0x7fffffff ? 0 : bad;
    if (status && cblk == 0 && tid == 0) status[b] = bad;
    if constexpr (RP) {
        if (!early_state) {
            int pbad = pbad_own;
            if (R.pn > 64) {
                pbad = 0x7fffffff;
#pragma unroll
                for (int q = 0; q < kThreads / 64; ++q) pbad = min(pbad, pbad_w[q]);
                pbad = pbad == 0x7fffffff ? 0 : pbad;
            }
            place_state_rows(pbad);
            __syncthreads();
        }
    }
    if (!has_c) return;
    if (bad) {
        for (int i = g; i < n; i += kConvLanes)
            *reinterpret_cast<uint4 *>(out + ((size_t)b * n + i) * Cc + c0) = make_uint4(0u, 0u, 0u, 0u);
        return;
    }
    uint4 wq[W];
#pragma unroll
    for (int q = 0; q < W; ++q) wq[q] = wsh[q * kConvVecs + v];
    const uint4 bq = wsh[W * kConvVecs + v];
    float wv[W][VEC];  // flat [e*W + j] = w[c0+e][j]
#pragma unroll
    for (int q = 0; q < W; ++q) Vec16<T>::unpack(wq[q], wv[q]);
    float bv[VEC];
    Vec16<T>::unpack(bq, bv);
    for (int i = g; i < n; i += kConvLanes) {
        float acc[VEC];
#pragma unroll
        for (int e = 0; e < VEC; ++e) acc[e] = bv[e];
        int node = i, above = 0;
        uint4 rk[W];                    // row of the k-th ancestor, or of the rows over the root
#pragma unroll
        for (int k = 0; k < W; ++k) {
            int row;
            if (node >= 0) {
                row = node;
                node = par[node];
            } else {
                ++above;
                row = n + above - 1;
            }
            rk[k] = rows[row * kConvVecs + v];
        }
        if constexpr (W == 4 && VEC == 8) {
            const uint32_t ww[16] = {wq[0].x, wq[0].y, wq[0].z, wq[0].w, wq[1].x, wq[1].y, wq[1].z, wq[1].w,
                                     wq[2].x, wq[2].y, wq[2].z, wq[2].w, wq[3].x, wq[3].y, wq[3].z, wq[3].w};
            conv4_bf16_dot(acc, rk[0], rk[1], rk[2], rk[3], ww);
        } else {
#pragma unroll
            for (int k = 0; k < W; ++k) {
                float r[VEC];
                Vec16<T>::unpack(rk[k], r);
#pragma unroll
                for (int e = 0; e < VEC; ++e) acc[e] = fmaf((&wv[0][0])[e * W + (W - 1 - k)], r[e], acc[e]);
            }
        }
        if (silu) {
#pragma unroll
            for (int e = 0; e < VEC; ++e)   // z * sigmoid(z); hardware reciprocal (1 ulp) instead of a division
                acc[e] = acc[e] * __builtin_amdgcn_rcpf(1.f + __expf(-acc[e]));
        }
        store_written_through16(out + ((size_t)b * n + i) * Cc + c0, Vec16<T>::pack(acc));
    }
}

template <typename T, bool RP>
static hipError_t launch_conv_t(const stree_dims &d, const int32_t *parent, const void *xbc_pre,
                                const void *conv_state, const void *conv_w, const void *conv_b,
                                void *xbc_out, int32_t *status, const ConvReplay &R, hipStream_t st) {
    constexpr int VEC = Vec16<T>::N;
    const int Cc = d.nheads * d.headdim + 2 * d.ngroups * d.dstate;
    const int cblocks = (Cc / VEC + kConvVecs - 1) / kConvVecs;
    const dim3 grid(cblocks * d.batch);
    // (at most (256 + 3) rows of 128 bytes: inside the default limit on dynamic LDS)
    const size_t lds = (size_t)(d.nnodes + d.conv_width - 1) * kConvVecs * sizeof(uint4);
    static_assert((kMaxNodes + 3) * kConvVecs * sizeof(uint4) <= 48 * 1024, "the conv rows outgrow the default LDS limit");
    const int silu = (d.flags & STREE_FLAG_CONV_SILU) ? 1 : 0;
#define STREE_CONV_CASE(WW)                                                                                   \
    case WW:                                                                                                  \
        hipLaunchKernelGGL((tree_conv_kernel<T, WW, RP>), grid, dim3(kThreads), lds, st, parent, d.nnodes, Cc, \
                           silu, (const T *)xbc_pre, (const T *)conv_state, (const T *)conv_w,                \
                           (const T *)conv_b, (T *)xbc_out, status, R);                                       \
        break;
    switch (d.conv_width) {
        STREE_CONV_CASE(2)
        STREE_CONV_CASE(3)
        STREE_CONV_CASE(4)
        default: return hipErrorInvalidValue;
    }
#undef STREE_CONV_CASE
    return hipGetLastError();
}

hipError_t launch_tree_conv(const stree_dims &d, const int32_t *parent, const void *xbc_pre,
                            const void *conv_state, const void *conv_w, const void *conv_b, void *xbc_out,
                            int32_t *status, hipStream_t st) {
    const ConvReplay none = {};
    if (d.io_dtype == STREE_BF16)
        return launch_conv_t<bf16_t, false>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, none, st);
    return launch_conv_t<float, false>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, none, st);
}

hipError_t launch_tree_conv_replay(const stree_dims &d, int prev_nnodes, const int32_t *prev_parent,
                                   const int32_t *prev_accepted, const void *prev_xbc_pre, const int32_t *parent,
                                   const void *xbc_pre, const void *conv_state, const void *conv_w,
                                   const void *conv_b, void *xbc_out, void *conv_state_out, int32_t *status,
                                   int32_t *replay_status, hipStream_t st) {
    const ConvReplay R = {prev_parent, prev_accepted, prev_xbc_pre, conv_state_out, replay_status, prev_nnodes};
    if (d.io_dtype == STREE_BF16)
        return launch_conv_t<bf16_t, true>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, R, st);
    return launch_conv_t<float, true>(d, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out, status, R, st);
}

}  // namespace stree
