// stree_commit_state: state of the accepted node, recomputed from the cached
// activations of the verified tree (activation replay), plus the conv tail.
//
//   h_out = exp(s_k) h0 + sum_{j on path(k)} dt_j exp(s_k - s_j) x_j (outer) B_j
//
// Streaming kernel: the P x S fp32 state is read once and written once; the
// rank-(depth+1) update comes from a handful of x / B rows staged in LDS.
#include "common.hpp"
#include "launch.hpp"

namespace stree {

constexpr int kQ = 8;               // state rows per thread (one float4 of each)
constexpr int kPathChunk = 16;     // path nodes staged in LDS at a time

// conv tail: out row r (oldest first) = pre-conv row of the (W-2-r)-th ancestor of k, or the old
// state row once above the root.  One workgroup covers VEC*256 channels of one sequence.
// `status` (null unless the call has no state part, whose workgroups report otherwise): the first
// channel block of a sequence writes 0, the first bad node + 1, or -1 for an accepted index
// outside [-1, n).
template <typename T, int VEC>
__device__ __forceinline__ void conv_tail(int b, int cblk, const int32_t *__restrict__ parent,
                                          const int32_t *__restrict__ accepted, int n, int Cc, int W,
                                          const T *__restrict__ xbc_pre, const T *conv_state, T *conv_state_out,
                                          int32_t *__restrict__ status) {
    __shared__ int par[kMaxNodes];
    __shared__ int first_bad;
    const int tid = threadIdx.x;
    if (tid == 0) first_bad = 0x7fffffff;
    __syncthreads();
    int ok = 1;
    if (tid < n) {
        const int p = parent[(size_t)b * n + tid];
        ok = (tid == 0) ? (p == -1) : (p >= 0 && p < tid);
        par[tid] = ok ? p : -1;
        if (!ok) atomicMin(&first_bad, tid + 1);
    }
    const int any_bad = __syncthreads_or(!ok);
    const int k = accepted[b];
    if (status && cblk == 0 && tid == 0) status[b] = any_bad ? first_bad : ((k < -1 || k >= n) ? -1 : 0);
    const int c0 = (cblk * kThreads + tid) * VEC;
    if (c0 >= Cc) return;
    const bool pass = any_bad || k < 0 || k >= n;
    uint4 rows[3];  // W - 1 <= 3 rows of 16 bytes
    int v = pass ? -1 : k, above = 0;
    for (int m = 0; m < W - 1; ++m) {  // m-th ancestor of k feeds out row W-2-m
        const T *src;
        if (v >= 0) {
            src = xbc_pre + ((size_t)b * n + v) * Cc + c0;
            v = par[v];
        } else {
            ++above;
            src = conv_state + ((size_t)b * (W - 1) + (W - 1 - above)) * Cc + c0;
        }
        rows[m] = *reinterpret_cast<const uint4 *>(src);
    }
    for (int m = 0; m < W - 1; ++m)
        *reinterpret_cast<uint4 *>(conv_state_out + ((size_t)b * (W - 1) + (W - 2 - m)) * Cc + c0) = rows[m];
}

struct ConvTailArgs {      // conv part folded into the state kernel's grid (cblocks = 0: none)
    const void *xbc_pre, *conv_state;
    void *conv_state_out;
    int Cc, W, cblocks, batch;
    int state_z;           // z slices of the grid that belong to the state (batch, or 0 with no state)
};

// grid (slabs, H, B [+ conv-tail slices]); dynamic LDS = kPathChunk * (P + S) floats.
// A thread owns one 4-wide piece s4 of the state index and kQ consecutive rows p, so that per
// path node it needs one B piece and kQ x values: three 16-byte LDS reads for 4*kQ FMAs.  A
// workgroup covers rows_wg = kQ * (256 / (S/4)) rows; slabs = ceil(P / rows_wg).
// The z slices behind the batch, when present, carry the conv tail: their first cblocks * B
// workgroups each copy one channel block of one sequence, so that the whole commit is one launch.
// (They follow the state's workgroups rather than alternate with them: workgroups go to the eight
// XCDs in turn, and a grid that alternates would put all of the state on every other XCD.)
//
// FAST (every thread owns kQ rows inside the state, 16-byte aligned x / B rows; see
// commit_fast_shape): nothing on the way from the state loads to the state stores is predicated.
// The small parent / dt loads go out ahead of the state loads, so that the wave that works out
// the path waits for those alone; the path rows are fetched as 16-byte pieces, all requested
// before any is waited for; the stores follow each other with no wait between them.  (With
// per-row bounds branches the compiler had put a full wait in front of every load of the path rows
// and of every store: a dozen serial round trips per workgroup.)
// NS = 16-byte pieces of a chunk of path rows per thread (0: the general, predicated kernel).  With
// two pieces the kernel needs under 102 registers, i.e. five workgroups per CU: at 80 heads x
// batch 16 every workgroup of the launch is resident at once.  (Forcing that budget on the compiler
// where it does not come by itself is worse than four per CU: the spills wait on the state loads.)
template <typename T, typename HT, bool WAVE, int NS, bool SPL>
__global__ __launch_bounds__(kThreads) void commit_h_kernel(
    const int32_t *__restrict__ parent, const int32_t *__restrict__ accepted, int n, int H, int P, int S,
    int G, const T *__restrict__ x, long x_sn, const float *__restrict__ dt, const float *__restrict__ dt_bias,
    const float *__restrict__ A, const T *__restrict__ Bm, long b_sn, const HT *h0, HT *h_out,
    int32_t *__restrict__ status, int slabs, ConvTailArgs ct) {
    constexpr bool FAST = NS > 0;
    constexpr int kStageMax = NS ? NS : 1;
    if ((int)blockIdx.z >= ct.state_z) {               // the conv-tail slices at the end of the grid
        const int idx = (((int)blockIdx.z - ct.state_z) * (int)gridDim.y + (int)blockIdx.y) * (int)gridDim.x + (int)blockIdx.x;
        if (idx < ct.cblocks * ct.batch)
            conv_tail<T, 16 / (int)sizeof(T)>(idx / ct.cblocks, idx % ct.cblocks, parent, accepted, n, ct.Cc, ct.W,
                                              (const T *)ct.xbc_pre, (const T *)ct.conv_state,
                                              (T *)ct.conv_state_out, ct.state_z == 0 ? status : nullptr);
        return;
    }
    extern __shared__ __align__(16) float rows[];     // xs[kPathChunk][P] then bs[kPathChunk][S]
    __shared__ int path[kMaxNodes];
    __shared__ float coef[kMaxNodes];
    float *xs = rows, *bs = rows + kPathChunk * P;
    const int tid = threadIdx.x, lane = tid & 63, h = blockIdx.y, b = blockIdx.z;
    const int g = h / (H / G);

    const int S4 = S >> 2, RP = kThreads / S4;
    const int s4 = tid % S4, p0 = (blockIdx.x * RP + tid / S4) * kQ;   // rows p0 .. p0 + kQ - 1
    const bool owner = FAST || tid < RP * S4;          // S/4 need not divide the thread count
    const size_t sbase = ((size_t)b * H + h) * P * S + (size_t)s4 * 4;
    const size_t ubase = ((size_t)b * H + h) * P * S;              // FAST: the head's state, uniform
    const uint32_t loff = (uint32_t)(p0 * S + s4 * 4) * (uint32_t)sizeof(HT);   // and this thread's place in it, bytes
    // n <= 64: every wave asks for the parents and step sizes (wave 0 uses them), ahead of the state
    int par_j = -1;
    float dt_j = 0.f;
    if constexpr (WAVE) {
        const int node = min(lane, n - 1);
        par_j = parent[(size_t)b * n + node];
        dt_j = dt[((size_t)b * n + node) * H + h];
    }
    // the state rows: these loads fly while the path is worked out (read once: streaming hint,
    // as for the store of the result below)
    float4 acc[kQ];
    if constexpr (FAST) {
        const HT *src = h0 ? h0 : h_out;              // no initial state: any readable rows, zeroed below
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            // (uniform row pointer + one 32-bit lane offset: one address register for all kQ rows)
            acc[q] = load_state4(reinterpret_cast<const HT *>(
                reinterpret_cast<const char *>(src + ubase + (size_t)q * S) + loff));
        }
    } else {
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int p = p0 + q;
            acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (h0 && owner && p < P) acc[q] = load_state4(h0 + sbase + (size_t)p * S);
        }
    }

    const int k = accepted[b];
    const bool k_bad = (k < -1) || (k >= n);
    const float A_h = A[h];
    float bias_h = 0.f;
    if constexpr (SPL) bias_h = dt_bias[h];
    int bad, len = 0;
    float decay = 1.f;
    if constexpr (WAVE) {
        // n <= 64: every wave finds the path in registers (all of them use the parent / dt values, so
        // their loads stay where they were issued, ahead of the state); wave 0 publishes it
        int pos;
        float cf;
        if constexpr (SPL) dt_j = softplus_step(dt_j + bias_h);      // raw projection -> step size
        bad = wave_path(lane, n, (k >= 0 && !k_bad) ? k : 0, par_j, dt_j, A_h, pos, cf, len, decay);
        if (tid < 64 && bad == 0 && pos >= 0) {
            path[pos] = lane;
            coef[pos] = cf;
        }
        __syncthreads();
    } else {
        __shared__ TreeLds tree;
        __shared__ uint32_t mask[kMaxNodes * kMaxWords];
        const int words = (n + 31) / 32;
        const float dt_raw = tid < n ? dt[((size_t)b * n + tid) * H + h] : 0.f;
        const float dt_i = (SPL && tid < n) ? softplus_step(dt_raw + bias_h) : dt_raw;
        bad = build_tree_index(tree, mask, parent + (size_t)b * n, n, n, words, dt_i, A_h);
        len = 0;
        if (!bad && k >= 0 && !k_bad) {
            // compact path(k) (ancestors have smaller labels, so ascending label = root first)
            if (tid < n && mask_bit(mask, words, k, tid)) {
                int pos = 0;
                for (int w = 0; w < (tid >> 5); ++w) pos += __popc(mask[k * words + w]);
                pos += __popc(mask[k * words + (tid >> 5)] & ((1u << (tid & 31)) - 1u));
                path[pos] = tid;
                coef[pos] = tree.dt[tid];              // the step size for now, the weight below
            }
            len = tree.cnt[k];
        }
        __syncthreads();
        // exp(s_k - s_j) as the exponential of the sum of dt_m A over the path nodes BEHIND j, summed
        // along the path itself (thread = position on the path from here on): its rounding error is
        // relative to that sum, which is small wherever the weight is not negligible, while the
        // difference of two prefix sums carries the error of |s_k| (hundreds on a long chain with a
        // strong decay: 1e-4 in the weight).  Suffix sums inside each wave, then the later waves' totals.
        __shared__ float wave_total[kThreads / 64];
        const float dt_p = tid < len ? coef[tid] : 0.f;
        float suf = dt_p * A_h;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float t = __shfl_down(suf, off);
            if (lane + off < 64) suf += t;
        }
        float behind = __shfl_down(suf, 1);
        if (lane == 63) behind = 0.f;
        if (lane == 0) wave_total[tid >> 6] = suf;
        __syncthreads();
        float whole = 0.f;
#pragma unroll
        for (int w = kThreads / 64 - 1; w >= 0; --w) {
            if (w > (tid >> 6)) behind += wave_total[w];
            whole += wave_total[w];
        }
        if (tid < len) coef[tid] = dt_p * __expf(behind);
        decay = __expf(whole);                         // (no path: exp(0) = 1)
        __syncthreads();
    }
    if (status && blockIdx.x == 0 && h == 0 && tid == 0) status[b] = bad ? bad : (k_bad ? -1 : 0);

    const bool pass = bad || k < 0 || k_bad;          // the state goes through unchanged
    if (pass && h_out == h0 && h0) return;
    if constexpr (FAST) {
        if (!h0) {                                     // (here, not at the loads: this is their first use)
#pragma unroll
            for (int q = 0; q < kQ; ++q) acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
    const T *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
    const T *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
    bool scaled = false;
    for (int c0 = 0; !pass && c0 < len; c0 += kPathChunk) {
        const int cn = min(kPathChunk, len - c0);
        if constexpr (FAST) {
            constexpr int EPV = 16 / (int)sizeof(T);   // elements of a 16-byte piece
            const int px = P / EPV, ppn = (P + S) / EPV, total = cn * ppn;
            uint4 piece[kStageMax];
#pragma unroll
            for (int q = 0; q < kStageMax; ++q) {      // (clamped: the last piece again past the end)
                const int idx = min(q * kThreads + tid, total - 1);
                const int t = idx / ppn, c = idx % ppn;
                const int node = path[c0 + t];
                const T *src = c < px ? xb + (size_t)node * x_sn + c * EPV : Bb + (size_t)node * b_sn + (c - px) * EPV;
                piece[q] = *reinterpret_cast<const uint4 *>(src);
            }
            // (the decay is made opaque here so that the scaling of the state below, which waits for
            // the state loads, is not scheduled in front of these requests)
            asm volatile("" : "+v"(decay) : : "memory");
#pragma unroll
            for (int q = 0; q < kStageMax; ++q) {
                const int idx = q * kThreads + tid;
                if (idx < total) {
                    const int t = idx / ppn, c = idx % ppn;
                    const float w = c < px ? 1.f : coef[c0 + t];
                    float *dst = c < px ? xs + t * P + c * EPV : bs + t * S + (c - px) * EPV;
                    float f[8];
                    if constexpr (sizeof(T) == 2) {
                        f[0] = bf16_lo(piece[q].x); f[1] = bf16_hi(piece[q].x); f[2] = bf16_lo(piece[q].y); f[3] = bf16_hi(piece[q].y);
                        f[4] = bf16_lo(piece[q].z); f[5] = bf16_hi(piece[q].z); f[6] = bf16_lo(piece[q].w); f[7] = bf16_hi(piece[q].w);
                    } else {
                        f[0] = __uint_as_float(piece[q].x); f[1] = __uint_as_float(piece[q].y);
                        f[2] = __uint_as_float(piece[q].z); f[3] = __uint_as_float(piece[q].w);
                    }
#pragma unroll
                    for (int e = 0; e < EPV; e += 4)
                        *reinterpret_cast<float4 *>(dst + e) = make_float4(w * f[e], w * f[e + 1], w * f[e + 2], w * f[e + 3]);
                }
            }
        } else {
            for (int idx = tid; idx < cn * (P + S); idx += kThreads) {
                const int t = idx / (P + S), col = idx % (P + S);
                const int node = path[c0 + t];
                if (col < P) xs[t * P + col] = to_f32(xb[(size_t)node * x_sn + col]);
                else bs[t * S + col - P] = coef[c0 + t] * to_f32(Bb[(size_t)node * b_sn + (col - P)]);
            }
        }
        if (!scaled) {   // the state loads are first needed here
#pragma unroll
            for (int q = 0; q < kQ; ++q) {
                acc[q].x *= decay; acc[q].y *= decay; acc[q].z *= decay; acc[q].w *= decay;
            }
            scaled = true;
        }
        __syncthreads();
        if (owner && p0 < P) {
            for (int t = 0; t < cn; ++t) {
                const float4 bv = *reinterpret_cast<const float4 *>(&bs[t * S + s4 * 4]);
                float xv[kQ];
                if (P % kQ == 0) {   // kQ consecutive rows, 16-byte aligned: p0 is a multiple of kQ
#pragma unroll
                    for (int q = 0; q < kQ; q += 4) {
                        const float4 v = *reinterpret_cast<const float4 *>(&xs[t * P + p0 + q]);
                        xv[q] = v.x; xv[q + 1] = v.y; xv[q + 2] = v.z; xv[q + 3] = v.w;
                    }
                } else {
#pragma unroll
                    for (int q = 0; q < kQ; ++q) xv[q] = xs[t * P + min(p0 + q, P - 1)];
                }
#pragma unroll
                for (int q = 0; q < kQ; ++q) {
                    acc[q].x = fmaf(xv[q], bv.x, acc[q].x);
                    acc[q].y = fmaf(xv[q], bv.y, acc[q].y);
                    acc[q].z = fmaf(xv[q], bv.z, acc[q].z);
                    acc[q].w = fmaf(xv[q], bv.w, acc[q].w);
                }
            }
        }
        __syncthreads();
    }
    if constexpr (FAST) {
#pragma unroll
        for (int q = 0; q < kQ; ++q)
            store_state4(reinterpret_cast<HT *>(reinterpret_cast<char *>(h_out + ubase + (size_t)q * S) + loff), acc[q]);
    } else if (owner) {
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int p = p0 + q;
            if (p < P) store_state4(h_out + sbase + (size_t)p * S, acc[q]);
        }
    }
}

// Shapes of the unpredicated kernel: the threads tile the state exactly (S/4 divides the workgroup,
// its kQ-row slabs divide P), x and B rows are whole 16-byte pieces at 16-byte addresses, and a
// chunk of path rows is at most four pieces per thread.  Returns that number of pieces (2 or 4), or 0.
static int commit_fast_shape(const stree_dims &d, const void *x, const void *Bm, const void *h0,
                              const void *h_out) {
    const int S4 = d.dstate / 4;
    if (d.dstate % 4 != 0 || S4 > kThreads || kThreads % S4 != 0) return 0;
    const int rows_wg = kQ * (kThreads / S4);
    if (d.headdim % rows_wg != 0) return 0;
    const int epv = d.io_dtype == STREE_BF16 ? 8 : 4;
    if (d.headdim % epv != 0 || d.dstate % epv != 0 || d.x_stride_n % epv != 0 || d.b_stride_n % epv != 0)
        return 0;
    if (((uintptr_t)x | (uintptr_t)Bm | (uintptr_t)h0 | (uintptr_t)h_out) % 16 != 0) return 0;
    const int pieces = kPathChunk * ((d.headdim + d.dstate) / epv);
    return pieces <= 2 * kThreads ? 2 : pieces <= 4 * kThreads ? 4 : 0;
}

hipError_t launch_commit_state(const stree_dims &d, const int32_t *parent, const int32_t *accepted,
                               const void *x, const float *dt, const float *A, const void *Bm,
                               const void *h0, void *h_out, const void *xbc_pre, const void *conv_state,
                               void *conv_state_out, int32_t *status, hipStream_t st) {
    const int rows_wg = kQ * (kThreads / (d.dstate / 4));   // state rows per workgroup
    const int slabs = h_out ? (d.headdim + rows_wg - 1) / rows_wg : 0;
    const int Cc = d.nheads * d.headdim + 2 * d.ngroups * d.dstate;
    const int vec = d.io_dtype == STREE_BF16 ? 8 : 4;
    // channel blocks of the conv tail; never more than heads: Cc = H*P + 2*G*S <= H*(P + 2*S) and
    // P, S <= 256 give Cc / (vec*256) <= 0.75 * H
    const int cblocks = conv_state_out ? (Cc / vec + kThreads - 1) / kThreads : 0;
    if (slabs + cblocks == 0) return hipSuccess;
    const int gx = slabs ? slabs : cblocks, gy = slabs ? d.nheads : 1, state_z = slabs ? d.batch : 0;
    const int tail_z = (cblocks * d.batch + gx * gy - 1) / (gx * gy);
    if (state_z + tail_z > 65535) return hipErrorInvalidValue;
    ConvTailArgs ct = {xbc_pre, conv_state, conv_state_out, Cc, d.conv_width, cblocks, d.batch, state_z};
    const dim3 grid(gx, gy, state_z + tail_z);
    const size_t lds = (size_t)kPathChunk * (d.headdim + d.dstate) * sizeof(float);
    // (the in-kernel softplus is a variant of its own: compiled into the common one, even unused, it costs time)
#define STREE_COMMIT_LAUNCH_SP(TT, HT, WV, NS, SPL)                                                              \
    hipLaunchKernelGGL((commit_h_kernel<TT, HT, WV, NS, SPL>), grid, dim3(kThreads), lds, st, parent, accepted,  \
                       d.nnodes, d.nheads, d.headdim, d.dstate, d.ngroups, (const TT *)x, (long)d.x_stride_n,    \
                       dt, step_bias(d), A, (const TT *)Bm, (long)d.b_stride_n, (const HT *)h0, (HT *)h_out,     \
                       status, slabs, ct)
#define STREE_COMMIT_LAUNCH(TT, HT, WV, NS)                             \
    do {                                                                \
        if (step_bias(d)) STREE_COMMIT_LAUNCH_SP(TT, HT, WV, NS, true); \
        else STREE_COMMIT_LAUNCH_SP(TT, HT, WV, NS, false);             \
    } while (0)
    const bool wave = d.nnodes <= 64;
    const int ns = slabs > 0 ? commit_fast_shape(d, x, Bm, h0, h_out) : 0;
#define STREE_COMMIT_NS(TT, HT, WV)                                 \
    do {                                                            \
        if (ns == 2) STREE_COMMIT_LAUNCH(TT, HT, WV, 2);            \
        else if (ns == 4) STREE_COMMIT_LAUNCH(TT, HT, WV, 4);       \
        else STREE_COMMIT_LAUNCH(TT, HT, WV, 0);                    \
    } while (0)
#define STREE_COMMIT_WV(TT, HT)                 \
    do {                                        \
        if (wave) STREE_COMMIT_NS(TT, HT, true); \
        else STREE_COMMIT_NS(TT, HT, false);    \
    } while (0)
    if (d.io_dtype == STREE_BF16) {
        if (d.state_dtype == STREE_BF16) STREE_COMMIT_WV(bf16_t, bf16_t);   // (a bf16 state goes with bf16 io only)
        else STREE_COMMIT_WV(bf16_t, float);
    } else {
        STREE_COMMIT_WV(float, float);
    }
#undef STREE_COMMIT_WV
#undef STREE_COMMIT_NS
#undef STREE_COMMIT_LAUNCH
#undef STREE_COMMIT_LAUNCH_SP
    return hipGetLastError();
}

}  // namespace stree
