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
template <typename T, int VEC>
__device__ __forceinline__ void conv_tail(int b, int cblk, const int32_t *__restrict__ parent,
                                          const int32_t *__restrict__ accepted, int n, int Cc, int W,
                                          const T *__restrict__ xbc_pre, const T *conv_state, T *conv_state_out) {
    __shared__ int par[kMaxNodes];
    const int tid = threadIdx.x;
    int ok = 1;
    if (tid < n) {
        const int p = parent[(size_t)b * n + tid];
        ok = (tid == 0) ? (p == -1) : (p >= 0 && p < tid);
        par[tid] = ok ? p : -1;
    }
    const int any_bad = __syncthreads_or(!ok);
    const int k = accepted[b];
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
    int Cc, W, cblocks;
};

// grid (slabs [+ 1], H, B); dynamic LDS = kPathChunk * (P + S) floats.
// A thread owns one 4-wide piece s4 of the state index and kQ consecutive rows p, so that per
// path node it needs one B piece and kQ x values: three 16-byte LDS reads for 4*kQ FMAs.  A
// workgroup covers rows_wg = kQ * (256 / (S/4)) rows; slabs = ceil(P / rows_wg).
// The extra x index, when present, carries the conv tail: its workgroups with h < cblocks each copy
// one channel block, so that the whole commit is one launch.
template <typename T, bool WAVE>
__global__ __launch_bounds__(kThreads) void commit_h_kernel(
    const int32_t *__restrict__ parent, const int32_t *__restrict__ accepted, int n, int H, int P, int S,
    int G, const T *__restrict__ x, long x_sn, const float *__restrict__ dt, const float *__restrict__ A,
    const T *__restrict__ Bm, long b_sn, const float *h0, float *h_out, int32_t *__restrict__ status,
    int slabs, ConvTailArgs ct) {
    if ((int)blockIdx.x >= slabs) {                    // the conv-tail slot of the grid
        if ((int)blockIdx.y < ct.cblocks)
            conv_tail<T, 16 / (int)sizeof(T)>(blockIdx.z, blockIdx.y, parent, accepted, n, ct.Cc, ct.W,
                                              (const T *)ct.xbc_pre, (const T *)ct.conv_state,
                                              (T *)ct.conv_state_out);
        return;
    }
    extern __shared__ __align__(16) float rows[];     // xs[kPathChunk][P] then bs[kPathChunk][S]
    __shared__ int path[kMaxNodes];
    __shared__ float coef[kMaxNodes];
    __shared__ float scal[2];                          // decay, then path length (as int bits)
    __shared__ int bad_s;
    float *xs = rows, *bs = rows + kPathChunk * P;
    const int tid = threadIdx.x, lane = tid & 63, h = blockIdx.y, b = blockIdx.z;
    const int g = h / (H / G);

    // the state rows first: these loads fly while the path is worked out
    const int S4 = S >> 2, RP = kThreads / S4;
    const int s4 = tid % S4, p0 = (blockIdx.x * RP + tid / S4) * kQ;   // rows p0 .. p0 + kQ - 1
    const bool owner = tid < RP * S4;                  // S/4 need not divide the thread count
    const size_t sbase = ((size_t)b * H + h) * P * S + (size_t)s4 * 4;
    float4 acc[kQ];
#pragma unroll
    for (int q = 0; q < kQ; ++q) {
        const int p = p0 + q;
        acc[q] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (h0 && owner && p < P) {   // read once: streaming hint (as for the store of the result below)
            const uint4 v = load_stream16(h0 + sbase + (size_t)p * S);
            acc[q] = make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
        }
    }

    const int k = accepted[b];
    const bool k_bad = (k < -1) || (k >= n);
    const float A_h = A[h];
    int bad, len;
    float decay;
    if constexpr (WAVE) {
        // n <= 64: wave 0 finds the path in registers and publishes it
        if (tid < 64) {
            const int node = min(lane, n - 1);
            const int par_j = parent[(size_t)b * n + node];
            const float dt_j = dt[((size_t)b * n + node) * H + h];
            int pos, ln;
            float cf, dc;
            const int st = wave_path(lane, n, (k >= 0 && !k_bad) ? k : 0, par_j, dt_j, A_h, pos, cf, ln, dc);
            if (st == 0 && pos >= 0) {
                path[pos] = lane;
                coef[pos] = cf;
            }
            if (lane == 0) {
                bad_s = st;
                scal[0] = dc;
                scal[1] = __int_as_float(ln);
            }
        }
        __syncthreads();
        bad = bad_s;
        decay = scal[0];
        len = __float_as_int(scal[1]);
    } else {
        __shared__ TreeLds tree;
        __shared__ uint32_t mask[kMaxNodes * kMaxWords];
        const int words = (n + 31) / 32;
        const float dt_i = tid < n ? dt[((size_t)b * n + tid) * H + h] : 0.f;
        bad = build_tree_index(tree, mask, parent + (size_t)b * n, n, n, words, dt_i, A_h);
        len = 0;
        decay = 1.f;
        if (!bad && k >= 0 && !k_bad) {
            // compact path(k) (ancestors have smaller labels, so ascending label = root first)
            const float s_k = tree.s[k];
            if (tid < n && mask_bit(mask, words, k, tid)) {
                int pos = 0;
                for (int w = 0; w < (tid >> 5); ++w) pos += __popc(mask[k * words + w]);
                pos += __popc(mask[k * words + (tid >> 5)] & ((1u << (tid & 31)) - 1u));
                path[pos] = tid;
                coef[pos] = tree.dt[tid] * __expf(s_k - tree.s[tid]);
            }
            len = tree.cnt[k];
            decay = __expf(s_k);
        }
        __syncthreads();
    }
    if (status && blockIdx.x == 0 && h == 0 && tid == 0) status[b] = bad ? bad : (k_bad ? -1 : 0);

    const bool pass = bad || k < 0 || k_bad;          // the state goes through unchanged
    if (pass && h_out == h0 && h0) return;
    const T *xb = x + (size_t)b * n * x_sn + (size_t)h * P;
    const T *Bb = Bm + (size_t)b * n * b_sn + (size_t)g * S;
    bool scaled = false;
    for (int c0 = 0; !pass && c0 < len; c0 += kPathChunk) {
        const int cn = min(kPathChunk, len - c0);
        for (int idx = tid; idx < cn * (P + S); idx += kThreads) {
            const int t = idx / (P + S), col = idx % (P + S);
            const int node = path[c0 + t];
            if (col < P) xs[t * P + col] = to_f32(xb[(size_t)node * x_sn + col]);
            else bs[t * S + col - P] = coef[c0 + t] * to_f32(Bb[(size_t)node * b_sn + (col - P)]);
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
    if (owner) {
#pragma unroll
        for (int q = 0; q < kQ; ++q) {
            const int p = p0 + q;
            if (p < P)
                store_stream16(h_out + sbase + (size_t)p * S,
                               make_uint4(__float_as_uint(acc[q].x), __float_as_uint(acc[q].y),
                                          __float_as_uint(acc[q].z), __float_as_uint(acc[q].w)));
        }
    }
}

hipError_t launch_commit_state(const stree_dims &d, const int32_t *parent, const int32_t *accepted,
                               const void *x, const float *dt, const float *A, const void *Bm,
                               const float *h0, float *h_out, const void *xbc_pre, const void *conv_state,
                               void *conv_state_out, int32_t *status, hipStream_t st) {
    const int rows_wg = kQ * (kThreads / (d.dstate / 4));   // state rows per workgroup
    const int slabs = h_out ? (d.headdim + rows_wg - 1) / rows_wg : 0;
    const int Cc = d.nheads * d.headdim + 2 * d.ngroups * d.dstate;
    const int vec = d.io_dtype == STREE_BF16 ? 8 : 4;
    // channel blocks of the conv tail; never more than heads: Cc = H*P + 2*G*S <= H*(P + 2*S) and
    // P, S <= 256 give Cc / (vec*256) <= 0.75 * H
    const int cblocks = conv_state_out ? (Cc / vec + kThreads - 1) / kThreads : 0;
    if (cblocks > d.nheads) return hipErrorInvalidValue;
    ConvTailArgs ct = {xbc_pre, conv_state, conv_state_out, Cc, d.conv_width, cblocks};
    if (slabs + cblocks == 0) return hipSuccess;
    const dim3 grid(slabs + (cblocks ? 1 : 0), slabs ? d.nheads : cblocks, d.batch);
    const size_t lds = (size_t)kPathChunk * (d.headdim + d.dstate) * sizeof(float);
#define STREE_COMMIT_LAUNCH(TT, WV)                                                                           \
    hipLaunchKernelGGL((commit_h_kernel<TT, WV>), grid, dim3(kThreads), lds, st, parent, accepted, d.nnodes,     \
                       d.nheads, d.headdim, d.dstate, d.ngroups, (const TT *)x, (long)d.x_stride_n, dt, A,      \
                       (const TT *)Bm, (long)d.b_stride_n, h0, h_out, status, slabs, ct)
    const bool wave = d.nnodes <= 64;
    if (d.io_dtype == STREE_BF16) {
        if (wave) STREE_COMMIT_LAUNCH(bf16_t, true);
        else STREE_COMMIT_LAUNCH(bf16_t, false);
    } else {
        if (wave) STREE_COMMIT_LAUNCH(float, true);
        else STREE_COMMIT_LAUNCH(float, false);
    }
#undef STREE_COMMIT_LAUNCH
    return hipGetLastError();
}

}  // namespace stree
