// Shared device helpers for the libstree kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/stree.h"

namespace stree {

constexpr int kThreads = 256;  // every kernel here runs 256-thread workgroups (4 waves)
constexpr int kMaxNodes = STREE_MAX_NODES;
constexpr int kMaxWords = kMaxNodes / 32;

typedef __bf16 bf16_t;
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

__device__ __forceinline__ float to_f32(float v) { return v; }
__device__ __forceinline__ float to_f32(bf16_t v) { return (float)v; }
__device__ __forceinline__ void from_f32(float v, float &o) { o = v; }
__device__ __forceinline__ void from_f32(float v, bf16_t &o) { o = (bf16_t)v; }  // round to nearest even

__device__ __forceinline__ float bf16_lo(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __uint_as_float(w & 0xffff0000u); }

// ---------------------------------------------------------------------------
// Tree index of one sequence, built cooperatively by a 256-thread workgroup in
// LDS.  Thread i owns node i.  Pointer doubling over the parent array: every
// node keeps a jump pointer and the aggregate (log-decay sum, node count,
// ancestor bit set) of the path segment from itself up to, not including, the
// jump target; each round merges the target's segment and doubles the jump.
// ceil(log2(depth+1)) rounds.  The aggregates are the tree mask row L_i, the
// depth, and s_i = sum over path(i) of dt*A (the paper's A_tree, Eq. a_tree).
// ---------------------------------------------------------------------------
struct __align__(16) TreeLds {
    float s[kMaxNodes];           // cumulative log-decay (A_tree)_i
    float dt[kMaxNodes];          // dt of each node for this head (0 beyond N)
    int cnt[kMaxNodes];           // nodes on path(i); depth = cnt - 1
    int jump[kMaxNodes];
    int bad;                      // first invalid node + 1, or INT_MAX
};
// The ancestor bit rows live in a separate LDS array `mask` of npad*words words
// (row i at mask[i*words ..)), so that kernels size it to the tree at hand.

// Loads and validates parent[], returns the (uniform) status: 0 or bad node + 1.
// On return (after the internal barriers) s/cnt/mask are final for i < n; rows
// n..npad-1 of s, dt, mask are zero.  `dtA` is this thread's dt_i * A_h (any
// value for i >= n).
__device__ __forceinline__ int build_tree_index(TreeLds &T, uint32_t *mask, const int32_t *__restrict__ parent,
                                                int n, int npad, int words, float dt_i, float A_h) {
    const int i = threadIdx.x;
    if (i == 0) T.bad = 0x7fffffff;
    __syncthreads();
    int p = -1;
    uint32_t m[kMaxWords];
#pragma unroll
    for (int w = 0; w < kMaxWords; ++w) m[w] = 0u;
    float s = 0.f;
    int cnt = 1;
    if (i < n) {
        p = parent[i];
        const bool ok = (i == 0) ? (p == -1) : (p >= 0 && p < i);
        if (!ok) {
            atomicMin(&T.bad, i + 1);
            p = -1;
        }
        s = dt_i * A_h;
#pragma unroll
        for (int w = 0; w < kMaxWords; ++w)
            if (w == (i >> 5)) m[w] = 1u << (i & 31);
    }
    if (i < npad) {
        T.s[i] = (i < n) ? s : 0.f;
        T.dt[i] = (i < n) ? dt_i : 0.f;
        T.cnt[i] = cnt;
        T.jump[i] = p;
#pragma unroll
        for (int w = 0; w < kMaxWords; ++w)
            if (w < words) mask[i * words + w] = m[w];
    }
    __syncthreads();
    const int bad = T.bad;
    if (bad != 0x7fffffff) return bad;
    // at most 8 rounds: depth < 256
    for (int round = 0; round < 8; ++round) {
        if (!__syncthreads_or(p >= 0)) break;
        float rs = 0.f;
        int rc = 0, rp = -1;
        uint32_t rm[kMaxWords];
#pragma unroll
        for (int w = 0; w < kMaxWords; ++w) rm[w] = 0u;
        if (p >= 0) {
            rs = T.s[p];
            rc = T.cnt[p];
            rp = T.jump[p];
#pragma unroll
            for (int w = 0; w < kMaxWords; ++w)
                if (w < words) rm[w] = mask[p * words + w];
        }
        __syncthreads();
        if (p >= 0) {
            s += rs;
            cnt += rc;
            p = rp;
            T.s[i] = s;
            T.cnt[i] = cnt;
            T.jump[i] = p;
#pragma unroll
            for (int w = 0; w < kMaxWords; ++w)
                if (w < words) {
                    m[w] |= rm[w];
                    mask[i * words + w] = m[w];
                }
        }
    }
    __syncthreads();
    return 0;
}

__device__ __forceinline__ bool mask_bit(const uint32_t *mask, int words, int i, int j) {
    return (mask[i * words + (j >> 5)] >> (j & 31)) & 1u;
}

}  // namespace stree
