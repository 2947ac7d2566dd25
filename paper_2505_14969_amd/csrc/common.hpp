// Shared device helpers for the libstree kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/stree.h"

namespace stree {

constexpr int kThreads = 256;  // workgroup size of the kernels that do not set their own (the persistent scan runs 512)
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

// Step size of a token from the raw projection, softplus(raw + bias_h): Mamba2's discretisation of the
// recurrence of Eq. ssm, used by the kernel variants that the caller selects with a bias vector.
//   softplus(v) = max(v, 0) + log1p(exp(-|v|)),   log1p(t) = log(1 + t) * t / ((1 + t) - 1)
// (the quotient restores what the rounding of 1 + t lost; 1 + t == 1: log1p(t) = t).  A dozen instructions,
// no branch, hardware exp2 / log2 / reciprocal: a few ulp, far inside the tolerance of the state (1e-4) --
// it sits on the chain parents -> path -> rows -> state that the commit kernels are bound by.
__device__ __forceinline__ float softplus_step(float v) {
    const float t = __expf(-fabsf(v));
    const float u = 1.f + t;
    const float l = (u == 1.f) ? t : __logf(u) * __fdividef(t, u - 1.f);
    return fmaxf(v, 0.f) + l;
}
__device__ __forceinline__ float step_size(float raw, const float *__restrict__ bias, int h) {
    return bias ? softplus_step(raw + bias[h]) : raw;
}

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

// Validates the parents (thread i passes parent[i]; any value for i >= n) and
// returns the (uniform) status: 0 or bad node + 1.  On return (after the
// internal barriers) s/cnt/mask are final for i < n; rows n..npad-1 of s, dt,
// mask are zero.  dt_i is this thread's step size (any value for i >= n).
__device__ __forceinline__ int build_tree_index(TreeLds &T, uint32_t *mask, int parent_i, int n, int npad,
                                                int words, float dt_i, float A_h) {
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
        p = parent_i;
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

// The same, with thread i loading parent[i] itself.
__device__ __forceinline__ int build_tree_index(TreeLds &T, uint32_t *mask, const int32_t *__restrict__ parent,
                                                int n, int npad, int words, float dt_i, float A_h) {
    const int i = threadIdx.x;
    return build_tree_index(T, mask, i < n ? parent[i] : -1, n, npad, words, dt_i, A_h);
}

__device__ __forceinline__ bool mask_bit(const uint32_t *mask, int words, int i, int j) {
    return (mask[i * words + (j >> 5)] >> (j & 31)) & 1u;
}

// 16-byte load of data that is read once (the state tiles): the streaming hint keeps it from
// displacing the B / C rows that the heads of a group share in L2.
__device__ __forceinline__ uint4 load_stream16(const void *p) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

// 16-byte store of data that this kernel does not read again.
__device__ __forceinline__ void store_stream16(void *p, uint4 v) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 vv = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(vv, reinterpret_cast<u32x4 *>(p));
}

// Four consecutive values of the recurrent state, which is kept in fp32 (16 bytes) or in bf16 (8 bytes):
// read once and written once per call, both with the streaming hint.  A bf16 state is widened exactly
// on the way in and rounded to nearest even on the way out.
__device__ __forceinline__ uint2 load_stream8(const void *p) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 v = __builtin_nontemporal_load(reinterpret_cast<const u32x2 *>(p));
    return make_uint2(v.x, v.y);
}
__device__ __forceinline__ void store_stream8(void *p, uint2 v) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 vv = {v.x, v.y};
    __builtin_nontemporal_store(vv, reinterpret_cast<u32x2 *>(p));
}
__device__ __forceinline__ uint2 pack_bf16x4(float a, float b, float c, float d) {
    typedef __bf16 bf16x4_t __attribute__((ext_vector_type(4)));
    bf16x4_t o;
    o[0] = (__bf16)a; o[1] = (__bf16)b; o[2] = (__bf16)c; o[3] = (__bf16)d;
    return __builtin_bit_cast(uint2, o);
}
__device__ __forceinline__ float4 load_state4(const float *p) {
    const uint4 v = load_stream16(p);
    return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
}
__device__ __forceinline__ float4 load_state4(const __bf16 *p) {
    const uint2 v = load_stream8(p);
    return make_float4(__uint_as_float(v.x << 16), __uint_as_float(v.x & 0xffff0000u), __uint_as_float(v.y << 16),
                       __uint_as_float(v.y & 0xffff0000u));
}
__device__ __forceinline__ void store_state4(float *p, float4 v) {
    store_stream16(p, make_uint4(__float_as_uint(v.x), __float_as_uint(v.y), __float_as_uint(v.z), __float_as_uint(v.w)));
}
__device__ __forceinline__ void store_state4(__bf16 *p, float4 v) { store_stream8(p, pack_bf16x4(v.x, v.y, v.z, v.w)); }

// Output stores that write through L2 (system scope) with the streaming hint: y and the replayed
// state are never read again by this kernel, and lines left dirty in the eight L2s would all be
// written back at once when the kernel ends.  (Measured on the 64-node / 80-head / batch-16 shape:
// the hint on these stores and on the h0 loads takes the scan from 18.4 to 15.8 us and the fused
// replay + scan from 33.2 to 27.6 us; on the x loads, whose lines the replay of the next step's
// kernel reads again, it costs time.)  The store is inline assembly, so the compiler does not know that it reads
// four data registers after issue: the trailing s_nop keeps the next instruction from overwriting
// them in that window (the wait states a store of more than 8 bytes needs).
__device__ __forceinline__ void store_through16(void *p, uint4 v) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 vv = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1 nt\n\ts_nop 1" ::"v"(p), "v"(vv) : "memory");
}

// The 8-byte form (a state kept in bf16).  A store of at most 8 bytes needs no wait states behind it.
__device__ __forceinline__ void store_through8(void *p, uint2 v) {
    typedef unsigned u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 vv = {v.x, v.y};
    asm volatile("global_store_dwordx2 %0, %1, off sc0 sc1 nt" ::"v"(p), "v"(vv) : "memory");
}

// The same store as a raw buffer store, the cache bits riding on an instruction the compiler knows.
// (The compiler's wait-count pass treats the operand registers of inline assembly as if a memory
// operation of unknown age still read them: the next write to any of them -- they are ordinary
// temporaries -- becomes a wait for EVERYTHING in flight, prefetches included.  A store it knows it
// counts exactly.)  `rsrc` covers `bytes` bytes from `base` (uniform); stores past the end are dropped.
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_store_rsrc(void *base, uint32_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(base, 0, (int)bytes, 0x00020000);
}
// A read-only array as a raw buffer: loads at byte offsets >= `bytes` return zeros (and a null
// array with bytes = 0 reads as all zeros).
__device__ __forceinline__ __amdgpu_buffer_rsrc_t make_buffer(const void *base, size_t bytes) {
    return __builtin_amdgcn_make_buffer_rsrc(const_cast<void *>(base), 0, (int)(uint32_t)bytes, 0x00020000);
}
__device__ __forceinline__ uint4 buffer_load16(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)off, 0, 0);
    return make_uint4(v.x, v.y, v.z, v.w);
}
__device__ __forceinline__ int buffer_load4(__amdgpu_buffer_rsrc_t rsrc, uint32_t off) {
    return (int)__builtin_amdgcn_raw_buffer_load_b32(rsrc, (int)off, 0, 0);
}
__device__ __forceinline__ void buffer_store_through16(__amdgpu_buffer_rsrc_t rsrc, uint32_t off, uint4 v) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 vv = {v.x, v.y, v.z, v.w};
    __builtin_amdgcn_raw_buffer_store_b128(vv, rsrc, (int)off, 0, 1 | 2 | 16);   // sc0 | nt | sc1
}

// 16-byte store that writes through L2 to memory (system scope) and keeps the default temporal
// policy: for an output that the next kernel reads.  The line stays in L2 for that reader, but not
// dirty: lines left dirty are all written back when the kernel ends, and the kernel is not over
// until they are.  (Measured on the 64-node / 80-head / batch-16 conv: 8.7 -> 7.5 us, and the scan
// behind it is none the slower; with the streaming hint added the scan loses what the conv wins.)
// Inline assembly: the compiler has no builtin for these cache bits; the trailing s_nop keeps the
// next instruction from overwriting the four data registers while the store still reads them.
__device__ __forceinline__ void store_written_through16(void *p, uint4 v) {
    typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
    const u32x4 vv = {v.x, v.y, v.z, v.w};
    asm volatile("global_store_dwordx4 %0, %1, off sc0 sc1\n\ts_nop 1" ::"v"(p), "v"(vv) : "memory");
}

// Four-tap conv of 8 bf16 channels on the packed dot unit (v_dot2c_f32_bf16: d += a.lo b.lo + a.hi b.hi):
//   a[e] += w[e][3] r0[e] + w[e][2] r1[e] + w[e][1] r2[e] + w[e][0] r3[e]
// r0 = the node's own row, r1..r3 its first three ancestors (8 bf16 each); ww = the 32 weights as 16
// dwords, bf16 number e * 4 + j = w[e][j].  Per channel two byte permutes pair the rows' values with
// the weight pairs as they lie in memory, instead of eight conversions and four FMAs.
__device__ __forceinline__ void conv4_bf16_dot(float (&a)[8], const uint4 &r0, const uint4 &r1, const uint4 &r2,
                                               const uint4 &r3, const uint32_t (&ww)[16]) {
    typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
    const uint32_t q0[4] = {r0.x, r0.y, r0.z, r0.w}, q1[4] = {r1.x, r1.y, r1.z, r1.w};
    const uint32_t q2[4] = {r2.x, r2.y, r2.z, r2.w}, q3[4] = {r3.x, r3.y, r3.z, r3.w};
#pragma unroll
    for (int d = 0; d < 4; ++d) {
#pragma unroll
        for (int hi = 0; hi < 2; ++hi) {
            const int e = 2 * d + hi;
            const uint32_t sel = hi ? 0x07060302u : 0x05040100u;     // (lo, hi) = (second row, first row)[channel e]
            const uint32_t x10 = __builtin_amdgcn_perm(q0[d], q1[d], sel);   // pairs with (w[e][2], w[e][3])
            const uint32_t x32 = __builtin_amdgcn_perm(q2[d], q3[d], sel);   // pairs with (w[e][0], w[e][1])
            float acc = a[e];
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ww[2 * e + 1]),
                                                  __builtin_bit_cast(bf16x2_t, x10), acc, false);
            acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, ww[2 * e]),
                                                  __builtin_bit_cast(bf16x2_t, x32), acc, false);
            a[e] = acc;
        }
    }
}

// Cross-lane read within a wave of 64: value `v` of lane `src` (0..63).  Unlike __shfl this
// needs no lane id of the caller, so nothing lane-derived stays live around it.
__device__ __forceinline__ int wave_read(int v, int src) { return __builtin_amdgcn_ds_bpermute(src << 2, v); }
__device__ __forceinline__ uint32_t wave_read(uint32_t v, int src) {
    return (uint32_t)__builtin_amdgcn_ds_bpermute(src << 2, (int)v);
}
__device__ __forceinline__ float wave_read(float v, int src) {
    return __int_as_float(__builtin_amdgcn_ds_bpermute(src << 2, __float_as_int(v)));
}
__device__ __forceinline__ unsigned long long wave_read(unsigned long long v, int src) {
    const uint32_t lo = wave_read((uint32_t)v, src), hi = wave_read((uint32_t)(v >> 32), src);
    return ((unsigned long long)hi << 32) | lo;
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves (no LDS
// round trips): shifts by 1, 2, 4, 8 inside each row of 16 lanes (zeros shifted in), then lane 15
// of rows 0 and 2 broadcast to rows 1 and 3, then lane 31 to the upper half.
template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ float dpp_move(float a) {     // lanes the move does not reach read 0
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(a), CTRL, ROW_MASK, 0xf, BOUND));
}
__device__ __forceinline__ float wave_inclusive_sum(float v) {
    v += dpp_move<0x111, 0xf, true>(v);    // row_shr:1
    v += dpp_move<0x112, 0xf, true>(v);    // row_shr:2
    v += dpp_move<0x114, 0xf, true>(v);    // row_shr:4
    v += dpp_move<0x118, 0xf, true>(v);    // row_shr:8
    v += dpp_move<0x142, 0xa, false>(v);   // row_bcast:15 into rows 1 and 3
    v += dpp_move<0x143, 0xc, false>(v);   // row_bcast:31 into rows 2 and 3
    return v;
}

// Sum of the lanes ABOVE each lane (exclusive suffix sum), same moves in the other direction: shifts
// towards lower lanes inside each row of 16, the totals of the rows above added from scalars, then
// one shift of the whole wave.  `total` = the sum over all 64 lanes.
__device__ __forceinline__ float wave_exclusive_suffix_sum(float v, float &total) {
    v += dpp_move<0x101, 0xf, true>(v);    // row_shl:1
    v += dpp_move<0x102, 0xf, true>(v);    // row_shl:2
    v += dpp_move<0x104, 0xf, true>(v);    // row_shl:4
    v += dpp_move<0x108, 0xf, true>(v);    // row_shl:8
    const float r1 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 16));
    const float r2 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 32));
    const float r3 = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 48));
    const int row = (int)(__lane_id() >> 4);
    v += row == 0 ? r1 + (r2 + r3) : row == 1 ? r2 + r3 : row == 2 ? r3 : 0.f;
    total = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 0));
    return dpp_move<0x130, 0xf, true>(v);  // wave_shl:1: lane l reads lane l + 1, lane 63 reads 0
}

// Transposing store of one 16-byte row piece (8 bf16 of row r, columns c8 .. c8+7) into an LDS
// tile laid out [column][row] with `ld` elements per column.  Two-byte scatter writes would put
// two lanes into every LDS word and serialise; instead the lanes holding rows r and r^1 of the
// same columns (lane ^ VPR, VPR = 16-byte pieces per row) swap half of their data, and each
// writes four full words (row pair, one column each).  Every lane of the wave must call it.
//
// SWZ: the tile's 16-byte groups of a column (8 rows each) are permuted by the column's group of 8,
//   group g of column c lies at group g ^ ((c >> 3) & 7)       (transposed_at() below),
// because without it the lanes of a wave that hold the same rows of different column groups all
// write to the same banks (8 columns x ld elements is a multiple of 32 words whatever the padding):
// 8- to 16-way conflicts on every transposing store.  Readers of a swizzled tile address it
// through transposed_at(); a 16-byte read of 8 consecutive rows stays one aligned group.
template <bool SWZ>
__device__ __forceinline__ int transposed_at(int ld, int c, int r) {     // element index of (column c, row r)
    return c * ld + (SWZ ? ((((r >> 3) ^ (c >> 3)) & 7) << 3) | (r & ~63) | (r & 7) : r);
}
template <int VPR, bool SWZ = false>
__device__ __forceinline__ void store_transposed_pair(unsigned short *tile, int ld, int r, int c8, uint4 v, int lane) {
    const bool odd = r & 1;
    const uint32_t r0 = wave_read(odd ? v.x : v.z, lane ^ VPR), r1 = wave_read(odd ? v.y : v.w, lane ^ VPR);
    // even row: columns c8..c8+3, own values low; odd row: columns c8+4..c8+7, own values high
    const uint32_t lo0 = odd ? r0 : v.x, lo1 = odd ? r1 : v.y, hi0 = odd ? v.z : r0, hi1 = odd ? v.w : r1;
    uint32_t *dst = reinterpret_cast<uint32_t *>(tile + transposed_at<SWZ>(ld, c8 + (odd ? 4 : 0), r & ~1));
    const int ldw = ld / 2;
    dst[0] = (lo0 & 0xffffu) | (hi0 << 16);
    dst[ldw] = (lo0 >> 16) | (hi0 & 0xffff0000u);
    dst[2 * ldw] = (lo1 & 0xffffu) | (hi1 << 16);
    dst[3 * ldw] = (lo1 >> 16) | (hi1 & 0xffff0000u);
}

// Path of the accepted node k for trees of at most 64 nodes, by one wave with no LDS and no
// barrier: lane j owns node j; pointer doubling over the parent array with cross-lane reads
// gives every lane s_j (the paper's A_tree) and its ancestor bit row; lane k's values are then
// broadcast.  Returns the tree status (uniform).  On success lane j holds in `coef` the weight
// dt_j * exp(s_k - s_j) of node j if it lies on path(k) and its position on the path (root
// first) in `pos`, else pos = -1; `len` = nodes on the path, `decay` = exp(s_k).
__device__ __forceinline__ int wave_path(int lane, int n, int k, int parent_j, float dt_j, float A_h, int &pos,
                                         float &coef, int &len, float &decay) {
    int p = -1;
    bool ok = true;
    if (lane < n) {
        p = parent_j;
        ok = (lane == 0) ? (p == -1) : (p >= 0 && p < lane);
        if (!ok) p = -1;
    }
    const unsigned long long badmask = __ballot(!ok);
    if (badmask) return __ffsll((long long)badmask);
    float s = lane < n ? dt_j * A_h : 0.f;
    unsigned long long m = lane < n ? (1ull << lane) : 0ull;
    for (int round = 0; round < 6; ++round) {
        if (!__any(p >= 0)) break;
        const int q = p >= 0 ? p : lane;
        const float rs = wave_read(s, q);
        const int rp = wave_read(p, q);
        const unsigned long long rm = wave_read(m, q);
        if (p >= 0) {
            s += rs;
            m |= rm;
            p = rp;
        }
    }
    const float s_k = wave_read(s, k);
    const unsigned long long m_k = wave_read(m, k);
    const bool on = (m_k >> lane) & 1ull;
    pos = on ? __popcll(m_k & ((1ull << lane) - 1ull)) : -1;   // ancestors have smaller labels
    coef = on ? dt_j * __expf(s_k - s) : 0.f;
    len = __popcll(m_k);
    decay = __expf(s_k);
    return 0;
}

}  // namespace stree
