// stree_gate_norm: output gate and grouped RMS norm of the Mamba2 block behind the tree scan,
//   v   = y * silu(z)
//   out = v / sqrt(mean over the channel group of v^2 + eps) * w
// per node, the H*P channels split into `ngroups` runs of consecutive channels.
//
// Streaming kernel: y and z are read once, out is written once.  A norm group spans the heads of a
// group (all heads when ngroups = 1), i.e. many (batch, head) units of the scan kernels, so the
// step cannot ride on a unit's y store; fused there it would move the z read into the scan and save
// no byte.  One workgroup per (node, group) segment; the gated values stay in registers between the
// sum of squares and the scaling.
#include "common.hpp"
#include "launch.hpp"

namespace stree {

namespace {

template <typename T>
struct Pack16;
template <>
struct Pack16<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4 &v, float (&o)[4]) {
        o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&o)[4]) {
        return make_uint4(__float_as_uint(o[0]), __float_as_uint(o[1]), __float_as_uint(o[2]), __float_as_uint(o[3]));
    }
};
template <>
struct Pack16<bf16_t> {
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

__device__ __forceinline__ float gate(float y, float z) { return y * z * __builtin_amdgcn_rcpf(1.f + __expf(-z)); }

// sum over the workgroup (4 waves); every thread gets the result
__device__ __forceinline__ float block_sum(float v) {
    __shared__ float part[kThreads / 64];
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = v;
    __syncthreads();
    float s = 0.f;
#pragma unroll
    for (int w = 0; w < kThreads / 64; ++w) s += part[w];
    return s;
}

// CPT = 16-byte chunks of a segment per thread (the segment has at most CPT * 256 chunks)
template <typename T, int CPT>
__global__ __launch_bounds__(kThreads) void gate_norm_kernel(const T *__restrict__ y, const T *__restrict__ z, long z_sn,
                                                             const T *__restrict__ w, T *out, int d, int G, int gs,
                                                             float eps) {
    constexpr int EPV = Pack16<T>::N;
    const int row = blockIdx.x / G, g = blockIdx.x % G;
    const size_t oy = (size_t)row * d + (size_t)g * gs, oz = (size_t)row * z_sn + (size_t)g * gs;
    const int chunks = gs / EPV;
    float v[CPT][EPV];
    uint4 ry[CPT], rz[CPT];
#pragma unroll
    for (int q = 0; q < CPT; ++q) {      // every load goes out before anything is waited for
        const int c = min(q * kThreads + (int)threadIdx.x, chunks - 1);
        ry[q] = load_stream16(y + oy + (size_t)c * EPV);
        rz[q] = load_stream16(z + oz + (size_t)c * EPV);
    }
    float ss = 0.f;
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        float fy[EPV], fz[EPV];
        Pack16<T>::unpack(ry[q], fy);
        Pack16<T>::unpack(rz[q], fz);
        const bool live = q * kThreads + (int)threadIdx.x < chunks;
#pragma unroll
        for (int e = 0; e < EPV; ++e) {
            v[q][e] = live ? gate(fy[e], fz[e]) : 0.f;
            ss = fmaf(v[q][e], v[q][e], ss);
        }
    }
    const float scale = rsqrtf(block_sum(ss) / (float)gs + eps);
#pragma unroll
    for (int q = 0; q < CPT; ++q) {
        const int c = q * kThreads + (int)threadIdx.x;
        if (c < chunks) {
            float fw[EPV], o[EPV];
            Pack16<T>::unpack(*reinterpret_cast<const uint4 *>(w + (size_t)g * gs + (size_t)c * EPV), fw);
#pragma unroll
            for (int e = 0; e < EPV; ++e) o[e] = v[q][e] * scale * fw[e];
            store_stream16(out + oy + (size_t)c * EPV, Pack16<T>::pack(o));
        }
    }
}

// any group size, any alignment: two passes over the segment, one element at a time
template <typename T>
__global__ __launch_bounds__(kThreads) void gate_norm_plain_kernel(const T *__restrict__ y, const T *__restrict__ z,
                                                                   long z_sn, const T *__restrict__ w, T *out, int d,
                                                                   int G, int gs, float eps) {
    const int row = blockIdx.x / G, g = blockIdx.x % G;
    const size_t oy = (size_t)row * d + (size_t)g * gs, oz = (size_t)row * z_sn + (size_t)g * gs;
    float ss = 0.f;
    for (int c = threadIdx.x; c < gs; c += kThreads) {
        const float v = gate(to_f32(y[oy + c]), to_f32(z[oz + c]));
        ss = fmaf(v, v, ss);
    }
    const float scale = rsqrtf(block_sum(ss) / (float)gs + eps);
    for (int c = threadIdx.x; c < gs; c += kThreads) {
        const float v = gate(to_f32(y[oy + c]), to_f32(z[oz + c]));
        T o;
        from_f32(v * scale * to_f32(w[(size_t)g * gs + c]), o);
        out[oy + c] = o;
    }
}

template <typename T>
hipError_t launch_t(const stree_dims &d, const void *y, const void *z, long z_sn, const void *w, float eps, void *out,
                    hipStream_t st) {
    constexpr int EPV = Pack16<T>::N;
    const int dd = d.nheads * d.headdim, G = d.ngroups, gs = dd / G;
    const long rows = (long)d.batch * d.nnodes;
    const dim3 grid((unsigned)(rows * G));
    const bool vec = gs % EPV == 0 && z_sn % EPV == 0 &&
                     (((uintptr_t)y | (uintptr_t)z | (uintptr_t)w | (uintptr_t)out) % 16) == 0;
    const int cpt = vec ? (gs / EPV + kThreads - 1) / kThreads : 0;
#define STREE_GN_LAUNCH(K)                                                                                        \
    hipLaunchKernelGGL(K, grid, dim3(kThreads), 0, st, (const T *)y, (const T *)z, z_sn, (const T *)w, (T *)out, dd, G, \
                       gs, eps)
    if (cpt == 1) STREE_GN_LAUNCH((gate_norm_kernel<T, 1>));
    else if (cpt == 2) STREE_GN_LAUNCH((gate_norm_kernel<T, 2>));
    else if (cpt == 3) STREE_GN_LAUNCH((gate_norm_kernel<T, 3>));
    else if (cpt == 4) STREE_GN_LAUNCH((gate_norm_kernel<T, 4>));
    else STREE_GN_LAUNCH((gate_norm_plain_kernel<T>));
#undef STREE_GN_LAUNCH
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gate_norm(const stree_dims &d, const void *y, const void *z, long z_sn, const void *w, float eps,
                            void *out, hipStream_t st) {
    if (d.io_dtype == STREE_BF16) return launch_t<bf16_t>(d, y, z, z_sn, w, eps, out, st);
    return launch_t<float>(d, y, z, z_sn, w, eps, out, st);
}

}  // namespace stree
