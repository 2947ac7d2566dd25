// Host-side launchers, one per kernel family.  Arguments are already validated
// by the C-ABI layer (api.hip); strides are resolved (never 0).
#pragma once
#include <hip/hip_runtime.h>

#include <mutex>

#include "../../include/stree.h"

namespace stree {

// the per-head bias of the in-kernel softplus, or null when `dt` already holds step sizes
inline const float *step_bias(const stree_dims &d) {
    return (d.flags & STREE_FLAG_DT_SOFTPLUS) ? d.dt_bias : nullptr;
}

// The dynamic-LDS limit of one kernel (64 KB unless raised), raised on demand with hipFuncSetAttribute.
// The limit only ever grows, under a lock, so a launch from another host thread never finds it lowered;
// it is tracked per device, each device holding its own copy of the kernel and of its attributes.
struct LdsLimit {
    static constexpr int kDevices = 64;
    std::mutex mu;
    size_t set[kDevices] = {};
    hipError_t raise(const void *kernel, size_t bytes) {
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= kDevices) return hipErrorInvalidDevice;
        std::lock_guard<std::mutex> hold(mu);
        if (bytes > set[dev]) {
            e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
            if (e != hipSuccess) return e;
            set[dev] = bytes;
        }
        return hipSuccess;
    }
};

// raise, on the current device, every limit that a launcher below would otherwise raise at its first launch
hipError_t prepare_tree_ssd_mfma();
hipError_t prepare_tree_ssd_fma();

hipError_t launch_tree_index(const stree_dims &d, const int32_t *parent, int32_t *depth_out,
                             uint32_t *mask_out, int32_t *anc_out, int32_t *status, hipStream_t st);

hipError_t launch_tree_conv(const stree_dims &d, const int32_t *parent, const void *xbc_pre,
                            const void *conv_state, const void *conv_w, const void *conv_b, void *xbc_out,
                            int32_t *status, hipStream_t st);

// conv with the conv-tail update of the previous tree's commit folded in
hipError_t launch_tree_conv_replay(const stree_dims &d, int prev_nnodes, const int32_t *prev_parent,
                                   const int32_t *prev_accepted, const void *prev_xbc_pre, const int32_t *parent,
                                   const void *xbc_pre, const void *conv_state, const void *conv_w,
                                   const void *conv_b, void *xbc_out, void *conv_state_out, int32_t *status,
                                   int32_t *replay_status, hipStream_t st);

hipError_t launch_tree_ssd_fma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                               const float *A, const void *Bm, const void *Cm, const float *D,
                               const void *h0, void *y, int32_t *status, hipStream_t st);

// true when the MFMA kernel covers these dims / alignments
bool tree_ssd_mfma_supported(const stree_dims &d, const void *x, const void *Bm, const void *Cm,
                             const void *h0, const void *y);
hipError_t launch_tree_ssd_mfma(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                const float *A, const void *Bm, const void *Cm, const float *D,
                                const void *h0, void *y, int32_t *status, hipStream_t st);

// single node block (n <= 64), persistent and software-pipelined
bool tree_ssd_mfma64_supported(const stree_dims &d);
hipError_t launch_tree_ssd_mfma64(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D,
                                  const void *h0, void *y, int32_t *status, hipStream_t st);

// 65 .. 256 nodes: the persistent kernel over (row block, column block) pairs
bool tree_ssd_blocks_supported(const stree_dims &d);
hipError_t launch_tree_ssd_blocks(const stree_dims &d, const int32_t *parent, const void *x, const float *dt,
                                  const float *A, const void *Bm, const void *Cm, const float *D, const void *h0,
                                  void *y, int32_t *status, hipStream_t st);

// fused replay + scan: `dp` describes the previous tree (its node count and strides)
bool tree_ssd_replay_fused_supported(const stree_dims &d, const stree_dims &dp, const void *px, const void *pB,
                                     const void *x, const void *Bm, const void *Cm, const void *y, const void *h0,
                                     const void *h_out);
hipError_t launch_tree_ssd_replay_fused(const stree_dims &d, const stree_dims &dp, const int32_t *pparent,
                                        const int32_t *paccepted, const void *px, const float *pdt, const void *pB,
                                        const int32_t *parent, const void *x, const float *dt, const float *A,
                                        const void *Bm, const void *Cm, const float *D, const void *h0,
                                        void *h_out, void *y, int32_t *status, int32_t *rstatus, hipStream_t st);

// chunked causal scan of a long sequence (d.nnodes = T tokens)
bool linear_ssd_supported(const stree_dims &d, const void *x, const void *Bm, const void *Cm, const void *y,
                          const void *h0, const void *h_out);
hipError_t launch_linear_ssd(const stree_dims &d, const void *x, const float *dt, const float *A, const void *Bm,
                             const void *Cm, const float *D, const void *h0, void *y, void *h_out, hipStream_t st);

// output gate + grouped RMS norm behind the scan; z_sn = token stride of z in elements
hipError_t launch_gate_norm(const stree_dims &d, const void *y, const void *z, long z_sn, const void *w, float eps,
                            void *out, hipStream_t st);

// h_out == NULL: conv tail only
hipError_t launch_commit_state(const stree_dims &d, const int32_t *parent, const int32_t *accepted,
                               const void *x, const float *dt, const float *A, const void *Bm,
                               const void *h0, void *h_out, const void *xbc_pre, const void *conv_state,
                               void *conv_state_out, int32_t *status, hipStream_t st);

}  // namespace stree
