// C-ABI entry points of libstree: argument validation and kernel dispatch.
// Nothing here computes; every step of the path runs in the HIP kernels.
#include <hip/hip_runtime.h>

#include "../../include/stree.h"
#include "launch.hpp"

namespace {

enum ConvCheck { kNoConv = 0, kConvWidth = 1, kConvChannels = 2 };

int check_dims(const stree_dims *d, int need_conv) {
    if (!d) return STREE_ERR_NULL_ARG;
    if (d->io_dtype != STREE_F32 && d->io_dtype != STREE_BF16) return STREE_ERR_BAD_DTYPE;
    if (d->state_dtype != STREE_F32 && !(d->state_dtype == STREE_BF16 && d->io_dtype == STREE_BF16))
        return STREE_ERR_BAD_DTYPE;                 // (a bf16 state goes with bf16 io only)
    if (d->batch < 0 || d->batch > 65535) return STREE_ERR_BAD_SHAPE;
    if (d->nnodes < 1 || d->nnodes > STREE_MAX_NODES) return STREE_ERR_BAD_SHAPE;
    if (d->nheads < 1 || d->nheads > 65535 || d->ngroups < 1 || d->nheads % d->ngroups != 0)
        return STREE_ERR_BAD_SHAPE;
    if (d->headdim < 1 || d->headdim > 256 || d->dstate < 1 || d->dstate > 256) return STREE_ERR_BAD_SHAPE;
    // the kernels index dt, and the rows of one sequence, with 32-bit offsets
    if ((int64_t)d->batch * d->nnodes * d->nheads > 0x7fffffffLL) return STREE_ERR_BAD_SHAPE;
    if ((int64_t)d->nnodes * ((int64_t)d->nheads * d->headdim + 2 * (int64_t)d->ngroups * d->dstate) > (1LL << 29))
        return STREE_ERR_BAD_SHAPE;
    if (need_conv) {
        if (d->conv_width < 2 || d->conv_width > 4) return STREE_ERR_BAD_SHAPE;
    }
    if (need_conv == kConvChannels) {
        const int cc = d->nheads * d->headdim + 2 * d->ngroups * d->dstate;
        if (cc % (d->io_dtype == STREE_BF16 ? 8 : 4) != 0) return STREE_ERR_BAD_SHAPE;
    }
    return STREE_OK;
}

// fills in dense strides and checks that rows fit
int resolve_strides(stree_dims &d) {
    if (d.x_stride_n == 0) d.x_stride_n = (int64_t)d.nheads * d.headdim;
    if (d.b_stride_n == 0) d.b_stride_n = (int64_t)d.ngroups * d.dstate;
    if (d.c_stride_n == 0) d.c_stride_n = (int64_t)d.ngroups * d.dstate;
    if (d.x_stride_n < (int64_t)d.nheads * d.headdim) return STREE_ERR_BAD_STRIDE;
    if (d.b_stride_n < (int64_t)d.ngroups * d.dstate) return STREE_ERR_BAD_STRIDE;
    if (d.c_stride_n < (int64_t)d.ngroups * d.dstate) return STREE_ERR_BAD_STRIDE;
    // a tree's rows are addressed with 32-bit byte offsets from the sequence's first row (the prefix scan,
    // whose sequences are longer than a tree, uses 64-bit ones)
    const int64_t widest = d.x_stride_n > d.b_stride_n ? (d.x_stride_n > d.c_stride_n ? d.x_stride_n : d.c_stride_n)
                                                       : (d.b_stride_n > d.c_stride_n ? d.b_stride_n : d.c_stride_n);
    if (d.nnodes <= STREE_MAX_NODES && (int64_t)d.nnodes * widest > (1LL << 29)) return STREE_ERR_BAD_STRIDE;
    return STREE_OK;
}

// entry points that read dt: the in-kernel softplus needs its bias vector
bool step_bias_missing(const stree_dims *d) { return (d->flags & STREE_FLAG_DT_SOFTPLUS) && !d->dt_bias; }

// a state kept in bf16 is moved 8 or 16 bytes at a time by every kernel: its arrays start on 16-byte boundaries
bool state_aligned(const stree_dims &d, const void *h0, const void *h_out) {
    return d.state_dtype != STREE_BF16 || (((uintptr_t)h0 | (uintptr_t)h_out) % 16) == 0;
}

int hip_status(hipError_t e) { return e == hipSuccess ? STREE_OK : STREE_ERR_HIP; }

// true when the byte ranges [a, a + na) and [b, b + nb) share a byte
bool ranges_overlap(const void *a, size_t na, const void *b, size_t nb) {
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// bytes spanned by `rows` rows of `row` elements that lie `stride` elements apart
size_t span_bytes(int64_t rows, int64_t stride, int64_t row, size_t elem) {
    return rows > 0 ? (size_t)((rows - 1) * stride + row) * elem : 0;
}

}  // namespace

extern "C" {

int stree_version(void) { return 2; }

size_t stree_workspace_bytes(const stree_dims *dims) {
    // every intermediate of every kernel lives in LDS or registers: no entry point needs device scratch
    return check_dims(dims, kNoConv) == STREE_OK ? 0 : (size_t)-1;
}

int stree_prepare(void) {
    hipError_t e = stree::prepare_tree_ssd_mfma();
    if (e == hipSuccess) e = stree::prepare_tree_ssd_fma();
    return hip_status(e);
}

const char *stree_status_string(int status) {
    switch (status) {
        case STREE_OK: return "ok";
        case STREE_ERR_NULL_ARG: return "a required pointer is NULL";
        case STREE_ERR_BAD_SHAPE: return "a dimension is outside the supported envelope";
        case STREE_ERR_BAD_DTYPE: return "unknown io_dtype or unsupported state_dtype";
        case STREE_ERR_BAD_STRIDE: return "a token stride is smaller than its row";
        case STREE_ERR_HIP: return "a HIP call failed";
        case STREE_ERR_BAD_ALIAS: return "an output overlaps an input that the same call still reads";
    }
    return "unknown status";
}

int stree_tree_index(const stree_dims *dims, const int32_t *parent, int32_t *depth_out,
                     uint32_t *ancmask_out, int32_t *anc_out, int32_t *tree_status, void *hip_stream) {
    int rc = check_dims(dims, anc_out ? kConvWidth : kNoConv);
    if (rc) return rc;
    if (!parent) return STREE_ERR_NULL_ARG;
    if (dims->batch == 0) return STREE_OK;
    return hip_status(stree::launch_tree_index(*dims, parent, depth_out, ancmask_out, anc_out, tree_status,
                                               (hipStream_t)hip_stream));
}

int stree_tree_conv(const stree_dims *dims, const int32_t *parent, const void *xbc_pre,
                    const void *conv_state, const void *conv_w, const void *conv_b, void *xbc_out,
                    int32_t *tree_status, void *hip_stream) {
    int rc = check_dims(dims, kConvChannels);
    if (rc) return rc;
    if (!parent || !xbc_pre || !conv_state || !conv_w || !xbc_out) return STREE_ERR_NULL_ARG;
    if (dims->batch == 0) return STREE_OK;
    return hip_status(stree::launch_tree_conv(*dims, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out,
                                              tree_status, (hipStream_t)hip_stream));
}

int stree_tree_ssd(const stree_dims *dims, const int32_t *parent, const void *x, const float *dt,
                   const float *A, const void *Bm, const void *Cm, const float *D, const void *h0, void *y,
                   int32_t *tree_status, void *hip_stream) {
    int rc = check_dims(dims, kNoConv);
    if (rc) return rc;
    if (!parent || !x || !dt || !A || !Bm || !Cm || !y || step_bias_missing(dims)) return STREE_ERR_NULL_ARG;
    stree_dims d = *dims;
    rc = resolve_strides(d);
    if (rc) return rc;
    if (!state_aligned(d, h0, nullptr)) return STREE_ERR_BAD_SHAPE;
    if (d.batch == 0) return STREE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    if (!(d.flags & STREE_FLAG_FORCE_FMA) && stree::tree_ssd_mfma_supported(d, x, Bm, Cm, h0, y))
        return hip_status(stree::launch_tree_ssd_mfma(d, parent, x, dt, A, Bm, Cm, D, h0, y, tree_status, st));
    return hip_status(stree::launch_tree_ssd_fma(d, parent, x, dt, A, Bm, Cm, D, h0, y, tree_status, st));
}

int stree_commit_state(const stree_dims *dims, const int32_t *parent, const int32_t *accepted, const void *x,
                       const float *dt, const float *A, const void *Bm, const void *h0, void *h_out,
                       const void *xbc_pre, const void *conv_state, void *conv_state_out,
                       int32_t *tree_status, void *hip_stream) {
    const bool conv = xbc_pre || conv_state || conv_state_out;
    int rc = check_dims(dims, conv ? kConvChannels : kNoConv);
    if (rc) return rc;
    const bool no_state = !x && !dt && !A && !Bm && !h0 && !h_out;   // conv tail only
    if (!parent || !accepted) return STREE_ERR_NULL_ARG;
    if (!no_state && (!x || !dt || !A || !Bm || !h_out || step_bias_missing(dims))) return STREE_ERR_NULL_ARG;
    if (no_state && !conv) return STREE_ERR_NULL_ARG;
    if (conv && (!xbc_pre || !conv_state || !conv_state_out)) return STREE_ERR_NULL_ARG;
    if (dims->dstate % 4 != 0) return STREE_ERR_BAD_SHAPE;
    stree_dims d = *dims;
    rc = resolve_strides(d);
    if (rc) return rc;
    if (!state_aligned(d, h0, h_out)) return STREE_ERR_BAD_SHAPE;
    if (d.batch == 0) return STREE_OK;
    return hip_status(stree::launch_commit_state(d, parent, accepted, x, dt, A, Bm, h0, h_out, xbc_pre,
                                                 conv_state, conv_state_out, tree_status,
                                                 (hipStream_t)hip_stream));
}

int stree_tree_ssd_replay(const stree_dims *dims, const stree_replay *prev, const int32_t *parent,
                          const void *x, const float *dt, const float *A, const void *Bm, const void *Cm,
                          const float *D, const void *h0, void *h_out, void *y, int32_t *tree_status,
                          int32_t *replay_status, void *hip_stream) {
    int rc = check_dims(dims, kNoConv);
    if (rc) return rc;
    if (!prev || !prev->parent || !prev->accepted || !prev->x || !prev->dt || !prev->Bm) return STREE_ERR_NULL_ARG;
    if (!parent || !x || !dt || !A || !Bm || !Cm || !y || !h0 || !h_out || step_bias_missing(dims))
        return STREE_ERR_NULL_ARG;
    if (prev->nnodes < 1 || prev->nnodes > STREE_MAX_NODES || dims->dstate % 4 != 0) return STREE_ERR_BAD_SHAPE;
    stree_dims d = *dims;
    rc = resolve_strides(d);
    if (rc) return rc;
    if (!state_aligned(d, h0, h_out)) return STREE_ERR_BAD_SHAPE;
    // the previous tree as a problem of its own: same heads and dtypes, its own node count and strides
    stree_dims dp = *dims;
    dp.nnodes = prev->nnodes;
    dp.x_stride_n = prev->x_stride_n;
    dp.b_stride_n = prev->b_stride_n;
    dp.c_stride_n = 0;
    rc = resolve_strides(dp);
    if (rc) return rc;
    if (d.batch == 0) return STREE_OK;
    hipStream_t st = (hipStream_t)hip_stream;
    if (!(d.flags & STREE_FLAG_FORCE_FMA) && stree::tree_ssd_replay_fused_supported(d, dp, prev->x, prev->Bm, x, Bm, Cm, y, h0, h_out))
        return hip_status(stree::launch_tree_ssd_replay_fused(d, dp, prev->parent, prev->accepted, prev->x, prev->dt,
                                                              prev->Bm, parent, x, dt, A, Bm, Cm, D, h0, h_out, y,
                                                              tree_status, replay_status, st));
    hipError_t e = stree::launch_commit_state(dp, prev->parent, prev->accepted, prev->x, prev->dt, A, prev->Bm, h0,
                                              h_out, nullptr, nullptr, nullptr, replay_status, st);
    if (e != hipSuccess) return STREE_ERR_HIP;
    if (stree::tree_ssd_mfma_supported(d, x, Bm, Cm, h_out, y) && !(d.flags & STREE_FLAG_FORCE_FMA))
        return hip_status(stree::launch_tree_ssd_mfma(d, parent, x, dt, A, Bm, Cm, D, h_out, y, tree_status, st));
    return hip_status(stree::launch_tree_ssd_fma(d, parent, x, dt, A, Bm, Cm, D, h_out, y, tree_status, st));
}

int stree_tree_conv_replay(const stree_dims *dims, const stree_replay *prev, const void *prev_xbc_pre,
                           const int32_t *parent, const void *xbc_pre, const void *conv_state, const void *conv_w,
                           const void *conv_b, void *xbc_out, void *conv_state_out, int32_t *tree_status,
                           int32_t *replay_status, void *hip_stream) {
    int rc = check_dims(dims, kConvChannels);
    if (rc) return rc;
    if (!prev || !prev->parent || !prev->accepted || !prev_xbc_pre) return STREE_ERR_NULL_ARG;
    if (!parent || !xbc_pre || !conv_state || !conv_w || !xbc_out || !conv_state_out) return STREE_ERR_NULL_ARG;
    if (prev->nnodes < 1 || prev->nnodes > STREE_MAX_NODES) return STREE_ERR_BAD_SHAPE;
    if (dims->batch == 0) return STREE_OK;
    return hip_status(stree::launch_tree_conv_replay(*dims, prev->nnodes, prev->parent, prev->accepted, prev_xbc_pre,
                                                     parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out,
                                                     conv_state_out, tree_status, replay_status,
                                                     (hipStream_t)hip_stream));
}

int stree_tree_step(const stree_dims *dims, const stree_replay *prev, const void *prev_xbc_pre,
                    const int32_t *parent, const void *xbc_pre, const void *conv_state, const void *conv_w,
                    const void *conv_b, void *xbc_out, void *conv_state_out, const float *dt, const float *A,
                    const float *D, const void *h0, void *h_out, void *y, int32_t *tree_status,
                    int32_t *replay_status, void *hip_stream) {
    int rc = check_dims(dims, kConvChannels);
    if (rc) return rc;
    if (!prev || !prev->parent || !prev->accepted || !prev->x || !prev->dt || !prev->Bm || !prev_xbc_pre)
        return STREE_ERR_NULL_ARG;
    if (!parent || !xbc_pre || !conv_state || !conv_w || !xbc_out || !conv_state_out) return STREE_ERR_NULL_ARG;
    if (!dt || !A || !h0 || !h_out || !y || step_bias_missing(dims)) return STREE_ERR_NULL_ARG;
    if (prev->nnodes < 1 || prev->nnodes > STREE_MAX_NODES || dims->dstate % 4 != 0) return STREE_ERR_BAD_SHAPE;
    // x, B, C of the scan: column ranges of the conv output
    stree_dims d = *dims;
    const int64_t Cc = (int64_t)d.nheads * d.headdim + 2 * (int64_t)d.ngroups * d.dstate;
    d.x_stride_n = d.b_stride_n = d.c_stride_n = Cc;
    stree_dims dp = *dims;
    dp.nnodes = prev->nnodes;
    dp.x_stride_n = prev->x_stride_n;
    dp.b_stride_n = prev->b_stride_n;
    dp.c_stride_n = 0;
    rc = resolve_strides(dp);
    if (rc) return rc;
    if (!state_aligned(d, h0, h_out)) return STREE_ERR_BAD_SHAPE;      // (before the conv is launched)
    if (d.batch == 0) return STREE_OK;
    {   // the conv overwrites xbc_out before the replay reads the previous step's x / B rows
        const size_t e = d.io_dtype == STREE_BF16 ? 2 : 4;
        const size_t out_bytes = (size_t)d.batch * d.nnodes * (size_t)Cc * e;
        const int64_t prows = (int64_t)d.batch * dp.nnodes;
        if (ranges_overlap(xbc_out, out_bytes, prev->x, span_bytes(prows, dp.x_stride_n, (int64_t)d.nheads * d.headdim, e)) ||
            ranges_overlap(xbc_out, out_bytes, prev->Bm, span_bytes(prows, dp.b_stride_n, (int64_t)d.ngroups * d.dstate, e)))
            return STREE_ERR_BAD_ALIAS;
    }
    rc = stree_tree_conv_replay(dims, prev, prev_xbc_pre, parent, xbc_pre, conv_state, conv_w, conv_b, xbc_out,
                                conv_state_out, tree_status, replay_status, hip_stream);
    if (rc) return rc;
    const size_t e = d.io_dtype == STREE_BF16 ? 2 : 4;
    const char *xo = static_cast<const char *>(xbc_out);
    return stree_tree_ssd_replay(&d, prev, parent, xo, dt, A, xo + (size_t)d.nheads * d.headdim * e,
                                 xo + ((size_t)d.nheads * d.headdim + (size_t)d.ngroups * d.dstate) * e, D, h0, h_out,
                                 y, tree_status, replay_status, hip_stream);
}

int stree_gate_norm(const stree_dims *dims, const void *y, const void *z, int64_t z_stride_n, const void *norm_w,
                    float eps, void *out, void *hip_stream) {
    int rc = check_dims(dims, kNoConv);
    if (rc) return rc;
    if (!y || !z || !norm_w || !out) return STREE_ERR_NULL_ARG;
    const int64_t d = (int64_t)dims->nheads * dims->headdim;
    if (z_stride_n == 0) z_stride_n = d;
    if (z_stride_n < d) return STREE_ERR_BAD_STRIDE;
    if (!(eps >= 0.f)) return STREE_ERR_BAD_SHAPE;
    if ((int64_t)dims->batch * dims->nnodes * dims->ngroups > 0x7fffffffLL) return STREE_ERR_BAD_SHAPE;
    if (dims->batch == 0) return STREE_OK;
    return hip_status(stree::launch_gate_norm(*dims, y, z, (long)z_stride_n, norm_w, eps, out, (hipStream_t)hip_stream));
}

int stree_linear_ssd(const stree_dims *dims, const void *x, const float *dt, const float *A, const void *Bm,
                     const void *Cm, const float *D, const void *h0, void *y, void *h_out, void *hip_stream) {
    if (!dims) return STREE_ERR_NULL_ARG;
    stree_dims d = *dims;
    const int T = d.nnodes;
    d.nnodes = 1;                        // the envelope check of the tree entry points, bar the node limit
    int rc = check_dims(&d, kNoConv);
    if (rc) return rc;
    if (T < 1 || T > (1 << 24)) return STREE_ERR_BAD_SHAPE;
    d.nnodes = T;
    if (!x || !dt || !A || !Bm || !h_out || (y && !Cm) || step_bias_missing(dims)) return STREE_ERR_NULL_ARG;
    rc = resolve_strides(d);
    if (rc) return rc;
    if (!stree::linear_ssd_supported(d, x, Bm, Cm, y, h0, h_out)) return STREE_ERR_BAD_SHAPE;
    if (d.batch == 0) return STREE_OK;
    return hip_status(stree::launch_linear_ssd(d, x, dt, A, Bm, Cm ? Cm : Bm, D, h0, y, h_out,
                                               (hipStream_t)hip_stream));
}

}  // extern "C"
