/*
 * libstree: tree-masked Mamba2 SSD verification pass for AMD MI355X (gfx950).
 *
 * One call scores a token tree that is packed into a sequence t_1..t_N (t_1 the
 * root) and described by a parent-index array, the compact form of the paper's
 * tree mask L (Sec. 3 "Formalization": L_ij = 1 iff t_j lies on the path from
 * the root to t_i, the path including t_i itself).
 *
 * C ABI, plain pointers and sizes.  Conventions for every entry point:
 *   - `dims` is HOST memory.  Every other pointer is DEVICE memory owned by the
 *     caller; the library never allocates, frees or synchronises.
 *   - All work is enqueued on `hip_stream` (a hipStream_t passed as void*; NULL
 *     is the default stream).  Outputs are fully overwritten; inputs are never
 *     written (except where aliasing is explicitly allowed below).
 *   - Return value: STREE_OK (0) or a host-detected error (> 0), in which case
 *     nothing was launched.
 *   - Trees are validated on the device: parent[b,0] == -1 and
 *     0 <= parent[b,i] < i.  Per sequence, `tree_status[b]` (may be NULL) gets 0,
 *     or (index of the first bad node) + 1, and that sequence's outputs are
 *     zero-filled (commit: state copied through unchanged).
 *   - Layouts are row-major with the last index contiguous.  Head h reads group
 *     g = h / (nheads / ngroups).  dt, A, D are always fp32; the SSM state (h0, h_out:
 *     "st" below) is fp32, or bf16 with state_dtype = STREE_BF16;
 *     `io_dtype` selects fp32 or bf16 for x, B, C, y and the conv tensors.
 *   - Envelope: 1 <= nnodes <= 256, batch >= 0 (0 is a no-op), nheads % ngroups
 *     == 0, 1 <= headdim <= 256, 1 <= dstate <= 256, conv_width in {2,3,4};
 *     batch * nnodes * nheads < 2^31 and nnodes * (token stride) <= 2^29 elements
 *     (32-bit offsets inside the kernels).
 *     An MFMA kernel is used when io_dtype is bf16, headdim in {32,64,128},
 *     dstate % 16 == 0 and pointers/strides are 16-byte aligned; every other
 *     case in the envelope runs a plain fp32-FMA kernel.  Among the MFMA
 *     shapes, the persistent kernels (the ones the benchmark prices) take
 *     headdim 64 with dstate 64, 128 or 256, and headdim 128 with dstate 128,
 *     at any node count; the remaining MFMA shapes (headdim 32, other dstates,
 *     ...) run one workgroup per (sequence, head) and are several times slower
 *     per node.  Results are the same to rounding on every route.
 */
#ifndef STREE_H
#define STREE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define STREE_MAX_NODES 256

enum stree_status {
    STREE_OK = 0,
    STREE_ERR_NULL_ARG = 1,   /* a required pointer is NULL */
    STREE_ERR_BAD_SHAPE = 2,  /* a dimension is outside the envelope */
    STREE_ERR_BAD_DTYPE = 3,  /* unknown io_dtype / unsupported state_dtype */
    STREE_ERR_BAD_STRIDE = 4, /* a token stride is smaller than its row */
    STREE_ERR_HIP = 5,        /* a HIP launch failed */
    STREE_ERR_BAD_ALIAS = 6   /* an output overlaps an input that the same call still reads */
};

enum stree_dtype { STREE_F32 = 0, STREE_BF16 = 1 };

enum stree_flags {
    STREE_FLAG_CONV_SILU = 1,    /* tree_conv applies z * sigmoid(z) */
    STREE_FLAG_DT_SOFTPLUS = 2,  /* every `dt` argument (and prev->dt) holds the RAW projection; the kernels use
                                    softplus(dt + dt_bias[h]) as the step size (see stree_dims.dt_bias) */
    STREE_FLAG_FORCE_FMA = 256,    /* tree_ssd: use the plain fp32-FMA kernel even where MFMA applies */
    STREE_FLAG_GENERAL_MFMA = 1024 /* tree_ssd: trees of more than 64 nodes take the one-workgroup-per-(b,h) MFMA
                                      kernel even where the persistent one applies (same results to rounding) */
};

/* Problem sizes.  POD, host memory. */
typedef struct stree_dims {
    int32_t batch;       /* B sequences, each with its own tree of exactly nnodes nodes */
    int32_t nnodes;      /* N */
    int32_t nheads;      /* H */
    int32_t headdim;     /* P */
    int32_t dstate;      /* S */
    int32_t ngroups;     /* G */
    int32_t conv_width;  /* W (ignored by tree_ssd; 0 allowed there) */
    int32_t io_dtype;    /* enum stree_dtype */
    int32_t state_dtype; /* type of h0 / h_out: STREE_F32, or STREE_BF16 (only with io_dtype = STREE_BF16).
                          * A bf16 state is widened exactly when read, all arithmetic stays fp32, and a new
                          * state is rounded to nearest even once, when written: every iteration adds that
                          * rounding (at most 2^-8 relative) to the state -- the caller's trade for half the traffic.
                          * bf16 state arrays start on 16-byte boundaries (STREE_ERR_BAD_SHAPE otherwise). */
    int32_t flags;       /* enum stree_flags */
    /* token strides in ELEMENTS of x, B, C (0 = dense: H*P, G*S, G*S).  They let
     * x | B | C be column ranges of one conv output buffer [B,N,H*P+2*G*S].  The
     * batch stride is nnodes * token stride. */
    int64_t x_stride_n, b_stride_n, c_stride_n;
    /* DEVICE pointer, f32 [H]: the per-head bias in front of the softplus.  Read only when
     * STREE_FLAG_DT_SOFTPLUS is set, and required then by every entry point that takes dt
     * (STREE_ERR_NULL_ARG otherwise); pass zeros
     * for a plain softplus.  The paper's Eq. ssm has no step size; this is Mamba2's discretisation,
     * dt = log(1 + exp(raw + bias_h)), evaluated in fp32 where dt is loaded (values above 20 pass
     * through, the difference being below fp32 resolution).  Without the flag `dt` is the step size itself. */
    const float *dt_bias;
} stree_dims;

int stree_version(void);
const char *stree_status_string(int status);

/*
 * Optional set-up for callers that capture the entry points into a HIP graph (or cannot afford a slow
 * first call).  Two of the kernels -- the one-workgroup-per-(sequence, head) MFMA kernel and the fp32-FMA
 * kernel, i.e. the shapes outside the persistent kernels -- need more dynamic LDS than the default limit
 * and raise it with hipFuncSetAttribute at their first launch that needs it.  This call raises every such
 * limit at once, on the CURRENT device (call it once per device used): afterwards no entry point calls
 * anything but kernel launches.  Launches nothing, allocates nothing.  Returns STREE_OK or STREE_ERR_HIP.
 */
int stree_prepare(void);

/*
 * Device scratch that the entry points below would need for a problem of these sizes
 * (the problem statement of Sec. 3 "Formalization" fixes the operands; this call sizes
 * what the library needs beyond them).  Every intermediate of every kernel -- the tree
 * index, the decay-weighted mask, the state tile -- lives in LDS or registers, so the
 * answer is 0 for every valid `dims`, and no entry point takes a workspace argument.
 * Invalid `dims` (NULL, unknown dtype, a dimension outside the envelope) return
 * (size_t)-1.  conv_width and flags are not looked at.  Launches nothing.
 */
size_t stree_workspace_bytes(const stree_dims *dims);

/*
 * Tree structure (the tree mask L of Sec. 3 "Formalization", in index form).
 *   parent     int32 [B,N]
 *   depth_out  int32 [B,N]               edges from the root            (or NULL)
 *   ancmask_out uint32 [B,N,ceil(N/32)]  bit j of row i = L_ij          (or NULL)
 *   anc_out    int32 [B,N,W]             k-th ancestor of i for k < W = conv_width,
 *                                        k = 0 is i itself; once the walk leaves the
 *                                        tree the entry is -m, "m rows above the
 *                                        root" (m = k - depth)          (or NULL)
 * Results are exact integers.
 */
int stree_tree_index(const stree_dims *dims, const int32_t *parent, int32_t *depth_out,
                     uint32_t *ancmask_out, int32_t *anc_out, int32_t *tree_status,
                     void *hip_stream);

/*
 * Depthwise causal conv1d taken along each node's ancestor chain (the Mamba2
 * block's conv in front of the SSM, applied to the packed tree of Sec. 3):
 *   out[b,i,c] = act( bias[c] + sum_{k=0}^{W-1} w[c,W-1-k] * src(i,k)[c] )
 * where src(i,k) is the pre-conv row of the k-th ancestor of i, or, above the
 * root, row (W-1) - (k - depth(i)) of conv_state.
 *   xbc_pre    io [B,N,Cc], Cc = H*P + 2*G*S
 *   conv_state io [B,W-1,Cc]  last W-1 pre-conv rows before the root, oldest first
 *   conv_w     io [Cc,W]      conv_w[c,W-1] multiplies the node's own row
 *   conv_b     io [Cc] or NULL
 *   xbc_out    io [B,N,Cc]    must not alias xbc_pre
 * Accumulation is fp32.  Cc must be a multiple of 8 (bf16) or 4 (fp32).
 */
int stree_tree_conv(const stree_dims *dims, const int32_t *parent, const void *xbc_pre,
                    const void *conv_state, const void *conv_w, const void *conv_b,
                    void *xbc_out, int32_t *tree_status, void *hip_stream);

/*
 * Tree scan (Sec. 3 "Tree decoding with State-space models"; Eq. a_tree and the
 * matrix form y = M_x x0 + M_u u):
 *   s_i  = sum_{j on path(i)} dt[j] * A[h]                        (A_tree)
 *   y_i  = exp(s_i) * h0 C_i
 *        + sum_{j on path(i)} exp(s_i - s_j) * dt[j] * <C_i,B_j> * x_j
 *        + D[h] * x_i
 *   x   io  [B,N,H,P] (token stride x_stride_n)    dt  f32 [B,N,H]: the step size (>= 0), or, with
 *                                                  STREE_FLAG_DT_SOFTPLUS, the raw projection
 *   A   f32 [H], negative                          Bm, Cm io [B,N,G,S] (strides b/c_stride_n)
 *   D   f32 [H] or NULL                            h0  st  [B,H,P,S] or NULL (zero state)
 *   y   io  [B,N,H,P] dense
 * bf16 mode: products on the bf16 MFMA units with fp32 accumulation; the state
 * and the decay-weighted mask are rounded to bf16 as MFMA operands.
 */
int stree_tree_ssd(const stree_dims *dims, const int32_t *parent, const void *x, const float *dt,
                   const float *A, const void *Bm, const void *Cm, const float *D,
                   const void *h0, void *y, int32_t *tree_status, void *hip_stream);

/*
 * State commit (the "activation replay" of Sec. 3 "Implementation" / Alg. 1: the
 * state after the last accepted token is recomputed from the cached x, dt, B of
 * the tree that was just verified).  For accepted node k = accepted[b]:
 *   h_out = exp(s_k) * h0 + sum_{j on path(k)} exp(s_k - s_j) * dt[j] * x_j (outer) B_j
 *   conv_state_out = last W-1 rows of [conv_state ; xbc_pre[path(k)]]
 * accepted[b] == -1 copies the state through.  An accepted index outside
 * [-1, N) sets tree_status[b] = -1 and copies the state through.
 *   accepted int32 [B]; x, dt, A, Bm as in stree_tree_ssd
 *   h0 st [B,H,P,S] or NULL; h_out st [B,H,P,S], MAY alias h0
 *   xbc_pre, conv_state, conv_state_out: all three NULL to skip the conv part;
 *   conv_state_out MAY alias conv_state.
 *   x, dt, A, Bm, h0, h_out: all six NULL to skip the state part (conv tail only,
 *   as used in front of stree_tree_ssd_replay).
 * dstate must be a multiple of 4.
 */
int stree_commit_state(const stree_dims *dims, const int32_t *parent, const int32_t *accepted,
                       const void *x, const float *dt, const float *A, const void *Bm,
                       const void *h0, void *h_out, const void *xbc_pre,
                       const void *conv_state, void *conv_state_out, int32_t *tree_status,
                       void *hip_stream);

/*
 * The previous iteration's tree and its cached activations: what Alg. 1 keeps so
 * that the state can be replayed at the start of the next iteration.  POD, host
 * memory; the pointers in it are device memory.  Batch, heads, headdim, dstate,
 * groups and io_dtype are those of the `dims` it is passed with.
 */
typedef struct stree_replay {
    int32_t nnodes;           /* nodes of the previous tree, 1..STREE_MAX_NODES */
    int32_t reserved;         /* 0 */
    const int32_t *parent;    /* int32 [B,nnodes] */
    const int32_t *accepted;  /* int32 [B]: accepted node of the previous tree, -1 = none */
    const void *x;            /* io [B,nnodes,H,P], token stride x_stride_n */
    const float *dt;          /* f32 [B,nnodes,H] */
    const void *Bm;           /* io [B,nnodes,G,S], token stride b_stride_n */
    int64_t x_stride_n, b_stride_n; /* elements; 0 = dense */
} stree_replay;

/*
 * Fused activation replay and tree scan (Alg. 1, "replay at the start of the next
 * iteration"; Sec. 3 "Implementation"): one pass over the state that does what
 * stree_commit_state on the previous tree followed by stree_tree_ssd on the
 * current tree would do, reading the state once instead of twice:
 *   h_out = state after the accepted path of `prev` starting from h0   (commit formula)
 *   y     = tree scan of the current tree starting from h_out          (scan formula)
 *   h0    st [B,H,P,S], required; h_out st [B,H,P,S], required, MAY alias h0
 *   replay_status int32 [B] or NULL: 0, (first bad node of the previous tree) + 1,
 *                 or -1 for an accepted index outside [-1, prev->nnodes); in the
 *                 last two cases the state passes through unchanged
 *   every other argument as in stree_tree_ssd; A is shared by both trees.
 * The single-pass kernel covers the shapes of a decoding step (both trees of at
 * most 64 nodes, bf16, the MFMA head shapes); every other shape in the envelope
 * runs the two separate kernels back to back on the stream, with the same result.
 * dstate must be a multiple of 4.
 */
int stree_tree_ssd_replay(const stree_dims *dims, const stree_replay *prev, const int32_t *parent,
                          const void *x, const float *dt, const float *A, const void *Bm,
                          const void *Cm, const float *D, const void *h0, void *h_out, void *y,
                          int32_t *tree_status, int32_t *replay_status, void *hip_stream);

/*
 * Tree conv with the conv-state part of the previous tree's commit folded in (the
 * replay of Alg. 1 applied to the conv in front of the SSM): the rows above the
 * root are taken from
 *   conv_state* = last W-1 rows of [conv_state ; prev_xbc_pre[path(accepted)]]
 * instead of conv_state, and conv_state* is written to conv_state_out.  Equal to
 * stree_commit_state (conv part) on the previous tree followed by stree_tree_conv.
 *   prev           only nnodes, parent and accepted are read
 *   prev_xbc_pre   io [B, prev->nnodes, Cc]  pre-conv rows of the previous tree
 *   conv_state_out io [B,W-1,Cc], must NOT alias conv_state
 *   replay_status  as in stree_tree_ssd_replay (the state passes through on error)
 *   every other argument as in stree_tree_conv.
 */
int stree_tree_conv_replay(const stree_dims *dims, const stree_replay *prev, const void *prev_xbc_pre,
                           const int32_t *parent, const void *xbc_pre, const void *conv_state,
                           const void *conv_w, const void *conv_b, void *xbc_out, void *conv_state_out,
                           int32_t *tree_status, int32_t *replay_status, void *hip_stream);

/*
 * One decoding step of the layer behind one call: stree_tree_conv_replay followed by
 * stree_tree_ssd_replay on the column ranges of its output (Sec. 3: tree conv, tree
 * scan; Alg. 1: replay at the start of the next iteration), with the same results:
 *   xbc_out        io [B,N,Cc]: conv output; x = columns [0, H*P), B = the next G*S,
 *                  C = the last G*S, each with token stride Cc (the strides in dims
 *                  are ignored)
 *   conv_state_out io [B,W-1,Cc], must NOT alias conv_state
 *   h_out          st [B,H,P,S], MAY alias h0;   y io [B,N,H,P] dense
 *   prev           the previous tree; prev->x and prev->Bm are the x and B columns of
 *                  the previous step's xbc_out (strides in prev), prev_xbc_pre its
 *                  pre-conv rows [B, prev->nnodes, Cc]
 *   tree_status, replay_status  as in stree_tree_ssd_replay
 * xbc_out must NOT overlap prev->x or prev->Bm: the conv overwrites xbc_out before the
 * replay reads the previous step's rows, so a caller that ping-pongs conv outputs needs
 * two buffers.  The overlap is detected on the host and returns STREE_ERR_BAD_ALIAS
 * with nothing launched.  (The same holds for a caller that makes the two calls itself;
 * there the library cannot see it.)
 * The two kernels run back to back on the stream.  A single kernel that also convolves
 * was built and measured on MI355X at 1.5 x the time of the two (every workgroup has to
 * redo the B / C columns of its group, or wait for another workgroup of the same launch):
 * it is not part of the library.
 */
int stree_tree_step(const stree_dims *dims, const stree_replay *prev, const void *prev_xbc_pre,
                    const int32_t *parent, const void *xbc_pre, const void *conv_state,
                    const void *conv_w, const void *conv_b, void *xbc_out, void *conv_state_out,
                    const float *dt, const float *A, const float *D, const void *h0, void *h_out,
                    void *y, int32_t *tree_status, int32_t *replay_status, void *hip_stream);

/*
 * Output gate and grouped RMS norm behind the scan (the Mamba2 block that the SSM of
 * Sec. 3 sits in -- Eq. in_proj names its projections; the paper does not print the
 * gate and the norm, they follow public Mamba2 practice): per node, the d = H*P
 * channels of y split into ngroups runs of d / ngroups consecutive channels,
 *   v   = y * z * sigmoid(z)
 *   out = v / sqrt(mean over the channel's group of v^2 + eps) * norm_w
 *   y      io [B,N,H,P] dense: the scan's output
 *   z      io [B,N,H,P] with token stride z_stride_n elements (0 = dense), so that z may
 *          be a column range of the input projection's output
 *   norm_w io [H*P];  eps >= 0
 *   out    io [B,N,H,P] dense, MAY alias y
 * fp32 arithmetic, one rounding of the result.  16-byte aligned pointers, a stride and a
 * group size that are multiples of 8 (bf16) or 4 (fp32) elements, and groups of at most
 * 8192 (bf16) / 4096 (fp32) channels take the single-pass kernel (y and z read once);
 * anything else a plain two-pass kernel with the same result.  No tree is involved, so
 * there is no tree_status.
 */
int stree_gate_norm(const stree_dims *dims, const void *y, const void *z, int64_t z_stride_n,
                    const void *norm_w, float eps, void *out, void *hip_stream);

/*
 * Linear prefix scan: the ordinary causal Mamba2 scan of T tokens per sequence (the
 * chain case of the tree mask, Sec. 3: a lower-triangular L is Mamba2 with an
 * initial state), chunked, with the state carried from chunk to chunk on chip.  It
 * is the prefix pass in front of tree decoding: the state it returns seeds
 * stree_tree_ssd.
 *   dims->nnodes = T, any T >= 1 (not limited to STREE_MAX_NODES); conv_width ignored
 *   x, dt, A, Bm, Cm, D, h0 as in stree_tree_ssd with T in place of N
 *   y      io [B,T,H,P] or NULL: state only (then Cm and D may be NULL too)
 *   h_out  st [B,H,P,S] state after token T-1, required, MAY alias h0
 * Shapes: bf16 io, (headdim, dstate) in {(64,64), (64,128), (64,256), (128,128)}, 16-byte
 * aligned pointers and strides; anything else returns STREE_ERR_BAD_SHAPE
 * (a chain tree through stree_tree_ssd / stree_commit_state covers it, 256
 * tokens at a time).  The state is carried in fp32 (the weighted inputs enter
 * the matrix units as two bf16 terms, value and rounding remainder: the state
 * after 4096 tokens is within 1e-4 of an fp64 scan); only its use in y is
 * rounded to bf16.
 */
int stree_linear_ssd(const stree_dims *dims, const void *x, const float *dt, const float *A,
                     const void *Bm, const void *Cm, const float *D, const void *h0, void *y,
                     void *h_out, void *hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* STREE_H */
