/*
 * CPU oracle for the tree-masked Mamba2 SSD verification pass (STree).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow, fp64
 * statement of what the hot path must compute, written from the paper's
 * definitions.  It shares no code with the HIP library and must never be
 * called from the product path; only tests, the smoke check and the CPU
 * baseline leg of the benchmark use it.
 *
 * What the method computes (Sec. 3 "Formalization" and "Tree decoding with
 * State-space models"): a token tree T packed as t_1..t_N with t_1 the root;
 * every node's output is the output the sequential state-space recurrence
 * (Eq. ssm, in the Mamba2 convention: scalar decay a_t = exp(dt_t * A_h) per
 * head, input term dt_t * x_t (outer) B_t, read-out C_t, skip D_h) would give
 * on the unique root-to-node path, started from the state h0.
 *
 * Functions and what pins them (see tests/test_oracle_*.py):
 *   orc_tree_index        naive parent walking; pinned by the closed forms of a
 *                         full binary tree and by brute-force path sets.
 *   orc_unroll_counts     leaves and unrolled tokens; pinned by the table in
 *                         Fig. "binary-tree" (left) of the paper.
 *   orc_linear_scan       ordinary causal scan of one sequence, no tree code;
 *                         pinned by closed forms (geometric series, dt = 0,
 *                         A -> -inf) and by the lower-triangular matrix form.
 *   orc_ssd_paths         PRIMARY ORACLE: unroll every root-to-leaf path and
 *                         run the sequential recurrence on it; pinned by
 *                         chain == orc_linear_scan (the paper's remark that a
 *                         lower-triangular mask is Mamba2 with a non-zero
 *                         initial state), by the numpy matrix form M_x, M_u
 *                         built from the definitions on every 3..7-node tree,
 *                         by closed forms and by invariants.
 *   orc_ssd_nodes         second formulation: one state per node in
 *                         topological order; must agree with orc_ssd_paths.
 *   orc_tree_conv         depthwise causal conv along each unrolled path;
 *                         pinned by torch.nn.functional.conv1d on the
 *                         concatenated [conv_state ; path] sequence.
 *   orc_commit            state after the accepted path + conv tail; pinned by
 *                         orc_linear_scan on the extracted path and by
 *                         commit-then-continue == grafted tree.
 *   orc_gate_norm         output gate and grouped RMS norm behind the scan (the
 *                         Mamba2 block that the SSM of Sec. 3 sits in; not in
 *                         the paper): pinned by torch's silu and rms_norm, by
 *                         a hand-worked 2 x 4 example and by closed forms.
 *   orc_step_size         step size from the raw projection, softplus(raw +
 *                         bias) (Mamba2's discretisation; the paper leaves the
 *                         step size out): pinned by ln 2 at zero, by
 *                         softplus(v) - softplus(-v) = v, by both tails and by
 *                         torch's softplus.
 *
 * Layouts (all contiguous, fp64 unless noted):
 *   parent int32 [B,N] (root -1, parent[i] < i)    x  [B,N,H,P]
 *   dt [B,N,H]   A [H]   D [H] or NULL             Bm, Cm [B,N,G,S]
 *   h0 [B,H,P,S] or NULL (zero state)              y  [B,N,H,P]
 *   head h reads group g = h / (H/G).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int orc_num_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* tree structure by naive parent walking                              */
/* ------------------------------------------------------------------ */

/* Returns 0 for a valid tree, else (index of the first bad node) + 1.
 * valid: parent[0] == -1 and 0 <= parent[i] < i for i > 0. */
int orc_tree_check(int N, const int32_t *parent) {
    for (int i = 0; i < N; ++i) {
        if (i == 0) {
            if (parent[0] != -1) return 1;
        } else if (parent[i] < 0 || parent[i] >= i) {
            return i + 1;
        }
    }
    return 0;
}

/* depth[i]   = edges from the root to i
 * ancmask    = [N][ceil(N/32)] bit j of row i set iff t_j lies on the path
 *              root..i (the tree mask L_ij, path inclusive of i itself)
 * anc[i][k]  = k-th ancestor of i (anc[i][0] = i), -1 - (k - depth[i] - 1)
 *              ... i.e. negative once the walk leaves the tree: -m means
 *              "m rows before the root" (m = k - depth[i]).
 * ancmask / anc may be NULL. */
int orc_tree_index(int N, const int32_t *parent, int W, int32_t *depth,
                   uint32_t *ancmask, int32_t *anc) {
    int bad = orc_tree_check(N, parent);
    if (bad) return bad;
    int words = (N + 31) / 32;
    if (ancmask) memset(ancmask, 0, sizeof(uint32_t) * (size_t)N * words);
    for (int i = 0; i < N; ++i) {
        int d = 0;
        for (int v = i; v >= 0; v = parent[v]) {
            if (ancmask) ancmask[(size_t)i * words + v / 32] |= (1u << (v % 32));
            if (parent[v] >= 0) ++d;
        }
        depth[i] = d;
        if (anc) {
            int v = i;
            for (int k = 0; k < W; ++k) {
                if (k <= d) {
                    anc[i * W + k] = v;
                    v = parent[v];
                } else {
                    anc[i * W + k] = -(k - d);
                }
            }
        }
    }
    return 0;
}

/* Number of root-to-leaf sequences and total tokens when the tree is unrolled
 * (Fig. "binary-tree", left table: "#. of States" and "Tokens Computed"). */
int orc_unroll_counts(int N, const int32_t *parent, int64_t *n_seq, int64_t *n_tok) {
    int bad = orc_tree_check(N, parent);
    if (bad) return bad;
    char *has_child = (char *)calloc((size_t)N, 1);
    for (int i = 1; i < N; ++i) has_child[parent[i]] = 1;
    int64_t seqs = 0, toks = 0;
    for (int i = 0; i < N; ++i) {
        if (has_child[i]) continue;
        ++seqs;
        for (int v = i; v >= 0; v = parent[v]) ++toks;
    }
    free(has_child);
    *n_seq = seqs;
    *n_tok = toks;
    return 0;
}

/* path root..node, root first; returns its length */
static int root_path(const int32_t *parent, int node, int32_t *path) {
    int len = 0;
    for (int v = node; v >= 0; v = parent[v]) path[len++] = v;
    for (int a = 0, b = len - 1; a < b; ++a, --b) {
        int32_t t = path[a];
        path[a] = path[b];
        path[b] = t;
    }
    return len;
}

/* ------------------------------------------------------------------ */
/* one step of the sequential recurrence (Eq. ssm, Mamba2 convention)  */
/*   h <- exp(dt*A) h + dt * x (outer) B ;  y = h C + D x              */
/* ------------------------------------------------------------------ */
static void ssm_step(int P, int S, double *h, double dt, double A, const double *x,
                     const double *Bv, const double *Cv, double Dh, int hasD, double *y) {
    double a = exp(dt * A);
    for (int p = 0; p < P; ++p) {
        double acc = 0.0;
        for (int s = 0; s < S; ++s) {
            double v = a * h[p * S + s] + dt * x[p] * Bv[s];
            h[p * S + s] = v;
            acc += v * Cv[s];
        }
        if (y) y[p] = acc + (hasD ? Dh * x[p] : 0.0);
    }
}

/* ------------------------------------------------------------------ */
/* ordinary causal scan of B independent sequences of length T         */
/* ------------------------------------------------------------------ */
void orc_linear_scan(int B, int T, int H, int P, int S, int G, const double *x,
                     const double *dt, const double *A, const double *Bm, const double *Cm,
                     const double *D, const double *h0, double *y, double *h_final) {
    int hpg = H / G;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            int g = h / hpg;
            double *st = (double *)malloc(sizeof(double) * (size_t)P * S);
            if (h0) memcpy(st, h0 + ((size_t)b * H + h) * P * S, sizeof(double) * (size_t)P * S);
            else memset(st, 0, sizeof(double) * (size_t)P * S);
            for (int t = 0; t < T; ++t) {
                size_t tok = (size_t)b * T + t;
                ssm_step(P, S, st, dt[tok * H + h], A[h], x + (tok * H + h) * P,
                         Bm + (tok * G + g) * S, Cm + (tok * G + g) * S, D ? D[h] : 0.0, D != NULL,
                         y ? y + (tok * H + h) * P : NULL);
            }
            if (h_final) memcpy(h_final + ((size_t)b * H + h) * P * S, st, sizeof(double) * (size_t)P * S);
            free(st);
        }
    }
}

/* ------------------------------------------------------------------ */
/* PRIMARY: unroll every root-to-leaf path, sequential recurrence      */
/* ------------------------------------------------------------------ */
/* rewrite_diff (may be NULL) receives the largest |difference| seen when a
 * node shared by several unrolled paths is written again (must be 0). */
int orc_ssd_paths(int B, int N, int H, int P, int S, int G, const int32_t *parent,
                  const double *x, const double *dt, const double *A, const double *Bm,
                  const double *Cm, const double *D, const double *h0, double *y,
                  double *rewrite_diff) {
    for (int b = 0; b < B; ++b) {
        int bad = orc_tree_check(N, parent + (size_t)b * N);
        if (bad) return bad;
    }
    int hpg = H / G;
    double worst = 0.0;
#pragma omp parallel for collapse(2) schedule(dynamic) reduction(max : worst)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const int32_t *par = parent + (size_t)b * N;
            int g = h / hpg;
            char *has_child = (char *)calloc((size_t)N, 1);
            char *written = (char *)calloc((size_t)N, 1);
            int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
            double *st = (double *)malloc(sizeof(double) * (size_t)P * S);
            double *yrow = (double *)malloc(sizeof(double) * (size_t)P);
            for (int i = 1; i < N; ++i) has_child[par[i]] = 1;
            for (int leaf = 0; leaf < N; ++leaf) {
                if (has_child[leaf]) continue;
                int len = root_path(par, leaf, path);
                if (h0) memcpy(st, h0 + ((size_t)b * H + h) * P * S, sizeof(double) * (size_t)P * S);
                else memset(st, 0, sizeof(double) * (size_t)P * S);
                for (int t = 0; t < len; ++t) {
                    size_t tok = (size_t)b * N + path[t];
                    ssm_step(P, S, st, dt[tok * H + h], A[h], x + (tok * H + h) * P,
                             Bm + (tok * G + g) * S, Cm + (tok * G + g) * S, D ? D[h] : 0.0,
                             D != NULL, yrow);
                    double *dst = y + (tok * H + h) * P;
                    if (written[path[t]]) {
                        for (int p = 0; p < P; ++p) {
                            double d = fabs(dst[p] - yrow[p]);
                            if (d > worst) worst = d;
                        }
                    }
                    memcpy(dst, yrow, sizeof(double) * (size_t)P);
                    written[path[t]] = 1;
                }
            }
            free(has_child); free(written); free(path); free(st); free(yrow);
        }
    }
    if (rewrite_diff) *rewrite_diff = worst;
    return 0;
}

/* ------------------------------------------------------------------ */
/* second formulation: one state per node, topological order           */
/*   h_i = a_i h_par(i) + dt_i x_i (outer) B_i,  h_par(root) = h0       */
/* ------------------------------------------------------------------ */
int orc_ssd_nodes(int B, int N, int H, int P, int S, int G, const int32_t *parent,
                  const double *x, const double *dt, const double *A, const double *Bm,
                  const double *Cm, const double *D, const double *h0, double *y) {
    for (int b = 0; b < B; ++b) {
        int bad = orc_tree_check(N, parent + (size_t)b * N);
        if (bad) return bad;
    }
    int hpg = H / G;
    size_t PS = (size_t)P * S;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const int32_t *par = parent + (size_t)b * N;
            int g = h / hpg;
            double *states = (double *)malloc(sizeof(double) * PS * (size_t)N);
            for (int i = 0; i < N; ++i) {
                double *hi = states + PS * (size_t)i;
                if (par[i] >= 0) memcpy(hi, states + PS * (size_t)par[i], sizeof(double) * PS);
                else if (h0) memcpy(hi, h0 + ((size_t)b * H + h) * PS, sizeof(double) * PS);
                else memset(hi, 0, sizeof(double) * PS);
                size_t tok = (size_t)b * N + i;
                ssm_step(P, S, hi, dt[tok * H + h], A[h], x + (tok * H + h) * P,
                         Bm + (tok * G + g) * S, Cm + (tok * G + g) * S, D ? D[h] : 0.0, D != NULL,
                         y + (tok * H + h) * P);
            }
            free(states);
        }
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* depthwise causal conv along each unrolled path                      */
/* ------------------------------------------------------------------ */
/* xbc_pre [B,N,Cc]; conv_state [B,W-1,Cc] = the last W-1 pre-conv rows before
 * the root, oldest first; w [Cc,W] with w[c][W-1] multiplying the newest row
 * (standard causal cross-correlation); bias [Cc] or NULL; silu != 0 applies
 * z*sigmoid(z).  For each root-to-leaf path the sequence [conv_state ; path]
 * is convolved; a node on several paths gets the same value on each. */
int orc_tree_conv(int B, int N, int Cc, int W, const int32_t *parent, const double *xbc_pre,
                  const double *conv_state, const double *w, const double *bias, int silu,
                  double *out) {
    for (int b = 0; b < B; ++b) {
        int bad = orc_tree_check(N, parent + (size_t)b * N);
        if (bad) return bad;
    }
#pragma omp parallel for schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        const int32_t *par = parent + (size_t)b * N;
        char *has_child = (char *)calloc((size_t)N, 1);
        int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
        double *seq = (double *)malloc(sizeof(double) * (size_t)(N + W - 1) * Cc);
        for (int i = 1; i < N; ++i) has_child[par[i]] = 1;
        for (int leaf = 0; leaf < N; ++leaf) {
            if (has_child[leaf]) continue;
            int len = root_path(par, leaf, path);
            /* sequence = state rows then the path's rows */
            for (int r = 0; r < W - 1; ++r)
                memcpy(seq + (size_t)r * Cc, conv_state + ((size_t)b * (W - 1) + r) * Cc,
                       sizeof(double) * (size_t)Cc);
            for (int t = 0; t < len; ++t)
                memcpy(seq + (size_t)(W - 1 + t) * Cc, xbc_pre + ((size_t)b * N + path[t]) * Cc,
                       sizeof(double) * (size_t)Cc);
            for (int t = 0; t < len; ++t) {
                double *dst = out + ((size_t)b * N + path[t]) * Cc;
                for (int c = 0; c < Cc; ++c) {
                    double acc = bias ? bias[c] : 0.0;
                    for (int k = 0; k < W; ++k) acc += w[(size_t)c * W + k] * seq[(size_t)(t + k) * Cc + c];
                    dst[c] = silu ? acc / (1.0 + exp(-acc)) : acc;
                }
            }
        }
        free(has_child); free(path); free(seq);
    }
    return 0;
}

/* ------------------------------------------------------------------ */
/* commit: state after the accepted root..k path, and the conv tail     */
/* ------------------------------------------------------------------ */
/* accepted[b] = node id k (whole path root..k accepted) or -1 (keep state).
 * h_out [B,H,P,S]; conv_state_out [B,W-1,Cc] = last W-1 rows of
 * [conv_state ; xbc_pre[path(k)]].  The conv part is skipped when xbc_pre is
 * NULL. */
int orc_commit(int B, int N, int H, int P, int S, int G, int W, int Cc, const int32_t *parent,
               const int32_t *accepted, const double *x, const double *dt, const double *A,
               const double *Bm, const double *h0, double *h_out, const double *xbc_pre,
               const double *conv_state, double *conv_state_out) {
    for (int b = 0; b < B; ++b) {
        int bad = orc_tree_check(N, parent + (size_t)b * N);
        if (bad) return bad;
        if (accepted[b] < -1 || accepted[b] >= N) return -1;
    }
    int hpg = H / G;
    size_t PS = (size_t)P * S;
#pragma omp parallel for collapse(2) schedule(dynamic)
    for (int b = 0; b < B; ++b) {
        for (int h = 0; h < H; ++h) {
            const int32_t *par = parent + (size_t)b * N;
            int g = h / hpg;
            double *st = h_out + ((size_t)b * H + h) * PS;
            if (h0) memcpy(st, h0 + ((size_t)b * H + h) * PS, sizeof(double) * PS);
            else memset(st, 0, sizeof(double) * PS);
            if (accepted[b] < 0) continue;
            int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
            int len = root_path(par, accepted[b], path);
            for (int t = 0; t < len; ++t) {
                size_t tok = (size_t)b * N + path[t];
                ssm_step(P, S, st, dt[tok * H + h], A[h], x + (tok * H + h) * P,
                         Bm + (tok * G + g) * S, Bm + (tok * G + g) * S, 0.0, 0, NULL);
            }
            free(path);
        }
    }
    if (xbc_pre) {
        for (int b = 0; b < B; ++b) {
            const int32_t *par = parent + (size_t)b * N;
            int32_t *path = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
            int len = accepted[b] >= 0 ? root_path(par, accepted[b], path) : 0;
            int total = W - 1 + len;
            for (int r = 0; r < W - 1; ++r) {
                int src = total - (W - 1) + r; /* index into [conv_state ; path rows] */
                const double *row = src < W - 1 ? conv_state + ((size_t)b * (W - 1) + src) * Cc
                                                : xbc_pre + ((size_t)b * N + path[src - (W - 1)]) * Cc;
                memcpy(conv_state_out + ((size_t)b * (W - 1) + r) * Cc, row, sizeof(double) * (size_t)Cc);
            }
            free(path);
        }
    }
    return 0;
}

/*
 * Output gate and grouped RMS norm of the Mamba2 block behind the SSM (not in
 * the paper; the block the scan of Sec. 3 sits in): per node, with the d = H*P
 * channels split into G groups of gs = d / G consecutive channels,
 *   v_c   = y_c * z_c * sigmoid(z_c)                       (gate: y * silu(z))
 *   out_c = v_c / sqrt(mean_{c' in group(c)} v_{c'}^2 + eps) * w_c
 * y, z, out [rows, d]; w [d].  Returns 1 when G does not divide d.
 */
int orc_gate_norm(int rows, int d, int G, const double *y, const double *z, const double *w, double eps,
                  double *out) {
    if (G < 1 || d % G != 0) return 1;
    const int gs = d / G;
#pragma omp parallel for schedule(static)
    for (int r = 0; r < rows; ++r) {
        for (int g = 0; g < G; ++g) {
            const double *yr = y + (size_t)r * d + (size_t)g * gs;
            const double *zr = z + (size_t)r * d + (size_t)g * gs;
            double *o = out + (size_t)r * d + (size_t)g * gs;
            double ss = 0.0;
            for (int c = 0; c < gs; ++c) {
                const double v = yr[c] * (zr[c] / (1.0 + exp(-zr[c])));
                o[c] = v;
                ss += v * v;
            }
            const double scale = 1.0 / sqrt(ss / gs + eps);
            for (int c = 0; c < gs; ++c) o[c] = o[c] * scale * w[g * gs + c];
        }
    }
    return 0;
}

/*
 * Step size of the discretised recurrence from the raw projection (Mamba2
 * practice; the paper's Eq. ssm carries no step size at all): per token and
 * head,
 *   dt = softplus(raw + bias_h) = log(1 + exp(raw + bias_h)),
 * written so that neither tail overflows or cancels.  raw, out [rows, H];
 * bias [H] or NULL (zero).
 */
void orc_step_size(int rows, int H, const double *raw, const double *bias, double *out) {
    for (int r = 0; r < rows; ++r)
        for (int h = 0; h < H; ++h) {
            const double v = raw[(size_t)r * H + h] + (bias ? bias[h] : 0.0);
            out[(size_t)r * H + h] = v > 0.0 ? v + log1p(exp(-v)) : log1p(exp(v));
        }
}
