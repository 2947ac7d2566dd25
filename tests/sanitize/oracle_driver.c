/* Exercises every routine of the CPU oracle on small deterministic inputs.  Built by
 * tests/test_sanitizers.py together with oracle/stree_oracle.c under
 * -fsanitize=address,undefined: the run must end without a sanitizer report. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

int orc_tree_check(int N, const int32_t *parent);
int orc_tree_index(int N, const int32_t *parent, int W, int32_t *depth, uint32_t *mask, int32_t *anc);
int orc_unroll_counts(int N, const int32_t *parent, int64_t *n_seq, int64_t *n_tok);
void orc_linear_scan(int B, int T, int H, int P, int S, int G, const double *x, const double *dt, const double *A,
                     const double *Bm, const double *Cm, const double *D, const double *h0, double *y, double *h_out);
int orc_ssd_paths(int B, int N, int H, int P, int S, int G, const int32_t *parent, const double *x, const double *dt,
                  const double *A, const double *Bm, const double *Cm, const double *D, const double *h0, double *y,
                  double *rewrite_diff);
int orc_ssd_nodes(int B, int N, int H, int P, int S, int G, const int32_t *parent, const double *x, const double *dt,
                  const double *A, const double *Bm, const double *Cm, const double *D, const double *h0, double *y);
int orc_tree_conv(int B, int N, int Cc, int W, const int32_t *parent, const double *xbc_pre, const double *conv_state,
                  const double *w, const double *bias, int silu, double *out);
int orc_commit(int B, int N, int H, int P, int S, int G, int W, int Cc, const int32_t *parent, const int32_t *accepted,
               const double *x, const double *dt, const double *A, const double *Bm, const double *h0, double *h_out,
               const double *xbc_pre, const double *conv_state, double *cs_out);
int orc_gate_norm(int rows, int d, int G, const double *y, const double *z, const double *w, double eps, double *out);

static uint64_t lcg = 88172645463325252ull;
static double rnd(void) {                      /* uniform in (-1, 1) */
    lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
    return ((double)(lcg >> 11) / 9007199254740992.0) * 2.0 - 1.0;
}
static double *vec(size_t n, double scale, double shift) {
    double *p = malloc(n * sizeof *p);
    for (size_t i = 0; i < n; ++i) p[i] = rnd() * scale + shift;
    return p;
}

static int run(int B, int N, int H, int P, int S, int G, int W) {
    const int Cc = H * P + 2 * G * S;
    int32_t *parent = malloc((size_t)B * N * sizeof *parent), *acc = malloc(B * sizeof *acc);
    for (int b = 0; b < B; ++b) {
        parent[b * N] = -1;
        for (int i = 1; i < N; ++i) {
            lcg = lcg * 6364136223846793005ull + 1442695040888963407ull;
            parent[b * N + i] = (b == 0) ? i - 1 : (int32_t)((lcg >> 33) % (uint64_t)i);   /* a chain, then random trees */
        }
        acc[b] = (b % 3 == 2) ? -1 : (N - 1 - b % N + N) % N;
    }
    double *x = vec((size_t)B * N * H * P, 1, 0), *dt = vec((size_t)B * N * H, 0.2, 0.25), *A = vec(H, 1, -2),
           *Bm = vec((size_t)B * N * G * S, 1, 0), *Cm = vec((size_t)B * N * G * S, 1, 0), *D = vec(H, 1, 0),
           *h0 = vec((size_t)B * H * P * S, 0.1, 0);
    double *y1 = vec((size_t)B * N * H * P, 0, 0), *y2 = vec((size_t)B * N * H * P, 0, 0), diff = 0;
    int bad = 0;
    for (int b = 0; b < B; ++b) bad |= orc_tree_check(N, parent + b * N);
    int32_t *depth = malloc(N * sizeof *depth), *anc = malloc((size_t)N * 4 * sizeof *anc);
    uint32_t *mask = calloc((size_t)N * ((N + 31) / 32), sizeof *mask);
    bad |= orc_tree_index(N, parent + (B - 1) * N, W > 1 ? W : 4, depth, mask, anc);
    int64_t ns, nt;
    bad |= orc_unroll_counts(N, parent, &ns, &nt);
    bad |= orc_ssd_paths(B, N, H, P, S, G, parent, x, dt, A, Bm, Cm, D, h0, y1, &diff);
    bad |= orc_ssd_nodes(B, N, H, P, S, G, parent, x, dt, A, Bm, Cm, NULL, NULL, y2);
    double *yl = vec((size_t)B * N * H * P, 0, 0), *hl = vec((size_t)B * H * P * S, 0, 0);
    orc_linear_scan(B, N, H, P, S, G, x, dt, A, Bm, Cm, D, h0, yl, hl);
    double sum = diff;
    for (size_t i = 0; i < (size_t)N * H * P; ++i) sum += fabs(y1[i] - yl[i]);    /* sequence 0 is a chain */
    double *hc = vec((size_t)B * H * P * S, 0, 0);
    if (W > 1) {
        double *xbc = vec((size_t)B * N * Cc, 1, 0), *cs = vec((size_t)B * (W - 1) * Cc, 1, 0), *w = vec((size_t)Cc * W, 0.5, 0),
               *bias = vec(Cc, 0.5, 0), *out = vec((size_t)B * N * Cc, 0, 0), *cso = vec((size_t)B * (W - 1) * Cc, 0, 0);
        bad |= orc_tree_conv(B, N, Cc, W, parent, xbc, cs, w, bias, 1, out);
        bad |= orc_tree_conv(B, N, Cc, W, parent, xbc, cs, w, NULL, 0, out);
        bad |= orc_commit(B, N, H, P, S, G, W, Cc, parent, acc, x, dt, A, Bm, h0, hc, xbc, cs, cso);
        free(xbc); free(cs); free(w); free(bias); free(out); free(cso);
    }
    bad |= orc_commit(B, N, H, P, S, G, 0, 0, parent, acc, x, dt, A, Bm, NULL, hc, NULL, NULL, NULL);
    double *z = vec((size_t)B * N * H * P, 2, 0), *nw = vec((size_t)H * P, 0.5, 1), *gn = vec((size_t)B * N * H * P, 0, 0);
    bad |= orc_gate_norm(B * N, H * P, G, y1, z, nw, 1e-5, gn);
    printf("B%d N%d H%d P%d S%d G%d W%d: status %d, chain vs linear scan %.3e\n", B, N, H, P, S, G, W, bad, sum);
    free(parent); free(acc); free(x); free(dt); free(A); free(Bm); free(Cm); free(D); free(h0); free(y1); free(y2);
    free(depth); free(anc); free(mask); free(yl); free(hl); free(hc); free(z); free(nw); free(gn);
    return bad != 0 || !(sum < 1e-9);
}

int main(void) {
    int fail = 0;
    fail |= run(1, 1, 1, 1, 1, 1, 2);
    fail |= run(3, 7, 2, 3, 5, 1, 4);
    fail |= run(2, 33, 4, 4, 8, 2, 3);
    fail |= run(4, 70, 2, 8, 4, 2, 0);
    return fail;
}
