"""Pins for the CPU oracle: everything here runs without a GPU and checks the
oracle against things other than itself -- the one table the paper prints, a
hand-worked example, closed forms, the paper's matrix form on every tiny tree,
the chain == causal-scan equivalence the paper states, library conv1d, and
structural invariants."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import matrix_form
from paper_2505_14969_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rows(name):
    with open(os.path.join(GOLDEN, name)) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def _rand(rng, B, N, H, P, S, G, h0=True, D=True):
    x = rng.standard_normal((B, N, H, P))
    dt = np.logaddexp(0, rng.standard_normal((B, N, H)) - 2)
    A = -np.exp(rng.uniform(0, 2, H))
    Bm = rng.standard_normal((B, N, G, S))
    Cm = rng.standard_normal((B, N, G, S))
    Dv = rng.standard_normal(H) if D else None
    h = 0.1 * rng.standard_normal((B, H, P, S)) if h0 else None
    return x, dt, A, Bm, Cm, Dv, h


def _close(a, b, tol=1e-12):
    scale = max(np.max(np.abs(b)), 1e-300)
    assert np.max(np.abs(a - b)) <= tol * scale, (np.max(np.abs(a - b)), scale)


# ----------------------------------------------------------------------- #
# the table the paper prints (Fig. "binary-tree", left)
# ----------------------------------------------------------------------- #
def test_unroll_counts_match_printed_table(oracle):
    for levels, packed, states, tokens, printed in _rows("unroll_table.txt"):
        parent = synth.full_binary_tree(int(levels))
        assert len(parent) == int(packed)
        n_seq, n_tok = oracle.unroll_counts(parent)
        assert n_seq == int(states)
        assert n_tok == int(tokens)
        # the 5-level row is printed as 90; leaves x levels gives 80
        assert n_tok == int(states) * int(levels)
        if int(levels) != 5:
            assert n_tok == int(printed)


def test_unroll_counts_chain_and_star(oracle):
    assert oracle.unroll_counts(synth.chain_tree(17)) == (1, 17)
    assert oracle.unroll_counts(synth.star_tree(9)) == (8, 16)


# ----------------------------------------------------------------------- #
# tree index
# ----------------------------------------------------------------------- #
def test_tree_index_full_binary_closed_form(oracle):
    parent = synth.full_binary_tree(6)
    st, depth, mask, anc = oracle.tree_index(parent, 4)
    assert st == 0
    for i in range(len(parent)):
        assert depth[i] == int(math.floor(math.log2(i + 1)))
        for k in range(4):
            want = ((i + 1) >> k) - 1 if k <= depth[i] else -(k - depth[i])
            assert anc[i, k] == want
        bits = {j for j in range(len(parent)) if (mask[i, j // 32] >> (j % 32)) & 1}
        assert bits == {((i + 1) >> k) - 1 for k in range(depth[i] + 1)}


def test_tree_index_matches_mask_definition(oracle):
    rng = np.random.default_rng(5)
    for n, d in ((64, 6), (100, 9), (256, 10)):
        parent = synth.gen_tree(n, d, 5, rng)
        st, depth, mask, _ = oracle.tree_index(parent, 4)
        assert st == 0 and depth.max() == d
        L = matrix_form.tree_mask(parent)
        bits = ((mask[:, np.arange(n) // 32] >> (np.arange(n) % 32)) & 1).astype(np.float64)
        assert np.array_equal(bits, L)
        assert np.array_equal(L.sum(1) - 1, depth)


def test_tree_index_rejects_bad_trees(oracle):
    assert oracle.tree_index(np.array([0, 0, 1]), 2)[0] == 1          # root must be -1
    assert oracle.tree_index(np.array([-1, 0, 2]), 2)[0] == 3         # self loop
    assert oracle.tree_index(np.array([-1, 2, 0]), 2)[0] == 2         # forward edge
    assert oracle.tree_index(np.array([-1, -1, 0]), 2)[0] == 2        # second root
    assert oracle.tree_index(np.array([-1, 0, 7]), 2)[0] == 3         # out of range


# ----------------------------------------------------------------------- #
# hand-worked example
# ----------------------------------------------------------------------- #
def test_hand_worked_three_node_tree(oracle):
    rows = np.array(_rows("hand_example.txt"), dtype=np.float64)
    parent = rows[:, 1].astype(np.int32)
    dt, x, Bv, Cv, h_exp, y_exp = (rows[:, k] for k in range(2, 8))
    args = dict(x=x.reshape(1, 3, 1, 1), dt=dt.reshape(1, 3, 1), A=np.array([-math.log(2.0)]),
                Bm=Bv.reshape(1, 3, 1, 1), Cm=Cv.reshape(1, 3, 1, 1), D=np.array([0.5]),
                h0=np.full((1, 1, 1, 1), 4.0))
    for fn in (oracle.ssd_paths, oracle.ssd_nodes):
        y = fn(parent, **args)
        _close(y.reshape(3), y_exp, 1e-14)
    _close(matrix_form.ssd_matrix(parent, args["x"][0], args["dt"][0], args["A"], args["Bm"][0],
                                  args["Cm"][0], args["D"], args["h0"][0]).reshape(3), y_exp, 1e-14)
    for k in range(3):
        h, _ = oracle.commit(parent, [k], args["x"], args["dt"], args["A"], args["Bm"], args["h0"])
        assert abs(h.item() - h_exp[k]) < 1e-13


# ----------------------------------------------------------------------- #
# linear scan: closed forms
# ----------------------------------------------------------------------- #
def test_linear_scan_geometric_series(oracle):
    T, dtv, A, h0 = 12, 0.3, -1.7, 2.5
    a = math.exp(dtv * A)
    x = np.ones((1, T, 1, 1)); dt = np.full((1, T, 1), dtv)
    Bm = np.ones((1, T, 1, 1)); Cm = np.ones((1, T, 1, 1))
    y, hf = oracle.linear_scan(x, dt, np.array([A]), Bm, Cm, None, np.full((1, 1, 1, 1), h0))
    t = np.arange(1, T + 1)
    want = a ** t * h0 + dtv * (1 - a ** t) / (1 - a)
    _close(y.reshape(T), want, 1e-13)
    assert abs(hf.item() - want[-1]) < 1e-13


def test_linear_scan_outer_product_orientation(oracle):
    # one step from a zero state: h = dt * x (outer) B with x along P and B along S
    P, S = 3, 5
    rng = np.random.default_rng(0)
    x = rng.standard_normal((1, 1, 1, P)); Bm = rng.standard_normal((1, 1, 1, S))
    Cm = rng.standard_normal((1, 1, 1, S))
    y, hf = oracle.linear_scan(x, np.full((1, 1, 1), 0.7), np.array([-1.0]), Bm, Cm, np.array([2.0]), None)
    _close(hf[0, 0], 0.7 * np.outer(x.reshape(P), Bm.reshape(S)), 1e-15)
    _close(y.reshape(P), 0.7 * x.reshape(P) * float(Bm.reshape(S) @ Cm.reshape(S)) + 2.0 * x.reshape(P), 1e-14)


def test_linear_scan_equals_lower_triangular_matrix_form(oracle):
    rng = np.random.default_rng(11)
    T, H, P, S, G = 9, 4, 3, 5, 2
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, T, H, P, S, G)
    y, _ = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0)
    ym = matrix_form.ssd_matrix(synth.chain_tree(T), x[0], dt[0], A, Bm[0], Cm[0], D, h0[0])
    _close(y[0], ym)


# ----------------------------------------------------------------------- #
# the paper's remark: a lower-triangular mask is Mamba2 with an initial state
# ----------------------------------------------------------------------- #
@pytest.mark.parametrize("n", [1, 2, 33, 256])
def test_chain_tree_equals_linear_scan(oracle, n):
    rng = np.random.default_rng(n)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 2, n, 4, 8, 16, 2)
    parent = np.stack([synth.chain_tree(n)] * 2)
    want, hf = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0)
    assert np.array_equal(oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0), want)
    assert np.array_equal(oracle.ssd_nodes(parent, x, dt, A, Bm, Cm, D, h0), want)
    hc, _ = oracle.commit(parent, [n - 1, n - 1], x, dt, A, Bm, h0)
    assert np.array_equal(hc, hf)


# ----------------------------------------------------------------------- #
# matrix form (M_x, M_u from the definitions) on EVERY tree with 3..7 nodes
# ----------------------------------------------------------------------- #
def _all_trees(n):
    for rest in itertools.product(*[range(i) for i in range(1, n)]):
        yield np.array((-1,) + rest, dtype=np.int32)


@pytest.mark.parametrize("n", [3, 4, 5, 6, 7])
def test_matrix_form_on_all_small_trees(oracle, n):
    rng = np.random.default_rng(100 + n)
    H, P, S, G = 2, 3, 4, 2
    count = 0
    for parent in _all_trees(n):
        x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, n, H, P, S, G)
        y, rewrite = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0, return_rewrite_diff=True)
        assert rewrite == 0.0          # shared nodes: identical on every path
        ym = matrix_form.ssd_matrix(parent, x[0], dt[0], A, Bm[0], Cm[0], D, h0[0])
        _close(y[0], ym)
        _close(oracle.ssd_nodes(parent, x, dt, A, Bm, Cm, D, h0)[0], ym)
        count += 1
    assert count == math.factorial(n - 1)


def test_paths_equals_nodes_on_workload_trees(oracle):
    rng = np.random.default_rng(21)
    for n, d, G in ((64, 6, 1), (128, 8, 2), (256, 10, 4)):
        parent = np.stack([synth.gen_tree(n, d, 4 + G, rng) for _ in range(2)])
        x, dt, A, Bm, Cm, D, h0 = _rand(rng, 2, n, 4, 8, 16, G)
        y1, rewrite = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0, return_rewrite_diff=True)
        assert rewrite == 0.0
        assert np.array_equal(y1, oracle.ssd_nodes(parent, x, dt, A, Bm, Cm, D, h0))


def test_matrix_form_on_random_64_node_tree(oracle):
    rng = np.random.default_rng(22)
    parent = synth.gen_tree(64, 6, 4, rng)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, 64, 4, 8, 16, 2)
    _close(oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)[0],
           matrix_form.ssd_matrix(parent, x[0], dt[0], A, Bm[0], Cm[0], D, h0[0]), 1e-11)


# ----------------------------------------------------------------------- #
# closed forms on trees
# ----------------------------------------------------------------------- #
def test_star_tree_closed_form(oracle):
    rng = np.random.default_rng(31)
    n, H, P, S = 7, 2, 3, 4
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, n, H, P, S, 1)
    y = oracle.ssd_paths(synth.star_tree(n), x, dt, A, Bm, Cm, D, h0)[0]
    for h in range(H):
        a = np.exp(dt[0, :, h] * A[h])
        h_root = a[0] * h0[0, h] + dt[0, 0, h] * np.outer(x[0, 0, h], Bm[0, 0, 0])
        _close(y[0, h], h_root @ Cm[0, 0, 0] + D[h] * x[0, 0, h], 1e-13)
        for i in range(1, n):
            hi = a[i] * h_root + dt[0, i, h] * np.outer(x[0, i, h], Bm[0, i, 0])
            _close(y[i, h], hi @ Cm[0, i, 0] + D[h] * x[0, i, h], 1e-13)


def test_zero_dt_reads_initial_state(oracle):
    rng = np.random.default_rng(32)
    parent = synth.gen_tree(20, 4, 3, rng)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, 20, 2, 3, 4, 1)
    dt[:] = 0.0
    y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)[0]
    want = np.einsum("hps,ns->nhp", h0[0], Cm[0, :, 0]) + D[None, :, None] * x[0]
    _close(y, want, 1e-14)
    hc, _ = oracle.commit(parent, [13], x, dt, A, Bm, h0)
    assert np.array_equal(hc, h0)      # bit-exact: exp(0) = 1, + 0


def test_infinite_decay_keeps_only_own_token(oracle):
    rng = np.random.default_rng(33)
    parent = synth.gen_tree(20, 4, 3, rng)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, 20, 2, 3, 4, 1)
    A[:] = -1e4
    dt = dt + 0.1
    y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)[0]
    cb = np.einsum("ns,ns->n", Cm[0, :, 0], Bm[0, :, 0])
    want = dt[0][:, :, None] * cb[:, None, None] * x[0] + D[None, :, None] * x[0]
    _close(y, want, 1e-14)


def test_no_decay_sums_ancestors(oracle):
    rng = np.random.default_rng(34)
    n, H, P, S = 30, 2, 3, 5
    parent = synth.gen_tree(n, 5, 3, rng)
    x, dt, A, Bm, Cm, _, _ = _rand(rng, 1, n, H, P, S, 1, h0=False, D=False)
    A[:] = 0.0
    Bm[:] = 1.0
    Cm[:] = 1.0
    y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, None, None)[0]
    L = matrix_form.tree_mask(parent)
    want = S * np.einsum("ij,jhp->ihp", L, dt[0][:, :, None] * x[0])
    _close(y, want, 1e-13)


# ----------------------------------------------------------------------- #
# invariants
# ----------------------------------------------------------------------- #
def test_relabelling_permutes_outputs(oracle):
    rng = np.random.default_rng(41)
    parent = synth.gen_tree(48, 6, 4, rng)              # BFS labels
    perm = synth.relabel_permutation(parent, synth.relabel_dfs)   # perm[new] = old
    parent_dfs = synth.relabel_dfs(parent)
    assert not np.array_equal(parent, parent_dfs)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, 48, 2, 4, 8, 1)
    y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    y2 = oracle.ssd_paths(parent_dfs, x[:, perm], dt[:, perm], A, Bm[:, perm], Cm[:, perm], D, h0)
    assert np.array_equal(y2, y[:, perm])


def test_perturbing_a_node_changes_only_its_subtree(oracle):
    rng = np.random.default_rng(42)
    n = 40
    parent = synth.gen_tree(n, 5, 4, rng)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, n, 2, 4, 8, 1)
    y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)[0]
    L = matrix_form.tree_mask(parent)
    for j in (0, 3, 17, n - 1):
        x2, Bm2, dt2 = x.copy(), Bm.copy(), dt.copy()
        x2[0, j] += 1.0; Bm2[0, j] -= 0.5; dt2[0, j] *= 1.5
        yj = oracle.ssd_paths(parent, x2, dt2, A, Bm2, Cm, D, h0)[0]
        changed = np.any(yj != y, axis=(1, 2))
        assert np.array_equal(changed, L[:, j] > 0)


# ----------------------------------------------------------------------- #
# conv: textbook causal depthwise conv1d on every unrolled path (library routine)
# ----------------------------------------------------------------------- #
@pytest.mark.parametrize("W,silu,bias", [(4, True, True), (4, False, False), (2, True, False), (3, False, True)])
def test_tree_conv_equals_library_conv1d_on_paths(oracle, W, silu, bias):
    import torch
    rng = np.random.default_rng(50 + W)
    n, Cc = 40, 12
    parent = synth.gen_tree(n, 6, 3, rng)
    xbc = rng.standard_normal((1, n, Cc)); cs = rng.standard_normal((1, W - 1, Cc))
    w = rng.uniform(-0.5, 0.5, (Cc, W)); b = rng.uniform(-0.5, 0.5, Cc) if bias else None
    out = oracle.tree_conv(parent, xbc, cs, w, b, silu)[0]
    kids = [[] for _ in range(n)]
    for i in range(1, n):
        kids[parent[i]].append(i)
    checked = np.zeros(n, dtype=bool)
    for leaf in [i for i in range(n) if not kids[i]]:
        path = []
        v = leaf
        while v >= 0:
            path.append(v); v = int(parent[v])
        path = path[::-1]
        seq = np.concatenate([cs[0], xbc[0, path]], axis=0)          # [W-1+len, Cc]
        z = torch.nn.functional.conv1d(torch.from_numpy(seq.T.copy())[None], torch.from_numpy(w)[:, None, :],
                                       None if b is None else torch.from_numpy(b), groups=Cc)[0].T
        if silu:
            z = torch.nn.functional.silu(z)
        _close(out[path], z.numpy(), 1e-13)
        checked[path] = True
    assert checked.all()


# ----------------------------------------------------------------------- #
# commit
# ----------------------------------------------------------------------- #
def test_commit_equals_linear_scan_of_the_accepted_path(oracle):
    rng = np.random.default_rng(61)
    n, H, P, S, G, W = 50, 4, 4, 8, 2, 4
    Cc = H * P + 2 * G * S
    parent = np.stack([synth.gen_tree(n, 7, 3, rng) for _ in range(3)])
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 3, n, H, P, S, G)
    xbc = rng.standard_normal((3, n, Cc)); cs = rng.standard_normal((3, W - 1, Cc))
    acc = np.array([n - 1, 0, -1], dtype=np.int32)
    hc, cso = oracle.commit(parent, acc, x, dt, A, Bm, h0, xbc, cs)
    for b in range(3):
        if acc[b] < 0:
            assert np.array_equal(hc[b], h0[b]) and np.array_equal(cso[b], cs[b])
            continue
        path = []
        v = int(acc[b])
        while v >= 0:
            path.append(v); v = int(parent[b, v])
        path = path[::-1]
        _, hf = oracle.linear_scan(x[b:b + 1, path], dt[b:b + 1, path], A, Bm[b:b + 1, path], Cm[b:b + 1, path],
                                   None, h0[b:b + 1])
        assert np.array_equal(hc[b], hf[0])
        seq = np.concatenate([cs[b], xbc[b, path]], axis=0)
        assert np.array_equal(cso[b], seq[-(W - 1):])


def test_commit_then_continue_equals_grafted_tree(oracle):
    """Outputs of a second tree verified from the committed state equal the
    outputs of those nodes when the second tree is grafted under the accepted
    node of the first (same for the conv)."""
    rng = np.random.default_rng(62)
    n1, n2, H, P, S, G, W = 20, 15, 2, 4, 8, 1, 4
    Cc = H * P + 2 * G * S
    p1 = synth.gen_tree(n1, 4, 3, rng); p2 = synth.gen_tree(n2, 4, 3, rng)
    k = 11
    big = np.concatenate([p1, np.where(p2 < 0, k, p2 + n1)]).astype(np.int32)
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, n1 + n2, H, P, S, G)
    y_big = oracle.ssd_paths(big, x, dt, A, Bm, Cm, D, h0)[0]
    hk, _ = oracle.commit(p1, [k], x[:, :n1], dt[:, :n1], A, Bm[:, :n1], h0)
    y2 = oracle.ssd_paths(p2, x[:, n1:], dt[:, n1:], A, Bm[:, n1:], Cm[:, n1:], D, hk)[0]
    _close(y2, y_big[n1:], 1e-13)
    xbc = rng.standard_normal((1, n1 + n2, Cc)); cs = rng.standard_normal((1, W - 1, Cc))
    w = rng.uniform(-0.5, 0.5, (Cc, W)); b = rng.uniform(-0.5, 0.5, Cc)
    c_big = oracle.tree_conv(big, xbc, cs, w, b, True)[0]
    _, cs_k = oracle.commit(p1, [k], x[:, :n1], dt[:, :n1], A, Bm[:, :n1], h0, xbc[:, :n1], cs)
    c2 = oracle.tree_conv(p2, xbc[:, n1:], cs_k, w, b, True)[0]
    assert np.array_equal(c2, c_big[n1:])


def test_prefix_in_chunks_equals_one_scan(oracle):
    rng = np.random.default_rng(63)
    T, chunk, H, P, S = 96, 32, 2, 4, 8
    x, dt, A, Bm, Cm, D, h0 = _rand(rng, 1, T, H, P, S, 1)
    _, hf = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0)
    h = h0
    for c in range(T // chunk):
        sl = slice(c * chunk, (c + 1) * chunk)
        h, _ = oracle.commit(synth.chain_tree(chunk), [chunk - 1], x[:, sl], dt[:, sl], A, Bm[:, sl], h)
    assert np.array_equal(h, hf)


# --------------------------------------------------------------------------- #
# output gate + grouped RMS norm behind the scan (the Mamba2 block; not in the paper)
# --------------------------------------------------------------------------- #
def test_gate_norm_hand_worked_example(oracle):
    """tests/golden/gate_norm_example.txt: 2 rows x 4 channels, 2 groups, worked by hand."""
    rows, w = [], None
    for line in open(os.path.join(GOLDEN, "gate_norm_example.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        f = line.split()
        if f[0] == "w":
            w = np.array([float(v) for v in f[1:]])
        else:
            rows.append([float(v) for v in f[1:]])
    rows = np.array(rows)
    y, z, want = rows[:, :4], rows[:, 4:8] * np.log(3.0), rows[:, 8:]
    got = oracle.gate_norm(y, z, w, 2, 0.0)
    assert np.allclose(got, want, rtol=0, atol=5e-10)


def test_gate_norm_against_torch_silu_and_rms_norm(oracle):
    """The two library routines the step is made of: silu, then rms_norm on each group."""
    import torch
    import torch.nn.functional as F
    rng = np.random.default_rng(70)
    for (rows, H, P, G, eps) in ((5, 4, 8, 1, 1e-5), (3, 6, 4, 3, 1e-6), (2, 8, 16, 8, 0.0), (4, 2, 3, 2, 1e-5)):
        d = H * P
        y = rng.standard_normal((rows, H, P)); z = 2.0 * rng.standard_normal((rows, H, P)); w = rng.uniform(0.5, 1.5, d)
        v = torch.from_numpy(y) * F.silu(torch.from_numpy(z))
        vg = v.reshape(rows, G, d // G)
        want = F.rms_norm(vg, (d // G,), eps=eps).reshape(rows, d) * torch.from_numpy(w)
        got = oracle.gate_norm(y, z, w, G, eps)
        assert got.shape == y.shape
        _close(got.reshape(rows, d), want.numpy(), 1e-13)


def test_gate_norm_closed_forms(oracle):
    rng = np.random.default_rng(71)
    rows, d, G = 4, 24, 3
    y = rng.standard_normal((rows, d)); z = rng.standard_normal((rows, d)); w = rng.uniform(0.5, 1.5, d)
    base = oracle.gate_norm(y, z, w, G, 0.0)
    # without eps the norm forgets the scale of y; each group has unit mean square before the weight
    _close(oracle.gate_norm(7.5 * y, z, w, G, 0.0), base, 1e-13)
    ms = np.mean((base / w).reshape(rows, G, d // G) ** 2, axis=-1)
    assert np.allclose(ms, 1.0, rtol=1e-12)
    # a group only sees its own channels
    y2 = y.copy(); y2[:, : d // G] *= -3.0
    other = oracle.gate_norm(y2, z, w, G, 0.0)
    assert np.array_equal(other[:, d // G:], base[:, d // G:]) and not np.allclose(other[:, : d // G], base[:, : d // G])
    # z = 0 closes the gate: silu(0) = 0, and with eps > 0 the output is exactly zero
    assert not oracle.gate_norm(y, np.zeros_like(z), w, G, 1e-5).any()
    # large z opens it: silu(z) -> z, so y * silu(z) -> y z
    zz = np.full_like(z, 40.0)
    v = y * 40.0
    want = v / np.sqrt(np.mean(v.reshape(rows, G, -1) ** 2, axis=-1, keepdims=True)).repeat(d // G, -1).reshape(rows, d) * w
    _close(oracle.gate_norm(y, zz, w, G, 0.0), want, 1e-12)
    with pytest.raises(ValueError):
        oracle.gate_norm(y, z, w, 5, 0.0)


def test_step_size_closed_forms_and_library_softplus(oracle):
    """softplus(raw + bias): ln 2 at zero, softplus(v) - softplus(-v) = v, both tails, the bias is per head
    (last index), and torch's softplus (its threshold switched off) on random values."""
    import torch
    assert oracle.step_size(np.zeros((1, 1)))[0, 0] == pytest.approx(math.log(2.0), rel=1e-15)
    v = np.linspace(-30, 30, 61).reshape(-1, 1)
    assert np.allclose(oracle.step_size(v) - oracle.step_size(-v), v, rtol=0, atol=1e-13)
    assert oracle.step_size(np.array([[50.0]]))[0, 0] == pytest.approx(50.0, rel=1e-15)
    assert oracle.step_size(np.array([[800.0]]))[0, 0] == 800.0                      # no overflow
    assert oracle.step_size(np.array([[-40.0]]))[0, 0] == pytest.approx(math.exp(-40.0), rel=1e-12)
    # bias indexed by head, added before the softplus: softplus(0 + b_h) with b = (0, ln(e - 1)) gives (ln 2, 1)
    got = oracle.step_size(np.zeros((3, 2)), np.array([0.0, math.log(math.e - 1.0)]))
    assert np.allclose(got, np.array([[math.log(2.0), 1.0]] * 3), rtol=1e-14, atol=0)
    rng = np.random.default_rng(77)
    raw, bias = rng.standard_normal((5, 7, 6)) * 4, rng.standard_normal(6)
    want = torch.nn.functional.softplus(torch.from_numpy(raw + bias), threshold=1e9).numpy()
    assert np.allclose(oracle.step_size(raw, bias), want, rtol=1e-13, atol=0)
