"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer results bit-exact; floating point within
1e-4 (fp32 io) or 2e-2 (bf16 io, fp32 accumulate) by the metric of
helpers.parity (max-abs and l2 error relative to the reference tensor)."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, split_xbc, split_xbc_dev, to_dev, to_host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def st():
    import torch
    from paper_2505_14969_amd import binding
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    binding.load()           # fail loudly when the HIP library is not built
    return binding


def _rand(seed, io, B, N, H, P, S, G, h0=True):
    rng = np.random.default_rng(seed)
    rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    x = rnd(rng.standard_normal((B, N, H, P)).astype(np.float32))
    Bm = rnd(rng.standard_normal((B, N, G, S)).astype(np.float32))
    Cm = rnd(rng.standard_normal((B, N, G, S)).astype(np.float32))
    dt = np.logaddexp(0, rng.standard_normal((B, N, H)) - 2).astype(np.float32)
    A = (-np.exp(rng.uniform(0, 2, H))).astype(np.float32)
    D = rng.standard_normal(H).astype(np.float32)
    h = (0.1 * rng.standard_normal((B, H, P, S))).astype(np.float32) if h0 else None
    return x, dt, A, Bm, Cm, D, h


def _trees(seed, B, N):
    rng = np.random.default_rng(seed)
    out = []
    for b in range(B):
        if N <= 2:
            out.append(synth.chain_tree(N))
            continue
        d = int(rng.integers(1, min(N - 1, 12) + 1))
        tree = synth.gen_tree(N, d, N, rng)
        out.append(synth.relabel_dfs(tree) if b % 2 else tree)
    return np.stack(out).astype(np.int32)


def _run_ssd(st, io, parent, x, dt, A, Bm, Cm, D, h0, **kw):
    y = st.stree_tree_ssd(to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io),
                          to_dev(D), to_dev(h0), **kw)
    return to_host(y)


# --------------------------------------------------------------------------- #
# tree index: exact integers
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("N", [1, 2, 15, 31, 64, 65, 100, 255, 256])
def test_tree_index_bit_exact(st, oracle, N):
    parent = _trees(7 + N, 5, N)
    parent[-1] = synth.chain_tree(N)
    depth, mask, anc, status = (to_host(t) for t in st.stree_tree_index(to_dev(parent), 4))
    for b in range(parent.shape[0]):
        s, d, m, a = oracle.tree_index(parent[b], 4)
        assert s == 0 and status[b] == 0
        assert np.array_equal(depth[b], d)
        assert np.array_equal(mask[b].view(np.uint32), m)
        assert np.array_equal(anc[b], a)


def test_tree_index_reports_bad_trees(st, oracle):
    good = synth.gen_tree(40, 5, 4, np.random.default_rng(3))
    bads = [good.copy() for _ in range(5)]
    bads[0][0] = 0           # root must be -1
    bads[1][7] = 7           # self loop
    bads[2][9] = 30          # forward edge
    bads[3][20] = -1         # second root
    bads[4][39] = 1000       # out of range
    parent = np.stack(bads + [good]).astype(np.int32)
    depth, mask, anc, status = (to_host(t) for t in st.stree_tree_index(to_dev(parent), 3))
    want = [oracle.tree_index(p, 3)[0] for p in parent]
    assert list(status) == want == [1, 8, 10, 21, 40, 0]
    assert not depth[:5].any() and not mask[:5].any()
    assert np.array_equal(depth[5], oracle.tree_index(good, 3)[1])


# --------------------------------------------------------------------------- #
# configuration 0: fp32, full binary tree, 1e-4
# --------------------------------------------------------------------------- #
def test_config0_fp32(st, oracle):
    wl = synth.config(0)
    want = oracle.ssd_paths(wl.parent, wl.x, wl.dt, wl.A, wl.Bm, wl.Cm, wl.D, wl.h0)
    got = _run_ssd(st, "f32", wl.parent, wl.x, wl.dt, wl.A, wl.Bm, wl.Cm, wl.D, wl.h0)
    assert_parity(got, want, TOL["f32"], "cfg0 y", kind="y")


@pytest.mark.parametrize("N,H,P,S,G", [(1, 2, 8, 8, 1), (13, 3, 24, 20, 1), (64, 4, 64, 64, 2),
                                       (100, 2, 32, 48, 1), (256, 2, 16, 16, 2)])
def test_fp32_fma_kernel_shapes(st, oracle, N, H, P, S, G):
    parent = _trees(N, 2, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(N + 1, "f32", 2, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "f32", parent, x, dt, A, Bm, Cm, D, h0)
    assert_parity(got, want, TOL["f32"], f"fp32 N={N}", kind="y")


def test_fp32_chain_256_against_linear_scan(st, oracle):
    N = 256
    parent = np.stack([synth.chain_tree(N)] * 2)
    x, dt, A, Bm, Cm, D, h0 = _rand(5, "f32", 2, N, 2, 32, 32, 1)
    want, _ = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "f32", parent, x, dt, A, Bm, Cm, D, h0)
    assert_parity(got, want, TOL["f32"], "fp32 chain", kind="y")


# --------------------------------------------------------------------------- #
# bf16 MFMA kernel: shapes spanning several tiles and ragged tails
# --------------------------------------------------------------------------- #
MFMA_SHAPES = [(1, 2, 64, 128, 1), (13, 4, 64, 128, 1), (63, 2, 64, 64, 2), (64, 8, 64, 128, 1),
               (65, 2, 64, 128, 1), (100, 4, 32, 16, 2), (128, 2, 128, 64, 1), (200, 2, 64, 256, 2),
               (256, 4, 64, 128, 4), (256, 2, 128, 256, 1), (96, 2, 32, 128, 1)]


@pytest.mark.parametrize("N,H,P,S,G", MFMA_SHAPES)
def test_bf16_mfma_kernel_shapes(st, oracle, N, H, P, S, G):
    parent = _trees(100 + N, 3, N)
    parent[2] = synth.chain_tree(N)
    x, dt, A, Bm, Cm, D, h0 = _rand(N + P, "bf16", 3, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0)
    assert_parity(got, want, TOL["bf16"], f"mfma N={N} P={P} S={S}", kind="y")
    # the plain-FMA kernel on the same bf16 inputs only rounds the output
    got2 = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, force_fma=True)
    assert_parity(got2, want, 6e-3, f"fma-bf16 N={N}", kind="y")


def test_bf16_mfma_kernel_skips_column_blocks_without_ancestors(st, oracle):
    # trees of several 64-node blocks in which whole (row block, column block) pairs hold no
    # ancestor: a star, two far-apart families (parent i - 128), and a chain hanging off node 0
    # that starts in the last block
    N, H, P, S, G = 250, 2, 64, 128, 1
    far = np.arange(N, dtype=np.int32) - 128
    far[:128] = np.arange(128, dtype=np.int32) - 1
    late = np.zeros(N, dtype=np.int32)
    late[0] = -1
    late[200:] = np.arange(199, N - 1, dtype=np.int32)
    late[200] = 0
    parent = np.stack([synth.star_tree(N), far, late]).astype(np.int32)
    x, dt, A, Bm, Cm, D, h0 = _rand(77, "bf16", 3, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0)
    assert_parity(got, want, TOL["bf16"], "mfma block skipping", kind="y")


def test_bf16_optional_arguments(st, oracle):
    N, H, P, S, G = 48, 2, 64, 64, 1
    parent = _trees(9, 2, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(10, "bf16", 2, N, H, P, S, G)
    for Dv, hv in ((None, h0), (D, None), (None, None)):
        want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, Dv, hv)
        got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, Dv, hv)
        assert_parity(got, want, TOL["bf16"], "optional args", kind="y")


def test_bad_tree_zero_fills_that_sequence_only(st, oracle):
    import torch
    N, H, P, S, G = 64, 2, 64, 128, 1
    parent = _trees(11, 3, N)
    parent[1, 20] = 33
    x, dt, A, Bm, Cm, D, h0 = _rand(12, "bf16", 3, N, H, P, S, G)
    for force in (False, True):
        status = torch.full((3,), -7, dtype=torch.int32, device="cuda")
        got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, status=status, force_fma=force)
        assert list(to_host(status)) == [0, 21, 0]
        assert not got[1].any()
        keep = [0, 2]
        want = oracle.ssd_paths(parent[keep], x[keep], dt[keep], A, Bm[keep], Cm[keep], D, h0[keep])
        assert_parity(got[keep], want, TOL["bf16"], "good sequences next to a bad one", kind="y")


def test_relabelling_permutes_gpu_outputs(st):
    N, H, P, S, G = 64, 2, 64, 128, 1
    tree = synth.gen_tree(N, 6, 4, np.random.default_rng(13))
    perm = synth.relabel_permutation(tree, synth.relabel_dfs)
    x, dt, A, Bm, Cm, D, h0 = _rand(14, "bf16", 1, N, H, P, S, G)
    y1 = _run_ssd(st, "bf16", tree[None], x, dt, A, Bm, Cm, D, h0)
    y2 = _run_ssd(st, "bf16", synth.relabel_dfs(tree)[None], x[:, perm], dt[:, perm], A, Bm[:, perm], Cm[:, perm],
                  D, h0)
    assert_parity(y2, y1[:, perm], 1e-2, "relabel", kind="y")


# --------------------------------------------------------------------------- #
# conv
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("io,W,silu,bias", [("bf16", 4, True, True), ("bf16", 2, False, False),
                                            ("f32", 4, True, True), ("f32", 3, False, True)])
def test_tree_conv(st, oracle, io, W, silu, bias):
    B, N, H, P, S, G = 3, (256 if W == 3 else 70), 4, 64, 32, 2
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(20 + W)
    rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    parent = _trees(21, B, N)
    xbc = rnd(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = rnd(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    w = rnd(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
    b = rnd(rng.uniform(-0.5, 0.5, Cc).astype(np.float32)) if bias else None
    want = oracle.tree_conv(parent, xbc, cs, w, b, silu)
    got = to_host(st.stree_tree_conv(to_dev(parent), to_dev(xbc, io), to_dev(cs, io), to_dev(w, io),
                                     to_dev(b, io), H, P, S, G, silu=silu))
    assert_parity(got, want, TOL[io] if io == "f32" else 4e-3, "conv")
    # elementwise: fp32 accumulation, then one rounding to the storage type
    ulp = 2.0 ** -8 if io == "bf16" else 2.0 ** -22
    assert np.all(np.abs(got - want) <= ulp * np.abs(want) + 1e-5)


# --------------------------------------------------------------------------- #
# commit
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_commit_state(st, oracle, io):
    import torch
    B, N, H, P, S, G, W = 5, 90, 4, 64, 128, 2, 4
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(30)
    rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    parent = _trees(31, B, N)
    parent[4] = synth.chain_tree(N)
    x, dt, A, Bm, Cm, D, h0 = _rand(32, io, B, N, H, P, S, G)
    xbc = rnd(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = rnd(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    acc = np.array([N - 1, 0, -1, 37, N - 1], dtype=np.int32)
    want_h, want_cs = oracle.commit(parent, acc, x, dt, A, Bm, h0, xbc, cs)
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    h, cso = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(dt), to_dev(A),
                                   to_dev(Bm, io), to_dev(h0), xbc_pre=to_dev(xbc, io), conv_state=to_dev(cs, io),
                                   status=status)
    assert not to_host(status).any()
    for b in range(B):
        assert_parity(to_host(h)[b], want_h[b], 1e-4, f"commit h b={b}", kind="state")
    assert np.array_equal(to_host(h)[2], h0[2])                  # -1 keeps the state bit-exactly
    assert np.array_equal(to_host(cso), want_cs.astype(np.float32))   # row copies: exact
    # in place
    h_io, cs_io = to_dev(h0), to_dev(cs, io)
    st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                          h_io, h_out=h_io, xbc_pre=to_dev(xbc, io), conv_state=cs_io, conv_state_out=cs_io)
    assert np.array_equal(to_host(h_io), to_host(h))
    assert np.array_equal(to_host(cs_io), to_host(cso))


def test_commit_edge_cases(st, oracle):
    import torch
    B, N, H, P, S, G = 3, 20, 2, 32, 64, 1
    parent = _trees(41, B, N)
    parent[1, 5] = 9                                              # bad tree
    x, dt, A, Bm, Cm, D, h0 = _rand(42, "bf16", B, N, H, P, S, G)
    acc = np.array([N + 3, 4, 6], dtype=np.int32)                # out of range, (bad tree), ok
    status = torch.zeros((B,), dtype=torch.int32, device="cuda")
    h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, "bf16"), to_dev(dt), to_dev(A),
                                 to_dev(Bm, "bf16"), to_dev(h0), status=status)
    assert list(to_host(status)) == [-1, 6, 0]
    h = to_host(h)
    assert np.array_equal(h[0], h0[0]) and np.array_equal(h[1], h0[1])
    want, _ = oracle.commit(parent[2:], acc[2:], x[2:], dt[2:], A, Bm[2:], h0[2:])
    assert_parity(h[2], want[0], 1e-4, "commit next to bad sequences", kind="state")
    # zero dt: the state comes back bit-exactly
    h2, _ = st.stree_commit_state(to_dev(parent[2:]), to_dev(acc[2:]), to_dev(x[2:], "bf16"),
                                  to_dev(np.zeros_like(dt[2:])), to_dev(A), to_dev(Bm[2:], "bf16"), to_dev(h0[2:]))
    assert np.array_equal(to_host(h2), h0[2:])
    # no initial state
    h3, _ = st.stree_commit_state(to_dev(parent[2:]), to_dev(acc[2:]), to_dev(x[2:], "bf16"), to_dev(dt[2:]),
                                  to_dev(A), to_dev(Bm[2:], "bf16"), None)
    want3, _ = oracle.commit(parent[2:], acc[2:], x[2:], dt[2:], A, Bm[2:], None)
    assert_parity(to_host(h3), want3, 1e-4, "commit without h0", kind="state")


@pytest.mark.parametrize("N", [30, 130])
def test_commit_conv_tail_alone_reports_status(st, oracle, N):
    """Conv tail only (all state pointers NULL): the per-sequence status is written by the conv-tail
    workgroups -- 0, first bad node + 1, or -1 for an accepted index outside [-1, N) -- and in the
    last two cases the conv state passes through."""
    import torch
    B, H, P, S, G, W = 5, 3, 64, 128, 1, 4
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(300 + N)
    parent = _trees(301 + N, B, N)
    parent[1, 7] = 12                                             # invalid: parent label above the node's
    parent[3, 0] = 0                                              # invalid root
    xbc = synth.round_to_bf16(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = synth.round_to_bf16(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    acc = np.array([N - 1, 3, N + 4, 2, -1], dtype=np.int32)
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    _, cso = st.stree_commit_state(to_dev(parent), to_dev(acc), None, None, None, None, xbc_pre=to_dev(xbc, "bf16"),
                                   conv_state=to_dev(cs, "bf16"), status=status, dims=(H, P, S, G))
    assert list(to_host(status)) == [0, 8, -1, 1, 0]
    got = to_host(cso)
    z = np.zeros((1, N, 1, 4), dtype=np.float32)                  # (the oracle's commit wants a state part: a dummy one)
    _, want = oracle.commit(parent[:1], acc[:1], z, z[..., 0], np.array([-1.0], dtype=np.float32), z, None, xbc[:1],
                            cs[:1])
    assert np.array_equal(got[0], want[0].astype(np.float32))
    for b in (1, 2, 3, 4):
        assert np.array_equal(got[b], cs[b])


@pytest.mark.parametrize("io", ["bf16", "f32"])
@pytest.mark.parametrize("N", [40, 100])
def test_commit_unpredicated_kernel_cases(st, oracle, io, N):
    """Shapes whose state the threads tile exactly (the kernel variant without bounds checks), on both
    tree-size branches: missing initial state, a bad tree, accepted = -1 and out of range, a long and a
    one-node path, several heads per group."""
    import torch
    B, H, P, S, G = 6, 6, 64, 128, 2
    parent = _trees(71, B, N)
    parent[0] = synth.chain_tree(N)
    parent[3, N // 2] = N - 1                                     # bad tree
    x, dt, A, Bm, Cm, D, h0 = _rand(72, io, B, N, H, P, S, G)
    acc = np.array([N - 1, 0, -1, 5, N + 2, N // 3], dtype=np.int32)
    good = [0, 1, 5]
    want, _ = oracle.commit(parent[good], acc[good], x[good], dt[good], A, Bm[good], h0[good])
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(dt), to_dev(A),
                                 to_dev(Bm, io), to_dev(h0), status=status)
    assert list(to_host(status)) == [0, 0, 0, N // 2 + 1, -1, 0]
    h = to_host(h)
    for i, b in enumerate(good):
        assert_parity(h[b], want[i], 1e-4, f"commit b={b}", kind="state")
    for b in (2, 3, 4):                                           # kept bit-exactly
        assert np.array_equal(h[b], h0[b])
    # no initial state: zeros for the sequences that keep it, the update alone for the others
    want0, _ = oracle.commit(parent[good], acc[good], x[good], dt[good], A, Bm[good], None)
    hz, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(dt), to_dev(A),
                                  to_dev(Bm, io), None,
                                  h_out=torch.full((B, H, P, S), float("nan"), dtype=torch.float32, device="cuda"))
    hz = to_host(hz)
    for i, b in enumerate(good):
        assert_parity(hz[b], want0[i], 1e-4, f"commit without h0 b={b}", kind="state")
    for b in (2, 3, 4):
        assert not hz[b].any()
    # x / B as strided views of one buffer whose rows are not a whole number of 16-byte pieces: the
    # predicated kernel takes over, same result
    pad = 4 if io == "bf16" else 2
    xw = torch.zeros((B, N, H * P + pad), dtype=to_dev(x, io).dtype, device="cuda")
    xw[..., :H * P] = to_dev(x, io).reshape(B, N, H * P)
    hv, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), xw[..., :H * P].view(B, N, H, P), to_dev(dt),
                                  to_dev(A), to_dev(Bm, io), to_dev(h0))
    assert_parity(to_host(hv)[good], h[good], 1e-6, "commit from a misaligned view", kind="state")


@pytest.mark.parametrize("N,H,P,S,G", [(13, 3, 24, 20, 1), (30, 2, 12, 48, 2), (64, 2, 256, 256, 1), (7, 4, 1, 4, 4)])
def test_commit_ragged_shapes(st, oracle, N, H, P, S, G):
    """State tiles that do not divide evenly over the threads of a workgroup."""
    B = 2
    parent = _trees(61, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(62, "f32", B, N, H, P, S, G)
    acc = np.array([N - 1, N // 2], dtype=np.int32)
    want, _ = oracle.commit(parent, acc, x, dt, A, Bm, h0)
    h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, "f32"), to_dev(dt), to_dev(A),
                                 to_dev(Bm, "f32"), to_dev(h0))
    assert_parity(to_host(h), want, 1e-4, f"commit P={P} S={S}", kind="state")


def test_commit_then_continue_on_gpu(st, oracle):
    """Verify a second tree from the committed state: equals the grafted big tree."""
    n1, n2, H, P, S, G = 40, 30, 2, 64, 128, 1
    rng = np.random.default_rng(50)
    p1, p2 = synth.gen_tree(n1, 5, 4, rng), synth.gen_tree(n2, 4, 3, rng)
    k = 23
    big = np.concatenate([p1, np.where(p2 < 0, k, p2 + n1)]).astype(np.int32)
    x, dt, A, Bm, Cm, D, h0 = _rand(51, "bf16", 1, n1 + n2, H, P, S, G)
    want = oracle.ssd_paths(big, x, dt, A, Bm, Cm, D, h0)[:, n1:]
    hk, _ = st.stree_commit_state(to_dev(p1[None]), to_dev(np.array([k], dtype=np.int32)),
                                  to_dev(x[:, :n1], "bf16"), to_dev(dt[:, :n1]), to_dev(A),
                                  to_dev(Bm[:, :n1], "bf16"), to_dev(h0))
    y2 = st.stree_tree_ssd(to_dev(p2[None]), to_dev(x[:, n1:], "bf16"), to_dev(dt[:, n1:]), to_dev(A),
                           to_dev(Bm[:, n1:], "bf16"), to_dev(Cm[:, n1:], "bf16"), to_dev(D), hk)
    assert_parity(to_host(y2), want, TOL["bf16"], "commit then continue", kind="y")

