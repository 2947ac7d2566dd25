"""GPU parity of the fused activation replay + tree scan (Alg. 1: the state is
advanced along the previous tree's accepted path at the start of the next
iteration).  The oracle has no fused routine: the expected values are its commit
followed by its path-unrolled scan from the committed state."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _case(seed, io, B, Np, N, H, P, S, G):
    prev = _rand(seed, io, B, Np, H, P, S, G)
    cur = _rand(seed + 1, io, B, N, H, P, S, G, h0=False)
    pp, p = _trees(seed + 2, B, Np), _trees(seed + 3, B, N)
    return prev, cur, pp, p


def _expect(oracle, pp, acc, prev, p, cur, A, D):
    px, pdt, _, pB, _, _, h0 = prev
    x, dt, _, Bm, Cm, _, _ = cur
    h_star, _ = oracle.commit(pp, acc, px, pdt, A, pB, h0)
    y = oracle.ssd_paths(p, x, dt, A, Bm, Cm, D, h_star)
    return h_star, y


def _run(st, io, pp, acc, prev, p, cur, A, D, h_io=None, **kw):
    px, pdt, _, pB, _, _, h0 = prev
    x, dt, _, Bm, Cm, _, _ = cur
    h_in = to_dev(h0) if h_io is None else h_io
    y, h = st.stree_tree_ssd_replay(to_dev(pp), to_dev(acc), to_dev(px, io), to_dev(pdt), to_dev(pB, io),
                                    to_dev(p), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), h_in, **kw)
    return to_host(y), to_host(h)


# single-pass kernel shapes (both trees of at most 64 nodes, bf16, MFMA head shapes), several
# units per workgroup, and shapes that take the two-kernel route
SHAPES = [("bf16", 5, 40, 64, 6, 64, 128, 2), ("bf16", 3, 64, 30, 4, 64, 64, 1), ("bf16", 2, 20, 64, 3, 128, 128, 1),
          ("bf16", 16, 33, 57, 80, 64, 128, 1), ("bf16", 2, 100, 64, 4, 64, 128, 1), ("bf16", 2, 30, 130, 4, 64, 128, 2),
          ("f32", 2, 25, 31, 3, 24, 20, 1), ("bf16", 4, 64, 64, 6, 64, 256, 2), ("bf16", 3, 17, 40, 3, 64, 256, 1)]


@pytest.mark.parametrize("io,B,Np,N,H,P,S,G", SHAPES)
def test_replay_matches_commit_then_scan(st, oracle, io, B, Np, N, H, P, S, G):
    import torch
    prev, cur, pp, p = _case(700 + B + N, io, B, Np, N, H, P, S, G)
    A, D = prev[2], prev[5]
    rng = np.random.default_rng(7)
    acc = rng.integers(0, Np, B).astype(np.int32)
    acc[0] = Np - 1
    if B > 2:
        acc[2] = -1                                   # nothing accepted: state passes through
        pp[1] = synth.chain_tree(Np)                  # longest possible path
        acc[1] = Np - 1
    want_h, want_y = _expect(oracle, pp, acc, prev, p, cur, A, D)
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    rstatus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    y, h = _run(st, io, pp, acc, prev, p, cur, A, D, status=status, replay_status=rstatus)
    assert not to_host(status).any() and not to_host(rstatus).any()
    for b in range(B):
        assert_parity(h[b], want_h[b], 1e-4, f"replayed state b={b}", kind="state")
        assert_parity(y[b], want_y[b], TOL[io], f"scan after replay b={b}", kind="y")
    if B > 2:
        assert np.array_equal(h[2], prev[6][2])       # bit-exact pass-through
    # in place: same bits
    h_io = to_dev(prev[6])
    y2, h2 = _run(st, io, pp, acc, prev, p, cur, A, D, h_io=h_io, h_out=h_io)
    assert np.array_equal(h2, h) and np.array_equal(y2, y)


def test_replay_edge_cases(st, oracle):
    """Bad previous tree, accepted index out of range, bad current tree: the state passes
    through (or is still replayed) and the scan of the other sequences is untouched."""
    import torch
    io, B, Np, N, H, P, S, G = "bf16", 4, 20, 24, 4, 64, 128, 1
    prev, cur, pp, p = _case(900, io, B, Np, N, H, P, S, G)
    A, D = prev[2], prev[5]
    acc = np.array([Np + 5, 7, 3, 11], dtype=np.int32)          # b=0 out of range
    pp[1, 6] = 9                                                 # b=1 bad previous tree
    p[2, 4] = 4                                                  # b=2 bad current tree
    status = torch.zeros((B,), dtype=torch.int32, device="cuda")
    rstatus = torch.zeros((B,), dtype=torch.int32, device="cuda")
    y, h = _run(st, io, pp, acc, prev, p, cur, A, D, status=status, replay_status=rstatus)
    assert list(to_host(rstatus)) == [-1, 7, 0, 0]
    assert list(to_host(status)) == [0, 0, 5, 0]
    h0 = prev[6]
    assert np.array_equal(h[0], h0[0]) and np.array_equal(h[1], h0[1])
    assert not y[2].any()
    # expected values sequence by sequence (the oracle rejects bad trees as a whole)
    x, dt, _, Bm, Cm, _, _ = cur
    for b in (0, 1):
        want = oracle.ssd_paths(p[b:b + 1], x[b:b + 1], dt[b:b + 1], A, Bm[b:b + 1], Cm[b:b + 1], D, h0[b:b + 1])
        assert_parity(y[b], want[0], TOL[io], f"scan from the untouched state b={b}", kind="y")
    px, pdt, _, pB, _, _, _ = prev
    for b in (2, 3):
        want_h, _ = oracle.commit(pp[b:b + 1], acc[b:b + 1], px[b:b + 1], pdt[b:b + 1], A, pB[b:b + 1], h0[b:b + 1])
        assert_parity(h[b], want_h[0], 1e-4, f"replayed state b={b}", kind="state")
    want = oracle.ssd_paths(p[3:4], x[3:4], dt[3:4], A, Bm[3:4], Cm[3:4], D, want_h)
    assert_parity(y[3], want[0], TOL[io], "scan after replay b=3", kind="y")


def test_replay_chain_of_iterations(st, oracle):
    """Three decoding iterations through the fused call, the state carried in place, against one
    oracle scan of the concatenated accepted paths (the linear-sequence special case)."""
    io, B, H, P, S, G, N = "bf16", 2, 4, 64, 128, 1, 48
    rng = np.random.default_rng(77)
    steps = [(_rand(950 + i, io, B, N, H, P, S, G), _trees(960 + i, B, N)) for i in range(4)]
    A, D = steps[0][0][2], steps[0][0][5]
    h0 = steps[0][0][6]
    accs = [rng.integers(0, N, B).astype(np.int32) for _ in range(3)]
    h_dev = to_dev(h0)
    for i in range(3):
        prev, pp = steps[i]
        cur, p = steps[i + 1]
        y, _ = st.stree_tree_ssd_replay(to_dev(pp), to_dev(accs[i]), to_dev(prev[0], io), to_dev(prev[1]),
                                        to_dev(prev[3], io), to_dev(p), to_dev(cur[0], io), to_dev(cur[1]),
                                        to_dev(A), to_dev(cur[3], io), to_dev(cur[4], io), to_dev(D), h_dev,
                                        h_out=h_dev)
    # oracle: accepted paths of the three trees as one sequence, then the last tree from that state
    want_h = np.empty_like(h0, dtype=np.float64)
    for b in range(B):
        xs, dts, Bs = [], [], []
        for i in range(3):
            prev, pp = steps[i]
            path, v = [], int(accs[i][b])
            while v >= 0:
                path.append(v)
                v = int(pp[b, v])
            path.reverse()
            xs.append(prev[0][b, path]); dts.append(prev[1][b, path]); Bs.append(prev[3][b, path])
        xs, dts, Bs = np.concatenate(xs)[None], np.concatenate(dts)[None], np.concatenate(Bs)[None]
        _, hf = oracle.linear_scan(xs, dts, A, Bs, np.zeros_like(Bs), None, h0[b:b + 1])
        want_h[b] = hf[0]
    assert_parity(to_host(h_dev), want_h, 1e-4, "state after three fused iterations", kind="state")
    cur, p = steps[3]
    want_y = oracle.ssd_paths(p, cur[0], cur[1], A, cur[3], cur[4], D, want_h)
    assert_parity(to_host(y), want_y, TOL[io], "scan of the fourth tree", kind="y")


@pytest.mark.parametrize("io,W,N,Np", [("bf16", 4, 70, 33), ("bf16", 2, 64, 64), ("f32", 3, 31, 100), ("bf16", 4, 256, 256)])
def test_conv_replay_matches_commit_then_conv(st, oracle, io, W, N, Np):
    """Tree conv seeded by the conv state after the previous tree's accepted path, and that state."""
    import torch
    B, H, P, S, G = 6, 3, 32, 16, 1
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(40 + W)
    rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    pp, p = _trees(41, B, Np), _trees(42, B, N)
    depth = np.stack([synth.tree_depths(pp[b]) for b in range(B)])
    # accepted: none, the root (one row), a child of the root (two rows), the deepest node, out of range, deep
    acc = np.array([-1, 0, int(np.argmax(depth[2] == 1)), int(depth[3].argmax()), Np + 2, int(depth[5].argmax())],
                   dtype=np.int32)
    pxbc = rnd(rng.standard_normal((B, Np, Cc)).astype(np.float32))
    xbc = rnd(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = rnd(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    w = rnd(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
    bias = rnd(rng.uniform(-0.5, 0.5, Cc).astype(np.float32))
    # oracle: conv part of the commit (state part on dummies), then the conv
    ok = acc < Np
    z = np.zeros((B, Np, 1, 1))
    want_cs = cs.astype(np.float64).copy()
    _, c = oracle.commit(pp[ok], acc[ok], z[ok], np.zeros((ok.sum(), Np, 1)), np.array([-1.0]), z[ok], None,
                         pxbc[ok], cs[ok])
    want_cs[ok] = c
    want = oracle.tree_conv(p, xbc, want_cs, w, bias, True)
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    rstatus = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    got, cso = st.stree_tree_conv_replay(to_dev(pp), to_dev(acc), to_dev(pxbc, io), to_dev(p), to_dev(xbc, io),
                                         to_dev(cs, io), to_dev(w, io), to_dev(bias, io), H, P, S, G, silu=True,
                                         status=status, replay_status=rstatus)
    assert not to_host(status).any()
    assert list(to_host(rstatus)) == [0, 0, 0, 0, -1, 0]
    assert np.array_equal(to_host(cso), want_cs.astype(np.float32))          # row copies: exact
    ulp = 2.0 ** -8 if io == "bf16" else 2.0 ** -22
    assert np.all(np.abs(to_host(got) - want) <= ulp * np.abs(want) + 1e-5)
    # a bad previous tree: the old state is used and passed through
    pp[1, 5] = 7
    got2, cso2 = st.stree_tree_conv_replay(to_dev(pp), to_dev(acc), to_dev(pxbc, io), to_dev(p), to_dev(xbc, io),
                                           to_dev(cs, io), to_dev(w, io), to_dev(bias, io), H, P, S, G, silu=True,
                                           replay_status=rstatus)
    assert int(to_host(rstatus)[1]) == 6
    assert np.array_equal(to_host(cso2)[1], cs[1])
    plain = st.stree_tree_conv(to_dev(p[1:2]), to_dev(xbc[1:2], io), to_dev(cs[1:2], io), to_dev(w, io),
                               to_dev(bias, io), H, P, S, G, silu=True)
    assert np.array_equal(to_host(got2)[1], to_host(plain)[0])


@pytest.mark.parametrize("B", [33, 96])
def test_fused_kernel_equals_commit_then_scan_at_large_batches(st, B):
    """Runs of 6 to 15 units per workgroup, and a unit count that does not divide over the eight
    XCDs: the fused kernel against stree_commit_state followed by stree_tree_ssd on the same
    device inputs (the replay arithmetic is the same chain of fp32 FMAs in path order in both)."""
    import torch
    N, H, P, S, G = 64, 80, 64, 128, 1
    rng = np.random.default_rng(900 + B)
    parent = np.stack([synth.gen_tree(N, int(rng.integers(4, 9)), 4, rng) for _ in range(B)]).astype(np.int32)
    pparent = np.roll(parent, 1, 0).copy()
    acc = rng.integers(-1, N, size=B).astype(np.int32)
    dev = torch.device("cuda")
    gen = torch.Generator(device=dev).manual_seed(901 + B)

    def randn(*shape):
        return torch.randn(shape, device=dev, generator=gen)

    x, px = randn(B, N, H, P).bfloat16(), randn(B, N, H, P).bfloat16()
    Bm, pB, Cm = randn(B, N, G, S).bfloat16(), randn(B, N, G, S).bfloat16(), randn(B, N, G, S).bfloat16()
    dt = torch.rand((B, N, H), device=dev, generator=gen) * 0.1 + 0.01
    pdt = torch.rand((B, N, H), device=dev, generator=gen) * 0.1 + 0.01
    A = -torch.rand(H, device=dev, generator=gen) - 0.5
    D = randn(H)
    h0 = randn(B, H, P, S) * 0.1
    tp, tpp, tacc = to_dev(parent), to_dev(pparent), to_dev(acc)
    y1, h1 = st.stree_tree_ssd_replay(tpp, tacc, px, pdt, pB, tp, x, dt, A, Bm, Cm, D, h0)
    h2, _ = st.stree_commit_state(tpp, tacc, px, pdt, A, pB, h0)
    y2 = st.stree_tree_ssd(tp, x, dt, A, Bm, Cm, D, h2)
    torch.cuda.synchronize()
    eh = ((h1 - h2).abs().max() / h2.abs().max()).item()
    ey = ((y1.float() - y2.float()).abs().max() / y2.float().abs().max()).item()
    assert eh <= 1e-6, f"state: {eh}"
    assert ey <= TOL["bf16"], f"y: {ey}"
