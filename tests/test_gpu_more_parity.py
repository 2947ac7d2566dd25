"""More GPU parity cases against the CPU oracle: identity steps (dt = 0) in every scan kernel,
views that are not 16-byte aligned (the vector kernels must hand over to the plain ones and give
the same result), conv width 3 in bf16, the fused replay + scan at a batch whose workgroup runs
are long, and a bounded seeded sweep over random shapes of all entry points."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _run_ssd, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("N,force_fma", [(40, False), (64, False), (64, True), (200, False)])
def test_scan_with_identity_steps(st, oracle, N, force_fma):
    """dt = 0 nodes are identity steps: decay 1, weight 0 (in the MFMA kernels u = +inf, exp2(-inf) = 0)."""
    B, H, P, S, G = 3, 4, 64, 128, 2
    parent = _trees(400 + N, B, N)
    parent[2] = synth.chain_tree(N)
    x, dt, A, Bm, Cm, D, h0 = _rand(401 + N, "bf16", B, N, H, P, S, G)
    dt[0, ::3] = 0.0
    dt[1, N // 2:] = 0.0
    dt[2, 1::2, :2] = 0.0
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, force_fma=force_fma)
    assert_parity(got, want, TOL["bf16"], f"scan with dt = 0 nodes, N={N}", kind="y")
    # all steps zero: y = C h0 + D x, whatever the tree
    z = np.zeros_like(dt)
    want0 = oracle.ssd_paths(parent, x, z, A, Bm, Cm, D, h0)
    got0 = _run_ssd(st, "bf16", parent, x, z, A, Bm, Cm, D, h0, force_fma=force_fma)
    assert_parity(got0, want0, TOL["bf16"], f"scan with dt = 0 everywhere, N={N}", kind="y")


@pytest.mark.parametrize("N", [50, 64, 130])
def test_scan_on_misaligned_views_equals_aligned(st, oracle, N):
    """x / B / C rows that start 4 bytes off a 16-byte boundary, or whose stride is not a whole number
    of 16-byte pieces: the MFMA kernels do not apply, the plain kernel runs; same result as on aligned
    copies to the rounding of y, and within tolerance of the oracle."""
    import torch
    B, H, P, S, G = 2, 3, 64, 128, 1
    parent = _trees(410 + N, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(411 + N, "bf16", B, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    aligned = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0)

    def off_view(a, pad_front, pad_back):
        t = to_dev(a, "bf16")
        Bn, Nn = t.shape[:2]
        row = t.shape[2] * t.shape[3]
        buf = torch.zeros((Bn, Nn, pad_front + row + pad_back), dtype=torch.bfloat16, device="cuda")
        buf[:, :, pad_front:pad_front + row] = t.reshape(Bn, Nn, row)
        return buf[:, :, pad_front:pad_front + row].unflatten(2, (t.shape[2], t.shape[3]))

    for pf, pb in ((2, 6), (0, 3)):                          # 4 bytes off; stride of odd length
        y = st.stree_tree_ssd(to_dev(parent), off_view(x, pf, pb), to_dev(dt), to_dev(A), off_view(Bm, pf, pb),
                              off_view(Cm, pf, pb), to_dev(D), to_dev(h0))
        got = to_host(y)
        assert_parity(got, want, TOL["bf16"], f"scan on a misaligned view ({pf},{pb})", kind="y")
        assert_parity(got, aligned.astype(np.float64), TOL["bf16"], "misaligned vs aligned", kind="y")


def test_replay_and_prefix_with_a_misaligned_state(st, oracle):
    """A state view 4 bytes off a 16-byte boundary: the fused replay + scan and the linear prefix
    kernel read and write the state 16 bytes at a time, so they must not take such a view."""
    import torch
    from paper_2505_14969_amd.binding import StreeError
    io, B, Np, N, H, P, S, G = "bf16", 2, 30, 48, 3, 64, 128, 1
    prev = _rand(420, io, B, Np, H, P, S, G)
    cur = _rand(421, io, B, N, H, P, S, G, h0=False)
    pp, p = _trees(422, B, Np), _trees(423, B, N)
    A, D = prev[2], prev[5]
    acc = np.array([Np - 1, 7], dtype=np.int32)
    px, pdt, _, pB, _, _, h0 = prev
    x, dt, _, Bm, Cm, _, _ = cur
    want_h, _ = oracle.commit(pp, acc, px, pdt, A, pB, h0)
    want_y = oracle.ssd_paths(p, x, dt, A, Bm, Cm, D, want_h)
    flat = torch.zeros(B * H * P * S + 1, dtype=torch.float32, device="cuda")
    flat[1:] = to_dev(h0).reshape(-1)
    h_view = flat[1:].view(B, H, P, S)                       # 4 bytes off
    assert h_view.data_ptr() % 16 == 4
    out = torch.zeros(B * H * P * S + 1, dtype=torch.float32, device="cuda")[1:].view(B, H, P, S)
    y, h = st.stree_tree_ssd_replay(to_dev(pp), to_dev(acc), to_dev(px, io), to_dev(pdt), to_dev(pB, io), to_dev(p),
                                    to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io), to_dev(D),
                                    h_view, h_out=out)
    assert_parity(to_host(h), want_h, 1e-4, "replayed state through misaligned views", kind="state")
    assert_parity(to_host(y), want_y, TOL[io], "scan after replay through misaligned views", kind="y")
    # the linear prefix kernel has no plain variant: it refuses the view
    with pytest.raises(StreeError) as e:
        st.stree_linear_ssd(to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io), None, h_view)
    assert e.value.code == 2


def test_tree_conv_width_3_bf16(st, oracle):
    B, N, H, P, S, G, W = 3, 90, 4, 64, 32, 2, 3
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(430)
    r = synth.round_to_bf16
    parent = _trees(431, B, N)
    xbc = r(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = r(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    w = r(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
    b = r(rng.uniform(-0.5, 0.5, Cc).astype(np.float32))
    for silu, bias in ((True, True), (False, True), (True, False)):
        want = oracle.tree_conv(parent, xbc, cs, w, b if bias else None, silu)
        got = to_host(st.stree_tree_conv(to_dev(parent), to_dev(xbc, "bf16"), to_dev(cs, "bf16"), to_dev(w, "bf16"),
                                         to_dev(b, "bf16") if bias else None, H, P, S, G, silu=silu))
        assert np.all(np.abs(got - want) <= 2.0 ** -8 * np.abs(want) + 1e-5), f"conv W=3 silu={silu} bias={bias}"


def test_fused_replay_scan_long_runs_against_oracle(st, oracle):
    """Batch 33 x 80 heads: 2640 units on 512 workgroups, runs of 5 and 6 units that cross sequences,
    and a unit count that does not divide over the eight XCDs -- against the oracle's commit followed
    by its path-unrolled scan (not against another GPU kernel)."""
    io, B, N, H, P, S, G = "bf16", 33, 64, 80, 64, 128, 1
    rng = np.random.default_rng(933)
    parent = np.stack([synth.gen_tree(N, int(rng.integers(4, 9)), 4, rng) for _ in range(B)]).astype(np.int32)
    pparent = np.roll(parent, 1, 0).copy()
    acc = rng.integers(-1, N, size=B).astype(np.int32)
    prev = _rand(934, io, B, N, H, P, S, G)
    cur = _rand(935, io, B, N, H, P, S, G, h0=False)
    A, D = prev[2], prev[5]
    px, pdt, _, pB, _, _, h0 = prev
    x, dt, _, Bm, Cm, _, _ = cur
    want_h, _ = oracle.commit(pparent, acc, px, pdt, A, pB, h0)
    want_y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, want_h)
    y, h = st.stree_tree_ssd_replay(to_dev(pparent), to_dev(acc), to_dev(px, io), to_dev(pdt), to_dev(pB, io),
                                    to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), to_dev(h0))
    assert_parity(to_host(h), want_h, 1e-4, "replayed state, batch 33", kind="state")
    assert_parity(to_host(y), want_y, TOL[io], "scan after replay, batch 33", kind="y")


def test_seeded_shape_sweep(st, oracle):
    """36 seeded random problems (fixed seeds; stops at the first failure): commit, scan and conv of
    every storage type, head shape, group count, tree size 1..256 and conv width, against the oracle."""
    rng = np.random.default_rng(424242)
    for it in range(36):
        io = "bf16" if it % 4 else "f32"
        P, S = [(64, 128), (64, 64), (128, 128), (32, 64), (64, 256), (32, 16)][int(rng.integers(0, 6))]
        G = int(rng.integers(1, 3))
        H = G * int(rng.integers(1, 4))
        B = int(rng.integers(1, 4))
        N = int(rng.integers(1, 257)) if it % 3 else int(rng.integers(60, 140))
        W = int(rng.integers(2, 5))
        parent = _trees(5000 + it, B, N)
        x, dt, A, Bm, Cm, D, h0 = _rand(6000 + it, io, B, N, H, P, S, G)
        acc = rng.integers(-1, N, B).astype(np.int32)
        tag = f"case {it}: {io} B{B} N{N} H{H} P{P} S{S} G{G} W{W}"
        want_h, _ = oracle.commit(parent, acc, x, dt, A, Bm, h0)
        h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                     to_dev(h0))
        assert_parity(to_host(h), want_h, 1e-4, "commit, " + tag, kind="state")
        want_y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
        y = st.stree_tree_ssd(to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io),
                              to_dev(D), to_dev(h0))
        assert_parity(to_host(y), want_y, TOL[io], "scan, " + tag, kind="y")
        Cc = H * P + 2 * G * S
        rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
        xbc = rnd(rng.standard_normal((B, N, Cc)).astype(np.float32))
        cs = rnd(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
        cw = rnd(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
        cb = rnd(rng.uniform(-0.5, 0.5, Cc).astype(np.float32))
        want_c = oracle.tree_conv(parent, xbc, cs, cw, cb, True)
        c = to_host(st.stree_tree_conv(to_dev(parent), to_dev(xbc, io), to_dev(cs, io), to_dev(cw, io), to_dev(cb, io),
                                       H, P, S, G, silu=True))
        bound = (2.0 ** -8 if io == "bf16" else 2e-5) * np.abs(want_c) + 1e-5
        assert np.all(np.abs(c - want_c) <= bound), "conv, " + tag


@pytest.mark.parametrize("N,kw", [(64, {}), (64, dict(force_fma=True)), (128, {}), (200, {}),
                                  (200, dict(general_mfma=True))])
def test_scan_with_extreme_decay_and_mixed_heads(st, oracle, N, kw):
    """dt A = -50 per node on some heads: every ancestor's contribution and the initial state vanish
    (exp(-50)), y_i = dt_i <C_i,B_i> x_i + D x_i (a closed form the oracle is pinned to), while for
    NON-ancestor pairs exp(s_i - s_j) overflows to +inf after a few levels -- which must be removed by
    the select, never multiplied by zero.  The other heads keep ordinary decays, and some of their
    steps are large (dt = 8: decay factors down to exp(-59))."""
    B, H, P, S, G = 3, 4, 64, 128, 2
    parent = _trees(480 + N, B, N)
    parent[1] = synth.chain_tree(N)
    x, dt, A, Bm, Cm, D, h0 = _rand(481 + N, "bf16", B, N, H, P, S, G)
    A[0] = A[2] = -100.0
    dt[:, :, 0] = dt[:, :, 2] = 0.5
    dt[:, ::5, 1] = 8.0
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    f8 = np.float64
    closed = (dt.astype(f8)[:, :, [0, 2], None] * np.einsum("bngs,bngs->bng", Cm.astype(f8), Bm.astype(f8))[:, :, [0, 1], None]
              + D.astype(f8)[[0, 2]][None, None, :, None]) * x.astype(f8)[:, :, [0, 2]]
    assert np.allclose(want[:, :, [0, 2]], closed, rtol=1e-9, atol=1e-15)
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, **kw)
    assert np.isfinite(got).all()
    assert_parity(got, want, TOL["bf16"], f"scan with extreme decays, N={N} {kw}", kind="y")


def test_commit_replay_and_prefix_scan_with_extreme_decay(st, oracle):
    """The same for the state: on a head with dt A = -50 per node the committed state is dt_k x_k
    (outer) B_k of the accepted node alone, through the commit kernel (both sizes), the fused replay
    and the chunked prefix scan.  (The prefix scan's chunk sums reach 4600 in log2 units there: as a
    difference of prefix sums its weights would be off by 2e-4.)"""
    import torch
    H, P, S, G = 4, 64, 128, 2
    for N in (48, 150):
        B = 3
        parent = _trees(490 + N, B, N)
        x, dt, A, Bm, Cm, D, h0 = _rand(491 + N, "bf16", B, N, H, P, S, G)
        A[1] = -100.0
        dt[:, :, 1] = 0.5
        acc = np.array([N - 1, 0, N // 2], dtype=np.int32)
        want_h, _ = oracle.commit(parent, acc, x, dt, A, Bm, h0, None, None)
        bidx = np.arange(B)
        closed = (dt.astype(np.float64)[bidx, acc, 1][:, None, None] * x.astype(np.float64)[bidx, acc, 1][:, :, None]
                  * Bm.astype(np.float64)[bidx, acc, 0][:, None, :])
        assert np.allclose(want_h[:, 1], closed, rtol=1e-9, atol=1e-15)
        h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, "bf16"), to_dev(dt), to_dev(A),
                                     to_dev(Bm, "bf16"), to_dev(h0))
        got = to_host(h)
        assert np.isfinite(got).all()
        assert_parity(got, want_h, 1e-4, f"commit with an extreme decay, N={N}", kind="state")
        if N <= 64:      # the fused replay + scan of a following tree from that state
            parent2 = _trees(495, B, 40)
            x2, dt2, _, B2, C2, _, _ = _rand(496, "bf16", B, 40, H, P, S, G)
            want_y = oracle.ssd_paths(parent2, x2, dt2, A, B2, C2, D, want_h)
            y, h2 = st.stree_tree_ssd_replay(to_dev(parent), to_dev(acc), to_dev(x, "bf16"), to_dev(dt),
                                             to_dev(Bm, "bf16"), to_dev(parent2), to_dev(x2, "bf16"), to_dev(dt2),
                                             to_dev(A), to_dev(B2, "bf16"), to_dev(C2, "bf16"), to_dev(D), to_dev(h0))
            assert_parity(to_host(h2), want_h, 1e-4, "fused replay with an extreme decay: state", kind="state")
            assert_parity(to_host(y), want_y, TOL["bf16"], "fused replay with an extreme decay: y", kind="y")
    # prefix scan: 300 tokens, one head with dt A = -50 per token, one with large steps
    B, T = 2, 300
    x, dt, A, Bm, Cm, D, h0 = _rand(499, "bf16", B, T, H, P, S, G)
    A[3] = -100.0
    dt[:, :, 3] = 0.5
    dt[:, ::7, 0] = 8.0
    want_y, want_h = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0)
    y, h = st.stree_linear_ssd(to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"), to_dev(Cm, "bf16"),
                               to_dev(D), to_dev(h0))
    assert np.isfinite(to_host(y)).all() and np.isfinite(to_host(h)).all()
    assert_parity(to_host(h), want_h, 1e-4, "prefix scan with extreme decays: state", kind="state")
    assert_parity(to_host(y), want_y, TOL["bf16"], "prefix scan with extreme decays: y", kind="y")
