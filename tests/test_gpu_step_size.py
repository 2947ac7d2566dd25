"""The step size taken inside the kernels: with a bias vector the `dt` arguments hold the raw
projection and every kernel uses softplus(dt + bias_h) (Mamba2's discretisation; the recurrence of
Eq. ssm itself has no step size).  Each entry point that reads `dt`, on each of its kernels, against
the oracle fed with the oracle's own fp64 softplus of the same raw values.  The raw values span both
tails: some above 20, where the kernels pass the argument through, some far below zero."""
import numpy as np
import pytest
import torch

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _raw(seed, B, N, H):
    """Raw projection and bias: softplus(raw + bias) mostly in the workload's range (around softplus(-2)),
    a few steps of 21..25 (pass-through branch) and a few of about exp(-30)."""
    rng = np.random.default_rng(seed)
    bias = rng.uniform(-3.0, -1.0, H).astype(np.float32)
    raw = rng.standard_normal((B, N, H)).astype(np.float32)
    pick = rng.random((B, N, H))
    raw = np.where(pick < 0.02, rng.uniform(23.0, 26.0, (B, N, H)), raw)
    raw = np.where(pick > 0.98, -28.0, raw).astype(np.float32)
    return raw, bias


SCAN_CASES = [
    # io, B, N, H, P, S, G, route
    ("bf16", 3, 64, 4, 64, 128, 1, {}),                         # persistent kernel, one node block
    ("bf16", 2, 37, 4, 128, 128, 2, {}),
    ("bf16", 2, 128, 4, 64, 128, 1, {}),                        # persistent kernel over node blocks
    ("bf16", 2, 200, 4, 64, 64, 2, {}),
    ("bf16", 2, 200, 4, 64, 128, 1, {"general_mfma": True}),    # one workgroup per (sequence, head)
    ("bf16", 2, 50, 3, 32, 64, 1, {}),
    ("bf16", 2, 90, 3, 64, 128, 1, {"force_fma": True}),        # fp32 FMA kernel, bf16 storage
    ("f32", 2, 15, 4, 64, 64, 1, {}),                           # fp32 path
]


@pytest.mark.parametrize("io,B,N,H,P,S,G,route", SCAN_CASES)
def test_scan_takes_softplus_of_raw_dt(st, oracle, io, B, N, H, P, S, G, route):
    parent = _trees(8100 + N, B, N)
    x, _, A, Bm, Cm, D, h0 = _rand(8200 + N, io, B, N, H, P, S, G)
    raw, bias = _raw(8300 + N, B, N, H)
    want = oracle.ssd_paths(parent, x, oracle.step_size(raw, bias), A, Bm, Cm, D, h0)
    y = st.stree_tree_ssd(to_dev(parent), to_dev(x, io), to_dev(raw), to_dev(A), to_dev(Bm, io), to_dev(Cm, io),
                          to_dev(D), to_dev(h0), dt_bias=to_dev(bias), **route)
    assert_parity(to_host(y), want, TOL[io], f"y, raw dt, N={N} {route}", kind="y")


@pytest.mark.parametrize("io,B,N,H,P,S,G", [("bf16", 3, 64, 4, 64, 128, 1), ("bf16", 2, 150, 4, 64, 128, 2),
                                            ("f32", 2, 40, 3, 32, 48, 1), ("bf16", 2, 256, 2, 128, 128, 1)])
def test_commit_takes_softplus_of_raw_dt(st, oracle, io, B, N, H, P, S, G):
    parent = _trees(8400 + N, B, N)
    x, _, A, Bm, _, _, h0 = _rand(8500 + N, io, B, N, H, P, S, G)
    raw, bias = _raw(8600 + N, B, N, H)
    acc = np.array([N - 1, N // 2, -1][:B], dtype=np.int32)
    want, _ = oracle.commit(parent, acc, x, oracle.step_size(raw, bias), A, Bm, h0)
    h, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, io), to_dev(raw), to_dev(A), to_dev(Bm, io),
                                 to_dev(h0), dt_bias=to_dev(bias))
    assert_parity(to_host(h), want, 1e-4, f"committed state, raw dt, N={N}", kind="state")


@pytest.mark.parametrize("Np,N", [(64, 64), (23, 50), (100, 40), (30, 130)])
def test_replay_and_step_take_softplus_of_raw_dt(st, oracle, Np, N):
    """The fused replay + scan (both trees within 64 nodes: one kernel; otherwise two), and the whole step in
    one call, which must equal the two fused calls bit for bit."""
    B, H, P, S, G, W = 3, 4, 64, 128, 1, 4
    io = "bf16"
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(8700 + N)
    r = synth.round_to_bf16
    pparent, parent = _trees(8701 + Np, B, Np), _trees(8702 + N, B, N)
    px, _, A, pB, _, D, h0 = _rand(8703 + Np, io, B, Np, H, P, S, G)
    x, _, _, Bm, Cm, _, _ = _rand(8704 + N, io, B, N, H, P, S, G)
    praw, bias = _raw(8705 + Np, B, Np, H)
    raw, _ = _raw(8706 + N, B, N, H)
    acc = np.array([Np - 1, Np // 3, -1], dtype=np.int32)
    h_want, _ = oracle.commit(pparent, acc, px, oracle.step_size(praw, bias), A, pB, h0)
    y_want = oracle.ssd_paths(parent, x, oracle.step_size(raw, bias), A, Bm, Cm, D, h_want)
    y, h = st.stree_tree_ssd_replay(to_dev(pparent), to_dev(acc), to_dev(px, io), to_dev(praw), to_dev(pB, io),
                                    to_dev(parent), to_dev(x, io), to_dev(raw), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), to_dev(h0), dt_bias=to_dev(bias))
    assert_parity(to_host(h), h_want, 1e-4, f"replayed state, raw dt, {Np}->{N}", kind="state")
    assert_parity(to_host(y), y_want, TOL[io], f"y after replay, raw dt, {Np}->{N}", kind="y")

    # the step in one call on conv inputs: equal to conv_replay followed by ssd_replay with the same bias
    ppre = r(rng.standard_normal((B, Np, Cc)).astype(np.float32))
    pre = r(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = r(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    cw = r(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
    cb = r(rng.uniform(-0.5, 0.5, Cc).astype(np.float32))
    d = {k: to_dev(v) for k, v in dict(pparent=pparent, parent=parent, acc=acc, praw=praw, raw=raw, A=A, D=D,
                                       h0=h0, bias=bias).items()}
    d.update({k: to_dev(v, io) for k, v in dict(ppre=ppre, pre=pre, cs=cs, cw=cw, cb=cb).items()})
    pout = st.stree_tree_conv(d["pparent"], d["ppre"], torch.zeros_like(d["cs"]), d["cw"], d["cb"], H, P, S, G)
    xbc, cso = st.stree_tree_conv_replay(d["pparent"], d["acc"], d["ppre"], d["parent"], d["pre"], d["cs"], d["cw"],
                                         d["cb"], H, P, S, G)
    cols = lambda t: (t[:, :, :H * P].unflatten(2, (H, P)), t[:, :, H * P:H * P + G * S].unflatten(2, (G, S)),  # noqa: E731
                      t[:, :, H * P + G * S:].unflatten(2, (G, S)))
    (pxv, pBv, _), (xv, Bv, Cv) = cols(pout), cols(xbc)
    y2, h2 = st.stree_tree_ssd_replay(d["pparent"], d["acc"], pxv, d["praw"], pBv, d["parent"], xv, d["raw"], d["A"],
                                      Bv, Cv, d["D"], d["h0"], dt_bias=d["bias"])
    y1, h1, xbc1, cso1 = st.stree_tree_step(d["pparent"], d["acc"], d["ppre"], pout, d["praw"], d["parent"], d["pre"],
                                            d["cs"], d["cw"], d["cb"], d["raw"], d["A"], d["D"], d["h0"], H, P, S, G,
                                            dt_bias=d["bias"])
    assert torch.equal(y1, y2) and torch.equal(h1, h2) and torch.equal(xbc1, xbc) and torch.equal(cso1, cso)
    # ... and it did read the bias: without it the raw values are step sizes (negative ones included)
    y3, _ = st.stree_tree_ssd_replay(d["pparent"], d["acc"], pxv, d["praw"], pBv, d["parent"], xv, d["raw"], d["A"],
                                     Bv, Cv, d["D"], d["h0"])
    assert not torch.equal(y3, y2)


@pytest.mark.parametrize("want_y", [True, False])
def test_linear_scan_takes_softplus_of_raw_dt(st, oracle, want_y):
    B, T, H, P, S, G = 2, 300, 3, 64, 128, 1
    x, _, A, Bm, Cm, D, h0 = _rand(8800, "bf16", B, T, H, P, S, G)
    raw, bias = _raw(8801, B, T, H)
    y_want, h_want = oracle.linear_scan(x, oracle.step_size(raw, bias), A, Bm, Cm, D, h0)
    y, h = st.stree_linear_ssd(to_dev(x, "bf16"), to_dev(raw), to_dev(A), to_dev(Bm, "bf16"),
                               to_dev(Cm, "bf16") if want_y else None, to_dev(D) if want_y else None, to_dev(h0),
                               want_y=want_y, dt_bias=to_dev(bias))
    assert_parity(to_host(h), h_want, 1e-4, "linear scan state, raw dt", kind="state")
    if want_y:
        assert_parity(to_host(y), y_want, TOL["bf16"], "linear scan y, raw dt", kind="y")
