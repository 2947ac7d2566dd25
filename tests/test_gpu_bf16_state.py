"""The SSM state kept in bf16 (`state_dtype`): h0 is widened exactly when read, all arithmetic stays
fp32, and a new state is rounded to nearest even once, when written.  So against the oracle on the
same (bf16-exact) initial state: y keeps the tolerance of the bf16 path, and a state that the library
writes is the oracle's within one bf16 rounding (2^-8 relative, element by element) on top of the
fp32 tolerance of the state (1e-4 of its largest element).  Every entry point that touches the state,
on each of its kernels."""
import numpy as np
import pytest
import torch

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _assert_rounded_state(got, want, what):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    assert np.isfinite(got).all()
    bound = 2.0 ** -8 * np.abs(want) * 1.001 + 1e-4 * np.max(np.abs(want))
    worst = np.max(np.abs(got - want) - bound)
    assert worst <= 0, f"{what}: {worst:.3e} beyond one bf16 rounding + 1e-4 of the largest element"


def _inputs(seed, B, N, H, P, S, G):
    x, dt, A, Bm, Cm, D, h0 = _rand(seed, "bf16", B, N, H, P, S, G)
    return x, dt, A, Bm, Cm, D, synth.round_to_bf16(h0)


SCAN_CASES = [
    (3, 64, 4, 64, 128, 1, {}),                         # persistent kernel, one node block
    (2, 37, 4, 128, 128, 2, {}),
    (2, 20, 4, 64, 64, 1, {}),
    (2, 128, 4, 64, 128, 1, {}),                        # persistent kernel over node blocks
    (2, 200, 4, 64, 64, 2, {}),
    (2, 200, 4, 64, 128, 1, {"general_mfma": True}),    # one workgroup per (sequence, head)
    (2, 50, 3, 32, 64, 1, {}),
    (2, 150, 2, 128, 128, 1, {}),
    (2, 64, 3, 64, 256, 1, {}),                         # dstate 256 on the persistent kernels
    (2, 180, 3, 64, 256, 1, {}),
    (2, 90, 3, 64, 128, 1, {"force_fma": True}),        # fp32 FMA kernel
    (2, 30, 3, 24, 40, 1, {}),                          # (a shape only the FMA kernel takes)
]


@pytest.mark.parametrize("B,N,H,P,S,G,route", SCAN_CASES)
def test_scan_from_a_bf16_state(st, oracle, B, N, H, P, S, G, route):
    parent = _trees(9100 + N, B, N)
    x, dt, A, Bm, Cm, D, h0 = _inputs(9200 + N, B, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    y = st.stree_tree_ssd(to_dev(parent), to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"),
                          to_dev(Cm, "bf16"), to_dev(D), to_dev(h0, "bf16"), **route)
    assert_parity(to_host(y), want, TOL["bf16"], f"y from a bf16 state, N={N} {route}", kind="y")
    # the same values handed over in fp32 go through the same arithmetic: the MFMA kernels round the state
    # to bf16 themselves, which changes nothing here
    y32 = st.stree_tree_ssd(to_dev(parent), to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"),
                            to_dev(Cm, "bf16"), to_dev(D), to_dev(h0), **route)
    if not route.get("force_fma") and P in (32, 64, 128) and S % 16 == 0:
        assert torch.equal(y, y32)


@pytest.mark.parametrize("B,N,H,P,S,G", [(3, 64, 4, 64, 128, 1), (3, 40, 4, 128, 128, 2), (2, 150, 4, 64, 128, 2),
                                         (2, 40, 3, 32, 48, 1), (2, 256, 2, 128, 128, 1), (3, 64, 3, 64, 64, 1)])
def test_commit_into_a_bf16_state(st, oracle, B, N, H, P, S, G):
    parent = _trees(9300 + N, B, N)
    x, dt, A, Bm, _, _, h0 = _inputs(9400 + N, B, N, H, P, S, G)
    acc = np.array([N - 1, N // 2, -1][:B], dtype=np.int32)
    want, _ = oracle.commit(parent, acc, x, dt, A, Bm, h0)
    args = (to_dev(parent), to_dev(acc), to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"))
    h0d = to_dev(h0, "bf16")
    h, _ = st.stree_commit_state(*args, h0d)
    assert h.dtype == torch.bfloat16
    _assert_rounded_state(to_host(h), want, f"committed bf16 state, N={N}")
    if B == 3:                                         # accepted = -1: the state passes through bit for bit
        assert torch.equal(h[2], h0d[2])
    hin = h0d.clone()                                  # in place
    st.stree_commit_state(*args, hin, h_out=hin)
    assert torch.equal(hin, h)
    hz, _ = st.stree_commit_state(*args, None, h_out=torch.empty_like(h0d))      # no initial state
    want0, _ = oracle.commit(parent, acc, x, dt, A, Bm, None)
    _assert_rounded_state(to_host(hz), want0, f"committed bf16 state from zero, N={N}")


@pytest.mark.parametrize("Np,N,P,S", [(64, 64, 64, 128), (23, 50, 64, 64), (40, 33, 128, 128), (100, 40, 64, 128),
                                      (30, 130, 64, 128), (50, 60, 64, 256), (40, 140, 64, 256)])
def test_replay_and_step_with_a_bf16_state(st, oracle, Np, N, P, S):
    """Fused replay + scan (one kernel when both trees have at most 64 nodes, otherwise two): the state it
    writes is the oracle's commit within one rounding, and y is the scan FROM THAT ROUNDED STATE (the value
    written back is the value scanned from).  The step in one call equals the two fused calls bit for bit."""
    B, H, G, W = 3, 4, 1, 4
    io = "bf16"
    Cc = H * P + 2 * G * S
    rng = np.random.default_rng(9500 + N)
    r = synth.round_to_bf16
    pparent, parent = _trees(9501 + Np, B, Np), _trees(9502 + N, B, N)
    px, pdt, A, pB, _, D, h0 = _inputs(9503 + Np, B, Np, H, P, S, G)
    x, dt, _, Bm, Cm, _, _ = _inputs(9504 + N, B, N, H, P, S, G)
    acc = np.array([Np - 1, Np // 3, -1], dtype=np.int32)
    h_want, _ = oracle.commit(pparent, acc, px, pdt, A, pB, h0)
    y, h = st.stree_tree_ssd_replay(to_dev(pparent), to_dev(acc), to_dev(px, io), to_dev(pdt), to_dev(pB, io),
                                    to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), to_dev(h0, io))
    assert h.dtype == torch.bfloat16
    _assert_rounded_state(to_host(h), h_want, f"replayed bf16 state, {Np}->{N}")
    y_want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, to_host(h))
    assert_parity(to_host(y), y_want, TOL[io], f"y after replay, bf16 state, {Np}->{N}", kind="y")
    # in place
    hin = to_dev(h0, io)
    y_in, _ = st.stree_tree_ssd_replay(to_dev(pparent), to_dev(acc), to_dev(px, io), to_dev(pdt), to_dev(pB, io),
                                       to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                       to_dev(Cm, io), to_dev(D), hin, h_out=hin)
    assert torch.equal(hin, h) and torch.equal(y_in, y)

    ppre = r(rng.standard_normal((B, Np, Cc)).astype(np.float32))
    pre = r(rng.standard_normal((B, N, Cc)).astype(np.float32))
    cs = r(rng.standard_normal((B, W - 1, Cc)).astype(np.float32))
    cw = r(rng.uniform(-0.5, 0.5, (Cc, W)).astype(np.float32))
    cb = r(rng.uniform(-0.5, 0.5, Cc).astype(np.float32))
    d = {k: to_dev(v) for k, v in dict(pparent=pparent, parent=parent, acc=acc, pdt=pdt, dt=dt, A=A, D=D).items()}
    d.update({k: to_dev(v, io) for k, v in dict(ppre=ppre, pre=pre, cs=cs, cw=cw, cb=cb, h0=h0).items()})
    pout = st.stree_tree_conv(d["pparent"], d["ppre"], torch.zeros_like(d["cs"]), d["cw"], d["cb"], H, P, S, G)
    xbc, cso = st.stree_tree_conv_replay(d["pparent"], d["acc"], d["ppre"], d["parent"], d["pre"], d["cs"], d["cw"],
                                         d["cb"], H, P, S, G)
    cols = lambda t: (t[:, :, :H * P].unflatten(2, (H, P)), t[:, :, H * P:H * P + G * S].unflatten(2, (G, S)),  # noqa: E731
                      t[:, :, H * P + G * S:].unflatten(2, (G, S)))
    (pxv, pBv, _), (xv, Bv, Cv) = cols(pout), cols(xbc)
    y2, h2 = st.stree_tree_ssd_replay(d["pparent"], d["acc"], pxv, d["pdt"], pBv, d["parent"], xv, d["dt"], d["A"],
                                      Bv, Cv, d["D"], d["h0"])
    y1, h1, xbc1, cso1 = st.stree_tree_step(d["pparent"], d["acc"], d["ppre"], pout, d["pdt"], d["parent"], d["pre"],
                                            d["cs"], d["cw"], d["cb"], d["dt"], d["A"], d["D"], d["h0"], H, P, S, G)
    assert h1.dtype == torch.bfloat16
    assert torch.equal(y1, y2) and torch.equal(h1, h2) and torch.equal(xbc1, xbc) and torch.equal(cso1, cso)


@pytest.mark.parametrize("P,S,T,with_h0,want_y", [(64, 128, 300, True, True), (64, 64, 129, False, True),
                                                  (128, 128, 64, True, False), (64, 256, 200, True, True)])
def test_linear_scan_with_a_bf16_state(st, oracle, P, S, T, with_h0, want_y):
    B, H, G = 2, 3, 1
    x, dt, A, Bm, Cm, D, h0 = _inputs(9600 + T, B, T, H, P, S, G)
    y_want, h_want = oracle.linear_scan(x, dt, A, Bm, Cm, D, h0 if with_h0 else None)
    y, h = st.stree_linear_ssd(to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"),
                               to_dev(Cm, "bf16") if want_y else None, to_dev(D) if want_y else None,
                               to_dev(h0, "bf16") if with_h0 else None, want_y=want_y,
                               h_out=torch.empty((B, H, P, S), dtype=torch.bfloat16, device="cuda"))
    _assert_rounded_state(to_host(h), h_want, f"linear scan, bf16 state, T={T}")
    if want_y:
        assert_parity(to_host(y), y_want, TOL["bf16"], f"linear scan y, bf16 state, T={T}", kind="y")


def test_three_iterations_with_a_bf16_state_stay_within_three_roundings(st, oracle):
    """Commit, commit, commit: each iteration rounds the state once more, so against the oracle carrying the
    state in fp64 the error grows by at most one rounding of the (decayed) state per iteration."""
    B, N, H, P, S, G = 2, 48, 4, 64, 128, 1
    _, _, A, _, _, _, h0 = _inputs(9700, B, N, H, P, S, G)
    hd, hw = to_dev(h0, "bf16"), h0.astype(np.float64)
    scale = 0.0
    for it in range(3):
        parent = _trees(9710 + it, B, N)
        x, dt, _, Bm, _, _, _ = _inputs(9720 + it, B, N, H, P, S, G)
        acc = np.array([N - 1 - it, 5 + it], dtype=np.int32)
        hw, _ = oracle.commit(parent, acc, x, dt, A, Bm, hw)
        hd, _ = st.stree_commit_state(to_dev(parent), to_dev(acc), to_dev(x, "bf16"), to_dev(dt), to_dev(A),
                                      to_dev(Bm, "bf16"), hd)
        scale = max(scale, float(np.max(np.abs(hw))))
        err = np.abs(to_host(hd).astype(np.float64) - hw)
        # a rounding of an earlier iteration is at most 2^-8 of that state's largest element, and decays
        assert np.max(err) <= (it + 1) * 2.0 ** -8 * scale * 1.01 + 1e-4 * scale, (it, np.max(err), scale)


def test_bf16_state_needs_bf16_io(st):
    B, N, H, P, S, G = 1, 15, 2, 64, 64, 1
    parent = to_dev(_trees(9800, B, N))
    x, dt, A, Bm, Cm, D, h0 = _rand(9801, "f32", B, N, H, P, S, G)
    with pytest.raises(Exception, match="dtype"):
        st.stree_tree_ssd(parent, to_dev(x), to_dev(dt), to_dev(A), to_dev(Bm), to_dev(Cm), to_dev(D),
                          to_dev(synth.round_to_bf16(h0), "bf16"))


def test_bf16_state_must_start_on_a_16_byte_boundary(st):
    """Every kernel moves a bf16 state 8 or 16 bytes at a time: a view that starts elsewhere is refused on the
    host, before anything is launched (the output keeps its fill)."""
    from paper_2505_14969_amd.binding import StreeError
    B, N, H, P, S, G = 1, 20, 2, 64, 64, 1
    parent = to_dev(_trees(9900, B, N))
    x, dt, A, Bm, Cm, D, h0 = _inputs(9901, B, N, H, P, S, G)
    flat = torch.zeros(B * H * P * S + 1, dtype=torch.bfloat16, device="cuda")
    flat[1:] = to_dev(h0, "bf16").reshape(-1)
    h_view = flat[1:].view(B, H, P, S)                       # 2 bytes off
    out = torch.full((B, N, H, P), 7.0, dtype=torch.bfloat16, device="cuda")
    with pytest.raises(StreeError) as e:
        st.stree_tree_ssd(parent, to_dev(x, "bf16"), to_dev(dt), to_dev(A), to_dev(Bm, "bf16"), to_dev(Cm, "bf16"),
                          to_dev(D), h_view, out=out)
    assert e.value.code == 2
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())


@pytest.mark.parametrize("Np,N", [(50, 64), (90, 140)])
def test_bf16_state_together_with_the_in_kernel_step_size(st, oracle, Np, N):
    """Both variants at once (raw dt + bias, state in bf16) through the fused replay + scan: one kernel for
    trees of at most 64 nodes, commit followed by the scan kernel of larger trees otherwise."""
    B, H, P, S, G = 2, 4, 64, 128, 1
    io = "bf16"
    rng = np.random.default_rng(9950 + N)
    pparent, parent = _trees(9951 + Np, B, Np), _trees(9952 + N, B, N)
    px, _, A, pB, _, D, h0 = _inputs(9953 + Np, B, Np, H, P, S, G)
    x, _, _, Bm, Cm, _, _ = _inputs(9954 + N, B, N, H, P, S, G)
    praw = rng.standard_normal((B, Np, H)).astype(np.float32)
    raw = rng.standard_normal((B, N, H)).astype(np.float32)
    bias = rng.uniform(-3.0, -1.0, H).astype(np.float32)
    acc = np.array([Np - 1, Np // 2], dtype=np.int32)
    h_want, _ = oracle.commit(pparent, acc, px, oracle.step_size(praw, bias), A, pB, h0)
    y, h = st.stree_tree_ssd_replay(to_dev(pparent), to_dev(acc), to_dev(px, io), to_dev(praw), to_dev(pB, io),
                                    to_dev(parent), to_dev(x, io), to_dev(raw), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), to_dev(h0, io), dt_bias=to_dev(bias))
    _assert_rounded_state(to_host(h), h_want, f"replayed bf16 state, raw dt, {Np}->{N}")
    y_want = oracle.ssd_paths(parent, x, oracle.step_size(raw, bias), A, Bm, Cm, D, to_host(h))
    assert_parity(to_host(y), y_want, TOL[io], f"y, bf16 state and raw dt, {Np}->{N}", kind="y")
