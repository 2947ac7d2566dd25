"""The launch configuration the benchmark times: every kernel of the step captured in a HIP graph
and replayed.  A replay must give what the same calls give when launched directly -- bit for bit,
the arithmetic being the same -- on every replay, also after the inputs were changed in place and
with the program's own eager work and synchronisations between the replays; and the first replay
is checked against the oracle.  Headline shape (batch 16 x 64 nodes, 80 heads x 64, dstate 128) for
the separate and the fused call sequences, a 128-node batch for the kernel of larger trees, and
the gate + norm kernel."""
import numpy as np
import pytest
import torch

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, split_xbc, to_dev, to_host
from test_gpu_parity import _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _capture(fn):
    fn()                                  # first launches outside the capture (one-time kernel attributes)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    torch.cuda.synchronize()
    return g


def _views(xbc, H, P, S, G):
    return (xbc[:, :, :H * P].unflatten(2, (H, P)), xbc[:, :, H * P:H * P + G * S].unflatten(2, (G, S)),
            xbc[:, :, H * P + G * S:].unflatten(2, (G, S)))


def test_graph_replays_of_both_step_sequences_equal_direct_launches(st, oracle):
    wl = synth.config(2)
    B, N, H, P, S, G = wl.batch, wl.nnodes, wl.nheads, wl.headdim, wl.dstate, wl.ngroups
    Cc = wl.conv_channels
    io = "bf16"
    par, acc = to_dev(wl.parent), to_dev(wl.accepted)
    pre, cs = to_dev(wl.xbc_pre, io), to_dev(wl.conv_state, io)
    cw, cb = to_dev(wl.conv_w, io), to_dev(wl.conv_b, io)
    dt, A, D, h0 = to_dev(wl.dt), to_dev(wl.A), to_dev(wl.D), to_dev(wl.h0)
    # the "previous tree" of the fused sequence: the same trees with the batch rolled by one
    ppar, pacc = torch.roll(par, 1, 0).contiguous(), torch.roll(acc, 1, 0).contiguous()
    ppre, pdt = torch.roll(pre, 1, 0).contiguous(), torch.roll(dt, 1, 0).contiguous()
    pxbc = st.stree_tree_conv(ppar, ppre, torch.zeros_like(cs), cw, cb, H, P, S, G, silu=True)
    px, pB, _ = _views(pxbc, H, P, S, G)

    def buffers():
        return dict(xbc=torch.zeros((B, N, Cc), dtype=torch.bfloat16, device="cuda"),
                    y=torch.zeros((B, N, H, P), dtype=torch.bfloat16, device="cuda"),
                    h=torch.zeros((B, H, P, S), dtype=torch.float32, device="cuda"), cso=torch.zeros_like(cs),
                    xbc_f=torch.zeros((B, N, Cc), dtype=torch.bfloat16, device="cuda"),
                    y_f=torch.zeros((B, N, H, P), dtype=torch.bfloat16, device="cuda"),
                    h_f=torch.zeros((B, H, P, S), dtype=torch.float32, device="cuda"), cso_f=torch.zeros_like(cs))

    def step(o):
        # separate: conv -> scan -> commit
        st.stree_tree_conv(par, pre, cs, cw, cb, H, P, S, G, silu=True, out=o["xbc"])
        x, Bm, Cm = _views(o["xbc"], H, P, S, G)
        st.stree_tree_ssd(par, x, dt, A, Bm, Cm, D, h0, out=o["y"])
        st.stree_commit_state(par, acc, x, dt, A, Bm, h0, h_out=o["h"], xbc_pre=pre, conv_state=cs,
                              conv_state_out=o["cso"])
        # fused: conv with the previous tree's conv tail -> scan with the previous tree's state replay
        st.stree_tree_conv_replay(ppar, pacc, ppre, par, pre, cs, cw, cb, H, P, S, G, silu=True, out=o["xbc_f"],
                                  conv_state_out=o["cso_f"])
        xf, Bf, Cf = _views(o["xbc_f"], H, P, S, G)
        st.stree_tree_ssd_replay(ppar, pacc, px, pdt, pB, par, xf, dt, A, Bf, Cf, D, h0, h_out=o["h_f"], out=o["y_f"])

    direct, graphed = buffers(), buffers()
    graph = _capture(lambda: step(graphed))
    for replay in range(3):
        if replay:                        # the inputs change in place: a replay must read them again
            pre.mul_(-1.0)
            dt.mul_(0.5)
            h0.add_(0.25)
        for t in graphed.values():        # eager work of the program between the replays
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        step(direct)
        torch.cuda.synchronize()
        for k in direct:
            assert torch.equal(direct[k], graphed[k]), f"replay {replay}: {k} differs from the direct launch"
        if replay == 0:                   # ... and the direct launch is right: against the oracle
            want_conv = oracle.tree_conv(wl.parent, wl.xbc_pre, wl.conv_state, wl.conv_w, wl.conv_b, True)
            got_conv = to_host(graphed["xbc"])
            assert np.all(np.abs(got_conv - want_conv) <= 2.0 ** -8 * np.abs(want_conv) + 1e-5)
            gx, gB, gC = split_xbc(got_conv, H, P, G, S)
            want_y = oracle.ssd_paths(wl.parent, gx, wl.dt, wl.A, gB, gC, wl.D, wl.h0.astype(np.float64))
            assert_parity(to_host(graphed["y"]), want_y, TOL[io], "graph replay: y", kind="y")
            want_h, want_cs = oracle.commit(wl.parent, wl.accepted, gx, wl.dt, wl.A, gB, wl.h0.astype(np.float64),
                                            wl.xbc_pre, wl.conv_state)
            assert_parity(to_host(graphed["h"]), want_h, 1e-4, "graph replay: committed state", kind="state")
            assert np.array_equal(to_host(graphed["cso"]), want_cs.astype(np.float32))


def test_graph_replays_of_the_large_tree_kernel_and_gate_norm(st, oracle):
    B, N, H, P, S, G = 8, 128, 80, 64, 128, 1
    rng = np.random.default_rng(404)
    r = synth.round_to_bf16
    parent = _trees(405, B, N)
    x = r(rng.standard_normal((B, N, H, P)).astype(np.float32))
    Bm = r(rng.standard_normal((B, N, G, S)).astype(np.float32))
    Cm = r(rng.standard_normal((B, N, G, S)).astype(np.float32))
    z = r(rng.standard_normal((B, N, H, P)).astype(np.float32))
    nw = r(rng.uniform(0.5, 1.5, H * P).astype(np.float32))
    dtn = np.logaddexp(0, rng.standard_normal((B, N, H)) - 2).astype(np.float32)
    An = (-np.exp(rng.uniform(0, 2, H))).astype(np.float32)
    Dn = rng.standard_normal(H).astype(np.float32)
    h0n = (0.1 * rng.standard_normal((B, H, P, S))).astype(np.float32)
    par, xd, Bd, Cd, zd, nwd = to_dev(parent), to_dev(x, "bf16"), to_dev(Bm, "bf16"), to_dev(Cm, "bf16"), \
        to_dev(z, "bf16"), to_dev(nw, "bf16")
    dt, A, D, h0 = to_dev(dtn), to_dev(An), to_dev(Dn), to_dev(h0n)

    def buffers():
        return dict(y=torch.zeros((B, N, H, P), dtype=torch.bfloat16, device="cuda"),
                    yn=torch.zeros((B, N, H, P), dtype=torch.bfloat16, device="cuda"))

    def work(o):
        st.stree_tree_ssd(par, xd, dt, A, Bd, Cd, D, h0, out=o["y"])
        st.stree_gate_norm(o["y"], zd, nwd, G, 1e-5, out=o["yn"])

    direct, graphed = buffers(), buffers()
    graph = _capture(lambda: work(graphed))
    for replay in range(3):
        if replay:
            dt.mul_(0.5)
            h0.add_(0.25)
        for t in graphed.values():
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        work(direct)
        torch.cuda.synchronize()
        for k in direct:
            assert torch.equal(direct[k], graphed[k]), f"replay {replay}: {k} differs from the direct launch"
        if replay == 0:
            want_y = oracle.ssd_paths(parent, x, dtn, An, Bm, Cm, Dn, h0n.astype(np.float64))
            assert_parity(to_host(graphed["y"]), want_y, TOL["bf16"], "graph replay: y (128 nodes)", kind="y")
            got_y = to_host(graphed["y"])
            want_n = oracle.gate_norm(got_y.reshape(B * N, H * P), z.reshape(B * N, H * P), nw, G, 1e-5)
            got_n = to_host(graphed["yn"]).reshape(B * N, H * P)
            assert np.all(np.abs(got_n - want_n) <= 2.0 ** -8 * np.abs(want_n) + 1e-5)


def test_capture_without_a_first_call_after_prepare(st, oracle):
    """stree_prepare raises the dynamic-LDS limits of the two kernels that would otherwise raise them at their
    first launch: after it their very first launch may sit inside a stream capture (run on its own, this test
    is that first launch).  The fp32 kernel at headdim = dstate = 256, its largest LDS tile, and the
    one-workgroup-per-(sequence, head) MFMA kernel on a 256-node tree with headdim 128."""
    from test_gpu_parity import _rand
    st.stree_prepare()
    cases = []
    for io, B, N, H, P, S, G in (("f32", 1, 40, 2, 256, 256, 1), ("bf16", 1, 256, 2, 128, 128, 1)):
        parent = _trees(406 + N, B, N)
        x, dt, A, Bm, Cm, D, h0 = _rand(407 + N, io, B, N, H, P, S, G)
        dev = [to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io), to_dev(D),
               to_dev(h0)]
        out = torch.zeros((B, N, H, P), dtype=dev[1].dtype, device="cuda")
        cases.append((io, parent, (x, dt, A, Bm, Cm, D, h0), dev, out))
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):             # no launch of these kernels before this capture
        for _, _, _, dev, out in cases:
            st.stree_tree_ssd(*dev, out=out)
    torch.cuda.synchronize()
    for replay in range(2):
        for _, _, _, _, out in cases:
            out.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for io, parent, (x, dt, A, Bm, Cm, D, h0), _, out in cases:
            want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
            assert_parity(to_host(out), want, TOL[io], f"captured first launch ({io}), replay {replay}", kind="y")


def test_entry_points_run_on_the_callers_stream(st, oracle):
    """The kernels are enqueued on the stream handed over (here torch's current stream, a non-blocking side
    stream of default priority): their inputs are finished by a long chain of small kernels on that same
    stream, so a launch anywhere else would read them half done."""
    from test_gpu_parity import _rand
    io, B, N, H, P, S, G = "bf16", 4, 64, 8, 64, 128, 1
    parent = _trees(430, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(431, io, B, N, H, P, S, G)
    acc = np.array([N - 1, 3, -1, 20], dtype=np.int32)
    want_y = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    want_h, _ = oracle.commit(parent, acc, x, dt, A, Bm, h0)
    par, accd, Ad, Dd = to_dev(parent), to_dev(acc), to_dev(A), to_dev(D)
    xd, Bd, Cd = to_dev(x, io), to_dev(Bm, io), to_dev(Cm, io)
    steps = 400
    side = torch.cuda.Stream()
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        # a chain of small kernels first; dt and h0 become valid only behind it (h0 even depends on its result)
        dtd = torch.zeros((B, N, H), dtype=torch.float32, device="cuda")
        h0d = torch.zeros((B, H, P, S), dtype=torch.float32, device="cuda")
        junk = torch.zeros_like(h0d)
        for _ in range(steps):
            junk.add_(1.0)
        dtd.copy_(to_dev(dt))             # the inputs become valid only behind the chain
        h0d.copy_(to_dev(h0))
        h0d.add_(junk.sub_(float(steps)))  # + 0 exactly, once the chain is through
        y = st.stree_tree_ssd(par, xd, dtd, Ad, Bd, Cd, Dd, h0d)
        h, _ = st.stree_commit_state(par, accd, xd, dtd, Ad, Bd, h0d)
    side.synchronize()
    assert_parity(to_host(y), want_y, TOL[io], "scan on a side stream", kind="y")
    assert_parity(to_host(h), want_h, 1e-4, "commit on a side stream", kind="state")
