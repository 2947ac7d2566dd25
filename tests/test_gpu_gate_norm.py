"""GPU parity of the output gate + grouped RMS norm behind the scan (stree_gate_norm) against the
CPU oracle's orc_gate_norm on the same seeded inputs."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu


def _inputs(seed, io, B, N, H, P):
    rng = np.random.default_rng(seed)
    rnd = synth.round_to_bf16 if io == "bf16" else (lambda a: a.astype(np.float32))
    y = rnd((2.0 * rng.standard_normal((B, N, H, P))).astype(np.float32))
    z = rnd((1.5 * rng.standard_normal((B, N, H, P))).astype(np.float32))
    w = rnd(rng.uniform(0.5, 1.5, H * P).astype(np.float32))
    return y, z, w


def _check(got, want, io, what):
    assert_parity(got, want, TOL[io], what)
    # fp32 arithmetic and one rounding of the result: elementwise, not only per tensor
    bound = (2.0 ** -8 if io == "bf16" else 2e-5) * np.abs(want) + 1e-5
    assert np.all(np.abs(got - want) <= bound), f"{what}: worst {np.max(np.abs(got - want) - bound):.3e} over the bound"


# (io, B, N, H, P, G): the headline layer shape at full size (one group of 5120 channels: three
# 16-byte pieces per thread), the 8-group shape, one head per group, fp32 storage, and group sizes
# that are not whole 16-byte pieces (the plain two-pass kernel)
SHAPES = [("bf16", 16, 64, 80, 64, 1), ("bf16", 4, 256, 128, 64, 8), ("bf16", 3, 5, 8, 64, 8), ("f32", 2, 15, 4, 64, 2),
          ("bf16", 2, 7, 3, 20, 3), ("f32", 2, 9, 5, 3, 1), ("bf16", 1, 3, 160, 64, 1), ("bf16", 1, 2, 320, 64, 1)]


@pytest.mark.parametrize("io,B,N,H,P,G", SHAPES)
def test_gate_norm_against_oracle(st, oracle, io, B, N, H, P, G):
    y, z, w = _inputs(B * 100 + H, io, B, N, H, P)
    want = oracle.gate_norm(y, z, w, G, 1e-5)
    got = to_host(st.stree_gate_norm(to_dev(y, io), to_dev(z, io), to_dev(w, io), G, 1e-5))
    _check(got, want, io, f"gate + norm {io} B={B} N={N} H={H} P={P} G={G}")


def test_gate_norm_strided_z_in_place_and_eps(st, oracle):
    """z as a column range of a wider buffer (the input projection's output), the result written over
    y, and eps = 0 with a closed gate elsewhere: z = 0 rows give zeros, not NaN, when eps > 0."""
    import torch
    io, B, N, H, P, G = "bf16", 2, 33, 8, 64, 2
    y, z, w = _inputs(5, io, B, N, H, P)
    z[1, 4] = 0.0                                            # the gate closed for a whole node
    d = H * P
    wide = torch.zeros((B, N, 2 * d + 24), dtype=torch.bfloat16, device="cuda")
    wide[:, :, 16:16 + d] = to_dev(z, io).reshape(B, N, d)
    zv = wide[:, :, 16:16 + d].unflatten(2, (H, P))
    y_io = to_dev(y, io)
    out = st.stree_gate_norm(y_io, zv, to_dev(w, io), G, 1e-5, out=y_io)
    assert out.data_ptr() == y_io.data_ptr()
    got = to_host(out)
    _check(got, oracle.gate_norm(y, z, w, G, 1e-5), io, "gate + norm in place, strided z")
    assert not got[1, 4].any()
    # a z view whose stride is not a whole number of 16-byte pieces takes the plain kernel: same result
    odd = torch.zeros((B, N, d + 3), dtype=torch.bfloat16, device="cuda")
    odd[:, :, :d] = to_dev(z, io).reshape(B, N, d)
    got2 = to_host(st.stree_gate_norm(to_dev(y, io), odd[:, :, :d].unflatten(2, (H, P)), to_dev(w, io), G, 1e-5))
    assert_parity(got2, got.astype(np.float64), 2.0 ** -7, "plain kernel vs single-pass kernel")


def test_scan_then_gate_norm(st, oracle):
    """The scan's own y (a 100-node tree: the multi-block kernel) through the gate and the norm, against
    the oracle chain ssd_paths -> round to bf16 -> gate_norm."""
    io, B, N, H, P, S, G = "bf16", 2, 100, 8, 64, 128, 2
    parent = _trees(9, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(10, io, B, N, H, P, S, G)
    _, z, w = _inputs(11, io, B, N, H, P)
    y_dev = st.stree_tree_ssd(to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io), to_dev(Cm, io),
                              to_dev(D), to_dev(h0))
    got = to_host(st.stree_gate_norm(y_dev, to_dev(z, io), to_dev(w, io), G, 1e-5))
    # stage-isolated: the norm checked on the y it actually saw
    _check(got, oracle.gate_norm(to_host(y_dev), z, w, G, 1e-5), io, "gate + norm of the scan's y")
    # end to end against the oracle's own scan
    y_ref = synth.round_to_bf16(oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0).astype(np.float32))
    assert_parity(got, oracle.gate_norm(y_ref, z, w, G, 1e-5), TOL[io], "scan + gate + norm")


def test_gate_norm_rejects_bad_arguments(st):
    import ctypes as C
    lib = st.load()
    d = st.make_dims(2, 8, 4, 64, 1, 1)
    fake = C.c_void_p(0x1000)
    call = lambda y=fake, z=fake, zs=0, w=fake, eps=1e-5, out=fake, dd=d: lib.stree_gate_norm(
        C.byref(dd), y, z, zs, w, C.c_float(eps), out, None)
    assert call(y=None) == 1 and call(z=None) == 1 and call(w=None) == 1 and call(out=None) == 1
    assert call(zs=100) == 4                                  # stride shorter than a row of 256 channels
    assert call(eps=-1.0) == 2
    assert call(dd=st.make_dims(2, 8, 4, 64, 1, 3)) == 2      # groups do not divide the heads
    assert call(dd=st.make_dims(0, 8, 4, 64, 1, 1)) == 0      # empty batch: nothing launched
