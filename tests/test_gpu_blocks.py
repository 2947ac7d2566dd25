"""GPU parity of the persistent tree-scan kernel for trees of 65 .. 256 nodes (several node blocks
per unit, several units per workgroup) against the CPU oracle, and against the
one-workgroup-per-unit MFMA kernel that it replaces for these shapes."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, _run_ssd, _trees, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

# (B, N, H, P, S, G): one and several units per workgroup run (the grid stops at 512 workgroups),
# runs that cross a sequence and a group boundary, ragged last blocks, every head shape the kernel takes
SHAPES = [(3, 65, 2, 64, 128, 1), (2, 100, 6, 64, 128, 3), (3, 128, 4, 64, 64, 2), (2, 129, 3, 64, 128, 1),
          (2, 192, 4, 64, 128, 2), (3, 255, 2, 64, 64, 1), (2, 256, 8, 64, 128, 8),
          (9, 70, 64, 64, 128, 4), (5, 130, 120, 64, 128, 1),
          # the wide tiles (one workgroup per CU): dstate 256, headdim 128; more units than workgroups
          (2, 100, 3, 64, 256, 1), (2, 256, 4, 64, 256, 2), (3, 129, 2, 128, 128, 1), (2, 250, 4, 128, 128, 2),
          (5, 70, 60, 128, 128, 2)]


@pytest.mark.parametrize("B,N,H,P,S,G", SHAPES)
def test_blocks_kernel_against_oracle(st, oracle, B, N, H, P, S, G):
    parent = _trees(900 + N + H, B, N)
    parent[B - 1] = synth.chain_tree(N)                  # depth N - 1: the longest pointer-doubling run
    x, dt, A, Bm, Cm, D, h0 = _rand(N + H, "bf16", B, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0)
    for b in range(B):
        assert_parity(got[b], want[b], TOL["bf16"], f"blocks kernel B={B} N={N} H={H} b={b}", kind="y")
    # the one-workgroup-per-unit kernel forms the same products; its decay weights come from expf
    # instead of exp2, so an operand may round to the neighbouring bf16 value
    other = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, general_mfma=True)
    assert_parity(got, other.astype(np.float64), TOL["bf16"], "blocks kernel vs general MFMA kernel", kind="y")


def test_blocks_kernel_optional_arguments_and_zero_steps(st, oracle):
    B, N, H, P, S, G = 2, 150, 4, 64, 128, 2
    parent = _trees(31, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(32, "bf16", B, N, H, P, S, G)
    dt[0, ::7] = 0.0                                     # identity steps: weight exp2(s - inf) = 0, decay 1
    dt[1, 100:] = 0.0
    for Dv, hv in ((None, h0), (D, None), (None, None), (D, h0)):
        want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, Dv, hv)
        got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, Dv, hv)
        assert_parity(got, want, TOL["bf16"], "blocks kernel, optional args / dt = 0", kind="y")


def test_blocks_kernel_bad_tree_zero_fills_that_sequence_only(st, oracle):
    import torch
    B, N, H, P, S, G = 4, 200, 3, 64, 128, 1
    parent = _trees(41, B, N)
    parent[1, 150] = 170                                 # first bad node in the third block
    parent[2, 0] = 5                                     # bad root
    x, dt, A, Bm, Cm, D, h0 = _rand(42, "bf16", B, N, H, P, S, G)
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    got = _run_ssd(st, "bf16", parent, x, dt, A, Bm, Cm, D, h0, status=status)
    assert list(to_host(status)) == [0, 151, 1, 0]
    assert not got[1].any() and not got[2].any()
    keep = [0, 3]
    want = oracle.ssd_paths(parent[keep], x[keep], dt[keep], A, Bm[keep], Cm[keep], D, h0[keep])
    assert_parity(got[keep], want, TOL["bf16"], "good sequences next to bad ones", kind="y")


def test_blocks_kernel_strided_views(st, oracle):
    """x | B | C as column ranges of one buffer (token stride = conv channels)."""
    import torch
    B, N, H, P, S, G = 2, 90, 4, 64, 128, 1
    parent = _trees(51, B, N)
    x, dt, A, Bm, Cm, D, h0 = _rand(52, "bf16", B, N, H, P, S, G)
    Cc = H * P + 2 * G * S
    buf = torch.empty((B, N, Cc), dtype=torch.bfloat16, device="cuda")
    buf[:, :, :H * P] = to_dev(x, "bf16").reshape(B, N, H * P)
    buf[:, :, H * P:H * P + G * S] = to_dev(Bm, "bf16").reshape(B, N, G * S)
    buf[:, :, H * P + G * S:] = to_dev(Cm, "bf16").reshape(B, N, G * S)
    y = st.stree_tree_ssd(to_dev(parent), buf[:, :, :H * P].unflatten(2, (H, P)), to_dev(dt), to_dev(A),
                          buf[:, :, H * P:H * P + G * S].unflatten(2, (G, S)),
                          buf[:, :, H * P + G * S:].unflatten(2, (G, S)), to_dev(D), to_dev(h0))
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    assert_parity(to_host(y), want, TOL["bf16"], "blocks kernel on strided views", kind="y")
