"""GPU parity on the tree shapes the paper measures (full binary trees of 15/31/63 tokens, beam
trees M x N, static trees): the packed scan against the oracle, and against the same GPU scan on
the tree unrolled into one chain per leaf -- every node of every unrolled path must reproduce the
packed output of that node (the property behind the paper's packed-vs-unrolled comparison)."""
import numpy as np
import pytest

from paper_2505_14969_amd import synth
from helpers import TOL, assert_parity, to_dev, to_host
from test_gpu_parity import _rand, st  # noqa: F401  (fixture)

pytestmark = pytest.mark.gpu

SHAPES = [("binary", 4), ("binary", 5), ("binary", 6), ("static", (3, 4)), ("static", (3, 5)), ("static", (4, 7)),
          ("beam", (2, 4)), ("beam", (3, 8)), ("beam", (5, 16)), ("beam", (4, 16))]


def _tree(kind, arg, rng):
    if kind == "binary":
        return synth.full_binary_tree(arg)
    if kind == "static":
        return synth.static_tree(*arg)
    return synth.beam_tree(arg[0], arg[1], rng)


@pytest.mark.parametrize("kind,arg", SHAPES)
def test_paper_tree_shapes_packed_and_unrolled(st, oracle, kind, arg):
    B, H, P, S, G, io = 2, 4, 64, 128, 1, "bf16"
    rng = np.random.default_rng(123)
    parent = np.stack([_tree(kind, arg, rng) for _ in range(B)]).astype(np.int32)
    N = parent.shape[1]
    x, dt, A, Bm, Cm, D, h0 = _rand(124, io, B, N, H, P, S, G)
    want = oracle.ssd_paths(parent, x, dt, A, Bm, Cm, D, h0)
    got = to_host(st.stree_tree_ssd(to_dev(parent), to_dev(x, io), to_dev(dt), to_dev(A), to_dev(Bm, io),
                                    to_dev(Cm, io), to_dev(D), to_dev(h0)))
    assert_parity(got, want, TOL[io], f"{kind}{arg} packed", kind="y")
    # unrolled: one chain per leaf of sequence 0, its own copy of the state
    ns, nt = oracle.unroll_counts(parent[0])
    has_child = np.zeros(N, dtype=bool)
    has_child[parent[0][parent[0] >= 0]] = True
    for leaf in np.nonzero(~has_child)[0][:6]:
        path, v = [], int(leaf)
        while v >= 0:
            path.append(v)
            v = int(parent[0, v])
        path = path[::-1]
        chain = synth.chain_tree(len(path))[None]
        yu = to_host(st.stree_tree_ssd(to_dev(chain), to_dev(x[:1, path], io), to_dev(dt[:1, path]), to_dev(A),
                                       to_dev(Bm[:1, path], io), to_dev(Cm[:1, path], io), to_dev(D), to_dev(h0[:1])))
        assert_parity(yu[0], want[0, path], TOL[io], f"{kind}{arg} unrolled path to leaf {leaf}", kind="y")
    assert ns == int((~has_child).sum())
