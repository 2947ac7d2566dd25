"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, and rejects bad arguments before launching
anything."""
import ctypes as C
import os
import re

import pytest

from paper_2505_14969_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "stree.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2505_14969_amd import build
        build.build()
    return binding.load()


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "stree.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(stree_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = _declared_symbols()
    assert {"stree_workspace_bytes", "stree_tree_conv", "stree_tree_ssd", "stree_commit_state", "stree_tree_index",
            "stree_version", "stree_status_string"} <= set(names)
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/stree.h but not exported"


def test_dims_struct_matches_header_layout(tmp_path):
    """Sizes and field offsets of the two argument structs: the ctypes mirror against the header itself,
    as the host C compiler lays it out."""
    import subprocess
    fields = {"stree_dims": ["batch", "flags", "x_stride_n", "c_stride_n", "dt_bias"],
              "stree_replay": ["nnodes", "parent", "accepted", "x", "dt", "Bm", "x_stride_n", "b_stride_n"]}
    src = ['#include <stdio.h>', '#include <stddef.h>', f'#include "{HEADER}"', 'int main(void) {']
    for st, fs in fields.items():
        src.append(f'printf("%zu\\n", sizeof({st}));')
        src += [f'printf("%zu\\n", offsetof({st}, {f}));' for f in fs]
    src += ['return 0; }']
    (tmp_path / "layout.c").write_text("\n".join(src))
    subprocess.run(["gcc", "-o", str(tmp_path / "layout"), str(tmp_path / "layout.c")], check=True)
    got = [int(v) for v in subprocess.run([str(tmp_path / "layout")], check=True, capture_output=True,
                                          text=True).stdout.split()]
    want = []
    for st, cls in (("stree_dims", binding.StreeDims), ("stree_replay", binding.StreeReplay)):
        want.append(C.sizeof(cls))
        want += [getattr(cls, f).offset for f in fields[st]]
    assert got == want
    # 10 int32 + 3 int64 + 1 pointer, naturally aligned
    assert C.sizeof(binding.StreeDims) == 10 * 4 + 3 * 8 + 8 and binding.StreeDims.dt_bias.offset == 64


def test_version_and_status_strings(lib):
    assert lib.stree_version() >= 1
    seen = {lib.stree_status_string(c) for c in range(7)}
    assert len(seen) == 7 and all(s for s in seen)
    assert lib.stree_status_string(99) not in seen


def test_workspace_bytes(lib):
    """No kernel uses device scratch: 0 for every valid shape, (size_t)-1 for invalid dims."""
    bad = C.c_size_t(-1).value
    for cfg in (dict(batch=1, nnodes=15, nheads=4, headdim=64, dstate=64, ngroups=1, io_dtype=binding.F32),
                dict(batch=16, nnodes=64, nheads=80, headdim=64, dstate=128, ngroups=1, conv_width=4),
                dict(batch=4, nnodes=256, nheads=128, headdim=64, dstate=128, ngroups=8),
                dict(batch=0, nnodes=1, nheads=1, headdim=1, dstate=1, ngroups=1)):
        assert binding.stree_workspace_bytes(binding.make_dims(**cfg)) == 0
    ok = dict(batch=1, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1)
    assert lib.stree_workspace_bytes(None) == bad
    for k, v in (("nnodes", 0), ("nnodes", 257), ("ngroups", 3), ("dstate", 512), ("batch", -1)):
        assert binding.stree_workspace_bytes(binding.make_dims(**{**ok, k: v})) == bad
    assert binding.stree_workspace_bytes(binding.make_dims(**ok, io_dtype=7)) == bad


FAKE = C.c_void_p(0x1000)   # never dereferenced: every call below fails validation first


def _ssd(lib, d, parent=FAKE, x=FAKE, dt=FAKE, A=FAKE, Bm=FAKE, Cm=FAKE, y=FAKE):
    return lib.stree_tree_ssd(C.byref(d), parent, x, dt, A, Bm, Cm, None, None, y, None, None)


def test_tree_ssd_rejects_bad_arguments(lib):
    ok = dict(batch=1, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1)
    assert lib.stree_tree_ssd(None, *([FAKE] * 6), None, None, FAKE, None, None) == 1
    assert _ssd(lib, binding.make_dims(**ok), x=None) == 1
    assert _ssd(lib, binding.make_dims(**ok), y=None) == 1
    assert _ssd(lib, binding.make_dims(**{**ok, "nnodes": 0})) == 2
    assert _ssd(lib, binding.make_dims(**{**ok, "nnodes": 257})) == 2
    assert _ssd(lib, binding.make_dims(**{**ok, "ngroups": 3})) == 2
    assert _ssd(lib, binding.make_dims(**{**ok, "headdim": 0})) == 2
    assert _ssd(lib, binding.make_dims(**{**ok, "dstate": 512})) == 2
    assert _ssd(lib, binding.make_dims(**{**ok, "batch": -1})) == 2
    assert _ssd(lib, binding.make_dims(**ok, io_dtype=7)) == 3
    d = binding.make_dims(**ok)
    d.state_dtype = 7
    assert _ssd(lib, d) == 3
    d = binding.make_dims(**ok, io_dtype=binding.F32)      # a bf16 state goes with bf16 io only
    d.state_dtype = binding.BF16
    assert _ssd(lib, d) == 3
    assert _ssd(lib, binding.make_dims(**ok, x_stride_n=8)) == 4
    assert _ssd(lib, binding.make_dims(**ok, b_stride_n=64)) == 4
    # the in-kernel softplus needs its bias vector
    assert _ssd(lib, binding.make_dims(**ok, flags=binding.FLAG_DT_SOFTPLUS)) == 1
    # batch 0 is a valid no-op and launches nothing
    assert _ssd(lib, binding.make_dims(**{**ok, "batch": 0})) == 0


def test_tree_conv_rejects_bad_arguments(lib):
    ok = dict(batch=1, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1, conv_width=4)

    def conv(d, out=FAKE):
        return lib.stree_tree_conv(C.byref(d), FAKE, FAKE, FAKE, FAKE, None, out, None, None)

    assert conv(binding.make_dims(**ok), out=None) == 1
    assert conv(binding.make_dims(**{**ok, "conv_width": 1})) == 2
    assert conv(binding.make_dims(**{**ok, "conv_width": 5})) == 2
    assert conv(binding.make_dims(**{**ok, "headdim": 3, "dstate": 1})) == 2   # Cc not a vector multiple
    assert conv(binding.make_dims(**{**ok, "batch": 0})) == 0


def test_commit_rejects_bad_arguments(lib):
    ok = dict(batch=1, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1, conv_width=4)

    def commit(d, accepted=FAKE, h_out=FAKE, xbc=None, cs=None, cso=None):
        return lib.stree_commit_state(C.byref(d), FAKE, accepted, FAKE, FAKE, FAKE, FAKE, None, h_out,
                                      xbc, cs, cso, None, None)

    assert commit(binding.make_dims(**ok), accepted=None) == 1
    assert commit(binding.make_dims(**ok), h_out=None) == 1
    assert commit(binding.make_dims(**ok), xbc=FAKE) == 1            # conv part needs all three
    assert commit(binding.make_dims(**{**ok, "dstate": 30})) == 2
    assert commit(binding.make_dims(**{**ok, "conv_width": 7}), xbc=FAKE, cs=FAKE, cso=FAKE) == 2
    assert commit(binding.make_dims(**{**ok, "batch": 0})) == 0


def test_tree_index_rejects_bad_arguments(lib):
    d = binding.make_dims(1, 300, 1, 1, 1, 1, 4, binding.F32)
    assert lib.stree_tree_index(C.byref(d), FAKE, FAKE, None, None, None, None) == 2
    d = binding.make_dims(1, 30, 1, 1, 1, 1, 9, binding.F32)
    assert lib.stree_tree_index(C.byref(d), FAKE, None, None, FAKE, None, None) == 2
    d = binding.make_dims(1, 30, 1, 1, 1, 1, 4, binding.F32)
    assert lib.stree_tree_index(C.byref(d), None, FAKE, None, None, None, None) == 1


def test_replay_entry_points_reject_bad_arguments(lib):
    ok = dict(batch=1, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1, conv_width=4)
    d = binding.make_dims(**ok)
    prev = binding.StreeReplay(64, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0, 0)

    def ssd(d=d, prev=prev, h0=FAKE, h_out=FAKE, y=FAKE):
        pr = C.byref(prev) if prev is not None else None
        return lib.stree_tree_ssd_replay(C.byref(d), pr, FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, None, h0, h_out, y,
                                         None, None, None)

    assert ssd(prev=None) == 1
    assert ssd(h0=None) == 1 and ssd(h_out=None) == 1 and ssd(y=None) == 1
    assert ssd(prev=binding.StreeReplay(64, 0, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0, 0)) == 1
    assert ssd(prev=binding.StreeReplay(0, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0, 0)) == 2
    assert ssd(prev=binding.StreeReplay(257, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 0, 0)) == 2
    assert ssd(prev=binding.StreeReplay(64, 0, 0x1000, 0x1000, 0x1000, 0x1000, 0x1000, 8, 0)) == 4
    assert ssd(d=binding.make_dims(**{**ok, "dstate": 30})) == 2
    assert ssd(d=binding.make_dims(**{**ok, "batch": 0})) == 0

    def conv(d=d, prev=prev, pxbc=FAKE, cso=FAKE):
        pr = C.byref(prev) if prev is not None else None
        return lib.stree_tree_conv_replay(C.byref(d), pr, pxbc, FAKE, FAKE, FAKE, FAKE, None, FAKE, cso, None, None,
                                          None)

    assert conv(prev=None) == 1 and conv(pxbc=None) == 1 and conv(cso=None) == 1
    assert conv(prev=binding.StreeReplay(300, 0, 0x1000, 0x1000, 0, 0, 0, 0, 0)) == 2
    assert conv(d=binding.make_dims(**{**ok, "conv_width": 5})) == 2
    assert conv(d=binding.make_dims(**{**ok, "batch": 0})) == 0
    # conv tail alone through stree_commit_state: state pointers all NULL
    assert lib.stree_commit_state(C.byref(d), FAKE, FAKE, None, None, None, None, None, None, FAKE, FAKE, None,
                                  None, None) == 1          # conv_state_out missing
    assert lib.stree_commit_state(C.byref(d), FAKE, FAKE, None, None, None, None, None, None, None, None, None,
                                  None, None) == 1          # nothing to do


def test_step_rejects_overlapping_conv_outputs(lib):
    """xbc_out overlapping the previous step's x / B rows is caught on the host (status 6)."""
    ok = dict(batch=2, nnodes=64, nheads=8, headdim=64, dstate=128, ngroups=1, conv_width=4)
    d = binding.make_dims(**ok)
    Cc = 8 * 64 + 2 * 128
    nbytes = 2 * 64 * Cc * 2
    base = 0x100000

    def step(xbc_out, px, pB, d=d):
        prev = binding.StreeReplay(64, 0, 0x1000, 0x1000, px, 0x1000, pB, Cc, Cc)
        return lib.stree_tree_step(C.byref(d), C.byref(prev), FAKE, FAKE, FAKE, FAKE, FAKE, None,
                                   C.c_void_p(xbc_out), FAKE, FAKE, FAKE, None, FAKE, FAKE, FAKE, None, None, None)

    assert step(base, base, base + 8 * 64 * 2) == 6                      # the same buffer
    assert step(base, base + nbytes - 16, base + 4 * nbytes) == 6        # x rows start inside xbc_out
    assert step(base, base + 4 * nbytes, base - 256) == 6                # B rows run into xbc_out
    assert step(base, None, base) == 1                                   # (NULL is reported first)
    assert step(base, base, base, d=binding.make_dims(**{**ok, "batch": 0})) == 0
