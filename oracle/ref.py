"""ctypes wrapper of the C oracle (``stree_oracle.c``).  TEST INFRASTRUCTURE ONLY.

All tensor arguments are numpy arrays of any float dtype; they are widened to
contiguous fp64 here.  Shapes follow the paper's problem statement (Sec. 3):
packed tree of N nodes given by ``parent`` (root -1, parent[i] < i), per-node
inputs x [B,N,H,P], dt [B,N,H], B/C [B,N,G,S], per-head A, D, initial state
h0 [B,H,P,S].
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Optional, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "stree_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP over (batch, head))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_num_threads.restype = C.c_int
    return _lib


def num_threads() -> int:
    return int(lib().orc_num_threads())


def _f64(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    return None if a is None else np.ascontiguousarray(a, dtype=np.float64)


def _i32(a: np.ndarray) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.int32)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _parent2d(parent: np.ndarray) -> np.ndarray:
    parent = _i32(parent)
    return parent[None, :] if parent.ndim == 1 else parent


def tree_index(parent: np.ndarray, width: int = 4) -> Tuple[int, np.ndarray, np.ndarray, np.ndarray]:
    """One tree.  Returns (status, depth[N], ancmask[N, ceil(N/32)] uint32,
    anc[N, width]); anc[i,k] is the k-th ancestor of i, or -m when the walk is
    m rows above the root."""
    parent = _i32(parent)
    n = parent.shape[0]
    depth = np.zeros(n, dtype=np.int32)
    mask = np.zeros((n, (n + 31) // 32), dtype=np.uint32)
    anc = np.zeros((n, width), dtype=np.int32)
    st = lib().orc_tree_index(C.c_int(n), _p(parent), C.c_int(width), _p(depth), _p(mask), _p(anc))
    return int(st), depth, mask, anc


def unroll_counts(parent: np.ndarray) -> Tuple[int, int]:
    parent = _i32(parent)
    ns, nt = C.c_int64(0), C.c_int64(0)
    st = lib().orc_unroll_counts(C.c_int(parent.shape[0]), _p(parent), C.byref(ns), C.byref(nt))
    if st:
        raise ValueError(f"invalid tree at node {st - 1}")
    return int(ns.value), int(nt.value)


def _ssd_args(parent, x, dt, A, Bm, Cm, D, h0):
    parent = _parent2d(parent)
    x, dt, A, Bm, Cm, D, h0 = map(_f64, (x, dt, A, Bm, Cm, D, h0))
    B, N = parent.shape
    if x.ndim == 3:
        x, dt, Bm, Cm = x[None], dt[None], Bm[None], Cm[None]
        if h0 is not None:
            h0 = h0[None]
    _, _, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    assert x.shape == (B, N, H, P) and dt.shape == (B, N, H) and A.shape == (H,)
    assert Bm.shape == (B, N, G, S) and Cm.shape == (B, N, G, S) and H % G == 0
    assert D is None or D.shape == (H,)
    assert h0 is None or h0.shape == (B, H, P, S)
    return parent, x, dt, A, Bm, Cm, D, h0, (B, N, H, P, S, G)


def ssd_paths(parent, x, dt, A, Bm, Cm, D=None, h0=None, return_rewrite_diff: bool = False):
    """PRIMARY ORACLE: every root-to-leaf path unrolled through the sequential
    recurrence.  Returns y [B,N,H,P] fp64."""
    parent, x, dt, A, Bm, Cm, D, h0, (B, N, H, P, S, G) = _ssd_args(parent, x, dt, A, Bm, Cm, D, h0)
    y = np.full((B, N, H, P), np.nan)
    diff = C.c_double(0.0)
    st = lib().orc_ssd_paths(*(C.c_int(v) for v in (B, N, H, P, S, G)), _p(parent), _p(x), _p(dt), _p(A),
                             _p(Bm), _p(Cm), _p(D), _p(h0), _p(y), C.byref(diff))
    if st:
        raise ValueError(f"invalid tree at node {st - 1}")
    return (y, float(diff.value)) if return_rewrite_diff else y


def ssd_nodes(parent, x, dt, A, Bm, Cm, D=None, h0=None):
    """Second formulation: h_i = a_i h_parent(i) + dt_i x_i (outer) B_i per node."""
    parent, x, dt, A, Bm, Cm, D, h0, (B, N, H, P, S, G) = _ssd_args(parent, x, dt, A, Bm, Cm, D, h0)
    y = np.full((B, N, H, P), np.nan)
    st = lib().orc_ssd_nodes(*(C.c_int(v) for v in (B, N, H, P, S, G)), _p(parent), _p(x), _p(dt), _p(A),
                             _p(Bm), _p(Cm), _p(D), _p(h0), _p(y))
    if st:
        raise ValueError(f"invalid tree at node {st - 1}")
    return y


def linear_scan(x, dt, A, Bm, Cm, D=None, h0=None):
    """Ordinary causal scan of B sequences of length T (no tree code).
    Returns (y [B,T,H,P], h_final [B,H,P,S])."""
    x, dt, A, Bm, Cm, D, h0 = map(_f64, (x, dt, A, Bm, Cm, D, h0))
    B, T, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    assert dt.shape == (B, T, H) and Bm.shape == (B, T, G, S) and Cm.shape == (B, T, G, S) and H % G == 0
    y = np.full((B, T, H, P), np.nan)
    hf = np.full((B, H, P, S), np.nan)
    lib().orc_linear_scan(*(C.c_int(v) for v in (B, T, H, P, S, G)), _p(x), _p(dt), _p(A), _p(Bm), _p(Cm),
                          _p(D), _p(h0), _p(y), _p(hf))
    return y, hf


def tree_conv(parent, xbc_pre, conv_state, w, bias=None, silu: bool = True):
    """Depthwise causal conv along each unrolled path.  xbc_pre [B,N,Cc],
    conv_state [B,W-1,Cc] oldest first, w [Cc,W].  Returns [B,N,Cc] fp64."""
    parent = _parent2d(parent)
    xbc_pre, conv_state, w, bias = map(_f64, (xbc_pre, conv_state, w, bias))
    B, N = parent.shape
    Cc, W = w.shape
    assert xbc_pre.shape == (B, N, Cc) and conv_state.shape == (B, W - 1, Cc)
    out = np.full((B, N, Cc), np.nan)
    st = lib().orc_tree_conv(C.c_int(B), C.c_int(N), C.c_int(Cc), C.c_int(W), _p(parent), _p(xbc_pre),
                             _p(conv_state), _p(w), _p(bias), C.c_int(1 if silu else 0), _p(out))
    if st:
        raise ValueError(f"invalid tree at node {st - 1}")
    return out


def commit(parent, accepted, x, dt, A, Bm, h0=None, xbc_pre=None, conv_state=None):
    """State after the accepted root..k path (k = accepted[b], -1 keeps the
    state) and, when xbc_pre is given, the new conv state.
    Returns (h_out [B,H,P,S], conv_state_out [B,W-1,Cc] or None)."""
    parent = _parent2d(parent)
    accepted = _i32(np.atleast_1d(accepted))
    x, dt, A, Bm, h0, xbc_pre, conv_state = map(_f64, (x, dt, A, Bm, h0, xbc_pre, conv_state))
    B, N = parent.shape
    _, _, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    assert H % G == 0
    h_out = np.full((B, H, P, S), np.nan)
    W = Cc = 0
    cs_out = None
    if xbc_pre is not None:
        W, Cc = conv_state.shape[1] + 1, conv_state.shape[2]
        assert xbc_pre.shape == (B, N, Cc)
        cs_out = np.full((B, W - 1, Cc), np.nan)
    st = lib().orc_commit(*(C.c_int(v) for v in (B, N, H, P, S, G, W, Cc)), _p(parent), _p(accepted), _p(x),
                          _p(dt), _p(A), _p(Bm), _p(h0), _p(h_out), _p(xbc_pre), _p(conv_state), _p(cs_out))
    if st:
        raise ValueError("invalid tree or accepted index")
    return h_out, cs_out


def gate_norm(y, z, w, ngroups: int, eps: float = 1e-5):
    """Output gate and grouped RMS norm of the Mamba2 block behind the scan:
    out = rmsnorm_per_group(y * silu(z)) * w.  y, z [..., H, P] (or [..., d]); w [d];
    groups are ngroups runs of d / ngroups consecutive channels.  Returns y's shape."""
    y, z, w = map(_f64, (y, z, w))
    d = w.shape[0]
    rows = y.size // d
    assert y.shape == z.shape and y.size == rows * d
    out = np.full((rows, d), np.nan)
    st = lib().orc_gate_norm(C.c_int(rows), C.c_int(d), C.c_int(ngroups), _p(y.reshape(rows, d)),
                             _p(z.reshape(rows, d)), _p(w), C.c_double(eps), _p(out))
    if st:
        raise ValueError("ngroups does not divide the channel count")
    return out.reshape(y.shape)


def step_size(raw, bias=None):
    """Step size from the raw projection: softplus(raw + bias[h]) in fp64.  raw [..., H]; bias [H] or None."""
    raw = _f64(raw)
    H = raw.shape[-1]
    bias = None if bias is None else _f64(bias)
    assert bias is None or bias.shape == (H,)
    out = np.full(raw.shape, np.nan)
    lib().orc_step_size(C.c_int(raw.size // H), C.c_int(H), _p(raw), _p(bias), _p(out))
    return out
