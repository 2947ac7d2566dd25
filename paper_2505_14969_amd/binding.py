"""Thin ctypes binding of libstree.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU, passes their
device pointers and the current HIP stream through the C ABI declared in
``include/stree.h`` and returns the output tensors.  No step of the path is
computed here, and there is no CPU fallback: if the library is missing,
``load()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstree.so")

F32, BF16 = 0, 1
FLAG_CONV_SILU = 1
FLAG_DT_SOFTPLUS = 2
FLAG_FORCE_FMA = 256
FLAG_GENERAL_MFMA = 1024
MAX_NODES = 256


class StreeDims(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "nnodes", "nheads", "headdim", "dstate", "ngroups",
                                         "conv_width", "io_dtype", "state_dtype", "flags")] + \
               [(n, C.c_int64) for n in ("x_stride_n", "b_stride_n", "c_stride_n")] + [("dt_bias", C.c_void_p)]


class StreeReplay(C.Structure):
    _fields_ = [("nnodes", C.c_int32), ("reserved", C.c_int32), ("parent", C.c_void_p), ("accepted", C.c_void_p),
                ("x", C.c_void_p), ("dt", C.c_void_p), ("Bm", C.c_void_p),
                ("x_stride_n", C.c_int64), ("b_stride_n", C.c_int64)]


class StreeError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = load().stree_status_string(code).decode()
        super().__init__(f"{where}: status {code} ({msg})")


_lib = None
_VP = C.c_void_p


def load() -> C.CDLL:
    """Load libstree.so (build it first with ``python -m paper_2505_14969_amd.build``
    or ``__graft_entry__.build()``).  Raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise FileNotFoundError(f"{LIB_PATH} is not built; run paper_2505_14969_amd/build.py")
        lib = C.CDLL(LIB_PATH)
        lib.stree_version.restype = C.c_int
        lib.stree_status_string.restype = C.c_char_p
        lib.stree_status_string.argtypes = [C.c_int]
        lib.stree_workspace_bytes.restype = C.c_size_t
        lib.stree_prepare.restype = C.c_int
        lib.stree_prepare.argtypes = []
        lib.stree_workspace_bytes.argtypes = [C.POINTER(StreeDims)]
        dp = C.POINTER(StreeDims)
        lib.stree_tree_index.argtypes = [dp] + [_VP] * 6
        lib.stree_tree_conv.argtypes = [dp] + [_VP] * 8
        lib.stree_tree_ssd.argtypes = [dp] + [_VP] * 11
        lib.stree_commit_state.argtypes = [dp] + [_VP] * 13
        lib.stree_tree_ssd_replay.argtypes = [dp, C.POINTER(StreeReplay)] + [_VP] * 13
        lib.stree_tree_conv_replay.argtypes = [dp, C.POINTER(StreeReplay)] + [_VP] * 11
        lib.stree_tree_step.argtypes = [dp, C.POINTER(StreeReplay)] + [_VP] * 17
        lib.stree_linear_ssd.argtypes = [dp] + [_VP] * 10
        lib.stree_linear_ssd.restype = C.c_int
        lib.stree_gate_norm.argtypes = [dp, _VP, _VP, C.c_int64, _VP, C.c_float, _VP, _VP]
        lib.stree_gate_norm.restype = C.c_int
        for f in (lib.stree_tree_index, lib.stree_tree_conv, lib.stree_tree_ssd, lib.stree_commit_state,
                  lib.stree_tree_ssd_replay, lib.stree_tree_conv_replay, lib.stree_tree_step):
            f.restype = C.c_int
        _lib = lib
    return _lib


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else _VP(t.data_ptr())


def _stream() -> _VP:
    return _VP(torch.cuda.current_stream().cuda_stream)


def _io_code(t) -> int:
    dt = t.dtype if isinstance(t, torch.Tensor) else t
    if dt == torch.float32:
        return F32
    if dt == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {dt}")


def _state_code(*states) -> int:
    """Type code of the SSM state from the state tensors of a call (those that are given must agree)."""
    dts = {t.dtype for t in states if t is not None}
    assert len(dts) <= 1, "h0 and h_out must have the same dtype"
    return _io_code(next(iter(dts))) if dts else F32


def _token_stride(t: torch.Tensor, nnodes: int) -> int:
    """Element stride between tokens of a [B,N,a,b] view whose last two dims are
    dense and whose batch stride is N * token stride."""
    assert t.dim() == 4 and t.stride(3) == 1 and t.stride(2) == t.shape[3], "inner dims must be dense"
    sn = t.stride(1)
    if nnodes == 1 and t.shape[0] > 1:
        sn = t.stride(0)     # (the stride torch keeps for a dimension of size 1 means nothing)
    assert t.shape[0] == 1 or t.stride(0) == nnodes * sn, "batch stride must be N * token stride"
    return sn


def make_dims(batch, nnodes, nheads, headdim, dstate, ngroups, conv_width=0, io_dtype=BF16, flags=0,
              x_stride_n=0, b_stride_n=0, c_stride_n=0, dt_bias: Optional[torch.Tensor] = None,
              state_dtype=F32) -> StreeDims:
    """`dt_bias` (f32 [H] on the GPU) switches the in-kernel softplus on: the dt arguments of the call are
    then the raw projection and the step size is softplus(dt + dt_bias[h])."""
    if dt_bias is not None:
        assert dt_bias.dtype == torch.float32 and dt_bias.is_contiguous() and dt_bias.numel() == nheads
        flags |= FLAG_DT_SOFTPLUS
    return StreeDims(batch, nnodes, nheads, headdim, dstate, ngroups, conv_width, io_dtype, state_dtype, flags,
                     x_stride_n, b_stride_n, c_stride_n, None if dt_bias is None else dt_bias.data_ptr())


def stree_prepare() -> None:
    """Raise, on the current device, the dynamic-LDS limits that two of the kernels otherwise raise at their
    first launch: afterwards every entry point only launches kernels (what a stream capture wants)."""
    _check(load().stree_prepare(), "stree_prepare")


def stree_workspace_bytes(d: StreeDims) -> int:
    """Device scratch the entry points need for these sizes: 0 for every valid shape."""
    return int(load().stree_workspace_bytes(C.byref(d)))


def _check(rc: int, where: str):
    if rc != 0:
        raise StreeError(rc, where)


def stree_tree_index(parent: torch.Tensor, conv_width: int = 4
                     ) -> Tuple[torch.Tensor, torch.Tensor, torch.Tensor, torch.Tensor]:
    """parent int32 [B,N] -> (depth [B,N], ancmask uint32-as-int32 [B,N,ceil(N/32)],
    anc [B,N,W], status [B])."""
    B, N = parent.shape
    dev = parent.device
    depth = torch.empty((B, N), dtype=torch.int32, device=dev)
    mask = torch.empty((B, N, (N + 31) // 32), dtype=torch.int32, device=dev)
    anc = torch.empty((B, N, conv_width), dtype=torch.int32, device=dev)
    status = torch.empty((B,), dtype=torch.int32, device=dev)
    d = make_dims(B, N, 1, 1, 1, 1, conv_width, F32)
    _check(load().stree_tree_index(C.byref(d), _ptr(parent), _ptr(depth), _ptr(mask), _ptr(anc), _ptr(status),
                                   _stream()), "stree_tree_index")
    return depth, mask, anc, status


def stree_tree_conv(parent, xbc_pre, conv_state, conv_w, conv_b, nheads, headdim, dstate, ngroups,
                    silu: bool = True, out: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None):
    """xbc_pre [B,N,Cc], conv_state [B,W-1,Cc], conv_w [Cc,W], conv_b [Cc]|None -> xbc_out [B,N,Cc]."""
    B, N, Cc = xbc_pre.shape
    W = conv_w.shape[1]
    assert Cc == nheads * headdim + 2 * ngroups * dstate
    assert xbc_pre.is_contiguous() and conv_state.is_contiguous() and conv_w.is_contiguous()
    if out is None:
        out = torch.empty_like(xbc_pre)
    d = make_dims(B, N, nheads, headdim, dstate, ngroups, W, _io_code(xbc_pre), FLAG_CONV_SILU if silu else 0)
    _check(load().stree_tree_conv(C.byref(d), _ptr(parent), _ptr(xbc_pre), _ptr(conv_state), _ptr(conv_w),
                                  _ptr(conv_b), _ptr(out), _ptr(status), _stream()), "stree_tree_conv")
    return out


def stree_tree_ssd(parent, x, dt, A, Bm, Cm, D=None, h0=None, out: Optional[torch.Tensor] = None,
                   status: Optional[torch.Tensor] = None, force_fma: bool = False, general_mfma: bool = False,
                   dt_bias: Optional[torch.Tensor] = None):
    """x [B,N,H,P], dt [B,N,H] f32, A [H] f32, Bm/Cm [B,N,G,S], D [H]|None, h0 [B,H,P,S] f32 or bf16|None
    -> y [B,N,H,P].  x, Bm, Cm may be column views of one [B,N,Cc] buffer.  With dt_bias [H] f32, dt is
    the raw projection and the kernels take softplus(dt + dt_bias[h]) as the step size (here and in
    every function below that has this argument)."""
    B, N, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    if out is None:
        out = torch.empty((B, N, H, P), dtype=x.dtype, device=x.device)
    d = make_dims(B, N, H, P, S, G, 0, _io_code(x),
                  (FLAG_FORCE_FMA if force_fma else 0) | (FLAG_GENERAL_MFMA if general_mfma else 0),
                  _token_stride(x, N), _token_stride(Bm, N), _token_stride(Cm, N), dt_bias, _state_code(h0))
    assert dt.is_contiguous() and dt.dtype == torch.float32 and out.is_contiguous()
    _check(load().stree_tree_ssd(C.byref(d), _ptr(parent), _ptr(x), _ptr(dt), _ptr(A), _ptr(Bm), _ptr(Cm),
                                 _ptr(D), _ptr(h0), _ptr(out), _ptr(status), _stream()), "stree_tree_ssd")
    return out


def stree_commit_state(parent, accepted, x, dt, A, Bm, h0=None, h_out: Optional[torch.Tensor] = None,
                       xbc_pre=None, conv_state=None, conv_state_out: Optional[torch.Tensor] = None,
                       status: Optional[torch.Tensor] = None, dims: Optional[tuple] = None,
                       dt_bias: Optional[torch.Tensor] = None):
    """-> (h_out [B,H,P,S] in the dtype of h0, conv_state_out [B,W-1,Cc] | None).  h_out may be h0 itself
    (in place), conv_state_out may be conv_state itself.  With x, dt, A, Bm all None only the conv
    tail is updated; `dims` = (H, P, S, G) then names the head shapes."""
    if x is None:
        B, N = parent.shape
        H, P, S, G = dims
        W = conv_state.shape[1] + 1
        if conv_state_out is None:
            conv_state_out = torch.empty_like(conv_state)
        d = make_dims(B, N, H, P, S, G, W, _io_code(xbc_pre))
        _check(load().stree_commit_state(C.byref(d), _ptr(parent), _ptr(accepted), None, None, None, None, None,
                                         None, _ptr(xbc_pre), _ptr(conv_state), _ptr(conv_state_out),
                                         _ptr(status), _stream()), "stree_commit_state")
        return None, conv_state_out
    B, N, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    if h_out is None:
        h_out = torch.empty((B, H, P, S), dtype=torch.float32 if h0 is None else h0.dtype, device=x.device)
    W = 0
    if xbc_pre is not None:
        W = conv_state.shape[1] + 1
        if conv_state_out is None:
            conv_state_out = torch.empty_like(conv_state)
    d = make_dims(B, N, H, P, S, G, W, _io_code(x), 0, _token_stride(x, N), _token_stride(Bm, N), 0, dt_bias,
                  _state_code(h0, h_out))
    _check(load().stree_commit_state(C.byref(d), _ptr(parent), _ptr(accepted), _ptr(x), _ptr(dt), _ptr(A),
                                     _ptr(Bm), _ptr(h0), _ptr(h_out), _ptr(xbc_pre), _ptr(conv_state),
                                     _ptr(conv_state_out), _ptr(status), _stream()), "stree_commit_state")
    return h_out, conv_state_out


def stree_tree_ssd_replay(prev_parent, prev_accepted, prev_x, prev_dt, prev_Bm, parent, x, dt, A, Bm, Cm, D, h0,
                          h_out: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                          status: Optional[torch.Tensor] = None, replay_status: Optional[torch.Tensor] = None,
                          force_fma: bool = False, dt_bias: Optional[torch.Tensor] = None):
    """Commit of the previous tree's accepted path fused with the scan of the current tree.
    -> (y [B,N,H,P], h_out [B,H,P,S] in the dtype of h0).  h_out may be h0 itself (in place)."""
    B, N, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    Np = prev_x.shape[1]
    assert prev_x.shape == (B, Np, H, P) and prev_Bm.shape == (B, Np, G, S) and prev_x.dtype == x.dtype
    assert prev_dt.is_contiguous() and prev_dt.dtype == torch.float32 and prev_dt.shape == (B, Np, H)
    assert dt.is_contiguous() and dt.dtype == torch.float32 and h0.is_contiguous()
    if out is None:
        out = torch.empty((B, N, H, P), dtype=x.dtype, device=x.device)
    if h_out is None:
        h_out = torch.empty_like(h0)
    d = make_dims(B, N, H, P, S, G, 0, _io_code(x), FLAG_FORCE_FMA if force_fma else 0,
                  _token_stride(x, N), _token_stride(Bm, N), _token_stride(Cm, N), dt_bias, _state_code(h0, h_out))
    r = StreeReplay(Np, 0, prev_parent.data_ptr(), prev_accepted.data_ptr(), prev_x.data_ptr(), prev_dt.data_ptr(),
                    prev_Bm.data_ptr(), _token_stride(prev_x, Np), _token_stride(prev_Bm, Np))
    _check(load().stree_tree_ssd_replay(C.byref(d), C.byref(r), _ptr(parent), _ptr(x), _ptr(dt), _ptr(A), _ptr(Bm),
                                        _ptr(Cm), _ptr(D), _ptr(h0), _ptr(h_out), _ptr(out), _ptr(status),
                                        _ptr(replay_status), _stream()), "stree_tree_ssd_replay")
    return out, h_out


def stree_tree_conv_replay(prev_parent, prev_accepted, prev_xbc_pre, parent, xbc_pre, conv_state, conv_w, conv_b,
                           nheads, headdim, dstate, ngroups, silu: bool = True, out: Optional[torch.Tensor] = None,
                           conv_state_out: Optional[torch.Tensor] = None, status: Optional[torch.Tensor] = None,
                           replay_status: Optional[torch.Tensor] = None):
    """Tree conv seeded by the conv state after the previous tree's accepted path.
    -> (xbc_out [B,N,Cc], conv_state_out [B,W-1,Cc]); conv_state_out must not be conv_state."""
    B, N, Cc = xbc_pre.shape
    W = conv_w.shape[1]
    Np = prev_xbc_pre.shape[1]
    assert Cc == nheads * headdim + 2 * ngroups * dstate and prev_xbc_pre.shape == (B, Np, Cc)
    assert xbc_pre.is_contiguous() and conv_state.is_contiguous() and conv_w.is_contiguous()
    assert prev_xbc_pre.is_contiguous()
    if out is None:
        out = torch.empty_like(xbc_pre)
    if conv_state_out is None:
        conv_state_out = torch.empty_like(conv_state)
    assert conv_state_out.data_ptr() != conv_state.data_ptr()
    d = make_dims(B, N, nheads, headdim, dstate, ngroups, W, _io_code(xbc_pre), FLAG_CONV_SILU if silu else 0)
    r = StreeReplay(Np, 0, prev_parent.data_ptr(), prev_accepted.data_ptr(), None, None, None, 0, 0)
    _check(load().stree_tree_conv_replay(C.byref(d), C.byref(r), _ptr(prev_xbc_pre), _ptr(parent), _ptr(xbc_pre),
                                         _ptr(conv_state), _ptr(conv_w), _ptr(conv_b), _ptr(out),
                                         _ptr(conv_state_out), _ptr(status), _ptr(replay_status), _stream()),
           "stree_tree_conv_replay")
    return out, conv_state_out


def stree_tree_step(prev_parent, prev_accepted, prev_xbc_pre, prev_xbc_out, prev_dt, parent, xbc_pre, conv_state,
                    conv_w, conv_b, dt, A, D, h0, nheads, headdim, dstate, ngroups, silu: bool = True,
                    xbc_out: Optional[torch.Tensor] = None, conv_state_out: Optional[torch.Tensor] = None,
                    h_out: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None,
                    status: Optional[torch.Tensor] = None, replay_status: Optional[torch.Tensor] = None,
                    force_fma: bool = False, dt_bias: Optional[torch.Tensor] = None):
    """One decoding step in one call: tree conv (seeded by the conv state after the previous tree's
    accepted path), state replay along that path and tree scan.  prev_xbc_out is the previous step's
    conv output [B,Np,Cc] (its x and B columns are replayed; it must not be xbc_out).
    -> (y [B,N,H,P], h_out [B,H,P,S] in the dtype of h0, xbc_out [B,N,Cc], conv_state_out [B,W-1,Cc])."""
    B, N, Cc = xbc_pre.shape
    W = conv_w.shape[1]
    Np = prev_xbc_pre.shape[1]
    H, P, S, G = nheads, headdim, dstate, ngroups
    assert Cc == H * P + 2 * G * S and prev_xbc_pre.shape == (B, Np, Cc) and prev_xbc_out.shape == (B, Np, Cc)
    for t_ in (xbc_pre, conv_state, conv_w, prev_xbc_pre, prev_xbc_out, prev_dt, dt, h0):
        assert t_.is_contiguous()
    assert dt.dtype == torch.float32 and prev_dt.dtype == torch.float32 and prev_dt.shape == (B, Np, H)
    if xbc_out is None:
        xbc_out = torch.empty_like(xbc_pre)
    if conv_state_out is None:
        conv_state_out = torch.empty_like(conv_state)
    if h_out is None:
        h_out = torch.empty_like(h0)
    if out is None:
        out = torch.empty((B, N, H, P), dtype=xbc_pre.dtype, device=xbc_pre.device)
    assert xbc_out.is_contiguous() and out.is_contiguous() and h_out.is_contiguous()
    assert conv_state_out.data_ptr() != conv_state.data_ptr()
    flags = (FLAG_CONV_SILU if silu else 0) | (FLAG_FORCE_FMA if force_fma else 0)
    d = make_dims(B, N, H, P, S, G, W, _io_code(xbc_pre), flags, dt_bias=dt_bias, state_dtype=_state_code(h0, h_out))
    prev_B = prev_xbc_out[:, :, H * P:H * P + G * S]
    r = StreeReplay(Np, 0, prev_parent.data_ptr(), prev_accepted.data_ptr(), prev_xbc_out.data_ptr(),
                    prev_dt.data_ptr(), prev_B.data_ptr(), Cc, Cc)
    _check(load().stree_tree_step(C.byref(d), C.byref(r), _ptr(prev_xbc_pre), _ptr(parent), _ptr(xbc_pre),
                                  _ptr(conv_state), _ptr(conv_w), _ptr(conv_b), _ptr(xbc_out), _ptr(conv_state_out),
                                  _ptr(dt), _ptr(A), _ptr(D), _ptr(h0), _ptr(h_out), _ptr(out), _ptr(status),
                                  _ptr(replay_status), _stream()), "stree_tree_step")
    return out, h_out, xbc_out, conv_state_out


def stree_gate_norm(y, z, norm_w, ngroups: int, eps: float = 1e-5, out: Optional[torch.Tensor] = None):
    """Output gate and grouped RMS norm: y [B,N,H,P] dense, z [B,N,H,P] (may be a column view with its
    own token stride), norm_w [H*P] -> out [B,N,H,P]; out may be y itself."""
    B, N, H, P = y.shape
    assert y.is_contiguous() and z.shape == y.shape and z.dtype == y.dtype and norm_w.numel() == H * P
    if out is None:
        out = torch.empty_like(y)
    d = make_dims(B, N, H, P, 1, ngroups, 0, _io_code(y))
    _check(load().stree_gate_norm(C.byref(d), _ptr(y), _ptr(z), _token_stride(z, N), _ptr(norm_w), C.c_float(eps),
                                  _ptr(out), _stream()), "stree_gate_norm")
    return out


def stree_linear_ssd(x, dt, A, Bm, Cm=None, D=None, h0=None, want_y: bool = True,
                     out: Optional[torch.Tensor] = None, h_out: Optional[torch.Tensor] = None,
                     dt_bias: Optional[torch.Tensor] = None):
    """Causal scan of T tokens per sequence: x [B,T,H,P], dt [B,T,H] f32, Bm/Cm [B,T,G,S].
    -> (y [B,T,H,P] or None, h_out [B,H,P,S] in the dtype of h0).  h_out may be h0 itself."""
    B, T, H, P = x.shape
    G, S = Bm.shape[2], Bm.shape[3]
    assert dt.is_contiguous() and dt.dtype == torch.float32 and dt.shape == (B, T, H)
    if want_y and out is None:
        out = torch.empty((B, T, H, P), dtype=x.dtype, device=x.device)
    if h_out is None:
        h_out = torch.empty((B, H, P, S), dtype=torch.float32 if h0 is None else h0.dtype, device=x.device)
    d = make_dims(B, T, H, P, S, G, 0, _io_code(x), 0, _token_stride(x, T), _token_stride(Bm, T),
                  _token_stride(Cm, T) if Cm is not None else 0, dt_bias, _state_code(h0, h_out))
    _check(load().stree_linear_ssd(C.byref(d), _ptr(x), _ptr(dt), _ptr(A), _ptr(Bm), _ptr(Cm), _ptr(D), _ptr(h0),
                                   _ptr(out) if want_y else None, _ptr(h_out), _stream()), "stree_linear_ssd")
    return (out if want_y else None), h_out
