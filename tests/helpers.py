"""Shared helpers for the parity tests: moving seeded numpy inputs to the GPU in
the library's storage types, reading results back, and the parity metric."""
from __future__ import annotations

import numpy as np

from paper_2505_14969_amd import synth

TOL = {"f32": 1e-4, "bf16": 2e-2}


def to_dev(a, io: str = "f32"):
    """numpy fp32 (already rounded when io == 'bf16') -> cuda tensor in storage type."""
    import torch
    if a is None:
        return None
    a = np.ascontiguousarray(a)
    if a.dtype in (np.int32, np.int64):
        return torch.from_numpy(a.astype(np.int32)).cuda()
    if io == "bf16":
        bits = synth.f32_to_bf16_bits(a.astype(np.float32))
        assert np.array_equal(synth.bf16_bits_to_f32(bits), a.astype(np.float32)), "input was not bf16-exact"
        return torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a.astype(np.float32)).cuda()


def to_host(t) -> np.ndarray:
    """cuda tensor (f32 / bf16 / int32) -> numpy (fp32 for floats)."""
    import torch
    if t.dtype == torch.bfloat16:
        return synth.bf16_bits_to_f32(t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16))
    return t.contiguous().cpu().numpy()


def parity(got: np.ndarray, want: np.ndarray):
    """(max-abs error / max-abs reference, l2 error / l2 reference) of one tensor."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.isfinite(got).all(), "non-finite values in the result"
    scale = max(float(np.max(np.abs(want))), 1e-30)
    l2 = max(float(np.linalg.norm(want.ravel())), 1e-30)
    return float(np.max(np.abs(got - want))) / scale, float(np.linalg.norm((got - want).ravel())) / l2


_BLOCK_AXES = {"y": (-3, -1), "state": (-2, -1), None: None}


def elementwise(got: np.ndarray, want: np.ndarray, kind=None) -> float:
    """Worst |err| / (|ref| + rms(ref)), the rms taken over the block an element belongs to:
    kind "y" ([.., N, H, P]): the outputs of one (sequence, head); kind "state" ([.., H, P, S]): the
    state of one (sequence, head); None: the whole tensor.  Unlike the ratio to the tensor's maximum
    this does not let an error hide in a head whose outputs are small next to another head's.  (A
    finer block does not work as a scale: one node's row of y is (dt <C,B> + D) x_i + ..., and where
    that scalar nearly cancels the whole row is small next to the terms whose rounding it carries.)"""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    rms = np.sqrt(np.mean(want * want, axis=_BLOCK_AXES[kind], keepdims=True))
    den = np.abs(want) + rms
    err = np.abs(got - want)
    return float(np.max(np.where(err == 0.0, 0.0, err / np.maximum(den, 1e-300))))


def assert_parity(got, want, tol: float, what: str = "", kind=None, ew_tol=None):
    """Per tensor: max-abs and l2 error relative to the reference's, AND elementwise
    |err| <= ew_tol * (|ref| + rms(ref of the element's block)), see elementwise(); ew_tol = tol
    unless a test states another bound and why."""
    emax, el2 = parity(got, want)
    assert emax <= tol and el2 <= tol, f"{what}: max-rel {emax:.3e}, l2-rel {el2:.3e} > tol {tol:g}"
    ew_tol = tol if ew_tol is None else ew_tol
    ew = elementwise(got, want, kind)
    assert ew <= ew_tol, f"{what}: elementwise |err| / (|ref| + rms) {ew:.3e} > tol {ew_tol:g}"
    return emax, el2


def split_xbc(xbc: np.ndarray, H: int, P: int, G: int, S: int):
    """Column ranges x | B | C of a [B,N,Cc] conv output (numpy views)."""
    B, N, _ = xbc.shape
    x = xbc[:, :, : H * P].reshape(B, N, H, P)
    Bm = xbc[:, :, H * P: H * P + G * S].reshape(B, N, G, S)
    Cm = xbc[:, :, H * P + G * S:].reshape(B, N, G, S)
    return x, Bm, Cm


def split_xbc_dev(xbc, H: int, P: int, G: int, S: int):
    """Same split on a cuda tensor: strided views, no copies."""
    B, N, _ = xbc.shape
    x = xbc[:, :, : H * P].unflatten(2, (H, P))
    Bm = xbc[:, :, H * P: H * P + G * S].unflatten(2, (G, S))
    Cm = xbc[:, :, H * P + G * S:].unflatten(2, (G, S))
    return x, Bm, Cm
