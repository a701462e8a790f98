"""Python binding of the offline GQA -> MLA conversion (``include/mla_convert_gfx950.h``).

Argument marshalling only: fp64 torch tensors on the GPU in, device pointers and
the current HIP stream to the C entry point of the same name, output tensors out.
No arithmetic happens here and there is no fallback path.
"""
from __future__ import annotations

import ctypes
from typing import Optional

import torch

from .mla import _check, _stream, lib as _base_lib

EXPORTS = ("mla_conv_project", "mla_conv_rope_moments", "mla_conv_sym_eig_workspace_bytes", "mla_conv_sym_eig",
           "mla_conv_rotate_rows", "mla_conv_kv_balance", "mla_conv_joint_moment",
           "mla_conv_top_eig_workspace_bytes", "mla_conv_top_eig", "mla_conv_apply_workspace_bytes", "mla_conv_apply",
           "mla_convert_layer_workspace_bytes", "mla_convert_layer")

_ready = False


def lib() -> ctypes.CDLL:
    global _ready
    L = _base_lib()
    if not _ready:
        vp, i, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.mla_conv_project.restype = i
        L.mla_conv_project.argtypes = [vp, vp, vp, i, i, i, i, vp]
        L.mla_conv_rope_moments.restype = i
        L.mla_conv_rope_moments.argtypes = [vp, vp, i, i, i, i, vp]
        L.mla_conv_sym_eig_workspace_bytes.restype = sz
        L.mla_conv_sym_eig_workspace_bytes.argtypes = [i, i]
        L.mla_conv_sym_eig.restype = i
        L.mla_conv_sym_eig.argtypes = [vp, vp, vp, sz, vp, i, i, i, vp]
        L.mla_conv_rotate_rows.restype = i
        L.mla_conv_rotate_rows.argtypes = [vp, vp, vp, i, i, i, i, i, vp]
        L.mla_conv_kv_balance.restype = i
        L.mla_conv_kv_balance.argtypes = [vp, i, vp, i, vp, vp, i, i, i, vp]
        L.mla_conv_joint_moment.restype = i
        L.mla_conv_joint_moment.argtypes = [vp, i, vp, i, vp, vp, vp, i, i, i, vp]
        L.mla_conv_top_eig_workspace_bytes.restype = sz
        L.mla_conv_top_eig_workspace_bytes.argtypes = [i, i]
        L.mla_conv_top_eig.restype = i
        L.mla_conv_top_eig.argtypes = [vp, vp, vp, vp, vp, sz, vp, i, i, i, i, vp]
        L.mla_conv_apply_workspace_bytes.restype = sz
        L.mla_conv_apply_workspace_bytes.argtypes = [i, i]
        L.mla_conv_apply.restype = i
        L.mla_conv_apply.argtypes = [vp, vp, vp, vp, sz, i, i, vp]
        L.mla_convert_layer_workspace_bytes.restype = sz
        L.mla_convert_layer_workspace_bytes.argtypes = [i, i, i, i, i, i, i, i, i]
        L.mla_convert_layer.restype = i
        L.mla_convert_layer.argtypes = [vp] * 14 + [vp, sz, vp] + [i] * 10 + [vp]
        _ready = True
    return L


def _f64(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda or t.dtype != torch.float64 or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous float64 GPU tensor")
    return t.data_ptr()


def _new(ref: torch.Tensor, *shape) -> torch.Tensor:
    return torch.empty(shape, dtype=torch.float64, device=ref.device)


def _bytes(ref: torch.Tensor, n: int) -> torch.Tensor:
    return torch.empty(max(int(n), 256), dtype=torch.uint8, device=ref.device)


def project(X: torch.Tensor, W: torch.Tensor) -> torch.Tensor:
    n, D = X.shape
    m = W.shape[0]
    assert W.shape[1] == D
    Y = _new(X, n, m)
    _check(lib().mla_conv_project(_f64(X, "X"), _f64(W, "W"), Y.data_ptr(), n, D, m, m, _stream(X)), "mla_conv_project")
    return Y


def rope_moments(K: torch.Tensor, g: int, d: int, M: int = 1) -> torch.Tensor:
    n = K.shape[0]
    assert K.shape[1] == g * d
    sigma = _new(K, d // (2 * M), M * g, M * g)
    _check(lib().mla_conv_rope_moments(_f64(K, "K"), sigma.data_ptr(), n, g, d, M, _stream(K)), "mla_conv_rope_moments")
    return sigma


def sym_eig(A: torch.Tensor, max_sweeps: int = 60):
    """A [batch, m, m] symmetric (left untouched) -> (evals [batch, m] descending, U [batch, m, m], info [batch])."""
    batch, m, _ = A.shape
    U = A.clone()
    evals = _new(A, batch, m)
    info = torch.empty(batch, dtype=torch.int32, device=A.device)
    nbytes = lib().mla_conv_sym_eig_workspace_bytes(batch, m)
    work = _bytes(A, nbytes)
    _check(lib().mla_conv_sym_eig(_f64(U, "A"), evals.data_ptr(), work.data_ptr(), nbytes, info.data_ptr(),
                                  batch, m, max_sweeps, _stream(A)), "mla_conv_sym_eig")
    return evals, U, info


def rotate_rows(W: torch.Tensor, U: torch.Tensor, g: int, d: int, M: int = 1, keep: Optional[int] = None) -> torch.Tensor:
    assert W.shape[0] == g * d
    out = torch.empty_like(W)
    keep = M if keep is None else keep
    _check(lib().mla_conv_rotate_rows(_f64(W, "W"), _f64(U, "U"), out.data_ptr(), g, d, M, keep, W.shape[1], _stream(W)),
           "mla_conv_rotate_rows")
    return out


def kv_balance(K_nope: torch.Tensor, V: torch.Tensor):
    """-> (alpha [1] on the device, row_norms [2, n])."""
    n, a = K_nope.shape
    b = V.shape[1]
    alpha, norms = _new(V, 1), _new(V, 2, n)
    _check(lib().mla_conv_kv_balance(_f64(K_nope, "K_nope"), a, _f64(V, "V"), b, alpha.data_ptr(), norms.data_ptr(),
                                     n, a, b, _stream(V)), "mla_conv_kv_balance")
    return alpha, norms


def joint_moment(K_nope: torch.Tensor, V: torch.Tensor, alpha: torch.Tensor):
    """-> (S [(a+b), (a+b)], C [n, a+b])."""
    n, a = K_nope.shape
    b = V.shape[1]
    C, S = _new(V, n, a + b), _new(V, a + b, a + b)
    _check(lib().mla_conv_joint_moment(_f64(K_nope, "K_nope"), a, _f64(V, "V"), b, _f64(alpha, "alpha"),
                                       C.data_ptr(), S.data_ptr(), n, a, b, _stream(V)), "mla_conv_joint_moment")
    return S, C


def top_eig(S: torch.Tensor, Q0: torch.Tensor, r: int, iters: int):
    """-> (Ritz values [p] descending, R [m, r], info [2])."""
    m, p = Q0.shape
    assert S.shape == (m, m)
    evals, R = _new(S, p), _new(S, m, r)
    info = torch.empty(2, dtype=torch.int32, device=S.device)
    nbytes = lib().mla_conv_top_eig_workspace_bytes(m, p)
    ws = _bytes(S, nbytes)
    _check(lib().mla_conv_top_eig(_f64(S, "S"), _f64(Q0, "Q0"), evals.data_ptr(), R.data_ptr(), ws.data_ptr(), nbytes,
                                  info.data_ptr(), m, r, p, iters, _stream(S)), "mla_conv_top_eig")
    return evals, R, info


def apply_workspace_bytes(m: int, p: int) -> int:
    return lib().mla_conv_apply_workspace_bytes(m, p)


def apply(S: torch.Tensor, Q: torch.Tensor, out: Optional[torch.Tensor] = None,
          workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    m, p = Q.shape
    assert S.shape == (m, m)
    Y = out if out is not None else _new(S, m, p)
    ws_ptr, ws_bytes = (workspace.data_ptr(), workspace.numel()) if workspace is not None else (None, 0)
    _check(lib().mla_conv_apply(_f64(S, "S"), _f64(Q, "Q"), _f64(Y, "Y"), ws_ptr, ws_bytes, m, p, _stream(S)),
           "mla_conv_apply")
    return Y


def convert_layer(X: torch.Tensor, W_K: torch.Tensor, W_V: torch.Tensor, Q0: torch.Tensor,
                  g: int, h: int, d: int, M: int, r_kv: int, iters: int, workspace: Optional[torch.Tensor] = None,
                  keep: Optional[int] = None):
    """The whole chain; returns a dict of the tensors named in the header.  keep (default M): components per
    FreqFold group that stay under RoPE; the RoPE key is d_rope = keep * d / M wide."""
    n, D = X.shape
    mj, p = Q0.shape
    keep = M if keep is None else keep
    d_rope = keep * (d // M)
    assert W_K.shape == (g * d, D) and W_V.shape == (g * d, D) and mj == 2 * g * d - d_rope
    groups, Mg = d // (2 * M), M * g
    out = dict(W_KR=_new(X, d_rope, D), W_QR=_new(X, h, d_rope, d), W_DKV=_new(X, r_kv, D), W_UK=_new(X, h, d, r_kv),
               W_UV=_new(X, h, r_kv, d), alpha=_new(X, 1), evals_rope=_new(X, groups, Mg), U=_new(X, groups, Mg, Mg),
               evals_joint=_new(X, p), R_KV=_new(X, mj, r_kv),
               info=torch.empty(groups + 2, dtype=torch.int32, device=X.device))
    nbytes = lib().mla_convert_layer_workspace_bytes(n, D, g, h, d, M, keep, r_kv, p)
    ws = workspace if workspace is not None else _bytes(X, nbytes)
    _check(lib().mla_convert_layer(
        _f64(X, "X"), _f64(W_K, "W_K"), _f64(W_V, "W_V"), _f64(Q0, "Q0"),
        out["W_KR"].data_ptr(), out["W_QR"].data_ptr(), out["W_DKV"].data_ptr(), out["W_UK"].data_ptr(),
        out["W_UV"].data_ptr(), out["alpha"].data_ptr(), out["evals_rope"].data_ptr(), out["U"].data_ptr(),
        out["evals_joint"].data_ptr(), out["R_KV"].data_ptr(), ws.data_ptr(), ws.numel(), out["info"].data_ptr(),
        n, D, g, h, d, M, keep, r_kv, p, iters, _stream(X)), "mla_convert_layer")
    return out
