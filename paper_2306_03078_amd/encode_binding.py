"""ctypes binding of the quantiser entry points (include/spqr_encode.h): argument marshalling only.

Every step of Alg. 1 runs in the library's kernels; this module allocates the output tensors (torch supplies
device memory and streams) and passes pointers.  No CPU fallback: a missing libspqr.so raises.
"""
from __future__ import annotations

import ctypes as C
from types import SimpleNamespace

import numpy as np

from .binding import SpQRError, _stream_ptr, load_library


class spqr_quantized_t(C.Structure):
    _fields_ = [(k, C.c_void_p) for k in ("Q", "s_q", "z_q", "s_s", "z_s", "s_z", "z_z", "outlier_mask", "outlier_val",
                                          "row_ptr", "W_final")]


_ready = False


def _lib():
    global _ready
    lib = load_library()
    if not _ready:
        i32, vp, dbl, sz = C.c_int32, C.c_void_p, C.c_double, C.c_size_t
        lib.spqr_hessian.restype = C.c_int
        lib.spqr_hessian.argtypes = [vp, i32, i32, vp, vp]
        lib.spqr_inverse_cholesky_workspace_bytes.restype = sz
        lib.spqr_inverse_cholesky_workspace_bytes.argtypes = [i32]
        lib.spqr_inverse_cholesky.restype = C.c_int
        lib.spqr_inverse_cholesky.argtypes = [vp, i32, dbl, vp, vp, sz, vp]
        lib.spqr_quantize_workspace_bytes.restype = sz
        lib.spqr_quantize_workspace_bytes.argtypes = [i32, i32]
        lib.spqr_quantize.restype = C.c_int
        lib.spqr_quantize.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, dbl, C.POINTER(spqr_quantized_t), vp, sz, vp]
        lib.spqr_gather_outliers.restype = C.c_int
        lib.spqr_gather_outliers.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
        lib.spqr_act_order_workspace_bytes.restype = sz
        lib.spqr_act_order_workspace_bytes.argtypes = [i32]
        lib.spqr_act_order.restype = C.c_int
        lib.spqr_act_order.argtypes = [vp, i32, vp, vp, sz, vp]
        lib.spqr_permute_columns.restype = C.c_int
        lib.spqr_permute_columns.argtypes = [vp, i32, i32, vp, vp, vp]
        lib.spqr_permute_symmetric.restype = C.c_int
        lib.spqr_permute_symmetric.argtypes = [vp, i32, vp, vp, vp]
        _ready = True
    return lib


def _check(rc, where):
    if rc != 0:
        raise SpQRError(int(rc), where)


def spqr_hessian(X, stream=None):
    """H[n, n] = 2 X X^T for a float64 device tensor X[n, d] (Alg. 1 line 2)."""
    import torch
    assert X.dtype == torch.float64 and X.is_contiguous() and X.dim() == 2
    n, d = X.shape
    H = torch.empty((n, n), dtype=torch.float64, device=X.device)
    _check(_lib().spqr_hessian(X.data_ptr(), n, d, H.data_ptr(), _stream_ptr(stream)), "spqr_hessian")
    return H


def spqr_inverse_cholesky(H, lam: float, workspace=None, stream=None):
    """The upper triangular H^ic with H^ic^T H^ic = (H + lam I)^-1 (Alg. 1 line 3)."""
    import torch
    assert H.dtype == torch.float64 and H.is_contiguous() and H.dim() == 2 and H.shape[0] == H.shape[1]
    n = int(H.shape[0])
    need = int(_lib().spqr_inverse_cholesky_workspace_bytes(n))
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=H.device)
    U = torch.empty((n, n), dtype=torch.float64, device=H.device)
    _check(_lib().spqr_inverse_cholesky(H.data_ptr(), n, float(lam), U.data_ptr(), workspace.data_ptr(),
                                        workspace.numel(), _stream_ptr(stream)), "spqr_inverse_cholesky")
    return U


def spqr_act_order(H, stream=None):
    """perm (int32 device tensor [n]): the columns in the order of decreasing diag(H), ties to the smaller index."""
    import torch
    assert H.dtype == torch.float64 and H.is_contiguous() and H.dim() == 2 and H.shape[0] == H.shape[1]
    n = int(H.shape[0])
    ws = torch.empty(max(256, int(_lib().spqr_act_order_workspace_bytes(n))), dtype=torch.uint8, device=H.device)
    perm = torch.empty(n, dtype=torch.int32, device=H.device)
    _check(_lib().spqr_act_order(H.data_ptr(), n, perm.data_ptr(), ws.data_ptr(), ws.numel(), _stream_ptr(stream)), "spqr_act_order")
    s = torch.cuda.current_stream() if stream is None else stream
    s.synchronize()                           # the scratch goes out of scope here
    return perm


def spqr_permute_columns(W, perm, stream=None):
    """W[:, perm] for a float64 device tensor W[m, n]."""
    import torch
    assert W.dtype == torch.float64 and W.is_contiguous() and perm.dtype == torch.int32 and perm.numel() == W.shape[1]
    out = torch.empty_like(W)
    _check(_lib().spqr_permute_columns(W.data_ptr(), int(W.shape[0]), int(W.shape[1]), perm.data_ptr(), out.data_ptr(),
                                       _stream_ptr(stream)), "spqr_permute_columns")
    return out


def spqr_permute_symmetric(H, perm, stream=None):
    """H[perm][:, perm] for a float64 device tensor H[n, n]."""
    import torch
    assert H.dtype == torch.float64 and H.is_contiguous() and perm.dtype == torch.int32 and perm.numel() == H.shape[0]
    out = torch.empty_like(H)
    _check(_lib().spqr_permute_symmetric(H.data_ptr(), int(H.shape[0]), perm.data_ptr(), out.data_ptr(), _stream_ptr(stream)),
           "spqr_permute_symmetric")
    return out


def spqr_quantize_device(W, Hic, w_bits, beta1, beta2, tau, s_bits=3, z_bits=3, want_final=True, workspace=None,
                         outputs=None, stream=None):
    """Alg. 1 lines 4-20 on device tensors W[m, n], Hic[n, n] (float64): enqueues the sweep and returns the
    dictionary of output device tensors (see spqr_quantized_t in include/spqr_encode.h).  Asynchronous."""
    import torch
    assert W.dtype == torch.float64 and W.is_contiguous() and Hic.dtype == torch.float64 and Hic.is_contiguous()
    m, n = (int(v) for v in W.shape)
    dev = W.device
    lib = _lib()
    ng, nt = n // max(1, beta1), m // max(1, beta2)
    t = outputs
    if t is None:
        t = dict(Q=torch.empty((m, n), dtype=torch.uint8, device=dev),
                 s_q=torch.empty((m, ng), dtype=torch.uint8, device=dev), z_q=torch.empty((m, ng), dtype=torch.uint8, device=dev),
                 s_s=torch.empty((nt, ng), dtype=torch.float16, device=dev), z_s=torch.empty((nt, ng), dtype=torch.float16, device=dev),
                 s_z=torch.empty((nt, ng), dtype=torch.float16, device=dev), z_z=torch.empty((nt, ng), dtype=torch.float16, device=dev),
                 outlier_mask=torch.empty((m, n), dtype=torch.uint8, device=dev),
                 outlier_val=torch.empty((m, n), dtype=torch.float16, device=dev),
                 row_ptr=torch.empty(m + 1, dtype=torch.int32, device=dev),
                 W_final=torch.empty((m, n), dtype=torch.float64, device=dev) if want_final else None)
    out = spqr_quantized_t(**{k: (None if v is None else v.data_ptr()) for k, v in t.items()})
    need = int(lib.spqr_quantize_workspace_bytes(m, n))
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=dev)
    _check(lib.spqr_quantize(W.data_ptr(), Hic.data_ptr(), m, n, w_bits, s_bits, z_bits, beta1, beta2, float(tau),
                             C.byref(out), workspace.data_ptr(), workspace.numel(), _stream_ptr(stream)), "spqr_quantize")
    t["workspace"] = workspace                # keeps the scratch alive while the kernels run
    return t


def spqr_quantize(W, Hic, w_bits, beta1, beta2, tau, s_bits=3, z_bits=3, want_final=True, workspace=None, stream=None):
    """spqr_quantize_device + spqr_gather_outliers, results copied to the host: the logical SpQR arrays
    (group_axis 0) as NumPy arrays in the form spqr_synth.SpQRLogical / the oracles use, plus W_final."""
    import torch
    m, n = (int(v) for v in W.shape)
    dev = W.device
    lib = _lib()
    t = spqr_quantize_device(W, Hic, w_bits, beta1, beta2, tau, s_bits, z_bits, want_final, workspace, None, stream)
    t.pop("workspace")
    s = torch.cuda.current_stream() if stream is None else stream
    s.synchronize()
    nnz = int(t["row_ptr"][-1].item())
    col = torch.empty(max(nnz, 1), dtype=torch.int16, device=dev)
    val = torch.empty(max(nnz, 1), dtype=torch.float16, device=dev)
    if nnz:
        _check(lib.spqr_gather_outliers(t["outlier_mask"].data_ptr(), t["outlier_val"].data_ptr(), t["row_ptr"].data_ptr(),
                                        m, n, col.data_ptr(), val.data_ptr(), _stream_ptr(stream)), "spqr_gather_outliers")
    s.synchronize()
    host = {k: (None if v is None else v.cpu().numpy()) for k, v in t.items()}
    return SimpleNamespace(
        m=m, n=n, w_bits=w_bits, s_bits=s_bits, z_bits=z_bits, beta1=beta1, beta2=beta2, group_axis=0,
        Q=host["Q"], s_q=host["s_q"], z_q=host["z_q"], s_s=host["s_s"], z_s=host["z_s"], s_z=host["s_z"], z_z=host["z_z"],
        row_ptr=host["row_ptr"], col_idx=col[:nnz].cpu().numpy().view(np.uint16), val=val[:nnz].cpu().numpy(),
        is_outlier=host["outlier_mask"].astype(bool), W_final=host["W_final"], stat_layout="bilevel", perm=None)
