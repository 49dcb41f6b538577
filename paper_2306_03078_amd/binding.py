"""ctypes binding of the C ABI declared in include/spqr.h (same names).

Argument marshalling only.  There is no CPU fallback: if libspqr.so is missing
the first call raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(HERE, "libspqr.so")
_lib = None

SPQR_F32, SPQR_F16 = 0, 1
SPQR_CHECK_CSR, SPQR_CHECK_NONFINITE, SPQR_CHECK_PERM = 1, 2, 4
SPQR_OUT_CODES_U8, SPQR_OUT_SCALE_F32, SPQR_OUT_ZERO_F32 = 0, 1, 2
SPQR_OUT_DENSE_F32, SPQR_OUT_DENSE_F16, SPQR_OUT_WITH_OUTLIERS = 3, 4, 0x100
SPQR_LAYOUT_V1, SPQR_LAYOUT_ROUND_ZERO, SPQR_LAYOUT_STATS16 = 1, 2, 3
_LAYOUT_OF = {"bilevel": SPQR_LAYOUT_V1, "round_zero": SPQR_LAYOUT_ROUND_ZERO, "stats16": SPQR_LAYOUT_STATS16}
SPQR_OPT_BATCH_PATH, SPQR_OPT_FORCE_GENERIC, SPQR_OPT_BATCH_STEPS, SPQR_OPT_DENSE_ROWS, SPQR_OPT_GEMV_PLAN = 0, 1, 2, 3, 4
SPQR_BATCH_PATH_AUTO, SPQR_BATCH_PATH_VECTOR, SPQR_BATCH_PATH_MATRIX, SPQR_BATCH_PATH_DENSE = 0, 1, 2, 3
SPQR_ERR_WORKSPACE = -11
SPQR_STATIC_SCRATCH_BYTES = 32 * 1024 * 1024


class SpQRError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {spqr_strerror(status)} (status {status})")


class spqr_matrix_t(C.Structure):
    _fields_ = [
        ("m", C.c_int32), ("n", C.c_int32),
        ("w_bits", C.c_int32), ("s_bits", C.c_int32), ("z_bits", C.c_int32),
        ("beta1", C.c_int32), ("beta2", C.c_int32),
        ("group_axis", C.c_int32), ("layout_version", C.c_int32), ("max_row_nnz", C.c_int32),
        ("packed", C.c_void_p), ("packed_bytes", C.c_int64),
        ("row_ptr", C.c_void_p), ("col_idx", C.c_void_p), ("out_val", C.c_void_p),
        ("nnz", C.c_int64), ("perm", C.c_void_p),
    ]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libspqr.so (built in-tree by paper_2306_03078_amd.build)."""
    global _lib
    if _lib is not None:
        return _lib
    # PyTorch ships its own HIP runtime; importing it first makes the dynamic
    # linker resolve libspqr.so against that same runtime instead of loading a
    # second one (two runtimes in one process cannot share streams or memory).
    import torch  # noqa: F401
    if not os.path.exists(_LIB_PATH):
        raise FileNotFoundError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2306_03078_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    P = C.POINTER(spqr_matrix_t)
    i32, i64, vp = C.c_int32, C.c_int64, C.c_void_p
    lib.spqr_packed_bytes.restype = i64
    lib.spqr_packed_bytes.argtypes = [i32] * 8
    lib.spqr_pack_host.restype = C.c_int
    lib.spqr_pack_host.argtypes = [i32] * 8 + [vp] * 8 + [i64]
    lib.spqr_packed_bytes_layout.restype = i64
    lib.spqr_packed_bytes_layout.argtypes = [i32] * 9
    lib.spqr_pack_host_layout.restype = C.c_int
    lib.spqr_pack_host_layout.argtypes = [i32] * 9 + [vp] * 8 + [i64]
    lib.spqr_strerror.restype = C.c_char_p
    lib.spqr_strerror.argtypes = [C.c_int]
    lib.spqr_version.restype = i32
    lib.spqr_version.argtypes = []
    lib.spqr_pack_check.restype = C.c_int
    lib.spqr_pack_check.argtypes = [P, C.c_uint32, vp]
    lib.spqr_gemv.restype = C.c_int
    lib.spqr_gemv.argtypes = [P, vp, vp, C.c_int, vp]
    lib.spqr_gemm_smallbatch.restype = C.c_int
    lib.spqr_gemm_smallbatch.argtypes = [P, vp, C.c_int, vp, C.c_int, vp]
    lib.spqr_gemv_fused.restype = C.c_int
    lib.spqr_gemv_fused.argtypes = [C.POINTER(P), C.c_int, vp, C.POINTER(vp), C.c_int, vp]
    lib.spqr_gemm_fused.restype = C.c_int
    lib.spqr_gemm_fused.argtypes = [C.POINTER(P), C.c_int, vp, C.c_int, C.POINTER(vp), C.c_int, vp]
    lib.spqr_dequant_dense.restype = C.c_int
    lib.spqr_dequant_dense.argtypes = [P, C.c_int, vp, vp]
    lib.spqr_plan_batch_steps.restype = C.c_int
    lib.spqr_plan_batch_steps.argtypes = [C.c_int] * 5
    lib.spqr_set_option.restype = C.c_int
    lib.spqr_set_option.argtypes = [C.c_int, C.c_int]
    lib.spqr_workspace_bytes.restype = i64
    lib.spqr_workspace_bytes.argtypes = [C.POINTER(P), C.c_int, C.c_int]
    lib.spqr_gemm_smallbatch_ws.restype = C.c_int
    lib.spqr_gemm_smallbatch_ws.argtypes = [P, vp, C.c_int, vp, C.c_int, vp, i64, vp]
    lib.spqr_gemm_fused_ws.restype = C.c_int
    lib.spqr_gemm_fused_ws.argtypes = [C.POINTER(P), C.c_int, vp, C.c_int, C.POINTER(vp), C.c_int, vp, i64, vp]
    lib.spqr_gemv_grouped.restype = C.c_int
    lib.spqr_gemv_grouped.argtypes = [C.POINTER(P), C.c_int, C.POINTER(vp), C.POINTER(vp), C.c_int, vp]
    lib.spqr_gemm_smallbatch_noalloc.restype = C.c_int
    lib.spqr_gemm_smallbatch_noalloc.argtypes = [P, vp, C.c_int, vp, C.c_int, vp]
    _lib = lib
    return lib


def spqr_strerror(status: int) -> str:
    return load_library().spqr_strerror(int(status)).decode()


def packed_bytes(m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis, layout_version=SPQR_LAYOUT_V1) -> int:
    lib = load_library()
    if layout_version == SPQR_LAYOUT_V1:
        r = lib.spqr_packed_bytes(m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis)
    else:
        r = lib.spqr_packed_bytes_layout(layout_version, m, n, w_bits, s_bits, z_bits, beta1, beta2, group_axis)
    if r < 0:
        raise SpQRError(int(r), "spqr_packed_bytes")
    return int(r)


def _np_ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


def layout_version_of(fmt) -> int:
    return _LAYOUT_OF[getattr(fmt, "stat_layout", "bilevel")]


def pack_host(fmt) -> np.ndarray:
    """Logical arrays (spqr_synth.SpQRLogical-like) -> packed uint8 host buffer."""
    lib = load_library()
    lv = layout_version_of(fmt)
    nbytes = packed_bytes(fmt.m, fmt.n, fmt.w_bits, fmt.s_bits, fmt.z_bits, fmt.beta1, fmt.beta2,
                          fmt.group_axis, lv)
    out = np.empty(nbytes, dtype=np.uint8)
    Q = np.ascontiguousarray(fmt.Q, dtype=np.uint8)
    if lv == SPQR_LAYOUT_STATS16:
        first = [np.ascontiguousarray(a, dtype=np.float16).view(np.uint16) for a in (fmt.s16, fmt.z16)]
    else:
        first = [np.ascontiguousarray(a, dtype=np.uint8) for a in (fmt.s_q, fmt.z_q)]
    st = [None if a is None else np.ascontiguousarray(a, dtype=np.float16).view(np.uint16)
          for a in (fmt.s_s, fmt.z_s, fmt.s_z, fmt.z_z)]
    if lv == SPQR_LAYOUT_V1:
        rc = lib.spqr_pack_host(fmt.m, fmt.n, fmt.w_bits, fmt.s_bits, fmt.z_bits, fmt.beta1, fmt.beta2,
                                fmt.group_axis, _np_ptr(Q), _np_ptr(first[0]), _np_ptr(first[1]),
                                *[_np_ptr(a) for a in st], _np_ptr(out), nbytes)
    else:
        rc = lib.spqr_pack_host_layout(lv, fmt.m, fmt.n, fmt.w_bits, fmt.s_bits, fmt.z_bits, fmt.beta1,
                                       fmt.beta2, fmt.group_axis, _np_ptr(Q), _np_ptr(first[0]),
                                       _np_ptr(first[1]), *[_np_ptr(a) for a in st], _np_ptr(out), nbytes)
    if rc != 0:
        raise SpQRError(rc, "spqr_pack_host")
    return out


def _stream_ptr(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


class SpQRMatrix:
    """Device-resident SpQR matrix: torch tensors own the memory, the
    descriptor points into them."""

    def __init__(self, m, n, w_bits, beta1, beta2, group_axis, packed, row_ptr, col_idx, val,
                 perm=None, s_bits=3, z_bits=3, layout_version=SPQR_LAYOUT_V1, max_row_nnz=0):
        self.m, self.n = int(m), int(n)
        self.w_bits, self.s_bits, self.z_bits = int(w_bits), int(s_bits), int(z_bits)
        self.beta1, self.beta2, self.group_axis = int(beta1), int(beta2), int(group_axis)
        self.packed, self.row_ptr, self.col_idx, self.val, self.perm = packed, row_ptr, col_idx, val, perm
        self.nnz = int(col_idx.numel())
        d = spqr_matrix_t()
        d.m, d.n = self.m, self.n
        d.w_bits, d.s_bits, d.z_bits = self.w_bits, self.s_bits, self.z_bits
        d.beta1, d.beta2, d.group_axis = self.beta1, self.beta2, self.group_axis
        self.layout_version = int(layout_version)
        self.max_row_nnz = int(max_row_nnz)
        d.layout_version, d.max_row_nnz = self.layout_version, self.max_row_nnz
        d.packed, d.packed_bytes = packed.data_ptr(), packed.numel()
        d.row_ptr = row_ptr.data_ptr()
        d.col_idx = col_idx.data_ptr() if self.nnz else None
        d.out_val = val.data_ptr() if self.nnz else None
        d.nnz = self.nnz
        d.perm = perm.data_ptr() if perm is not None else None
        self.desc = d

    @property
    def device(self):
        return self.packed.device

    def compressed_bytes(self) -> int:
        """Bytes of the representation: packed tiles + CSR arrays (App. D accounting)."""
        return self.packed.numel() + 4 * (self.m + 1) + 4 * self.nnz

    @classmethod
    def from_logical(cls, fmt, device="cuda:0"):
        import torch
        packed = torch.from_numpy(pack_host(fmt)).to(device)
        row_ptr = torch.from_numpy(np.ascontiguousarray(fmt.row_ptr, dtype=np.int32)).to(device)
        col = torch.from_numpy(np.ascontiguousarray(fmt.col_idx, dtype=np.uint16).view(np.int16)).to(device)
        val = torch.from_numpy(np.ascontiguousarray(fmt.val, dtype=np.float16)).to(device)
        perm = None
        if getattr(fmt, "perm", None) is not None:
            perm = torch.from_numpy(np.ascontiguousarray(fmt.perm, dtype=np.int32)).to(device)
        return cls(fmt.m, fmt.n, fmt.w_bits, fmt.beta1, fmt.beta2, fmt.group_axis, packed, row_ptr,
                   col, val, perm, fmt.s_bits, fmt.z_bits, layout_version_of(fmt),
                   int(np.diff(np.asarray(fmt.row_ptr, dtype=np.int64)).max()) if fmt.m > 0 else 0)

    def clone(self):
        """A second copy of all device buffers (distinct addresses)."""
        return SpQRMatrix(self.m, self.n, self.w_bits, self.beta1, self.beta2, self.group_axis,
                          self.packed.clone(), self.row_ptr.clone(), self.col_idx.clone(),
                          self.val.clone(), None if self.perm is None else self.perm.clone(),
                          self.s_bits, self.z_bits, self.layout_version, self.max_row_nnz)


def _check(rc: int, where: str):
    if rc != 0:
        raise SpQRError(int(rc), where)


def spqr_pack_check(A: SpQRMatrix, flags: int = SPQR_CHECK_CSR | SPQR_CHECK_NONFINITE | SPQR_CHECK_PERM,
                    stream=None) -> int:
    """Returns the status code (0 = valid); does not raise on a failed check."""
    return int(load_library().spqr_pack_check(C.byref(A.desc), flags, _stream_ptr(stream)))


def _out_dtype(y_dtype):
    import torch
    return torch.float32 if y_dtype == SPQR_F32 else torch.float16


def spqr_gemv(A: SpQRMatrix, x, out=None, y_dtype: int = SPQR_F32, stream=None):
    """y[m] = W_hat . x, x: float16 device tensor [n]."""
    import torch
    assert x.dtype == torch.float16 and x.is_contiguous() and x.numel() == A.n
    if out is None:
        out = torch.empty(A.m, dtype=_out_dtype(y_dtype), device=x.device)
    _check(load_library().spqr_gemv(C.byref(A.desc), x.data_ptr(), out.data_ptr(), y_dtype,
                                    _stream_ptr(stream)), "spqr_gemv")
    return out


def spqr_gemm_smallbatch(A: SpQRMatrix, X, out=None, y_dtype: int = SPQR_F32, stream=None):
    """Y[b, m] = X[b, :] . W_hat^T, X: float16 device tensor [b, n], 1 <= b <= SPQR_MAX_BATCH (256)."""
    import torch
    assert X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == A.n
    b = int(X.shape[0])
    if out is None:
        out = torch.empty((b, A.m), dtype=_out_dtype(y_dtype), device=X.device)
    _check(load_library().spqr_gemm_smallbatch(C.byref(A.desc), X.data_ptr(), b, out.data_ptr(),
                                               y_dtype, _stream_ptr(stream)), "spqr_gemm_smallbatch")
    return out


def spqr_gemv_fused(As, x, outs=None, y_dtype: int = SPQR_F32, stream=None):
    """y_i[m_i] = W_hat_i . x for matrices sharing the input vector; one launch when possible."""
    import torch
    As = list(As)
    assert x.dtype == torch.float16 and x.is_contiguous() and x.numel() == As[0].n
    if outs is None:
        outs = [torch.empty(A.m, dtype=_out_dtype(y_dtype), device=x.device) for A in As]
    lib = load_library()
    k = len(As)
    descs = (C.POINTER(spqr_matrix_t) * k)(*[C.pointer(A.desc) for A in As])
    ys = (C.c_void_p * k)(*[o.data_ptr() for o in outs])
    _check(lib.spqr_gemv_fused(descs, k, x.data_ptr(), ys, y_dtype, _stream_ptr(stream)), "spqr_gemv_fused")
    return outs


def spqr_gemm_fused(As, X, outs=None, y_dtype: int = SPQR_F32, stream=None):
    """Y_i[b, m_i] = X[b, :] . W_hat_i^T for matrices sharing the batch X (float16 device tensor [b, n])."""
    import torch
    As = list(As)
    assert X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == As[0].n
    b = int(X.shape[0])
    if outs is None:
        outs = [torch.empty((b, A.m), dtype=_out_dtype(y_dtype), device=X.device) for A in As]
    lib = load_library()
    k = len(As)
    descs = (C.POINTER(spqr_matrix_t) * k)(*[C.pointer(A.desc) for A in As])
    ys = (C.c_void_p * k)(*[o.data_ptr() for o in outs])
    _check(lib.spqr_gemm_fused(descs, k, X.data_ptr(), b, ys, y_dtype, _stream_ptr(stream)), "spqr_gemm_fused")
    return outs


def spqr_set_option(option: int, value: int) -> None:
    """Process-wide tuning / test switch (SPQR_OPT_*)."""
    _check(load_library().spqr_set_option(int(option), int(value)), "spqr_set_option")


def spqr_workspace_bytes(As, b: int) -> int:
    """Device scratch the *_ws calls need at most for these matrices (one SpQRMatrix or a list) at batch b."""
    As = [As] if isinstance(As, SpQRMatrix) else list(As)
    k = len(As)
    descs = (C.POINTER(spqr_matrix_t) * k)(*[C.pointer(A.desc) for A in As])
    r = load_library().spqr_workspace_bytes(descs, k, int(b))
    if r < 0:
        raise SpQRError(int(r), "spqr_workspace_bytes")
    return int(r)


def _ws_args(workspace):
    if workspace is None:
        return None, 0
    return workspace.data_ptr(), workspace.numel() * workspace.element_size()


def spqr_gemm_smallbatch_ws(A: SpQRMatrix, X, workspace, out=None, y_dtype: int = SPQR_F32, stream=None):
    """spqr_gemm_smallbatch with scratch in `workspace` (a device tensor, or None where none is needed)."""
    import torch
    assert X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == A.n
    b = int(X.shape[0])
    if out is None:
        out = torch.empty((b, A.m), dtype=_out_dtype(y_dtype), device=X.device)
    wp, wb = _ws_args(workspace)
    _check(load_library().spqr_gemm_smallbatch_ws(C.byref(A.desc), X.data_ptr(), b, out.data_ptr(), y_dtype, wp, wb,
                                                  _stream_ptr(stream)), "spqr_gemm_smallbatch_ws")
    return out


def spqr_gemm_fused_ws(As, X, workspace, outs=None, y_dtype: int = SPQR_F32, stream=None):
    """spqr_gemm_fused with scratch in `workspace`."""
    import torch
    As = list(As)
    assert X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == As[0].n
    b = int(X.shape[0])
    if outs is None:
        outs = [torch.empty((b, A.m), dtype=_out_dtype(y_dtype), device=X.device) for A in As]
    k = len(As)
    descs = (C.POINTER(spqr_matrix_t) * k)(*[C.pointer(A.desc) for A in As])
    ys = (C.c_void_p * k)(*[o.data_ptr() for o in outs])
    wp, wb = _ws_args(workspace)
    _check(load_library().spqr_gemm_fused_ws(descs, k, X.data_ptr(), b, ys, y_dtype, wp, wb, _stream_ptr(stream)),
           "spqr_gemm_fused_ws")
    return outs


def spqr_gemm_smallbatch_noalloc(A: SpQRMatrix, X, out, y_dtype: int = SPQR_F32, stream=None):
    """spqr_gemm_smallbatch with scratch in the library's static device array; `out` is the caller's."""
    import torch
    assert X.dtype == torch.float16 and X.is_contiguous() and X.dim() == 2 and X.shape[1] == A.n
    _check(load_library().spqr_gemm_smallbatch_noalloc(C.byref(A.desc), X.data_ptr(), int(X.shape[0]), out.data_ptr(),
                                                       y_dtype, _stream_ptr(stream)), "spqr_gemm_smallbatch_noalloc")
    return out


def spqr_gemv_grouped(As, xs, outs=None, y_dtype: int = SPQR_F32, stream=None):
    """y_i[m_i] = W_hat_i . x_i for matrices with an input vector each; as few launches as possible."""
    import torch
    As, xs = list(As), list(xs)
    assert len(As) == len(xs)
    for A, x in zip(As, xs):
        assert x.dtype == torch.float16 and x.is_contiguous() and x.numel() == A.n
    if outs is None:
        outs = [torch.empty(A.m, dtype=_out_dtype(y_dtype), device=x.device) for A, x in zip(As, xs)]
    k = len(As)
    descs = (C.POINTER(spqr_matrix_t) * k)(*[C.pointer(A.desc) for A in As])
    xp = (C.c_void_p * k)(*[x.data_ptr() for x in xs])
    ys = (C.c_void_p * k)(*[o.data_ptr() for o in outs])
    _check(load_library().spqr_gemv_grouped(descs, k, xp, ys, y_dtype, _stream_ptr(stream)), "spqr_gemv_grouped")
    return outs


def spqr_dequant_dense(A: SpQRMatrix, what: int, stream=None):
    """Debug decode; returns a new device tensor shaped for the selector."""
    import torch
    sel = what & 0xFF
    gshape = (A.m, A.n // A.beta1) if A.group_axis == 0 else (A.m // A.beta1, A.n)
    shape, dt = {
        SPQR_OUT_CODES_U8: ((A.m, A.n), torch.uint8),
        SPQR_OUT_SCALE_F32: (gshape, torch.float32),
        SPQR_OUT_ZERO_F32: (gshape, torch.float32),
        SPQR_OUT_DENSE_F32: ((A.m, A.n), torch.float32),
        SPQR_OUT_DENSE_F16: ((A.m, A.n), torch.float16),
    }.get(sel, ((1,), torch.uint8))
    out = torch.empty(shape, dtype=dt, device=A.device)
    _check(load_library().spqr_dequant_dense(C.byref(A.desc), what, out.data_ptr(),
                                             _stream_ptr(stream)), "spqr_dequant_dense")
    return out


def spqr_plan_batch_steps(groups: int, nsteps: int, slots_one_step: int, slots: int, long_workgroups: int) -> int:
    """Steps per workgroup the batch path's dense launch would take (host arithmetic, no device needed)."""
    rc = load_library().spqr_plan_batch_steps(groups, nsteps, slots_one_step, slots, long_workgroups)
    if rc < 0:
        _check(rc, "spqr_plan_batch_steps")
    return rc
