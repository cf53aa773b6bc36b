"""ctypes binding of libsga.so: argument marshalling only.

The `sga_*` functions mirror the C entry points one to one (raw addresses and
sizes in, status code out).  The un-prefixed helpers take torch tensors, check
shapes, allocate outputs and raise SgaError on a non-zero status.  There is no
CPU fallback: if the library is missing or cannot be built, loading raises.
"""
import ctypes
import os

from sga_inputs.masks import MaskSpec

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("SGA_LIB", os.path.join(_HERE, "libsga.so"))
_lib = None

PATH_AUTO, PATH_GATHER, PATH_TILE, PATH_TILE_SPLIT = 0, 1, 2, 3
_DTYPE_CODE = {"f32": 0, "f16": 1}


class SgaError(RuntimeError):
    def __init__(self, status, where):
        self.status = status
        super().__init__(f"{where}: {sga_status_string(status)} (status {status})")


class _MaskDesc(ctypes.Structure):
    _fields_ = [
        ("struct_bytes", ctypes.c_uint32), ("kind", ctypes.c_int32),
        ("L", ctypes.c_int64), ("window", ctypes.c_int32), ("stride", ctypes.c_int32),
        ("n_global", ctypes.c_int32), ("block", ctypes.c_int32),
        ("window_blocks", ctypes.c_int32), ("n_global_blocks", ctypes.c_int32),
        ("n_random_blocks", ctypes.c_int32), ("seed", ctypes.c_uint64),
    ]


def lib_path():
    return _LIB_PATH


def load():
    """Load libsga.so (building it first only if no built library exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build_lib
        build_lib()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64, f32 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float
    P = ctypes.POINTER
    lib.sga_status_string.restype = ctypes.c_char_p
    lib.sga_status_string.argtypes = [ctypes.c_int]
    lib.sga_mask_nnz.restype = ctypes.c_int
    lib.sga_mask_nnz.argtypes = [P(_MaskDesc), P(ctypes.c_int64)]
    lib.sga_build_mask.restype = ctypes.c_int
    lib.sga_build_mask.argtypes = [P(_MaskDesc), vp, vp, i64, vp]
    lib.sga_workspace_bytes.restype = ctypes.c_int
    lib.sga_workspace_bytes.argtypes = [i64, i32, i32, i32, i64, P(ctypes.c_size_t)]
    lib.sga_attention_forward.restype = ctypes.c_int
    lib.sga_attention_forward.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, f32, vp,
                                          i32, vp, vp, ctypes.c_size_t, i32]
    lib.sga_attention_forward_implicit.restype = ctypes.c_int
    lib.sga_attention_forward_implicit.argtypes = [vp, vp, vp, P(_MaskDesc), vp, i64, i32, i32,
                                                   f32, vp, i32, vp, vp, ctypes.c_size_t, i32]
    lib.sga_attention_accumulate.restype = ctypes.c_int
    lib.sga_attention_accumulate.argtypes = lib.sga_attention_forward.argtypes
    lib.sga_attention_accumulate_implicit.restype = ctypes.c_int
    lib.sga_attention_accumulate_implicit.argtypes = lib.sga_attention_forward_implicit.argtypes
    lib.sga_profile_enable.restype = ctypes.c_int
    lib.sga_profile_enable.argtypes = [i32]
    lib.sga_profile_collect.restype = ctypes.c_int
    lib.sga_profile_collect.argtypes = [P(ctypes.c_float), i32, P(ctypes.c_int32)]
    _lib = lib
    return lib


def _desc(spec: MaskSpec) -> _MaskDesc:
    return _MaskDesc(ctypes.sizeof(_MaskDesc), spec.kind, spec.L, spec.window, spec.stride,
                     spec.n_global, spec.block, spec.window_blocks, spec.n_global_blocks,
                     spec.n_random_blocks, spec.seed & ((1 << 64) - 1))


# ---- raw entry points (same names and argument order as include/sga.h) ----------
def sga_status_string(status):
    return load().sga_status_string(int(status)).decode()


def sga_mask_nnz(spec: MaskSpec):
    """-> (status, nnz)"""
    d = _desc(spec)
    out = ctypes.c_int64(0)
    st = load().sga_mask_nnz(ctypes.byref(d), ctypes.byref(out))
    return st, out.value


def sga_build_mask(spec: MaskSpec, row_ptr_addr, col_idx_addr, col_capacity, stream):
    d = _desc(spec)
    return load().sga_build_mask(ctypes.byref(d), row_ptr_addr, col_idx_addr, col_capacity, stream)


def sga_workspace_bytes(L, H, d, dtype_code, nnz):
    """-> (status, bytes)"""
    out = ctypes.c_size_t(0)
    st = load().sga_workspace_bytes(L, H, d, dtype_code, nnz, ctypes.byref(out))
    return st, out.value


def sga_attention_forward(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype_code,
                          lse, workspace, workspace_bytes_, path):
    return load().sga_attention_forward(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream,
                                        dtype_code, lse, workspace, workspace_bytes_, path)


def sga_attention_forward_implicit(Q, K, V, spec, O, L, H, d, scale, stream, dtype_code, lse,
                                   workspace, workspace_bytes_, path):
    dsc = _desc(spec)
    return load().sga_attention_forward_implicit(Q, K, V, ctypes.byref(dsc), O, L, H, d, scale,
                                                 stream, dtype_code, lse, workspace,
                                                 workspace_bytes_, path)


def sga_attention_accumulate(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype_code,
                             lse, workspace, workspace_bytes_, path):
    return load().sga_attention_accumulate(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream,
                                           dtype_code, lse, workspace, workspace_bytes_, path)


def sga_attention_accumulate_implicit(Q, K, V, spec, O, L, H, d, scale, stream, dtype_code, lse,
                                      workspace, workspace_bytes_, path):
    dsc = _desc(spec)
    return load().sga_attention_accumulate_implicit(Q, K, V, ctypes.byref(dsc), O, L, H, d, scale,
                                                    stream, dtype_code, lse, workspace,
                                                    workspace_bytes_, path)


def sga_profile_enable(on):
    return load().sga_profile_enable(int(on))


def sga_profile_collect(capacity=4096):
    """-> (status, [kernel durations in ms])"""
    buf = (ctypes.c_float * capacity)()
    n = ctypes.c_int32(0)
    st = load().sga_profile_collect(buf, capacity, ctypes.byref(n))
    return st, [buf[i] for i in range(n.value)]


# ---- tensor-level helpers ---------------------------------------------------------
def _stream():
    import torch
    return torch.cuda.current_stream().cuda_stream


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return 0
    if t.dtype == torch.float16:
        return 1
    raise TypeError(f"unsupported storage dtype {t.dtype}")


def mask_nnz(spec: MaskSpec) -> int:
    st, n = sga_mask_nnz(spec)
    if st != 0:
        raise SgaError(st, "sga_mask_nnz")
    return n


def build_mask(spec: MaskSpec, device="cuda"):
    """Build the CSR of the mask on `device`.  Returns (row_ptr int64 [L+1], col_idx int32 [nnz])."""
    import torch
    nnz = mask_nnz(spec)
    row_ptr = torch.empty(spec.L + 1, dtype=torch.int64, device=device)
    col_idx = torch.empty(max(nnz, 1), dtype=torch.int32, device=device)
    with torch.cuda.device(row_ptr.device):
        st = sga_build_mask(spec, row_ptr.data_ptr(), col_idx.data_ptr(), col_idx.numel(), _stream())
    if st != 0:
        raise SgaError(st, "sga_build_mask")
    return row_ptr, col_idx[:nnz]


def workspace_bytes(L, H, d, dtype, nnz=-1) -> int:
    st, n = sga_workspace_bytes(L, H, d, _DTYPE_CODE[dtype] if isinstance(dtype, str) else dtype, nnz)
    if st != 0:
        raise SgaError(st, "sga_workspace_bytes")
    return n


def alloc_workspace(L, H, d, dtype, nnz=-1, device="cuda"):
    import torch
    n = workspace_bytes(L, H, d, dtype, nnz)
    return torch.empty(n, dtype=torch.uint8, device=device)


def _check_qkv(Q, K, V):
    if not (Q.is_cuda and K.is_cuda and V.is_cuda):
        raise ValueError("Q, K, V must be device tensors")
    if Q.dim() != 3 or Q.shape != K.shape or Q.shape != V.shape:
        raise ValueError("Q, K, V must all be [H, L, d]")
    if not (Q.is_contiguous() and K.is_contiguous() and V.is_contiguous()):
        raise ValueError("Q, K, V must be contiguous")
    if not (Q.dtype == K.dtype == V.dtype):
        raise ValueError("Q, K, V must share a dtype")


def _col_ptr(row_ptr, col_idx):
    # a mask without edges has an empty col_idx, whose address is null; the entry points want a
    # device address even though they will not read through it
    return col_idx.data_ptr() if col_idx.numel() > 0 else row_ptr.data_ptr()


def attention_forward(Q, K, V, row_ptr, col_idx, scale, O=None, lse=None, workspace=None,
                      path=PATH_AUTO, want_lse=False):
    """Masked attention over an explicit CSR mask.  Returns O (and lse if requested)."""
    import torch
    _check_qkv(Q, K, V)
    H, L, d = Q.shape
    if row_ptr.dtype != torch.int64 or row_ptr.numel() != L + 1 or not row_ptr.is_contiguous():
        raise ValueError("row_ptr must be contiguous int64 [L+1]")
    if col_idx.dtype != torch.int32 or not col_idx.is_contiguous():
        raise ValueError("col_idx must be contiguous int32")
    if O is None:
        O = torch.empty_like(Q)
    if want_lse and lse is None:
        lse = torch.empty((H, L), dtype=torch.float32, device=Q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(Q.device):
        st = sga_attention_forward(Q.data_ptr(), K.data_ptr(), V.data_ptr(), row_ptr.data_ptr(),
                                   _col_ptr(row_ptr, col_idx), O.data_ptr(), L, H, d, float(scale),
                                   _stream(), _dtype_code(Q),
                                   lse.data_ptr() if lse is not None else None, ws_ptr, ws_n, path)
    if st != 0:
        raise SgaError(st, "sga_attention_forward")
    return (O, lse) if (want_lse or lse is not None) else O


def attention_forward_implicit(Q, K, V, spec: MaskSpec, scale, O=None, lse=None, workspace=None,
                               path=PATH_AUTO, want_lse=False):
    """Masked attention with neighbours generated in the kernel (sliding / dilated windows)."""
    import torch
    _check_qkv(Q, K, V)
    H, L, d = Q.shape
    if O is None:
        O = torch.empty_like(Q)
    if want_lse and lse is None:
        lse = torch.empty((H, L), dtype=torch.float32, device=Q.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(Q.device):
        st = sga_attention_forward_implicit(Q.data_ptr(), K.data_ptr(), V.data_ptr(), spec,
                                            O.data_ptr(), L, H, d, float(scale), _stream(),
                                            _dtype_code(Q),
                                            lse.data_ptr() if lse is not None else None,
                                            ws_ptr, ws_n, path)
    if st != 0:
        raise SgaError(st, "sga_attention_forward_implicit")
    return (O, lse) if (want_lse or lse is not None) else O


def _check_state(Q, O, lse):
    import torch
    H, L, d = Q.shape
    if O.shape != Q.shape or O.dtype != Q.dtype or not O.is_contiguous() or O.device != Q.device:
        raise ValueError("O must match Q in shape, dtype and device")
    if (lse.shape != (H, L) or lse.dtype != torch.float32 or not lse.is_contiguous()
            or lse.device != Q.device):
        raise ValueError("lse must be contiguous float32 [H, L] on Q's device")


def attention_accumulate(Q, K, V, row_ptr, col_idx, scale, O, lse, workspace=None, path=PATH_AUTO):
    """Continue the (O, lse) state over the edges of an explicit CSR mask, in place."""
    import torch
    _check_qkv(Q, K, V)
    _check_state(Q, O, lse)
    H, L, d = Q.shape
    if row_ptr.dtype != torch.int64 or row_ptr.numel() != L + 1 or not row_ptr.is_contiguous():
        raise ValueError("row_ptr must be contiguous int64 [L+1]")
    if col_idx.dtype != torch.int32 or not col_idx.is_contiguous():
        raise ValueError("col_idx must be contiguous int32")
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(Q.device):
        st = sga_attention_accumulate(Q.data_ptr(), K.data_ptr(), V.data_ptr(), row_ptr.data_ptr(),
                                      _col_ptr(row_ptr, col_idx), O.data_ptr(), L, H, d, float(scale),
                                      _stream(), _dtype_code(Q), lse.data_ptr(), ws_ptr, ws_n, path)
    if st != 0:
        raise SgaError(st, "sga_attention_accumulate")
    return O, lse


def attention_accumulate_implicit(Q, K, V, spec: MaskSpec, scale, O, lse, workspace=None,
                                  path=PATH_AUTO):
    """Continue the (O, lse) state over the edges of an implicit mask, in place."""
    import torch
    _check_qkv(Q, K, V)
    _check_state(Q, O, lse)
    H, L, d = Q.shape
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(Q.device):
        st = sga_attention_accumulate_implicit(Q.data_ptr(), K.data_ptr(), V.data_ptr(), spec,
                                               O.data_ptr(), L, H, d, float(scale), _stream(),
                                               _dtype_code(Q), lse.data_ptr(), ws_ptr, ws_n, path)
    if st != 0:
        raise SgaError(st, "sga_attention_accumulate_implicit")
    return O, lse
