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


class GraphPlan(ctypes.Structure):
    """sga_graph_plan: host record of a prepared tile graph (see include/sga.h)."""
    _fields_ = [
        ("struct_bytes", ctypes.c_uint32), ("magic", ctypes.c_uint32),
        ("L", ctypes.c_int64), ("nnz", ctypes.c_int64),
        ("H", ctypes.c_int32), ("d", ctypes.c_int32), ("dtype", ctypes.c_int32),
        ("tiles_left", ctypes.c_uint32), ("multi_tiles", ctypes.c_uint32),
        ("tile_parts", ctypes.c_uint32), ("long_rows", ctypes.c_uint32),
        ("row_chunks", ctypes.c_uint32), ("flags", ctypes.c_uint32),
        ("row_ptr", ctypes.c_void_p), ("col_idx", ctypes.c_void_p),
        ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t),
    ]


GRAPH_TILES_COVER_ALL, GRAPH_TILE_PARTS_FIT, GRAPH_ROW_CHUNKS_FIT = 1, 2, 4


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
    lib.sga_validate_csr.restype = ctypes.c_int
    lib.sga_validate_csr.argtypes = [vp, vp, i64, i64, vp, P(ctypes.c_int64), vp]
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
    lib.sga_graph_prepare.restype = ctypes.c_int
    lib.sga_graph_prepare.argtypes = [vp, vp, i64, i32, i32, i32, vp, ctypes.c_size_t, vp, P(GraphPlan)]
    lib.sga_attention_forward_prepared.restype = ctypes.c_int
    lib.sga_attention_forward_prepared.argtypes = lib.sga_attention_forward.argtypes + [P(GraphPlan)]
    lib.sga_attention_accumulate_prepared.restype = ctypes.c_int
    lib.sga_attention_accumulate_prepared.argtypes = lib.sga_attention_forward.argtypes + [P(GraphPlan)]
    lib.sga_profile_enable.restype = ctypes.c_int
    lib.sga_profile_enable.argtypes = [i32]
    lib.sga_profile_collect.restype = ctypes.c_int
    lib.sga_profile_collect.argtypes = [P(ctypes.c_float), i32, P(ctypes.c_int32)]
    lib.sga_static_scratch_init.restype = ctypes.c_int
    lib.sga_static_scratch_init.argtypes = []
    lib.sga_static_scratch_bytes.restype = ctypes.c_size_t
    lib.sga_static_scratch_bytes.argtypes = []
    lib.sga_attention_forward_static.restype = ctypes.c_int
    lib.sga_attention_forward_static.argtypes = [vp, vp, vp, vp, vp, vp, i64, i32, i32, f32, vp,
                                                 i32, vp, i64, i32]
    lib.sga_profile_last_kernel.restype = ctypes.c_char_p
    lib.sga_profile_last_kernel.argtypes = []
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


def sga_validate_csr(row_ptr_addr, col_idx_addr, L, col_capacity, scratch_addr, stream):
    """-> (status, bad_row)"""
    bad = ctypes.c_int64(-2)
    st = load().sga_validate_csr(row_ptr_addr, col_idx_addr, L, col_capacity, scratch_addr, ctypes.byref(bad), stream)
    return st, bad.value


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


def sga_graph_prepare(row_ptr, col_idx, L, H, d, dtype_code, workspace, workspace_bytes_, stream):
    """-> (status, GraphPlan)"""
    plan = GraphPlan()
    st = load().sga_graph_prepare(row_ptr, col_idx, L, H, d, dtype_code, workspace, workspace_bytes_,
                                  stream, ctypes.byref(plan))
    return st, plan


def sga_attention_forward_prepared(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype_code,
                                   lse, workspace, workspace_bytes_, path, plan):
    return load().sga_attention_forward_prepared(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream,
                                                 dtype_code, lse, workspace, workspace_bytes_, path,
                                                 ctypes.byref(plan))


def sga_attention_accumulate_prepared(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream,
                                      dtype_code, lse, workspace, workspace_bytes_, path, plan):
    return load().sga_attention_accumulate_prepared(Q, K, V, row_ptr, col_idx, O, L, H, d, scale,
                                                    stream, dtype_code, lse, workspace,
                                                    workspace_bytes_, path, ctypes.byref(plan))


def sga_static_scratch_init():
    return load().sga_static_scratch_init()


def sga_static_scratch_bytes():
    return int(load().sga_static_scratch_bytes())


def sga_attention_forward_static(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream, dtype_code,
                                 lse, nnz, path):
    return load().sga_attention_forward_static(Q, K, V, row_ptr, col_idx, O, L, H, d, scale, stream,
                                               dtype_code, lse, nnz, path)


def sga_profile_enable(on):
    return load().sga_profile_enable(int(on))


def sga_profile_collect(capacity=4096):
    """-> (status, [kernel durations in ms])"""
    buf = (ctypes.c_float * capacity)()
    n = ctypes.c_int32(0)
    st = load().sga_profile_collect(buf, capacity, ctypes.byref(n))
    return st, [buf[i] for i in range(min(n.value, capacity))]


def sga_profile_last_kernel():
    return load().sga_profile_last_kernel().decode()


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


def validate_csr(row_ptr, col_idx) -> int:
    """-1 if (row_ptr, col_idx) is a valid mask for the forward calls, else the smallest row that
    breaks the contract (L if row_ptr[0] or row_ptr[L] does).  Waits for the current stream."""
    import torch
    if not (row_ptr.is_cuda and col_idx.is_cuda and row_ptr.device == col_idx.device):
        raise ValueError("row_ptr and col_idx must be tensors of one device")
    if row_ptr.dtype != torch.int64 or col_idx.dtype != torch.int32 or row_ptr.dim() != 1 or col_idx.dim() != 1:
        raise ValueError("row_ptr must be int64 [L+1], col_idx int32 [nnz]")
    if not (row_ptr.is_contiguous() and col_idx.is_contiguous()) or row_ptr.numel() < 2:
        raise ValueError("row_ptr and col_idx must be contiguous, L >= 1")
    scratch = torch.empty(2, dtype=torch.int64, device=row_ptr.device)
    with torch.cuda.device(row_ptr.device):
        st, bad = sga_validate_csr(row_ptr.data_ptr(), _col_ptr(row_ptr, col_idx), row_ptr.numel() - 1,
                                   col_idx.numel(), scratch.data_ptr(), _stream())
    if st != 0 and bad < 0:
        raise SgaError(st, "sga_validate_csr")
    return bad


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


def _check_csr(Q, row_ptr, col_idx):
    import torch
    L = Q.shape[1]
    if row_ptr.dtype != torch.int64 or row_ptr.numel() != L + 1 or not row_ptr.is_contiguous():
        raise ValueError("row_ptr must be contiguous int64 [L+1]")
    if col_idx.dtype != torch.int32 or not col_idx.is_contiguous():
        raise ValueError("col_idx must be contiguous int32")
    if row_ptr.device != Q.device or (col_idx.numel() > 0 and col_idx.device != Q.device):
        raise ValueError("row_ptr and col_idx must be on Q's device")


def _check_outputs(Q, O, lse, workspace):
    """Caller-supplied output and scratch buffers: the kernels write H*L*d elements of O and H*L
    floats of lse without further checks, so a wrong shape here would be an out-of-bounds write."""
    import torch
    H, L, d = Q.shape
    if O is not None and (O.shape != Q.shape or O.dtype != Q.dtype or not O.is_contiguous()
                          or O.device != Q.device):
        raise ValueError("O must match Q in shape, dtype and device, and be contiguous")
    if lse is not None and (lse.shape != (H, L) or lse.dtype != torch.float32
                            or not lse.is_contiguous() or lse.device != Q.device):
        raise ValueError("lse must be contiguous float32 [H, L] on Q's device")
    if workspace is not None and (workspace.device != Q.device or not workspace.is_contiguous()):
        raise ValueError("workspace must be a contiguous tensor on Q's device")


def attention_forward(Q, K, V, row_ptr, col_idx, scale, O=None, lse=None, workspace=None,
                      path=PATH_AUTO, want_lse=False):
    """Masked attention over an explicit CSR mask.  Returns O (and lse if requested)."""
    import torch
    _check_qkv(Q, K, V)
    H, L, d = Q.shape
    _check_csr(Q, row_ptr, col_idx)
    _check_outputs(Q, O, lse, workspace)
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
    _check_outputs(Q, O, lse, workspace)
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
    _check_csr(Q, row_ptr, col_idx)
    _check_outputs(Q, None, None, workspace)
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
    _check_outputs(Q, None, None, workspace)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_n = workspace.numel() * workspace.element_size() if workspace is not None else 0
    with torch.cuda.device(Q.device):
        st = sga_attention_accumulate_implicit(Q.data_ptr(), K.data_ptr(), V.data_ptr(), spec,
                                               O.data_ptr(), L, H, d, float(scale), _stream(),
                                               _dtype_code(Q), lse.data_ptr(), ws_ptr, ws_n, path)
    if st != 0:
        raise SgaError(st, "sga_attention_accumulate_implicit")
    return O, lse


def graph_prepare(row_ptr, col_idx, H, d, dtype, workspace):
    """Prepare the tile graph of an explicit mask once (waits for the stream).  Returns the
    GraphPlan to pass to attention_forward_prepared / attention_accumulate_prepared together with
    the same row_ptr, col_idx and workspace."""
    import torch
    L = row_ptr.numel() - 1
    if row_ptr.dtype != torch.int64 or not row_ptr.is_contiguous() or not row_ptr.is_cuda:
        raise ValueError("row_ptr must be a contiguous int64 device tensor")
    if col_idx.dtype != torch.int32 or not col_idx.is_contiguous():
        raise ValueError("col_idx must be contiguous int32")
    if workspace is None or workspace.device != row_ptr.device or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous tensor on row_ptr's device")
    code = _DTYPE_CODE[dtype] if isinstance(dtype, str) else dtype
    with torch.cuda.device(row_ptr.device):
        st, plan = sga_graph_prepare(row_ptr.data_ptr(), _col_ptr(row_ptr, col_idx), L, H, d, code,
                                     workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                     _stream())
    if st != 0:
        raise SgaError(st, "sga_graph_prepare")
    return plan


def _prepared_call(fn, name, Q, K, V, row_ptr, col_idx, scale, plan, O, lse, workspace, path):
    import torch
    H, L, d = Q.shape
    with torch.cuda.device(Q.device):
        st = fn(Q.data_ptr(), K.data_ptr(), V.data_ptr(), row_ptr.data_ptr(), _col_ptr(row_ptr, col_idx),
                O.data_ptr(), L, H, d, float(scale), _stream(), _dtype_code(Q),
                lse.data_ptr() if lse is not None else None, workspace.data_ptr(),
                workspace.numel() * workspace.element_size(), path, plan)
    if st != 0:
        raise SgaError(st, name)


def attention_forward_prepared(Q, K, V, row_ptr, col_idx, scale, plan, workspace, O=None, lse=None,
                               path=PATH_AUTO, want_lse=False):
    """attention_forward on a graph prepared by graph_prepare (same row_ptr, col_idx, workspace)."""
    import torch
    _check_qkv(Q, K, V)
    H, L, d = Q.shape
    _check_csr(Q, row_ptr, col_idx)
    _check_outputs(Q, O, lse, workspace)
    if O is None:
        O = torch.empty_like(Q)
    if want_lse and lse is None:
        lse = torch.empty((H, L), dtype=torch.float32, device=Q.device)
    _prepared_call(sga_attention_forward_prepared, "sga_attention_forward_prepared", Q, K, V, row_ptr,
                   col_idx, scale, plan, O, lse, workspace, path)
    return (O, lse) if (want_lse or lse is not None) else O


def attention_accumulate_prepared(Q, K, V, row_ptr, col_idx, scale, plan, workspace, O, lse,
                                  path=PATH_AUTO):
    """attention_accumulate on a prepared graph, in place."""
    _check_qkv(Q, K, V)
    _check_state(Q, O, lse)
    _check_csr(Q, row_ptr, col_idx)
    _check_outputs(Q, None, None, workspace)
    _prepared_call(sga_attention_accumulate_prepared, "sga_attention_accumulate_prepared", Q, K, V,
                   row_ptr, col_idx, scale, plan, O, lse, workspace, path)
    return O, lse
