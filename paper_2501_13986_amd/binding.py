"""ctypes binding of libcgtp.so: the functions of include/cgtp.h under the same names.

Argument marshalling only: torch tensors supply device memory and the current stream, every
step of the computation runs in the library's kernels.  There is no fallback: if the shared
library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libcgtp.so")

CGTP_F32, CGTP_F64 = 0, 1
CGTP_UVU, CGTP_UVW = 0, 1
CGTP_MUL_IR, CGTP_IR_MUL = 0, 1
K_TP_FWD, K_TP_BWD, K_CONV_FWD, K_CONV_BWD, K_CONV_FWD_ATOMIC, K_CONV_BWD_ATOMIC, K_TP_DBL_BWD = 0, 1, 2, 3, 4, 5, 6
K_CONV_DBL_FWD, K_CONV_DBL_BWD = 7, 8
STATUS = {0: "CGTP_OK", 1: "CGTP_EINVAL", 2: "CGTP_EUNSUPPORTED", 3: "CGTP_ECOMPILE", 4: "CGTP_ERUNTIME", 5: "CGTP_ENOMEM"}

EXPORTS = [
    "cgtp_plan_create", "cgtp_plan_create_ex", "cgtp_plan_destroy", "cgtp_plan_dim", "cgtp_plan_num_paths", "cgtp_plan_get_path",
    "cgtp_plan_path_nonzeros", "cgtp_plan_flops", "cgtp_plan_source", "cgtp_plan_kernel_info",
    "tp_forward", "tp_backward", "tp_double_backward", "conv_forward", "conv_forward_static", "conv_backward", "conv_forward_perm", "conv_backward_perm", "conv_double_backward", "conv_forward_atomic", "conv_backward_atomic",
    "cgtp_csr_from_coo", "cgtp_csr_from_coo_async", "cgtp_csr_workspace_bytes", "cgtp_last_error", "cgtp_check_code_object",
]


class CgtpError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__(f"{STATUS.get(status, status)}: {msg}")
        self.status = status


class cgtp_options(C.Structure):
    _fields_ = [("struct_size", C.c_int32), ("kahan_conv", C.c_int32)]


class cgtp_path(C.Structure):
    _fields_ = [("ix", C.c_int32), ("iy", C.c_int32), ("iz", C.c_int32), ("mode", C.c_int32), ("coeff", C.c_double)]


_lib = None


def lib() -> C.CDLL:
    """Loads libcgtp.so (built by paper_2501_13986_amd.build) and declares the prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2501_13986_amd.build`")
    L = C.CDLL(LIB_PATH)
    vp, i64, i32 = C.c_void_p, C.c_int64, C.c_int32
    L.cgtp_last_error.restype = C.c_char_p
    L.cgtp_check_code_object.argtypes = [C.c_char_p, C.c_char_p, C.c_size_t]
    L.cgtp_plan_create.argtypes = [C.c_char_p, C.c_char_p, C.c_char_p, C.POINTER(cgtp_path), i32, i32, i32, i32, i32, C.c_uint32,
                                   C.POINTER(vp)]
    L.cgtp_plan_create_ex.argtypes = [C.c_char_p, C.c_char_p, C.c_char_p, C.POINTER(cgtp_path), i32, i32, i32, i32, i32, C.c_uint32,
                                      C.POINTER(cgtp_options), C.POINTER(vp)]
    L.cgtp_plan_destroy.argtypes = [vp]
    L.cgtp_plan_dim.argtypes = [vp, i32]
    L.cgtp_plan_dim.restype = i64
    L.cgtp_plan_num_paths.argtypes = [vp]
    L.cgtp_plan_get_path.argtypes = [vp, i32, C.POINTER(cgtp_path), C.POINTER(i32), C.POINTER(i32), C.POINTER(i64)]
    L.cgtp_plan_path_nonzeros.argtypes = [vp, i32, i32, C.POINTER(i32), C.POINTER(i32), C.POINTER(i32), C.POINTER(C.c_double)]
    L.cgtp_plan_flops.argtypes = [vp, i32]
    L.cgtp_plan_flops.restype = i64
    L.cgtp_plan_source.argtypes = [vp, i32]
    L.cgtp_plan_source.restype = C.c_char_p
    L.cgtp_plan_kernel_info.argtypes = [vp, i32, C.POINTER(i32)]
    L.tp_forward.argtypes = [vp, vp, vp, vp, vp, i64, vp]
    L.tp_backward.argtypes = [vp] + [vp] * 7 + [i64, vp]
    L.tp_double_backward.argtypes = [vp] + [vp] * 11 + [i64, vp]
    L.conv_forward.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
    L.conv_forward_static.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
    L.conv_backward.argtypes = [vp] + [vp] * 7 + [i64, i64, vp, vp, vp, vp, vp]
    L.conv_forward_perm.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp, vp]
    L.conv_backward_perm.argtypes = [vp] + [vp] * 7 + [i64, i64, vp, vp, vp, vp, vp, vp]
    L.conv_double_backward.argtypes = [vp] + [vp] * 11 + [i64, i64, vp, vp, vp, vp, vp]
    L.conv_forward_atomic.argtypes = [vp, vp, vp, vp, vp, i64, i64, vp, vp, vp]
    L.conv_backward_atomic.argtypes = [vp] + [vp] * 7 + [i64, i64, vp, vp, vp]
    L.cgtp_csr_from_coo.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, vp, vp]
    L.cgtp_csr_workspace_bytes.argtypes = [i64, i64]
    L.cgtp_csr_workspace_bytes.restype = C.c_size_t
    L.cgtp_csr_from_coo_async.argtypes = [vp, vp, i64, i64, vp, vp, vp, vp, vp, vp, C.c_size_t, vp, vp]
    _lib = L
    return L


def _check(status: int):
    if status != 0:
        raise CgtpError(status, lib().cgtp_last_error().decode())


def _ptr(t) -> int:
    return 0 if t is None else t.data_ptr()


def _stream() -> int:
    import torch
    return torch.cuda.current_stream().cuda_stream


class Plan:
    """Owns a cgtp_plan.  device=-1: plan + source only; -2: also compile into the kernel cache;
    >= 0: compile and load on that GPU."""

    def __init__(self, irreps_x: str, irreps_y: str, irreps_z: str, paths: Optional[Sequence[Tuple]] = None,
                 mode: int = CGTP_UVU, shared_weights: bool = False, dtype: int = CGTP_F32, device: int = 0,
                 kahan_conv: bool = False, flags: int = CGTP_MUL_IR):
        L = lib()
        arr, n = None, 0
        if paths:
            n = len(paths)
            arr = (cgtp_path * n)()
            for t, q in enumerate(paths):
                q = tuple(q)
                arr[t] = cgtp_path(q[0], q[1], q[2], q[3] if len(q) > 3 else mode, q[4] if len(q) > 4 else 1.0)
        h = C.c_void_p()
        if kahan_conv:
            opt = cgtp_options(C.sizeof(cgtp_options), 1)
            _check(L.cgtp_plan_create_ex(irreps_x.encode(), irreps_y.encode(), irreps_z.encode(), arr, n, mode,
                                         int(shared_weights), dtype, device, flags, C.byref(opt), C.byref(h)))
        else:
            _check(L.cgtp_plan_create(irreps_x.encode(), irreps_y.encode(), irreps_z.encode(), arr, n, mode,
                                      int(shared_weights), dtype, device, flags, C.byref(h)))
        self._h = h
        self.dtype = dtype
        self.dim_x, self.dim_y, self.dim_z, self.n_w = (L.cgtp_plan_dim(h, t) for t in range(4))
        self.num_paths = L.cgtp_plan_num_paths(h)

    def close(self):
        if getattr(self, "_h", None):
            lib().cgtp_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:      # interpreter shutdown: module globals may already be gone
            pass

    def path(self, p: int):
        q, l = cgtp_path(), (C.c_int32 * 3)()
        nnz, woff = C.c_int32(), C.c_int64()
        _check(lib().cgtp_plan_get_path(self._h, p, C.byref(q), l, C.byref(nnz), C.byref(woff)))
        return dict(ix=q.ix, iy=q.iy, iz=q.iz, mode=q.mode, coeff=q.coeff, l=tuple(l), nnz=nnz.value, w_offset=woff.value)

    def path_nonzeros(self, p: int):
        n = lib().cgtp_plan_path_nonzeros(self._h, p, 0, None, None, None, None)
        i, j, k, v = (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_int32 * n)(), (C.c_double * n)()
        lib().cgtp_plan_path_nonzeros(self._h, p, n, i, j, k, v)
        return [(i[t], j[t], k[t], v[t]) for t in range(n)]

    def flops(self, which: int) -> int:
        return lib().cgtp_plan_flops(self._h, which)

    def source(self, kernel: int) -> Optional[str]:
        s = lib().cgtp_plan_source(self._h, kernel)
        return None if s is None else s.decode()

    def kernel_info(self, kernel: int):
        a = (C.c_int32 * 6)()
        _check(lib().cgtp_plan_kernel_info(self._h, kernel, a))
        return dict(vgprs=a[0], sgprs=a[1], lds=a[2], scratch=a[3], wg=a[4], blocks_per_cu=a[5])


def tp_forward(plan: Plan, x, y, W, z, B: Optional[int] = None):
    _check(lib().tp_forward(plan._h, _ptr(x), _ptr(y), _ptr(W), _ptr(z), x.shape[0] if B is None else B, _stream()))
    return z


def tp_backward(plan: Plan, x, y, W, gz, gx, gy, gW, B: Optional[int] = None):
    _check(lib().tp_backward(plan._h, _ptr(x), _ptr(y), _ptr(W), _ptr(gz), _ptr(gx), _ptr(gy), _ptr(gW),
                             x.shape[0] if B is None else B, _stream()))
    return gx, gy, gW


def tp_double_backward(plan: Plan, x, y, W, gz, La, Lb, LC, Lx, Ly, LW, Lgz, B: Optional[int] = None):
    _check(lib().tp_double_backward(plan._h, _ptr(x), _ptr(y), _ptr(W), _ptr(gz), _ptr(La), _ptr(Lb), _ptr(LC), _ptr(Lx),
                                    _ptr(Ly), _ptr(LW), _ptr(Lgz), x.shape[0] if B is None else B, _stream()))
    return Lx, Ly, LW, Lgz


def conv_forward(plan: Plan, x_nodes, y_edges, W_edges, z_nodes, row_ptr, col):
    V, E = z_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_forward(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(z_nodes), V, E,
                              _ptr(row_ptr), _ptr(col), _stream()))
    return z_nodes


def conv_forward_static(plan: Plan, x_nodes, y_edges, W_edges, z_nodes, row_ptr, col):
    V, E = z_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_forward_static(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(z_nodes), V, E,
                                     _ptr(row_ptr), _ptr(col), _stream()))
    return z_nodes


def conv_backward(plan: Plan, x_nodes, y_edges, W_edges, gz_nodes, gx_nodes, gy_edges, gW_edges, row_ptr, col,
                  t_row_ptr, t_perm):
    V, E = x_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_backward(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(gz_nodes), _ptr(gx_nodes),
                               _ptr(gy_edges), _ptr(gW_edges), V, E, _ptr(row_ptr), _ptr(col), _ptr(t_row_ptr),
                               _ptr(t_perm), _stream()))
    return gx_nodes, gy_edges, gW_edges


def conv_forward_perm(plan: Plan, x_nodes, y_edges, W_edges, z_nodes, row_ptr, col, edge_perm):
    V, E = z_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_forward_perm(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(z_nodes), V, E,
                                   _ptr(row_ptr), _ptr(col), _ptr(edge_perm), _stream()))
    return z_nodes


def conv_backward_perm(plan: Plan, x_nodes, y_edges, W_edges, gz_nodes, gx_nodes, gy_edges, gW_edges, row_ptr, col,
                       t_row_ptr, t_perm, edge_perm):
    V, E = x_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_backward_perm(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(gz_nodes), _ptr(gx_nodes),
                                    _ptr(gy_edges), _ptr(gW_edges), V, E, _ptr(row_ptr), _ptr(col), _ptr(t_row_ptr),
                                    _ptr(t_perm), _ptr(edge_perm), _stream()))
    return gx_nodes, gy_edges, gW_edges


def conv_double_backward(plan: Plan, x_nodes, y_edges, W_edges, gz_nodes, La_nodes, Lb_edges, LC_edges, Lx_nodes, Ly_edges,
                         LW_edges, Lgz_nodes, row_ptr, col, t_row_ptr, t_perm):
    V, E = x_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_double_backward(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(gz_nodes), _ptr(La_nodes),
                                      _ptr(Lb_edges), _ptr(LC_edges), _ptr(Lx_nodes), _ptr(Ly_edges), _ptr(LW_edges),
                                      _ptr(Lgz_nodes), V, E, _ptr(row_ptr), _ptr(col), _ptr(t_row_ptr), _ptr(t_perm),
                                      _stream()))
    return Lx_nodes, Ly_edges, LW_edges, Lgz_nodes


def conv_forward_atomic(plan: Plan, x_nodes, y_edges, W_edges, z_nodes, recv, send):
    V, E = z_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_forward_atomic(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(z_nodes), V, E,
                                     _ptr(recv), _ptr(send), _stream()))
    return z_nodes


def conv_backward_atomic(plan: Plan, x_nodes, y_edges, W_edges, gz_nodes, gx_nodes, gy_edges, gW_edges, recv, send):
    V, E = x_nodes.shape[0], y_edges.shape[0]
    _check(lib().conv_backward_atomic(plan._h, _ptr(x_nodes), _ptr(y_edges), _ptr(W_edges), _ptr(gz_nodes), _ptr(gx_nodes),
                                      _ptr(gy_edges), _ptr(gW_edges), V, E, _ptr(recv), _ptr(send), _stream()))
    return gx_nodes, gy_edges, gW_edges


def check_code_object(path: str) -> str:
    """The library's check of compiled code on a code object file: the first vector instruction placed where the
    execution mask is empty, or an empty string."""
    buf = C.create_string_buffer(256)
    _check(lib().cgtp_check_code_object(path.encode(), buf, 256))
    return buf.value.decode()


def cgtp_csr_from_coo(recv, send, V: int):
    """recv, send: int64 CUDA tensors [E].  Returns (row_ptr, col, perm, t_row_ptr, t_perm) on the same device."""
    import torch
    E = recv.shape[0]
    dev = recv.device
    row_ptr = torch.empty(V + 1, dtype=torch.int64, device=dev)
    t_row_ptr = torch.empty(V + 1, dtype=torch.int64, device=dev)
    col, perm, t_perm = (torch.empty(E, dtype=torch.int64, device=dev) for _ in range(3))
    _check(lib().cgtp_csr_from_coo(_ptr(recv), _ptr(send), E, V, _ptr(row_ptr), _ptr(col), _ptr(perm), _ptr(t_row_ptr),
                                   _ptr(t_perm), _stream()))
    return row_ptr, col, perm, t_row_ptr, t_perm


def cgtp_csr_workspace_bytes(E: int, V: int) -> int:
    return lib().cgtp_csr_workspace_bytes(E, V)


def cgtp_csr_from_coo_async(recv, send, V: int, out, workspace, bad_flag=None, transpose: bool = True):
    """Asynchronous variant on caller-owned buffers: out = (row_ptr, col, perm, t_row_ptr, t_perm) int64 CUDA tensors
    (t_row_ptr, t_perm ignored when transpose is False), workspace a uint8 CUDA tensor of at least
    cgtp_csr_workspace_bytes(E, V) bytes, bad_flag an optional int32 CUDA tensor [1].  Nothing is allocated or awaited."""
    row_ptr, col, perm, t_row_ptr, t_perm = out
    _check(lib().cgtp_csr_from_coo_async(_ptr(recv), _ptr(send), recv.shape[0], V, _ptr(row_ptr), _ptr(col), _ptr(perm),
                                         _ptr(t_row_ptr) if transpose else 0, _ptr(t_perm) if transpose else 0,
                                         _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(bad_flag), _stream()))
    return out
