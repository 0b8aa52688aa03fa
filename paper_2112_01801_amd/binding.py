"""ctypes binding of libpicassomesh.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/picassomesh.h).  PyTorch is
used for device memory and streams; all arithmetic runs in the HIP kernels.  There is no CPU
fallback: if the library has not been built the import of this module's `lib()` raises.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass
from typing import Optional

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpicassomesh.so")

PM_F32, PM_BF16 = 0, 1
PM_SH_PAPER, PM_SH_ORTHONORMAL = 0, 1
PM_OP_ADJACENCY, PM_OP_F2V, PM_OP_F2V_BWD, PM_OP_V2F, PM_OP_V2F_BWD, PM_OP_F2F, PM_OP_F2F_BWD = range(7)
PM_OP_F2V_SEP, PM_OP_F2V_SEP_BWD, PM_OP_V2F_SEP, PM_OP_V2F_SEP_BWD = 7, 8, 9, 10
PM_MAX_L = 5

EXPORTS = [
    "pm_status_string", "pm_last_error", "pm_workspace_bytes", "pm_validate_mesh", "pm_build_vf_adjacency",
    "pm_sh_basis", "pm_sh_basis_dirs", "pm_sh_basis_bwd", "pm_f2v", "pm_f2v_bwd", "pm_v2f", "pm_v2f_noalloc", "pm_v2f_bwd",
    "pm_f2f", "pm_f2f_bwd", "pm_profile_enable", "pm_profile_filter", "pm_profile_count", "pm_profile_read", "pm_profile_reset",
    "pm_peak_probe", "pm_f2v_sep", "pm_f2v_sep_bwd", "pm_v2f_sep", "pm_v2f_sep_bwd",
    "pm_cluster_ws_bytes", "pm_validate_clusters", "pm_build_cluster_map", "pm_pool", "pm_pool_bwd", "pm_unpool",
    "pm_unpool_bwd", "pm_pcloud_ws_bytes", "pm_reverse_ws_bytes", "pm_build_reverse_neighbors", "pm_validate_neighbors", "pm_pcloud_conv", "pm_pcloud_conv_bwd",
    "pm_facet_geometry", "pm_texture_ws_bytes", "pm_texture_layout", "pm_texture_bary",
    "pm_v2v_sep_ws_bytes", "pm_v2v_sep", "pm_v2v_sep_bwd",
]


class PmError(RuntimeError):
    def __init__(self, status: int, msg: str):
        super().__init__("%s (%d): %s" % (_status_name(status), status, msg))
        self.status = status


class _PmMesh(C.Structure):
    _fields_ = [("n_mesh", C.c_int32), ("n_vert", C.c_int64), ("n_facet", C.c_int64), ("vert", C.c_void_p),
                ("facet", C.c_void_p), ("vert_off", C.c_void_p), ("facet_off", C.c_void_p)]


class _PmAdj(C.Structure):
    _fields_ = [("row_ptr", C.c_void_p), ("col", C.c_void_p)]


class _PmNbr(C.Structure):
    _fields_ = [("n_query", C.c_int64), ("n_source", C.c_int64), ("nnz", C.c_int64), ("xq", C.c_void_p),
                ("xs", C.c_void_p), ("ptr", C.c_void_p), ("idx", C.c_void_p), ("rho", C.c_float),
                ("rev_ptr", C.c_void_p), ("rev_col", C.c_void_p), ("owner", C.c_void_p)]


class _PmClusterMap(C.Structure):
    _fields_ = [("n_in", C.c_int64), ("n_out", C.c_int64), ("target", C.c_void_p), ("row_ptr", C.c_void_p),
                ("col", C.c_void_p)]


_lib = None


def lib():
    """Load the HIP library; fails loudly when it has not been built (no fallback exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libpicassomesh.so is missing: run `python -m paper_2112_01801_amd.build` "
                               "(or __graft_entry__.build()) first; there is no CPU fallback")
        l = C.CDLL(LIB_PATH)
        l.pm_status_string.restype = C.c_char_p
        l.pm_status_string.argtypes = [C.c_int32]
        l.pm_last_error.restype = C.c_char_p
        l.pm_workspace_bytes.restype = C.c_size_t
        l.pm_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int, C.c_int, C.c_int, C.c_int]
        vp, i32, i64, sz = C.c_void_p, C.c_int, C.c_int64, C.c_size_t
        mp, ap = C.POINTER(_PmMesh), C.POINTER(_PmAdj)
        sig = {
            "pm_validate_mesh": [mp, vp, sz, vp],
            "pm_build_vf_adjacency": [mp, vp, vp, vp, sz, vp],
            "pm_sh_basis": [mp, i32, i32, vp, vp],
            "pm_sh_basis_dirs": [i64, vp, i32, i32, vp, vp],
            "pm_sh_basis_bwd": [i64, vp, i32, i32, vp, vp, vp],
            "pm_f2v": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp],
            "pm_f2v_bwd": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp],
            "pm_v2f": [mp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp],
            "pm_v2f_noalloc": [mp, i32, i32, i32, i32, i32, vp, vp, vp, vp],
            "pm_v2f_bwd": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp],
            "pm_f2f": [i64, i64, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, sz, vp],
            "pm_f2f_bwd": [i64, i64, vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp],
            "pm_f2v_sep": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, sz, vp],
            "pm_f2v_sep_bwd": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
            "pm_v2f_sep": [mp, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, sz, vp],
            "pm_v2f_sep_bwd": [mp, ap, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp],
        }
        cp = C.POINTER(_PmClusterMap)
        sig.update({"pm_validate_clusters": [i64, i64, vp, vp, vp, sz, vp],
                    "pm_build_cluster_map": [i64, i64, vp, vp, vp, vp, vp, vp, sz, vp],
                    "pm_pool": [cp, i32, i32, i32, vp, vp, vp, vp],
                    "pm_pool_bwd": [cp, i32, i32, i32, vp, vp, vp, vp],
                    "pm_unpool": [cp, i32, i32, vp, vp, vp],
                    "pm_unpool_bwd": [cp, i32, i32, vp, vp, vp]})
        sig.update({"pm_facet_geometry": [mp, i32, i32, vp, vp],
                    "pm_texture_layout": [mp, i32, i32, vp, vp, vp, sz, vp],
                    "pm_texture_bary": [i64, vp, vp, i64, vp, vp]})
        npt = C.POINTER(_PmNbr)
        sig.update({"pm_validate_neighbors": [npt, vp, sz, vp],
                    "pm_build_reverse_neighbors": [npt, vp, vp, vp, vp, sz, vp],
                    "pm_pcloud_conv": [npt, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, sz, vp],
                    "pm_pcloud_conv_bwd": [npt, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]})
        ep = C.POINTER(_PmEpilogue)
        sig.update({"pm_v2v_sep": [mp, ap, i32, i32, i32, i32, i32, i32, vp, vp, vp, ep, vp, vp, ep, vp, vp, vp, vp, sz, vp],
                    "pm_v2v_sep_bwd": [mp, ap, i32, i32, i32, i32, i32, i32, vp, vp, vp, ep, vp, vp, ep, vp, vp, vp, vp,
                                       vp, vp, vp, vp, vp, vp, sz, vp]})
        l.pm_v2v_sep_ws_bytes.restype = C.c_size_t
        l.pm_v2v_sep_ws_bytes.argtypes = [i32, i64, i64, i32, i32, i32, i32, i32]
        l.pm_reverse_ws_bytes.restype = C.c_size_t
        l.pm_reverse_ws_bytes.argtypes = [i64, i64]
        l.pm_pcloud_ws_bytes.restype = C.c_size_t
        l.pm_pcloud_ws_bytes.argtypes = [i32, i64, i64, i64, i32, i32, i32, i32]
        l.pm_texture_ws_bytes.restype = C.c_size_t
        l.pm_texture_ws_bytes.argtypes = [i64, C.c_int32]
        l.pm_cluster_ws_bytes.restype = C.c_size_t
        l.pm_cluster_ws_bytes.argtypes = [i64, i64]
        sig.update({"pm_profile_enable": [i32], "pm_profile_filter": [C.c_char_p], "pm_profile_count": [], "pm_profile_reset": [],
                    "pm_profile_read": [i32, C.c_char_p, sz, C.POINTER(C.c_float)],
                    "pm_peak_probe": [i32, vp, sz, C.POINTER(C.c_double), C.POINTER(C.c_double), vp]})
        for name, args in sig.items():
            f = getattr(l, name)
            f.restype = C.c_int32
            f.argtypes = args
        _lib = l
    return _lib


def _status_name(s: int) -> str:
    return lib().pm_status_string(s).decode()


def _check(s: int):
    if s != 0:
        raise PmError(s, lib().pm_last_error().decode())


def _ptr(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device-resident contiguous tensors only"
    return C.c_void_p(t.data_ptr())


def _stream(stream=None):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def torch_dtype(dtype: int):
    return torch.bfloat16 if dtype == PM_BF16 else torch.float32


@dataclass
class Mesh:
    """Device-resident packed mesh batch and the struct the C ABI takes."""
    vert: Optional[torch.Tensor]      # [V,3] float32
    facet: torch.Tensor               # [F,3] int32
    vert_off: Optional[torch.Tensor]  # [n_mesh+1] int32
    facet_off: Optional[torch.Tensor]
    n_vert: int
    n_mesh: int = 1

    @property
    def n_facet(self) -> int:
        return int(self.facet.shape[0])

    def c(self) -> _PmMesh:
        m = _PmMesh()
        m.n_mesh, m.n_vert, m.n_facet = self.n_mesh, self.n_vert, self.n_facet
        m.vert = self.vert.data_ptr() if self.vert is not None else None
        m.facet = self.facet.data_ptr() if self.facet.numel() else None
        m.vert_off = self.vert_off.data_ptr() if self.vert_off is not None else None
        m.facet_off = self.facet_off.data_ptr() if self.facet_off is not None else None
        return m


@dataclass
class Adjacency:
    row_ptr: torch.Tensor
    col: torch.Tensor

    def c(self) -> _PmAdj:
        a = _PmAdj()
        a.row_ptr = self.row_ptr.data_ptr()
        a.col = self.col.data_ptr() if self.col.numel() else None
        return a


def mesh_to_device(batch, device="cuda") -> Mesh:
    """Upload a meshgen.MeshBatch (numpy) to the GPU."""
    import numpy as np
    vert = torch.from_numpy(np.ascontiguousarray(batch.vert)).to(device)
    facet = torch.from_numpy(np.ascontiguousarray(batch.facet)).to(device)
    vo = torch.from_numpy(np.ascontiguousarray(batch.vert_off)).to(device)
    fo = torch.from_numpy(np.ascontiguousarray(batch.facet_off)).to(device)
    return Mesh(vert, facet, vo, fo, int(batch.vert.shape[0]), int(batch.n_mesh))


def pm_workspace_bytes(op: int, n_vert: int, n_facet: int, n_tex: int, L: int, cin: int, cout: int, dtype: int) -> int:
    return int(lib().pm_workspace_bytes(op, n_vert, n_facet, n_tex, L, cin, cout, dtype))


def alloc_workspace(nbytes: int, device="cuda") -> torch.Tensor:
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def pm_validate_mesh(mesh: Mesh, stream=None) -> None:
    ws = alloc_workspace(256, mesh.facet.device)
    m = mesh.c()
    _check(lib().pm_validate_mesh(C.byref(m), _ptr(ws), ws.numel(), _stream(stream)))


def pm_build_vf_adjacency(mesh: Mesh, ws: Optional[torch.Tensor] = None, stream=None) -> Adjacency:
    dev = mesh.facet.device
    row_ptr = torch.empty(mesh.n_vert + 1, dtype=torch.int32, device=dev)
    col = torch.empty(3 * mesh.n_facet, dtype=torch.int32, device=dev)
    if ws is None:
        ws = alloc_workspace(pm_workspace_bytes(PM_OP_ADJACENCY, mesh.n_vert, mesh.n_facet, 0, 0, 1, 1, PM_F32), dev)
    m = mesh.c()
    _check(lib().pm_build_vf_adjacency(C.byref(m), _ptr(row_ptr), C.c_void_p(col.data_ptr()), _ptr(ws), ws.numel(),
                                       _stream(stream)))
    return Adjacency(row_ptr, col)


def pm_sh_basis(mesh: Mesh, L: int, norm: int = PM_SH_PAPER, stream=None) -> torch.Tensor:
    K = (L + 1) ** 2
    out = torch.empty((mesh.n_facet, K), dtype=torch.float32, device=mesh.facet.device)
    m = mesh.c()
    _check(lib().pm_sh_basis(C.byref(m), L, norm, C.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def pm_sh_basis_dirs(dirs: torch.Tensor, L: int, norm: int = PM_SH_PAPER, stream=None) -> torch.Tensor:
    K = (L + 1) ** 2
    out = torch.empty((dirs.shape[0], K), dtype=torch.float32, device=dirs.device)
    _check(lib().pm_sh_basis_dirs(dirs.shape[0], _ptr(dirs), L, norm, C.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def pm_sh_basis_bwd(dirs: torch.Tensor, L: int, dbasis: torch.Tensor, norm: int = PM_SH_PAPER, stream=None):
    out = torch.empty_like(dirs)
    _check(lib().pm_sh_basis_bwd(dirs.shape[0], _ptr(dirs), L, norm, _ptr(dbasis), C.c_void_p(out.data_ptr()),
                                 _stream(stream)))
    return out


def _ws(op, V, F, P, L, cin, cout, dtype, ws, dev):
    need = pm_workspace_bytes(op, V, F, P, L, cin, cout, dtype)
    if ws is None:
        ws = alloc_workspace(need, dev)
    return ws


def pm_f2v(mesh: Mesh, adj: Adjacency, L: int, h_facet: torch.Tensor, W: torch.Tensor, dtype: int,
           norm: int = PM_SH_PAPER, out: Optional[torch.Tensor] = None, ws: Optional[torch.Tensor] = None, stream=None):
    K, cin, cout = W.shape
    dev = h_facet.device
    if out is None:
        out = torch.empty((mesh.n_vert, cout), dtype=torch_dtype(dtype), device=dev)
    ws = _ws(PM_OP_F2V, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_f2v(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_facet), _ptr(W),
                        C.c_void_p(out.data_ptr()), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def pm_f2v_bwd(mesh: Mesh, adj: Adjacency, L: int, h_facet, W, dg_vert, dtype: int, norm: int = PM_SH_PAPER,
               want_dh=True, want_dW=True, dh=None, dW=None, ws=None, stream=None):
    K, cin, cout = W.shape
    dev = h_facet.device
    if want_dh and dh is None:
        dh = torch.empty((mesh.n_facet, cin), dtype=torch_dtype(dtype), device=dev)
    if want_dW and dW is None:
        dW = torch.empty((K, cin, cout), dtype=torch.float32, device=dev)
    ws = _ws(PM_OP_F2V_BWD, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_f2v_bwd(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_facet), _ptr(W), _ptr(dg_vert),
                            _ptr(dh) if want_dh else None, _ptr(dW) if want_dW else None, _ptr(ws), ws.numel(),
                            _stream(stream)))
    return (dh if want_dh else None), (dW if want_dW else None)


def pm_v2f(mesh: Mesh, L: int, h_vert, W, dtype: int, norm: int = PM_SH_PAPER, out=None, ws=None, stream=None):
    K, cin, cout = W.shape
    dev = h_vert.device
    if out is None:
        out = torch.empty((mesh.n_facet, cout), dtype=torch_dtype(dtype), device=dev)
    ws = _ws(PM_OP_V2F, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m = mesh.c()
    _check(lib().pm_v2f(C.byref(m), L, norm, cin, cout, dtype, _ptr(h_vert), _ptr(W), C.c_void_p(out.data_ptr()),
                        _ptr(ws), ws.numel(), _stream(stream)))
    return out


def pm_v2f_noalloc(mesh: Mesh, L: int, h_vert, W, dtype: int, out, norm: int = PM_SH_PAPER, stream=None):
    """pm_v2f without a workspace: the library's static scratch array holds the coefficient image; `out` is the caller's."""
    K, cin, cout = W.shape
    m = mesh.c()
    _check(lib().pm_v2f_noalloc(C.byref(m), L, norm, cin, cout, dtype, _ptr(h_vert), _ptr(W), C.c_void_p(out.data_ptr()),
                                _stream(stream)))
    return out


def pm_v2f_bwd(mesh: Mesh, adj: Adjacency, L: int, h_vert, W, dg_facet, dtype: int, norm: int = PM_SH_PAPER,
               want_dh=True, want_dW=True, dh=None, dW=None, ws=None, stream=None):
    K, cin, cout = W.shape
    dev = h_vert.device
    if want_dh and dh is None:
        dh = torch.empty((mesh.n_vert, cin), dtype=torch_dtype(dtype), device=dev)
    if want_dW and dW is None:
        dW = torch.empty((K, cin, cout), dtype=torch.float32, device=dev)
    ws = _ws(PM_OP_V2F_BWD, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_v2f_bwd(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_vert), _ptr(W), _ptr(dg_facet),
                            _ptr(dh) if want_dh else None, _ptr(dW) if want_dW else None, _ptr(ws), ws.numel(),
                            _stream(stream)))
    return (dh if want_dh else None), (dW if want_dW else None)


def pm_f2f(tex_off: torch.Tensor, bary: torch.Tensor, L: int, h_tex, W, dtype: int, norm: int = PM_SH_PAPER, out=None,
           ws=None, stream=None):
    K, cin, cout = W.shape
    F, P = int(tex_off.shape[0]) - 1, int(bary.shape[0])
    dev = tex_off.device
    if out is None:
        out = torch.empty((F, cout), dtype=torch_dtype(dtype), device=dev)
    ws = _ws(PM_OP_F2F, 0, F, P, L, cin, cout, dtype, ws, dev)
    _check(lib().pm_f2f(F, P, _ptr(tex_off), _ptr(bary) if P else None, L, norm, cin, cout, dtype,
                        _ptr(h_tex) if P else None, _ptr(W), C.c_void_p(out.data_ptr()), _ptr(ws), ws.numel(),
                        _stream(stream)))
    return out


def pm_f2f_bwd(tex_off, bary, L: int, h_tex, W, dg_facet, dtype: int, norm: int = PM_SH_PAPER, want_dh=True,
               want_dW=True, dh=None, dW=None, ws=None, stream=None):
    K, cin, cout = W.shape
    F, P = int(tex_off.shape[0]) - 1, int(bary.shape[0])
    dev = tex_off.device
    if want_dh and dh is None:
        dh = torch.empty((P, cin), dtype=torch_dtype(dtype), device=dev)
    if want_dW and dW is None:
        dW = torch.empty((K, cin, cout), dtype=torch.float32, device=dev)
    ws = _ws(PM_OP_F2F_BWD, 0, F, P, L, cin, cout, dtype, ws, dev)
    _check(lib().pm_f2f_bwd(F, P, _ptr(tex_off), _ptr(bary) if P else None, L, norm, cin, cout, dtype,
                            _ptr(h_tex) if P else None, _ptr(W), _ptr(dg_facet), _ptr(dh) if want_dh else None,
                            _ptr(dW) if want_dW else None, _ptr(ws), ws.numel(), _stream(stream)))
    return (dh if want_dh else None), (dW if want_dW else None)


def _check_sep(alpha, P, dtype):
    assert alpha.dtype == torch.float32, "alpha is always fp32"
    assert P.dtype == torch_dtype(dtype) and alpha.shape[1] == P.shape[0]


def pm_f2v_sep(mesh: Mesh, adj: Adjacency, L: int, h_facet, alpha, P, dtype: int, norm: int = PM_SH_PAPER, out=None,
               ws=None, stream=None, save_z: bool = False):
    """Depth-wise separable facet2vertex: alpha [K,cin] fp32, P [cin,cout] in the feature dtype.
    With save_z the vertex means before the point-wise matrix come back too: (g, z), z for pm_f2v_sep_bwd."""
    _check_sep(alpha, P, dtype)
    cin, cout = P.shape
    dev = h_facet.device
    if out is None:
        out = torch.empty((mesh.n_vert, cout), dtype=torch_dtype(dtype), device=dev)
    z = torch.empty((mesh.n_vert, cin), dtype=torch_dtype(dtype), device=dev) if save_z else None
    ws = _ws(PM_OP_F2V_SEP, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_f2v_sep(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_facet), _ptr(alpha), _ptr(P),
                            C.c_void_p(out.data_ptr()), C.c_void_p(z.data_ptr()) if z is not None and z.numel() else None,
                            _ptr(ws), ws.numel(), _stream(stream)))
    return (out, z) if save_z else out


def pm_f2v_sep_bwd(mesh: Mesh, adj: Adjacency, L: int, h_facet, alpha, P, dg_vert, dtype: int, norm: int = PM_SH_PAPER,
                   want_dh=True, want_dw=True, ws=None, stream=None, z_saved=None):
    """Returns (dh, dalpha, dP); dalpha and dP are fp32 and come together.  z_saved: the z of pm_f2v_sep(save_z)."""
    _check_sep(alpha, P, dtype)
    cin, cout = P.shape
    K = alpha.shape[0]
    dev = h_facet.device
    dh = torch.empty((mesh.n_facet, cin), dtype=torch_dtype(dtype), device=dev) if want_dh else None
    da = torch.empty((K, cin), dtype=torch.float32, device=dev) if want_dw else None
    dP = torch.empty((cin, cout), dtype=torch.float32, device=dev) if want_dw else None
    ws = _ws(PM_OP_F2V_SEP_BWD, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_f2v_sep_bwd(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_facet), _ptr(alpha), _ptr(P),
                                _ptr(dg_vert), _ptr(z_saved) if z_saved is not None and z_saved.numel() else None,
                                _ptr(dh), _ptr(da), _ptr(dP), _ptr(ws), ws.numel(), _stream(stream)))
    return dh, da, dP


def pm_v2f_sep(mesh: Mesh, L: int, h_vert, alpha, P, dtype: int, norm: int = PM_SH_PAPER, out=None, ws=None,
               stream=None):
    _check_sep(alpha, P, dtype)
    cin, cout = P.shape
    dev = h_vert.device
    if out is None:
        out = torch.empty((mesh.n_facet, cout), dtype=torch_dtype(dtype), device=dev)
    ws = _ws(PM_OP_V2F_SEP, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m = mesh.c()
    _check(lib().pm_v2f_sep(C.byref(m), L, norm, cin, cout, dtype, _ptr(h_vert), _ptr(alpha), _ptr(P),
                            C.c_void_p(out.data_ptr()), _ptr(ws), ws.numel(), _stream(stream)))
    return out


def pm_v2f_sep_bwd(mesh: Mesh, adj: Adjacency, L: int, h_vert, alpha, P, dg_facet, dtype: int, norm: int = PM_SH_PAPER,
                   want_dh=True, want_dw=True, ws=None, stream=None):
    _check_sep(alpha, P, dtype)
    cin, cout = P.shape
    K = alpha.shape[0]
    dev = h_vert.device
    dh = torch.empty((mesh.n_vert, cin), dtype=torch_dtype(dtype), device=dev) if want_dh else None
    da = torch.empty((K, cin), dtype=torch.float32, device=dev) if want_dw else None
    dP = torch.empty((cin, cout), dtype=torch.float32, device=dev) if want_dw else None
    ws = _ws(PM_OP_V2F_SEP_BWD, mesh.n_vert, mesh.n_facet, 0, L, cin, cout, dtype, ws, dev)
    m, a = mesh.c(), adj.c()
    _check(lib().pm_v2f_sep_bwd(C.byref(m), C.byref(a), L, norm, cin, cout, dtype, _ptr(h_vert), _ptr(alpha), _ptr(P),
                                _ptr(dg_facet), _ptr(dh), _ptr(da), _ptr(dP), _ptr(ws), ws.numel(), _stream(stream)))
    return dh, da, dP


class _PmEpilogue(C.Structure):
    _fields_ = [("scale", C.c_void_p), ("shift", C.c_void_p), ("relu", C.c_int)]


class Epilogue:
    """Per-channel affine map (fp32 device vectors or None) and optional ReLU after a stage of pm_v2v_sep."""

    def __init__(self, scale=None, shift=None, relu=False):
        for t in (scale, shift):
            assert t is None or (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous())
        self.scale, self.shift, self.relu = scale, shift, bool(relu)

    def c(self):
        return _PmEpilogue(self.scale.data_ptr() if self.scale is not None else None,
                           self.shift.data_ptr() if self.shift is not None else None, int(self.relu))


def _ep(e):
    return C.byref(e.c()) if e is not None else None


def pm_v2v_sep(mesh: Mesh, adj: Adjacency, L: int, h_vert, alpha1, P1, ep1, alpha2, P2, ep2, dtype: int,
               norm: int = PM_SH_PAPER, ws=None, stream=None, save: bool = False):
    """Separable vertex2vertex block (vertex2facet -> epilogue -> facet2vertex -> epilogue); ep1 / ep2: Epilogue or None.
    With save the activated facet features and the vertex means come back too, (out, g, z), for pm_v2v_sep_bwd."""
    _check_sep(alpha1, P1, dtype)
    _check_sep(alpha2, P2, dtype)
    cin, cmid = P1.shape
    cout = P2.shape[1]
    assert P2.shape[0] == cmid
    dev, td = h_vert.device, torch_dtype(dtype)
    out = torch.empty((mesh.n_vert, cout), dtype=td, device=dev)
    g = torch.empty((mesh.n_facet, cmid), dtype=td, device=dev) if save else None
    z = torch.empty((mesh.n_vert, cmid), dtype=td, device=dev) if save else None
    if ws is None:
        ws = alloc_workspace(lib().pm_v2v_sep_ws_bytes(0, mesh.n_vert, mesh.n_facet, L, cin, cmid, cout, dtype), dev)
    m, a = mesh.c(), adj.c()
    opt = lambda t: _ptr(t) if t is not None and t.numel() else None
    _check(lib().pm_v2v_sep(C.byref(m), C.byref(a), L, norm, cin, cmid, cout, dtype, _ptr(h_vert), _ptr(alpha1), _ptr(P1),
                            _ep(ep1), _ptr(alpha2), _ptr(P2), _ep(ep2), C.c_void_p(out.data_ptr()), opt(g), opt(z),
                            _ptr(ws), ws.numel(), _stream(stream)))
    return (out, g, z) if save else out


def pm_v2v_sep_bwd(mesh: Mesh, adj: Adjacency, L: int, h_vert, alpha1, P1, ep1, alpha2, P2, ep2, g_saved, z_saved,
                   out_saved, d_out, dtype: int, norm: int = PM_SH_PAPER, want_dh=True, want_dw=True, ws=None, stream=None):
    """Returns (dh, dalpha1, dP1, dalpha2, dP2) for fixed epilogue coefficients; the weight gradients are fp32."""
    _check_sep(alpha1, P1, dtype)
    _check_sep(alpha2, P2, dtype)
    cin, cmid = P1.shape
    cout = P2.shape[1]
    K = alpha1.shape[0]
    dev = h_vert.device
    f32 = dict(dtype=torch.float32, device=dev)
    dh = torch.empty((mesh.n_vert, cin), dtype=torch_dtype(dtype), device=dev) if want_dh else None
    da1 = torch.empty((K, cin), **f32) if want_dw else None
    dP1 = torch.empty((cin, cmid), **f32) if want_dw else None
    da2 = torch.empty((K, cmid), **f32) if want_dw else None
    dP2 = torch.empty((cmid, cout), **f32) if want_dw else None
    if ws is None:
        ws = alloc_workspace(lib().pm_v2v_sep_ws_bytes(1, mesh.n_vert, mesh.n_facet, L, cin, cmid, cout, dtype), dev)
    m, a = mesh.c(), adj.c()
    opt = lambda t: _ptr(t) if t is not None and t.numel() else None
    _check(lib().pm_v2v_sep_bwd(C.byref(m), C.byref(a), L, norm, cin, cmid, cout, dtype, _ptr(h_vert), _ptr(alpha1),
                                _ptr(P1), _ep(ep1), _ptr(alpha2), _ptr(P2), _ep(ep2), opt(g_saved), opt(z_saved),
                                opt(out_saved), opt(d_out), opt(dh), _ptr(da1), _ptr(dP1), _ptr(da2), _ptr(dP2),
                                _ptr(ws), ws.numel(), _stream(stream)))
    return dh, da1, dP1, da2, dP2


# ---- pooling / unpooling over vertex clusters -------------------------------------------------------
PM_POOL_MAX, PM_POOL_AVG = 0, 1


@dataclass
class ClusterMap:
    n_in: int
    n_out: int
    target: torch.Tensor
    row_ptr: torch.Tensor
    col: torch.Tensor

    def c(self) -> _PmClusterMap:
        m = _PmClusterMap()
        m.n_in, m.n_out = self.n_in, self.n_out
        m.target = self.target.data_ptr() if self.n_in else None
        m.row_ptr = self.row_ptr.data_ptr()
        m.col = self.col.data_ptr() if self.n_in else None
        return m


def pm_cluster_ws_bytes(n_in: int, n_out: int) -> int:
    return int(lib().pm_cluster_ws_bytes(n_in, n_out))


def pm_validate_clusters(vcluster: torch.Tensor, iomap: torch.Tensor, n_out: int, stream=None) -> None:
    n_in = vcluster.shape[0]
    ws = alloc_workspace(pm_cluster_ws_bytes(n_in, n_out), vcluster.device)
    _check(lib().pm_validate_clusters(n_in, n_out, _ptr(vcluster), _ptr(iomap), _ptr(ws), ws.numel(), _stream(stream)))


def pm_build_cluster_map(vcluster: torch.Tensor, iomap: torch.Tensor, n_out: int, ws=None, stream=None) -> ClusterMap:
    assert vcluster.dtype == torch.int32 and iomap.dtype == torch.int32 and vcluster.shape == iomap.shape
    n_in, dev = vcluster.shape[0], vcluster.device
    target = torch.empty(n_in, dtype=torch.int32, device=dev)
    row_ptr = torch.empty(n_out + 1, dtype=torch.int32, device=dev)
    col = torch.empty(n_in, dtype=torch.int32, device=dev)
    if ws is None:
        ws = alloc_workspace(pm_cluster_ws_bytes(n_in, n_out), dev)
    _check(lib().pm_build_cluster_map(n_in, n_out, _ptr(vcluster), _ptr(iomap), C.c_void_p(target.data_ptr()),
                                      _ptr(row_ptr), C.c_void_p(col.data_ptr()), _ptr(ws), ws.numel(), _stream(stream)))
    return ClusterMap(n_in, n_out, target, row_ptr, col)


def pm_pool(cm: ClusterMap, mode: int, h_in: torch.Tensor, dtype: int, want_argmax: bool = True, stream=None):
    """(h_out [n_out, C], argmax [n_out, C] int32 or None)."""
    Cc = h_in.shape[1]
    assert h_in.dtype == torch_dtype(dtype) and h_in.shape[0] == cm.n_in
    out = torch.empty((cm.n_out, Cc), dtype=h_in.dtype, device=h_in.device)
    arg = torch.empty((cm.n_out, Cc), dtype=torch.int32, device=h_in.device) if (mode == PM_POOL_MAX and want_argmax) else None
    m = cm.c()
    _check(lib().pm_pool(C.byref(m), mode, Cc, dtype, C.c_void_p(h_in.data_ptr()), C.c_void_p(out.data_ptr()),
                         C.c_void_p(arg.data_ptr()) if arg is not None else None, _stream(stream)))
    return out, arg


def pm_pool_bwd(cm: ClusterMap, mode: int, dg_out: torch.Tensor, dtype: int, argmax=None, stream=None) -> torch.Tensor:
    Cc = dg_out.shape[1]
    assert dg_out.dtype == torch_dtype(dtype) and dg_out.shape[0] == cm.n_out
    out = torch.empty((cm.n_in, Cc), dtype=dg_out.dtype, device=dg_out.device)
    m = cm.c()
    _check(lib().pm_pool_bwd(C.byref(m), mode, Cc, dtype, C.c_void_p(dg_out.data_ptr()),
                             C.c_void_p(argmax.data_ptr()) if argmax is not None else None,
                             C.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def pm_unpool(cm: ClusterMap, h_coarse: torch.Tensor, dtype: int, stream=None) -> torch.Tensor:
    Cc = h_coarse.shape[1]
    assert h_coarse.dtype == torch_dtype(dtype) and h_coarse.shape[0] == cm.n_out
    out = torch.empty((cm.n_in, Cc), dtype=h_coarse.dtype, device=h_coarse.device)
    m = cm.c()
    _check(lib().pm_unpool(C.byref(m), Cc, dtype, C.c_void_p(h_coarse.data_ptr()), C.c_void_p(out.data_ptr()),
                           _stream(stream)))
    return out


def pm_unpool_bwd(cm: ClusterMap, dg_fine: torch.Tensor, dtype: int, stream=None) -> torch.Tensor:
    Cc = dg_fine.shape[1]
    assert dg_fine.dtype == torch_dtype(dtype) and dg_fine.shape[0] == cm.n_in
    out = torch.empty((cm.n_out, Cc), dtype=dg_fine.dtype, device=dg_fine.device)
    m = cm.c()
    _check(lib().pm_unpool_bwd(C.byref(m), Cc, dtype, C.c_void_p(dg_fine.data_ptr()), C.c_void_p(out.data_ptr()),
                               _stream(stream)))
    return out


# ---- point-cloud convolution with the radial term ----------------------------------------------------
@dataclass
class Neighbors:
    """Caller-supplied neighbour lists of a range search: xq [M,3], xs [N,3] fp32, ptr [M+1], idx [nnz] int32."""
    xq: torch.Tensor
    xs: torch.Tensor
    ptr: torch.Tensor
    idx: torch.Tensor
    rho: float
    rev_ptr: Optional[torch.Tensor] = None      # reverse lists (pm_build_reverse_neighbors), optional
    rev_col: Optional[torch.Tensor] = None
    owner: Optional[torch.Tensor] = None

    def c(self) -> _PmNbr:
        n = _PmNbr()
        n.n_query, n.n_source, n.nnz = self.xq.shape[0], self.xs.shape[0], self.idx.shape[0]
        n.xq = self.xq.data_ptr() if self.xq.numel() else None
        n.xs = self.xs.data_ptr() if self.xs.numel() else None
        n.ptr = self.ptr.data_ptr()
        n.idx = self.idx.data_ptr() if self.idx.numel() else None
        n.rho = float(self.rho)
        if self.rev_ptr is not None:
            n.rev_ptr = self.rev_ptr.data_ptr()
            n.rev_col = self.rev_col.data_ptr() if self.rev_col.numel() else None
            n.owner = self.owner.data_ptr() if self.owner.numel() else None
        return n


def pm_validate_neighbors(nb: Neighbors, stream=None) -> None:
    ws = alloc_workspace(256, nb.ptr.device)
    n = nb.c()
    _check(lib().pm_validate_neighbors(C.byref(n), _ptr(ws), ws.numel(), _stream(stream)))


def pm_build_reverse_neighbors(nb: Neighbors, stream=None) -> Neighbors:
    """The same lists with the reverse lists attached (built once, reused by every backward call)."""
    dev, nnz, N = nb.ptr.device, nb.idx.shape[0], nb.xs.shape[0]
    rev_ptr = torch.empty(N + 1, dtype=torch.int32, device=dev)
    rev_col = torch.empty(nnz, dtype=torch.int32, device=dev)
    owner = torch.empty(nnz, dtype=torch.int32, device=dev)
    ws = alloc_workspace(int(lib().pm_reverse_ws_bytes(N, nnz)), dev)
    n = nb.c()
    vp = lambda t: C.c_void_p(t.data_ptr()) if t.numel() else None
    _check(lib().pm_build_reverse_neighbors(C.byref(n), _ptr(rev_ptr), vp(rev_col), vp(owner), _ptr(ws), ws.numel(),
                                            _stream(stream)))
    return Neighbors(nb.xq, nb.xs, nb.ptr, nb.idx, nb.rho, rev_ptr, rev_col, owner)


def _pc_ws(bwd, nb, L, cin, cout, dtype, ws):
    if ws is None:
        ws = alloc_workspace(int(lib().pm_pcloud_ws_bytes(bwd, nb.xq.shape[0], nb.xs.shape[0], nb.idx.shape[0], L, cin,
                                                          cout, dtype)), nb.ptr.device)
    return ws


def pm_pcloud_conv(nb: Neighbors, L: int, h, alpha, c0, P, dtype: int, norm: int = PM_SH_PAPER, ws=None, stream=None,
                   save_y: bool = False):
    """g [M, cout]: alpha [K,cin] and c0 [cin] fp32, P [cin,cout] and h [N,cin] in the feature dtype.
    With save_y the depth-wise output comes back too: (g, y), y for pm_pcloud_conv_bwd."""
    _check_sep(alpha, P, dtype)
    assert c0.dtype == torch.float32 and c0.shape[0] == P.shape[0]
    cin, cout = P.shape
    out = torch.empty((nb.xq.shape[0], cout), dtype=torch_dtype(dtype), device=h.device)
    y = torch.empty((nb.xq.shape[0], cin), dtype=torch_dtype(dtype), device=h.device) if save_y else None
    ws = _pc_ws(0, nb, L, cin, cout, dtype, ws)
    n = nb.c()
    _check(lib().pm_pcloud_conv(C.byref(n), L, norm, cin, cout, dtype, C.c_void_p(h.data_ptr()), _ptr(alpha), _ptr(c0),
                                _ptr(P), C.c_void_p(out.data_ptr()),
                                C.c_void_p(y.data_ptr()) if y is not None and y.numel() else None, _ptr(ws), ws.numel(),
                                _stream(stream)))
    return (out, y) if save_y else out


def pm_pcloud_conv_bwd(nb: Neighbors, L: int, h, alpha, c0, P, dg, dtype: int, norm: int = PM_SH_PAPER,
                       want_dh: bool = True, want_dw: bool = True, ws=None, stream=None, y_saved=None):
    """(dh [N,cin], dalpha [K,cin], dc0 [cin], dP [cin,cout]); the parameter gradients come together or not at all.
    y_saved: the y of pm_pcloud_conv(save_y)."""
    _check_sep(alpha, P, dtype)
    cin, cout = P.shape
    dev = h.device
    dh = torch.empty((nb.xs.shape[0], cin), dtype=torch_dtype(dtype), device=dev) if want_dh else None
    da = torch.empty(alpha.shape, dtype=torch.float32, device=dev) if want_dw else None
    dc = torch.empty(c0.shape, dtype=torch.float32, device=dev) if want_dw else None
    dP = torch.empty((cin, cout), dtype=torch.float32, device=dev) if want_dw else None
    ws = _pc_ws(1, nb, L, cin, cout, dtype, ws)
    n = nb.c()
    vp = lambda t: C.c_void_p(t.data_ptr()) if t is not None else None
    _check(lib().pm_pcloud_conv_bwd(C.byref(n), L, norm, cin, cout, dtype, vp(h), _ptr(alpha), _ptr(c0), _ptr(P), vp(dg),
                                    vp(y_saved) if y_saved is not None and y_saved.numel() else None,
                                    vp(dh), vp(da), vp(dc), vp(dP), _ptr(ws), ws.numel(), _stream(stream)))
    return dh, da, dc, dP


# ---- input preparation -------------------------------------------------------------------------------
def pm_facet_geometry(mesh: Mesh, dtype: int, with_heights: bool = False, stream=None) -> torch.Tensor:
    """[n_facet, 9 or 12]: edge lengths, inner-angle cosines, unit normal, optionally corner heights (Eq. 9)."""
    out = torch.empty((mesh.n_facet, 12 if with_heights else 9), dtype=torch_dtype(dtype), device=mesh.facet.device)
    m = mesh.c()
    _check(lib().pm_facet_geometry(C.byref(m), 1 if with_heights else 0, dtype, C.c_void_p(out.data_ptr()), _stream(stream)))
    return out


def pm_texture_layout(mesh: Mesh, alpha: int, beta: int, stream=None):
    """(gamma [F] int32, tex_off [F+1] int32, bary [P, 3] fp32) of Eq. 8; reads the point total back once."""
    dev = mesh.facet.device
    gamma = torch.empty(mesh.n_facet, dtype=torch.int32, device=dev)
    tex_off = torch.empty(mesh.n_facet + 1, dtype=torch.int32, device=dev)
    ws = alloc_workspace(int(lib().pm_texture_ws_bytes(mesh.n_facet, mesh.n_mesh)), dev)
    m = mesh.c()
    _check(lib().pm_texture_layout(C.byref(m), alpha, beta, C.c_void_p(gamma.data_ptr()), _ptr(tex_off), _ptr(ws),
                                   ws.numel(), _stream(stream)))
    n_tex = int(tex_off[-1].item())
    bary = torch.empty((n_tex, 3), dtype=torch.float32, device=dev)
    _check(lib().pm_texture_bary(mesh.n_facet, C.c_void_p(gamma.data_ptr()), _ptr(tex_off), n_tex,
                                 C.c_void_p(bary.data_ptr()), _stream(stream)))
    return gamma, tex_off, bary


def pm_profile_enable(on: bool) -> None:
    _check(lib().pm_profile_enable(1 if on else 0))


def pm_profile_filter(label_part: str = "") -> None:
    """Record only kernels whose "<entry point>/<kernel>" label contains `label_part` ("" = all)."""
    _check(lib().pm_profile_filter(label_part.encode()))


def pm_profile_reset() -> None:
    _check(lib().pm_profile_reset())


PM_PEAK_MFMA_BF16_ONES, PM_PEAK_MFMA_BF16_RANDOM, PM_PEAK_MFMA_F32, PM_PEAK_HBM_COPY = 0, 1, 2, 3


def pm_peak_probe(kind: int, ws: torch.Tensor, stream=None):
    """(rate, shader clock in MHz) of one issue-loop probe; rate in TFLOP/s, or GB/s for the copy."""
    val, clk = C.c_double(), C.c_double()
    _check(lib().pm_peak_probe(kind, _ptr(ws), ws.numel() * ws.element_size(), C.byref(val), C.byref(clk),
                               _stream(stream)))
    return float(val.value), float(clk.value)


def pm_profile_read():
    """All records since the last reset as a list of (label, milliseconds)."""
    out = []
    buf = C.create_string_buffer(64)
    ms = C.c_float()
    for i in range(lib().pm_profile_count()):
        _check(lib().pm_profile_read(i, buf, 64, C.byref(ms)))
        out.append((buf.value.decode(), float(ms.value)))
    return out
