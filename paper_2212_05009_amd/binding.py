"""ctypes binding of include/gcn.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libgcn.so")

F32, BF16 = 0, 1
BUILD_CSC = 1
EPI_NONE, EPI_RELU, EPI_MASK = 0, 1, 2
PART_LOCAL, PART_HALO = 1, 2
ACT_NONE, ACT_RELU = 0, 1


class GcnError(RuntimeError):
    pass


class ProfileRec(C.Structure):
    """Mirror of gcn_profile_rec."""
    _fields_ = [("kind", C.c_int32), ("d", C.c_int32), ("dtype", C.c_int32), ("reserved", C.c_int32),
                ("rows", C.c_int64), ("inner", C.c_int64), ("alg_bytes", C.c_double),
                ("touched_bytes", C.c_double), ("flops", C.c_double), ("ms", C.c_double)]


KIND_NAMES = ["spmm", "spmm_t", "spmm_finish", "gemm_nn", "gemm_tn", "gemm_tn_sum", "softmax_xent", "gather", "other"]


def library_path() -> str:
    return _LIB_PATH


def _load():
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            f"{_LIB_PATH} is missing: build the HIP library first "
            "(python -m paper_2212_05009_amd.build); there is no fallback path")
    lib = C.CDLL(_LIB_PATH)
    i32p, i64p, f32p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_int64), C.POINTER(C.c_float), C.c_void_p
    lib.gcn_last_error.restype = C.c_char_p
    lib.gcn_last_error.argtypes = []
    lib.gcn_csr_build.argtypes = [vp, vp, C.c_int64, C.c_int64, C.c_int64, C.c_int64, vp, C.c_int, vp, C.POINTER(vp)]
    lib.gcn_csr_info.argtypes = [vp, i64p, i64p, i64p]
    lib.gcn_csr_arrays.argtypes = [vp] + [C.POINTER(vp)] * 8
    lib.gcn_csr_free.argtypes = [vp]
    lib.gcn_spmm.argtypes = [vp, vp, C.c_int64, C.c_int, C.c_int, vp, C.c_int64, C.c_int, vp, vp, C.c_int64, vp]
    lib.gcn_spmm_noalloc.argtypes = [vp, vp, C.c_int64, C.c_int, C.c_int, vp, C.c_int64, C.c_int, vp, vp, C.c_int64, vp]
    lib.gcn_spmm_noalloc.restype = C.c_int
    lib.gcn_spmm_t.argtypes = [vp, vp, C.c_int64, C.c_int, C.c_int, vp, C.c_int64, C.c_int, vp, C.c_int64, vp]
    lib.gcn_halo_gather.argtypes = [vp, C.c_int64, C.c_int64, C.c_int, C.c_int, vp, C.c_int64, vp, C.c_int64, vp]
    lib.gcn_layer_fwd.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp]
    lib.gcn_layer_bwd.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, vp]
    lib.gcn_layer_fwd_ld.argtypes = [vp, vp, C.c_int64, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, C.c_int64, vp, C.c_int64,
                                     vp, C.c_int64, vp]
    lib.gcn_layer_fwd_ld.restype = C.c_int
    lib.gcn_layer_bwd_ld.argtypes = [vp, vp, C.c_int64, vp, C.c_int64, vp, C.c_int, C.c_int, C.c_int, vp, C.c_int64, vp, C.c_int64,
                                     vp, vp, vp, C.c_int64, vp]
    lib.gcn_layer_bwd_ld.restype = C.c_int
    lib.gcn_softmax_xent.argtypes = [vp, C.c_int64, C.c_int64, C.c_int, C.c_int, vp, C.c_float, vp, vp, C.c_int64, vp]
    lib.gcn_spmm_part.argtypes = [vp, C.c_int, vp, C.c_int64, C.c_int, C.c_int, vp, C.c_int64, C.c_int, vp, vp, C.c_int64, vp]
    lib.gcn_spmm_part.restype = C.c_int
    lib.gcn_dense_fwd.argtypes = [vp, C.c_int64, C.c_int64, vp, vp, C.c_int, C.c_int, C.c_int, C.c_int, vp, vp, C.c_int64, vp]
    lib.gcn_dense_fwd.restype = C.c_int
    lib.gcn_layer_bwd_pull.argtypes = [vp, C.c_int, vp, C.c_int64, vp, C.c_int, C.c_int, C.c_int, vp, C.c_int64, vp, vp, vp, vp, vp, vp]
    lib.gcn_layer_bwd_pull.restype = C.c_int
    lib.gcn_partition_stats.argtypes = [vp, vp, C.c_int, vp, vp, vp, vp, vp, vp, vp]
    lib.gcn_partition_stats.restype = C.c_int
    lib.gcn_csr_induced.argtypes = [vp, vp, C.c_int64, C.c_int, vp, C.POINTER(C.c_void_p)]
    lib.gcn_csr_induced.restype = C.c_int
    lib.gcn_sgd_update.argtypes = [vp, vp, C.c_int64, C.c_float, vp]
    lib.gcn_sgd_update.restype = C.c_int
    lib.gcn_profile_enable.argtypes = [C.c_int]
    lib.gcn_profile_enable.restype = C.c_int
    lib.gcn_profile_filter.argtypes = [C.c_int, C.c_int]
    lib.gcn_profile_filter.restype = C.c_int
    lib.gcn_profile_count.argtypes = [i64p]
    lib.gcn_profile_count.restype = C.c_int64
    lib.gcn_profile_get.argtypes = [C.c_int64, C.POINTER(ProfileRec)]
    lib.gcn_profile_get.restype = C.c_int
    lib.gcn_debug_max_grid_x.argtypes = [C.c_int64]
    lib.gcn_debug_max_grid_x.restype = C.c_int
    lib.gcn_feature_ld.argtypes = [C.c_int, C.c_int]
    lib.gcn_feature_ld.restype = C.c_int64
    lib.gcn_debug_set_tuning.argtypes = [C.c_char_p, C.c_int]
    lib.gcn_debug_set_tuning.restype = C.c_int
    for name in ("gcn_csr_build", "gcn_csr_info", "gcn_csr_arrays", "gcn_csr_free", "gcn_spmm", "gcn_spmm_t",
                 "gcn_halo_gather", "gcn_layer_fwd", "gcn_layer_bwd", "gcn_softmax_xent"):
        getattr(lib, name).restype = C.c_int
    return lib


_lib = _load()
_hip = C.CDLL("libamdhip64.so.7")     # already loaded by torch; same runtime instance as the library's
_hip.hipMemcpy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int]
_hip.hipMemcpy.restype = C.c_int


def _hip_memcpy(dst: int, src: int, nbytes: int) -> int:
    return _hip.hipMemcpy(C.c_void_p(dst), C.c_void_p(src), C.c_size_t(nbytes), 3)   # 3 = device to device


def _check(rc: int, what: str):
    if rc != 0:
        raise GcnError(f"{what} failed ({rc}): {_lib.gcn_last_error().decode()}")


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dtype_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported feature dtype {t.dtype}")


def _dev(t: torch.Tensor, dtype=None, what="tensor"):
    if not t.is_cuda:
        raise TypeError(f"{what} must live on the GPU")
    if dtype is not None and t.dtype != dtype:
        raise TypeError(f"{what} must have dtype {dtype}, got {t.dtype}")
    return t


def _rowmajor(t: torch.Tensor, what="matrix"):
    """(ld, d): accepts 2-D tensors whose rows are contiguous (row stride >= number of columns)."""
    if t.dim() != 2 or (t.shape[1] > 1 and t.stride(1) != 1) or t.stride(0) < t.shape[1]:
        raise TypeError(f"{what} must be a row-major 2-D tensor")
    return t.stride(0), t.shape[1]


class Csr:
    """Owning wrapper of a gcn_csr_t handle."""

    def __init__(self, handle, device):
        self._h = handle
        self.device = device
        nr, nh, nnz = C.c_int64(), C.c_int64(), C.c_int64()
        _check(_lib.gcn_csr_info(self._h, C.byref(nr), C.byref(nh), C.byref(nnz)), "gcn_csr_info")
        self.nr, self.nh, self.nnz = nr.value, nh.value, nnz.value
        self.nc = self.nr + self.nh

    @property
    def handle(self):
        if self._h is None:
            raise GcnError("handle already freed")
        return self._h

    def arrays(self):
        """Copies of the device arrays as torch tensors (for inspection and parity checks)."""
        ptrs = [C.c_void_p() for _ in range(8)]
        _check(_lib.gcn_csr_arrays(self.handle, *[C.byref(p) for p in ptrs]), "gcn_csr_arrays")
        spec = [("rowptr", torch.int64, self.nr + 1), ("col", torch.int32, self.nnz), ("val", torch.float32, self.nnz),
                ("deg", torch.int32, self.nr), ("halo_gid", torch.int32, self.nh),
                ("colptr", torch.int64, self.nc + 1), ("rowidx", torch.int32, self.nnz), ("val_t", torch.float32, self.nnz)]
        out = {}
        torch.cuda.synchronize()
        for p, (name, dt, n) in zip(ptrs, spec):
            if not p.value:
                out[name] = None
                continue
            t = torch.empty(n, dtype=dt, device=self.device)
            if n:
                rc = _hip_memcpy(t.data_ptr(), p.value, n * t.element_size())
                if int(rc) != 0:
                    raise GcnError(f"copy of {name} failed: {rc}")
            out[name] = t
        return out

    def free(self):
        if self._h is not None:
            _lib.gcn_csr_free(self._h)
            self._h = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def gcn_csr_build(src: torch.Tensor, dst: torch.Tensor, n_global: int, row_lo: int = 0, row_hi: int | None = None,
                  deg_global: torch.Tensor | None = None, flags: int = BUILD_CSC) -> Csr:
    _dev(src, torch.int32, "src"); _dev(dst, torch.int32, "dst")
    if src.numel() != dst.numel() or not src.is_contiguous() or not dst.is_contiguous():
        raise TypeError("src/dst must be contiguous int32 vectors of equal length")
    if deg_global is not None:
        _dev(deg_global, torch.int32, "deg_global")
        if deg_global.numel() != n_global or not deg_global.is_contiguous():
            raise TypeError("deg_global must be a contiguous int32 vector of length n_global")
    row_hi = n_global if row_hi is None else row_hi
    out = C.c_void_p()
    with torch.cuda.device(src.device):
        rc = _lib.gcn_csr_build(_ptr(src), _ptr(dst), src.numel(), n_global, row_lo, row_hi, _ptr(deg_global), flags,
                                _stream(), C.byref(out))
    _check(rc, "gcn_csr_build")
    return Csr(out, src.device)


def gcn_csr_induced(A: Csr, vertices: torch.Tensor, flags: int = BUILD_CSC) -> Csr:
    _dev(vertices, torch.int32, "vertices")
    if vertices.dim() != 1 or not vertices.is_contiguous():
        raise TypeError("vertices must be a contiguous int32 vector")
    out = C.c_void_p()
    with torch.cuda.device(vertices.device):
        rc = _lib.gcn_csr_induced(A.handle, _ptr(vertices), vertices.numel(), flags, _stream(), C.byref(out))
    _check(rc, "gcn_csr_induced")
    return Csr(out, vertices.device)


def gcn_spmm(A: Csr, X: torch.Tensor, Y: torch.Tensor, epilogue: int = EPI_NONE, bias: torch.Tensor | None = None,
             Zprev: torch.Tensor | None = None):
    ldx, d = _rowmajor(_dev(X), "X"); ldy, dy = _rowmajor(_dev(Y), "Y")
    if X.shape[0] != A.nc or Y.shape[0] != A.nr or dy != d or Y.dtype != X.dtype:
        raise TypeError("gcn_spmm: X must be [nc, d] and Y [nr, d] of the same dtype")
    ldz = 0
    if Zprev is not None:
        ldz, dz = _rowmajor(_dev(Zprev, X.dtype, "Zprev"), "Zprev")
        if Zprev.shape[0] != A.nr or dz != d:
            raise TypeError("gcn_spmm: Zprev must be [nr, d]")
    if bias is not None and (_dev(bias, torch.float32, "bias").numel() != d or not bias.is_contiguous()):
        raise TypeError("gcn_spmm: bias must be a contiguous f32 vector of length d")
    _check(_lib.gcn_spmm(A.handle, _ptr(X), ldx, d, _dtype_code(X), _ptr(Y), ldy, epilogue, _ptr(bias), _ptr(Zprev),
                         ldz, _stream()), "gcn_spmm")
    return Y


def gcn_spmm_noalloc(A: Csr, X: torch.Tensor, Y: torch.Tensor, epilogue: int = EPI_NONE, bias: torch.Tensor | None = None,
                     Zprev: torch.Tensor | None = None):
    """gcn_spmm through the entry point that allocates nothing (its scratch is a fixed array of the library)."""
    ldx, d = _rowmajor(_dev(X), "X"); ldy, dy = _rowmajor(_dev(Y), "Y")
    if X.shape[0] != A.nc or Y.shape[0] != A.nr or dy != d or Y.dtype != X.dtype:
        raise TypeError("gcn_spmm_noalloc: X must be [nc, d] and Y [nr, d] of the same dtype")
    ldz = 0
    if Zprev is not None:
        ldz, dz = _rowmajor(_dev(Zprev, X.dtype, "Zprev"), "Zprev")
        if Zprev.shape[0] != A.nr or dz != d:
            raise TypeError("gcn_spmm_noalloc: Zprev must be [nr, d]")
    if bias is not None and (_dev(bias, torch.float32, "bias").numel() != d or not bias.is_contiguous()):
        raise TypeError("gcn_spmm_noalloc: bias must be a contiguous f32 vector of length d")
    _check(_lib.gcn_spmm_noalloc(A.handle, _ptr(X), ldx, d, _dtype_code(X), _ptr(Y), ldy, epilogue, _ptr(bias), _ptr(Zprev),
                                 ldz, _stream()), "gcn_spmm_noalloc")
    return Y


def gcn_spmm_part(A: Csr, part: int, X: torch.Tensor, Y: torch.Tensor, epilogue: int = EPI_NONE,
                  bias: torch.Tensor | None = None, Zprev: torch.Tensor | None = None):
    ldx, d = _rowmajor(_dev(X), "X"); ldy, dy = _rowmajor(_dev(Y), "Y")
    if X.shape[0] != A.nc or Y.shape[0] != A.nr or dy != d or Y.dtype != X.dtype:
        raise TypeError("gcn_spmm_part: X must be [nc, d] and Y [nr, d] of the same dtype")
    ldz = 0
    if Zprev is not None:
        ldz, dz = _rowmajor(_dev(Zprev, X.dtype, "Zprev"), "Zprev")
        if Zprev.shape[0] != A.nr or dz != d:
            raise TypeError("gcn_spmm_part: Zprev must be [nr, d]")
    if bias is not None and (_dev(bias, torch.float32, "bias").numel() != d or not bias.is_contiguous()):
        raise TypeError("gcn_spmm_part: bias must be a contiguous f32 vector of length d")
    _check(_lib.gcn_spmm_part(A.handle, int(part), _ptr(X), ldx, d, _dtype_code(X), _ptr(Y), ldy, epilogue, _ptr(bias),
                              _ptr(Zprev), ldz, _stream()), "gcn_spmm_part")
    return Y


def gcn_dense_fwd(X: torch.Tensor, W: torch.Tensor, Out: torch.Tensor, bias: torch.Tensor | None = None,
                  act: int = ACT_NONE, Z: torch.Tensor | None = None):
    ldx, d_in = _rowmajor(_dev(X), "X"); ldo, d_out = _rowmajor(_dev(Out, X.dtype, "Out"), "Out")
    if _dev(W, torch.float32, "W").shape != (d_in, d_out) or not W.is_contiguous():
        raise TypeError("gcn_dense_fwd: W must be a contiguous f32 [d_in, d_out]")
    if Out.shape[0] != X.shape[0]:
        raise TypeError("gcn_dense_fwd: Out must have the rows of X")
    if Z is not None and (_dev(Z, X.dtype, "Z").shape != (X.shape[0], d_out) or not Z.is_contiguous()):
        raise TypeError("gcn_dense_fwd: Z must be a contiguous [rows, d_out]")
    if bias is not None and (_dev(bias, torch.float32, "bias").numel() != d_out or not bias.is_contiguous()):
        raise TypeError("gcn_dense_fwd: bias must be a contiguous f32 vector of length d_out")
    _check(_lib.gcn_dense_fwd(_ptr(X), ldx, X.shape[0], _ptr(W), _ptr(bias), d_in, d_out, act, _dtype_code(X), _ptr(Z),
                              _ptr(Out), ldo, _stream()), "gcn_dense_fwd")
    return Out


def gcn_spmm_t(A: Csr, X: torch.Tensor, Y: torch.Tensor, epilogue: int = EPI_NONE, Zprev: torch.Tensor | None = None):
    ldx, d = _rowmajor(_dev(X), "X"); ldy, dy = _rowmajor(_dev(Y), "Y")
    if X.shape[0] != A.nr or Y.shape[0] != A.nc or dy != d or Y.dtype != X.dtype:
        raise TypeError("gcn_spmm_t: X must be [nr, d] and Y [nc, d] of the same dtype")
    ldz = 0
    if Zprev is not None:
        ldz, dz = _rowmajor(_dev(Zprev, X.dtype, "Zprev"), "Zprev")
        if Zprev.shape[0] != A.nr or dz != d:
            raise TypeError("gcn_spmm_t: Zprev must be [nr, d]")
    _check(_lib.gcn_spmm_t(A.handle, _ptr(X), ldx, d, _dtype_code(X), _ptr(Y), ldy, epilogue, _ptr(Zprev), ldz,
                           _stream()), "gcn_spmm_t")
    return Y


def gcn_halo_gather(table: torch.Tensor, idx: torch.Tensor, recv: torch.Tensor):
    """table may be a GPU tensor or a pinned host tensor."""
    if not (table.is_cuda or table.is_pinned()):
        raise TypeError("table must be a GPU tensor or pinned host memory")
    ld, d = _rowmajor(table, "table"); ldr, dr = _rowmajor(_dev(recv), "recv")
    _dev(idx, torch.int32, "idx")
    if dr != d or recv.shape[0] != idx.numel() or recv.dtype != table.dtype or not idx.is_contiguous():
        raise TypeError("gcn_halo_gather: recv must be [len(idx), d] of the table's dtype")
    _check(_lib.gcn_halo_gather(_ptr(table), ld, table.shape[0], d, _dtype_code(table), _ptr(idx), idx.numel(),
                                _ptr(recv), ldr, _stream()), "gcn_halo_gather")
    return recv


def _dense(t, rows, cols, dtype, what):
    _dev(t, dtype, what)
    if t.shape != (rows, cols) or not t.is_contiguous():
        raise TypeError(f"{what} must be a contiguous [{rows}, {cols}] tensor")
    return t


def gcn_layer_fwd(A: Csr, H: torch.Tensor, W: torch.Tensor, Hout: torch.Tensor, act: int = ACT_RELU,
                  bias: torch.Tensor | None = None, Z: torch.Tensor | None = None, AH_save: torch.Tensor | None = None):
    ldh, d_in = _rowmajor(_dev(H), "H")
    if H.shape[0] != A.nc:
        raise TypeError("gcn_layer_fwd: H must have nc rows")
    d_out = W.shape[1]
    _dense(W, d_in, d_out, torch.float32, "W")
    _dense(Hout, A.nr, d_out, H.dtype, "Hout")
    if Z is not None:
        _dense(Z, A.nr, d_out, H.dtype, "Z")
    if AH_save is not None:
        _dense(AH_save, A.nr, d_in, H.dtype, "AH_save")
    if bias is not None:
        _dense(bias.view(1, -1), 1, d_out, torch.float32, "bias")
    _check(_lib.gcn_layer_fwd(A.handle, _ptr(H), ldh, _ptr(W), _ptr(bias), d_in, d_out, act, _dtype_code(H), _ptr(Z),
                              _ptr(Hout), _ptr(AH_save), _stream()), "gcn_layer_fwd")
    return Hout


def gcn_layer_bwd(A: Csr, H: torch.Tensor, W: torch.Tensor, G: torch.Tensor, dW: torch.Tensor,
                  dH: torch.Tensor | None = None, Zprev: torch.Tensor | None = None,
                  AH_saved: torch.Tensor | None = None, dbias: torch.Tensor | None = None):
    ldh, d_in = _rowmajor(_dev(H), "H")
    if H.shape[0] != A.nc:
        raise TypeError("gcn_layer_bwd: H must have nc rows")
    d_out = W.shape[1]
    _dense(W, d_in, d_out, torch.float32, "W")
    _dense(G, A.nr, d_out, H.dtype, "G")
    _dense(dW, d_in, d_out, torch.float32, "dW")
    if dH is not None:
        _dense(dH, A.nc, d_in, H.dtype, "dH")
    if Zprev is not None:
        _dense(Zprev, A.nr, d_in, H.dtype, "Zprev")
    if AH_saved is not None:
        _dense(AH_saved, A.nr, d_in, H.dtype, "AH_saved")
    if dbias is not None:
        _dense(dbias.view(1, -1), 1, d_out, torch.float32, "dbias")
    _check(_lib.gcn_layer_bwd(A.handle, _ptr(H), ldh, _ptr(AH_saved), _ptr(W), d_in, d_out, _dtype_code(H), _ptr(G),
                              _ptr(Zprev), _ptr(dW), _ptr(dbias), _ptr(dH), _stream()), "gcn_layer_bwd")
    return dW


def _pitched(t, rows, cols, dtype, what):
    """(pointer, ld) of a [rows, cols] tensor with contiguous rows and any row pitch; (None, 0) for None."""
    if t is None:
        return None, 0
    ld, c = _rowmajor(_dev(t, dtype, what), what)
    if t.shape[0] != rows or c != cols:
        raise TypeError(f"{what} must be [{rows}, {cols}]")
    return _ptr(t), ld


def gcn_layer_fwd_ld(A: Csr, H: torch.Tensor, W: torch.Tensor, Hout: torch.Tensor, act: int = ACT_RELU,
                     bias: torch.Tensor | None = None, Z: torch.Tensor | None = None, AH_save: torch.Tensor | None = None):
    """gcn_layer_fwd for feature tensors of any row pitch (e.g. feature_buffer views)."""
    ldh, d_in = _rowmajor(_dev(H), "H")
    if H.shape[0] != A.nc:
        raise TypeError("gcn_layer_fwd_ld: H must have nc rows")
    d_out = W.shape[1]
    _dense(W, d_in, d_out, torch.float32, "W")
    po, ldo = _pitched(Hout, A.nr, d_out, H.dtype, "Hout")
    pz, ldz = _pitched(Z, A.nr, d_out, H.dtype, "Z")
    pa, ldah = _pitched(AH_save, A.nr, d_in, H.dtype, "AH_save")
    if bias is not None:
        _dense(bias.view(1, -1), 1, d_out, torch.float32, "bias")
    _check(_lib.gcn_layer_fwd_ld(A.handle, _ptr(H), ldh, _ptr(W), _ptr(bias), d_in, d_out, act, _dtype_code(H), pz, ldz,
                                 po, ldo, pa, ldah, _stream()), "gcn_layer_fwd_ld")
    return Hout


def gcn_layer_bwd_ld(A: Csr, H: torch.Tensor, W: torch.Tensor, G: torch.Tensor, dW: torch.Tensor,
                     dH: torch.Tensor | None = None, Zprev: torch.Tensor | None = None,
                     AH_saved: torch.Tensor | None = None, dbias: torch.Tensor | None = None):
    """gcn_layer_bwd for feature tensors of any row pitch."""
    ldh, d_in = _rowmajor(_dev(H), "H")
    if H.shape[0] != A.nc:
        raise TypeError("gcn_layer_bwd_ld: H must have nc rows")
    d_out = W.shape[1]
    _dense(W, d_in, d_out, torch.float32, "W")
    _dense(dW, d_in, d_out, torch.float32, "dW")
    pg, ldg = _pitched(G, A.nr, d_out, H.dtype, "G")
    pd, lddh = _pitched(dH, A.nc, d_in, H.dtype, "dH")
    pz, ldzp = _pitched(Zprev, A.nr, d_in, H.dtype, "Zprev")
    pa, ldah = _pitched(AH_saved, A.nr, d_in, H.dtype, "AH_saved")
    if dbias is not None:
        _dense(dbias.view(1, -1), 1, d_out, torch.float32, "dbias")
    _check(_lib.gcn_layer_bwd_ld(A.handle, _ptr(H), ldh, pa, ldah, _ptr(W), d_in, d_out, _dtype_code(H), pg, ldg,
                                 pz, ldzp, _ptr(dW), _ptr(dbias), pd, lddh, _stream()), "gcn_layer_bwd_ld")
    return dW


def gcn_layer_bwd_pull(A: Csr, H: torch.Tensor, W: torch.Tensor, G: torch.Tensor, T: torch.Tensor, dW: torch.Tensor,
                       dH: torch.Tensor | None = None, Zprev: torch.Tensor | None = None,
                       dbias: torch.Tensor | None = None, phase: int = 0):
    """H needs only its nr owned rows ([>= nr, d_in]); G is [nc, d_out]; T [nr, d_out]; dH [nr, d_in]."""
    ldh, d_in = _rowmajor(_dev(H), "H")
    ldg, d_out = _rowmajor(_dev(G, H.dtype, "G"), "G")
    if H.shape[0] < A.nr or G.shape[0] != A.nc:
        raise TypeError("gcn_layer_bwd_pull: H must hold the nr owned rows and G all nc rows")
    _dense(W, d_in, d_out, torch.float32, "W"); _dense(dW, d_in, d_out, torch.float32, "dW")
    _dense(T, A.nr, d_out, H.dtype, "T")
    if dH is not None:
        _dense(dH, A.nr, d_in, H.dtype, "dH")
    if Zprev is not None:
        _dense(Zprev, A.nr, d_in, H.dtype, "Zprev")
    if dbias is not None:
        _dense(dbias.view(1, -1), 1, d_out, torch.float32, "dbias")
    _check(_lib.gcn_layer_bwd_pull(A.handle, int(phase), _ptr(H), ldh, _ptr(W), d_in, d_out, _dtype_code(H), _ptr(G), ldg,
                                   _ptr(Zprev), _ptr(T), _ptr(dW), _ptr(dbias), _ptr(dH), _stream()), "gcn_layer_bwd_pull")
    return dW


def gcn_softmax_xent(Z: torch.Tensor, y: torch.Tensor, scale: float, loss: torch.Tensor, G: torch.Tensor):
    ldz, Cn = _rowmajor(_dev(Z), "Z"); ldg, cg = _rowmajor(_dev(G, Z.dtype, "G"), "G")
    _dev(y, torch.int32, "y"); _dev(loss, torch.float32, "loss")
    if cg != Cn or G.shape[0] != Z.shape[0] or y.numel() != Z.shape[0] or not y.is_contiguous() or loss.numel() != 1:
        raise TypeError("gcn_softmax_xent: shape mismatch")
    _check(_lib.gcn_softmax_xent(_ptr(Z), ldz, Z.shape[0], Cn, _dtype_code(Z), _ptr(y), float(scale), _ptr(loss),
                                 _ptr(G), ldg, _stream()), "gcn_softmax_xent")
    return loss


def gcn_partition_stats(A: Csr, part: torch.Tensor, p: int):
    """Returns a dict of int64 GPU tensors: load, send_rows, recv_rows, send_msgs, recv_msgs ([p] each), totals ([2])."""
    _dev(part, torch.int32, "part")
    if part.dim() != 1 or part.numel() != A.nr or not part.is_contiguous():
        raise TypeError("gcn_partition_stats: part must be a contiguous int32 vector with one entry per vertex")
    out = {k: torch.empty(2 if k == "totals" else max(int(p), 0), dtype=torch.int64, device=part.device)
           for k in ("load", "send_rows", "recv_rows", "send_msgs", "recv_msgs", "totals")}
    _check(_lib.gcn_partition_stats(A.handle, _ptr(part), int(p), _ptr(out["load"]), _ptr(out["send_rows"]),
                                    _ptr(out["recv_rows"]), _ptr(out["send_msgs"]), _ptr(out["recv_msgs"]),
                                    _ptr(out["totals"]), _stream()), "gcn_partition_stats")
    return out


def gcn_sgd_update(W: torch.Tensor, dW: torch.Tensor, lr: float):
    _dev(W, torch.float32, "W"); _dev(dW, torch.float32, "dW")
    if W.shape != dW.shape or not W.is_contiguous() or not dW.is_contiguous():
        raise TypeError("gcn_sgd_update: W and dW must be contiguous and of one shape")
    _check(_lib.gcn_sgd_update(_ptr(W), _ptr(dW), W.numel(), float(lr), _stream()), "gcn_sgd_update")
    return W


def gcn_debug_max_grid_x(blocks: int):
    """Test hook: most blocks in the x dimension of a launch (0 restores the default of 2^22)."""
    _check(_lib.gcn_debug_max_grid_x(int(blocks)), "gcn_debug_max_grid_x")


def gcn_feature_ld(d: int, dtype: torch.dtype = torch.float32) -> int:
    """Row pitch (elements) the sparse products gather best from for rows of d elements."""
    ld = int(_lib.gcn_feature_ld(int(d), BF16 if dtype == torch.bfloat16 else F32))
    if ld < 0:
        raise GcnError("gcn_feature_ld: bad argument")
    return ld


def feature_buffer(rows: int, d: int, dtype: torch.dtype = torch.float32, device=None) -> torch.Tensor:
    """An uninitialised [rows, d] view of a buffer whose row pitch is gcn_feature_ld(d, dtype) (allocation only)."""
    return torch.empty(rows, gcn_feature_ld(d, dtype), dtype=dtype, device=device)[:, :d]


TUNE_DEFAULT = -2147483648


def gcn_debug_set_tuning(name: str, value: int | None):
    """Test and experiment hook: override one kernel-selection rule (value None restores the default)."""
    _check(_lib.gcn_debug_set_tuning(name.encode(), TUNE_DEFAULT if value is None else int(value)), "gcn_debug_set_tuning")


def gcn_profile_enable(on: bool):
    _check(_lib.gcn_profile_enable(1 if on else 0), "gcn_profile_enable")


def gcn_profile_filter(kinds=None, d: int = -1):
    """Record only launches of the named kinds (None: all) and, if d >= 0, of that feature width."""
    mask = -1 if kinds is None else sum(1 << KIND_NAMES.index(k) for k in kinds)
    _check(_lib.gcn_profile_filter(mask, int(d)), "gcn_profile_filter")


def gcn_profile_records():
    """All records held by the library, as dicts (synchronises with each record's stop event)."""
    dropped = C.c_int64()
    n = _lib.gcn_profile_count(C.byref(dropped))
    out = []
    rec = ProfileRec()
    for i in range(n):
        _check(_lib.gcn_profile_get(i, C.byref(rec)), "gcn_profile_get")
        out.append({"kind": KIND_NAMES[rec.kind], "d": rec.d, "dtype": rec.dtype, "rows": rec.rows, "inner": rec.inner,
                    "alg_bytes": rec.alg_bytes, "touched_bytes": rec.touched_bytes, "flops": rec.flops, "ms": rec.ms})
    return out, dropped.value
