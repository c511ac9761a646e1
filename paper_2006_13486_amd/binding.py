"""Thin ctypes binding over the C-ABI library (include/rbgp.h): argument
marshalling only, same names as the C entry points.  Every step of the path
runs inside librbgp.so; there is no Python or CPU fallback.  torch is used by
callers for device memory and streams, this module only passes raw pointers."""
from __future__ import annotations

import ctypes
import os

import numpy as np

F32, BF16_F32ACC, BF16 = 0, 1, 2   # BF16: as BF16_F32ACC with O stored as bf16 bits
KERNEL_AUTO, KERNEL_GENERIC, KERNEL_MFMA, KERNEL_MFMA_REG, KERNEL_MFMA_TILE, KERNEL_MFMA_REG_FILLED = 0, 1, 2, 3, 4, 5
TUNE_COLS_PER_LANE, TUNE_COLS_PER_WORKGROUP, TUNE_GROUPS_PER_WORKGROUP, TUNE_ROW_PAIRING = 0, 1, 2, 3
TUNE_ROW_GROUPS, TUNE_K_SPLIT, TUNE_COLUMN_TILES, TUNE_REGISTER_SETS = 4, 5, 6, 7
SPEC_OK, SPEC_COMPLETE, SPEC_DEGENERATE, SPEC_PRODUCT = 0, 1, 2, 3
OK, EINVAL, ENOMEM, ENOTRAMANUJAN, ESHAPE, EHIP, EUNSUPPORTED, EINTERNAL, ETOOLARGE = 0, -1, -2, -3, -4, -5, -6, -7, -8

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "librbgp.so")
_lib = None

_i32p = ctypes.POINTER(ctypes.c_int32)
_i64p = ctypes.POINTER(ctypes.c_int64)
_f64p = ctypes.POINTER(ctypes.c_double)
_intp = ctypes.POINTER(ctypes.c_int)
_vp = ctypes.c_void_p

SIGNATURES = {
    "rbgp_make_mask": (ctypes.c_int, [_i32p, _i32p, _i32p, ctypes.c_uint64, ctypes.c_int32, ctypes.POINTER(_vp)]),
    "rbgp_make_mask_k": (ctypes.c_int, [ctypes.c_int32, _i32p, _i32p, _i32p, _i32p, ctypes.c_uint64, ctypes.c_int32,
                                        ctypes.POINTER(_vp)]),
    "rbgp_mask_num_base": (ctypes.c_int, [_vp]),
    "rbgp_mask_base": (ctypes.c_int, [_vp, ctypes.c_int, _i32p, _i32p, _i32p, _i32p, ctypes.POINTER(_i32p),
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                      ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int),
                                      ctypes.POINTER(ctypes.c_int)]),
    "rbgp_mask_free": (None, [_vp]),
    "rbgp_mask_shape": (ctypes.c_int, [_vp, _i64p, _i64p, _i64p, _i64p, _i64p]),
    "rbgp_mask_factor": (ctypes.c_int, [_vp, ctypes.c_int, _i32p, _i32p, _i32p, ctypes.POINTER(_i32p)]),
    "rbgp_mask_spectrum": (ctypes.c_int, [_vp, ctypes.c_int, _f64p, _f64p, _f64p, _intp, _intp]),
    "rbgp_mask_columns": (ctypes.c_int, [_vp, _vp]),
    "rbgp_mask_dense": (ctypes.c_int, [_vp, _vp]),
    "rbgp_mask_set_kernel": (ctypes.c_int, [_vp, ctypes.c_int]),
    "rbgp_mask_kernel": (ctypes.c_int, [_vp, ctypes.c_int]),
    "rbgp_mask_tune": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int]),
    "rbgp_packed_bytes": (ctypes.c_size_t, [_vp, ctypes.c_int]),
    "rbgp_pack_layout": (ctypes.c_int, [_vp, ctypes.c_int, _vp]),
    "rbgp_pack": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, _vp]),
    "rbgp_pack_device": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, _vp]),
    "rbgp_mask_transpose": (ctypes.c_int, [_vp, ctypes.POINTER(_vp)]),
    "rbgp_mask_conv3x3_transpose": (ctypes.c_int, [_vp, ctypes.POINTER(_vp)]),
    "rbgp_mask_original_order": (ctypes.c_int, [_vp, _vp]),
    "rbgp_transpose_order": (ctypes.c_int, [_vp, _vp]),
    "rbgp_pack_transposed": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, _vp]),
    "rbgp_pack_transposed_device": (ctypes.c_int, [_vp, ctypes.c_int, _vp, _vp, _vp]),
    "rbgp_sddmm": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                  _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp, _vp]),
    "rbgp_sddmm_static": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                         _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp, _vp]),
    "rbgp_spmm": (ctypes.c_int, [_vp, ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                 _vp, _vp, ctypes.c_int64, _vp, ctypes.c_int64, _vp]),
    "rbgp_conv3x3": (ctypes.c_int, [_vp, ctypes.c_int] + [ctypes.c_int64] * 5 + [_vp, _vp, _vp, ctypes.c_int64, _vp]),
    "rbgp_conv3x3_sddmm": (ctypes.c_int, [_vp, ctypes.c_int] + [ctypes.c_int64] * 5 + [_vp, ctypes.c_int64, _vp, _vp, _vp]),
    "rbgp_mask_reg_plan": (ctypes.c_int, [_vp, ctypes.POINTER(ctypes.c_int32)]),
    "rbgp_mask_check_tables": (ctypes.c_int, [_vp]),
    "rbgp_strerror": (ctypes.c_char_p, [ctypes.c_int]),
    "rbgp_last_hip_error": (ctypes.c_char_p, []),
}


class RbgpError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        lib = load()
        msg = lib.rbgp_strerror(code).decode()
        if code == EHIP:
            msg += ": " + lib.rbgp_last_hip_error().decode()
        super().__init__(f"{where}: {msg} ({code})")


def load():
    """Load librbgp.so (built by paper_2006_13486_amd.build); fails loudly if absent."""
    global _lib
    if _lib is None:
        # RBGP_LIB names another build of the same library (the host-only sanitizer build of the CPU tests)
        path = os.environ.get("RBGP_LIB") or _LIB_PATH
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'`")
        # torch bundles its own HIP runtime (SONAME libamdhip64.so.7).  Import it first so
        # that librbgp.so binds to that copy: two HIP runtimes in one process do not share
        # the device and the second one reports "no ROCm-capable device".
        # (RBGP_NO_TORCH: the host-only sanitizer run loads the library without torch in the process)
        if not os.environ.get("RBGP_NO_TORCH"):
            import torch  # noqa: F401
        lib = ctypes.CDLL(path)
        for name, (res, args) in SIGNATURES.items():
            fn = getattr(lib, name)
            fn.restype = res
            fn.argtypes = args
        _lib = lib
    return _lib


def _check(code: int, where: str):
    if code != OK:
        raise RbgpError(code, where)


def _i32x4(v):
    arr = (ctypes.c_int32 * 4)(*[int(x) for x in v])
    return arr


class Mask:
    """Owner of one rbgp_mask_t*."""

    def __init__(self, handle):
        self.handle = handle

    def __del__(self):
        h, self.handle = getattr(self, "handle", None), None
        if h and _lib is not None:
            _lib.rbgp_mask_free(h)


def rbgp_make_mask(rows, cols, row_deg, seed: int, max_tries: int = 0) -> Mask:
    out = _vp()
    _check(load().rbgp_make_mask(_i32x4(rows), _i32x4(cols), _i32x4(row_deg), int(seed), int(max_tries),
                                 ctypes.byref(out)), "rbgp_make_mask")
    return Mask(out)


def rbgp_make_mask_k(rows, cols, row_deg, roles, seed: int, max_tries: int = 0) -> Mask:
    n = len(rows)
    arr = lambda v: (ctypes.c_int32 * n)(*[int(x) for x in v])
    out = _vp()
    _check(load().rbgp_make_mask_k(n, arr(rows), arr(cols), arr(row_deg), arr(roles), int(seed), int(max_tries),
                                   ctypes.byref(out)), "rbgp_make_mask_k")
    return Mask(out)


def rbgp_mask_num_base(mask: Mask) -> int:
    return int(load().rbgp_mask_num_base(mask.handle))


def rbgp_mask_base(mask: Mask, i: int) -> dict:
    r, c, d, role = (ctypes.c_int32() for _ in range(4))
    adj = _i32p()
    s1, s2, b = (ctypes.c_double() for _ in range(3))
    st, tr = ctypes.c_int(), ctypes.c_int()
    _check(load().rbgp_mask_base(mask.handle, i, *[ctypes.byref(x) for x in (r, c, d, role, adj, s1, s2, b, st, tr)]),
           "rbgp_mask_base")
    a = np.ctypeslib.as_array(adj, shape=(r.value, d.value)).copy()
    return dict(rows=r.value, cols=c.value, deg=d.value, role=role.value, adj=a, sigma1=s1.value, sigma2=s2.value,
                bound=b.value, status=st.value, tries=tr.value)


def rbgp_mask_free(mask: Mask):
    h, mask.handle = mask.handle, None
    if h:
        load().rbgp_mask_free(h)


def rbgp_mask_shape(mask: Mask) -> dict:
    v = [ctypes.c_int64() for _ in range(5)]
    _check(load().rbgp_mask_shape(mask.handle, *[ctypes.byref(x) for x in v]), "rbgp_mask_shape")
    return dict(zip(("M", "K", "rowdeg", "coldeg", "nnz"), (int(x.value) for x in v)))


def rbgp_mask_factor(mask: Mask, i: int):
    r, c, d = ctypes.c_int32(), ctypes.c_int32(), ctypes.c_int32()
    adj = _i32p()
    _check(load().rbgp_mask_factor(mask.handle, i, ctypes.byref(r), ctypes.byref(c), ctypes.byref(d),
                                   ctypes.byref(adj)), "rbgp_mask_factor")
    a = np.ctypeslib.as_array(adj, shape=(r.value, d.value)).copy()
    return int(r.value), int(c.value), int(d.value), a


def rbgp_mask_reg_plan(mask: Mask) -> list:
    info = (ctypes.c_int32 * 16)()
    _check(load().rbgp_mask_reg_plan(mask.handle, info), "rbgp_mask_reg_plan")
    return [int(v) for v in info]


def rbgp_mask_check_tables(mask: Mask) -> None:
    _check(load().rbgp_mask_check_tables(mask.handle), "rbgp_mask_check_tables")


def rbgp_mask_spectrum(mask: Mask, i: int) -> dict:
    s1, s2, b = ctypes.c_double(), ctypes.c_double(), ctypes.c_double()
    st, tr = ctypes.c_int(), ctypes.c_int()
    _check(load().rbgp_mask_spectrum(mask.handle, i, ctypes.byref(s1), ctypes.byref(s2), ctypes.byref(b),
                                     ctypes.byref(st), ctypes.byref(tr)), "rbgp_mask_spectrum")
    return dict(sigma1=s1.value, sigma2=s2.value, bound=b.value, status=st.value, tries=tr.value)


def rbgp_mask_columns(mask: Mask) -> np.ndarray:
    sh = rbgp_mask_shape(mask)
    out = np.empty((sh["M"], sh["rowdeg"]), dtype=np.int32)
    _check(load().rbgp_mask_columns(mask.handle, out.ctypes.data), "rbgp_mask_columns")
    return out


def rbgp_mask_dense(mask: Mask) -> np.ndarray:
    sh = rbgp_mask_shape(mask)
    out = np.empty((sh["M"], sh["K"]), dtype=np.uint8)
    _check(load().rbgp_mask_dense(mask.handle, out.ctypes.data), "rbgp_mask_dense")
    return out


def rbgp_mask_set_kernel(mask: Mask, kernel: int):
    _check(load().rbgp_mask_set_kernel(mask.handle, kernel), "rbgp_mask_set_kernel")


def rbgp_mask_kernel(mask: Mask, dtype: int) -> int:
    return int(load().rbgp_mask_kernel(mask.handle, dtype))


def rbgp_mask_tune(mask: Mask, knob: int, value: int):
    _check(load().rbgp_mask_tune(mask.handle, knob, value), "rbgp_mask_tune")


def rbgp_packed_bytes(mask: Mask, dtype: int) -> int:
    return int(load().rbgp_packed_bytes(mask.handle, dtype))


def rbgp_pack_layout(mask: Mask, dtype: int) -> np.ndarray:
    """int32 array, one entry per element of the packed buffer: canonical index or -1 (padding)."""
    n = rbgp_packed_bytes(mask, dtype) // (4 if dtype == F32 else 2)
    out = np.empty(n, dtype=np.int32)
    _check(load().rbgp_pack_layout(mask.handle, dtype, out.ctypes.data_as(_vp)), "rbgp_pack_layout")
    return out


def rbgp_pack(mask: Mask, dtype: int, host_values: np.ndarray, dev_packed_ptr: int, stream: int = 0):
    """host_values: contiguous numpy array, float32 (F32) or uint16 bf16 bits (BF16_F32ACC)."""
    want = np.float32 if dtype == F32 else np.uint16
    if host_values.dtype != want or not host_values.flags["C_CONTIGUOUS"]:
        raise TypeError(f"host_values must be C-contiguous {want}")
    if host_values.size != rbgp_mask_shape(mask)["nnz"]:
        raise ValueError("host_values must hold M*rowdeg elements")
    _check(load().rbgp_pack(mask.handle, dtype, host_values.ctypes.data, dev_packed_ptr, stream), "rbgp_pack")


def rbgp_pack_device(mask: Mask, dtype: int, dev_values_ptr: int, dev_packed_ptr: int, stream: int = 0):
    _check(load().rbgp_pack_device(mask.handle, dtype, dev_values_ptr, dev_packed_ptr, stream), "rbgp_pack_device")


def rbgp_mask_transpose(mask: Mask) -> Mask:
    out = _vp()
    _check(load().rbgp_mask_transpose(mask.handle, ctypes.byref(out)), "rbgp_mask_transpose")
    return Mask(out)


def rbgp_mask_conv3x3_transpose(mask: Mask) -> Mask:
    out = _vp()
    _check(load().rbgp_mask_conv3x3_transpose(mask.handle, ctypes.byref(out)), "rbgp_mask_conv3x3_transpose")
    return Mask(out)


def rbgp_mask_original_order(derived: Mask) -> np.ndarray:
    out = np.empty(rbgp_mask_shape(derived)["nnz"], dtype=np.int32)
    _check(load().rbgp_mask_original_order(derived.handle, out.ctypes.data), "rbgp_mask_original_order")
    return out


def rbgp_transpose_order(mask: Mask) -> np.ndarray:
    out = np.empty(rbgp_mask_shape(mask)["nnz"], dtype=np.int32)
    _check(load().rbgp_transpose_order(mask.handle, out.ctypes.data), "rbgp_transpose_order")
    return out


def rbgp_pack_transposed(mask_t: Mask, dtype: int, host_values: np.ndarray, dev_packed_ptr: int, stream: int = 0):
    """host_values: the kept values in the ORIGINAL mask's canonical order."""
    want = np.float32 if dtype == F32 else np.uint16
    if host_values.dtype != want or not host_values.flags["C_CONTIGUOUS"]:
        raise TypeError(f"host_values must be C-contiguous {want}")
    if host_values.size != rbgp_mask_shape(mask_t)["nnz"]:
        raise ValueError("host_values must hold nnz elements")
    _check(load().rbgp_pack_transposed(mask_t.handle, dtype, host_values.ctypes.data, dev_packed_ptr, stream),
           "rbgp_pack_transposed")


def rbgp_pack_transposed_device(mask_t: Mask, dtype: int, dev_values_ptr: int, dev_packed_ptr: int, stream: int = 0):
    _check(load().rbgp_pack_transposed_device(mask_t.handle, dtype, dev_values_ptr, dev_packed_ptr, stream),
           "rbgp_pack_transposed_device")


def rbgp_sddmm(mask: Mask, dtype: int, M: int, K: int, N: int, dev_dO_ptr: int, ld_dO: int, dev_I_ptr: int, ldI: int,
               dev_dW_ptr: int, stream: int = 0):
    _check(load().rbgp_sddmm(mask.handle, dtype, M, K, N, dev_dO_ptr, ld_dO, dev_I_ptr, ldI, dev_dW_ptr, stream),
           "rbgp_sddmm")


def rbgp_sddmm_static(mask: Mask, dtype: int, M: int, K: int, N: int, dev_dO_ptr: int, ld_dO: int, dev_I_ptr: int,
                      ldI: int, dev_dW_ptr: int, stream: int = 0):
    _check(load().rbgp_sddmm_static(mask.handle, dtype, M, K, N, dev_dO_ptr, ld_dO, dev_I_ptr, ldI, dev_dW_ptr, stream),
           "rbgp_sddmm_static")


def rbgp_conv3x3(mask: Mask, dtype: int, channels_out: int, channels_in: int, images: int, height: int, width: int,
                 dev_packed_ptr: int, dev_X_ptr: int, dev_O_ptr: int, ldO: int, stream: int = 0):
    _check(load().rbgp_conv3x3(mask.handle, dtype, channels_out, channels_in, images, height, width,
                               dev_packed_ptr, dev_X_ptr, dev_O_ptr, ldO, stream), "rbgp_conv3x3")


def rbgp_conv3x3_sddmm(mask: Mask, dtype: int, channels_out: int, channels_in: int, images: int, height: int, width: int,
                       dev_dO_ptr: int, ld_dO: int, dev_X_ptr: int, dev_dW_ptr: int, stream: int = 0):
    _check(load().rbgp_conv3x3_sddmm(mask.handle, dtype, channels_out, channels_in, images, height, width,
                                     dev_dO_ptr, ld_dO, dev_X_ptr, dev_dW_ptr, stream), "rbgp_conv3x3_sddmm")


def rbgp_spmm(mask: Mask, dtype: int, M: int, K: int, N: int, dev_packed_ptr: int, dev_I_ptr: int, ldI: int,
              dev_O_ptr: int, ldO: int, stream: int = 0):
    _check(load().rbgp_spmm(mask.handle, dtype, M, K, N, dev_packed_ptr, dev_I_ptr, ldI, dev_O_ptr, ldO, stream),
           "rbgp_spmm")
