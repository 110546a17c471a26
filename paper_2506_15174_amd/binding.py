"""ctypes binding of the C ABI in include/spmm.h.

Argument marshalling only: every step of the product runs inside the shared
library (host inspector in C++, executor in HIP for gfx950).  There is no
Python or CPU fallback: if the library is missing, loading fails.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "lib", "libspmm_cdna4.so")

SPMM_OK = 0
SPMM_ERR_INVALID_ARG = 1
SPMM_ERR_INVALID_CSR = 2
SPMM_ERR_ALLOC = 3
SPMM_ERR_HIP = 4
SPMM_ERR_UNSUPPORTED = 5

ARRAY_HDR, ARRAY_STREAM, ARRAY_WINS, ARRAY_ITEMS, ARRAY_ROWMAP, ARRAY_CROSS = 0, 1, 2, 3, 4, 5

EXPORTS = ("spmm_plan_create", "spmm_plan_create_ex", "spmm_execute", "spmm_execute_static",
           "spmm_plan_destroy", "spmm_plan_describe", "spmm_plan_get_groups",
           "spmm_plan_get_array", "spmm_status_string")


class PlanInfo(ctypes.Structure):
    _fields_ = [("M", ctypes.c_int64), ("K", ctypes.c_int64), ("nnz", ctypes.c_int64),
                ("ufi", ctypes.c_int32), ("ufk", ctypes.c_int32),
                ("group_nnz", ctypes.c_int32), ("group_panels", ctypes.c_int32),
                ("n_groups", ctypes.c_int64), ("n_blocks", ctypes.c_int64),
                ("n_split", ctypes.c_int64),
                ("n_enum", ctypes.c_int64), ("n_chunks", ctypes.c_int64),
                ("stream_words", ctypes.c_int64), ("device_bytes", ctypes.c_int64),
                ("sorted_rows", ctypes.c_int64), ("n_cross", ctypes.c_int64),
                ("scratch_bytes", ctypes.c_int64), ("k_slices", ctypes.c_int64),
                ("slice_rows", ctypes.c_int64), ("slice_cols", ctypes.c_int64)]

    def as_dict(self):
        return {name: int(getattr(self, name)) for name, _ in self._fields_}


class Options(ctypes.Structure):
    _fields_ = [("group_nnz", ctypes.c_int32), ("group_panels", ctypes.c_int32),
                ("host_only", ctypes.c_int32), ("ufi", ctypes.c_int32),
                ("n_hint", ctypes.c_int32), ("sort_rows", ctypes.c_int32),
                ("force_wide", ctypes.c_int32), ("threads", ctypes.c_int32), ("depth", ctypes.c_int32),
                ("cross", ctypes.c_int32), ("ufk", ctypes.c_int32), ("probe", ctypes.c_int32),
                ("kslices", ctypes.c_int32)]


class SpmmError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, status_string(status), status))


_lib = None


def load():
    """Load the shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            "HIP library %s is missing: run `python -m paper_2506_15174_amd.build` "
            "(there is no fallback path)" % LIB_PATH)
    # PyTorch ships its own copy of the HIP runtime (same soname as the system
    # one).  The tensors and streams handed to spmm_execute belong to that copy,
    # so it must be the one already resident when this library is mapped.
    import torch  # noqa: F401
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.spmm_plan_create.restype = ctypes.c_int
    lib.spmm_plan_create.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp]
    lib.spmm_plan_create_ex.restype = ctypes.c_int
    lib.spmm_plan_create_ex.argtypes = [ctypes.POINTER(vp), i64, i64, vp, vp, vp,
                                        ctypes.POINTER(Options)]
    lib.spmm_execute.restype = ctypes.c_int
    lib.spmm_execute.argtypes = [vp, vp, i32, vp, vp]
    lib.spmm_execute_static.restype = ctypes.c_int
    lib.spmm_execute_static.argtypes = [vp, vp, i32, vp, vp]
    lib.spmm_plan_destroy.restype = ctypes.c_int
    lib.spmm_plan_destroy.argtypes = [vp]
    lib.spmm_plan_describe.restype = ctypes.c_int
    lib.spmm_plan_describe.argtypes = [vp, ctypes.POINTER(PlanInfo)]
    lib.spmm_plan_get_groups.restype = ctypes.c_int
    lib.spmm_plan_get_groups.argtypes = [vp, vp, i64]
    lib.spmm_plan_get_array.restype = ctypes.c_int
    lib.spmm_plan_get_array.argtypes = [vp, i32, vp, i64, ctypes.POINTER(i64)]
    lib.spmm_status_string.restype = ctypes.c_char_p
    lib.spmm_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def status_string(status):
    return load().spmm_status_string(int(status)).decode()


def _check(status, where):
    if status != SPMM_OK:
        raise SpmmError(status, where)


def _ptr(arr):
    return None if arr is None or arr.size == 0 else arr.ctypes.data


class Plan:
    """Owner of one spmm_plan_t*.  Same calls as the C ABI, numpy/torch marshalled."""

    def __init__(self, handle):
        self._h = handle
        self._info = None

    @property
    def handle(self):
        return self._h

    def describe(self):
        if self._info is None:  # a plan is immutable: ask once
            info = PlanInfo()
            _check(load().spmm_plan_describe(self._h, ctypes.byref(info)), "spmm_plan_describe")
            self._info = info.as_dict()
        return dict(self._info)

    def get_groups(self):
        n = self.describe()["n_groups"]
        out = np.zeros((n, 5), dtype=np.int32)
        _check(load().spmm_plan_get_groups(self._h, out.ctypes.data, n), "spmm_plan_get_groups")
        return out

    def get_array(self, which):
        """spmm_plan_get_array: one of the plan's arrays (ARRAY_*) as uint32; host-only plans only."""
        n = ctypes.c_int64(0)
        _check(load().spmm_plan_get_array(self._h, which, None, 0, ctypes.byref(n)),
               "spmm_plan_get_array")
        out = np.zeros(n.value, dtype=np.uint32)
        _check(load().spmm_plan_get_array(self._h, which, out.ctypes.data, n.value, None),
               "spmm_plan_get_array")
        return out

    def execute_raw(self, B_ptr, N, C_ptr, stream_ptr=None):
        """spmm_execute with raw device addresses (ints)."""
        st = _lib.spmm_execute(self._h, B_ptr, N, C_ptr, stream_ptr)
        if st != SPMM_OK:
            raise SpmmError(st, "spmm_execute")

    def execute_static_raw(self, B_ptr, N, C_ptr, stream_ptr=None):
        """spmm_execute_static with raw device addresses (ints)."""
        st = _lib.spmm_execute_static(self._h, B_ptr, N, C_ptr, stream_ptr)
        if st != SPMM_OK:
            raise SpmmError(st, "spmm_execute_static")

    def execute(self, B, C=None, stream=None):
        """spmm_execute on torch tensors (device memory and stream plumbing only).

        B: float32 CUDA/HIP tensor (K x N, contiguous).  C: optional output
        tensor (M x N); allocated when omitted.  Runs on `stream` or on torch's
        current stream.  Returns C.
        """
        import torch
        if not (B.is_cuda and B.dtype == torch.float32 and B.is_contiguous() and B.dim() == 2):
            raise ValueError("B must be a contiguous 2-D float32 device tensor")
        info = self._info or self.describe()
        if B.shape[0] != info["K"]:
            raise ValueError("B has %d rows, A has %d columns" % (B.shape[0], info["K"]))
        N = B.shape[1]
        if C is None:
            C = torch.empty((info["M"], N), dtype=torch.float32, device=B.device)
        if not (C.is_cuda and C.dtype == torch.float32 and C.is_contiguous()
                and tuple(C.shape) == (info["M"], N)):
            raise ValueError("C must be a contiguous float32 device tensor of shape (M, N)")
        s = stream if stream is not None else torch.cuda.current_stream(B.device)
        self.execute_raw(B.data_ptr() or None, N, C.data_ptr() or None, s.cuda_stream or None)
        return C

    def destroy(self):
        if self._h is not None:
            _check(load().spmm_plan_destroy(self._h), "spmm_plan_destroy")
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def plan_create(M, K, row_ptr, col_idx, vals, group_nnz=0, group_panels=0, host_only=False, ufi=0,
                n_hint=0, sort_rows=0, force_wide=False, threads=0, depth=0, cross=0, ufk=0, probe=False,
                kslices=0):
    """spmm_plan_create / spmm_plan_create_ex on numpy host arrays."""
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    vals = np.ascontiguousarray(vals, dtype=np.float32)
    handle = ctypes.c_void_p()
    lib = load()
    if group_nnz or group_panels or host_only or ufi or n_hint or sort_rows or force_wide or threads or depth \
            or cross or ufk or probe or kslices:
        opts = Options(int(group_nnz), int(group_panels), 1 if host_only else 0, int(ufi), int(n_hint),
                       int(sort_rows), 1 if force_wide else 0, int(threads), int(depth), int(cross), int(ufk), 1 if probe else 0,
                       int(kslices))
        st = lib.spmm_plan_create_ex(ctypes.byref(handle), int(M), int(K), _ptr(row_ptr),
                                     _ptr(col_idx), _ptr(vals), ctypes.byref(opts))
    else:
        st = lib.spmm_plan_create(ctypes.byref(handle), int(M), int(K), _ptr(row_ptr),
                                  _ptr(col_idx), _ptr(vals))
    _check(st, "spmm_plan_create")
    return Plan(handle)
