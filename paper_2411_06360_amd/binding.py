"""ctypes binding of ``librsr.so`` (C ABI: ``include/rsr.h``).  Marshalling only.

Host arrays are numpy; device buffers are anything with ``data_ptr()`` (torch tensors on the
GPU) or a plain integer address; streams are an integer ``hipStream_t`` (``None``/0 = default,
``torch.cuda.current_stream().cuda_stream`` for torch's).
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_NAME = "librsr.so"
_lib: Optional[ctypes.CDLL] = None

RSR_OK = 0


class RsrError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"rsr error {code}: {message}")
        self.code = code
        self.message = message


class RsrInfo(ctypes.Structure):
    _fields_ = [
        ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
        ("k", ctypes.c_int32), ("parts", ctypes.c_int32),
        ("nblocks", ctypes.c_int64),
        ("last_block_width", ctypes.c_int32), ("lo_bits", ctypes.c_int32), ("hi_bits", ctypes.c_int32),
        ("stored_rows", ctypes.c_int64), ("segments", ctypes.c_int64), ("work_units", ctypes.c_int64),
        ("index_bytes", ctypes.c_int64), ("segment_bytes", ctypes.c_int64),
        ("schedule_bytes", ctypes.c_int64), ("table_bytes", ctypes.c_int64),
        ("device", ctypes.c_int32), ("compute_units", ctypes.c_int32),
        ("row_tiles", ctypes.c_int32), ("reserved", ctypes.c_int32),
    ]

    def as_dict(self) -> dict:
        return {name: getattr(self, name) for name, _ in self._fields_}


# numpy view of the 32-byte unit descriptors (csrc/rsr_format.h)
UNIT_DTYPE = np.dtype(
    [
        ("stream_off", "<u4"), ("block", "<u4"), ("window", "<u2"), ("part", "u1"), ("npos", "u1"),
        ("units_in_block", "<u2"), ("index_in_block", "<u2"), ("slot0", "<u2"), ("reserved0", "<u2"),
        ("nrows", "<u4"), ("nheads", "<u4"), ("nentries", "<u4"),
    ]
)
assert UNIT_DTYPE.itemsize == 32


def lib_path() -> str:
    """The built library, next to this file."""
    return os.path.join(HERE, _LIB_NAME)


def load(path: Optional[str] = None) -> ctypes.CDLL:
    """Load the built library (once per process; `path` names another build of the same sources and
    only counts on the first call).  Never builds and never falls back to anything else."""
    global _lib
    if _lib is not None:
        return _lib
    path = path or lib_path()
    if not os.path.exists(path):
        raise RuntimeError(
            f"{path} is missing: the HIP library has not been built "
            "(run `python -m paper_2411_06360_amd.build`); there is no CPU fallback"
        )
    # One HIP runtime per process: PyTorch ships its own libamdhip64 and owns the device buffers
    # and streams handed to this library, so its copy has to be the one that is already loaded
    # when librsr.so resolves its dependency (same SONAME).  Loading in the other order leaves
    # two runtimes in the process and torch then finds no GPU.
    import torch  # noqa: F401

    L = ctypes.CDLL(path)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    L.rsr_preprocess.argtypes = [vp, i64, i64, ci]
    L.rsr_preprocess.restype = vp
    L.rsr_preprocess_device.argtypes = [vp, i64, i64, ci]
    L.rsr_preprocess_device.restype = vp
    L.rsr_matvec.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_matvec.restype = ci
    L.rsr_matvec_i8.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_matvec_i8.restype = ci
    L.rsr_matvec_multi.argtypes = [vp, ci, ci, vp]
    L.rsr_matvec_multi.restype = ci
    L.rsr_matvec_multi_i8.argtypes = [vp, ci, ci, vp]
    L.rsr_matvec_multi_i8.restype = ci
    L.rsr_set_step2.argtypes = [vp, ci]
    L.rsr_set_step2.restype = ci
    L.rsr_model_k.argtypes = [i64, ci, ci]
    L.rsr_model_k.restype = ci
    L.rsr_autotune_k.argtypes = [vp, i64, i64, ci, ci, ci, ci, ci, ctypes.POINTER(ci), vp]
    L.rsr_autotune_k.restype = ci
    L.rsr_destroy.argtypes = [vp]
    L.rsr_destroy.restype = None
    L.rsr_last_error.argtypes = []
    L.rsr_last_error.restype = ctypes.c_char_p
    L.rsr_info.argtypes = [vp, ctypes.POINTER(RsrInfo)]
    L.rsr_info.restype = ci
    L.rsr_export_block.argtypes = [vp, ci, i64, vp, vp]
    L.rsr_export_block.restype = ci
    L.rsr_host_pack.argtypes = [vp, i64, i64, ci]
    L.rsr_host_pack.restype = vp
    L.rsr_host_free.argtypes = [vp]
    L.rsr_host_free.restype = None
    L.rsr_host_info.argtypes = [vp, ctypes.POINTER(RsrInfo)]
    L.rsr_host_info.restype = ci
    L.rsr_host_export_block.argtypes = [vp, ci, i64, vp, vp]
    L.rsr_host_export_block.restype = ci
    L.rsr_host_streams.argtypes = ([vp, ci] + [ctypes.POINTER(vp), ctypes.POINTER(i64)] * 2 + [ctypes.POINTER(vp)]
                                   + [ctypes.POINTER(i64)] * 2)
    L.rsr_host_streams.restype = ci
    L.rsr_matvec_acc.argtypes = [vp, vp, vp, ctypes.c_float, ci, vp]
    L.rsr_matvec_acc.restype = ci
    L.rsr_matvec_acc_i8.argtypes = [vp, vp, vp, ctypes.c_int32, ci, vp]
    L.rsr_matvec_acc_i8.restype = ci
    L.rsr_qbit_preprocess.argtypes = [vp, i64, i64, ci, ci]
    L.rsr_qbit_preprocess.restype = vp
    L.rsr_qbit_matvec.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_qbit_matvec.restype = ci
    L.rsr_qbit_matvec_i8.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_qbit_matvec_i8.restype = ci
    L.rsr_qbit_planes.argtypes = [vp]
    L.rsr_qbit_planes.restype = ci
    L.rsr_qbit_table_bytes.argtypes = [vp]
    L.rsr_qbit_table_bytes.restype = i64
    L.rsr_qbit_destroy.argtypes = [vp]
    L.rsr_qbit_destroy.restype = None
    L.rsr_dense_preprocess.argtypes = [vp, i64, i64]
    L.rsr_dense_preprocess.restype = vp
    L.rsr_dense_matvec.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_dense_matvec.restype = ci
    L.rsr_dense_matvec_i8.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_dense_matvec_i8.restype = ci
    L.rsr_dense_matvec_static.argtypes = [vp, vp, vp, ci, vp]
    L.rsr_dense_matvec_static.restype = ci
    L.rsr_dense_table_bytes.argtypes = [vp]
    L.rsr_dense_table_bytes.restype = i64
    L.rsr_dense_destroy.argtypes = [vp]
    L.rsr_dense_destroy.restype = None
    _lib = L
    return L


def rsr_last_error() -> str:
    return (load().rsr_last_error() or b"").decode("utf-8", "replace")


def _check(code: int) -> None:
    if code != RSR_OK:
        raise RsrError(code, rsr_last_error())


def _host_matrix(A) -> np.ndarray:
    A = np.asarray(A)
    if A.dtype != np.int8:
        raise TypeError("A must be int8")
    if A.ndim != 2:
        raise ValueError("A must be 2-D (rows x cols)")
    return np.ascontiguousarray(A)


def _addr(x) -> int:
    if x is None:
        return 0
    if hasattr(x, "data_ptr"):
        return int(x.data_ptr())
    return int(x)


def rsr_preprocess(A, k: int) -> int:
    """``A``: host int8 array ``rows x cols``.  Returns the handle (an integer address)."""
    A = _host_matrix(A)
    h = load().rsr_preprocess(A.ctypes.data, A.shape[0], A.shape[1], int(k))
    if not h:
        raise RsrError(-1, rsr_last_error())
    return int(h)


def rsr_preprocess_device(A_dev, rows: int, cols: int, k: int) -> int:
    """``A_dev``: device int8 buffer ``rows x cols`` (row-major).  Returns the handle."""
    h = load().rsr_preprocess_device(_addr(A_dev), int(rows), int(cols), int(k))
    if not h:
        raise RsrError(-1, rsr_last_error())
    return int(h)


def rsr_matvec(handle: int, v, out, batch: int, stream=None) -> None:
    """``v``: device float32 ``[batch][rows]``; ``out``: device float32 ``[batch][cols]``."""
    _check(load().rsr_matvec(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_matvec_i8(handle: int, v, out, batch: int, stream=None) -> None:
    """``v``: device int8 ``[batch][rows]``; ``out``: device int32 ``[batch][cols]``."""
    _check(load().rsr_matvec_i8(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_matvec_acc(handle: int, v, out, scale: float, batch: int, stream=None) -> None:
    """``out += scale * (v . A)`` on device float32 buffers."""
    _check(load().rsr_matvec_acc(handle, _addr(v), _addr(out), float(scale), int(batch), _addr(stream)))


def rsr_matvec_acc_i8(handle: int, v, out, scale: int, batch: int, stream=None) -> None:
    """``out += scale * (v . A)`` for device int8 activations and int32 results."""
    _check(load().rsr_matvec_acc_i8(handle, _addr(v), _addr(out), int(scale), int(batch), _addr(stream)))


# ---- q-bit matrices as weighted binary planes (include/rsr_qbit.h) ----
def rsr_qbit_preprocess(A, k: int, q: int) -> int:
    A = _host_matrix(A)
    h = load().rsr_qbit_preprocess(A.ctypes.data, A.shape[0], A.shape[1], int(k), int(q))
    if not h:
        raise RsrError(-1, rsr_last_error())
    return int(h)


def rsr_qbit_matvec(handle: int, v, out, batch: int, stream=None) -> None:
    _check(load().rsr_qbit_matvec(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_qbit_matvec_i8(handle: int, v, out, batch: int, stream=None) -> None:
    _check(load().rsr_qbit_matvec_i8(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_qbit_planes(handle: int) -> int:
    return int(load().rsr_qbit_planes(handle))


def rsr_qbit_table_bytes(handle: int) -> int:
    return int(load().rsr_qbit_table_bytes(handle))


def rsr_qbit_destroy(handle: Optional[int]) -> None:
    if handle:
        load().rsr_qbit_destroy(handle)


RSR_STEP2_FOLD, RSR_STEP2_PLAIN = 0, 1


def rsr_set_step2(handle: int, step2: int) -> None:
    """Step 2 as the RSR++ fold (RSR_STEP2_FOLD, default) or as the plain product (RSR_STEP2_PLAIN)."""
    _check(load().rsr_set_step2(handle, int(step2)))


def rsr_model_k(rows: int, k_min: int, k_max: int) -> int:
    k = load().rsr_model_k(int(rows), int(k_min), int(k_max))
    if k < 0:
        raise RsrError(k, rsr_last_error())
    return k


def rsr_autotune_k(A, batch: int, k_min: int, k_max: int, reps: int = 50, cold: bool = True):
    """Returns (best k, {k: microseconds per product})."""
    A = _host_matrix(A)
    best = ctypes.c_int(0)
    us = np.zeros(k_max - k_min + 1, dtype=np.float64)
    _check(load().rsr_autotune_k(A.ctypes.data, A.shape[0], A.shape[1], int(batch), int(k_min), int(k_max), int(reps),
                                 1 if cold else 0, ctypes.byref(best), us.ctypes.data))
    return int(best.value), {k_min + i: float(x) for i, x in enumerate(us)}


# ---- the bit-packed comparator (include/rsr_dense.h) ----
def rsr_dense_preprocess(A) -> int:
    A = _host_matrix(A)
    h = load().rsr_dense_preprocess(A.ctypes.data, A.shape[0], A.shape[1])
    if not h:
        raise RsrError(-1, rsr_last_error())
    return int(h)


def rsr_dense_matvec(handle: int, v, out, batch: int, stream=None) -> None:
    _check(load().rsr_dense_matvec(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_dense_matvec_i8(handle: int, v, out, batch: int, stream=None) -> None:
    _check(load().rsr_dense_matvec_i8(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_dense_matvec_static(handle: int, v, out, batch: int, stream=None) -> None:
    """As rsr_dense_matvec, with the partial sums in the library's static device buffer (allocates nothing)."""
    _check(load().rsr_dense_matvec_static(handle, _addr(v), _addr(out), int(batch), _addr(stream)))


def rsr_dense_table_bytes(handle: int) -> int:
    return int(load().rsr_dense_table_bytes(handle))


def rsr_dense_destroy(handle: Optional[int]) -> None:
    if handle:
        load().rsr_dense_destroy(handle)


class RsrJob(ctypes.Structure):
    _fields_ = [("h", ctypes.c_void_p), ("v", ctypes.c_void_p), ("out", ctypes.c_void_p)]


def make_jobs(jobs):
    """A C array of rsr_job from (handle, v, out) triples; keep it alive while it is in use."""
    arr = (RsrJob * len(jobs))()
    for i, (h, v, out) in enumerate(jobs):
        arr[i].h, arr[i].v, arr[i].out = int(h), _addr(v), _addr(out)
    return arr


def rsr_matvec_multi(jobs, batch: int, stream=None) -> None:
    """``jobs``: (handle, v, out) triples with float activations, or an array made by make_jobs."""
    arr = jobs if isinstance(jobs, ctypes.Array) else make_jobs(jobs)
    _check(load().rsr_matvec_multi(ctypes.cast(arr, ctypes.c_void_p), len(arr), int(batch), _addr(stream)))


def rsr_matvec_multi_i8(jobs, batch: int, stream=None) -> None:
    arr = jobs if isinstance(jobs, ctypes.Array) else make_jobs(jobs)
    _check(load().rsr_matvec_multi_i8(ctypes.cast(arr, ctypes.c_void_p), len(arr), int(batch), _addr(stream)))


def rsr_destroy(handle: Optional[int]) -> None:
    if handle:
        load().rsr_destroy(handle)


def rsr_info(handle: int) -> RsrInfo:
    info = RsrInfo()
    _check(load().rsr_info(handle, ctypes.byref(info)))
    return info


def _export(fn, handle: int, part: int, block: int, rows: int, width: int) -> Tuple[np.ndarray, np.ndarray]:
    sigma = np.empty(rows, dtype=np.int32)
    L = np.empty((1 << width) + 1, dtype=np.int32)
    _check(fn(handle, int(part), int(block), sigma.ctypes.data, L.ctypes.data))
    return sigma, L


def rsr_export_block(handle: int, part: int, block: int) -> Tuple[np.ndarray, np.ndarray]:
    """``(sigma, L)`` of one block, counted from 0; ``L`` has ``2^width + 1`` entries."""
    info = rsr_info(handle)
    width = info.last_block_width if block == info.nblocks - 1 else info.k
    return _export(load().rsr_export_block, handle, part, block, info.rows, width)


def rsr_host_pack(A, k: int) -> int:
    A = _host_matrix(A)
    x = load().rsr_host_pack(A.ctypes.data, A.shape[0], A.shape[1], int(k))
    if not x:
        raise RsrError(-1, rsr_last_error())
    return int(x)


def rsr_host_free(x: Optional[int]) -> None:
    if x:
        load().rsr_host_free(x)


def rsr_host_info(x: int) -> RsrInfo:
    info = RsrInfo()
    _check(load().rsr_host_info(x, ctypes.byref(info)))
    return info


def rsr_host_export_block(x: int, part: int, block: int) -> Tuple[np.ndarray, np.ndarray]:
    info = rsr_host_info(x)
    width = info.last_block_width if block == info.nblocks - 1 else info.k
    return _export(load().rsr_host_export_block, x, part, block, info.rows, width)


def rsr_host_streams(x: int, tile: int = 0) -> dict:
    """Copies of the packed streams of one row tile as numpy arrays: stream (uint16), units (structured),
    blk_unit, and the tile's first row and height."""
    vp, i64 = ctypes.c_void_p, ctypes.c_int64
    pe, pu, pb = vp(), vp(), vp()
    ne, nu, r0, nr = i64(), i64(), i64(), i64()
    _check(load().rsr_host_streams(x, int(tile), ctypes.byref(pe), ctypes.byref(ne), ctypes.byref(pu), ctypes.byref(nu),
                                   ctypes.byref(pb), ctypes.byref(r0), ctypes.byref(nr)))
    info = rsr_host_info(x)

    def view(ptr, count, dtype):
        if count == 0:
            return np.empty(0, dtype=dtype)
        nbytes = count * np.dtype(dtype).itemsize
        buf = (ctypes.c_char * nbytes).from_address(ptr.value)
        return np.frombuffer(buf, dtype=dtype, count=count).copy()

    return {
        "stream": view(pe, ne.value, np.uint16),
        "units": view(pu, nu.value, UNIT_DTYPE),
        "blk_unit": view(pb, info.nblocks + 1, np.uint32),
        "row0": int(r0.value),
        "rows": int(nr.value),
    }
