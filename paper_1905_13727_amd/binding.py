"""ctypes binding of libpsgd.so: same names as include/psgd.h, argument
marshalling only.  Every step of the path runs in the library's HIP kernels;
there is no CPU fallback: if the library is missing the import fails loudly.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpsgd.so")

PSGD_OK, PSGD_EINVAL, PSGD_ENOMEM, PSGD_EHIP, PSGD_EUNSUPPORTED = range(5)
PSGD_F32, PSGD_BF16 = 0, 1
PSGD_MAX_RANK = 64
PSGD_N_KERNELS = 8


class psgd_shape(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64)]


class psgd_sizes(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "n_mat_elems", "n_vec_elems", "grad_stride", "err_stride", "out_elems", "p_elems", "q_elems",
        "workspace_bytes", "n_matrices", "n_vectors", "payload_elems", "compressed_elems",
        "bytes_min", "bytes_stream", "kept_elems")]


class PsgdError(RuntimeError):
    def __init__(self, status: int, where: str, detail: str = ""):
        self.status = status
        msg = "%s: %s" % (where, status_string(status))
        if detail:
            msg += " (" + detail + ")"
        super().__init__(msg)


_lib = None


def load_library(path: Optional[str] = None):
    """Load libpsgd.so built in-tree.  Builds it first only if it is absent."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    path = path or LIB_PATH
    if not os.path.exists(path):
        from . import build as _build
        _build.build_library()
    lib = C.CDLL(path)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.psgd_plan_create.restype = C.c_int
    lib.psgd_plan_create.argtypes = [C.POINTER(psgd_shape), i32, i32, i32, C.c_int, C.c_int, C.POINTER(vp)]
    lib.psgd_plan_destroy.restype = None
    lib.psgd_plan_destroy.argtypes = [vp]
    lib.psgd_plan_sizes.restype = C.c_int
    lib.psgd_plan_sizes.argtypes = [vp, C.POINTER(psgd_sizes)]
    lib.psgd_plan_offsets.restype = C.c_int
    lib.psgd_plan_offsets.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i64), C.POINTER(i64), C.POINTER(i32)]
    lib.psgd_plan_set_tuning.restype = C.c_int
    lib.psgd_plan_set_tuning.argtypes = [vp, C.c_char_p, i64]
    lib.psgd_compress.restype = C.c_int
    lib.psgd_compress.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_decompress.restype = C.c_int
    lib.psgd_decompress.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_step.restype = C.c_int
    lib.psgd_step.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_step_iterations.restype = C.c_int
    lib.psgd_step_iterations.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32]
    lib.psgd_random_block_step.restype = C.c_int
    lib.psgd_random_block_step.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_random_k_step.restype = C.c_int
    lib.psgd_random_k_step.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_plan_path.restype = C.c_int
    lib.psgd_plan_path.argtypes = [vp, C.POINTER(i32)]
    lib.psgd_plan_kept.restype = C.c_int
    lib.psgd_plan_kept.argtypes = [vp, i32, C.POINTER(i64), C.POINTER(i64)]
    lib.psgd_step_static.restype = C.c_int
    lib.psgd_step_static.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.psgd_plan_set_profiling.restype = C.c_int
    lib.psgd_iterate.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.psgd_iterate.restype = C.c_int
    lib.psgd_step_update.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_float, C.c_float, vp, vp]
    lib.psgd_step_update.restype = C.c_int
    lib.psgd_decompress_update.argtypes = [vp, vp, vp, vp, vp, vp, vp, C.c_float, C.c_float, vp, vp]
    lib.psgd_decompress_update.restype = C.c_int
    lib.psgd_plan_set_profiling.argtypes = [vp, i32]
    lib.psgd_plan_kernel_times.restype = C.c_int
    lib.psgd_plan_kernel_times.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.psgd_kernel_name.restype = C.c_char_p
    lib.psgd_kernel_name.argtypes = [i32]
    lib.psgd_plan_check.restype = C.c_int
    lib.psgd_plan_check.argtypes = [vp, vp, C.POINTER(i32)]
    lib.psgd_plan_read_trace.restype = C.c_int
    lib.psgd_plan_read_trace.argtypes = [vp, C.POINTER(C.c_uint64), i64, C.POINTER(i64)]
    lib.psgd_status_string.restype = C.c_char_p
    lib.psgd_status_string.argtypes = [C.c_int]
    lib.psgd_plan_last_error.restype = C.c_char_p
    lib.psgd_plan_last_error.argtypes = [vp]
    if path == LIB_PATH:
        _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().psgd_status_string(int(status)).decode()


def _ptr(x) -> Optional[int]:
    """Device/host address of a torch tensor, or an int address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


class Plan:
    """Owner of one psgd_plan*.  Methods mirror the C entry points."""

    def __init__(self, shapes: Sequence[Tuple[int, ...]], rank: int, workers: int = 1,
                 grad_dtype: int = PSGD_F32, out_dtype: int = PSGD_F32):
        self._lib = load_library()
        self._h = C.c_void_p()
        arr = (psgd_shape * max(1, len(shapes)))()
        for i, s in enumerate(shapes):
            s = tuple(int(v) for v in s)
            if len(s) == 1:
                arr[i].rows, arr[i].cols = s[0], 1
            else:
                rows, cols = s[0], 1
                for v in s[1:]:
                    cols *= v
                arr[i].rows, arr[i].cols = rows, cols
        st = self._lib.psgd_plan_create(arr, len(shapes), int(rank), int(workers), int(grad_dtype),
                                        int(out_dtype), C.byref(self._h))
        if st != PSGD_OK:
            self._h = C.c_void_p()
            raise PsgdError(st, "psgd_plan_create")
        self.n_tensors = len(shapes)
        self.rank = int(rank)
        self.workers = int(workers)
        self.sizes = self.plan_sizes()

    # -- psgd_plan_* ---------------------------------------------------------
    def plan_sizes(self) -> psgd_sizes:
        s = psgd_sizes()
        self._check(self._lib.psgd_plan_sizes(self._h, C.byref(s)), "psgd_plan_sizes")
        return s

    def offsets(self, tensor: int):
        f, p, q, r = C.c_int64(), C.c_int64(), C.c_int64(), C.c_int32()
        self._check(self._lib.psgd_plan_offsets(self._h, int(tensor), C.byref(f), C.byref(p), C.byref(q),
                                                C.byref(r)), "psgd_plan_offsets")
        return f.value, p.value, q.value, r.value

    def set_tuning(self, key: str, value: int):
        self._check(self._lib.psgd_plan_set_tuning(self._h, key.encode(), int(value)), "psgd_plan_set_tuning")
        self.sizes = self.plan_sizes()

    def destroy(self):
        if self._h:
            self._lib.psgd_plan_destroy(self._h)
            self._h = C.c_void_p()

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    # -- psgd_compress / psgd_decompress / psgd_step ---------------------------
    def compress(self, grad, err, q, p, workspace, stream=None):
        self._check(self._lib.psgd_compress(self._h, _ptr(grad), _ptr(err), _ptr(q), _ptr(p), _ptr(workspace),
                                            _ptr(stream)), "psgd_compress")

    def decompress(self, p, q, err, grad, out, workspace, stream=None):
        self._check(self._lib.psgd_decompress(self._h, _ptr(p), _ptr(q), _ptr(err), _ptr(grad), _ptr(out),
                                              _ptr(workspace), _ptr(stream)), "psgd_decompress")

    def step(self, grad, err, q, p, out, workspace, stream=None):
        self._check(self._lib.psgd_step(self._h, _ptr(grad), _ptr(err), _ptr(q), _ptr(p), _ptr(out),
                                        _ptr(workspace), _ptr(stream)), "psgd_step")

    def step_iterations(self, grad, err, q, p, out, workspace, iterations, stream=None):
        self._check(self._lib.psgd_step_iterations(self._h, _ptr(grad), _ptr(err), _ptr(q), _ptr(p), _ptr(out),
                                                   _ptr(workspace), _ptr(stream), int(iterations)),
                    "psgd_step_iterations")

    def random_block_step(self, grad, err, starts, vals, out, stream=None):
        self._check(self._lib.psgd_random_block_step(self._h, _ptr(grad), _ptr(err), _ptr(starts), _ptr(vals), _ptr(out),
                                                     _ptr(stream)), "psgd_random_block_step")

    def random_k_step(self, grad, err, indices, vals, out, stream=None):
        self._check(self._lib.psgd_random_k_step(self._h, _ptr(grad), _ptr(err), _ptr(indices), _ptr(vals), _ptr(out),
                                                 _ptr(stream)), "psgd_random_k_step")

    def path(self) -> str:
        """'streaming', 'resident' or 'matrix cores': the kernels psgd_step runs for this plan."""
        r = C.c_int32()
        self._check(self._lib.psgd_plan_path(self._h, C.byref(r)), "psgd_plan_path")
        return ("streaming", "resident", "matrix cores")[r.value]

    def kept(self, tensor: int):
        off, n = C.c_int64(), C.c_int64()
        self._check(self._lib.psgd_plan_kept(self._h, int(tensor), C.byref(off), C.byref(n)), "psgd_plan_kept")
        return off.value, n.value

    def step_static(self, grad, err, q, p, out, stream=None):
        self._check(self._lib.psgd_step_static(self._h, _ptr(grad), _ptr(err), _ptr(q), _ptr(p), _ptr(out),
                                               _ptr(stream)), "psgd_step_static")

    def iterate(self, err, q, p, workspace, stream=None):
        self._check(self._lib.psgd_iterate(self._h, _ptr(err), _ptr(q), _ptr(p), _ptr(workspace), _ptr(stream)),
                    "psgd_iterate")

    def step_update(self, grad, err, q, p, mom, param, lr, momentum, workspace, stream=None):
        self._check(self._lib.psgd_step_update(self._h, _ptr(grad), _ptr(err), _ptr(q), _ptr(p), _ptr(mom), _ptr(param),
                                               float(lr), float(momentum), _ptr(workspace), _ptr(stream)),
                    "psgd_step_update")

    def decompress_update(self, p, q, err, grad, mom, param, lr, momentum, workspace, stream=None):
        self._check(self._lib.psgd_decompress_update(self._h, _ptr(p), _ptr(q), _ptr(err), _ptr(grad), _ptr(mom),
                                                     _ptr(param), float(lr), float(momentum), _ptr(workspace),
                                                     _ptr(stream)), "psgd_decompress_update")

    def set_profiling(self, enable: bool):
        self._check(self._lib.psgd_plan_set_profiling(self._h, 1 if enable else 0), "psgd_plan_set_profiling")

    def kernel_times(self):
        """(dict kernel name -> accumulated ms, number of steps); clears the accumulators."""
        ms = (C.c_double * PSGD_N_KERNELS)()
        steps = C.c_int64()
        self._check(self._lib.psgd_plan_kernel_times(self._h, ms, C.byref(steps)), "psgd_plan_kernel_times")
        names = [self._lib.psgd_kernel_name(i).decode() for i in range(PSGD_N_KERNELS)]
        return dict(zip(names, list(ms))), steps.value

    def check(self, stream=None) -> bool:
        """Uploads the plan's tables if no GPU call has done so yet; synchronises the stream, raises if a kernel
        whose workgroups wait for each other gave up; returns True if the plan's psgd_step runs in resident mode."""
        r = C.c_int32()
        self._check(self._lib.psgd_plan_check(self._h, _ptr(stream), C.byref(r)), "psgd_plan_check")
        return bool(r.value)

    def read_trace(self, capacity=1 << 18):
        """Diagnostic timestamps of the last resident step: list of per-workgroup lists (see psgd.h)."""
        buf = (C.c_uint64 * capacity)()
        n = C.c_int64()
        self._check(self._lib.psgd_plan_read_trace(self._h, buf, capacity, C.byref(n)), "psgd_plan_read_trace")
        vals = list(buf[: n.value])
        return [vals[i: i + 16] for i in range(0, len(vals), 16)]

    def last_error(self) -> str:
        return self._lib.psgd_plan_last_error(self._h).decode()

    def _check(self, st: int, where: str):
        if st != PSGD_OK:
            raise PsgdError(st, where, self.last_error() if self._h else "")
