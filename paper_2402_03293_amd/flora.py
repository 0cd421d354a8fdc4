"""ctypes binding of libflora.so (include/flora.h): argument marshalling only.

Every step of the method runs in the HIP kernels behind the C ABI.  PyTorch is
used by callers for device memory and streams; this module only needs
``tensor.data_ptr()`` and a stream handle.  There is no CPU fallback: if the
library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
from pathlib import Path
from typing import Optional, Sequence

F32 = 0
BF16 = 1
OK = 0
ERR_INVALID = -1
ERR_UNSUPPORTED = -2
ERR_DEVICE = -3
ERR_TOO_LARGE = -4
STATIC_SCRATCH_BYTES = 32 << 20
RULE_SGD = 0
RULE_FACTORED = 1
RULE_UNFACTORED = 2
INPUT_IDENTITY = 0
INPUT_SQUARE = 1

_LIB_PATH = Path(__file__).resolve().parent / "libflora.so"


class Matrix(ctypes.Structure):
    """flora_matrix_t"""
    _fields_ = [
        ("grad", ctypes.c_void_p),
        ("weight", ctypes.c_void_p),
        ("state", ctypes.c_void_p),
        ("row_stat", ctypes.c_void_p),
        ("col_stat", ctypes.c_void_p),
        ("n", ctypes.c_int64),
        ("m", ctypes.c_int64),
        ("seed", ctypes.c_uint64),
        ("seed_next", ctypes.c_uint64),
        ("second_moment", ctypes.c_void_p),
        ("weight_sumsq", ctypes.c_void_p),
    ]


class Update(ctypes.Structure):
    """flora_update_t"""
    _fields_ = [
        ("rule", ctypes.c_int),
        ("lr", ctypes.c_float),
        ("alpha", ctypes.c_float),
        ("beta2", ctypes.c_float),
        ("eps1", ctypes.c_float),
        ("clip_d", ctypes.c_float),
        ("zero_state_after", ctypes.c_int),
        ("scale_parameter", ctypes.c_int),
        ("eps2", ctypes.c_float),
        ("step_weight_mib", ctypes.c_float),
    ]


class FloraError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().flora_status_string(status).decode()
        extra = ""
        if status == ERR_DEVICE:
            extra = " (hipError %d)" % lib().flora_last_device_error()
        super().__init__("%s: %s%s" % (where, msg, extra))


_lib = None


def lib():
    """The loaded C library.  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not _LIB_PATH.exists():
            raise ImportError(
                "libflora.so is missing at %s: build it with "
                "`python -m paper_2402_03293_amd.build` (needs hipcc)" % _LIB_PATH)
        L = ctypes.CDLL(str(_LIB_PATH))
        MP = ctypes.POINTER(Matrix)
        vp, ci, cf = ctypes.c_void_p, ctypes.c_int, ctypes.c_float
        L.flora_compress.argtypes = [MP, ci, ci, ci, cf, cf, vp]
        L.flora_compress.restype = ci
        L.flora_compress_mapped.argtypes = [MP, ci, ci, ci, ci, cf, cf, vp]
        L.flora_compress_mapped.restype = ci
        L.flora_decompress.argtypes = [MP, ci, ci, cf, ctypes.POINTER(vp), ci, vp]
        L.flora_decompress.restype = ci
        L.flora_momentum_transfer.argtypes = [MP, ci, ci, vp]
        L.flora_momentum_transfer.restype = ci
        L.flora_transfer_accumulate.argtypes = [MP, ci, ci, cf, cf, ctypes.POINTER(vp), vp]
        L.flora_transfer_accumulate.restype = ci
        L.flora_apply_update.argtypes = [MP, ci, ci, ci, ctypes.POINTER(Update), vp]
        L.flora_apply_update.restype = ci
        L.flora_fused_step.argtypes = [MP, ci, ci, ci, ci, cf, cf, ci, ctypes.POINTER(Update), vp]
        L.flora_fused_step.restype = ci
        L.flora_weight_sumsq.argtypes = [MP, ci, ci, vp]
        L.flora_weight_sumsq.restype = ci
        L.flora_adafactor_schedule.argtypes = [ctypes.c_uint64, ctypes.POINTER(cf), ctypes.POINTER(cf)]
        L.flora_adafactor_schedule.restype = None
        L.flora_debug_generate.argtypes = [ctypes.c_uint64, ctypes.c_int64, ci, vp, vp, vp]
        L.flora_debug_generate.restype = ci
        L.flora_debug_work_items.argtypes = [ci, MP, ci, ci, ci, vp, ctypes.c_int64, vp]
        L.flora_debug_work_items.restype = ctypes.c_int64
        L.flora_debug_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.flora_debug_copy.restype = ci
        L.flora_debug_read.argtypes = [vp, ctypes.c_size_t, ci, ctypes.c_size_t, ci, vp, vp]
        L.flora_debug_read.restype = ci
        L.flora_debug_compute_loop.argtypes = [ci, ci, vp, ctypes.POINTER(ctypes.c_double), vp]
        L.flora_debug_compute_loop.restype = ci
        L.flora_derive_seed.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ctypes.c_uint64]
        L.flora_derive_seed.restype = ctypes.c_uint64
        L.flora_derive_seeds.argtypes = [ctypes.c_uint64, ctypes.c_uint64, ci, ctypes.c_uint64, vp]
        L.flora_derive_seeds.restype = None
        L.flora_workspace_bytes.argtypes = [MP, ci, ci]
        L.flora_workspace_bytes.restype = ctypes.c_size_t
        L.flora_momentum_transfer_static.argtypes = [MP, ci, ci, vp]
        L.flora_momentum_transfer_static.restype = ci
        L.flora_debug_plan_bytes.argtypes = [ci, MP, ci, ci, ci]
        L.flora_debug_plan_bytes.restype = ctypes.c_int64
        L.flora_set_workspace.argtypes = [vp, ctypes.c_size_t]
        L.flora_set_workspace.restype = ci
        L.flora_set_tuning.argtypes = [ctypes.c_char_p, ci]
        L.flora_set_tuning.restype = ci
        L.flora_last_device_error.argtypes = []
        L.flora_last_device_error.restype = ci
        L.flora_status_string.argtypes = [ci]
        L.flora_status_string.restype = ctypes.c_char_p
        L.flora_shutdown.argtypes = []
        L.flora_shutdown.restype = None
        L.flora_version.argtypes = []
        L.flora_version.restype = ci
        _lib = L
    return _lib


EXPORTS = [
    "flora_compress", "flora_compress_mapped", "flora_decompress", "flora_momentum_transfer", "flora_transfer_accumulate",
    "flora_apply_update",
    "flora_fused_step", "flora_weight_sumsq", "flora_adafactor_schedule", "flora_debug_generate",
    "flora_debug_work_items", "flora_debug_copy", "flora_debug_read", "flora_debug_compute_loop", "flora_derive_seed", "flora_derive_seeds",
    "flora_workspace_bytes", "flora_set_workspace", "flora_set_tuning", "flora_momentum_transfer_static",
    "flora_debug_plan_bytes",
    "flora_last_device_error", "flora_status_string", "flora_shutdown", "flora_version",
]


def _ptr(t) -> Optional[int]:
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def matrices(n_m: Sequence, grads=None, weights=None, states=None, row_stats=None, col_stats=None,
             seeds=None, seeds_next=None, second_moments=None, weight_sumsqs=None):
    """Builds a ctypes array of flora_matrix_t.  Each argument is a sequence of
    torch tensors (or raw device addresses) or None."""
    count = len(n_m)
    arr = (Matrix * count)()
    for l, (n, m) in enumerate(n_m):
        arr[l].n, arr[l].m = int(n), int(m)
        arr[l].grad = _ptr(grads[l]) if grads is not None else None
        arr[l].weight = _ptr(weights[l]) if weights is not None else None
        arr[l].state = _ptr(states[l]) if states is not None else None
        arr[l].row_stat = _ptr(row_stats[l]) if row_stats is not None else None
        arr[l].col_stat = _ptr(col_stats[l]) if col_stats is not None else None
        arr[l].second_moment = _ptr(second_moments[l]) if second_moments is not None else None
        arr[l].weight_sumsq = _ptr(weight_sumsqs[l]) if weight_sumsqs is not None else None
        arr[l].seed = int(seeds[l]) if seeds is not None else 0
        arr[l].seed_next = int(seeds_next[l]) if seeds_next is not None else 0
    return arr


def _check(status: int, where: str):
    if status != OK:
        raise FloraError(status, where)


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return stream.cuda_stream or None          # torch.cuda.Stream


def compress(mats, r: int, grad_dtype: int, a: float = 1.0, b: float = 1.0, stream=None):
    _check(lib().flora_compress(mats, len(mats), r, grad_dtype, a, b, _stream(stream)), "flora_compress")


def compress_mapped(mats, r: int, grad_dtype: int, input_map: int, a: float = 1.0, b: float = 1.0, stream=None):
    _check(lib().flora_compress_mapped(mats, len(mats), r, grad_dtype, input_map, a, b, _stream(stream)),
           "flora_compress_mapped")


def decompress(mats, r: int, alpha: float, outs, out_dtype: int, stream=None):
    count = len(mats)
    arr = (ctypes.c_void_p * count)(*[_ptr(o) for o in outs])
    _check(lib().flora_decompress(mats, count, r, alpha, arr, out_dtype, _stream(stream)), "flora_decompress")


def momentum_transfer(mats, r: int, stream=None):
    _check(lib().flora_momentum_transfer(mats, len(mats), r, _stream(stream)), "flora_momentum_transfer")


def momentum_transfer_static(mats, r: int, stream=None):
    """flora_momentum_transfer_static: the transfer out of the library's fixed scratch array."""
    _check(lib().flora_momentum_transfer_static(mats, len(mats), r, _stream(stream)), "flora_momentum_transfer_static")


def debug_plan_bytes(plan_kind: int, shapes, r: int, grad_dtype: int = F32) -> int:
    mats = matrices(shapes)
    n = int(lib().flora_debug_plan_bytes(plan_kind, mats, len(mats), r, grad_dtype))
    if n < 0:
        raise FloraError(n, "flora_debug_plan_bytes")
    return n


def transfer_accumulate(mats, r: int, a: float, b: float, dsts, stream=None):
    count = len(mats)
    arr = (ctypes.c_void_p * count)(*[_ptr(d) for d in dsts])
    _check(lib().flora_transfer_accumulate(mats, count, r, a, b, arr, _stream(stream)),
           "flora_transfer_accumulate")


def apply_update(mats, r: int, weight_dtype: int, update: Update, stream=None):
    _check(lib().flora_apply_update(mats, len(mats), r, weight_dtype, ctypes.byref(update), _stream(stream)),
           "flora_apply_update")


def fused_step(mats, r: int, grad_dtype: int, weight_dtype: int, a: float, b: float, do_transfer: bool,
               update: Update, stream=None):
    _check(lib().flora_fused_step(mats, len(mats), r, grad_dtype, weight_dtype, a, b, int(do_transfer),
                                  ctypes.byref(update), _stream(stream)), "flora_fused_step")


def debug_generate(seed: int, m: int, r: int, A_out=None, raw_out=None, stream=None):
    _check(lib().flora_debug_generate(seed, m, r, _ptr(A_out), _ptr(raw_out), _stream(stream)),
           "flora_debug_generate")


def debug_work_items(kind: int, shapes, r: int, grad_dtype: int = F32):
    """(items, info): the work table for these shapes as an int64 array [workgroups, 12] and the
    launch-shape info (host only, no GPU).  Columns: mat, row0, rows, col0, slice, rblock, col1,
    part, nparts, cidx, poff, 0."""
    import numpy as np
    mats = matrices(shapes)
    info = np.zeros(5, dtype=np.int64)
    n = lib().flora_debug_work_items(kind, mats, len(mats), r, grad_dtype, None, 0, info.ctypes.data)
    if n < 0:
        raise FloraError(int(n), "flora_debug_work_items")
    out = np.zeros((int(n), 12), dtype=np.int64)
    lib().flora_debug_work_items(kind, mats, len(mats), r, grad_dtype, out.ctypes.data, int(n), info.ctypes.data)
    return out, info


def debug_copy(src, dst, nbytes: int, stream=None):
    _check(lib().flora_debug_copy(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "flora_debug_copy")


def debug_read(src, nbytes: int, sink, pattern: int = 0, row_bytes: int = 0, chunk_bytes: int = 0, stream=None):
    _check(lib().flora_debug_read(_ptr(src), nbytes, pattern, row_bytes, chunk_bytes, _ptr(sink), _stream(stream)),
           "flora_debug_read")


def debug_compute_loop(kind: int, iters: int, sink, stream=None) -> float:
    """Launches the loop and returns the flops (kinds 0-2) or normals (kind 3) it performs."""
    work = ctypes.c_double(0.0)
    _check(lib().flora_debug_compute_loop(kind, iters, _ptr(sink), ctypes.byref(work), _stream(stream)),
           "flora_debug_compute_loop")
    return work.value


def derive_seed(global_seed: int, matrix_id: int, epoch: int) -> int:
    return int(lib().flora_derive_seed(global_seed, matrix_id, epoch))


def derive_seeds(global_seed: int, first_matrix_id: int, count: int, epoch: int):
    """numpy uint64 array of `count` seeds (one C call)."""
    import numpy as np
    out = np.empty(count, dtype=np.uint64)
    lib().flora_derive_seeds(global_seed, first_matrix_id, count, epoch, out.ctypes.data)
    return out


def fields(mats):
    """A numpy structured view of a flora_matrix_t array: `fields(mats)["seed"][:] = seeds`
    rewrites one field of every descriptor without a Python loop."""
    import numpy as np
    dt = np.dtype([("grad", np.uint64), ("weight", np.uint64), ("state", np.uint64),
                   ("row_stat", np.uint64), ("col_stat", np.uint64), ("n", np.int64), ("m", np.int64),
                   ("seed", np.uint64), ("seed_next", np.uint64),
                   ("second_moment", np.uint64), ("weight_sumsq", np.uint64)])
    return np.frombuffer(mats, dtype=dt)


def workspace_bytes(mats, r: int) -> int:
    return int(lib().flora_workspace_bytes(mats, len(mats), r))


def set_workspace(buf, nbytes: int = 0):
    """Hands the library a caller-owned device buffer (a torch tensor or a raw address) for all its
    private device memory; ``set_workspace(None)`` returns to library-allocated memory."""
    if buf is None:
        _check(lib().flora_set_workspace(None, 0), "flora_set_workspace")
        return
    if not nbytes:
        nbytes = buf.numel() * buf.element_size()
    _check(lib().flora_set_workspace(_ptr(buf), nbytes), "flora_set_workspace")


def sgd_update(lr: float, alpha: float = 1.0, zero_state_after: bool = False, step_weight_mib: float = 0.0) -> Update:
    return Update(RULE_SGD, lr, alpha, 0.0, 0.0, 0.0, int(zero_state_after), 0, 0.0, step_weight_mib)


def factored_update(lr: float, alpha: float, beta2: float, eps1: float, clip_d: float,
                    zero_state_after: bool = False, scale_parameter: bool = False,
                    eps2: float = 1e-3, step_weight_mib: float = 0.0) -> Update:
    return Update(RULE_FACTORED, lr, alpha, beta2, eps1, clip_d, int(zero_state_after),
                  int(scale_parameter), eps2, step_weight_mib)


def unfactored_update(lr: float, alpha: float, beta2: float, eps1: float, clip_d: float,
                      zero_state_after: bool = False, scale_parameter: bool = False,
                      eps2: float = 1e-3, step_weight_mib: float = 0.0) -> Update:
    return Update(RULE_UNFACTORED, lr, alpha, beta2, eps1, clip_d, int(zero_state_after),
                  int(scale_parameter), eps2, step_weight_mib)


def weight_sumsq(mats, weight_dtype: int = F32, stream=None):
    _check(lib().flora_weight_sumsq(mats, len(mats), weight_dtype, _stream(stream)), "flora_weight_sumsq")


def adafactor_schedule(t: int):
    """(rho_t, beta2_t) of the published schedules for step t = 1, 2, ..."""
    rho, beta2 = ctypes.c_float(0.0), ctypes.c_float(0.0)
    lib().flora_adafactor_schedule(int(t), ctypes.byref(rho), ctypes.byref(beta2))
    return rho.value, beta2.value


def set_tuning(name: str, value: int):
    _check(lib().flora_set_tuning(name.encode(), value), "flora_set_tuning")


def shutdown():
    lib().flora_shutdown()


def version() -> int:
    return lib().flora_version()
