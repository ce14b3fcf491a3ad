"""Thin ctypes binding of the C ABI in include/stripe.h.

Argument marshalling only: every step of a block's evaluation runs in the HIP
library.  The functions keep the C names; `StripeBlock` is a small
convenience wrapper that owns a handle.  PyTorch appears only as the owner of
device memory and streams (callers pass tensor.data_ptr() and a stream handle).

The library is loaded from this directory.  If it has not been built the import
of this module fails loudly; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libstripe_hip.so")

STRIPE_OK = 0
STATUS_NAMES = {0: "OK", 1: "ERR_NULL", 2: "ERR_INVALID_DESC", 3: "ERR_UNSUPPORTED", 4: "ERR_OUT_OF_BOUNDS",
                5: "ERR_ASSIGN_CONFLICT", 6: "ERR_HIP", 7: "ERR_NOMEM"}
PATHS = {"auto": 0, "generic": 1, "mfma_gemm": 2, "mfma_conv": 3, "pool": 4}
PATH_NAMES = {v: k for k, v in PATHS.items()}

_DIR = {"in": 0, "out": 1}
_DTYPE = {"i8": 0, "i32": 1, "bf16": 2, "f32": 3}
_AGG = {"assign": 0, "add": 1, "max": 2, "min": 3}
_INTR = {"mul": 0, "copy": 1, "add": 2}

EXPORTS = ("stripe_block_create", "stripe_block_create_for_path", "stripe_block_run", "stripe_block_query",
           "stripe_block_destroy", "stripe_status_string", "stripe_last_error", "stripe_device_copy")


class stripe_refinement_t(C.Structure):
    _fields_ = [("dir", C.c_int), ("dtype", C.c_int), ("agg", C.c_int), ("ndim", C.c_int32),
                ("access_coeff", C.POINTER(C.c_int64)), ("access_const", C.POINTER(C.c_int64)),
                ("sizes", C.POINTER(C.c_int64)), ("strides", C.POINTER(C.c_int64))]


class stripe_block_desc_t(C.Structure):
    pass


stripe_block_desc_t._fields_ = [
    ("n_idx", C.c_int32), ("ranges", C.POINTER(C.c_int64)),
    ("n_passed", C.c_int32), ("passed_coeff", C.POINTER(C.c_int64)), ("passed_const", C.POINTER(C.c_int64)),
    ("n_constraints", C.c_int32), ("cons_coeff", C.POINTER(C.c_int64)), ("cons_const", C.POINTER(C.c_int64)),
    ("n_refs", C.c_int32), ("refs", C.POINTER(stripe_refinement_t)),
    ("intrinsic", C.c_int), ("child", C.POINTER(stripe_block_desc_t))]


class stripe_block_info_t(C.Structure):
    _fields_ = [("path", C.c_int32), ("n_idx", C.c_int32), ("n_out_idx", C.c_int32), ("n_red_idx", C.c_int32),
                ("hull_points", C.c_int64), ("work_points", C.c_int64), ("output_elements", C.c_int64),
                ("algorithmic_bytes", C.c_int64),
                ("tile_m", C.c_int32), ("tile_n", C.c_int32), ("tile_k", C.c_int32),
                ("frag_m", C.c_int32), ("frag_n", C.c_int32), ("frag_k", C.c_int32),
                ("lds_bytes", C.c_int32), ("workgroup_size", C.c_int32), ("grid", C.c_int64),
                ("kernel", C.c_char * 64)]


class StripeError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"stripe: {STATUS_NAMES.get(status, status)}: {detail}")
        self.status = status
        self.detail = detail


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1903_06498_amd.build` "
                          "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    handle = C.c_void_p
    lib.stripe_block_create.restype = C.c_int
    lib.stripe_block_create.argtypes = [C.POINTER(stripe_block_desc_t), C.POINTER(handle)]
    lib.stripe_block_create_for_path.restype = C.c_int
    lib.stripe_block_create_for_path.argtypes = [C.POINTER(stripe_block_desc_t), C.c_int, C.POINTER(handle)]
    lib.stripe_block_run.restype = C.c_int
    lib.stripe_block_run.argtypes = [handle, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]
    lib.stripe_block_query.restype = C.c_int
    lib.stripe_block_query.argtypes = [handle, C.POINTER(stripe_block_info_t)]
    lib.stripe_block_destroy.restype = None
    lib.stripe_block_destroy.argtypes = [handle]
    lib.stripe_status_string.restype = C.c_char_p
    lib.stripe_status_string.argtypes = [C.c_int]
    lib.stripe_last_error.restype = C.c_char_p
    lib.stripe_last_error.argtypes = []
    lib.stripe_device_copy.restype = C.c_int
    lib.stripe_device_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    return lib


lib = _load()


def _i64(values, keep):
    flat = [int(v) for v in values]
    arr = (C.c_int64 * max(1, len(flat)))(*flat)
    keep.append(arr)
    return C.cast(arr, C.POINTER(C.c_int64))


def marshal(block, keep: list) -> stripe_block_desc_t:
    """A block description (workloads.Block or anything with its attributes) as C structs."""
    d = stripe_block_desc_t()
    d.n_idx = len(block.idx_names)
    d.ranges = _i64(block.ranges, keep)
    d.n_passed = len(block.passed_names)
    d.passed_coeff = _i64([v for row in block.passed_coeff for v in row], keep)
    d.passed_const = _i64(block.passed_const, keep)
    d.n_constraints = len(block.cons_coeff)
    d.cons_coeff = _i64([v for row in block.cons_coeff for v in row], keep)
    d.cons_const = _i64(block.cons_const, keep)
    d.n_refs = len(block.refs)
    refs = (stripe_refinement_t * max(1, len(block.refs)))()
    keep.append(refs)
    for i, r in enumerate(block.refs):
        refs[i].dir = _DIR[r.dir]
        refs[i].dtype = _DTYPE[r.dtype]
        refs[i].agg = _AGG[r.agg]
        refs[i].ndim = len(r.sizes)
        refs[i].access_coeff = _i64([v for row in r.access_coeff for v in row], keep)
        refs[i].access_const = _i64(r.access_const, keep)
        refs[i].sizes = _i64(r.sizes, keep)
        refs[i].strides = _i64(r.strides, keep)
    d.refs = C.cast(refs, C.POINTER(stripe_refinement_t))
    d.intrinsic = _INTR[block.intrinsic] if block.intrinsic is not None else 0
    if block.child is not None:
        child = marshal(block.child, keep)
        keep.append(child)
        d.child = C.pointer(child)
    return d


def stripe_last_error() -> str:
    return lib.stripe_last_error().decode()


def stripe_status_string(status: int) -> str:
    return lib.stripe_status_string(int(status)).decode()


def _check(status: int):
    if status != STRIPE_OK:
        raise StripeError(status, stripe_last_error())


def stripe_block_create(block, path: str = "auto") -> C.c_void_p:
    keep: list = []
    desc = marshal(block, keep)
    h = C.c_void_p()
    if path == "auto":
        _check(lib.stripe_block_create(C.byref(desc), C.byref(h)))
    else:
        _check(lib.stripe_block_create_for_path(C.byref(desc), PATHS[path], C.byref(h)))
    return h


def stripe_block_run(handle, input_ptrs: Sequence[int], output_ptr: int, stream: int = 0) -> None:
    arr = (C.c_void_p * len(input_ptrs))(*[C.c_void_p(int(p)) for p in input_ptrs])
    _check(lib.stripe_block_run(handle, arr, C.c_void_p(int(output_ptr)), C.c_void_p(int(stream))))


def stripe_block_query(handle) -> dict:
    info = stripe_block_info_t()
    _check(lib.stripe_block_query(handle, C.byref(info)))
    out = {name: getattr(info, name) for name, _ in stripe_block_info_t._fields_}
    out["kernel"] = info.kernel.decode()
    out["path_name"] = PATH_NAMES.get(info.path, str(info.path))
    return out


def stripe_block_destroy(handle) -> None:
    lib.stripe_block_destroy(handle)


def stripe_device_copy(src_ptr: int, dst_ptr: int, n_bytes: int, stream: int = 0) -> None:
    _check(lib.stripe_device_copy(C.c_void_p(int(src_ptr)), C.c_void_p(int(dst_ptr)), C.c_size_t(int(n_bytes)),
                                  C.c_void_p(int(stream))))


class StripeBlock:
    """Owns one handle.  run() takes torch CUDA tensors (or raw device pointers)."""

    def __init__(self, block, path: str = "auto"):
        self.handle = stripe_block_create(block, path)
        self.info = stripe_block_query(self.handle)
        self._n_in = len(block.refs) - 1
        self._in_arr = (C.c_void_p * self._n_in)()      # reused on every run: marshalling cost matters for tiny blocks

    def run(self, inputs, output, stream: Optional[int] = None) -> None:
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        if len(inputs) != self._n_in:
            raise ValueError(f"expected {self._n_in} inputs")
        arr = self._in_arr
        for i, t in enumerate(inputs):
            arr[i] = t if isinstance(t, int) else t.data_ptr()
        out = output if isinstance(output, int) else output.data_ptr()
        st = lib.stripe_block_run(self.handle, arr, out, stream)
        if st != STRIPE_OK:
            raise StripeError(st, stripe_last_error())

    def close(self) -> None:
        if self.handle is not None:
            stripe_block_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
