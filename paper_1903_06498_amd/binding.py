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
                5: "ERR_ASSIGN_CONFLICT", 6: "ERR_HIP", 7: "ERR_NOMEM", 8: "ERR_MISALIGNED"}
PATHS = {"auto": 0, "generic": 1, "mfma_gemm": 2, "mfma_conv": 3, "pool": 4}
PATH_NAMES = {v: k for k, v in PATHS.items()}

_DIR = {"in": 0, "out": 1, "temp": 2}
_DTYPE = {"i8": 0, "i32": 1, "bf16": 2, "f32": 3}
_AGG = {"assign": 0, "add": 1, "max": 2, "min": 3, "mul": 4}
_INTR = {"mul": 0, "copy": 1, "add": 2, "add_relu": 3}

EXPORTS = ("stripe_block_create", "stripe_block_create_for_path", "stripe_block_run", "stripe_block_run_static", "stripe_block_query",
           "stripe_block_workspace_size", "stripe_block_set_workspace",
           "stripe_block_destroy", "stripe_status_string", "stripe_last_error", "stripe_device_copy", "stripe_device_stream", "stripe_device_mfma",
           "stripe_tile_cost", "stripe_tile_search", "stripe_block_tile", "stripe_desc_free")


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
    ("intrinsic", C.c_int), ("child", C.POINTER(stripe_block_desc_t)),
    ("next", C.POINTER(stripe_block_desc_t)), ("parent_refs", C.POINTER(C.c_int32))]


class stripe_block_info_t(C.Structure):
    _fields_ = [("path", C.c_int32), ("n_idx", C.c_int32), ("n_out_idx", C.c_int32), ("n_red_idx", C.c_int32),
                ("hull_points", C.c_int64), ("work_points", C.c_int64), ("output_elements", C.c_int64),
                ("algorithmic_bytes", C.c_int64),
                ("tile_m", C.c_int32), ("tile_n", C.c_int32), ("tile_k", C.c_int32),
                ("frag_m", C.c_int32), ("frag_n", C.c_int32), ("frag_k", C.c_int32),
                ("lds_bytes", C.c_int32), ("workgroup_size", C.c_int32), ("grid", C.c_int64),
                ("kernel", C.c_char * 96), ("workspace_bytes", C.c_int64)]


class stripe_tile_model_t(C.Structure):
    _fields_ = [("line_elems", C.c_int64), ("mem_cap_elems", C.c_int64), ("counted_refs", C.c_uint32),
                ("tiled_idx", C.c_uint32), ("power_of_two", C.c_int32), ("multiple_of", C.POINTER(C.c_int64))]


class stripe_tile_cost_t(C.Structure):
    _fields_ = [("tiles", C.c_int64), ("lines_per_tile", C.c_int64), ("footprint_elems", C.c_int64),
                ("work", C.c_int64), ("cost", C.c_double), ("admissible", C.c_int32)]


class StripeError(RuntimeError):
    def __init__(self, status: int, detail: str):
        super().__init__(f"stripe: {STATUS_NAMES.get(status, status)}: {detail}")
        self.status = status
        self.detail = detail


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_1903_06498_amd.build` "
                          "(there is no CPU fallback)")
    # PyTorch wheels bundle their own copy of the HIP runtime.  If this library pulled in the system's copy
    # first, a later `import torch` would bring a second runtime into the process and every GPU call would
    # fail ("no ROCm-capable device").  Loading torch first makes its runtime the one both sides share.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(LIB_PATH)
    handle = C.c_void_p
    lib.stripe_block_create.restype = C.c_int
    lib.stripe_block_create.argtypes = [C.POINTER(stripe_block_desc_t), C.POINTER(handle)]
    lib.stripe_block_create_for_path.restype = C.c_int
    lib.stripe_block_create_for_path.argtypes = [C.POINTER(stripe_block_desc_t), C.c_int, C.POINTER(handle)]
    lib.stripe_block_run.restype = C.c_int
    lib.stripe_block_run.argtypes = [handle, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]
    lib.stripe_block_run_static.restype = C.c_int
    lib.stripe_block_run_static.argtypes = [handle, C.POINTER(C.c_void_p), C.c_void_p, C.c_void_p]
    lib.stripe_block_query.restype = C.c_int
    lib.stripe_block_query.argtypes = [handle, C.POINTER(stripe_block_info_t)]
    lib.stripe_block_workspace_size.restype = C.c_int
    lib.stripe_block_workspace_size.argtypes = [handle, C.POINTER(C.c_size_t)]
    lib.stripe_block_set_workspace.restype = C.c_int
    lib.stripe_block_set_workspace.argtypes = [handle, C.c_void_p, C.c_size_t]
    lib.stripe_block_destroy.restype = None
    lib.stripe_block_destroy.argtypes = [handle]
    lib.stripe_status_string.restype = C.c_char_p
    lib.stripe_status_string.argtypes = [C.c_int]
    lib.stripe_last_error.restype = C.c_char_p
    lib.stripe_last_error.argtypes = []
    lib.stripe_device_copy.restype = C.c_int
    lib.stripe_device_copy.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_void_p]
    lib.stripe_device_mfma.restype = C.c_int
    lib.stripe_device_mfma.argtypes = [C.c_void_p, C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
    lib.stripe_device_stream.restype = C.c_int
    lib.stripe_device_stream.argtypes = [C.c_void_p, C.c_void_p, C.c_size_t, C.c_int, C.c_int, C.c_int, C.c_void_p]
    lib.stripe_tile_cost.restype = C.c_int
    lib.stripe_tile_cost.argtypes = [C.POINTER(stripe_block_desc_t), C.POINTER(C.c_int64), C.POINTER(stripe_tile_model_t),
                                     C.POINTER(stripe_tile_cost_t)]
    lib.stripe_tile_search.restype = C.c_int
    lib.stripe_tile_search.argtypes = [C.POINTER(stripe_block_desc_t), C.POINTER(stripe_tile_model_t), C.POINTER(C.c_int64),
                                       C.POINTER(stripe_tile_cost_t)]
    lib.stripe_block_tile.restype = C.c_int
    lib.stripe_block_tile.argtypes = [C.POINTER(stripe_block_desc_t), C.POINTER(C.c_int64),
                                      C.POINTER(C.POINTER(stripe_block_desc_t))]
    lib.stripe_desc_free.restype = None
    lib.stripe_desc_free.argtypes = [C.POINTER(stripe_block_desc_t)]
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
    nxt = getattr(block, "next", None)
    if nxt is not None:
        sibling = marshal(nxt, keep)
        keep.append(sibling)
        d.next = C.pointer(sibling)
    uses = getattr(block, "parent_refs", None)
    if uses is not None:
        arr = (C.c_int32 * len(uses))(*[int(v) for v in uses])
        keep.append(arr)
        d.parent_refs = C.cast(arr, C.POINTER(C.c_int32))
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


def stripe_block_run_static(handle, input_ptrs: Sequence[int], output_ptr: int, stream: int = 0) -> None:
    arr = (C.c_void_p * len(input_ptrs))(*[C.c_void_p(int(p)) for p in input_ptrs])
    _check(lib.stripe_block_run_static(handle, arr, C.c_void_p(int(output_ptr)), C.c_void_p(int(stream))))


def stripe_block_workspace_size(handle) -> int:
    n = C.c_size_t(0)
    _check(lib.stripe_block_workspace_size(handle, C.byref(n)))
    return int(n.value)


def stripe_block_set_workspace(handle, device_ptr: int, n_bytes: int) -> None:
    _check(lib.stripe_block_set_workspace(handle, C.c_void_p(int(device_ptr)), C.c_size_t(int(n_bytes))))


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


def stripe_device_stream(src_ptr: int, dst_ptr: int, n_vectors: int, reads: int, write: int, grid: int, stream: int = 0) -> None:
    _check(lib.stripe_device_stream(C.c_void_p(int(src_ptr)), C.c_void_p(int(dst_ptr)), C.c_size_t(int(n_vectors)), int(reads), int(write),
                                    int(grid), C.c_void_p(int(stream))))


def stripe_device_mfma(operands_ptr: int, out_ptr: int, iters: int, grid: int, stream: int = 0, from_lds: bool = False) -> None:
    _check(lib.stripe_device_mfma(C.c_void_p(int(operands_ptr)), C.c_void_p(int(out_ptr)), int(iters), int(bool(from_lds)), int(grid),
                                  C.c_void_p(int(stream))))


# ---- autotiling (host only) ------------------------------------------------
_DIR_NAMES = {v: k for k, v in _DIR.items()}
_DTYPE_NAMES = {v: k for k, v in _DTYPE.items()}
_AGG_NAMES = {v: k for k, v in _AGG.items()}
_INTR_NAMES = {v: k for k, v in _INTR.items()}


def _model(model: dict, n_idx: int, keep: list) -> stripe_tile_model_t:
    """model: dict(line_elems, mem_cap_elems=0, counted_refs=[ref numbers], tiled_idx=[index numbers],
    power_of_two=False, multiple_of=None or a list per index)."""
    m = stripe_tile_model_t()
    m.line_elems = int(model["line_elems"])
    m.mem_cap_elems = int(model.get("mem_cap_elems", 0))
    m.counted_refs = sum(1 << int(r) for r in model["counted_refs"])
    m.tiled_idx = sum(1 << int(j) for j in model["tiled_idx"])
    m.power_of_two = 1 if model.get("power_of_two") else 0
    mult = model.get("multiple_of")
    m.multiple_of = _i64(mult, keep) if mult is not None else None
    if mult is not None and len(mult) != n_idx:
        raise ValueError("multiple_of needs one entry per index")
    return m


def _cost_dict(c: stripe_tile_cost_t) -> dict:
    return {name: getattr(c, name) for name, _ in stripe_tile_cost_t._fields_}


def stripe_tile_cost(block, tile: Sequence[int], model: dict) -> dict:
    keep: list = []
    desc = marshal(block, keep)
    out = stripe_tile_cost_t()
    _check(lib.stripe_tile_cost(C.byref(desc), _i64(tile, keep), C.byref(_model(model, len(tile), keep)), C.byref(out)))
    return _cost_dict(out)


def stripe_tile_search(block, model: dict):
    keep: list = []
    desc = marshal(block, keep)
    n = len(block.child.ranges)
    best_tile = (C.c_int64 * n)()
    out = stripe_tile_cost_t()
    _check(lib.stripe_tile_search(C.byref(desc), C.byref(_model(model, n, keep)), best_tile, C.byref(out)))
    return list(best_tile), _cost_dict(out)


def unmarshal(desc: stripe_block_desc_t, parent_vars: int = 0, names=None):
    """C descriptor -> workloads.Block (index and buffer names are not part of the C form: generic ones)."""
    from .workloads import Block, Refinement
    n_vars = desc.n_idx + desc.n_passed

    def mat(ptr, n_rows, n_cols):
        return [[int(ptr[r * n_cols + c]) for c in range(n_cols)] for r in range(n_rows)]

    refs = []
    for i in range(desc.n_refs):
        r = desc.refs[i]
        refs.append(Refinement(name=(names[i] if names else f"T{i}"), dir=_DIR_NAMES[r.dir], dtype=_DTYPE_NAMES[r.dtype],
                               agg=_AGG_NAMES[r.agg], access_coeff=mat(r.access_coeff, r.ndim, n_vars),
                               access_const=[int(r.access_const[d]) for d in range(r.ndim)],
                               sizes=[int(r.sizes[d]) for d in range(r.ndim)], strides=[int(r.strides[d]) for d in range(r.ndim)]))
    child = unmarshal(desc.child.contents, n_vars, names) if desc.child else None
    return Block(idx_names=[f"i{j}" for j in range(desc.n_idx)], ranges=[int(desc.ranges[j]) for j in range(desc.n_idx)],
                 passed_names=[f"p{j}" for j in range(desc.n_passed)], passed_coeff=mat(desc.passed_coeff, desc.n_passed, parent_vars),
                 passed_const=[int(desc.passed_const[j]) for j in range(desc.n_passed)],
                 cons_coeff=mat(desc.cons_coeff, desc.n_constraints, n_vars),
                 cons_const=[int(desc.cons_const[j]) for j in range(desc.n_constraints)], refs=refs,
                 intrinsic=_INTR_NAMES[desc.intrinsic] if child is None else None, child=child)


def stripe_block_tile(block, tile: Sequence[int]):
    """The tiling rewrite; returns the nest as a workloads.Block (the C result is freed before returning)."""
    keep: list = []
    desc = marshal(block, keep)
    out = C.POINTER(stripe_block_desc_t)()
    _check(lib.stripe_block_tile(C.byref(desc), _i64(tile, keep), C.byref(out)))
    try:
        return unmarshal(out.contents, 0, [r.name for r in block.refs])
    finally:
        lib.stripe_desc_free(out)


def stripe_desc_free(desc_ptr) -> None:
    lib.stripe_desc_free(desc_ptr)


class StripeBlock:
    """Owns one handle.  run() takes torch CUDA tensors (or raw device pointers)."""

    def __init__(self, block, path: str = "auto"):
        self.handle = stripe_block_create(block, path)
        self.info = stripe_block_query(self.handle)
        self._n_in = sum(1 for r in block.refs if r.dir == "in")
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

    def run_static(self, inputs, output, stream: Optional[int] = None) -> None:
        """As run(), through stripe_block_run_static: temporaries in the library's static scratch array."""
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        if len(inputs) != self._n_in:
            raise ValueError(f"expected {self._n_in} inputs")
        arr = self._in_arr
        for i, t in enumerate(inputs):
            arr[i] = t if isinstance(t, int) else t.data_ptr()
        out = output if isinstance(output, int) else output.data_ptr()
        st = lib.stripe_block_run_static(self.handle, arr, out, stream)
        if st != STRIPE_OK:
            raise StripeError(st, stripe_last_error())

    def set_workspace(self, tensor) -> None:
        """Hand the handle a caller-owned device workspace (a torch CUDA tensor, kept alive here), or None."""
        self._ws = tensor
        if tensor is None:
            stripe_block_set_workspace(self.handle, 0, 0)
        else:
            stripe_block_set_workspace(self.handle, tensor.data_ptr(), tensor.numel() * tensor.element_size())

    def close(self) -> None:
        if self.handle is not None:
            stripe_block_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
