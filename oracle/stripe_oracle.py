"""Python face of the Stripe block oracle -- TEST INFRASTRUCTURE, not the product.

Marshals a block description (any object with the attributes used below:
idx_names, ranges, passed_*, cons_*, refs, intrinsic, child) into the C
oracle's structs and runs it.  Nothing here or in the C file is shared with,
or imported from, the GPU library and its binding.

Threads: evaluate(..., threads=T, split_index=j) cuts the range of index j of
the first block level into T windows and runs the C oracle on each in its own
thread, every thread with a private result image.  The images are merged
afterwards and the merge fails if two windows touched the same output
element, i.e. if j was not an index the output address depends on
injectively.  Within one output element the order of aggregation is the same
as in a single-threaded run.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
import threading
from typing import List, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libstripe_oracle.so")

_DIR = {"in": 0, "out": 1}
_DTYPE = {"i8": 0, "i32": 1, "bf16": 2, "f32": 3}
_NP_DTYPE = {"i8": np.int8, "i32": np.int32, "bf16": np.uint16, "f32": np.float32}
_AGG = {"assign": 0, "add": 1, "max": 2, "min": 3, "mul": 4}
_INTR = {"mul": 0, "copy": 1, "add": 2, "add_relu": 3}

ERR_NAMES = {1: "bad block", 2: "out of bounds", 3: "assign conflict", 4: "int32 overflow"}


class OracleError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"oracle: {ERR_NAMES.get(code, code)}: {msg}")
        self.code = code


class _Ref(C.Structure):
    _fields_ = [("dir", C.c_int32), ("dtype", C.c_int32), ("agg", C.c_int32), ("ndim", C.c_int32),
                ("access_coeff", C.POINTER(C.c_int64)), ("access_const", C.POINTER(C.c_int64)),
                ("sizes", C.POINTER(C.c_int64)), ("strides", C.POINTER(C.c_int64))]


class _Block(C.Structure):
    pass


_Block._fields_ = [("n_idx", C.c_int32), ("ranges", C.POINTER(C.c_int64)),
                   ("n_passed", C.c_int32), ("passed_coeff", C.POINTER(C.c_int64)),
                   ("passed_const", C.POINTER(C.c_int64)),
                   ("n_cons", C.c_int32), ("cons_coeff", C.POINTER(C.c_int64)),
                   ("cons_const", C.POINTER(C.c_int64)),
                   ("n_refs", C.c_int32), ("refs", C.POINTER(_Ref)),
                   ("intrinsic", C.c_int32), ("child", C.POINTER(_Block))]


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (building the checker is not using it)."""
    src = os.path.join(_HERE, "stripe_oracle.c")
    hdr = os.path.join(_HERE, "stripe_oracle.h")
    if force or not os.path.exists(_LIB_PATH) or \
            os.path.getmtime(_LIB_PATH) < max(os.path.getmtime(src), os.path.getmtime(hdr)):
        subprocess.check_call(["gcc", "-O2", "-Wall", "-Wextra", "-fPIC", "-shared", "-o", _LIB_PATH, src])
    return _LIB_PATH


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB_PATH)
        lib.so_output_extent.restype = C.c_int64
        lib.so_output_extent.argtypes = [C.POINTER(_Block)]
        lib.so_eval.restype = C.c_int
        lib.so_eval.argtypes = [C.POINTER(_Block), C.POINTER(C.c_void_p), C.POINTER(C.c_double),
                                C.POINTER(C.c_int64), C.POINTER(C.c_uint8), C.POINTER(C.c_int64),
                                C.POINTER(C.c_int64), C.POINTER(C.c_int64), C.c_char_p, C.c_size_t]
        _lib = lib
    return _lib


def _i64(values, keep) -> "C.POINTER(C.c_int64)":
    flat = [int(v) for v in values]
    arr = (C.c_int64 * max(1, len(flat)))(*flat)
    keep.append(arr)
    return C.cast(arr, C.POINTER(C.c_int64))


def _marshal(block, keep: list) -> _Block:
    """Nested description -> chain of C structs (kept alive through `keep`)."""
    cb = _Block()
    nv = len(block.idx_names) + len(block.passed_names)
    cb.n_idx = len(block.idx_names)
    cb.ranges = _i64(block.ranges, keep)
    cb.n_passed = len(block.passed_names)
    cb.passed_coeff = _i64([v for row in block.passed_coeff for v in row], keep)
    cb.passed_const = _i64(block.passed_const, keep)
    cb.n_cons = len(block.cons_coeff)
    for row in block.cons_coeff:
        assert len(row) == nv
    cb.cons_coeff = _i64([v for row in block.cons_coeff for v in row], keep)
    cb.cons_const = _i64(block.cons_const, keep)
    cb.n_refs = len(block.refs)
    refs = (_Ref * max(1, len(block.refs)))()
    keep.append(refs)
    for i, r in enumerate(block.refs):
        refs[i].dir = _DIR[r.dir]
        refs[i].dtype = _DTYPE[r.dtype]
        refs[i].agg = _AGG[r.agg]
        refs[i].ndim = len(r.sizes)
        for row in r.access_coeff:
            assert len(row) == nv
        refs[i].access_coeff = _i64([v for row in r.access_coeff for v in row], keep)
        refs[i].access_const = _i64(r.access_const, keep)
        refs[i].sizes = _i64(r.sizes, keep)
        refs[i].strides = _i64(r.strides, keep)
    cb.refs = C.cast(refs, C.POINTER(_Ref))
    cb.intrinsic = _INTR[block.intrinsic] if block.intrinsic is not None else 0
    if block.child is not None:
        child = _marshal(block.child, keep)
        keep.append(child)
        cb.child = C.pointer(child)
    return cb


def output_extent(root) -> int:
    keep: list = []
    cb = _marshal(root, keep)
    return int(_load().so_output_extent(C.byref(cb)))


class Result:
    """out: fp64 (float blocks) or int64 (integer blocks) image of the output
    buffer, flat, addressed in elements; touched: 1 where an iteration wrote;
    n_points: leaf points executed."""

    def __init__(self, out, touched, n_points):
        self.out, self.touched, self.n_points = out, touched, n_points


def _eval_once(cb, in_ptrs, is_int, out, touched, win):
    lib = _load()
    err = C.create_string_buffer(256)
    npts = C.c_int64(0)
    lo = hi = None
    if win is not None:
        lo = (C.c_int64 * len(win[0]))(*[int(v) for v in win[0]])
        hi = (C.c_int64 * len(win[1]))(*[int(v) for v in win[1]])
    rc = lib.so_eval(C.byref(cb), in_ptrs,
                     None if is_int else out.ctypes.data_as(C.POINTER(C.c_double)),
                     out.ctypes.data_as(C.POINTER(C.c_int64)) if is_int else None,
                     touched.ctypes.data_as(C.POINTER(C.c_uint8)), lo, hi, C.byref(npts), err, 256)
    return rc, err.value.decode(), int(npts.value)


def statements(root) -> list:
    """The statement list of the root block (Section 3.2: a block's statements execute as if in serial)."""
    out, s = [], root.child
    while s is not None:
        out.append(s)
        s = getattr(s, "next", None)
    return out


def evaluate_program(root, inputs: Sequence[np.ndarray], out: Optional[np.ndarray] = None, threads: int = 1) -> Result:
    """A root block with several statements and temporaries ('temp' refinements of the root).

    The statements run one after the other, each evaluated exactly like a single block.  A statement names the
    root buffers it uses through `parent_refs`.  What a statement writes is stored in the buffer's declared
    element type (a temporary declared f32 holds the fp64 result rounded to fp32; integers stay exact), and later
    statements read that.  The result returned is the last statement's: the program's output, in fp64 / int64,
    not yet rounded to the output buffer's type."""
    import copy
    stmts = statements(root)
    held = {}                      # root refinement number -> array in its declared element type
    it = iter(inputs)
    for j, r in enumerate(root.refs):
        if r.dir == "in":
            held[j] = np.ascontiguousarray(next(it))
    res = None
    for si, st in enumerate(stmts):
        uses = list(st.parent_refs) if getattr(st, "parent_refs", None) is not None else list(range(len(st.refs)))
        sub_refs = []
        for lr, j in zip(st.refs, uses):
            rr = copy.copy(root.refs[j])
            rr.dir = lr.dir                    # a temporary is 'out' for the statement that writes it, 'in' later
            sub_refs.append(rr)
        single = copy.copy(st)
        single.next = None
        single.parent_refs = None
        sub_root = type(root)(idx_names=[], ranges=[], refs=sub_refs, child=single)
        ins = []
        for lr, j in zip(st.refs[:-1], uses[:-1]):
            if j not in held:
                raise OracleError(1, f"statement {si} reads root buffer {j} before anything wrote it")
            ins.append(held[j])
        last = si == len(stmts) - 1
        res = evaluate(sub_root, ins, out=out if last else None, threads=threads)
        jo = uses[-1]
        odt = root.refs[jo].dtype
        if not last:
            if not res.touched.all():
                raise OracleError(1, f"statement {si} leaves elements of temporary {jo} unwritten")
            if odt == "f32":
                held[jo] = res.out.astype(np.float32)
            elif odt == "i32":
                held[jo] = res.out.astype(np.int32)
            else:
                raise OracleError(1, "temporaries are f32 or i32")
    return res


def evaluate(root, inputs: Sequence[np.ndarray], out: Optional[np.ndarray] = None,
             window: Optional[Sequence[Sequence[int]]] = None, threads: int = 1,
             split_index: int = 0) -> Result:
    """Run the oracle.  inputs: numpy arrays in the declared element types
    (bf16 as uint16 bit patterns).  out: optional pre-filled image (fp64/int64,
    extent elements) whose untouched elements are kept; default zeros.
    window: (lo[], hi[]) per index of the first block level."""
    keep: list = []
    cb = _marshal(root, keep)
    ext = int(_load().so_output_extent(C.byref(cb)))
    if ext < 1:
        raise OracleError(1, "bad output declaration")
    is_int = root.refs[-1].dtype == "i32"
    arrs: List[np.ndarray] = []
    for r, a in zip(root.refs[:-1], inputs):
        a = np.ascontiguousarray(a)
        if a.dtype != _NP_DTYPE[r.dtype]:
            raise TypeError(f"input {r.name}: expected {_NP_DTYPE[r.dtype]}, got {a.dtype}")
        need = sum((c + n - 1) * s for c, n, s in zip(r.access_const, r.sizes, r.strides)) + 1
        if a.size < need:
            raise ValueError(f"input {r.name}: {a.size} elements, the declaration needs {need}")
        arrs.append(a)
    if len(arrs) != len(root.refs) - 1:
        raise ValueError("one array per input refinement")
    in_ptrs = (C.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])
    odt = np.int64 if is_int else np.float64
    if out is None:
        out = np.zeros(ext, dtype=odt)
    else:
        if out.dtype != odt or out.size != ext or not out.flags.c_contiguous:
            raise ValueError("out must be a flat contiguous image of the output buffer")
        out = out.reshape(-1)
    touched = np.zeros(ext, dtype=np.uint8)
    first = root.child
    full = ([0] * len(first.ranges), list(first.ranges))
    if window is None:
        window = full
    window = ([int(v) for v in window[0]], [int(v) for v in window[1]])

    span = window[1][split_index] - window[0][split_index] if first.ranges else 0
    threads = max(1, min(int(threads), span)) if first.ranges else 1
    if threads == 1:
        rc, msg, npts = _eval_once(cb, in_ptrs, is_int, out, touched, window)
        if rc:
            raise OracleError(rc, msg)
        return Result(out, touched, npts)

    cuts = [window[0][split_index] + (span * t) // threads for t in range(threads + 1)]
    results = [None] * threads
    outs = [np.zeros(ext, dtype=odt) for _ in range(threads)]
    tchs = [np.zeros(ext, dtype=np.uint8) for _ in range(threads)]

    def work(t):
        lo, hi = list(window[0]), list(window[1])
        lo[split_index], hi[split_index] = cuts[t], cuts[t + 1]
        results[t] = _eval_once(cb, in_ptrs, is_int, outs[t], tchs[t], (lo, hi))

    ths = [threading.Thread(target=work, args=(t,)) for t in range(threads)]
    for th in ths:
        th.start()
    for th in ths:
        th.join()
    npts = 0
    for t in range(threads):
        rc, msg, n = results[t]
        if rc:
            raise OracleError(rc, msg)
        npts += n
        if np.any(touched & tchs[t]):
            raise OracleError(3, "two thread windows wrote the same element: split on an output index")
        sel = tchs[t].astype(bool)
        out[sel] = outs[t][sel]
        touched |= tchs[t]
    return Result(out, touched, npts)
