"""Block descriptions and seeded synthetic inputs.

This module holds DATA only: how a Stripe block is written down (index names
and ranges, affine constraints, refinements with affine accesses, sizes and
strides, the leaf intrinsic, the aggregation operation; paper Section 3.2 and
Figure 5) and how the synthetic input tensors of the benchmark configurations
are drawn.  It evaluates nothing: no point of an iteration space is visited
here and no element of a result is computed.  Both the GPU binding and the
test oracle are fed from these descriptions; neither is imported here.
"""
from __future__ import annotations

import re
from dataclasses import dataclass, field
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

DTYPES = ("i8", "i32", "bf16", "f32")
AGGS = ("assign", "add", "max", "min", "mul")
INTRINSICS = ("mul", "copy", "add", "add_relu")


@dataclass
class Refinement:
    """A buffer as one nesting level sees it (Section 3.2, "refinements")."""
    name: str
    dir: str                       # "in" | "out"
    dtype: str                     # one of DTYPES
    agg: str                       # one of AGGS; meaningful for the output
    access_coeff: List[List[int]]  # [ndim][n_idx + n_passed]
    access_const: List[int]        # [ndim]
    sizes: List[int]               # extent of the view handed on (root: the buffer; leaf: 1s)
    strides: List[int]             # elements


@dataclass
class Block:
    """One nesting level.  Variables = own indexes, then passed parent values."""
    idx_names: List[str]
    ranges: List[int]
    passed_names: List[str] = field(default_factory=list)
    passed_coeff: List[List[int]] = field(default_factory=list)  # over the parent's variables
    passed_const: List[int] = field(default_factory=list)
    cons_coeff: List[List[int]] = field(default_factory=list)
    cons_const: List[int] = field(default_factory=list)
    refs: List[Refinement] = field(default_factory=list)
    intrinsic: Optional[str] = None   # leaf only
    child: Optional["Block"] = None
    next: Optional["Block"] = None    # next statement of the parent's statement list (statements run in order)
    parent_refs: Optional[List[int]] = None   # which parent refinement each of `refs` refines; None: same positions

    @property
    def var_names(self) -> List[str]:
        return list(self.idx_names) + list(self.passed_names)

    def levels(self) -> List["Block"]:
        out, b = [], self
        while b is not None:
            out.append(b)
            b = b.child
        return out


# --------------------------------------------------------------------------
# Writing affine expressions as text: "x + i - 1", "12 - x - i", "3*x".
# --------------------------------------------------------------------------
_TOKEN = re.compile(r"\s*(?:(\d+)|([A-Za-z_][A-Za-z_0-9]*)|([+\-*]))")


def parse_affine(expr: str, var_names: Sequence[str]) -> Tuple[List[int], int]:
    """Split an affine expression into one coefficient per variable and a constant."""
    coeff = {v: 0 for v in var_names}
    const = 0
    pos, sign = 0, 1
    text = expr.strip()
    if text == "":
        raise ValueError("empty affine expression")
    pending_num: Optional[int] = None
    expect_term = True
    while pos < len(text):
        m = _TOKEN.match(text, pos)
        if not m:
            raise ValueError(f"cannot read affine expression {expr!r} at {pos}")
        pos = m.end()
        num, name, op = m.groups()
        if op in ("+", "-"):
            if pending_num is not None:
                const += sign * pending_num
                pending_num = None
            sign = 1 if op == "+" else -1
            expect_term = True
        elif op == "*":
            if pending_num is None:
                raise ValueError(f"'*' needs a number on its left in {expr!r}")
        elif num is not None:
            pending_num = int(num)
            expect_term = False
        else:
            if name not in coeff:
                raise ValueError(f"unknown variable {name!r} in {expr!r}")
            coeff[name] += sign * (pending_num if pending_num is not None else 1)
            pending_num = None
            expect_term = False
    if pending_num is not None:
        const += sign * pending_num
    if expect_term:
        raise ValueError(f"dangling operator in {expr!r}")
    return [coeff[v] for v in var_names], const


def contiguous_strides(sizes: Sequence[int]) -> List[int]:
    strides, s = [], 1
    for n in reversed(list(sizes)):
        strides.append(s)
        s *= int(n)
    return list(reversed(strides))


@dataclass
class Buffer:
    """A buffer declaration of the root block (Figure 5: 'in I[0,0,0] i8(12,16,8):(128,8,1)')."""
    name: str
    dir: str
    dtype: str
    sizes: Sequence[int]
    strides: Optional[Sequence[int]] = None
    agg: str = "assign"


def make_level(idx: Dict[str, int], refs: Sequence[Tuple], *, buffers: Sequence[Buffer],
               constraints: Sequence[str] = (), passed: Optional[Dict[str, str]] = None,
               parent: Optional[Block] = None, intrinsic: Optional[str] = None,
               child: Optional[Block] = None) -> Block:
    """Write one level.

    refs: one tuple per buffer, in the buffers' order: (accesses, agg) or
    (accesses, agg, sizes); accesses is a list of affine texts, one per
    dimension, in this level's variables.  sizes default to all 1 (scalar
    views, as at a leaf).  constraints are texts "expr >= 0".  passed maps a
    new name to an affine text in the PARENT's variables.
    """
    passed = passed or {}
    idx_names, ranges = list(idx.keys()), [int(v) for v in idx.values()]
    b = Block(idx_names=idx_names, ranges=ranges, passed_names=list(passed.keys()))
    if passed:
        if parent is None:
            raise ValueError("passed values need the parent level")
        for text in passed.values():
            co, c0 = parse_affine(text, parent.var_names)
            b.passed_coeff.append(co)
            b.passed_const.append(c0)
    vn = b.var_names
    for text in constraints:
        lhs = text.replace(" ", "")
        if not lhs.endswith(">=0"):
            raise ValueError(f"constraint must read 'expr >= 0': {text!r}")
        co, c0 = parse_affine(lhs[:-3], vn)
        b.cons_coeff.append(co)
        b.cons_const.append(c0)
    if len(refs) != len(buffers):
        raise ValueError("one refinement per declared buffer")
    for buf, r in zip(buffers, refs):
        accesses, agg = r[0], r[1]
        sizes = list(r[2]) if len(r) > 2 else [1] * len(buf.sizes)
        if len(accesses) != len(buf.sizes):
            raise ValueError(f"{buf.name}: one access per dimension")
        cos, c0s = [], []
        for a in accesses:
            co, c0 = parse_affine(str(a), vn)
            cos.append(co)
            c0s.append(c0)
        strides = list(buf.strides) if buf.strides is not None else contiguous_strides(buf.sizes)
        b.refs.append(Refinement(buf.name, buf.dir, buf.dtype, agg, cos, c0s, [int(s) for s in sizes], strides))
    b.intrinsic = intrinsic
    b.child = child
    return b


def make_root(buffers: Sequence[Buffer], child: Block) -> Block:
    """The declaring root block: no indexes, one iteration (Figure 5, 'block []:1')."""
    root = Block(idx_names=[], ranges=[])
    for buf in buffers:
        nd = len(buf.sizes)
        strides = list(buf.strides) if buf.strides is not None else contiguous_strides(buf.sizes)
        root.refs.append(Refinement(buf.name, buf.dir, buf.dtype, buf.agg, [[] for _ in range(nd)],
                                    [0] * nd, [int(s) for s in buf.sizes], strides))
    root.child = child
    return root


def embed(root: Block, origins: Sequence[Sequence[int]], parent_sizes: Sequence[Sequence[int]]) -> Block:
    """Declare every buffer of `root` as a window of a larger, contiguous tensor: buffer r starts at coordinate
    origins[r] of a tensor of extents parent_sizes[r].  The root refinement then carries that origin as its
    constant (Figure 5 writes it 'in I[0, 0, 0]' for a window at the tensor's own origin) and every level the parent
    tensor's strides; the declared sizes stay the window's.  The arrays handed to an evaluator are the parents."""
    for r, (org, psz) in enumerate(zip(origins, parent_sizes)):
        top = root.refs[r]
        if len(org) != len(top.sizes) or len(psz) != len(top.sizes):
            raise ValueError(f"{top.name}: one origin and one parent extent per dimension")
        if any(o < 0 or o + n > p for o, n, p in zip(org, top.sizes, psz)):
            raise ValueError(f"{top.name}: the window leaves its parent tensor")
        strides = contiguous_strides(psz)
        for lv in root.levels():
            lv.refs[r].strides = list(strides)
        top.access_const = [int(o) for o in org]
    return root


def flat_block(buffers: Sequence[Buffer], idx: Dict[str, int], refs: Sequence[Tuple],
               constraints: Sequence[str] = (), intrinsic: str = "mul") -> Block:
    """A root declaration with one un-nested block below it (Figure 5a's shape)."""
    leaf = make_level(idx, refs, buffers=buffers, constraints=constraints, intrinsic=intrinsic)
    return make_root(buffers, leaf)


# --------------------------------------------------------------------------
# The shapes the benchmark configurations are made of.
# --------------------------------------------------------------------------
def conv2d_block(N, H, W, Ci, Co, R, S, stride, pad, in_dtype, out_dtype, filter_layout="RSKC") -> Block:
    """NHWC cross-correlation O[n,y,x,k] += I[n, s*y+i-p, s*x+j-p, c] * F[i,j,k,c].

    Padding is not materialised: taps that would read outside the input are
    removed from the iteration space by four affine constraints (Section 3.2,
    last paragraph but one; Figure 5a).  filter_layout "RSKC" is the layout
    of Figure 5 (F[i,j,k,c], c innermost); "RSCK" has k innermost.
    """
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    fsz = (R, S, Co, Ci) if filter_layout == "RSKC" else (R, S, Ci, Co)
    facc = ["i", "j", "k", "c"] if filter_layout == "RSKC" else ["i", "j", "c", "k"]
    bufs = [Buffer("I", "in", in_dtype, (N, H, W, Ci)), Buffer("F", "in", in_dtype, fsz),
            Buffer("O", "out", out_dtype, (N, Ho, Wo, Co))]
    s, p = stride, pad
    ya = f"{s}*y + i - {p}"
    xa = f"{s}*x + j - {p}"
    cons = [f"{ya} >= 0", f"{H - 1 + p} - {s}*y - i >= 0", f"{xa} >= 0", f"{W - 1 + p} - {s}*x - j >= 0"]
    return flat_block(bufs, dict(n=N, y=Ho, x=Wo, i=R, j=S, c=Ci, k=Co),
                      [(["n", ya, xa, "c"], "assign"), (facc, "assign"), (["n", "y", "x", "k"], "add")],
                      constraints=cons, intrinsic="mul")


def matmul_block(M, N, K, in_dtype, out_dtype, b_transposed=False) -> Block:
    """C[m,n] += A[m,k] * B[k,n], all row-major, no constraints.  With b_transposed the second operand is
    stored as [n][k] (C = A * B^T, the layout of a Linear layer's weights)."""
    bufs = [Buffer("A", "in", in_dtype, (M, K)), Buffer("B", "in", in_dtype, (N, K) if b_transposed else (K, N)),
            Buffer("C", "out", out_dtype, (M, N))]
    return flat_block(bufs, dict(m=M, n=N, k=K),
                      [(["m", "k"], "assign"), (["n", "k"] if b_transposed else ["k", "n"], "assign"), (["m", "n"], "add")],
                      intrinsic="mul")


def batched_matmul_block(batch, M, N, K, in_dtype, out_dtype, b_transposed=False, shared_b=False) -> Block:
    """C[b,m,n] += A[b,m,k] * B[b,k,n]: a batch of independent products (with shared_b every product uses one B)."""
    bshape = (N, K) if b_transposed else (K, N)
    bacc = ["n", "k"] if b_transposed else ["k", "n"]
    bufs = [Buffer("A", "in", in_dtype, (batch, M, K)), Buffer("B", "in", in_dtype, bshape if shared_b else (batch,) + bshape),
            Buffer("C", "out", out_dtype, (batch, M, N))]
    return flat_block(bufs, dict(b=batch, m=M, n=N, k=K),
                      [(["b", "m", "k"], "assign"), (bacc if shared_b else ["b"] + bacc, "assign"), (["b", "m", "n"], "add")],
                      intrinsic="mul")


def maxpool_block(N, H, W, C, R, stride, pad, dtype="f32", agg="max") -> Block:
    """O[n,y,x,c] = max (or another aggregation) over in-bounds taps of I[n, s*y+i-p, s*x+j-p, c]; body load -> store."""
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - R) // stride + 1
    bufs = [Buffer("I", "in", dtype, (N, H, W, C)), Buffer("O", "out", dtype, (N, Ho, Wo, C))]
    s, p = stride, pad
    ya = f"{s}*y + i - {p}"
    xa = f"{s}*x + j - {p}"
    cons = [f"{ya} >= 0", f"{H - 1 + p} - {s}*y - i >= 0", f"{xa} >= 0", f"{W - 1 + p} - {s}*x - j >= 0"]
    return flat_block(bufs, dict(n=N, y=Ho, x=Wo, c=C, i=R, j=R),
                      [(["n", ya, xa, "c"], "assign"), (["n", "y", "x", "c"], agg)],
                      constraints=cons, intrinsic="copy")


def depthwise_conv_block(N, H, W, C, R, S, stride, pad, dtype="f32", dilation=1) -> Block:
    """O[n,y,x,c] += I[n, s*y + d*i - p, s*x + d*j - p, c] * F[i,j,c]: a convolution without a reduction over channels
    (every channel has its own R x S filter); the same affine-access block shape as any other (Section 3.2)."""
    d = dilation
    Ho = (H + 2 * pad - d * (R - 1) - 1) // stride + 1
    Wo = (W + 2 * pad - d * (S - 1) - 1) // stride + 1
    out_dtype = "i32" if dtype in ("i8", "i32") else "f32"
    bufs = [Buffer("I", "in", dtype, (N, H, W, C)), Buffer("F", "in", dtype, (R, S, C)), Buffer("O", "out", out_dtype, (N, Ho, Wo, C))]
    ya, xa = f"{stride}*y + {d}*i - {pad}", f"{stride}*x + {d}*j - {pad}"
    cons = [f"{ya} >= 0", f"{H - 1 + pad} - {stride}*y - {d}*i >= 0", f"{xa} >= 0", f"{W - 1 + pad} - {stride}*x - {d}*j >= 0"]
    return flat_block(bufs, dict(n=N, y=Ho, x=Wo, c=C, i=R, j=S),
                      [(["n", ya, xa, "c"], "assign"), (["i", "j", "c"], "assign"), (["n", "y", "x", "c"], "add")],
                      constraints=cons, intrinsic="mul")


def avgpool_block(N, H, W, C, R, stride, pad, dtype="f32") -> Block:
    """Average pooling as sum aggregation of scaled taps: O[n,y,x,c] += I[n, s*y+i-p, s*x+j-p, c] * K[0], the scale
    1/(R*R) held in a one-element buffer K.  Taps outside the image are removed by the constraints, so a border
    window sums fewer taps but is scaled like an interior one."""
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - R) // stride + 1
    bufs = [Buffer("I", "in", dtype, (N, H, W, C)), Buffer("K", "in", dtype, (1,)), Buffer("O", "out", "f32", (N, Ho, Wo, C))]
    ya, xa = f"{stride}*y + i - {pad}", f"{stride}*x + j - {pad}"
    cons = [f"{ya} >= 0", f"{H - 1 + pad} - {stride}*y - i >= 0", f"{xa} >= 0", f"{W - 1 + pad} - {stride}*x - j >= 0"]
    return flat_block(bufs, dict(n=N, y=Ho, x=Wo, c=C, i=R, j=R),
                      [(["n", ya, xa, "c"], "assign"), (["0"], "assign"), (["n", "y", "x", "c"], "add")],
                      constraints=cons, intrinsic="mul")


# --------------------------------------------------------------------------
# The paper's worked example (Figure 5): a 3x3 convolution over a 12x16
# spatial extent, 8 -> 16 channels, before and after the 3x4 output tiling.
# Element types follow the benchmark contract: i8 inputs, i32 accumulation.
# The printed upper bound of the second spatial index in the un-tiled form
# ("12 - y - j") is read as "16 - y - j": the index has range 16 and the tiled
# form prints 16.
# --------------------------------------------------------------------------
def _fig5_buffers(out_dtype="i32", in_dtype="i8"):
    return [Buffer("I", "in", in_dtype, (12, 16, 8), (128, 8, 1)),
            Buffer("F", "in", in_dtype, (3, 3, 16, 8), (384, 128, 8, 1)),
            Buffer("O", "out", out_dtype, (12, 16, 16), (256, 16, 1), agg="assign")]


def fig5_flat(in_dtype="i8", out_dtype="i32", printed_typo=False) -> Block:
    bufs = _fig5_buffers(out_dtype, in_dtype)
    ymax = 12 if printed_typo else 16
    return flat_block(bufs, dict(x=12, y=16, i=3, j=3, c=8, k=16),
                      [(["x+i-1", "y+j-1", "c"], "assign"), (["i", "j", "k", "c"], "assign"),
                       (["x", "y", "k"], "add")],
                      constraints=["-1 + x + i >= 0", "12 - x - i >= 0", "-1 + y + j >= 0", f"{ymax} - y - j >= 0"],
                      intrinsic="mul")


def fig5_tiled(in_dtype="i8", out_dtype="i32") -> Block:
    bufs = _fig5_buffers(out_dtype, in_dtype)
    outer = make_level(dict(x=4, y=4, i=1, j=1, c=1, k=1),
                       [(["3*x - 1", "4*y - 1", "0"], "assign", (5, 6, 8)),
                        (["0", "0", "0", "0"], "assign", (3, 3, 16, 8)),
                        (["3*x", "4*y", "0"], "add", (3, 4, 16))], buffers=bufs)
    inner = make_level(dict(x=3, y=4, i=3, j=3, c=8, k=16),
                       [(["x + i", "y + j", "c"], "assign"), (["i", "j", "k", "c"], "assign"),
                        (["x", "y", "k"], "add")],
                       buffers=bufs, passed=dict(xo="3*x", yo="4*y"), parent=outer,
                       constraints=["-1 + xo + x + i >= 0", "12 - xo - x - i >= 0",
                                    "-1 + yo + y + j >= 0", "16 - yo - y - j >= 0"],
                       intrinsic="mul")
    outer.child = inner
    return make_root(bufs, outer)


# --------------------------------------------------------------------------
# The five benchmark configurations and their seeded inputs.
# --------------------------------------------------------------------------
CONFIG_NAMES = ("tiny_conv_f32", "gemm_bf16_4096", "resnet_conv_bf16", "conv7x7_s2_int8", "maxpool_f32")


def config_block(name: str) -> Block:
    if name == "tiny_conv_f32":
        return conv2d_block(1, 16, 16, 8, 16, 3, 3, 1, 1, "f32", "f32")
    if name == "gemm_bf16_4096":
        return matmul_block(4096, 4096, 4096, "bf16", "f32")
    if name == "resnet_conv_bf16":
        return conv2d_block(32, 56, 56, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    if name == "conv7x7_s2_int8":
        return conv2d_block(16, 224, 224, 3, 64, 7, 7, 2, 3, "i8", "i32")
    if name == "maxpool_f32":
        return maxpool_block(32, 112, 112, 64, 3, 2, 1, "f32")
    raise KeyError(name)


def conv_bias_relu_program(N, H, W, Ci, Co, R, S, stride, pad, in_dtype="bf16", out_dtype="bf16") -> Block:
    """Two statements under one root (Section 3.2: statements run as if in serial; Section 2.3: fusion and
    scalarisation are what an implementation may do with them):
        0:  T[n,y,x,k] += I[n, s*y+i-p, s*x+j-p, c] * F[i,j,k,c]      (T: an f32 temporary of the root)
        1:  O[n,y,x,k]  = relu(T[n,y,x,k] + B[k])
    Root buffers, in order: I, F, B (inputs), T (temporary), O (output).  Integer inputs give an i32 temporary,
    bias and output."""
    acc = "i32" if in_dtype in ("i8", "i32") else "f32"
    if acc == "i32":
        out_dtype = "i32"
    Ho = (H + 2 * pad - R) // stride + 1
    Wo = (W + 2 * pad - S) // stride + 1
    bufs = [Buffer("I", "in", in_dtype, (N, H, W, Ci)), Buffer("F", "in", in_dtype, (R, S, Co, Ci)),
            Buffer("B", "in", acc, (Co,)), Buffer("T", "temp", acc, (N, Ho, Wo, Co)),
            Buffer("O", "out", out_dtype, (N, Ho, Wo, Co))]
    s_, p_ = stride, pad
    ya, xa = f"{s_}*y + i - {p_}", f"{s_}*x + j - {p_}"
    cons = [f"{ya} >= 0", f"{H - 1 + p_} - {s_}*y - i >= 0", f"{xa} >= 0", f"{W - 1 + p_} - {s_}*x - j >= 0"] if pad else []
    conv_bufs = [bufs[0], bufs[1], Buffer("T", "out", acc, (N, Ho, Wo, Co))]
    s0 = make_level(dict(n=N, y=Ho, x=Wo, i=R, j=S, c=Ci, k=Co),
                    [(["n", ya, xa, "c"], "assign"), (["i", "j", "k", "c"], "assign"), (["n", "y", "x", "k"], "add")],
                    buffers=conv_bufs, constraints=cons, intrinsic="mul")
    s0.parent_refs = [0, 1, 3]
    ew_bufs = [Buffer("T", "in", acc, (N, Ho, Wo, Co)), bufs[2], bufs[4]]
    s1 = make_level(dict(n=N, y=Ho, x=Wo, k=Co),
                    [(["n", "y", "x", "k"], "assign"), (["k"], "assign"), (["n", "y", "x", "k"], "assign")],
                    buffers=ew_bufs, intrinsic="add_relu")
    s1.parent_refs = [3, 2, 4]
    s0.next = s1
    return make_root(bufs, s0)


def linear_bias_relu_program(M, N, K, out_dtype="bf16", b_transposed=True) -> Block:
    """A Linear layer with activation as two statements:  T[m,n] += X[m,k] * W[n,k]  (W as stored by a Linear layer;
    row-major [k][n] with b_transposed=False), then  O[m,n] = relu(T[m,n] + B[n]).  Root buffers: X, W, B, T (f32
    temporary), O."""
    wshape, wacc = ((N, K), ["n", "k"]) if b_transposed else ((K, N), ["k", "n"])
    bufs = [Buffer("X", "in", "bf16", (M, K)), Buffer("W", "in", "bf16", wshape), Buffer("B", "in", "f32", (N,)),
            Buffer("T", "temp", "f32", (M, N)), Buffer("O", "out", out_dtype, (M, N))]
    s0 = make_level(dict(m=M, n=N, k=K), [(["m", "k"], "assign"), (wacc, "assign"), (["m", "n"], "add")],
                    buffers=[bufs[0], bufs[1], Buffer("T", "out", "f32", (M, N))], intrinsic="mul")
    s0.parent_refs = [0, 1, 3]
    s1 = make_level(dict(m=M, n=N), [(["m", "n"], "assign"), (["n"], "assign"), (["m", "n"], "assign")],
                    buffers=[Buffer("T", "in", "f32", (M, N)), bufs[2], bufs[4]], intrinsic="add_relu")
    s1.parent_refs = [3, 2, 4]
    s0.next = s1
    return make_root(bufs, s0)


# Further shapes the kernel families cover, for measurements beyond the five configurations (bench.py --workload).
EXTRA_NAMES = ("gemm_bf16_4096_bt", "gemm_bf16_4000_ragged", "gemm_i8_4096_bt", "pointwise_conv_bf16", "transposed_conv_f32",
               "resnet_conv_bias_relu_bf16", "resnet_conv_bias_relu_f32", "conv3x3_bias_relu_bf16_128to128", "gemm_bf16_1024", "gemm_bf16_2048",
               "linear_bias_relu_4096", "gemm_bf16_256x256x65536", "gemm_i8_256x256x65536_bt", "gemm_bf16_1024x1024x8192", "conv3x3_bf16_128to128", "conv3x3_s2_bf16_64to128", "conv1x7_bf16_64to64",
               "conv3x3_bf16_w112", "conv5x5_bf16_32to32", "conv3x3_i8_64to64", "conv3x3_bf16_128to192", "conv3x3_bf16_128to256_56", "conv3x3_bf16_256to256_56", "depthwise3x3_f32", "avgpool3x3s2_f32", "maxpool2x2s2_f32", "maxpool3x3s1_f32")


# convolution shapes beyond the two tuned ones (the general matrix-core convolution kernel)
CONV_FAMILY = {   # name: (N, H, W, Ci, Co, R, S, stride, pad, dtype)
    "conv3x3_bf16_128to128": (32, 28, 28, 128, 128, 3, 3, 1, 1, "bf16"),
    "conv3x3_s2_bf16_64to128": (32, 56, 56, 64, 128, 3, 3, 2, 1, "bf16"),
    "conv1x7_bf16_64to64": (32, 56, 56, 64, 64, 1, 7, 1, 3, "bf16"),
    "conv3x3_bf16_w112": (8, 112, 112, 64, 64, 3, 3, 1, 1, "bf16"),
    "conv5x5_bf16_32to32": (32, 56, 56, 32, 32, 5, 5, 1, 2, "bf16"),
    "conv3x3_i8_64to64": (32, 56, 56, 64, 64, 3, 3, 1, 1, "i8"),
    "conv3x3_bf16_128to256_56": (16, 56, 56, 128, 256, 3, 3, 1, 1, "bf16"),   # 784 tiles of 128 x 128 (or 392 of 256 x 128: two rounds of workgroups)
    "conv3x3_bf16_256to256_56": (32, 56, 56, 256, 256, 3, 3, 1, 1, "bf16"),   # 392 tiles of 256 x 256, 72 K tiles: the contraction kernel's convolution mode
    "conv3x3_bf16_128to192": (32, 28, 28, 128, 192, 3, 3, 1, 1, "bf16"),   # 192 channels: one and a half 128-wide tiles or three 64-wide ones; 196 tiles of 256 x 128
}


def extra_block(name: str) -> Block:
    if name == "gemm_bf16_4096_bt":
        return matmul_block(4096, 4096, 4096, "bf16", "f32", b_transposed=True)
    if name in ("gemm_bf16_1024", "gemm_bf16_2048"):      # fewer 256 x 256 tiles than CUs: the 128 x 128-tile kernel
        n = int(name.rsplit("_", 1)[1])
        return matmul_block(n, n, n, "bf16", "f32")
    if name in CONV_FAMILY:
        N, H, Wd, Ci, Co, R, S, st, pad, dt = CONV_FAMILY[name]
        return conv2d_block(N, H, Wd, Ci, Co, R, S, st, pad, dt, "i32" if dt == "i8" else "f32")
    if name == "maxpool2x2s2_f32":             # other windows over the max-pooling config's tensor
        return maxpool_block(32, 112, 112, 64, 2, 2, 0)
    if name == "maxpool3x3s1_f32":
        return maxpool_block(32, 112, 112, 64, 3, 1, 1)
    if name == "depthwise3x3_f32":             # 3x3 depthwise convolution over the max-pooling config's tensor
        return depthwise_conv_block(32, 112, 112, 64, 3, 3, 1, 1, "f32")
    if name == "avgpool3x3s2_f32":             # the max-pooling config's window as an average (sum of taps times 1/9)
        return avgpool_block(32, 112, 112, 64, 3, 2, 1)
    if name == "gemm_bf16_256x256x65536":      # few output tiles, long reduction index: the reduction is split over workgroups
        return matmul_block(256, 256, 65536, "bf16", "f32")
    if name == "gemm_i8_256x256x65536_bt":
        return matmul_block(256, 256, 65536, "i8", "i32", b_transposed=True)
    if name == "gemm_bf16_1024x1024x8192":
        return matmul_block(1024, 1024, 8192, "bf16", "f32")
    if name == "gemm_bf16_4000_ragged":
        return matmul_block(4000, 4000, 4096, "bf16", "f32")
    if name == "gemm_i8_4096_bt":
        return matmul_block(4096, 4096, 4096, "i8", "i32", b_transposed=True)
    if name == "resnet_conv_bias_relu_bf16":   # the ResNet block followed by O = relu(T + bias), bf16 output: two statements
        return conv_bias_relu_program(32, 56, 56, 64, 64, 3, 3, 1, 1, "bf16", "bf16")
    if name == "linear_bias_relu_4096":        # relu(X * W^T + b), 4096^3, bf16 output: two statements fused into the GEMM
        return linear_bias_relu_program(4096, 4096, 4096, "bf16", b_transposed=True)
    if name == "conv3x3_bias_relu_bf16_128to128":   # the same two statements on a shape of the general convolution kernel
        return conv_bias_relu_program(32, 28, 28, 128, 128, 3, 3, 1, 1, "bf16", "bf16")
    if name == "resnet_conv_bias_relu_f32":    # the same with an fp32 output
        return conv_bias_relu_program(32, 56, 56, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    if name == "pointwise_conv_bf16":          # 1x1 convolution, 256 -> 64 channels on the ResNet block's 32 x 56 x 56 pixels
        bufs = [Buffer("I", "in", "bf16", (32, 56, 56, 256)), Buffer("F", "in", "bf16", (64, 256)),
                Buffer("O", "out", "f32", (32, 56, 56, 64))]
        return flat_block(bufs, dict(n=32, y=56, x=56, c=256, k=64),
                          [(["n", "y", "x", "c"], "assign"), (["k", "c"], "assign"), (["n", "y", "x", "k"], "add")], intrinsic="mul")
    if name == "transposed_conv_f32":          # stride-2 transposed 3x3 convolution: output elements shared between index tuples
        bufs = [Buffer("I", "in", "f32", (8, 28, 28, 32)), Buffer("F", "in", "f32", (3, 3, 32, 32)),
                Buffer("O", "out", "f32", (8, 57, 57, 32))]
        return flat_block(bufs, dict(n=8, y=28, x=28, i=3, j=3, c=32, k=32),
                          [(["n", "y", "x", "c"], "assign"), (["i", "j", "c", "k"], "assign"),
                           (["n", "2*y + i", "2*x + j", "k"], "add")], intrinsic="mul")
    raise KeyError(name)


def extra_inputs(name: str):
    if name in ("resnet_conv_bias_relu_bf16", "resnet_conv_bias_relu_f32"):
        return config_inputs("resnet_conv_bf16") + [seeded_tensor((64,), "f32", 2)]
    blk = extra_block(name)
    if name == "conv3x3_bias_relu_bf16_128to128":
        return [seeded_tensor((32, 28, 28, 128), "bf16", 0),
                (seeded_tensor((3, 3, 128, 128), "bf16", 1).float() * (2.0 / 1152.0) ** 0.5).to(seeded_tensor((1,), "bf16", 0).dtype),
                seeded_tensor((128,), "f32", 2)]
    if name == "avgpool3x3s2_f32":
        import torch
        return [seeded_tensor(blk.refs[0].sizes, "f32", 0), torch.full((1,), 1.0 / 9.0, dtype=torch.float32)]
    return [seeded_tensor(r.sizes, r.dtype, seed) for seed, r in enumerate(blk.refs) if r.dir == "in"]


def config_inputs(name: str):
    """Seeded torch CPU tensors for a configuration: seed 0 for the first
    tensor, seed 1 for the second; bf16 by round-to-nearest-even of the fp32 draw."""
    import torch

    def gen(seed):
        g = torch.Generator(device="cpu")
        g.manual_seed(seed)
        return g

    if name == "tiny_conv_f32":
        i = torch.rand((1, 16, 16, 8), generator=gen(0), dtype=torch.float32) * 2 - 1
        f = torch.rand((3, 3, 16, 8), generator=gen(1), dtype=torch.float32) * 2 - 1
        return [i, f]
    if name == "gemm_bf16_4096":
        a = torch.randn((4096, 4096), generator=gen(0), dtype=torch.float32).to(torch.bfloat16)
        b = torch.randn((4096, 4096), generator=gen(1), dtype=torch.float32).to(torch.bfloat16)
        return [a, b]
    if name == "resnet_conv_bf16":
        i = torch.relu(torch.randn((32, 56, 56, 64), generator=gen(0), dtype=torch.float32)).to(torch.bfloat16)
        f = (torch.randn((3, 3, 64, 64), generator=gen(1), dtype=torch.float32) * (2.0 / 576.0) ** 0.5).to(torch.bfloat16)
        return [i, f]
    if name == "conv7x7_s2_int8":
        i = torch.randint(-128, 128, (16, 224, 224, 3), generator=gen(0), dtype=torch.int8)
        f = torch.randint(-128, 128, (7, 7, 64, 3), generator=gen(1), dtype=torch.int8)
        return [i, f]
    if name == "maxpool_f32":
        return [torch.randn((32, 112, 112, 64), generator=gen(0), dtype=torch.float32)]
    raise KeyError(name)


def seeded_tensor(shape, dtype: str, seed: int, dist: str = "normal"):
    """One seeded torch CPU tensor of a block dtype ("i8","i32","bf16","f32")."""
    import torch
    g = torch.Generator(device="cpu")
    g.manual_seed(seed)
    if dtype == "i8":
        return torch.randint(-128, 128, tuple(shape), generator=g, dtype=torch.int8)
    if dtype == "i32":
        return torch.randint(-1000, 1001, tuple(shape), generator=g, dtype=torch.int32)
    x = torch.randn(tuple(shape), generator=g, dtype=torch.float32) if dist == "normal" else \
        torch.rand(tuple(shape), generator=g, dtype=torch.float32) * 2 - 1
    return x.to(torch.bfloat16) if dtype == "bf16" else x


def to_numpy(t) -> np.ndarray:
    """A torch CPU tensor as a numpy array; bf16 travels as its uint16 bit pattern."""
    import torch
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def buffer_extent(ref: Refinement) -> int:
    """Elements a root buffer must hold: largest declared address + 1 (the root constant is the window's origin)."""
    return sum((c + n - 1) * s for c, n, s in zip(ref.access_const, ref.sizes, ref.strides)) + 1


def output_extent(root: Block) -> int:
    """Elements the output buffer must hold."""
    return buffer_extent(root.refs[-1])
