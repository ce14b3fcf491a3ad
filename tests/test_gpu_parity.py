"""GPU parity: the HIP library, called through its C ABI, against the CPU oracle
on the same seeded inputs.  Tolerances are stated in tests/util.py.

Small cases span several tiles plus ragged tails and are compared element by
element; the benchmark-size cases run in the launch configuration bench.py
times and are compared on oracle-computed slabs plus size-independent
properties (identity operand, all-ones tap counts).
"""
import math
import random
import sys

import numpy as np
import pytest
import torch

from oracle import stripe_oracle as O
from paper_1903_06498_amd import binding as B
from paper_1903_06498_amd import workloads as W
from tests import brute
from tests.util import SENTINEL_F, SENTINEL_I, abs_inputs, compare, parity, run_gpu

pytestmark = pytest.mark.gpu


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


_FAMILY_ORACLE = {}   # oracle results of cases that run through several kernel variants (see tests.util.parity)


def taps(y, s, p, R, H):
    return sum(1 for i in range(R) if 0 <= s * y + i - p < H)


# ------------------------------------------------------------------ generic path
def test_tiny_conv_f32_config():
    name = "tiny_conv_f32"
    info, score = parity(W.config_block(name), W.config_inputs(name), what=name)
    say(f"{name}: {info['kernel']} rel err {score:.2e}")
    assert info["work_points"] == 270848


@pytest.mark.parametrize("form", ["flat", "tiled"])
def test_figure5_forms_int8(form):
    blk = W.fig5_flat() if form == "flat" else W.fig5_tiled()
    ins = [W.seeded_tensor((12, 16, 8), "i8", 0), W.seeded_tensor((3, 3, 16, 8), "i8", 1)]
    info, _ = parity(blk, ins, what=f"fig5 {form}")
    assert info["work_points"] == 200192 and info["n_idx"] == 6


@pytest.mark.parametrize("seed", range(60))
def test_random_tiny_blocks_generic(seed, monkeypatch):
    """Random small (nested) integer blocks, passed values, constraints, negative
    coefficients: bit-exact, untouched elements kept; or rejected at create.
    Every other group of seven seeds runs the 64-bit index variant."""
    monkeypatch.setenv("STRIPE_TUNE", f"generic_i64={(seed // 7) % 2}")
    rng = random.Random(1000 + seed)
    agg = ["add", "max", "min", "mul"][seed % 4]
    intrinsic = ["mul", "copy", "add"][(seed // 3) % 3]
    blk = brute.random_block(rng, seed % 2 == 1, "i32", "i32", agg, intrinsic, injective_out=True, max_range=6)
    nrng = np.random.default_rng(seed)
    lo, hi = (-1, 3) if agg == "mul" else (-3, 4)          # products of many factors must stay inside int32
    ins = [torch.from_numpy(nrng.integers(lo, hi, size=int(np.prod(r.sizes)), dtype=np.int32)) for r in blk.refs[:-1]]
    try:
        gpu = run_gpu(blk, ins, "generic")
    except B.StripeError as e:
        assert e.status == 5, str(e)   # assign with a reduction
        pytest.skip(f"rejected at create: {e}")
    try:
        res = O.evaluate(blk, [W.to_numpy(t) for t in ins], out=np.full(W.output_extent(blk), SENTINEL_I, np.int64))
    except O.OracleError as e:
        assert e.code == 4 and agg == "mul", str(e)
        pytest.skip("a product leaves int32: outside what the oracle defines")
    assert np.array_equal(gpu.astype(np.int64), res.out)


@pytest.mark.parametrize("seed", range(40))
def test_random_tiny_blocks_shared_outputs(seed, monkeypatch):
    """Random small (nested) integer blocks whose output maps are NOT injective on the output indexes
    (accesses like O[x + i], O[2*a - b]): partial results are combined atomically.  Bit-exact for every
    aggregation, untouched elements kept; 'assign' with several writers is refused at create."""
    monkeypatch.setenv("STRIPE_TUNE", f"generic_i64={(seed // 5) % 2}")
    rng = random.Random(5000 + seed)
    agg = ["add", "max", "min", "mul"][seed % 4]
    intrinsic = ["mul", "copy", "add"][(seed // 3) % 3]
    blk = brute.random_block(rng, seed % 2 == 1, "i32", "i32", agg, intrinsic, injective_out=False, max_range=5)
    nrng = np.random.default_rng(seed)
    lo, hi = (-1, 3) if agg == "mul" else (-3, 4)
    ins = [torch.from_numpy(nrng.integers(lo, hi, size=int(np.prod(r.sizes)), dtype=np.int32)) for r in blk.refs[:-1]]
    try:
        gpu, sb = run_gpu(blk, ins, "generic", return_block=True)
    except B.StripeError as e:
        assert e.status == 5, str(e)
        pytest.skip(f"rejected at create: {e}")
    try:
        res = O.evaluate(blk, [W.to_numpy(t) for t in ins], out=np.full(W.output_extent(blk), SENTINEL_I, np.int64))
    except O.OracleError as e:
        assert e.code == 4 and agg == "mul", str(e)
        pytest.skip("a product leaves int32: outside what the oracle defines")
    assert np.array_equal(gpu.astype(np.int64), res.out), sb.info["kernel"]


@pytest.mark.parametrize("dtype,agg", [("i8", "add"), ("f32", "add"), ("bf16", "add"), ("f32", "max"), ("i8", "min")])
def test_transposed_convolution_shape(dtype, agg):
    """O[n, 2y+i, 2x+j, k] (agg)= I[n, y, x, c] * F[i, j, c, k]: a stride-2 transposed convolution, the classic
    block whose output elements are shared between index tuples.  Integers and max/min exact, float sums by tolerance."""
    N, H, Wd, Ci, Co, R = 2, 9, 7, 5, 6, 3
    odt = "i32" if dtype == "i8" else "f32"
    bufs = [W.Buffer("I", "in", dtype, (N, H, Wd, Ci)), W.Buffer("F", "in", dtype, (R, R, Ci, Co)),
            W.Buffer("O", "out", odt, (N, 2 * H + 1, 2 * Wd + 1, Co))]
    blk = W.flat_block(bufs, dict(n=N, y=H, x=Wd, i=R, j=R, c=Ci, k=Co),
                       [(["n", "y", "x", "c"], "assign"), (["i", "j", "c", "k"], "assign"),
                        (["n", "2*y + i", "2*x + j", "k"], agg)], intrinsic="mul")
    ins = [W.seeded_tensor((N, H, Wd, Ci), dtype, 0), W.seeded_tensor((R, R, Ci, Co), dtype, 1)]
    info, _ = parity(blk, ins, what=f"transposed conv {dtype} {agg}")
    assert info["kernel"].endswith("_atomic") and info["path_name"] == "generic", info


@pytest.mark.parametrize("wide", [0, 1])
@pytest.mark.parametrize("dtype,lanes_hint", [("f32", "conv"), ("bf16", "conv"), ("i8", "conv")])
def test_generic_conv_shapes(dtype, lanes_hint, wide, monkeypatch):
    """Ragged, asymmetric convolution on the generic kernel (wave-per-output mapping), with 32-bit index
    arithmetic (the planner proves it is enough here) and with the 64-bit variant forced."""
    monkeypatch.setenv("STRIPE_TUNE", f"generic_i64={wide}")
    N, H, Wd, Ci, Co, R, S, s, p = 2, 19, 13, 24, 10, 3, 5, 2, 2
    odt = "i32" if dtype == "i8" else "f32"
    blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, s, p, dtype, odt)
    ins = [W.seeded_tensor((N, H, Wd, Ci), dtype, 0), W.seeded_tensor((R, S, Co, Ci), dtype, 1)]
    info, score = parity(blk, ins, "generic", what=f"generic conv {dtype}")
    assert info["kernel"].endswith("_i64") == bool(wide)
    say(f"generic conv {dtype}: {info['kernel']} score {score:.2e}")


@pytest.mark.parametrize("wide", [0, 1])
def test_generic_filter_layout_k_innermost(wide, monkeypatch):
    monkeypatch.setenv("STRIPE_TUNE", f"generic_i64={wide}")
    N, H, Wd, Ci, Co, R, S = 1, 9, 8, 5, 32, 3, 3
    blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, 1, 1, "f32", "f32", filter_layout="RSCK")
    ins = [W.seeded_tensor((N, H, Wd, Ci), "f32", 0), W.seeded_tensor((R, S, Ci, Co), "f32", 1)]
    info, _ = parity(blk, ins, "generic", what="RSCK conv")
    assert "lane_per_output" in info["kernel"]


@pytest.mark.parametrize("M,N,K,dtype", [(70, 90, 130, "f32"), (65, 33, 257, "bf16"), (40, 50, 60, "i8"), (1, 1, 1, "f32")])
def test_generic_matmul_ragged(M, N, K, dtype):
    odt = "i32" if dtype == "i8" else "f32"
    blk = W.matmul_block(M, N, K, dtype, odt)
    ins = [W.seeded_tensor((M, K), dtype, 0), W.seeded_tensor((K, N), dtype, 1)]
    parity(blk, ins, "generic", what=f"generic matmul {dtype}")


# ------------------------------------------------------------------ register-tiled generic contraction
TILED_SEEN = []


@pytest.mark.parametrize("seed", range(48))
def test_tiled_generic_random_blocks(seed, monkeypatch):
    """Random small (nested) integer sum-of-products blocks forced onto the 4 x 4 register-tiled kernel (it is
    normally reserved for large blocks): ragged patches, negative strides, constraints on the blocked index,
    untouched rows.  Bit-exact; blocks without the index roles the kernel needs stay on the plain kernel."""
    monkeypatch.setenv("STRIPE_TUNE", "generic_tiled=2")
    rng = random.Random(7000 + seed)
    blk = brute.random_block(rng, seed % 4 == 3, "i32", "i32", "add", "mul", injective_out=True, max_range=9,
                             contraction_roles=True)
    nrng = np.random.default_rng(seed)
    ins = [torch.from_numpy(nrng.integers(-3, 4, size=int(np.prod(r.sizes)), dtype=np.int32)) for r in blk.refs[:-1]]
    try:
        gpu, sb = run_gpu(blk, ins, "generic", return_block=True)
    except B.StripeError as e:
        assert e.status == 5, str(e)
        pytest.skip(f"rejected at create: {e}")
    TILED_SEEN.append(sb.info["kernel"].startswith("generic_tiled"))
    res = O.evaluate(blk, [W.to_numpy(t) for t in ins], out=np.full(W.output_extent(blk), SENTINEL_I, np.int64))
    assert np.array_equal(gpu.astype(np.int64), res.out), sb.info["kernel"]
    say(f"seed {seed}: {sb.info['kernel']}")


def test_tiled_generic_random_blocks_reached_the_tiled_kernel():
    """Runs after the 48 cases above: a fair share of them must really have used the tiled kernel."""
    assert len(TILED_SEEN) >= 40 and sum(TILED_SEEN) >= 15, (len(TILED_SEEN), sum(TILED_SEEN))


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i8"])
@pytest.mark.parametrize("shape", ["conv_ragged", "conv_vec", "matmul", "matmul_bt", "transposed_filter"])
def test_tiled_generic_shapes(shape, dtype, monkeypatch):
    """Convolutions (strided, asymmetric, padded), matmuls and a filter layout with k innermost on the tiled kernel,
    with and without 4-element loads."""
    monkeypatch.setenv("STRIPE_TUNE", "generic_tiled=2")
    odt = "i32" if dtype == "i8" else "f32"
    if shape == "conv_ragged":
        N, H, Wd, Ci, Co, R, S, s, p = 2, 19, 13, 6, 10, 3, 5, 2, 2
        blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, s, p, dtype, odt)
        ins = [W.seeded_tensor((N, H, Wd, Ci), dtype, 0), W.seeded_tensor((R, S, Co, Ci), dtype, 1)]
        want = "generic_tiled_4x4"
    elif shape == "conv_vec":
        N, H, Wd, Ci, Co, R, S, s, p = 1, 9, 11, 8, 7, 3, 3, 1, 1
        blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, s, p, dtype, odt)
        ins = [W.seeded_tensor((N, H, Wd, Ci), dtype, 0), W.seeded_tensor((R, S, Co, Ci), dtype, 1)]
        want = "generic_tiled_4x4_v4"
    elif shape == "matmul":
        blk = W.matmul_block(70, 90, 52, dtype, odt)
        ins = [W.seeded_tensor((70, 52), dtype, 0), W.seeded_tensor((52, 90), dtype, 1)]
        want = "generic_tiled_4x4"
    elif shape == "matmul_bt":
        blk = W.matmul_block(33, 21, 64, dtype, odt, b_transposed=True)
        ins = [W.seeded_tensor((33, 64), dtype, 0), W.seeded_tensor((21, 64), dtype, 1)]
        want = "generic_tiled_4x4_v4"
    else:
        N, H, Wd, Ci, Co, R, S = 1, 9, 8, 5, 32, 3, 3
        blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, 1, 1, dtype, odt, filter_layout="RSCK")
        ins = [W.seeded_tensor((N, H, Wd, Ci), dtype, 0), W.seeded_tensor((R, S, Ci, Co), dtype, 1)]
        want = "generic_tiled_4x4"
    info, score = parity(blk, ins, "generic", what=f"tiled {shape} {dtype}")
    assert info["kernel"] == want, info["kernel"]


@pytest.mark.parametrize("dtype", ["f32", "bf16", "i8", "i32"])
@pytest.mark.parametrize("intrinsic", ["copy", "add", "mul", "add_relu"])
@pytest.mark.parametrize("broadcast", ["none", "second_over_rows", "second_scalar_per_row"])
def test_pointwise_blocks_four_per_lane(intrinsic, dtype, broadcast):
    """O[a,b,c] = f(A[a,b,c], B[...]) without reduction: the four-outputs-per-lane kernel with a full second operand,
    one broadcast over the outer indexes (B[c]) and one broadcast along the fastest index (B[a,b]); and the plain
    kernel when the fastest range is not a multiple of 4.  Exact for integers, copy and add of exact values."""
    odt = "i32" if dtype in ("i8", "i32") else "f32"
    for shape in ((5, 7, 24), (3, 4, 10)):
        a_, b_, c_ = shape
        bshape, bacc = {"none": (shape, ["a", "b", "c"]), "second_over_rows": ((c_,), ["c"]),
                        "second_scalar_per_row": ((a_, b_), ["a", "b"])}[broadcast]
        bufs = [W.Buffer("A", "in", dtype, shape)] + ([] if intrinsic == "copy" else [W.Buffer("B", "in", dtype, bshape)]) + \
               [W.Buffer("O", "out", odt, shape)]
        refs = [(["a", "b", "c"], "assign")] + ([] if intrinsic == "copy" else [(bacc, "assign")]) + [(["a", "b", "c"], "assign")]
        blk = W.flat_block(bufs, dict(a=a_, b=b_, c=c_), refs, intrinsic=intrinsic)
        ins = [W.seeded_tensor(shape, dtype, 0)] + ([] if intrinsic == "copy" else [W.seeded_tensor(bshape, dtype, 1)])
        if dtype == "i32":
            ins = [t // 40 for t in ins]                      # keep products inside int32
        info, _ = parity(blk, ins, "generic", what=f"pointwise {intrinsic} {dtype} {broadcast} {shape}")
        assert (info["kernel"] == "generic_pointwise_x4") == (c_ % 4 == 0), info["kernel"]


def test_product_aggregation_float():
    """O[a] = prod over r of (A[a, r] + B[r]) in fp32 against the fp64 oracle; and a shared-output form O[a + r]."""
    bufs = [W.Buffer("A", "in", "f32", (50, 9)), W.Buffer("B", "in", "f32", (9,)), W.Buffer("O", "out", "f32", (58,))]
    a = 1.0 + 0.2 * W.seeded_tensor((50, 9), "f32", 0)
    b = 0.1 * W.seeded_tensor((9,), "f32", 1)
    for out_access in ("a", "a + r"):
        blk = W.flat_block(bufs, dict(a=50, r=9), [(["a", "r"], "assign"), (["r"], "assign"), ([out_access], "mul")], intrinsic="add")
        info, _ = parity(blk, [a, b], threads=1, what=f"product O[{out_access}]")
        assert info["kernel"].endswith("_atomic") == (out_access != "a")


def test_misaligned_buffers_are_refused_not_launched():
    """The matrix-core and pooling kernels load 16 bytes at a time: a buffer that is not 16-byte aligned must come
    back as the misalignment status from run (nothing is launched), while the generic path takes any element-aligned
    pointer."""
    dev = torch.device("cuda:0")
    blk = W.matmul_block(256, 256, 128, "bf16", "f32")
    sb = B.StripeBlock(blk)
    a = torch.zeros(256 * 128 + 8, dtype=torch.bfloat16, device=dev)
    b = torch.zeros(128 * 256, dtype=torch.bfloat16, device=dev)
    out = torch.zeros(256 * 256, dtype=torch.float32, device=dev)
    with pytest.raises(B.StripeError) as e:
        sb.run([a.data_ptr() + 2, b], out)
    assert e.value.status == 8
    sb.run([a, b], out)                                   # the handle is still usable
    torch.cuda.synchronize()
    gen = B.StripeBlock(blk, "generic")
    ones = torch.ones(256 * 128 + 8, dtype=torch.bfloat16, device=dev)
    gen.run([ones.data_ptr() + 2, torch.ones(128 * 256, dtype=torch.bfloat16, device=dev)], out)
    torch.cuda.synchronize()
    assert torch.all(out == 128.0)
    with pytest.raises(B.StripeError) as e:
        sb.run([0, b], out)                               # NULL input
    assert e.value.status == 1


def test_unwritten_elements_keep_their_contents():
    bufs = [W.Buffer("A", "in", "i32", (70,)), W.Buffer("O", "out", "i32", (70,))]
    blk = W.flat_block(bufs, dict(x=70, r=3), [(["x"], "assign"), (["x"], "add")],
                       constraints=["x + r - 40 >= 0"], intrinsic="copy")
    a = torch.arange(70, dtype=torch.int32)
    gpu = run_gpu(blk, [a])
    want = np.array([SENTINEL_I if x < 38 else x * sum(1 for r in range(3) if x + r >= 40) for x in range(70)])
    assert np.array_equal(gpu.astype(np.int64), want)
    res = O.evaluate(blk, [a.numpy()], out=np.full(70, SENTINEL_I, np.int64))
    assert np.array_equal(res.out, want)


def test_empty_block_launches_nothing():
    blk = W.matmul_block(3, 0, 5, "f32", "f32")
    blk.refs[1].sizes = [5, 1]
    blk.refs[2].sizes = [3, 1]
    gpu = run_gpu(blk, [torch.zeros(15), torch.zeros(5)])
    assert np.all(gpu == np.float32(SENTINEL_F))


# ------------------------------------------------------------------ buffers declared as windows of larger tensors
def _embedded_case(case):
    """(block, parent tensors, kernel-family expectation) with every buffer a window at a non-zero origin."""
    if case == "generic_matmul_f32":
        blk = W.embed(W.matmul_block(19, 23, 31, "f32", "f32"), [(2, 3), (1, 5), (3, 1)], [(24, 35), (40, 30), (25, 27)])
        return blk, [W.seeded_tensor((24, 35), "f32", 0), W.seeded_tensor((40, 30), "f32", 1)], "generic"
    if case == "tiny_conv_f32":
        blk = W.embed(W.conv2d_block(1, 16, 16, 8, 16, 3, 3, 1, 1, "f32", "f32"), [(1, 2, 3, 1), (1, 0, 2, 3), (0, 1, 2, 5)],
                      [(2, 19, 21, 11), (4, 3, 19, 12), (1, 18, 19, 23)])
        return blk, [W.seeded_tensor((2, 19, 21, 11), "f32", 0, "uniform"), W.seeded_tensor((4, 3, 19, 12), "f32", 1, "uniform")], "generic"
    if case == "fig5_tiled_i8":
        blk = W.embed(W.fig5_tiled(), [(2, 1, 3), (0, 1, 0, 2), (1, 0, 4)], [(15, 18, 12), (3, 4, 16, 11), (13, 17, 21)])
        return blk, [W.seeded_tensor((15, 18, 12), "i8", 0), W.seeded_tensor((3, 4, 16, 11), "i8", 1)], "generic"
    if case in ("gemm_bf16_aligned", "gemm_bf16_unaligned", "gemm_bf16_t256_aligned"):
        oa, ob = ((8, 16), (16, 8)) if case.endswith("_aligned") else ((8, 3), (16, 8))
        blk = W.embed(W.matmul_block(256, 384, 128, "bf16", "f32"), [oa, ob, (3, 5)], [(300, 200), (160, 400), (260, 391)])
        return blk, [W.seeded_tensor((300, 200), "bf16", 0), W.seeded_tensor((160, 400), "bf16", 1)], \
            "mfma_gemm" if case.endswith("_aligned") else "generic"
    if case in ("conv_bf16_aligned", "conv_bf16_unaligned"):
        oi = (1, 2, 3, 64) if case.endswith("_aligned") else (1, 2, 3, 60)
        blk = W.embed(W.conv2d_block(2, 10, 13, 64, 64, 3, 3, 1, 1, "bf16", "f32"), [oi, (2, 0, 0, 0), (1, 1, 2, 64)],
                      [(3, 14, 20, 128), (5, 3, 64, 64), (3, 12, 18, 128)])
        return blk, [W.seeded_tensor((3, 14, 20, 128), "bf16", 0), W.seeded_tensor((5, 3, 64, 64), "bf16", 1)], \
            "mfma_conv" if case.endswith("_aligned") else "generic"
    if case == "conv_i8_aligned":
        blk = W.embed(W.conv2d_block(2, 10, 64, 3, 64, 7, 7, 2, 3, "i8", "i32"), [(1, 2, 16, 0), (1, 0, 0, 0), (0, 1, 2, 64)],
                      [(3, 13, 96, 3), (8, 7, 64, 3), (2, 7, 36, 128)])
        return blk, [W.seeded_tensor((3, 13, 96, 3), "i8", 0), W.seeded_tensor((8, 7, 64, 3), "i8", 1)], "mfma_conv"
    if case in ("pool_aligned", "pool_unaligned"):
        oi = (1, 2, 1, 4) if case.endswith("_aligned") else (1, 2, 1, 3)
        blk = W.embed(W.maxpool_block(2, 30, 26, 8, 3, 2, 1), [oi, (0, 1, 2, 8)], [(3, 33, 28, 16), (2, 17, 16, 20)])
        return blk, [W.seeded_tensor((3, 33, 28, 16), "f32", 0)], "pool" if case.endswith("_aligned") else "generic"
    raise KeyError(case)


@pytest.mark.parametrize("case", ["generic_matmul_f32", "tiny_conv_f32", "fig5_tiled_i8", "gemm_bf16_aligned", "gemm_bf16_unaligned",
                                  "gemm_bf16_t256_aligned", "conv_bf16_aligned", "conv_bf16_unaligned", "conv_i8_aligned", "pool_aligned",
                                  "pool_unaligned"])
def test_root_origin_windows(case, monkeypatch):
    """The root refinement's constant is the origin of the buffer inside a larger tensor (Figure 5 prints it as
    'I[0, 0, 0]'): reads come from the window, writes go to the window, the rest of the output tensor keeps its
    contents.  Origins that keep 16-byte alignment stay on the specialised kernel families, others run generic."""
    if "_t256_" in case:
        monkeypatch.setenv("STRIPE_TUNE", "gemm_t128=0")       # the 256 x 256-tile kernel also for this small product
    blk, ins, family = _embedded_case(case)
    info, score = parity(blk, ins, what=f"root origin {case}")
    say(f"root origin {case}: {info['kernel']} score {score:.3g}")
    assert info["path_name"] == family, info


# ------------------------------------------------------------------ statement lists (two statements and a temporary)
def program_parity(N, H, Wd, Ci, Co, R, stride, pad, in_dt, out_dt, path="auto"):
    prog = W.conv_bias_relu_program(N, H, Wd, Ci, Co, R, R, stride, pad, in_dt, out_dt)
    acc = "i32" if in_dt == "i8" else "f32"
    ins = [W.seeded_tensor((N, H, Wd, Ci), in_dt, 0), W.seeded_tensor((R, R, Co, Ci), in_dt, 1)]
    bias = (W.seeded_tensor((Co,), "i32", 2) * 30) if acc == "i32" else W.seeded_tensor((Co,), "f32", 2)
    if acc == "f32" and in_dt == "bf16":
        ins[1] = (ins[1].float() * (2.0 / (R * R * Ci)) ** 0.5).to(torch.bfloat16)     # keep sums O(1), like the bias
    gpu, sb = run_gpu(prog, ins + [bias], path, return_block=True)
    res = O.evaluate_program(prog, [W.to_numpy(t).ravel() for t in ins] + [bias.numpy()], threads=8)
    assert res.touched.all()
    if acc == "i32":
        assert np.array_equal(gpu.astype(np.int64), res.out)
    else:
        err = np.abs(gpu.astype(np.float64) - res.out)
        K = R * R * Ci
        amax, bmax = float(ins[0].float().abs().max()), float(ins[1].float().abs().max())
        tol = (4e-3 * math.sqrt(K) * amax * bmax) if in_dt == "bf16" else 1e-4 * max(1.0, float(np.sqrt(np.mean(res.out ** 2))))
        if out_dt == "bf16":
            tol = tol + 2.0 ** -8 * np.abs(res.out)          # the store rounds to bf16: half an ulp, and a little
        assert np.all(err <= tol), float(np.max(err - tol))
        assert (gpu == 0).any() and (gpu > 0).any()          # the relu cut is exercised on both sides
    return sb.info


@pytest.mark.parametrize("in_dt,out_dt", [("f32", "f32"), ("bf16", "f32"), ("bf16", "bf16"), ("i8", "i32"), ("f32", "bf16")])
@pytest.mark.parametrize("shape", [(2, 9, 7, 5, 6, 3, 1, 1), (1, 12, 11, 8, 16, 3, 2, 0)])
def test_two_statement_program_small(shape, in_dt, out_dt):
    """convolution into an f32 (i32) temporary, then relu(T + bias) into the output, on general shapes (generic
    kernels): the statements run in order through a temporary the handle owns."""
    info = program_parity(*shape, in_dt, out_dt)
    assert " ; " in info["kernel"], info["kernel"]


@pytest.mark.parametrize("fuse", [1, 2, 0])
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
@pytest.mark.parametrize("N,H,Wd", [(2, 10, 13), (1, 7, 56), (2, 15, 31)])
def test_fused_convolution_bias_relu(N, H, Wd, out_dt, fuse, monkeypatch):
    """3x3, 64 -> 64 channels: the planner fuses the two statements into the matrix-core convolution kernel with a
    bias + relu epilogue (the temporary stays in the accumulators); with fuse=0 the same program runs as two
    launches through a real temporary; fuse=2 is the fused form on the rolling-row kernel.  All against the oracle's
    serial evaluation."""
    monkeypatch.setenv("STRIPE_TUNE", f"fuse={min(fuse, 1)},conv_ks={int(fuse == 2)}")
    info = program_parity(N, H, Wd, 64, 64, 3, 1, 1, "bf16", out_dt)
    if fuse:
        assert {1: "_dma_", 2: "_ksplit_"}[fuse] in info["kernel"], info["kernel"]
        assert info["kernel"].endswith("+bias_relu" + ("_bf16" if out_dt == "bf16" else "")) and info["path_name"] == "mfma_conv", info["kernel"]
    else:
        assert " ; " in info["kernel"], info["kernel"]


@pytest.mark.parametrize("fuse", [1, 2, 3, 0])
@pytest.mark.parametrize("out_dt", ["bf16", "f32"])
@pytest.mark.parametrize("shape", [(2, 14, 14, 128, 128, 3, 1, 1), (2, 17, 19, 64, 128, 3, 2, 1), (1, 12, 40, 32, 96, 5, 1, 2),
                                   (3, 9, 11, 64, 36, 1, 1, 0), (1, 30, 30, 32, 64, 3, 2, 0)])
def test_fused_convolution_bias_relu_general_kernel(shape, out_dt, fuse, monkeypatch):
    """The same two statements on shapes of the general matrix-core convolution kernel (channel counts, strides, filter
    extents and paddings the tuned kernel does not take; ragged pixel and channel tiles): fused into its store phase,
    (fuse=2: on the kernel's largest tile, 256 pixels x 128 channels), and unfused through a temporary; all against
    the oracle's serial evaluation."""
    monkeypatch.setenv("STRIPE_TUNE", f"fuse={min(fuse, 1)}" + (",conv_igemm_tn=128,conv_igemm_tm=256" if fuse == 2 else ",conv_gemm=2" if fuse == 3 else ""))
    info = program_parity(*shape, "bf16", out_dt)
    if fuse == 3 and (shape[5] * shape[5] * (shape[3] // 32)) % 4 == 0:
        # (fuse=3: the contraction kernel's convolution mode, which takes reductions of a multiple of four K tiles)
        assert info["kernel"].startswith("conv_gemm_bf16_256x256x32") and info["kernel"].endswith("+bias_relu" + ("_bf16" if out_dt == "bf16" else "")), info
    elif fuse:
        assert fuse != 2 or "_256x128x" in info["kernel"], info["kernel"]
        assert info["kernel"].startswith("conv_igemm_bf16_") and info["kernel"].endswith("+bias_relu" + ("_bf16" if out_dt == "bf16" else "")), info
    else:
        assert " ; " in info["kernel"] and "conv_igemm_bf16_" in info["kernel"], info["kernel"]


@pytest.mark.parametrize("fuse", [1, 2, 0])
@pytest.mark.parametrize("M,N,K,bt,out_dt", [(256, 256, 128, True, "bf16"), (300, 520, 256, True, "f32"), (512, 256, 128, False, "bf16"),
                                             (384, 640, 256, True, "f32"), (70, 264, 128, False, "f32"), (1024, 1024, 256, True, "bf16")])
def test_fused_linear_bias_relu(M, N, K, bt, out_dt, fuse, monkeypatch):
    """O = relu(X * W^T + b) as two statements: fused into the dense-contraction kernels' epilogue (all their float
    modes: 256 and 128 tiles, transposed / row-major W, ragged edges; fuse=2: with the 4-byte stores of the 256-tile
    kernel instead of its 16-byte ones), or unfused through a temporary."""
    monkeypatch.setenv("STRIPE_TUNE", f"fuse={min(fuse, 1)},gemm_epi16={-1 if fuse == 1 else 0}")
    prog = W.linear_bias_relu_program(M, N, K, out_dt, b_transposed=bt)
    x = W.seeded_tensor((M, K), "bf16", 0)
    w = (W.seeded_tensor((N, K) if bt else (K, N), "bf16", 1).float() * (1.0 / K) ** 0.5).to(torch.bfloat16)
    b = W.seeded_tensor((N,), "f32", 2)
    gpu, sb = run_gpu(prog, [x, w, b], return_block=True)
    assert ("+bias" in sb.info["kernel"]) == bool(fuse) and sb.info["path_name"] == "mfma_gemm", sb.info["kernel"]
    res = O.evaluate_program(prog, [W.to_numpy(x).ravel(), W.to_numpy(w).ravel(), b.numpy()], threads=8)
    err = np.abs(gpu.astype(np.float64) - res.out)
    tol = 4e-3 * math.sqrt(K) * float(x.float().abs().max()) * float(w.float().abs().max())
    if out_dt == "bf16":
        tol = tol + 2.0 ** -8 * np.abs(res.out)
    assert res.touched.all() and np.all(err <= tol), float(np.max(err - tol))
    assert (gpu == 0).any() and (gpu > 0).any()


def test_fused_convolution_bias_relu_full_size():
    """The ResNet-shaped block with a bf16 output, fused: all-ones closed form on every element, and the seeded
    inputs on every element against the oracle's serial evaluation of the two statements."""
    prog = W.extra_block("resnet_conv_bias_relu_bf16")
    ins = W.extra_inputs("resnet_conv_bias_relu_bf16")
    ones = [torch.ones_like(ins[0]), torch.ones_like(ins[1]), -40.0 * torch.arange(64, dtype=torch.float32)]
    gpu, sb = run_gpu(prog, ones, return_block=True)
    assert sb.info["kernel"].endswith("+bias_relu_bf16"), sb.info["kernel"]
    cy = np.array([taps(y, 1, 1, 3, 56) for y in range(56)])
    t = 64.0 * cy[:, None] * cy[None, :]
    want = np.maximum(t[:, :, None] - 40.0 * np.arange(64)[None, None, :], 0.0)          # all exactly representable in bf16
    assert np.array_equal(gpu.reshape(32, 56, 56, 64), np.broadcast_to(want[None], (32, 56, 56, 64)))
    fused = run_gpu(prog, ins)
    say("fused conv+bias+relu at full size: oracle (two statements, every element) ...")
    res = O.evaluate_program(prog, [W.to_numpy(t).ravel() for t in ins], threads=16)
    assert res.touched.all()
    err = np.abs(fused.astype(np.float64) - res.out)
    tol = 4e-3 * math.sqrt(576) * float(ins[0].float().abs().max()) * float(ins[1].float().abs().max()) + 2.0 ** -8 * np.abs(res.out)
    assert np.all(err <= tol), float(np.max(err - tol))
    say(f"  max err {err.max():.3e} (tolerance floor {tol.min():.3e})")
    assert (fused == 0).any() and (fused > 0).any()


# ------------------------------------------------------------------ blocks produced by the tiling rewrite
@pytest.mark.parametrize("case", ["pool_ragged", "conv_bf16", "matmul_f32", "fig5_ragged"])
def test_rewritten_nests_run_like_their_flat_forms(case):
    """A nest made by stripe_block_tile (Section 3.3's rewrite; ragged tiles add overflow constraints) goes through
    the same planner: it must land on the same kernel family as its flat form and match the oracle run on the NEST."""
    if case == "pool_ragged":
        flat, tile = W.maxpool_block(2, 45, 27, 12, 3, 2, 1), [1, 5, 4, 12, 3, 3]
        ins = [W.seeded_tensor((2, 45, 27, 12), "f32", 3)]
    elif case == "conv_bf16":
        flat, tile = W.conv2d_block(2, 10, 13, 64, 64, 3, 3, 1, 1, "bf16", "f32"), [1, 4, 5, 3, 3, 64, 32]
        ins = [W.seeded_tensor((2, 10, 13, 64), "bf16", 0), W.seeded_tensor((3, 3, 64, 64), "bf16", 1)]
    elif case == "matmul_f32":
        flat, tile = W.matmul_block(70, 90, 130, "f32", "f32"), [32, 16, 50]
        ins = [W.seeded_tensor((70, 130), "f32", 0), W.seeded_tensor((130, 90), "f32", 1)]
    else:
        flat, tile = W.fig5_flat(), [5, 3, 3, 3, 8, 16]
        ins = [W.seeded_tensor((12, 16, 8), "i8", 0), W.seeded_tensor((3, 3, 16, 8), "i8", 1)]
    assert len(tile) == len(flat.child.ranges)
    nest = B.stripe_block_tile(flat, tile)
    info, _ = parity(nest, ins, what=f"tiled {case}")
    flat_info = B.StripeBlock(flat).info
    assert info["path_name"] == flat_info["path_name"] and info["work_points"] == flat_info["work_points"], (info, flat_info)


# ------------------------------------------------------------------ pooling path
@pytest.mark.parametrize("N,H,Wd,C", [(2, 30, 26, 8), (1, 7, 9, 4), (3, 33, 35, 64), (1, 112, 112, 64)])
def test_pool_path_small(N, H, Wd, C):
    blk = W.maxpool_block(N, H, Wd, C, 3, 2, 1)
    x = W.seeded_tensor((N, H, Wd, C), "f32", 0)
    info, _ = parity(blk, [x], what=f"pool {N}x{H}x{Wd}x{C}")
    assert info["path_name"] == "pool", info
    ref = torch.nn.functional.max_pool2d(x.permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).contiguous()
    gpu = run_gpu(blk, [x])
    assert np.array_equal(gpu.reshape(ref.shape), ref.numpy())


@pytest.mark.parametrize("lean", [0, 1])
@pytest.mark.parametrize("ty", [1, 2, 3, 7])
def test_pool_strip_heights(ty, lean, monkeypatch):
    """Strip heights that divide and do not divide the 23 output rows; with selects for out-of-range taps
    (lean=0) and with clamped duplicate taps (lean=1, the default)."""
    monkeypatch.setenv("STRIPE_TUNE", f"pool_roll=0,pool_ty={ty},pool_nt=0,pool_lean={lean}")
    blk = W.maxpool_block(2, 45, 27, 12, 3, 2, 1)
    x = W.seeded_tensor((2, 45, 27, 12), "f32", 3)
    info, _ = parity(blk, [x], what=f"pool ty={ty}")
    assert f"ty{ty}" in info["kernel"] and not info["kernel"].endswith("_nt") and info["kernel"].endswith("_sel") != bool(lean)


@pytest.mark.parametrize("rows,wg", [(1, 0), (2, 64), (3, 128), (7, 0), (23, 512), (100, 0)])
def test_pool_rolling_chunks(rows, wg, monkeypatch):
    """The rolling kernel with chunks of 1 row (nothing carried), ragged last chunks, one chunk per image
    (rows clamps to the 23 output rows) and several workgroup sizes; odd H and W give a ragged bottom and right."""
    monkeypatch.setenv("STRIPE_TUNE", f"pool_roll=1,pool_roll_rows={rows},pool_roll_wg={wg}")
    blk = W.maxpool_block(2, 45, 27, 12, 3, 2, 1)
    x = W.seeded_tensor((2, 45, 27, 12), "f32", 3)
    info, _ = parity(blk, [x], what=f"pool roll rows={rows}")
    assert f"roll{min(rows, 23)}_" in info["kernel"], info["kernel"]
    ref = torch.nn.functional.max_pool2d(x.permute(0, 3, 1, 2), 3, 2, 1).permute(0, 2, 3, 1).contiguous()
    assert np.array_equal(run_gpu(blk, [x]).reshape(ref.shape), ref.numpy())


@pytest.mark.parametrize("R,stride,pad,agg", [(2, 2, 0, "max"), (2, 2, 1, "min"), (3, 1, 1, "max"), (3, 1, 0, "min"), (3, 2, 1, "min"),
                                              (3, 2, 0, "max"), (3, 1, 2, "max"), (3, 2, 1, "add"), (2, 2, 1, "add"), (3, 1, 2, "add")])
def test_pool_other_windows_and_min(R, stride, pad, agg):
    """2x2/s2 and 3x3/s1 windows, several paddings, max, min and sum on the pooling kernel: max/min exact and equal
    to the generic kernel's result; sums (taps outside the image contribute nothing) within the fp32 tolerance."""
    N, H, Wd, C = 2, 21, 18, 12
    blk = W.maxpool_block(N, H, Wd, C, R, stride, pad, agg=agg)
    x = W.seeded_tensor((N, H, Wd, C), "f32", 5)
    info, _ = parity(blk, [x], what=f"pool {R}x{R}s{stride}p{pad} {agg}")
    name = "sum" if agg == "add" else agg
    assert info["path_name"] == "pool" and info["kernel"].startswith(f"pool_{name}_f32_{R}x{R}s{stride}_ty"), info
    if agg != "add":
        assert np.array_equal(run_gpu(blk, [x], "pool"), run_gpu(blk, [x], "generic"))
    else:                    # all-ones: the sum is the number of in-range taps, exactly
        ones = torch.ones_like(x)
        got = run_gpu(blk, [ones], "pool").reshape(N, -1, info["output_elements"] // (N * C * ((H + 2 * pad - R) // stride + 1)), C)
        cy = np.array([taps(y, stride, pad, R, H) for y in range(got.shape[1])])
        cx = np.array([taps(xx, stride, pad, R, Wd) for xx in range(got.shape[2])])
        assert np.array_equal(got, np.broadcast_to((cy[:, None] * cx[None, :])[None, :, :, None], got.shape))


@pytest.mark.parametrize("yb", [1, 2, 4])
@pytest.mark.parametrize("ty", [1, 2, 3, 4])
@pytest.mark.parametrize("R,stride,pad,agg", [(2, 2, 0, "max"), (3, 1, 1, "min"), (3, 2, 1, "add"), (3, 1, 0, "add"), (3, 2, 1, "max")])
def test_pool_every_strip_shape(R, stride, pad, agg, ty, yb, monkeypatch):
    """Every strip shape the cost model may choose (rows per strip x strips per workgroup), forced through
    pool_ty / pool_yb, on row counts that leave ragged strips and ragged groups of strips."""
    monkeypatch.setenv("STRIPE_TUNE", f"pool_ty={ty},pool_yb={yb}")
    N, H, Wd, C = 3, 23, 10, 8
    blk = W.maxpool_block(N, H, Wd, C, R, stride, pad, agg=agg)
    info, _ = parity(blk, [W.seeded_tensor((N, H, Wd, C), "f32", 6)], what=f"pool {R}x{R}s{stride} {agg} ty{ty} yb{yb}")
    assert info["kernel"].endswith(f"_ty{ty}" + {1: "", 2: "x2", 4: "x4"}[yb]) and info["workgroup_size"] == 128 * yb, info


@pytest.mark.parametrize("rows", [1, 2, 4, 8])
@pytest.mark.parametrize("R,stride,pad,agg,C", [(2, 2, 0, "max", 8), (3, 1, 1, "min", 24), (3, 2, 1, "add", 8), (3, 2, 1, "max", 64), (3, 1, 0, "add", 4),
                                                (3, 2, 1, "max", 256)])
def test_pool_lds_staged_kernel(R, stride, pad, agg, C, rows, monkeypatch):
    """The LDS-staged strip kernel (input patch global -> LDS once, taps from LDS): every window, aggregation and
    number of rows per workgroup, channel counts that put several pixels, one pixel or a fraction of a pixel into a
    workgroup's 128 items, ragged row groups, clamped / zeroed taps on all four borders."""
    monkeypatch.setenv("STRIPE_TUNE", f"pool_lds={rows}")
    N, H, Wd = 2, 23, 21
    blk = W.maxpool_block(N, H, Wd, C, R, stride, pad, agg=agg)
    info, _ = parity(blk, [W.seeded_tensor((N, H, Wd, C), "f32", 6)], what=f"pool lds {R}x{R}s{stride} {agg} C{C} rows{rows}")
    staged = info["kernel"].endswith(f"_lds{rows}") and info["lds_bytes"] > 0
    assert staged or (rows == 8 and C >= 64), info          # a patch beyond 64 KB of LDS falls back to the register kernel


@pytest.mark.parametrize("yb", [1, 2, 4])
@pytest.mark.parametrize("ty", [1, 2, 3, 4])
@pytest.mark.parametrize("kind", ["depthwise_s1", "depthwise_s2", "avg_2x2"])
def test_weighted_windows_every_strip_shape(kind, ty, yb, monkeypatch):
    """Depthwise convolutions and an average pooling on every strip height and number of strips side by side."""
    monkeypatch.setenv("STRIPE_TUNE", f"pool_ty={ty},pool_yb={yb}")
    if kind == "avg_2x2":
        blk = W.avgpool_block(2, 23, 10, 8, 2, 2, 0)
        ins = [W.seeded_tensor((2, 23, 10, 8), "f32", 0), torch.full((1,), 0.25, dtype=torch.float32)]
    else:
        st = 1 if kind.endswith("s1") else 2
        blk = W.depthwise_conv_block(2, 23, 10, 8, 3, 3, st, 1, "f32")
        ins = [W.seeded_tensor((2, 23, 10, 8), "f32", 0), W.seeded_tensor((3, 3, 8), "f32", 1)]
    info, _ = parity(blk, ins, what=f"{kind} ty{ty} yb{yb}")
    assert info["path_name"] == "pool", info
    if kind == "avg_2x2" or yb < 4:
        assert info["kernel"].endswith(f"_ty{ty}" + {1: "", 2: "x2", 4: "x4"}[yb]), info
    else:                                                     # per-tap weights are offered one or two strips per workgroup
        assert info["kernel"].endswith(f"_ty{ty}") or info["kernel"].endswith(f"_ty{ty}x2"), info


@pytest.mark.parametrize("R,stride,pad,dtype", [(3, 1, 1, "f32"), (3, 2, 1, "f32"), (2, 2, 0, "f32"), (3, 1, 1, "bf16"), (3, 2, 1, "i8"),
                                               (5, 1, 2, "f32")])
def test_depthwise_convolution(R, stride, pad, dtype):
    """A convolution without a channel reduction: fp32 3x3 / 2x2 windows run on the window family's weighted kernel
    (a lane keeps the taps' weights of its four channels in registers), everything else on the generic kernels."""
    N, H, Wd, Cc = 2, 21, 18, 24
    blk = W.depthwise_conv_block(N, H, Wd, Cc, R, R, stride, pad, dtype)
    ins = [W.seeded_tensor((N, H, Wd, Cc), dtype, 0), W.seeded_tensor((R, R, Cc), dtype, 1)]
    info, score = parity(blk, ins, what=f"depthwise {R}x{R} s{stride} {dtype}")
    say(f"depthwise {R}x{R} s{stride} {dtype}: {info['kernel']} score {score:.3g}")
    special = dtype == "f32" and R in (2, 3)
    assert (info["path_name"] == "pool" and info["kernel"].startswith("depthwise")) == special, info
    if special:
        assert np.allclose(run_gpu(blk, ins), run_gpu(blk, ins, "generic"), rtol=1e-5, atol=1e-5)


def test_depthwise_convolution_dilated_runs_generic():
    blk = W.depthwise_conv_block(2, 17, 15, 8, 3, 3, 1, 2, "f32", dilation=2)
    ins = [W.seeded_tensor((2, 17, 15, 8), "f32", 0), W.seeded_tensor((3, 3, 8), "f32", 1)]
    info, _ = parity(blk, ins, what="dilated depthwise")
    assert info["path_name"] == "generic", info


@pytest.mark.parametrize("own_kernel", [0, 1])
@pytest.mark.parametrize("R,stride,pad", [(3, 2, 1), (2, 2, 0), (3, 1, 1), (4, 4, 0)])
def test_average_pooling_with_scale(R, stride, pad, own_kernel, monkeypatch):
    """Average pooling as a sum of scaled taps (the scale in a one-element buffer): the window family's strip kernel
    sums the in-range taps and scales once (own_kernel: the same in the weighted-window kernel's scaled form); windows
    it has no variant for run on the generic kernel."""
    if own_kernel:
        monkeypatch.setenv("STRIPE_TUNE", "pool_scaled_strip=0")
    N, H, Wd, Cc = 2, 24, 20, 16
    blk = W.avgpool_block(N, H, Wd, Cc, R, stride, pad)
    ins = [W.seeded_tensor((N, H, Wd, Cc), "f32", 0), torch.full((1,), 1.0 / (R * R), dtype=torch.float32)]
    info, score = parity(blk, ins, what=f"avgpool {R}x{R} s{stride}")
    say(f"avgpool {R}x{R} s{stride}: {info['kernel']} rel err {score:.2e}")
    assert (info["path_name"] == "pool" and info["kernel"].startswith("pool_scaled_sum")) == (R in (2, 3)), info
    ref = torch.nn.functional.avg_pool2d(ins[0].permute(0, 3, 1, 2), R, stride, pad, count_include_pad=True).permute(0, 2, 3, 1)
    assert np.allclose(run_gpu(blk, ins).reshape(ref.shape), ref.numpy(), rtol=1e-5, atol=1e-6)


def test_pool_all_negative_and_generic_agree():
    blk = W.maxpool_block(2, 21, 17, 8, 3, 2, 1)
    x = -torch.abs(W.seeded_tensor((2, 21, 17, 8), "f32", 1)) - 1
    a = run_gpu(blk, [x], "pool")
    b = run_gpu(blk, [x], "generic")
    assert np.array_equal(a, b) and np.all(a < 0)


def test_maxpool_config_full_size():
    name = "maxpool_f32"
    blk, ins = W.config_block(name), W.config_inputs(name)
    info, _ = parity(blk, ins, threads=16, what=name)
    say(f"{name}: {info['kernel']} grid {info['grid']}")
    assert info["path_name"] == "pool" and info["work_points"] == 57116672


# ------------------------------------------------------------------ dense contraction path
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (512, 768, 320), (1024, 512, 128), (128, 128, 128), (384, 640, 256), (1152, 128, 512)])
def test_gemm_mfma_small(M, N, K):
    blk = W.matmul_block(M, N, K, "bf16", "f32")
    ins = [W.seeded_tensor((M, K), "bf16", 0), W.seeded_tensor((K, N), "bf16", 1)]
    info, score = parity(blk, ins, threads=8, what=f"gemm {M}x{N}x{K}")
    say(f"gemm {M}x{N}x{K}: {info['kernel']} err/bound {score:.3f}")
    assert info["path_name"] == "mfma_gemm"


@pytest.mark.parametrize("tune,name", [("gemm_t128=0,gemm_dma_waves=4", "256x256x32_mfma32x32x16_w4_lds_direct"),
                                       ("gemm_t128=0,gemm_dma_waves=8", "w8_lds_direct"),
                                       ("gemm_t128=0,gemm_dma_waves=4,gemm_epi16=1", "256x256x32_mfma32x32x16_w4_lds_direct"),
                                       ("gemm_t128=0,gemm_dma_waves=8,gemm_epi16=1", "w8_lds_direct"),
                                       ("gemm_t128=0,gemm_sched=0", "w4_lds_direct_s0"), ("gemm_t128=0,gemm_sched=2", "w4_lds_direct_s2"),
                                       ("gemm_t128=0,gemm_sched=3", "w4_lds_direct_s3"),
                                       ("gemm_t128=1", "128x128x64_mfma32x32x16_w8_lds_direct"),
                                       ("gemm_t128=1,gemm_t128_kb=64", "128x128x32_mfma32x32x16_w8_lds_direct"),
                                       ("gemm_t128=1,gemm_t128_waves=4", "128x128x32_mfma32x32x16_w4_lds_direct"),
                                       ("gemm_dma=0,gemm_waves=4", "w4_swz2"), ("gemm_dma=0,gemm_waves=8,gemm_swz=1", "w8_swz1"),
                                       ("gemm_dma=0,gemm_waves=8,gemm_swz=0", "w8_swz0")])
def test_gemm_mfma_position_sensitive(tune, name, monkeypatch):
    """A[m,k] = small integers depending on (m,k), B = shifted identity: every
    output equals one specific input element, exactly, so any mix-up of rows,
    columns, fragments, K steps or tiles shows.  Run on every GEMM kernel variant."""
    monkeypatch.setenv("STRIPE_TUNE", tune)
    M = N = 512
    K = 512
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(torch.bfloat16)
    shift = 37
    b = torch.zeros((K, N), dtype=torch.bfloat16)
    b[(torch.arange(N) + shift) % K, torch.arange(N)] = 1.0
    blk = W.matmul_block(M, N, K, "bf16", "f32")
    gpu, sb = run_gpu(blk, [a, b], return_block=True)
    assert sb.info["path_name"] == "mfma_gemm" and sb.info["kernel"].endswith(name), sb.info["kernel"]
    want = a.float()[:, (torch.arange(N) + shift) % K].numpy()
    assert np.array_equal(gpu.reshape(M, N), want)
    ins = [W.seeded_tensor((M, K), "bf16", 0), W.seeded_tensor((K, N), "bf16", 1)]
    parity(blk, ins, what=f"gemm {tune}")


@pytest.mark.parametrize("M,N,K,bt", [(256, 256, 128, True), (512, 768, 384, True), (300, 520, 256, False), (2, 8, 128, False),
                                      (257, 264, 128, False), (300, 333, 256, True), (70, 9, 128, True), (511, 8, 128, True)])
def test_gemm_transposed_b_and_ragged_edges(M, N, K, bt, monkeypatch):
    """The LDS-direct kernel with B stored [n][k] and/or M, N that are not multiples of the 256 x 256 tile.
    Position-sensitive operands first (every output is one specific A element, exactly), then seeded data."""
    monkeypatch.setenv("STRIPE_TUNE", "gemm_t128=0")       # the 256 x 256 kernel's modes; the small-tile kernel is covered below
    blk = W.matmul_block(M, N, K, "bf16", "f32", b_transposed=bt)
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(torch.bfloat16)
    shift = 37
    sel = (torch.arange(N) + shift) % K
    b = torch.zeros((K, N), dtype=torch.bfloat16)
    b[sel, torch.arange(N)] = 1.0
    gpu, sb = run_gpu(blk, [a, b.t().contiguous() if bt else b], return_block=True)
    ragged = M % 256 != 0 or N % 256 != 0
    want_name = "lds_direct" + ("_bt" if bt else "") + ("_ragged" if ragged else "")
    assert sb.info["path_name"] == "mfma_gemm" and sb.info["kernel"].endswith(want_name), sb.info["kernel"]
    assert np.array_equal(gpu.reshape(M, N), a.float()[:, sel].numpy())
    ins = [W.seeded_tensor((M, K), "bf16", 0), W.seeded_tensor((N, K) if bt else (K, N), "bf16", 1)]
    parity(blk, ins, what=f"gemm {M}x{N}x{K} bt={bt}")          # also checks that nothing outside C[0:M, 0:N] changed


@pytest.mark.parametrize("t128", [1, 2, 0, -1])
@pytest.mark.parametrize("M,N,K", [(256, 256, 256), (512, 768, 512), (300, 333, 256), (70, 9, 512), (257, 8, 256), (128, 384, 256)])
def test_gemm_int8_transposed_b(M, N, K, t128, monkeypatch):
    """int8 x int8 -> int32 on the matrix cores (C = A * B^T, both operands k-contiguous): bit-exact, including
    extreme values (-128 * -128 summed over K) and edges that are not multiples of the tile; small aligned
    products on the 128 x 128-tile kernel (t128=1: K tiles 128 deep, as chosen for products of one round of
    workgroups; 2: 64 deep) and on the 256 x 256 one (0; -1: with its 16-byte stores)."""
    monkeypatch.setenv("STRIPE_TUNE", f"gemm_t128={min(max(t128, 0), 1)},gemm_epi16={int(t128 < 0)}" + (",gemm_t128_kb=64" if t128 == 2 else ""))
    deep = 64 if t128 == 2 else 128
    t128 = min(max(t128, 0), 1)
    blk = W.matmul_block(M, N, K, "i8", "i32", b_transposed=True)
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(torch.int8)
    sel = (torch.arange(N) + 37) % K
    b = torch.zeros((N, K), dtype=torch.int8)
    b[torch.arange(N), sel] = 1
    gpu, sb = run_gpu(blk, [a, b], return_block=True)
    ragged = M % 256 != 0 or N % 256 != 0
    small = bool(t128) and M % 128 == 0 and N % 128 == 0
    want = f"gemm_i8_128x128x{deep}_mfma32x32x32_w8_lds_direct_bt" if small else "gemm_i8_256x256x64_mfma32x32x32_w4_lds_direct_bt" + ("_ragged" if ragged else "")
    assert sb.info["path_name"] == "mfma_gemm" and sb.info["kernel"] == want, sb.info["kernel"]
    assert np.array_equal(gpu.reshape(M, N), a.to(torch.int32)[:, sel].numpy())
    ins = [W.seeded_tensor((M, K), "i8", 0), W.seeded_tensor((N, K), "i8", 1)]
    parity(blk, ins, what=f"int8 gemm {M}x{N}x{K}")
    lows = [torch.full((M, K), -128, dtype=torch.int8), torch.full((N, K), -128, dtype=torch.int8)]
    assert np.all(run_gpu(blk, lows) == 16384 * K)


@pytest.mark.parametrize("batch,M,N,K,dtype,bt,shared", [(3, 256, 256, 128, "bf16", False, False), (2, 300, 200, 128, "bf16", True, False),
                                                         (5, 70, 264, 256, "bf16", False, False), (2, 256, 256, 256, "i8", True, False),
                                                         (3, 130, 9, 512, "i8", True, False), (4, 64, 256, 128, "bf16", False, True)])
def test_batched_gemm(batch, M, N, K, dtype, bt, shared):
    """C[b] = A[b] * B[b] on the matrix cores: the batch index becomes the slowest part of the grid.  With a B shared
    by all products the batch merges into M and the block is a plain GEMM.  Position-sensitive operands per batch
    entry (different shifts), then seeded data against the oracle."""
    odt = "i32" if dtype == "i8" else "f32"
    tdt = torch.int8 if dtype == "i8" else torch.bfloat16
    blk = W.batched_matmul_block(batch, M, N, K, dtype, odt, b_transposed=bt, shared_b=shared)
    a = ((torch.arange(batch)[:, None, None] * 11 + torch.arange(M)[None, :, None] * 7 + torch.arange(K)[None, None, :] * 3) % 251 - 125).to(tdt)
    nb = 1 if shared else batch
    sel = (torch.arange(N)[None, :] + 37 + 5 * torch.arange(nb)[:, None]) % K
    b = torch.zeros((nb, K, N), dtype=tdt)
    for i in range(nb):
        b[i, sel[i], torch.arange(N)] = 1
    bb = (b.transpose(1, 2) if bt else b).contiguous()
    gpu, sb = run_gpu(blk, [a, bb[0] if shared else bb], return_block=True)
    assert sb.info["path_name"] == "mfma_gemm" and sb.info["kernel"].endswith("_batch") == (not shared), sb.info["kernel"]
    want = torch.stack([a[i].float()[:, sel[0 if shared else i]] for i in range(batch)]).numpy()
    assert np.array_equal(gpu.reshape(batch, M, N), want)
    ins = [W.seeded_tensor(r.sizes, dtype, s_) for s_, r in enumerate(blk.refs[:-1])]
    parity(blk, ins, what=f"batched gemm {batch}x{M}x{N}x{K} {dtype}")


@pytest.mark.parametrize("waves,deep", [(8, 64), (8, 32), (4, 32)])
@pytest.mark.parametrize("M,N,K,bt", [(128, 128, 128, False), (384, 640, 256, True), (1024, 256, 384, False), (256, 1152, 128, True), (512, 384, 1152, False)])
def test_gemm_small_tile_kernel(M, N, K, bt, waves, deep, monkeypatch):
    """Products with few 256 x 256 tiles run on the 128 x 128-tile kernel (row-major and transposed B, eight or four
    wavefronts, K tiles 64 or 32 deep): position-sensitive operands exactly, then seeded data."""
    monkeypatch.setenv("STRIPE_TUNE", f"gemm_t128_waves={waves},gemm_t128_kb={2 * deep}")
    blk = W.matmul_block(M, N, K, "bf16", "f32", b_transposed=bt)
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(torch.bfloat16)
    sel = (torch.arange(N) + 37) % K
    b = torch.zeros((K, N), dtype=torch.bfloat16)
    b[sel, torch.arange(N)] = 1.0
    gpu, sb = run_gpu(blk, [a, b.t().contiguous() if bt else b], return_block=True)
    assert sb.info["kernel"] == f"gemm_bf16_128x128x{deep}_mfma32x32x16_w{waves}_lds_direct" + ("_bt" if bt else ""), sb.info["kernel"]
    assert np.array_equal(gpu.reshape(M, N), a.float()[:, sel].numpy())
    ins = [W.seeded_tensor((M, K), "bf16", 0), W.seeded_tensor((N, K) if bt else (K, N), "bf16", 1)]
    parity(blk, ins, what=f"small-tile gemm {M}x{N}x{K} bt={bt}")


@pytest.mark.parametrize("M,N,K,dt,bt,tune", [(256, 256, 16384, "bf16", False, ""), (256, 256, 8192, "bf16", True, ""),
                                              (128, 256, 16384, "i8", True, ""), (200, 136, 8192, "bf16", False, ""),
                                              (300, 264, 4096, "i8", True, ""), (256, 384, 1536, "bf16", False, "gemm_splitk=3"),
                                              (512, 512, 2048, "bf16", True, "gemm_splitk=2,gemm_t128=0"),
                                              (256, 256, 1024, "i8", True, "gemm_splitk=4"),
                                              # threads per output item in the kernel that adds the slices: one, more than slices, some
                                              (256, 256, 16384, "bf16", False, "gemm_reduce_g=1"), (256, 384, 1536, "bf16", False, "gemm_splitk=3,gemm_reduce_g=16"),
                                              (300, 264, 4096, "i8", True, "gemm_reduce_g=4"), (70, 9, 8192, "bf16", True, "gemm_reduce_g=8")])
def test_split_reduction(M, N, K, dt, bt, tune, monkeypatch):
    """A product with few output tiles and a long reduction index: the reduction is cut into slices that run as
    separate workgroups, partial sums go through the handle's workspace and are added in slice order.  int8
    bit-exact, bf16 within tolerance; a shifted-identity operand that takes each output column from a different
    k (hence from different slices) must pass the first operand through exactly.  The caller-provided workspace and
    the static-scratch entry point give the same bits as the handle-owned workspace."""
    if tune:
        monkeypatch.setenv("STRIPE_TUNE", tune)
    odt = "i32" if dt == "i8" else "f32"
    blk = W.matmul_block(M, N, K, dt, odt, b_transposed=bt)
    tdt = torch.int8 if dt == "i8" else torch.bfloat16
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(tdt)
    sel = (torch.arange(N) * 613 + 37) % K
    b = torch.zeros((K, N), dtype=tdt)
    b[sel, torch.arange(N)] = 1
    gpu, sb = run_gpu(blk, [a, b.t().contiguous() if bt else b], return_block=True)
    assert "_splitk" in sb.info["kernel"] and sb.info["path_name"] == "mfma_gemm", sb.info["kernel"]
    S = int(sb.info["kernel"].rsplit("_splitk", 1)[1])
    assert sb.info["workspace_bytes"] == S * M * N * 4 == B.stripe_block_workspace_size(sb.handle)
    say(f"split reduction {M}x{N}x{K} {dt}: {sb.info['kernel']} grid {sb.info['grid']}")
    assert np.array_equal(gpu.reshape(M, N), a.float()[:, sel].numpy())
    ins = [W.seeded_tensor((M, K), dt, 0), W.seeded_tensor((N, K) if bt else (K, N), dt, 1)]
    parity(blk, ins, threads=16, what=f"split reduction {M}x{N}x{K} {dt}")
    # the three homes of the workspace give identical bits
    dev = torch.device("cuda:0")
    dins = [t.to(dev) for t in ins]
    outs = []
    for mode in ("owned", "caller", "static"):
        out = torch.zeros(M * N, dtype=torch.int32 if dt == "i8" else torch.float32, device=dev)
        if mode == "caller":
            sb.set_workspace(torch.empty(sb.info["workspace_bytes"] + 256, dtype=torch.uint8, device=dev))
        if mode == "static":
            if sb.info["workspace_bytes"] > 8 << 20:
                continue
            sb.run_static(dins, out)
        else:
            sb.run(dins, out)
        torch.cuda.synchronize()
        outs.append(out.cpu())
    assert all(torch.equal(outs[0], o) for o in outs[1:])
    sb.close()


def test_split_reduction_off_matches(monkeypatch):
    """gemm_splitk=0 runs the same block unsplit; both match the oracle (checked above) and each other closely."""
    blk = W.matmul_block(256, 256, 8192, "i8", "i32", b_transposed=True)
    ins = [W.seeded_tensor((256, 8192), "i8", 0), W.seeded_tensor((256, 8192), "i8", 1)]
    split, sb = run_gpu(blk, ins, return_block=True)
    assert "_splitk" in sb.info["kernel"]
    monkeypatch.setenv("STRIPE_TUNE", "gemm_splitk=0")
    whole, sb2 = run_gpu(blk, ins, return_block=True)
    assert "_splitk" not in sb2.info["kernel"] and sb2.info["workspace_bytes"] == 0
    assert np.array_equal(split, whole)


def test_pointwise_convolution_runs_on_the_gemm_kernel():
    """A 1x1 convolution O[n,y,x,k] += I[n,y,x,c] * F[k,c] canonicalises to C = A * B^T (pixels merge into one index)."""
    N, H, Wd, Ci, Co = 2, 12, 20, 128, 72
    bufs = [W.Buffer("I", "in", "bf16", (N, H, Wd, Ci)), W.Buffer("F", "in", "bf16", (Co, Ci)),
            W.Buffer("O", "out", "f32", (N, H, Wd, Co))]
    blk = W.flat_block(bufs, dict(n=N, y=H, x=Wd, c=Ci, k=Co),
                       [(["n", "y", "x", "c"], "assign"), (["k", "c"], "assign"), (["n", "y", "x", "k"], "add")], intrinsic="mul")
    ins = [W.seeded_tensor((N, H, Wd, Ci), "bf16", 0), W.seeded_tensor((Co, Ci), "bf16", 1)]
    info, _ = parity(blk, ins, what="1x1 conv")
    assert info["path_name"] == "mfma_gemm" and info["kernel"].endswith("_bt_ragged"), info


@pytest.mark.parametrize("M,N,K,dt", [(16384, 64, 256, "bf16"), (20000, 40, 128, "bf16"), (16500, 9, 64, "bf16"), (16384, 64, 256, "i8"), (17000, 33, 128, "i8")])
def test_narrow_product_runs_as_pointwise_convolution(M, N, K, dt, monkeypatch):
    """C = A * B^T with at most 64 columns and many rows: planned onto the general convolution kernel's 256 x 64 tile
    (rows as pixels) instead of the 256-wide tiles of the contraction kernels.  A selector operand takes each output
    column from one k (the first operand must come through exactly), then seeded data against the oracle; with
    gemm_narrow_conv=0 the contraction kernel gives the same integers / close floats."""
    odt = "i32" if dt == "i8" else "f32"
    blk = W.matmul_block(M, N, K, dt, odt, b_transposed=True)
    tdt = torch.int8 if dt == "i8" else torch.bfloat16
    a = ((torch.arange(M)[:, None] * 7 + torch.arange(K)[None, :] * 3) % 251 - 125).to(tdt)
    sel = (torch.arange(N) * 37 + 5) % K
    b = torch.zeros((N, K), dtype=tdt)
    b[torch.arange(N), sel] = 1
    gpu, sb = run_gpu(blk, [a, b], return_block=True)
    assert sb.info["path_name"] == "mfma_conv" and "conv_igemm" in sb.info["kernel"] and "_256x64x" in sb.info["kernel"], sb.info
    assert np.array_equal(gpu.reshape(M, N), a.float()[:, sel].numpy())
    ins = [W.seeded_tensor((M, K), dt, 0), W.seeded_tensor((N, K), dt, 1)]
    parity(blk, ins, threads=16, what=f"narrow product {M}x{N}x{K} {dt}")
    narrow = run_gpu(blk, ins)
    monkeypatch.setenv("STRIPE_TUNE", "gemm_narrow_conv=0")
    wide, sb2 = run_gpu(blk, ins, return_block=True)
    assert sb2.info["path_name"] in ("mfma_gemm", "generic"), sb2.info     # (a reduction shorter than the contraction kernels' ring: generic)
    if dt == "i8":
        assert np.array_equal(narrow, wide)
    else:
        assert np.allclose(narrow, wide, rtol=1e-4, atol=1e-3)


def test_gemm_config_full_size():
    """4096^3 in the benchmark's launch configuration: oracle slabs + identity property."""
    name = "gemm_bf16_4096"
    blk, ins = W.config_block(name), W.config_inputs(name)
    gpu, sb = run_gpu(blk, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']} grid {sb.info['grid']}")
    assert sb.info["path_name"] == "mfma_gemm"
    np_ins = [W.to_numpy(t).ravel() for t in ins]
    np_abs = abs_inputs(np_ins, ["bf16", "bf16"])
    # 64 full rows (all n) and 64 full columns (all m), every k: bands that straddle tile, wavefront and fragment
    # borders of the 256 x 256 tiling, plus the first and last row and column
    rows = [(0, 8), (120, 136), (1336, 1340), (2040, 2056), (3071, 3075), (4080, 4096)]
    cols = [(0, 8), (250, 266), (1023, 1027), (2168, 2184), (3583, 3587), (4080, 4096)]
    assert sum(b - a for a, b in rows) == 64 and sum(b - a for a, b in cols) == 64
    windows = [([a, 0, 0], [b, 4096, 4096]) for a, b in rows] + [([0, a, 0], [4096, b, 4096]) for a, b in cols]
    for lo, hi in windows:
        split = 1 if hi[0] - lo[0] < 4096 else 0
        res = O.evaluate(blk, np_ins, window=(lo, hi), threads=16, split_index=split)
        ares = O.evaluate(blk, np_abs, window=(lo, hi), threads=16, split_index=split)
        score = compare(blk, ins, gpu, res, what=f"{name} window {lo}", abs_res=ares)
        say(f"  window {lo}..{hi}: err/bound {score:.3f}")
    # identity operand passes A through bit-exactly, at full size
    eye = torch.eye(4096, dtype=torch.bfloat16)
    gpu = run_gpu(blk, [ins[0], eye])
    assert np.array_equal(gpu.reshape(4096, 4096), ins[0].float().numpy())


# ------------------------------------------------------------------ convolution path (matrix cores)
def conv_tune(w4):
    """STRIPE_TUNE string of one 3x3 kernel: 4 = rolling rows with the reduction split over the teams, 3 = row groups
    with LDS-direct staging (the default), 2 / 1 = row groups with register staging and two teams of wavefronts / one,
    0 = wavefront per row."""
    return f"conv_w4={min(w4, 1)},conv_w4_teams={min(max(w4, 1), 2)},conv_dma={int(w4 >= 3)},conv_ks={int(w4 == 4)}"


@pytest.mark.parametrize("w4", [4, 3, 2, 1, 0])
@pytest.mark.parametrize("N,H,Wd", [(2, 10, 13), (1, 7, 56), (3, 20, 64), (1, 2, 2), (2, 9, 33), (1, 15, 31), (2, 11, 58), (1, 8, 62)])
def test_conv_mfma_bf16_small(N, H, Wd, w4, monkeypatch):
    """3x3, 64 -> 64 channels, 'same' padding: ragged strips, both pixel fragments, halo on all four sides;
    every kernel of the shape (see conv_tune)."""
    monkeypatch.setenv("STRIPE_TUNE", conv_tune(w4))
    blk = W.conv2d_block(N, H, Wd, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    ins = [W.seeded_tensor((N, H, Wd, 64), "bf16", 0), W.seeded_tensor((3, 3, 64, 64), "bf16", 1)]
    info, score = parity(blk, ins, what=f"conv mfma {N}x{H}x{Wd}", cache=_FAMILY_ORACLE, key=("3x3c64", N, H, Wd))   # one oracle run per shape
    say(f"conv mfma {N}x{H}x{Wd}: {info['kernel']} err/bound {score:.3f}")
    patch = 9 * (Wd + 2) * 128
    if w4 >= 3:
        patch = (patch + 1023) // 1024 * 1024                    # whole 1 KB load blocks
    fits = 73728 + patch + 16384 <= 160 * 1024                   # filter + haloed strip + store buffers in LDS
    want = (f"_w{4 * min(w4, 2)}_" + ("ksplit_" if w4 == 4 else "dma_" if w4 == 3 else "mfma")) if (w4 and fits) else "_strip7_mfma"
    assert info["path_name"] == "mfma_conv" and want in info["kernel"], info


@pytest.mark.parametrize("w4", [4, 3, 2, 1, 0])
def test_conv_mfma_position_sensitive(w4, monkeypatch):
    """Delta input: the output is the (flipped) filter patch, exactly -- catches any mix-up of taps, pixels or channels."""
    monkeypatch.setenv("STRIPE_TUNE", conv_tune(w4))
    N, H, Wd = 1, 9, 40
    blk = W.conv2d_block(N, H, Wd, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    f = W.seeded_tensor((3, 3, 64, 64), "bf16", 1)
    i = torch.zeros((N, H, Wd, 64), dtype=torch.bfloat16)
    y0, x0, c0 = 4, 33, 17
    i[0, y0, x0, c0] = 1.0
    gpu, sb = run_gpu(blk, [i, f], return_block=True)
    assert sb.info["path_name"] == "mfma_conv"
    want = np.zeros((N, H, Wd, 64), np.float32)
    for y in range(H):
        for x in range(Wd):
            a, b = y0 - y + 1, x0 - x + 1
            if 0 <= a < 3 and 0 <= b < 3:
                want[0, y, x, :] = f[a, b, :, c0].float().numpy()
    assert np.array_equal(gpu.reshape(want.shape), want)


@pytest.mark.parametrize("N,H,Wd", [(2, 10, 64), (1, 6, 96), (1, 18, 224), (3, 4, 64)])
def test_conv_mfma_int8_small(N, H, Wd):
    """7x7 stride 2, 3 -> 64 channels, int8 -> int32: bit-exact, ragged strips, left/right/top/bottom halo."""
    blk = W.conv2d_block(N, H, Wd, 3, 64, 7, 7, 2, 3, "i8", "i32")
    ins = [W.seeded_tensor((N, H, Wd, 3), "i8", 0), W.seeded_tensor((7, 7, 64, 3), "i8", 1)]
    info, _ = parity(blk, ins, what=f"conv int8 {N}x{H}x{Wd}")
    assert info["path_name"] == "mfma_conv", info
    gen = run_gpu(blk, ins, "generic")
    assert np.array_equal(gen, run_gpu(blk, ins))


def test_conv_mfma_int8_extreme_values():
    """All operands -128: the largest magnitudes the block can produce, exact tap counts at every border."""
    N, H, Wd = 1, 20, 64
    blk = W.conv2d_block(N, H, Wd, 3, 64, 7, 7, 2, 3, "i8", "i32")
    ins = [torch.full((N, H, Wd, 3), -128, dtype=torch.int8), torch.full((7, 7, 64, 3), -128, dtype=torch.int8)]
    gpu = run_gpu(blk, ins).reshape(N, H // 2, Wd // 2, 64)
    cy = np.array([taps(y, 2, 3, 7, H) for y in range(H // 2)])
    cx = np.array([taps(x, 2, 3, 7, Wd) for x in range(Wd // 2)])
    want = 16384 * 3 * cy[:, None] * cx[None, :]
    assert np.array_equal(gpu, np.broadcast_to(want[None, :, :, None], gpu.shape))


# ------------------------------------------------------------------ the general matrix-core convolution kernel
IGEMM_CASES = {
    # name: (N, H, W, Ci, Co, R, S, stride, pad, dtype)
    "3x3_128to128": (2, 28, 28, 128, 128, 3, 3, 1, 1, "bf16"),
    "3x3_s2_64to128_56to28": (2, 56, 56, 64, 128, 3, 3, 2, 1, "bf16"),
    "1x7_64to64": (1, 20, 33, 64, 64, 1, 7, 1, 3, "bf16"),
    "3x3_w112": (1, 9, 112, 64, 64, 3, 3, 1, 1, "bf16"),
    "5x5_32to32": (2, 17, 19, 32, 32, 5, 5, 1, 2, "bf16"),
    "7x3_s2_nopad": (1, 23, 17, 32, 96, 7, 3, 2, 0, "bf16"),
    "1x1_96to40": (3, 10, 10, 96, 40, 1, 1, 1, 0, "bf16"),
    "3x3_32to200": (1, 12, 12, 32, 200, 3, 3, 1, 1, "bf16"),
    "3x3_i8_64to64": (2, 14, 14, 64, 64, 3, 3, 1, 1, "i8"),
    "5x5_s2_i8_128to72": (1, 19, 21, 128, 72, 5, 5, 2, 2, "i8"),
    "3x3_tiny_image": (1, 2, 3, 32, 8, 3, 3, 1, 1, "bf16"),
    "1x1_64to128_one_k_tile": (2, 10, 10, 64, 128, 1, 1, 1, 0, "bf16"),      # 128-byte K tile rows: the whole reduction is one tile
    "1x1_i8_128to72_one_k_tile": (1, 12, 9, 128, 72, 1, 1, 1, 0, "i8"),
    "1x3_64to128_three_k_tiles": (1, 9, 20, 64, 128, 1, 3, 1, 1, "bf16"),
    "3x3_128to264": (2, 19, 23, 128, 264, 3, 3, 1, 1, "bf16"),               # 36 K tiles; two channel tiles of 256, the second ragged
    "2x2_s2_64to72": (3, 20, 18, 64, 72, 2, 2, 2, 0, "bf16"),                 # 8 K tiles
    "3x3_pad2_128to40": (1, 21, 17, 128, 40, 3, 3, 1, 2, "bf16"),             # padding 2 of a 3x3: the pixels at the edges keep one tap
    "1x2_64to300": (2, 15, 20, 64, 300, 1, 2, 1, 0, "bf16"),                  # 4 K tiles: the shortest walk
}


@pytest.mark.parametrize("tile", ["chosen", "256x128", "128x128_k64", "contraction_kernel"])
@pytest.mark.parametrize("case", sorted(IGEMM_CASES))
def test_conv_family_on_the_matrix_cores(case, tile, monkeypatch):
    """Dense convolution-shaped blocks outside the two tuned shapes run on the general nested-tile kernel: other
    channel counts, filter extents, strides, image widths, ragged channel tiles, tiles that span rows and images.
    Position-sensitive first (a delta input reproduces the filter, exactly), then seeded data against the oracle."""
    N, H, Wd, Ci, Co, R, S, st, pad, dt = IGEMM_CASES[case]
    odt = "i32" if dt == "i8" else "f32"
    if tile == "256x128":   # the largest tile, which the selector keeps for blocks of 160 to 256 such tiles
        monkeypatch.setenv("STRIPE_TUNE", "conv_igemm_tn=128,conv_igemm_tm=256")
    elif tile == "128x128_k64":   # 64-byte K tile rows, which blocks of more than 256 tiles take also where 128-byte rows are possible
        monkeypatch.setenv("STRIPE_TUNE", "conv_igemm_tn=128,conv_igemm_tm=128,conv_igemm_kb=64")
    elif tile == "contraction_kernel":   # the 256 x 256-tile contraction kernel's convolution mode, chosen from 128 such tiles on
        monkeypatch.setenv("STRIPE_TUNE", "conv_gemm=2")
    blk = W.conv2d_block(N, H, Wd, Ci, Co, R, S, st, pad, dt, odt)
    Ho, Wo = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - S) // st + 1
    f = W.seeded_tensor((R, S, Co, Ci), dt, 1)
    i = torch.zeros((N, H, Wd, Ci), dtype=f.dtype)
    n0, y0, x0, c0 = N - 1, H // 2, Wd - 1, Ci - 3
    i[n0, y0, x0, c0] = 1
    gpu, sb = run_gpu(blk, [i, f], return_block=True)
    assert sb.info["path_name"] == "mfma_conv" and ("conv_igemm" in sb.info["kernel"] or tile == "contraction_kernel"), sb.info
    if tile == "contraction_kernel":   # bf16, the reduction a multiple of four 32-deep K tiles, every pixel written: else the general kernel
        takes = dt == "bf16" and (R * S * (Ci // 32)) % 4 == 0 and Co >= 8 and all(taps(y, st, pad, R, H) for y in range(Ho)) and all(taps(x, st, pad, S, Wd) for x in range(Wo))
        assert ("conv_gemm_bf16_256x256x32" in sb.info["kernel"]) == takes, sb.info
    assert tile != "256x128" or "_256x128x" in sb.info["kernel"], sb.info
    assert tile != "128x128_k64" or ("_128x128x64_" if dt == "i8" else "_128x128x32_") in sb.info["kernel"], sb.info
    say(f"conv family {case}: {sb.info['kernel']} grid {sb.info['grid']}")
    want = np.full((N, Ho, Wo, Co), float(SENTINEL_I) if dt == "i8" else float(np.float32(SENTINEL_F)), np.float64)
    for y in range(Ho):
        for x in range(Wo):
            if taps(y, st, pad, R, H) and taps(x, st, pad, S, Wd):        # else: no iteration writes this pixel
                want[:, y, x, :] = 0.0
            a, b = y0 - st * y + pad, x0 - st * x + pad
            if 0 <= a < R and 0 <= b < S:
                want[n0, y, x, :] = f[a, b, :, c0].double().numpy()
    assert np.array_equal(gpu.reshape(want.shape).astype(np.float64), want)
    ins = [W.seeded_tensor((N, H, Wd, Ci), dt, 0), f]
    parity(blk, ins, what=f"conv family {case}", threads=16, cache=_FAMILY_ORACLE, key=case)   # one oracle run per case, whatever the tile
    if dt == "i8":
        assert np.array_equal(run_gpu(blk, ins), run_gpu(blk, ins, "generic"))


def test_conv_family_dilated_and_strided_views():
    """A dilated 3x3 (taps two pixels apart), and a convolution whose tensors are windows of larger ones with more
    channels than the block uses (pixel strides larger than the channel count)."""
    N, H, Wd, Ci, Co = 2, 15, 13, 64, 48
    bufs = [W.Buffer("I", "in", "bf16", (N, H, Wd, Ci)), W.Buffer("F", "in", "bf16", (3, 3, Co, Ci)),
            W.Buffer("O", "out", "f32", (N, H, Wd, Co))]
    ya, xa = "y + 2*i - 2", "x + 2*j - 2"
    blk = W.flat_block(bufs, dict(n=N, y=H, x=Wd, i=3, j=3, c=Ci, k=Co),
                       [(["n", ya, xa, "c"], "assign"), (["i", "j", "k", "c"], "assign"), (["n", "y", "x", "k"], "add")],
                       constraints=[f"{ya} >= 0", f"{H + 1} - y - 2*i >= 0", f"{xa} >= 0", f"{Wd + 1} - x - 2*j >= 0"])
    ins = [W.seeded_tensor((N, H, Wd, Ci), "bf16", 0), W.seeded_tensor((3, 3, Co, Ci), "bf16", 1)]
    info, _ = parity(blk, ins, what="dilated conv")
    assert "conv_igemm" in info["kernel"], info
    ref = torch.nn.functional.conv2d(ins[0].float().permute(0, 3, 1, 2), ins[1].float().permute(2, 3, 0, 1), padding=2, dilation=2)
    gpu = run_gpu(blk, ins).reshape(N, H, Wd, Co)
    assert np.allclose(gpu, ref.permute(0, 2, 3, 1).numpy(), rtol=1e-3, atol=1e-2)
    blk = W.embed(W.conv2d_block(2, 10, 13, 32, 96, 3, 3, 1, 1, "bf16", "f32"), [(1, 2, 3, 64), (1, 0, 8, 32), (0, 1, 2, 4)],
                  [(3, 14, 20, 128), (4, 3, 112, 64), (2, 12, 18, 100)])
    ins = [W.seeded_tensor((3, 14, 20, 128), "bf16", 0), W.seeded_tensor((4, 3, 112, 64), "bf16", 1)]
    info, _ = parity(blk, ins, what="conv family windows")
    assert "conv_igemm" in info["kernel"], info


def test_conv_family_on_the_tuned_shapes(monkeypatch):
    """conv_tuned=0 sends the two benchmark shapes (small) through the general kernel too: same results as the tuned kernels."""
    blk = W.conv2d_block(2, 10, 13, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    ins = [W.seeded_tensor((2, 10, 13, 64), "bf16", 0), W.seeded_tensor((3, 3, 64, 64), "bf16", 1)]
    tuned = run_gpu(blk, ins)
    monkeypatch.setenv("STRIPE_TUNE", "conv_tuned=0")
    info, _ = parity(blk, ins, what="3x3 c64 on the general kernel")
    assert "conv_igemm" in info["kernel"], info
    assert np.allclose(run_gpu(blk, ins), tuned, rtol=1e-4, atol=1e-3)


# ------------------------------------------------------------------ convolution configs at full size
CONV_FAMILY_KERNELS = {   # the benchmark's shapes of the general kernel (one: of the contraction kernel) and the tile / K tile row the selectors give them
    "conv3x3_bf16_128to128": "_128x128x64_", "conv3x3_s2_bf16_64to128": "_128x128x64_", "conv1x7_bf16_64to64": "_256x64x32_",
    "conv3x3_bf16_w112": "_256x64x32_", "conv5x5_bf16_32to32": "_256x64x32_", "conv3x3_i8_64to64": "_256x64x64_",
    "conv3x3_bf16_128to192": "_256x128x32_", "conv3x3_bf16_128to256_56": "conv_gemm_bf16_256x256x32_", "conv3x3_bf16_256to256_56": "conv_gemm_bf16_256x256x32_",
}


@pytest.mark.parametrize("name", sorted(CONV_FAMILY_KERNELS))
def test_conv_family_bench_shapes_full_size(name):
    """The general kernel at the sizes and in the launch configurations bench.py times: all-ones operands give
    Ci * (taps inside the image) exactly on every element (pixels without any are left as they were); seeded data against the oracle on two whole images (the
    first, whose tiles start at pixel 0, and one in the middle, whose tiles straddle image borders; the two largest
    workloads: the middle one)."""
    N, H, Wd, Ci, Co, R, S, st, pad, dt = W.CONV_FAMILY[name]
    blk, ins = W.extra_block(name), W.extra_inputs(name)
    Ho, Wo = (H + 2 * pad - R) // st + 1, (Wd + 2 * pad - S) // st + 1
    ones = [torch.ones_like(ins[0]), torch.ones_like(ins[1])]
    gpu, sb = run_gpu(blk, ones, return_block=True)
    say(f"{name}: {sb.info['kernel']} grid {sb.info['grid']}")
    assert sb.info["path_name"] == "mfma_conv" and CONV_FAMILY_KERNELS[name] in sb.info["kernel"], sb.info
    cy = np.array([taps(y, st, pad, R, H) for y in range(Ho)])
    cx = np.array([taps(x, st, pad, S, Wd) for x in range(Wo)])
    want = float(Ci) * cy[:, None] * cx[None, :]
    want[want == 0] = float(SENTINEL_I) if dt == "i8" else float(np.float32(SENTINEL_F))   # no tap inside the image: no iteration writes the pixel
    assert np.array_equal(gpu.reshape(N, Ho, Wo, Co).astype(np.float64), np.broadcast_to(want[None, :, :, None], (N, Ho, Wo, Co)))
    gpu = run_gpu(blk, ins)
    np_ins = [W.to_numpy(t).ravel() for t in ins]
    np_abs = None if dt == "i8" else abs_inputs(np_ins, ["bf16", "bf16"])
    per_image = Ho * Wo * R * S * Ci * Co
    for n in ((0, N // 2 + 1) if per_image < 600e6 else (N // 2 + 1,)):      # (the largest: the middle image only)
        lo, hi = [n, 0, 0, 0, 0, 0, 0], [n + 1, Ho, Wo, R, S, Ci, Co]
        res = O.evaluate(blk, np_ins, window=(lo, hi), threads=16, split_index=1)
        ares = None if np_abs is None else O.evaluate(blk, np_abs, window=(lo, hi), threads=16, split_index=1)
        score = compare(blk, ins, gpu, res, what=f"{name} image {n}", abs_res=ares)
        say(f"  image {n}: err/bound {score:.3f}")


def test_resnet_conv_config_full_size():
    name = "resnet_conv_bf16"
    blk, ins = W.config_block(name), W.config_inputs(name)
    gpu, sb = run_gpu(blk, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']} grid {sb.info['grid']}")
    assert sb.info["work_points"] == 3611820032
    np_ins = [W.to_numpy(t).ravel() for t in ins]
    say("  oracle over the whole block (3.6 G points) ...")
    res = O.evaluate(blk, np_ins, threads=16, split_index=0)
    assert res.n_points == 3611820032 and res.touched.all()
    ares = O.evaluate(blk, abs_inputs(np_ins, ["bf16", "bf16"]), threads=16, split_index=0)
    score = compare(blk, ins, gpu, res, what=name, abs_res=ares)
    say(f"  every element: err/bound {score:.3f}")
    # all-ones: O = Ci * cy * cx exactly (in-bounds tap count), every element
    ones = [torch.ones_like(ins[0]), torch.ones_like(ins[1])]
    gpu = run_gpu(blk, ones).reshape(32, 56, 56, 64)
    cy = np.array([taps(y, 1, 1, 3, 56) for y in range(56)])
    want = 64.0 * cy[:, None] * cy[None, :]
    assert np.array_equal(gpu, np.broadcast_to(want[None, :, :, None], gpu.shape))


def test_tiled_generic_at_full_size():
    """The two convolution configurations on the register-tiled generic kernel (what a block gets when no
    matrix-core family fits): all-ones closed form on every element, int8 bit-exact against the matrix-core result,
    bf16 against an oracle window."""
    name = "resnet_conv_bf16"
    blk, ins = W.config_block(name), W.config_inputs(name)
    ones = [torch.ones_like(ins[0]), torch.ones_like(ins[1])]
    gpu, sb = run_gpu(blk, ones, "generic", return_block=True)
    assert sb.info["kernel"] == "generic_tiled_4x4_v4", sb.info["kernel"]
    cy = np.array([taps(y, 1, 1, 3, 56) for y in range(56)])
    want = 64.0 * cy[:, None] * cy[None, :]
    assert np.array_equal(gpu.reshape(32, 56, 56, 64), np.broadcast_to(want[None, :, :, None], (32, 56, 56, 64)))
    gpu = run_gpu(blk, ins, "generic")
    lo, hi = [13, 0, 50, 0, 0, 0, 0], [14, 56, 56, 3, 3, 64, 64]
    res = O.evaluate(blk, [W.to_numpy(t).ravel() for t in ins], window=(lo, hi), threads=16, split_index=1)
    compare(blk, ins, gpu, res, what="tiled generic resnet window")
    name = "conv7x7_s2_int8"
    blk, ins = W.config_block(name), W.config_inputs(name)
    a, sb = run_gpu(blk, ins, "generic", return_block=True)
    assert sb.info["kernel"] == "generic_tiled_4x4", sb.info["kernel"]
    assert np.array_equal(a, run_gpu(blk, ins))


def test_int8_conv_config_full_size():
    name = "conv7x7_s2_int8"
    blk, ins = W.config_block(name), W.config_inputs(name)
    gpu, sb = run_gpu(blk, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']} grid {sb.info['grid']}")
    assert sb.info["work_points"] == 1859432448
    np_ins = [W.to_numpy(t).ravel() for t in ins]
    say("  oracle over the whole block (1.9 G points) ...")
    res = O.evaluate(blk, np_ins, threads=16, split_index=0)
    assert res.n_points == 1859432448 and res.touched.all()
    compare(blk, ins, gpu, res, what=name)            # every element, bit-exact
    # all -128: O = 16384 * 3 * cy * cx exactly
    lowest = [torch.full_like(ins[0], -128), torch.full_like(ins[1], -128)]
    gpu = run_gpu(blk, lowest).reshape(16, 112, 112, 64)
    cy = np.array([taps(y, 2, 3, 7, 224) for y in range(112)])
    want = 16384 * 3 * cy[:, None] * cy[None, :]
    assert np.array_equal(gpu, np.broadcast_to(want[None, :, :, None], gpu.shape))


# ------------------------------------------------------------------ the benchmark's further workloads at full size
def _bands(extent, width):
    """Index bands at the start, around an unaligned middle and at the end."""
    if extent <= 3 * width:
        return [(0, extent)]
    mid = extent // 2 + 3
    return [(0, width), (mid, mid + width), (extent - width, extent)]


BENCH_FURTHER = ["gemm_bf16_4096_bt", "gemm_bf16_4000_ragged", "gemm_i8_4096_bt", "pointwise_conv_bf16", "transposed_conv_f32", "gemm_bf16_1024",
                 "gemm_bf16_2048", "gemm_bf16_256x256x65536", "gemm_i8_256x256x65536_bt", "gemm_bf16_1024x1024x8192", "depthwise3x3_f32",
                 "avgpool3x3s2_f32", "maxpool2x2s2_f32", "maxpool3x3s1_f32"]


@pytest.mark.parametrize("name", BENCH_FURTHER)
def test_bench_further_workloads_full_size(name):
    """bench.py's further single-statement workloads at the sizes and in the launch configurations it times, against
    the oracle on bands of the first index (for the products also of the second) that reach over every tile of the
    other indexes: first, an unaligned middle, last."""
    blk, ins = W.extra_block(name), W.extra_inputs(name)
    gpu, sb = run_gpu(blk, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']} grid {sb.info['grid']} path {sb.info['path_name']}")
    assert sb.info["path_name"] != "generic" or name == "transposed_conv_f32", sb.info
    lv = blk
    while not lv.idx_names:
        lv = lv.child
    ranges = list(lv.ranges)
    points = math.prod(ranges)
    np_ins = [W.to_numpy(t).ravel() for t in ins]
    in_dts = [r.dtype for r in blk.refs if r.dir == "in"]
    np_abs = abs_inputs(np_ins, in_dts) if in_dts[0] == "bf16" else None
    banded = [0, 1] if lv.idx_names[:3] == ["m", "n", "k"] else [0]
    for ax in banded:
        width = max(1, min(ranges[ax], int(3e8 / (points / ranges[ax]))))
        for a, b in _bands(ranges[ax], width):
            lo, hi = [0] * len(ranges), list(ranges)
            lo[ax], hi[ax] = a, b
            split = 1 if ax == 0 else 0          # the index the oracle's threads share out: an output index apart from the band's
            if name == "transposed_conv_f32":
                split = len(ranges) - 1          # O[2y+i, 2x+j]: y and i write the same elements, k does not
            res = O.evaluate(blk, np_ins, window=(lo, hi), threads=16, split_index=split)
            ares = None if np_abs is None else O.evaluate(blk, np_abs, window=(lo, hi), threads=16, split_index=split)
            score = compare(blk, ins, gpu, res, what=f"{name} index {ax} in [{a}, {b})", abs_res=ares)
            say(f"  index {lv.idx_names[ax]} in [{a}, {b}): {res.n_points} points, score {score:.3g}")


def test_bench_fused_programs_full_size(monkeypatch):
    """The two-statement workloads of bench.py beyond the ResNet-shaped one: the 128 -> 128 convolution + bias + relu
    on every element against the oracle's serial evaluation; the 4096^3 linear layer fused against the same
    program run as two launches (the product and the pointwise statement, each covered at full size on its own):
    the same sums in the same order, so equal bit for bit."""
    name = "conv3x3_bias_relu_bf16_128to128"
    prog, ins = W.extra_block(name), W.extra_inputs(name)
    fused, sb = run_gpu(prog, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']}")
    assert sb.info["kernel"].startswith("conv_igemm_bf16_") and sb.info["kernel"].endswith("+bias_relu_bf16"), sb.info["kernel"]
    res = O.evaluate_program(prog, [W.to_numpy(t).ravel() for t in ins], threads=16)
    assert res.touched.all()
    err = np.abs(fused.astype(np.float64) - res.out)
    tol = 4e-3 * math.sqrt(1152) * float(ins[0].float().abs().max()) * float(ins[1].float().abs().max()) + 2.0 ** -8 * np.abs(res.out)
    assert np.all(err <= tol), float(np.max(err - tol))
    assert (fused == 0).any() and (fused > 0).any()
    name = "linear_bias_relu_4096"
    prog, ins = W.extra_block(name), W.extra_inputs(name)
    fused, sb = run_gpu(prog, ins, return_block=True)
    say(f"{name}: {sb.info['kernel']}")
    assert "+bias_relu" in sb.info["kernel"] and " ; " not in sb.info["kernel"], sb.info["kernel"]
    monkeypatch.setenv("STRIPE_TUNE", "fuse=0")
    unfused, sb = run_gpu(prog, ins, return_block=True)
    assert " ; " in sb.info["kernel"], sb.info["kernel"]
    assert np.array_equal(fused, unfused)
    assert (fused == 0).any() and (fused > 0).any()


# ------------------------------------------------------------------ yardsticks
@pytest.mark.parametrize("from_lds", [False, True])
def test_matrix_core_yardstick_closed_form(from_lds):
    """All-ones operands: every accumulator element gains 16 per instruction (K = 16), a lane holds 256 elements."""
    iters, grid = 6, 3
    ops = torch.ones((16 * 256, 8), dtype=torch.bfloat16, device="cuda")
    out = torch.zeros(grid * 256, dtype=torch.float32, device="cuda")
    B.stripe_device_mfma(ops.data_ptr(), out.data_ptr(), iters, grid, torch.cuda.current_stream().cuda_stream, from_lds)
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 256 * 16 * iters)
    # two operand sets taking turns: set 0 ones, set 1 twos -> half of the passes contribute 4 x 16
    ops2 = ops.clone().reshape(2, 8 * 256, 8)
    ops2[1] = 2.0
    B.stripe_device_mfma(ops2.data_ptr(), out.data_ptr(), iters, grid, torch.cuda.current_stream().cuda_stream, from_lds)
    torch.cuda.synchronize()
    assert np.all(out.cpu().numpy() == 256 * 16 * (iters // 2) * (1 + 4))
    with pytest.raises(B.StripeError):
        B.stripe_device_mfma(ops.data_ptr(), out.data_ptr(), 3, grid)        # odd pass count


def test_streaming_yardstick_sums_its_streams():
    n16 = 1000
    src = torch.arange(4 * n16 * 4, dtype=torch.float32, device="cuda")
    dst = torch.zeros(n16 * 4, dtype=torch.float32, device="cuda")
    B.stripe_device_stream(src.data_ptr(), dst.data_ptr(), n16, 4, 1, 7, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    want = src.reshape(4, n16 * 4).sum(dim=0)
    assert torch.equal(dst, want)
