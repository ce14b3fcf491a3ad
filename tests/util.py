"""Helpers shared by the GPU parity tests: upload, run through the C ABI, compare.

Tolerances (stated once, used everywhere):
  integer blocks      bit-exact
  max / min blocks    exact equality of values (order-independent operation)
  fp32-input blocks   max |g - r| / max(|r|, rms(r)) <= 1e-4 against the fp64 oracle
  bf16-input blocks   |g - r| <= 4e-3 * sqrt(K) * max|a| * max|b|, K = reduction points per output
  bf16 output buffers the above plus 2^-8 * |r| (one rounding to bf16 on store; the oracle returns the unrounded value)
Elements no iteration writes must keep the sentinel the output was filled with.

Regression guard for bf16 sums of products (not the pass/fail bar, which stays the tolerance above): products of
bf16 values are exact in fp32, so all of the error is fp32 accumulation, which is bounded per element by
    MODEL_FACTOR * K * 2^-24 * sum |a * b|      (K terms, unit roundoff 2^-24, any summation order)
with sum |a * b| taken from a second oracle run on the inputs' absolute values.  At K = 4096 with N(0,1) inputs
this is about 0.7, an order of magnitude below the stated tolerance (about 6), so a dropped or doubled K tile,
which the tolerance alone would let through, fails here.
"""
from __future__ import annotations

import math

import numpy as np
import torch

from oracle import stripe_oracle as O
from paper_1903_06498_amd import binding as B
from paper_1903_06498_amd import workloads as W

SENTINEL_I = -123456789
SENTINEL_F = -9.87654321e30

_TORCH = {"i8": torch.int8, "i32": torch.int32, "bf16": torch.bfloat16, "f32": torch.float32}


def run_gpu(root, inputs, path="auto", return_block=False):
    """inputs: torch CPU tensors in the declared element types.  Returns the flat output image (numpy)."""
    dev = torch.device("cuda:0")
    blk = B.StripeBlock(root, path)
    ext = W.output_extent(root)
    odt = root.refs[-1].dtype
    out = torch.full((ext,), SENTINEL_I if odt == "i32" else SENTINEL_F, dtype=_TORCH[odt], device=dev)
    dins = []
    for r, t in zip(root.refs[:-1], inputs):
        assert t.dtype == _TORCH[r.dtype], (r.name, t.dtype)
        dins.append(t.contiguous().to(dev))
    blk.run(dins, out)
    torch.cuda.synchronize()
    res = (out.float() if odt == "bf16" else out).cpu().numpy()
    if return_block:
        return res, blk
    blk.close()
    return res


def reduction_points(root) -> int:
    """Hull reduction points per output element: product of ranges of indexes the output does not depend on."""
    k = 1
    for lv in root.levels()[1:]:
        o = lv.refs[-1]
        for j, rng in enumerate(lv.ranges):
            if all(row[j] == 0 for row in o.access_coeff):
                k *= rng
    return k


MODEL_FACTOR = 1.0


def abs_inputs(np_inputs, dtypes):
    """The inputs with every element replaced by its absolute value (bf16 travels as bit patterns)."""
    return [(a & np.uint16(0x7FFF)) if dt == "bf16" else np.abs(a) for a, dt in zip(np_inputs, dtypes)]


def is_sum_of_products(root) -> bool:
    agg = {lv.refs[-1].agg for lv in root.levels()} - {"assign"}
    return root.levels()[-1].intrinsic == "mul" and agg <= {"add"}


def compare(root, inputs, gpu_out, oracle_res, what="", abs_res=None):
    """Element-by-element comparison on the touched set; sentinel check on the rest.  abs_res: the oracle's
    result on the inputs' absolute values (same window), for the accumulation-error guard of bf16 blocks."""
    touched = oracle_res.touched.astype(bool)
    odt = root.refs[-1].dtype
    agg = {lv.refs[-1].agg for lv in root.levels()} - {"assign"}
    agg = agg.pop() if agg else "assign"
    g, r = gpu_out[touched], oracle_res.out[touched]
    if odt == "i32":
        assert np.array_equal(g.astype(np.int64), r), f"{what}: integer block not bit-exact"
        return 0.0
    in_dt = root.refs[0].dtype
    if agg in ("max", "min") and root.levels()[-1].intrinsic == "copy":
        assert np.array_equal(g.astype(np.float64), r), f"{what}: max/min block not exact"
        return 0.0
    err = np.abs(g.astype(np.float64) - r)
    if in_dt == "bf16":
        K = reduction_points(root)
        amax = max(float(np.max(np.abs(t.float().numpy()))) for t in inputs[:1])
        bmax = float(np.max(np.abs(inputs[1].float().numpy()))) if len(inputs) > 1 else 1.0
        bound = 4e-3 * math.sqrt(K) * amax * bmax
        if odt == "bf16":
            err = np.maximum(err - 2.0 ** -8 * np.abs(r), 0.0)
        assert err.max() <= bound, f"{what}: bf16 error {err.max():.3e} > bound {bound:.3e}"
        if abs_res is not None:
            model = MODEL_FACTOR * K * 2.0 ** -24 * abs_res.out[touched] + 1e-30
            worst = float(np.max(err / model))
            assert worst <= 1.0, f"{what}: fp32 accumulation error is {worst:.2f} x the model K * 2^-24 * sum|a*b|"
        return float(err.max() / bound)
    rms = math.sqrt(float(np.mean(r * r))) if r.size else 1.0
    rel = err / np.maximum(np.abs(r), rms if rms > 0 else 1.0)
    assert rel.max() <= 1e-4, f"{what}: fp32 relative error {rel.max():.3e} > 1e-4"
    return float(rel.max())


def check_untouched(gpu_out, oracle_res, odt):
    untouched = ~oracle_res.touched.astype(bool)
    if untouched.any():
        want = SENTINEL_I if odt == "i32" else np.float32(SENTINEL_F)
        assert np.all(gpu_out[untouched] == want), "an element no iteration writes was modified"


def parity(root, inputs, path="auto", window=None, threads=8, split_index=0, what="", cache=None, key=None):
    """Run GPU and oracle on the same inputs and compare.  With a window the
    oracle computes only a slab of outputs and only that slab is compared.
    cache / key: a dict that keeps the oracle's results for tests that run one block and one set of inputs through
    several kernel variants (the oracle does not depend on the variant; the GPU side runs every time)."""
    gpu, blk = run_gpu(root, inputs, path, return_block=True)
    info = dict(blk.info)
    blk.close()
    if cache is not None and key in cache:
        res, abs_res = cache[key]
    else:
        np_ins = [W.to_numpy(t).ravel() for t in inputs]
        res = O.evaluate(root, np_ins, window=window, threads=threads, split_index=split_index)
        abs_res = None
        if root.refs[0].dtype == "bf16" and is_sum_of_products(root):
            abs_res = O.evaluate(root, abs_inputs(np_ins, [r.dtype for r in root.refs[:-1]]), window=window, threads=threads,
                                 split_index=split_index)
        if cache is not None:
            cache[key] = (res, abs_res)
    score = compare(root, inputs, gpu, res, what, abs_res)
    if window is None:
        check_untouched(gpu, res, root.refs[-1].dtype)
    return info, score
