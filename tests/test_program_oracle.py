"""Pins for the oracle's statement lists (a root block with several statements and temporaries, Section 3.2) and
the add_relu leaf: closed forms, an integer library reference (exact), an fp64 library reference, error cases,
and agreement with the single-statement path.  CPU only; nothing here touches the HIP library."""
import numpy as np
import pytest
import torch

from oracle import stripe_oracle as O
from paper_1903_06498_amd import workloads as W


def taps(y, s, p, R, H):
    return sum(1 for i in range(R) if 0 <= s * y + i - p < H)


def test_all_ones_closed_form_with_relu_cut():
    """I = F = 1: T[n,y,x,k] = Ci * (taps in y) * (taps in x).  Bias -k*8 cuts some channels to zero exactly."""
    N, H, Wd, Ci, Co, R, s, p = 2, 7, 6, 3, 5, 3, 1, 1
    prog = W.conv_bias_relu_program(N, H, Wd, Ci, Co, R, R, s, p, "f32", "f32")
    bias = -8.0 * np.arange(Co, dtype=np.float32)
    res = O.evaluate_program(prog, [np.ones(N * H * Wd * Ci, np.float32), np.ones(R * R * Co * Ci, np.float32), bias])
    cy = np.array([taps(y, s, p, R, H) for y in range(H)])
    cx = np.array([taps(x, s, p, R, Wd) for x in range(Wd)])
    t = Ci * cy[:, None] * cx[None, :]
    want = np.maximum(t[None, :, :, None] + bias[None, None, None, :], 0.0) * np.ones((N, 1, 1, 1))
    assert res.touched.all() and np.array_equal(res.out.reshape(want.shape), want)
    assert (want == 0).any() and (want > 0).any()          # the cut is exercised on both sides


@pytest.mark.parametrize("stride,pad", [(1, 1), (2, 0), (2, 2)])
def test_integer_program_matches_integer_library_reference_exactly(stride, pad):
    N, H, Wd, Ci, Co, R = 2, 9, 8, 4, 6, 3
    prog = W.conv_bias_relu_program(N, H, Wd, Ci, Co, R, R, stride, pad, "i8", "i32")
    rng = np.random.default_rng(5)
    i = rng.integers(-128, 128, (N, H, Wd, Ci), dtype=np.int8)
    f = rng.integers(-128, 128, (R, R, Co, Ci), dtype=np.int8)
    b = rng.integers(-30000, 30000, (Co,), dtype=np.int32)
    res = O.evaluate_program(prog, [i.ravel(), f.ravel(), b])
    ref = torch.nn.functional.conv2d(torch.from_numpy(i.astype(np.int64)).permute(0, 3, 1, 2),
                                     torch.from_numpy(f.astype(np.int64)).permute(2, 3, 0, 1), stride=stride, padding=pad)
    ref = torch.clamp(ref + torch.from_numpy(b.astype(np.int64))[None, :, None, None], min=0).permute(0, 2, 3, 1).numpy()
    assert np.array_equal(res.out.reshape(ref.shape), ref)


def test_float_program_matches_fp64_library_reference():
    """The temporary is declared f32: the oracle rounds the first statement's fp64 sums to fp32 before the second
    statement reads them, and so does the reference."""
    N, H, Wd, Ci, Co, R = 2, 10, 7, 6, 5, 3
    prog = W.conv_bias_relu_program(N, H, Wd, Ci, Co, R, R, 1, 1, "bf16", "bf16")
    i, f = W.seeded_tensor((N, H, Wd, Ci), "bf16", 0), W.seeded_tensor((R, R, Co, Ci), "bf16", 1)
    b = W.seeded_tensor((Co,), "f32", 2)
    res = O.evaluate_program(prog, [W.to_numpy(i).ravel(), W.to_numpy(f).ravel(), b.numpy()])
    t = torch.nn.functional.conv2d(i.double().permute(0, 3, 1, 2), f.double().permute(2, 3, 0, 1), padding=1).float().double()
    ref = torch.relu(t + b.double()[None, :, None, None]).permute(0, 2, 3, 1).numpy()
    got = res.out.reshape(ref.shape)
    # identical up to the rare temporary whose fp64 sum sits within a summation-order error of an fp32 rounding boundary
    assert np.max(np.abs(got - ref)) <= 2.0 ** -22 * max(1.0, np.max(np.abs(ref)))
    assert np.mean(got == ref) > 0.99


def test_single_statement_program_is_the_plain_block():
    blk = W.conv2d_block(1, 6, 5, 3, 4, 3, 3, 1, 1, "f32", "f32")
    ins = [W.seeded_tensor((1, 6, 5, 3), "f32", 0).numpy().ravel(), W.seeded_tensor((3, 3, 4, 3), "f32", 1).numpy().ravel()]
    a, b = O.evaluate(blk, ins), O.evaluate_program(blk, ins)
    assert np.array_equal(a.out, b.out) and np.array_equal(a.touched, b.touched) and a.n_points == b.n_points


def test_reading_a_temporary_nobody_wrote_is_an_error():
    prog = W.conv_bias_relu_program(1, 5, 5, 2, 3, 3, 3, 1, 1, "f32", "f32")
    first, second = prog.child, prog.child.next
    prog.child, second.next = second, None                   # only the second statement: T was never written
    with pytest.raises(O.OracleError):
        O.evaluate_program(prog, [np.zeros(50, np.float32), np.zeros(54, np.float32), np.zeros(3, np.float32)])
    partial = W.conv_bias_relu_program(1, 5, 5, 2, 3, 3, 3, 1, 1, "f32", "f32")
    partial.child.ranges[1] = 4                              # the convolution now leaves a row of T unwritten
    with pytest.raises(O.OracleError):
        O.evaluate_program(partial, [np.zeros(50, np.float32), np.zeros(54, np.float32), np.zeros(3, np.float32)])
