"""stripe_block_run_static (the entry point for callers that cannot allocate device memory) against
stripe_block_run and the oracle: statement lists whose temporaries live in the library's static scratch array.
Two calls in a row on one GPU, the second with a smaller input, so stale contents of the shared array would show."""
import math

import numpy as np
import pytest
import torch

from oracle import stripe_oracle as O
from paper_1903_06498_amd import binding as B
from paper_1903_06498_amd import workloads as W

pytestmark = pytest.mark.gpu


def _program_case(N, H, Wd, Ci, Co, in_dt, out_dt):
    prog = W.conv_bias_relu_program(N, H, Wd, Ci, Co, 3, 3, 1, 1, in_dt, out_dt)
    acc = "i32" if in_dt == "i8" else "f32"
    ins = [W.seeded_tensor((N, H, Wd, Ci), in_dt, 0), W.seeded_tensor((3, 3, Co, Ci), in_dt, 1)]
    ins.append((W.seeded_tensor((Co,), "i32", 2) * 30) if acc == "i32" else W.seeded_tensor((Co,), "f32", 2))
    return prog, ins


def _run_both(prog, ins):
    """(output of stripe_block_run_static, output of stripe_block_run, kernel names) on fresh sentinel-filled outputs."""
    dev = torch.device("cuda:0")
    odt = {"i32": torch.int32, "f32": torch.float32, "bf16": torch.bfloat16}[prog.refs[-1].dtype]
    ext = W.output_extent(prog)
    dins = [t.contiguous().to(dev) for t in ins]
    sb = B.StripeBlock(prog)
    outs = []
    for fn in (sb.run_static, sb.run):
        out = torch.full((ext,), -7, dtype=odt, device=dev)
        fn(dins, out)
        torch.cuda.synchronize()
        outs.append((out.float() if odt == torch.bfloat16 else out).cpu().numpy())
    kernel = sb.info["kernel"]
    sb.close()
    return outs[0], outs[1], kernel


def _check_against_oracle(prog, ins, got, in_dt):
    res = O.evaluate_program(prog, [W.to_numpy(t).ravel() for t in ins], threads=4)
    assert res.touched.all()
    if prog.refs[-1].dtype == "i32":
        assert np.array_equal(got.astype(np.int64), res.out)          # integer blocks: bit-exact
        return
    err = np.abs(got.astype(np.float64) - res.out)
    rms = max(1.0, float(np.sqrt(np.mean(res.out ** 2))))
    K = 9 * ins[0].shape[-1]
    tol = 1e-4 * rms if in_dt == "f32" else 4e-3 * math.sqrt(K) * float(ins[0].float().abs().max()) * float(ins[1].float().abs().max())
    assert np.all(err <= tol), float(err.max())


@pytest.mark.parametrize("in_dt,out_dt", [("f32", "f32"), ("i8", "i32")])
def test_static_scratch_two_calls_second_smaller(in_dt, out_dt):
    """A larger program, then a smaller one, both through the static scratch: each equals the allocating entry
    point's result exactly (same kernels, same order of operations) and matches the oracle."""
    for shape in [(2, 19, 14, 5, 12), (1, 6, 5, 3, 4)]:
        prog, ins = _program_case(*shape, in_dt, out_dt)
        static, plain, kernel = _run_both(prog, ins)
        assert " ; " in kernel, kernel                               # two launches through a real temporary
        assert np.array_equal(static, plain), f"{shape}: static-scratch result differs from stripe_block_run"
        _check_against_oracle(prog, ins, static, in_dt)


def test_static_scratch_serves_single_blocks_and_fused_programs_without_scratch():
    blk = W.matmul_block(256, 256, 128, "bf16", "f32")
    ins = [W.seeded_tensor((256, 128), "bf16", 0), W.seeded_tensor((128, 256), "bf16", 1)]
    static, plain, _ = _run_both(blk, ins)
    assert np.array_equal(static, plain)
    prog = W.conv_bias_relu_program(1, 7, 20, 64, 64, 3, 3, 1, 1, "bf16", "f32")
    ins = [W.seeded_tensor((1, 7, 20, 64), "bf16", 0), (W.seeded_tensor((3, 3, 64, 64), "bf16", 1).float() / 24).to(torch.bfloat16),
           W.seeded_tensor((64,), "f32", 2)]
    static, plain, kernel = _run_both(prog, ins)
    assert "+bias_relu" in kernel and np.array_equal(static, plain)


def test_static_scratch_rejects_temporaries_beyond_its_size():
    """A temporary of 16 MiB does not fit the 8 MiB array: a clear error, nothing launched, and the allocating
    entry point still runs the same handle."""
    prog, ins = _program_case(4, 128, 128, 4, 64, "f32", "f32")         # temporary: 4*128*128*64 f32 = 16 MiB
    dev = torch.device("cuda:0")
    dins = [t.to(dev) for t in ins]
    out = torch.full((W.output_extent(prog),), -7.0, dtype=torch.float32, device=dev)
    sb = B.StripeBlock(prog)
    with pytest.raises(B.StripeError) as e:
        sb.run_static(dins, out)
    assert e.value.status == 7 and "static scratch" in str(e.value)
    torch.cuda.synchronize()
    assert torch.all(out == -7.0)                                       # nothing ran
    sb.run(dins, out)
    torch.cuda.synchronize()
    assert not torch.any(out == -7.0)
    sb.close()
