"""A second evaluator for tiny blocks, written differently from the C oracle.

It walks the joint product of all levels' index ranges at once, substitutes
passed values by hand, collects {output address: [values]} in a dictionary
and only then reduces each list.  Exact Python integers / fractions, so it
can be compared with the oracle for equality.  Used to pin the oracle
(Definition 2, rule 3) on inputs small enough to enumerate; also generates
random tiny blocks whose accesses are in bounds by construction.
"""
from __future__ import annotations

import itertools
import random
from fractions import Fraction
from functools import reduce

from paper_1903_06498_amd import workloads as W


def _dot(coeffs, vals, const):
    return const + sum(c * v for c, v in zip(coeffs, vals))


def enumerate_points(root):
    """Yield (addresses per refinement) of every executed leaf point."""
    levels = root.levels()[1:]
    all_ranges = [range(r) for lv in levels for r in lv.ranges]
    for joint in itertools.product(*all_ranges):
        pos, parent_vars, ok = 0, [], True
        per_level_vars = []
        for lv in levels:
            own = list(joint[pos:pos + len(lv.ranges)])
            pos += len(lv.ranges)
            passed = [_dot(co, parent_vars, c0) for co, c0 in zip(lv.passed_coeff, lv.passed_const)]
            vars_ = own + passed
            if any(_dot(co, vars_, c0) < 0 for co, c0 in zip(lv.cons_coeff, lv.cons_const)):
                ok = False
                break
            per_level_vars.append(vars_)
            parent_vars = vars_
        if not ok:
            continue
        addrs = []
        for r in range(len(root.refs)):
            top = root.refs[r]
            a = sum(s * c for s, c in zip(top.strides, top.access_const))
            for lv, vars_ in zip(levels, per_level_vars):
                ref = lv.refs[r]
                for d in range(len(ref.sizes)):
                    a += ref.strides[d] * _dot(ref.access_coeff[d], vars_, ref.access_const[d])
            addrs.append(a)
        yield addrs


def evaluate(root, inputs, exact=lambda v: Fraction(v)):
    """{output address: aggregated value}; inputs are flat sequences."""
    leaf = root.levels()[-1]
    aggs = {lv.refs[-1].agg for lv in root.levels()} - {"assign"}
    agg = aggs.pop() if aggs else "assign"
    written = {}
    for addrs in enumerate_points(root):
        a = exact(inputs[0][addrs[0]])
        if leaf.intrinsic == "copy":
            v = a
        else:
            b = exact(inputs[1][addrs[1]])
            v = a * b if leaf.intrinsic == "mul" else a + b
        written.setdefault(addrs[-1], []).append(v)
    ops = {"add": lambda x, y: x + y, "mul": lambda x, y: x * y, "max": max, "min": min}
    out = {}
    for e, vals in written.items():
        if len(vals) == 1:
            out[e] = vals[0]
        else:
            assert agg != "assign", "two writers under assign"
            out[e] = reduce(ops[agg], vals)
    return out


def random_block(rng: random.Random, nested: bool, dtype_in="i8", dtype_out="i32", agg="add", intrinsic="mul",
                 injective_out=False, max_range=4, contraction_roles=False, root_origin=0):
    """A random tiny block (every range <= 4, small integer coefficients).

    With injective_out every output dimension is moved by exactly one index
    (the shape the GPU library accepts without atomics).
    With contraction_roles (needs injective_out and two inputs) every output index is given a role as in a
    tensor contraction: it moves the first input only, the second input only, or both; the other indexes
    are reduction indexes.  Coefficients, signs and constraints stay random.
    With root_origin > 0 every buffer is declared as a window of a larger tensor: the root refinement gets a
    random origin in 0..root_origin per dimension and the strides are those of a parent tensor that holds the
    window at that origin (plus a little slack).
    Accesses are made in-bounds by measuring, per buffer dimension, the
    extreme coordinates over the executed points and sizing/offsetting the
    root buffer to contain them.  Views of intermediate levels are sized the
    same way, so that every view check of the oracle is exercised and passes.
    """
    n_in = 1 if intrinsic == "copy" else 2
    ndims = [rng.randint(1, 3) for _ in range(n_in + 1)]
    names = ["A", "B"][:n_in] + ["O"]
    dirs = ["in"] * n_in + ["out"]
    dts = [dtype_in] * n_in + [dtype_out]

    n_levels = 2 if nested else 1
    shapes = []
    for li in range(n_levels):
        n_idx = rng.randint(1, 3 if nested else 4)
        ranges = [rng.randint(1, max_range if not nested else max(2, max_range - 1)) for _ in range(n_idx)]
        n_passed = rng.randint(0, 2) if li > 0 else 0
        shapes.append((n_idx, ranges, n_passed))

    out_dim_of = {}   # (level, index) -> output dimension, when the output map is made injective
    if injective_out:
        cand = [(li, j) for li, (n_idx, _, _) in enumerate(shapes) for j in range(n_idx)]
        rng.shuffle(cand)
        chosen = cand[:rng.randint(2 if (contraction_roles and len(cand) >= 2) else 1, min(3, len(cand)))]
        for d, key in enumerate(chosen):
            out_dim_of[key] = d
        ndims[n_in] = len(chosen)
    role_of = {key: rng.choice(["first", "first", "second", "second", "both"]) for key in out_dim_of} if contraction_roles else {}
    if contraction_roles and len(out_dim_of) >= 2:      # at least one index of each one-sided role
        keys = list(out_dim_of)
        role_of[keys[0]], role_of[keys[1]] = "first", "second"

    def rand_level(li, var_count):
        acc = [[[rng.randint(-1, 2) for _ in range(var_count)] for _ in range(nd)] for nd in ndims]
        if injective_out:
            acc[n_in] = [[0] * var_count for _ in range(ndims[n_in])]
            for (l2, j), d in out_dim_of.items():
                if l2 == li:
                    acc[n_in][d][j] = rng.choice([1, 1, 2, -1])
                    if contraction_roles and n_in == 2:
                        silent = 1 if role_of[(l2, j)] == "first" else 0 if role_of[(l2, j)] == "second" else None
                        if silent is not None:
                            for row in acc[silent]:
                                row[j] = 0
        return acc

    lv_specs = []
    parent_nv = 0
    for li in range(n_levels):
        n_idx, ranges, n_passed = shapes[li]
        passed_coeff = [[rng.randint(-1, 2) for _ in range(parent_nv)] for _ in range(n_passed)]
        passed_const = [rng.randint(-1, 1) for _ in range(n_passed)]
        nv = n_idx + n_passed
        n_cons = rng.randint(0, 2)
        cons_coeff = [[rng.randint(-1, 1) for _ in range(nv)] for _ in range(n_cons)]
        if contraction_roles:                           # keep the constraints off the second input's own indexes
            for row in cons_coeff:
                for (l2, j), role in role_of.items():
                    if l2 == li and role == "second":
                        row[j] = 0
        cons_const = [rng.randint(0, 3) for _ in range(n_cons)]
        lv_specs.append(dict(n_idx=n_idx, ranges=ranges, passed_coeff=passed_coeff, passed_const=passed_const,
                             cons_coeff=cons_coeff, cons_const=cons_const, acc=rand_level(li, nv)))
        parent_nv = nv

    origin = [[rng.randint(0, root_origin) for _ in range(nd)] for nd in ndims]
    slack = [[rng.randint(0, 1) if root_origin else 0 for _ in range(nd)] for nd in ndims]

    # Build with provisional sizes, measure extremes, then fix sizes and offsets.
    def build(root_sizes, root_off, mid_sizes, mid_off):
        parent = [[n + o + s for n, o, s in zip(root_sizes[r], origin[r], slack[r])] for r in range(n_in + 1)]
        levels = []
        for li, sp in enumerate(lv_specs):
            refs = []
            for r in range(n_in + 1):
                nd = ndims[r]
                const = [0] * nd
                if li == 0:
                    const = [root_off[r][d] for d in range(nd)]
                if li == 1:
                    const = [mid_off[r][d] for d in range(nd)]
                sizes = [1] * nd if li == n_levels - 1 else mid_sizes[r]
                lv_agg = agg if r == n_in else "assign"
                refs.append(W.Refinement(names[r], dirs[r], dts[r], lv_agg, sp["acc"][r], const, list(sizes),
                                         W.contiguous_strides(parent[r])))
            b = W.Block(idx_names=[f"i{li}_{j}" for j in range(sp["n_idx"])], ranges=sp["ranges"],
                        passed_names=[f"p{li}_{j}" for j in range(len(sp["passed_coeff"]))],
                        passed_coeff=sp["passed_coeff"], passed_const=sp["passed_const"],
                        cons_coeff=sp["cons_coeff"], cons_const=sp["cons_const"], refs=refs)
            levels.append(b)
        levels[-1].intrinsic = intrinsic
        for a, b in zip(levels, levels[1:]):
            a.child = b
        root = W.Block(idx_names=[], ranges=[])
        for r in range(n_in + 1):
            nd = ndims[r]
            root.refs.append(W.Refinement(names[r], dirs[r], dts[r], "assign", [[] for _ in range(nd)], list(origin[r]),
                                          list(root_sizes[r]), W.contiguous_strides(parent[r])))
        root.child = levels[0]
        return root

    big = [[64] * nd for nd in ndims]
    zero = [[0] * nd for nd in ndims]
    probe = build(big, zero, big, zero)
    # Extremes of the total coordinate and of the inner level's own coordinate.
    levels = probe.levels()[1:]
    tot_lo = [[None] * nd for nd in ndims]
    tot_hi = [[None] * nd for nd in ndims]
    in_lo = [[None] * nd for nd in ndims]
    in_hi = [[None] * nd for nd in ndims]
    any_point = False
    all_ranges = [range(r) for lv in levels for r in lv.ranges]
    for joint in itertools.product(*all_ranges):
        pos, parent_vars, ok, per = 0, [], True, []
        for lv in levels:
            own = list(joint[pos:pos + len(lv.ranges)])
            pos += len(lv.ranges)
            vars_ = own + [_dot(co, parent_vars, c0) for co, c0 in zip(lv.passed_coeff, lv.passed_const)]
            if any(_dot(co, vars_, c0) < 0 for co, c0 in zip(lv.cons_coeff, lv.cons_const)):
                ok = False
                break
            per.append(vars_)
            parent_vars = vars_
        if not ok:
            continue
        any_point = True
        for r in range(n_in + 1):
            for d in range(ndims[r]):
                cs = [_dot(lv.refs[r].access_coeff[d], v, 0) for lv, v in zip(levels, per)]
                t, inner = sum(cs), cs[-1]
                tot_lo[r][d] = t if tot_lo[r][d] is None else min(tot_lo[r][d], t)
                tot_hi[r][d] = t if tot_hi[r][d] is None else max(tot_hi[r][d], t)
                in_lo[r][d] = inner if in_lo[r][d] is None else min(in_lo[r][d], inner)
                in_hi[r][d] = inner if in_hi[r][d] is None else max(in_hi[r][d], inner)
    if not any_point:
        return random_block(rng, nested, dtype_in, dtype_out, agg, intrinsic, injective_out, max_range, contraction_roles, root_origin)
    if nested:
        # The inner level's constant places its coordinate at the start of the
        # outer level's view; the outer level's constant places the total
        # coordinate at the start of the buffer.
        mid_off = [[-in_lo[r][d] for d in range(ndims[r])] for r in range(n_in + 1)]
        mid_sizes = [[in_hi[r][d] - in_lo[r][d] + 1 for d in range(ndims[r])] for r in range(n_in + 1)]
        # total coordinate after shifting = t + root_off + mid_off, must start at 0
        root_off = [[-tot_lo[r][d] - mid_off[r][d] for d in range(ndims[r])] for r in range(n_in + 1)]
    else:
        mid_off = zero
        mid_sizes = big
        root_off = [[-tot_lo[r][d] for d in range(ndims[r])] for r in range(n_in + 1)]
    root_sizes = [[tot_hi[r][d] - tot_lo[r][d] + 1 for d in range(ndims[r])] for r in range(n_in + 1)]
    return build(root_sizes, root_off, mid_sizes, mid_off)
