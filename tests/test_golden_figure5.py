"""The block descriptions used for the Figure 5 pins are the paper's: every number the figure prints (ranges,
constraint rows, access rows, view sizes, strides) is stored in tests/golden/figure5_facts.txt in a tabular
notation of this repository and compared here with what workloads.fig5_flat / fig5_tiled build.  CPU only."""
import os
import re

from paper_1903_06498_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "figure5_facts.txt")


def facts():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        if line.startswith("buffer"):
            _, name, direction, dtype, rest = line.split(None, 4)
            sizes, strides = rest.split("strides")
            out.setdefault("buffers", {})[name] = (direction, dtype, [int(v) for v in sizes.replace("sizes", "").split()],
                                                   [int(v) for v in strides.split()])
            continue
        key, body = re.match(r"\[(.+?)\]\s*(.*)", line).groups()
        out.setdefault(key, []).append(body)
    return out


def rows(body):
    """'a b c | k ; ...' -> ([[a, b, c], ...], [k, ...])"""
    coeff, const = [], []
    for part in body.split(";"):
        words = part.split()
        if words and not re.match(r"-?\d+$", words[0]):
            words = words[1:]                       # a passed value's name
        bar = words.index("|")
        coeff.append([int(v) for v in words[:bar]])
        const.append(int(words[bar + 1]))
    return coeff, const


def indexes(body):
    w = body.split()
    return w[0::2], [int(v) for v in w[1::2]]


def check_refs(level, f, prefix, views=None):
    for ref, name in zip(level.refs, "IFO"):
        coeff, const = rows(f[f"{prefix} access {name}"][0])
        assert ref.access_coeff == coeff and ref.access_const == const, (prefix, name)
        assert ref.strides == f["buffers"][name][3]
        if views:
            assert ref.sizes == [int(v) for v in f[f"{prefix} view {name}"][0].split()]
        else:
            assert ref.sizes == [1] * len(ref.sizes)          # scalar views at the leaf


def test_declaring_block_matches_the_figure():
    f = facts()
    for blk in (W.fig5_flat("i8", "i8"), W.fig5_tiled("i8", "i8")):
        assert blk.ranges == [] and blk.child is not None       # a root without indexes, one iteration
        for ref, name in zip(blk.refs, "IFO"):
            direction, dtype, sizes, strides = f["buffers"][name]
            assert (ref.dir, ref.dtype, ref.sizes, ref.strides) == (direction, dtype, sizes, strides)
            assert ref.access_const == [0] * len(sizes)


def test_flat_form_matches_figure_5a():
    f = facts()
    names, ranges = indexes(f["5a indexes"][0])
    for typo, last in ((True, "5a constraint printed"), (False, "5a constraint read")):
        leaf = W.fig5_flat(printed_typo=typo).child
        assert leaf.idx_names == names and leaf.ranges == ranges and leaf.child is None
        want = [rows(b) for b in f["5a constraint"]] + [rows(f[last][0])]
        assert leaf.cons_coeff == [c[0] for c, _ in want] and leaf.cons_const == [k[0] for _, k in want]
        check_refs(leaf, f, "5a")
        assert leaf.refs[-1].agg == f["5a aggregation"][0] and leaf.intrinsic == f["5a leaf"][0]


def test_tiled_form_matches_figure_5b():
    f = facts()
    outer = W.fig5_tiled().child
    inner = outer.child
    names, ranges = indexes(f["5b outer indexes"][0])
    assert outer.idx_names == names and outer.ranges == ranges and outer.cons_coeff == []
    check_refs(outer, f, "5b outer", views=True)
    names, ranges = indexes(f["5b inner indexes"][0])
    assert inner.idx_names == names and inner.ranges == ranges and inner.child is None
    pc, pk = rows(f["5b passed"][0])
    assert inner.passed_names == ["xo", "yo"] and inner.passed_coeff == pc and inner.passed_const == pk
    want = [rows(b) for b in f["5b inner constraint"]]
    assert inner.cons_coeff == [c[0] for c, _ in want] and inner.cons_const == [k[0] for _, k in want]
    check_refs(inner, f, "5b inner")
    # the tile of 5b: outer range x inner range covers the flat range exactly, the input view overlaps by the halo
    flat = dict(zip(*indexes(f["5a indexes"][0])))
    for n, ro, ri in zip(names, outer.ranges, inner.ranges):
        assert ro * ri == flat[n]
    assert outer.refs[0].sizes[0] == inner.ranges[0] + 2 and outer.refs[0].sizes[1] == inner.ranges[1] + 2
