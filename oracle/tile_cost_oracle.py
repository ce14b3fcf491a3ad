"""Brute-force oracle for the autotiling cost model (paper Section 3.3, Figure 4's caption).

TEST INFRASTRUCTURE ONLY: imported by tests/ (and nothing in the product path).  Shares no code with the
HIP library's closed-form cost; it counts by enumeration.

What is counted, for one tile of a flat block:
  * every point of the tile's index box is visited (tiled indexes 0..tile-1, the others over their whole
    range), constraints ignored: the figure shows tiles "including overflows", whose accesses the
    constraints remove at run time but which still cost;
  * for every counted tensor the coordinates the accesses reach give, per dimension, a lowest and a highest
    value; the tile's view is that box (the sizes Figure 5b prints for the middle block);
  * footprint = elements of the views; lines = the views' elements grouped along the stride-1 dimension
    into lines of `line_elems` starting at the view's origin, counted by inserting every element's line
    into a set;
  * tiles = product over indexes of ceil(range / tile); work = product of the ranges of the tiled indexes;
  * cost = tiles * lines / work.

Pinned by the two costs Figure 4 prints for admissible tiles (4.5 and 4.666) and by the tile it shows as excluded.
The figure's fourth cost, 5.625, is not reproduced by any tile under this reading of the caption: parity unpinned
for that one number.
"""
from itertools import product


def tile_cost(root, tile, line_elems, mem_cap_elems, counted_refs, tiled_idx):
    leaf = root.child
    assert root.ranges == [] and leaf.child is None, "flat form expected"
    n = len(leaf.ranges)
    box = [range(tile[j]) for j in range(n)]
    lows, highs = {}, {}
    for point in product(*box):
        for r in counted_refs:
            ref = leaf.refs[r]
            for d in range(len(ref.sizes)):
                v = sum(ref.access_coeff[d][j] * point[j] for j in range(n))     # relative to the tile's origin
                key = (r, d)
                lows[key] = min(lows.get(key, v), v)
                highs[key] = max(highs.get(key, v), v)
    footprint, lines = 0, 0
    for r in counted_refs:
        ref = leaf.refs[r]
        nd = len(ref.sizes)
        extents = [highs[(r, d)] - lows[(r, d)] + 1 for d in range(nd)]
        line_dim = [d for d in range(nd) if abs(ref.strides[d]) == 1]
        line_dim = line_dim[-1] if line_dim else None
        seen = set()
        count = 0
        for coord in product(*[range(e) for e in extents]):
            count += 1
            seen.add(tuple(c // line_elems if d == line_dim else c for d, c in enumerate(coord)))
        footprint += count
        lines += len(seen)
    tiles, work = 1, 1
    for j in range(n):
        tiles *= -(-leaf.ranges[j] // tile[j])
        if j in tiled_idx:
            work *= leaf.ranges[j]
    return {"tiles": tiles, "lines_per_tile": lines, "footprint_elems": footprint, "work": work,
            "cost": tiles * lines / work, "admissible": int(mem_cap_elems <= 0 or footprint <= mem_cap_elems)}
