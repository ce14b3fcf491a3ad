// Host-side planner: see plan.hpp.  Follows the paper's block definition
// (Section 3.2) and nesting rule (Section 3.1.3): refinement offsets compose
// down the nest, parent indexes enter a child only as passed affine values.
#include "plan.hpp"

#include <algorithm>
#include <cstdio>
#include <cstring>

namespace stripe {

namespace {

using i128 = __int128;

Affine zero_affine() {
  Affine a;
  std::memset(&a, 0, sizeof a);
  return a;
}

void add_scaled(Affine* dst, const Affine& src, int64_t s) {
  for (int j = 0; j < kMaxFlatIdx; ++j) dst->c[j] += s * src.c[j];
  dst->k += s * src.k;
}

bool same_affine(const Affine& a, const Affine& b, int n) {
  if (a.k != b.k) return false;
  for (int j = 0; j < n; ++j)
    if (a.c[j] != b.c[j]) return false;
  return true;
}

i128 lo_of(const FlatBlock& fb, const Affine& a) {
  i128 v = a.k;
  for (int j = 0; j < fb.n_idx; ++j)
    if (a.c[j] < 0) v += (i128)a.c[j] * (fb.range[j] - 1);
  return v;
}

i128 hi_of(const FlatBlock& fb, const Affine& a) {
  i128 v = a.k;
  for (int j = 0; j < fb.n_idx; ++j)
    if (a.c[j] > 0) v += (i128)a.c[j] * (fb.range[j] - 1);
  return v;
}

int64_t eval(const Affine& a, const int64_t* idx, int n) {
  int64_t v = a.k;
  for (int j = 0; j < n; ++j) v += a.c[j] * idx[j];
  return v;
}

std::string fmt(const char* f, long long a = 0, long long b = 0, long long c = 0) {
  char buf[256];
  std::snprintf(buf, sizeof buf, f, a, b, c);
  return buf;
}

stripe_status_t bad(std::string* err, stripe_status_t st, const std::string& msg) {
  if (err) *err = msg;
  return st;
}

bool is_int_type(int dt) { return dt == STRIPE_I8 || dt == STRIPE_I32; }

int dtype_bytes(int dt) { return dt == STRIPE_I8 ? 1 : dt == STRIPE_BF16 ? 2 : 4; }

// Enumerate the indexes in `sel` (others fixed at 0) and call f(idx); stops early when f returns false.
template <typename F>
bool for_each_point(const FlatBlock& fb, const std::vector<int>& sel, F f) {
  int64_t idx[kMaxFlatIdx] = {};
  for (int j : sel)
    if (fb.range[j] <= 0) return true;
  for (;;) {
    if (!f(idx)) return false;
    size_t p = 0;
    for (; p < sel.size(); ++p) {
      const int j = sel[p];
      if (++idx[j] < fb.range[j]) break;
      idx[j] = 0;
    }
    if (p == sel.size()) return true;
  }
}

// Is `a >= 0` at every point of the polyhedron?  Interval bound first, then the
// bound relative to one constraint (a = cons + (a - cons) with cons >= 0), then
// enumeration of the indexes involved when that is small.
bool prove_nonneg(const FlatBlock& fb, const Affine& a) {
  if (lo_of(fb, a) >= 0) return true;
  for (const Affine& q : fb.cons) {
    Affine d = a;
    add_scaled(&d, q, -1);
    if (lo_of(fb, d) >= 0) return true;
  }
  std::vector<bool> used(fb.n_idx, false);
  for (int j = 0; j < fb.n_idx; ++j)
    if (a.c[j]) used[j] = true;
  for (const Affine& q : fb.cons)
    for (int j = 0; j < fb.n_idx; ++j)
      if (q.c[j]) used[j] = true;
  std::vector<int> sel;
  i128 pts = 1;
  for (int j = 0; j < fb.n_idx; ++j)
    if (used[j]) {
      sel.push_back(j);
      pts *= fb.range[j];
      if (pts > ((i128)1 << 24)) return false;
    }
  return for_each_point(fb, sel, [&](const int64_t* idx) {
    for (const Affine& q : fb.cons)
      if (eval(q, idx, fb.n_idx) < 0) return true;  // not in the polyhedron
    return eval(a, idx, fb.n_idx) >= 0;
  });
}

}  // namespace

// --------------------------------------------------------------------------
// Descriptor -> flat form
// --------------------------------------------------------------------------
stripe_status_t flatten(const stripe_block_desc_t* root, FlatBlock* fb, std::string* err) {
  const stripe_block_desc_t* lvl[kMaxLevels];
  int L = 0;
  for (const stripe_block_desc_t* b = root; b; b = b->child) {
    if (L == kMaxLevels) return bad(err, STRIPE_ERR_INVALID_DESC, "nest deeper than 7 block levels");
    lvl[L++] = b;
  }
  if (L < 2) return bad(err, STRIPE_ERR_INVALID_DESC, "need the declaring root block and at least one block below it");
  if (root->n_idx != 0 || root->n_passed != 0 || root->n_constraints != 0)
    return bad(err, STRIPE_ERR_INVALID_DESC, "the root block only declares buffers: no indexes, passed values or constraints");
  const int R = root->n_refs;
  if (R < 2 || R > kMaxRefs) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement count %lld: expected 2 or 3", R));
  if (!root->refs) return bad(err, STRIPE_ERR_NULL, "root refs is NULL");

  *fb = FlatBlock();
  fb->n_refs = R;
  fb->n_levels = L;
  const stripe_block_desc_t* leaf = lvl[L - 1];
  fb->intrinsic = leaf->intrinsic;
  if (leaf->intrinsic != STRIPE_INTR_MUL && leaf->intrinsic != STRIPE_INTR_COPY && leaf->intrinsic != STRIPE_INTR_ADD &&
      leaf->intrinsic != STRIPE_INTR_ADD_RELU)
    return bad(err, STRIPE_ERR_INVALID_DESC, "unknown intrinsic");
  if ((leaf->intrinsic == STRIPE_INTR_COPY ? 1 : 2) != R - 1)
    return bad(err, STRIPE_ERR_INVALID_DESC, "COPY takes one input, MUL and ADD take two");

  // Buffers as declared at the root.
  for (int r = 0; r < R; ++r) {
    const stripe_refinement_t& t = root->refs[r];
    FlatRef& f = fb->ref[r];
    if (t.ndim < 1 || t.ndim > kMaxDims) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement %lld: ndim out of 1..8", r));
    if (!t.access_const || !t.sizes || !t.strides) return bad(err, STRIPE_ERR_NULL, fmt("refinement %lld: NULL array at the root", r));
    if (t.dir != (r == R - 1 ? STRIPE_OUT : STRIPE_IN))
      return bad(err, STRIPE_ERR_INVALID_DESC, "inputs come first, the single output last");
    if (t.dtype < STRIPE_I8 || t.dtype > STRIPE_F32) return bad(err, STRIPE_ERR_INVALID_DESC, "unknown element type");
    f.dir = t.dir;
    f.dtype = t.dtype;
    f.ndim = t.ndim;
    f.elements = 1;
    f.addr = zero_affine();
    for (int d = 0; d < t.ndim; ++d) {
      if (t.sizes[d] < 1 || t.sizes[d] > ((int64_t)1 << 40)) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement %lld dim %lld: bad size", r, d));
      if (t.strides[d] < 0 || t.strides[d] > ((int64_t)1 << 40)) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement %lld dim %lld: bad stride", r, d));
      if (t.access_const[d] < 0 || t.access_const[d] > ((int64_t)1 << 40)) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement %lld dim %lld: bad root offset", r, d));
      f.sizes[d] = t.sizes[d];
      f.strides[d] = t.strides[d];
      f.coord[d] = zero_affine();
      f.addr.k += t.strides[d] * t.access_const[d];
      f.elements *= t.sizes[d];
      if (f.elements > ((int64_t)1 << 46)) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("refinement %lld: buffer too large", r));
    }
  }
  const int odt = fb->ref[R - 1].dtype;
  if (odt != STRIPE_I32 && odt != STRIPE_F32 && odt != STRIPE_BF16) return bad(err, STRIPE_ERR_INVALID_DESC, "the output is i32, f32 or bf16");
  fb->int_mode = (odt == STRIPE_I32);
  fb->out_bf16 = (odt == STRIPE_BF16);
  for (int r = 0; r + 1 < R; ++r) {
    if (is_int_type(fb->ref[r].dtype) != fb->int_mode)
      return bad(err, STRIPE_ERR_INVALID_DESC, "integer inputs need an i32 output, float inputs an f32 or bf16 output");
    if (fb->ref[r].dtype != fb->ref[0].dtype)
      return bad(err, STRIPE_ERR_UNSUPPORTED, "both inputs must have the same element type");
  }

  // Walk the nest.  vars[l][v] = value of variable v of level l as an affine
  // function of the flat indexes; rel[l][r][d] = this level's own access.
  std::vector<std::vector<Affine>> vars(L);
  std::vector<Affine> level_coord((size_t)L * R * kMaxDims, zero_affine());
  auto LC = [&](int l, int r, int d) -> Affine& { return level_coord[((size_t)l * R + r) * kMaxDims + d]; };
  fb->agg = STRIPE_AGG_ASSIGN;
  for (int l = 0; l < L; ++l) {
    const stripe_block_desc_t* b = lvl[l];
    if (b->n_refs != R || !b->refs) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld: every level lists the root's buffers", l));
    if (b->n_idx < 0 || b->n_passed < 0 || b->n_constraints < 0) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld: negative count", l));
    if (b->n_idx && !b->ranges) return bad(err, STRIPE_ERR_NULL, fmt("level %lld: ranges is NULL", l));
    if (b->n_passed && (!b->passed_coeff || l == 0)) return bad(err, STRIPE_ERR_NULL, fmt("level %lld: passed_coeff is NULL", l));
    if (b->n_constraints && (!b->cons_coeff || !b->cons_const)) return bad(err, STRIPE_ERR_NULL, fmt("level %lld: constraint arrays are NULL", l));
    const int nv = b->n_idx + b->n_passed;
    if (nv > kMaxFlatIdx) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld: too many variables", l));
    vars[l].assign(nv, zero_affine());
    for (int j = 0; j < b->n_idx; ++j) {
      if (fb->n_idx == kMaxFlatIdx) return bad(err, STRIPE_ERR_UNSUPPORTED, "more than 24 indexes in the nest");
      if (b->ranges[j] < 0 || b->ranges[j] > 0x7fffffffLL) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld index %lld: range out of 0..2^31-1", l, j));
      const int f = fb->n_idx++;
      fb->range[f] = b->ranges[j];
      fb->level_of[f] = l;
      if (b->ranges[j] == 0) fb->empty = true;
      vars[l][j].c[f] = 1;
    }
    const int pnv = l ? lvl[l - 1]->n_idx + lvl[l - 1]->n_passed : 0;
    for (int p = 0; p < b->n_passed; ++p) {
      Affine a = zero_affine();
      a.k = b->passed_const ? b->passed_const[p] : 0;
      for (int v = 0; v < pnv; ++v) {
        const int64_t co = b->passed_coeff[(size_t)p * pnv + v];
        if (co > 0x7fffffffLL || co < -0x7fffffffLL) return bad(err, STRIPE_ERR_INVALID_DESC, "coefficient out of range");
        add_scaled(&a, vars[l - 1][v], co);
      }
      vars[l][b->n_idx + p] = a;
    }
    for (int q = 0; q < b->n_constraints; ++q) {
      Affine a = zero_affine();
      a.k = b->cons_const[q];
      for (int v = 0; v < nv; ++v) {
        const int64_t co = b->cons_coeff[(size_t)q * nv + v];
        if (co > 0x7fffffffLL || co < -0x7fffffffLL) return bad(err, STRIPE_ERR_INVALID_DESC, "coefficient out of range");
        add_scaled(&a, vars[l][v], co);
      }
      fb->cons.push_back(a);
    }
    for (int r = 0; r < R; ++r) {
      const stripe_refinement_t& t = b->refs[r];
      const stripe_refinement_t& top = root->refs[r];
      if (t.ndim != top.ndim || t.dtype != top.dtype || t.dir != top.dir)
        return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld refinement %lld: shape, type or direction differs from the root", l, r));
      if (!t.access_const || !t.sizes || !t.strides || (nv && !t.access_coeff))
        return bad(err, STRIPE_ERR_NULL, fmt("level %lld refinement %lld: NULL array", l, r));
      for (int d = 0; d < t.ndim; ++d) {
        if (t.strides[d] != top.strides[d]) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld refinement %lld: a view keeps its parent's strides", l, r));
        if (t.sizes[d] < 1) return bad(err, STRIPE_ERR_INVALID_DESC, fmt("level %lld refinement %lld: view sizes are positive", l, r));
        if (l == 0) continue;  // the root's constant is the buffer origin, already in addr.k
        Affine a = zero_affine();
        a.k = t.access_const[d];
        for (int v = 0; v < nv; ++v) {
          const int64_t co = t.access_coeff[(size_t)d * nv + v];
          if (co > 0x7fffffffLL || co < -0x7fffffffLL) return bad(err, STRIPE_ERR_INVALID_DESC, "coefficient out of range");
          add_scaled(&a, vars[l][v], co);
        }
        LC(l, r, d) = a;
      }
    }
    const int a = b->refs[R - 1].agg;
    if (a < STRIPE_AGG_ASSIGN || a > STRIPE_AGG_MUL) return bad(err, STRIPE_ERR_INVALID_DESC, "unknown aggregation");
    fb->level_agg[l] = a;
    if (a != STRIPE_AGG_ASSIGN) {
      if (fb->agg != STRIPE_AGG_ASSIGN && fb->agg != a)
        return bad(err, STRIPE_ERR_INVALID_DESC, "every level carries the nest's one aggregation operation or assign");
      fb->agg = a;
    }
  }

  // Absolute coordinates, addresses, and the containment checks of every enclosing view.
  for (int r = 0; r < R; ++r) {
    FlatRef& f = fb->ref[r];
    for (int d = 0; d < f.ndim; ++d) {
      Affine suffix = zero_affine();
      for (int l = L - 1; l >= 1; --l) {
        add_scaled(&suffix, LC(l, r, d), 1);
        RangeCheck ck;
        ck.rel = suffix;                      // sum of the accesses of levels l..leaf
        ck.size = lvl[l - 1]->refs[r].sizes[d];  // inside the view level l-1 handed on
        ck.ref = r;
        ck.dim = d;
        ck.level = l - 1;
        fb->checks.push_back(ck);
      }
      f.coord[d] = suffix;
      add_scaled(&f.addr, suffix, f.strides[d]);
    }
  }
  return STRIPE_OK;
}

// --------------------------------------------------------------------------
// Every executed access stays inside its buffer and inside every enclosing view.
// --------------------------------------------------------------------------
stripe_status_t prove_checks(const FlatBlock& fb, std::string* err) {
  if (fb.empty) return STRIPE_OK;
  for (const RangeCheck& ck : fb.checks) {
    if (hi_of(fb, ck.rel) > ((i128)1 << 60) || lo_of(fb, ck.rel) < -((i128)1 << 60))
      return bad(err, STRIPE_ERR_INVALID_DESC, "access coordinate overflows");
    Affine up = zero_affine();
    add_scaled(&up, ck.rel, -1);
    up.k += ck.size - 1;
    if (!prove_nonneg(fb, ck.rel) || !prove_nonneg(fb, up))
      return bad(err, STRIPE_ERR_OUT_OF_BOUNDS,
                 fmt("refinement %lld dim %lld: cannot prove the access stays inside the view of level %lld", ck.ref, ck.dim, ck.level));
  }
  return STRIPE_OK;
}

// A level whose output aggregation is 'assign' promises that its iterations
// write disjoint elements (Section 3.2).  Accepted when every index of that
// level (range > 1) moves the output address; together with the injectivity
// of the output map on those indexes (checked by make_plan) that is a proof.
stripe_status_t check_assign_levels(const FlatBlock& fb, std::string* err) {
  if (fb.empty) return STRIPE_OK;
  const Affine& o = fb.ref[fb.n_refs - 1].addr;
  for (int j = 0; j < fb.n_idx; ++j) {
    const int l = fb.level_of[j];
    if (fb.level_agg[l] == STRIPE_AGG_ASSIGN && fb.range[j] > 1 && o.c[j] == 0)
      return bad(err, STRIPE_ERR_ASSIGN_CONFLICT,
                 fmt("level %lld is 'assign' but one of its indexes (range %lld) does not move the output address", l, fb.range[j]));
  }
  return STRIPE_OK;
}

// --------------------------------------------------------------------------
// Canonical form: drop range-1 indexes, merge index pairs that every map uses
// as outer*range+inner (what a tiling pass splits), fold single-index
// constraints into ranges, drop constraints the ranges already imply.
// A tiled nest and its un-tiled form end up identical.
// --------------------------------------------------------------------------
namespace {

template <typename F>
void for_each_row(FlatBlock* fb, F f) {
  for (Affine& q : fb->cons) f(q);
  for (int r = 0; r < fb->n_refs; ++r) {
    for (int d = 0; d < fb->ref[r].ndim; ++d) f(fb->ref[r].coord[d]);
    f(fb->ref[r].addr);
  }
}

void remove_index(FlatBlock* fb, int j) {
  for_each_row(fb, [&](Affine& a) {
    for (int t = j; t + 1 < kMaxFlatIdx; ++t) a.c[t] = a.c[t + 1];
    a.c[kMaxFlatIdx - 1] = 0;
  });
  for (int t = j; t + 1 < fb->n_idx; ++t) {
    fb->range[t] = fb->range[t + 1];
    fb->level_of[t] = fb->level_of[t + 1];
  }
  fb->n_idx--;
}

bool try_merge(FlatBlock* fb) {
  for (int a = 0; a < fb->n_idx; ++a)
    for (int b = 0; b < fb->n_idx; ++b) {
      if (a == b) continue;
      if ((i128)fb->range[a] * fb->range[b] > 0x7fffffffLL) continue;
      bool ok = true, used = false;
      for_each_row(fb, [&](Affine& r) {
        if (r.c[a] != r.c[b] * fb->range[b]) ok = false;
        if (r.c[b]) used = true;
      });
      if (!ok || !used) continue;
      fb->range[b] *= fb->range[a];  // idx_b' = idx_a * range_b + idx_b keeps coefficient c[b]
      fb->level_of[b] = 0;
      remove_index(fb, a);
      return true;
    }
  return false;
}

bool fold_and_prune(FlatBlock* fb) {
  bool changed = false;
  for (size_t q = 0; q < fb->cons.size();) {
    Affine& c = fb->cons[q];
    int nz = 0, j = -1;
    for (int t = 0; t < fb->n_idx; ++t)
      if (c.c[t]) {
        ++nz;
        j = t;
      }
    bool drop = false;
    if (nz == 0) {
      if (c.k < 0) fb->empty = true;
      drop = true;
    } else if (nz == 1) {
      const int64_t co = c.c[j];
      if (co > 0) {  // idx >= ceil(-k / co)
        int64_t lo = (-c.k + co - 1) / co;
        if (-c.k <= 0) lo = 0;
        if (lo > 0) {
          if (lo >= fb->range[j]) {
            fb->empty = true;
          } else {
            for_each_row(fb, [&](Affine& r) { r.k += r.c[j] * lo; });  // idx = idx' + lo
            fb->range[j] -= lo;
          }
        }
      } else {  // idx <= floor(k / -co)
        if (c.k < 0) {
          fb->empty = true;
        } else {
          const int64_t ub = c.k / (-co);
          if (ub + 1 < fb->range[j]) fb->range[j] = ub + 1;
        }
      }
      drop = true;
    } else if (lo_of(*fb, c) >= 0) {
      drop = true;
    } else if (hi_of(*fb, c) < 0) {
      fb->empty = true;
      drop = true;
    }
    if (drop) {
      fb->cons.erase(fb->cons.begin() + q);
      changed = true;
    } else {
      ++q;
    }
    if (fb->empty) return false;
  }
  // identical constraints once
  for (size_t a = 0; a < fb->cons.size(); ++a)
    for (size_t b = a + 1; b < fb->cons.size();)
      if (same_affine(fb->cons[a], fb->cons[b], fb->n_idx)) {
        fb->cons.erase(fb->cons.begin() + b);
        changed = true;
      } else {
        ++b;
      }
  return changed;
}

}  // namespace

void canonicalize(FlatBlock* fb) {
  fb->checks.clear();
  if (fb->empty) return;
  for (int guard = 0; guard < 256; ++guard) {
    bool changed = false;
    for (int j = 0; j < fb->n_idx;) {
      if (fb->range[j] == 1) {
        remove_index(fb, j);
        changed = true;
      } else {
        ++j;
      }
    }
    if (fold_and_prune(fb)) changed = true;
    if (fb->empty) return;
    if (try_merge(fb)) changed = true;
    if (!changed) break;
  }
}

// --------------------------------------------------------------------------
// Counting the polyhedron's points: enumerate only the indexes constraints mention.
// --------------------------------------------------------------------------
int64_t count_points(const FlatBlock& fb, int64_t cap) {
  if (fb.empty) return 0;
  std::vector<int> sel;
  i128 rest = 1, pts = 1;
  for (int j = 0; j < fb.n_idx; ++j) {
    bool used = false;
    for (const Affine& q : fb.cons)
      if (q.c[j]) used = true;
    if (used) {
      sel.push_back(j);
      pts *= fb.range[j];
      if (pts > cap) return -1;
    } else {
      rest *= fb.range[j];
    }
  }
  int64_t n = 0;
  for_each_point(fb, sel, [&](const int64_t* idx) {
    for (const Affine& q : fb.cons)
      if (eval(q, idx, fb.n_idx) < 0) return true;
    ++n;
    return true;
  });
  const i128 total = rest * n;
  return total > (((i128)1) << 62) ? -1 : (int64_t)total;
}

// --------------------------------------------------------------------------
// Shape matchers for the specialised kernel families.  Strict: a block that
// is not exactly of the shape falls through to the generic kernel.
// --------------------------------------------------------------------------
namespace {

int single_term(const Affine& a, int n, int64_t* coef) {  // index of the only non-zero coefficient, -1 if none, -2 if several
  int j = -1;
  for (int t = 0; t < n; ++t)
    if (a.c[t]) {
      if (j >= 0) return -2;
      j = t;
    }
  if (j >= 0 && coef) *coef = a.c[j];
  return j;
}

struct Window2d {  // roles of the indexes of  X[n, sy*y + dy*i - py, sx*x + dx*j - px, c]
  int n = -1, y = -1, x = -1, c = -1, i = -1, j = -1;
  int64_t sy = 1, sx = 1, py = 0, px = 0, dy = 1, dx = 1;
  int64_t H = 1, W = 1, st_n = 0, st_y = 0, st_x = 0, st_c = 0;
};

bool match_window(const FlatBlock& fb, const FlatRef& in, const Affine& out_addr, Window2d* w) {
  if (in.ndim != 3 && in.ndim != 4) return false;
  const int nd = in.ndim;
  const int dy = nd - 3, dx = nd - 2, dc = nd - 1;
  int64_t co = 0;
  if (nd == 4) {
    if (in.coord[0].k != 0) return false;
    const int t = single_term(in.coord[0], fb.n_idx, &co);
    if (t == -2 || (t >= 0 && co != 1)) return false;
    w->n = t;
    w->st_n = in.strides[0];
  }
  {
    if (in.coord[dc].k != 0) return false;
    const int t = single_term(in.coord[dc], fb.n_idx, &co);
    if (t == -2 || (t >= 0 && co != 1)) return false;
    w->c = t;
    w->st_c = in.strides[dc];
  }
  for (int pass = 0; pass < 2; ++pass) {
    const int d = pass ? dx : dy;
    const Affine& a = in.coord[d];
    int o = -1, r = -1;
    int64_t s = 1, dil = 1;
    for (int t = 0; t < fb.n_idx; ++t) {
      if (!a.c[t]) continue;
      if (out_addr.c[t]) {  // an output index: the window's position
        if (o >= 0 || a.c[t] < 1) return false;
        o = t;
        s = a.c[t];
      } else {              // a reduction index: the tap (coefficient = dilation)
        if (r >= 0 || a.c[t] < 1) return false;
        r = t;
        dil = a.c[t];
      }
    }
    if (a.k > 0) return false;
    if (pass) {
      w->x = o; w->j = r; w->sx = s; w->dx = dil; w->px = -a.k; w->W = in.sizes[d]; w->st_x = in.strides[d];
    } else {
      w->y = o; w->i = r; w->sy = s; w->dy = dil; w->py = -a.k; w->H = in.sizes[d]; w->st_y = in.strides[d];
    }
  }
  // Constraints may only be the window's own bounds: coord >= 0 or size-1-coord >= 0.
  for (const Affine& q : fb.cons) {
    bool ok = false;
    for (int pass = 0; pass < 2 && !ok; ++pass) {
      const int d = pass ? dx : dy;
      Affine up = zero_affine();
      add_scaled(&up, in.coord[d], -1);
      up.k += in.sizes[d] - 1;
      if (same_affine(q, in.coord[d], fb.n_idx) || same_affine(q, up, fb.n_idx)) ok = true;
    }
    if (!ok) return false;
  }
  return true;
}

int64_t range_or_1(const FlatBlock& fb, int j) { return j >= 0 ? fb.range[j] : 1; }

bool distinct(std::initializer_list<int> ids) {
  std::vector<int> v;
  for (int t : ids)
    if (t >= 0) v.push_back(t);
  std::sort(v.begin(), v.end());
  return std::adjacent_find(v.begin(), v.end()) == v.end();
}

}  // namespace

// The block as its three address maps see it.  Indexes that all of them use as outer*range + inner are one index
// as far as addresses go, even when they are separate buffer dimensions (the pixels n, y, x of dense NHWC
// tensors): such pairs are merged until none is left or `target` indexes remain.  Constraint-free blocks only.
void address_form(const FlatBlock& fb, size_t target, std::vector<int64_t>* rng, std::vector<int64_t>* ca, std::vector<int64_t>* cb,
                  std::vector<int64_t>* cc) {
  rng->assign(fb.range, fb.range + fb.n_idx);
  ca->assign(fb.ref[0].addr.c, fb.ref[0].addr.c + fb.n_idx);
  cb->assign(fb.ref[1].addr.c, fb.ref[1].addr.c + fb.n_idx);
  cc->assign(fb.ref[2].addr.c, fb.ref[2].addr.c + fb.n_idx);
  for (bool merged = true; merged && rng->size() > target;) {
    merged = false;
    for (size_t o = 0; o < rng->size() && !merged; ++o)
      for (size_t i = 0; i < rng->size() && !merged; ++i) {
        if (o == i) continue;
        auto nests = [&](const std::vector<int64_t>& x) { return (i128)x[o] == (i128)x[i] * (*rng)[i]; };
        if (nests(*ca) && nests(*cb) && nests(*cc) && (i128)(*rng)[i] * (*rng)[o] < ((i128)1 << 62)) {
          (*rng)[i] *= (*rng)[o];
          for (auto* v : {rng, ca, cb, cc}) v->erase(v->begin() + o);
          merged = true;
        }
      }
  }
}

bool match_gemm(const FlatBlock& fb, GemmShape* g) {
  if (fb.empty || fb.n_refs != 3 || fb.intrinsic != STRIPE_INTR_MUL || fb.agg != STRIPE_AGG_ADD) return false;
  if (fb.n_idx < 3 || !fb.cons.empty()) return false;
  std::vector<int64_t> rng, ca, cb, cc;
  address_form(fb, 3, &rng, &ca, &cb, &cc);
  g->batch = 1;
  g->a_b = g->b_b = g->c_b = 0;
  if (rng.size() == 4) {   // one more index that moves all three operands: a batch of independent products
    int bi = -1;
    for (int j = 0; j < 4; ++j)
      if (ca[j] && cb[j] && cc[j]) bi = bi < 0 ? j : 4;
    if (bi < 0 || bi > 3 || ca[bi] < 0 || cb[bi] < 0 || cc[bi] < 0) return false;
    g->batch = rng[bi];
    g->a_b = ca[bi]; g->b_b = cb[bi]; g->c_b = cc[bi];
    for (auto* v : {&rng, &ca, &cb, &cc}) v->erase(v->begin() + bi);
  }
  if (rng.size() != 3) return false;
  int m = -1, n = -1, k = -1;
  for (int j = 0; j < 3; ++j) {
    if (cc[j] == 0) {
      if (k >= 0) return false;
      k = j;
    } else if (ca[j] && !cb[j]) {
      if (m >= 0) return false;
      m = j;
    } else if (cb[j] && !ca[j]) {
      if (n >= 0) return false;
      n = j;
    } else {
      return false;
    }
  }
  if (m < 0 || n < 0 || k < 0 || !ca[k] || !cb[k]) return false;
  g->M = rng[m]; g->N = rng[n]; g->K = rng[k];
  g->a_m = ca[m]; g->a_k = ca[k]; g->b_k = cb[k]; g->b_n = cb[n]; g->c_m = cc[m]; g->c_n = cc[n];
  g->a_base = fb.ref[0].addr.k; g->b_base = fb.ref[1].addr.k; g->c_base = fb.ref[2].addr.k;
  return g->a_m > 0 && g->a_k > 0 && g->b_k > 0 && g->b_n > 0 && g->c_m > 0 && g->c_n > 0;
}

bool match_conv2d(const FlatBlock& fb, Conv2dShape* c) {
  if (fb.empty || fb.n_refs != 3 || fb.intrinsic != STRIPE_INTR_MUL || fb.agg != STRIPE_AGG_ADD) return false;
  const FlatRef &I = fb.ref[0], &F = fb.ref[1], &O = fb.ref[2];
  Window2d w;
  if (!match_window(fb, I, O.addr, &w)) return false;
  // The filter: one dimension per role, each a single index with coefficient 1.
  int k = -1;
  int64_t f_r = 0, f_s = 0, f_k = 0, f_c = 0;
  for (int d = 0; d < F.ndim; ++d) {
    if (F.coord[d].k != 0) return false;
    int64_t co = 0;
    const int t = single_term(F.coord[d], fb.n_idx, &co);
    if (t == -2 || (t >= 0 && co != 1)) return false;
    if (t < 0) continue;
    if (t == w.i) f_r = F.strides[d];
    else if (t == w.j) f_s = F.strides[d];
    else if (t == w.c) f_c = F.strides[d];
    else if (O.addr.c[t] && !I.addr.c[t] && k < 0) { k = t; f_k = F.strides[d]; }
    else return false;
  }
  if (k < 0) return false;
  if (!distinct({w.n, w.y, w.x, w.c, w.i, w.j, k})) return false;
  int used = 0;
  for (int t : {w.n, w.y, w.x, w.c, w.i, w.j, k})
    if (t >= 0) ++used;
  if (used != fb.n_idx) return false;
  // Reduction indexes must reach the filter, window positions must not; the output takes n, y, x, k.
  for (int t : {w.i, w.j, w.c})
    if (t >= 0 && (F.addr.c[t] == 0 || O.addr.c[t] != 0)) return false;
  for (int t : {w.n, w.y, w.x})
    if (t >= 0 && (F.addr.c[t] != 0 || O.addr.c[t] <= 0)) return false;
  if (w.y < 0 || w.x < 0 || w.c < 0) return false;
  c->N = range_or_1(fb, w.n); c->Ho = fb.range[w.y]; c->Wo = fb.range[w.x]; c->Co = fb.range[k];
  c->R = range_or_1(fb, w.i); c->S = range_or_1(fb, w.j); c->Ci = fb.range[w.c];
  c->H = w.H; c->W = w.W;
  c->stride_y = w.sy; c->stride_x = w.sx; c->pad_y = w.py; c->pad_x = w.px;
  c->dil_y = w.dy; c->dil_x = w.dx;
  c->i_n = w.st_n; c->i_y = w.st_y; c->i_x = w.st_x; c->i_c = w.st_c;
  c->f_r = f_r; c->f_s = f_s; c->f_k = f_k; c->f_c = f_c;
  c->o_n = w.n >= 0 ? O.addr.c[w.n] : 0; c->o_y = O.addr.c[w.y]; c->o_x = O.addr.c[w.x]; c->o_k = O.addr.c[k];
  c->i_base = I.addr.k + 0; c->f_base = F.addr.k; c->o_base = O.addr.k;
  // I.addr.k contains -pad*stride terms; the kernels want the buffer origin.
  c->i_base = I.addr.k + w.py * w.st_y + w.px * w.st_x;
  return c->o_k > 0;
}

bool match_pool2d(const FlatBlock& fb, Pool2dShape* p) {
  if (fb.empty) return false;
  // plain windows: load -> store under max / min / add; weighted windows: load, load, mul -> store under add,
  // the second input moving with the taps and the channel only (depthwise convolution) or not at all (a scale)
  const bool weighted = fb.n_refs == 3 && fb.intrinsic == STRIPE_INTR_MUL && fb.agg == STRIPE_AGG_ADD;
  if (!weighted && (fb.n_refs != 2 || fb.intrinsic != STRIPE_INTR_COPY)) return false;
  if (fb.agg != STRIPE_AGG_MAX && fb.agg != STRIPE_AGG_MIN && fb.agg != STRIPE_AGG_ADD) return false;
  const FlatRef &I = fb.ref[0], &O = fb.ref[fb.n_refs - 1];
  Window2d w;
  if (!match_window(fb, I, O.addr, &w)) return false;
  if (!distinct({w.n, w.y, w.x, w.c, w.i, w.j})) return false;
  int used = 0;
  for (int t : {w.n, w.y, w.x, w.c, w.i, w.j})
    if (t >= 0) ++used;
  if (used != fb.n_idx) return false;
  if (w.y < 0 || w.x < 0 || w.c < 0) return false;
  for (int t : {w.n, w.y, w.x, w.c})
    if (t >= 0 && O.addr.c[t] <= 0) return false;
  p->N = range_or_1(fb, w.n); p->Ho = fb.range[w.y]; p->Wo = fb.range[w.x]; p->C = fb.range[w.c];
  p->R = range_or_1(fb, w.i); p->S = range_or_1(fb, w.j); p->H = w.H; p->W = w.W;
  p->stride_y = w.sy; p->stride_x = w.sx; p->pad_y = w.py; p->pad_x = w.px;
  p->dil_y = w.dy; p->dil_x = w.dx;
  p->i_n = w.st_n; p->i_y = w.st_y; p->i_x = w.st_x; p->i_c = w.st_c;
  p->o_n = w.n >= 0 ? O.addr.c[w.n] : 0; p->o_y = O.addr.c[w.y]; p->o_x = O.addr.c[w.x]; p->o_c = O.addr.c[w.c];
  p->i_base = I.addr.k + w.py * w.st_y + w.px * w.st_x;
  p->o_base = O.addr.k;
  p->agg = fb.agg;
  p->w_mode = 0;
  p->w_base = p->w_r = p->w_s = p->w_c = 0;
  if (weighted) {
    const Affine& wa = fb.ref[1].addr;
    for (int t : {w.n, w.y, w.x})
      if (t >= 0 && wa.c[t] != 0) return false;
    p->w_base = wa.k;
    p->w_r = w.i >= 0 ? wa.c[w.i] : 0;
    p->w_s = w.j >= 0 ? wa.c[w.j] : 0;
    p->w_c = wa.c[w.c];
    if (p->w_r < 0 || p->w_s < 0 || p->w_c < 0) return false;
    p->w_mode = (p->w_r == 0 && p->w_s == 0 && p->w_c == 0) ? 1 : 2;
  }
  return true;
}

// --------------------------------------------------------------------------
// Planning on the canonical form
// --------------------------------------------------------------------------
stripe_status_t make_plan(const FlatBlock& fb, stripe_path_t forced, Plan* plan, std::string* err) {
  plan->flat = fb;
  stripe_block_info_t& info = plan->info;
  std::memset(&info, 0, sizeof info);
  const int R = fb.n_refs;
  plan->in_dtype = fb.ref[0].dtype;
  info.n_idx = fb.n_idx;
  for (int r = 0; r + 1 < R; ++r) info.algorithmic_bytes += fb.ref[r].elements * dtype_bytes(fb.ref[r].dtype);
  if (fb.empty) {
    plan->noop = true;
    info.path = STRIPE_PATH_GENERIC;
    std::snprintf(info.kernel, sizeof info.kernel, "none (empty iteration space)");
    info.algorithmic_bytes = 0;
    return STRIPE_OK;
  }
  const Affine& o = fb.ref[R - 1].addr;
  std::vector<int> out_idx, red_idx;
  i128 hull = 1, outs = 1;
  for (int j = 0; j < fb.n_idx; ++j) {
    hull *= fb.range[j];
    if (o.c[j]) {
      out_idx.push_back(j);
      outs *= fb.range[j];
    } else {
      red_idx.push_back(j);
    }
  }
  if (hull > ((i128)1 << 62)) return bad(err, STRIPE_ERR_UNSUPPORTED, "iteration space larger than 2^62 points");
  info.n_out_idx = (int)out_idx.size();
  info.n_red_idx = (int)red_idx.size();
  info.hull_points = (int64_t)hull;
  info.output_elements = (int64_t)outs;
  info.work_points = fb.cons.empty() ? (int64_t)hull : count_points(fb, (int64_t)1 << 26);
  info.algorithmic_bytes += (int64_t)outs * dtype_bytes(fb.ref[R - 1].dtype);

  // The output map must be injective on the output indexes: sorted by |stride|,
  // each stride exceeds the span of all smaller ones (mixed-radix condition).
  std::sort(out_idx.begin(), out_idx.end(), [&](int a, int b) {
    const int64_t x = o.c[a] < 0 ? -o.c[a] : o.c[a], y = o.c[b] < 0 ? -o.c[b] : o.c[b];
    return x != y ? x < y : a < b;
  });
  bool injective = true;
  i128 span = 0;
  for (int j : out_idx) {
    const i128 s = o.c[j] < 0 ? -(i128)o.c[j] : (i128)o.c[j];
    if (s <= span) injective = false;
    span += s * (fb.range[j] - 1);
  }
  if (!injective) {
    // Several index tuples reach one output element through different output indexes (an access like
    // O[x + i]).  The aggregation still defines the result (Definition 2, rule 3); the generic kernel then
    // combines the per-tuple partial results with atomic operations.  'assign' allows a single writer only.
    if (fb.agg == STRIPE_AGG_ASSIGN)
      return bad(err, STRIPE_ERR_ASSIGN_CONFLICT, "'assign' output reached by several index tuples through different output indexes");
    if (span + 1 < outs) info.output_elements = (int64_t)(span + 1);   // at most the addresses between the extremes
    info.algorithmic_bytes -= (int64_t)(outs - info.output_elements) * dtype_bytes(fb.ref[R - 1].dtype);
  }
  if (fb.agg == STRIPE_AGG_ASSIGN && !red_idx.empty())
    return bad(err, STRIPE_ERR_ASSIGN_CONFLICT, "'assign' output with an index that does not move the output address");

  // the specialised families store fp32 / int32; a bf16 output buffer runs on the generic kernel
  if (fb.out_bf16 && !injective)
    return bad(err, STRIPE_ERR_UNSUPPORTED, "a bf16 output shared between index tuples (no 16-bit atomic aggregation)");
  const bool plain_out = injective && !fb.out_bf16;
  const bool is_gemm = plain_out && match_gemm(fb, &plan->gemm);
  const bool is_conv = plain_out && match_conv2d(fb, &plan->conv);
  const bool is_pool = plain_out && match_pool2d(fb, &plan->pool);
  plan->is_gemm = is_gemm;
  plan->is_conv = is_conv;
  plan->is_pool = is_pool;
  stripe_path_t path = forced;
  if (path == STRIPE_PATH_AUTO) {
    path = is_gemm ? STRIPE_PATH_MFMA_GEMM : is_conv ? STRIPE_PATH_MFMA_CONV : is_pool ? STRIPE_PATH_POOL : STRIPE_PATH_GENERIC;
  } else if ((path == STRIPE_PATH_MFMA_GEMM && !is_gemm) || (path == STRIPE_PATH_MFMA_CONV && !is_conv) ||
             (path == STRIPE_PATH_POOL && !is_pool)) {
    return bad(err, STRIPE_ERR_UNSUPPORTED, "the block does not have the shape of the requested kernel family");
  }
  info.path = path;

  // Generic parameters are always prepared: the specialised families fall back
  // to the generic kernel when a shape detail (tile divisibility, layout) is
  // outside what they cover.
  GenericParams& g = plan->gen;
  std::memset(&g, 0, sizeof g);
  bool gen_ok = true;
  std::string gen_why;
  if ((int)out_idx.size() > kGenIdx || (int)red_idx.size() > kGenIdx || (int)fb.cons.size() > kGenCons) {
    gen_ok = false;
    gen_why = "more than 8 output indexes, 8 reduction indexes or 8 constraints after canonicalisation";
  }
  if (gen_ok) {
    const Affine& A = fb.ref[0].addr;
    const Affine* B = R == 3 ? &fb.ref[1].addr : nullptr;
    // innermost reduction index: smallest input stride, so consecutive lanes/steps touch consecutive elements
    std::sort(red_idx.begin(), red_idx.end(), [&](int a, int b) {
      auto key = [&](int j) {
        int64_t x = A.c[j] < 0 ? -A.c[j] : A.c[j];
        if (B) {
          const int64_t y = B->c[j] < 0 ? -B->c[j] : B->c[j];
          x = std::max(x, y);
        }
        return x;
      };
      const int64_t x = key(a), y = key(b);
      return x != y ? x < y : a > b;
    });
    for (int t = 0; t < kGenIdx; ++t) g.out_range[t] = g.red_range[t] = 1;
    g.n_out = (int)out_idx.size();
    g.n_red = (int)red_idx.size();
    i128 red_total = 1;
    for (int t = 0; t < g.n_out; ++t) {
      const int j = out_idx[t];
      g.out_range[t] = (int32_t)fb.range[j];
      g.a_out[t] = A.c[j];
      g.b_out[t] = B ? B->c[j] : 0;
      g.o_out[t] = o.c[j];
    }
    for (int t = 0; t < g.n_red; ++t) {
      const int j = red_idx[t];
      g.red_range[t] = (int32_t)fb.range[j];
      g.a_red[t] = A.c[j];
      g.b_red[t] = B ? B->c[j] : 0;
      red_total *= fb.range[j];
    }
    if (red_total > 0x7fffffffLL) {
      gen_ok = false;
      gen_why = "more than 2^31 reduction points per output element";
    }
    g.red_total = (uint32_t)red_total;
    g.inner_range = g.n_red ? (uint32_t)g.red_range[0] : 1u;
    g.a_base = A.k;
    g.b_base = B ? B->k : 0;
    g.o_base = o.k;
    g.n_outputs = (int64_t)outs;
    for (size_t q = 0; q < fb.cons.size() && gen_ok; ++q) {
      const Affine& c = fb.cons[q];
      g.cons_const[q] = c.k;
      for (int t = 0; t < g.n_out; ++t) g.cons_out[q][t] = (int32_t)c.c[out_idx[t]];
      for (int t = 0; t < g.n_red; ++t) g.cons_red[q][t] = (int32_t)c.c[red_idx[t]];
      // the kernel holds constraint coefficients in 32 bits; flattening multiplies passed coefficients into them
      for (int j = 0; j < fb.n_idx; ++j)
        if (c.c[j] > 0x7fffffffLL || c.c[j] < -0x7fffffffLL) {
          gen_ok = false;
          gen_why = "a constraint coefficient exceeds 32 bits after substituting passed values";
        }
    }
    // One lane per output when neighbouring outputs read neighbouring (or the
    // same) input elements; otherwise one wavefront per output with the lanes
    // spread along the reduction and a cross-lane reduction at the end.
    bool lane_per_output_coalesces = true;
    if (g.n_out) {
      const int64_t sa = g.a_out[0] < 0 ? -g.a_out[0] : g.a_out[0];
      const int64_t sb = g.b_out[0] < 0 ? -g.b_out[0] : g.b_out[0];
      if (sa > 1 || sb > 1) lane_per_output_coalesces = false;
    }
    g.lanes = (!lane_per_output_coalesces && g.red_total >= 64) ? 64 : 1;
    if (gen_ok && (g.lanes == 64 ? (outs + 3) / 4 : (outs + 255) / 256) > (i128)0x7fffffff) {
      gen_ok = false;
      gen_why = "more than 2^31 workgroups: split the block on an output index";
    }
    // 32-bit index arithmetic when nothing the kernel computes can leave int32:
    // largest |offset| of each tensor, largest |value| of each constraint, the output count.
    auto reach = [&](const Affine& f) {
      i128 m = f.k < 0 ? -(i128)f.k : (i128)f.k;
      for (int j = 0; j < fb.n_idx; ++j) m += (f.c[j] < 0 ? -(i128)f.c[j] : (i128)f.c[j]) * (fb.range[j] - 1);
      return m;
    };
    const i128 lim = (i128)0x3fffffff;   // one extra loop step past a range stays representable
    bool narrow = (i128)outs + 256 <= lim && reach(A) <= lim && reach(o) <= lim && (!B || reach(*B) <= lim);
    for (const Affine& c : fb.cons) narrow = narrow && reach(c) <= lim;
    g.narrow = narrow ? 1 : 0;
    g.atomic = injective ? 0 : 1;
    g.out_bf16 = fb.out_bf16 ? 1 : 0;
    // Pointwise blocks (every index moves the output, no constraints): four consecutive outputs per lane when the
    // fastest output index has unit stride in the output, stride 0 or 1 in the inputs, and everything else keeps
    // 4-element alignment.
    {
      bool p4 = narrow && injective && g.n_red == 0 && fb.cons.empty() && g.n_out >= 1 && g.out_range[0] % 4 == 0 && g.o_out[0] == 1 &&
                (g.a_out[0] == 0 || g.a_out[0] == 1) && (!B || g.b_out[0] == 0 || g.b_out[0] == 1) && g.o_base % 4 == 0 &&
                (g.a_out[0] == 0 || g.a_base % 4 == 0) && (!B || g.b_out[0] == 0 || g.b_base % 4 == 0);
      for (int t = 1; t < g.n_out && p4; ++t)
        p4 = g.o_out[t] % 4 == 0 && (g.a_out[0] == 0 || g.a_out[t] % 4 == 0) && (!B || g.b_out[0] == 0 || g.b_out[t] % 4 == 0);
      g.point4 = p4 ? 1 : 0;
    }

    // Register-tiled variant for sum-of-products blocks with enough parallelism (see TiledParams).
    TiledParams& tp = plan->tiled;
    std::memset(&tp, 0, sizeof tp);
    if (narrow && injective && B && fb.intrinsic == STRIPE_INTR_MUL && fb.agg == STRIPE_AGG_ADD && !fb.out_bf16) {
      auto absv = [](int64_t v) { return v < 0 ? -v : v; };
      auto in_cons = [&](int j) {
        for (const Affine& c : fb.cons)
          if (c.c[j]) return true;
        return false;
      };
      int pm = -1, pn = -1;
      for (int j : out_idx) {   // out_idx is sorted by |output stride|: the first fit has the smallest
        const bool inA = A.c[j] != 0, inB = B->c[j] != 0;
        if (inA && !inB && pm < 0) pm = j;
        if (!inA && inB && pn < 0 && !in_cons(j)) pn = j;
      }
      // innermost reduction index: free of constraints; unit stride in both operands is best (vector loads)
      int r0 = -1;
      for (int j : red_idx) {
        if (in_cons(j)) continue;
        const bool unit = absv(A.c[j]) == 1 && absv(B->c[j]) == 1;
        if (r0 < 0 || (unit && !(absv(A.c[r0]) == 1 && absv(B->c[r0]) == 1))) r0 = j;
      }
      std::vector<int> reds;
      if (r0 >= 0) reds.push_back(r0);
      for (int j : red_idx)
        if (j != r0) reds.push_back(j);
      const int first_real = r0 >= 0 ? 0 : 1;   // without a constraint-free index level 0 stays a dummy of range 1
      std::vector<int> outers;
      for (int j : out_idx)
        if (j != pm && j != pn) outers.push_back(j);
      if (pm >= 0 && pn >= 0 && (int)reds.size() + first_real <= kTiledRed && (int)outers.size() <= kTiledOuter) {
        tp.n_outer = (int)outers.size();
        tp.n_cons = (int)fb.cons.size();
        i128 items = 1;
        for (int t = 0; t < kTiledOuter; ++t) tp.outer_range[t] = 1;
        for (int t = 0; t < tp.n_outer; ++t) {
          const int j = outers[t];
          tp.outer_range[t] = (int32_t)fb.range[j];
          tp.a_outer[t] = (int32_t)A.c[j]; tp.b_outer[t] = (int32_t)B->c[j]; tp.o_outer[t] = (int32_t)o.c[j];
          for (int q = 0; q < tp.n_cons; ++q) tp.cons_outer[q][t] = (int32_t)fb.cons[q].c[j];
          items *= fb.range[j];
        }
        tp.pm_range = (int32_t)fb.range[pm]; tp.pn_range = (int32_t)fb.range[pn];
        tp.pm_blocks = (tp.pm_range + 3) / 4; tp.pn_blocks = (tp.pn_range + 3) / 4;
        items *= (i128)tp.pm_blocks * tp.pn_blocks;
        tp.a_pm = (int32_t)A.c[pm]; tp.o_pm = (int32_t)o.c[pm]; tp.b_pn = (int32_t)B->c[pn]; tp.o_pn = (int32_t)o.c[pn];
        for (int q = 0; q < tp.n_cons; ++q) {
          tp.cons_pm[q] = (int32_t)fb.cons[q].c[pm];
          tp.cons_const[q] = (int32_t)fb.cons[q].k;
        }
        for (int t = 0; t < kTiledRed; ++t) tp.red_range[t] = 1;
        for (size_t t = 0; t < reds.size(); ++t) {
          const int j = reds[t], lvl = (int)t + first_real;
          tp.red_range[lvl] = (int32_t)fb.range[j];
          tp.a_red[lvl] = (int32_t)A.c[j]; tp.b_red[lvl] = (int32_t)B->c[j];
          for (int q = 0; q < tp.n_cons; ++q) tp.cons_red[q][lvl] = (int32_t)fb.cons[q].c[j];
        }
        tp.a_base = (int32_t)A.k; tp.b_base = (int32_t)B->k; tp.o_base = (int32_t)o.k;
        tp.n_items = (int64_t)items;
        // four elements per load when the innermost reduction index is unit-stride in both operands and every
        // other address term keeps 4-element alignment
        bool vec = r0 >= 0 && A.c[r0] == 1 && B->c[r0] == 1 && fb.range[r0] % 4 == 0 && A.k % 4 == 0 && B->k % 4 == 0;
        for (int j = 0; j < fb.n_idx && vec; ++j)
          if (j != r0 && (A.c[j] % 4 || B->c[j] % 4)) vec = false;
        tp.vec = vec ? 4 : 1;
        // worth it only with enough lanes to fill the chip; small blocks stay on the wavefront-per-output mapping
        tp.use = (items >= 16384 && items < ((i128)1 << 31)) ? 1 : 0;
      }
    }
  }
  if (path == STRIPE_PATH_GENERIC && !gen_ok) return bad(err, STRIPE_ERR_UNSUPPORTED, gen_why);
  if (!gen_ok) g.n_outputs = -1;  // marks "no generic fallback"
  return STRIPE_OK;
}

}  // namespace stripe
