// Autotiling for a flat Stripe block (paper Section 3.3): the cache-line cost
// model of Figure 4, an exhaustive tile search under its admissibility rules,
// and the rewrite of Figure 5a into the nest of Figure 5b.  Host-only integer
// code; nothing here touches the GPU.
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <new>
#include <string>
#include <vector>

#include "plan.hpp"

namespace stripe {
namespace {

struct FlatForm {
  const stripe_block_desc_t* root = nullptr;
  const stripe_block_desc_t* leaf = nullptr;
  int n = 0;   // leaf indexes
};

stripe_status_t flat_form(const stripe_block_desc_t* root, FlatForm* f) {
  if (!root) return api_fail(STRIPE_ERR_NULL, "root is NULL");
  if (root->n_idx != 0 || !root->child || root->child->child || root->child->n_passed != 0)
    return api_fail(STRIPE_ERR_INVALID_DESC, "tiling takes the flat form: a root without indexes whose child is the leaf");
  const stripe_block_desc_t* leaf = root->child;
  if (leaf->n_idx < 1 || leaf->n_idx > 31 || leaf->n_refs < 2 || leaf->n_refs > 3 || leaf->n_refs != root->n_refs || !leaf->ranges ||
      !leaf->refs || !root->refs || (leaf->n_constraints > 0 && (!leaf->cons_coeff || !leaf->cons_const)))
    return api_fail(STRIPE_ERR_INVALID_DESC, "leaf needs 1..31 indexes and the root's 2 or 3 refinements");
  for (int r = 0; r < leaf->n_refs; ++r) {
    const stripe_refinement_t& q = leaf->refs[r];
    if (q.ndim < 1 || q.ndim != root->refs[r].ndim || !q.access_coeff || !q.access_const || !q.strides || !root->refs[r].sizes)
      return api_fail(STRIPE_ERR_INVALID_DESC, "refinement without access rows, strides or root sizes");
  }
  for (int j = 0; j < leaf->n_idx; ++j)
    if (leaf->ranges[j] < 1) return api_fail(STRIPE_ERR_INVALID_DESC, "tiling needs non-empty ranges");
  f->root = root;
  f->leaf = leaf;
  f->n = leaf->n_idx;
  return STRIPE_OK;
}

stripe_status_t check_tile(const FlatForm& f, const int64_t* tile) {
  if (!tile) return api_fail(STRIPE_ERR_NULL, "tile is NULL");
  for (int j = 0; j < f.n; ++j)
    if (tile[j] < 1 || tile[j] > f.leaf->ranges[j]) return api_fail(STRIPE_ERR_INVALID_DESC, "tile size outside 1..range");
  return STRIPE_OK;
}

// Span of dimension d of refinement r over one tile: [lo, hi] relative to the tile's origin.
void span_of(const FlatForm& f, int r, int d, const int64_t* tile, int64_t* lo, int64_t* hi) {
  const int64_t* row = f.leaf->refs[r].access_coeff + (size_t)d * f.n;
  *lo = *hi = 0;
  for (int j = 0; j < f.n; ++j) {
    const int64_t reach = row[j] * (tile[j] - 1);
    if (reach < 0) *lo += reach; else *hi += reach;
  }
}

bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

TileProblem problem_of(const FlatForm& f) {
  TileProblem pr;
  pr.range.assign(f.leaf->ranges, f.leaf->ranges + f.n);
  for (int r = 0; r < f.leaf->n_refs; ++r) {
    const stripe_refinement_t& q = f.leaf->refs[r];
    TileRef t;
    t.coeff.assign(q.access_coeff, q.access_coeff + (size_t)q.ndim * f.n);
    t.stride.assign(q.strides, q.strides + q.ndim);
    pr.refs.push_back(t);
  }
  return pr;
}

}  // namespace

// The cost of one tile (Figure 4's caption): tiles * lines per tile / work, with footprint and admissibility.
void tile_cost_of(const TileProblem& pr, const int64_t* tile, const stripe_tile_model_t& m, stripe_tile_cost_t* c) {
  const int n = (int)pr.range.size();
  c->tiles = 1;
  c->work = 1;
  c->admissible = 1;
  for (int j = 0; j < n; ++j) {
    const int64_t range = pr.range[j];
    c->tiles *= (range + tile[j] - 1) / tile[j];
    if (m.tiled_idx >> j & 1) c->work *= range;
    if (tile[j] != range) {
      const int64_t mult = (m.multiple_of && m.multiple_of[j] > 1) ? m.multiple_of[j] : 1;
      if (tile[j] % mult) c->admissible = 0;
      if (m.power_of_two && !is_pow2(tile[j])) c->admissible = 0;
    }
  }
  c->lines_per_tile = 0;
  c->footprint_elems = 0;
  for (size_t r = 0; r < pr.refs.size(); ++r) {
    if (!(m.counted_refs >> r & 1)) continue;
    const TileRef& q = pr.refs[r];
    const int ndim = (int)q.stride.size();
    int line_dim = -1;
    for (int d = 0; d < ndim; ++d)
      if (q.stride[d] == 1 || q.stride[d] == -1) line_dim = d;
    int64_t lines = 1, elems = 1;
    for (int d = 0; d < ndim; ++d) {
      int64_t lo = 0, hi = 0;   // span of the dimension over one tile, relative to the tile's origin
      for (int j = 0; j < n; ++j) {
        const int64_t reach = q.coeff[(size_t)d * n + j] * (tile[j] - 1);
        if (reach < 0) lo += reach; else hi += reach;
      }
      const int64_t extent = hi - lo + 1;
      elems *= extent;
      lines *= (d == line_dim) ? (extent + m.line_elems - 1) / m.line_elems : extent;
    }
    c->lines_per_tile += lines;
    c->footprint_elems += elems;
  }
  if (m.mem_cap_elems > 0 && c->footprint_elems > m.mem_cap_elems) c->admissible = 0;
  c->cost = (double)c->tiles * (double)c->lines_per_tile / (double)c->work;
}

// Exhaustive minimum over the cross product of the candidate sizes; ties go to fewer tiles, then to the
// lexicographically larger tile.  False if no candidate is admissible.
bool tile_search_in(const TileProblem& pr, const stripe_tile_model_t& m, const std::vector<std::vector<int64_t>>& cand,
                    std::vector<int64_t>* best_tile, stripe_tile_cost_t* best) {
  const int n = (int)pr.range.size();
  std::vector<size_t> pos(n, 0);
  std::vector<int64_t> tile(n);
  best_tile->assign(n, 0);
  bool found = false;
  for (;;) {
    for (int j = 0; j < n; ++j) tile[j] = cand[j][pos[j]];
    stripe_tile_cost_t c;
    tile_cost_of(pr, tile.data(), m, &c);
    if (c.admissible) {
      bool better = !found || c.cost < best->cost || (c.cost == best->cost && c.tiles < best->tiles);
      if (found && c.cost == best->cost && c.tiles == best->tiles)
        better = std::lexicographical_compare(best_tile->begin(), best_tile->end(), tile.begin(), tile.end());
      if (better) {
        *best = c;
        *best_tile = tile;
        found = true;
      }
    }
    int j = n - 1;
    while (j >= 0 && ++pos[j] == cand[j].size()) pos[j--] = 0;
    if (j < 0) break;
  }
  return found;
}

namespace {

stripe_status_t check_model(const stripe_tile_model_t* m) {
  if (!m) return api_fail(STRIPE_ERR_NULL, "model is NULL");
  if (m->line_elems < 1 || m->mem_cap_elems < 0) return api_fail(STRIPE_ERR_INVALID_DESC, "line_elems >= 1 and mem_cap_elems >= 0 required");
  return STRIPE_OK;
}

// The rewritten nest and everything its pointers refer to, in one allocation unit.
struct OwnedNest {
  stripe_block_desc_t root;     // first member: the pointer handed out is the pointer freed
  stripe_block_desc_t outer, inner;
  std::vector<stripe_refinement_t> root_refs, outer_refs, inner_refs;
  std::vector<std::vector<int64_t>> store;   // every coefficient / size / stride array
  const int64_t* keep(std::vector<int64_t> v) {
    if (v.empty()) v.push_back(0);
    store.push_back(std::move(v));
    return store.back().data();
  }
};

}  // namespace
}  // namespace stripe

using namespace stripe;

extern "C" {

stripe_status_t stripe_tile_cost(const stripe_block_desc_t* root, const int64_t* tile, const stripe_tile_model_t* model,
                                 stripe_tile_cost_t* out) {
  if (!out) return api_fail(STRIPE_ERR_NULL, "out is NULL");
  FlatForm f;
  stripe_status_t st = flat_form(root, &f);
  if (st == STRIPE_OK) st = check_model(model);
  if (st == STRIPE_OK) st = check_tile(f, tile);
  if (st != STRIPE_OK) return st;
  tile_cost_of(problem_of(f), tile, *model, out);
  return STRIPE_OK;
}

stripe_status_t stripe_tile_search(const stripe_block_desc_t* root, const stripe_tile_model_t* model, int64_t* best_tile,
                                   stripe_tile_cost_t* best) {
  if (!best_tile || !best) return api_fail(STRIPE_ERR_NULL, "best_tile or best is NULL");
  FlatForm f;
  stripe_status_t st = flat_form(root, &f);
  if (st == STRIPE_OK) st = check_model(model);
  if (st != STRIPE_OK) return st;
  // candidate sizes per index
  std::vector<std::vector<int64_t>> cand(f.n);
  double space = 1;
  for (int j = 0; j < f.n; ++j) {
    const int64_t range = f.leaf->ranges[j];
    if (model->tiled_idx >> j & 1) {
      const int64_t mult = (model->multiple_of && model->multiple_of[j] > 1) ? model->multiple_of[j] : 1;
      for (int64_t t = 1; t < range; ++t)
        if (t % mult == 0 && (!model->power_of_two || is_pow2(t))) cand[j].push_back(t);
    }
    cand[j].push_back(range);
    space *= (double)cand[j].size();
  }
  if (space > (double)(1 << 22)) return api_fail(STRIPE_ERR_UNSUPPORTED, "more than 2^22 candidate tiles: restrict tiled_idx, multiple_of or power_of_two");
  std::vector<int64_t> tile;
  const bool found = tile_search_in(problem_of(f), *model, cand, &tile, best);
  if (found) std::memcpy(best_tile, tile.data(), sizeof(int64_t) * f.n);
  if (!found) return api_fail(STRIPE_ERR_UNSUPPORTED, "no admissible tile under this model");
  return STRIPE_OK;
}

stripe_status_t stripe_block_tile(const stripe_block_desc_t* root, const int64_t* tile, stripe_block_desc_t** out) {
  if (!out) return api_fail(STRIPE_ERR_NULL, "out is NULL");
  *out = nullptr;
  FlatForm f;
  stripe_status_t st = flat_form(root, &f);
  if (st == STRIPE_OK) st = check_tile(f, tile);
  if (st != STRIPE_OK) return st;
  OwnedNest* nest = new (std::nothrow) OwnedNest();
  if (!nest) return api_fail(STRIPE_ERR_NOMEM, "out of host memory");
  const stripe_block_desc_t* leaf = f.leaf;
  const int n = f.n, R = leaf->n_refs;

  // indexes that get a passed outer value: several tiles AND (used by a constraint OR tile does not divide the range)
  std::vector<int> passed_of(n, -1);
  int n_passed = 0;
  for (int j = 0; j < n; ++j) {
    const int64_t range = leaf->ranges[j];
    if (tile[j] == range) continue;
    bool used = range % tile[j] != 0;
    for (int q = 0; q < leaf->n_constraints && !used; ++q) used = leaf->cons_coeff[(size_t)q * n + j] != 0;
    if (used) passed_of[j] = n_passed++;
  }
  const int inner_vars = n + n_passed;

  // root: a copy of the caller's
  nest->root_refs.resize(R);
  for (int r = 0; r < R; ++r) {
    const stripe_refinement_t& q = root->refs[r];
    stripe_refinement_t& d = nest->root_refs[r];
    d = q;
    d.access_coeff = nest->keep({});
    d.access_const = nest->keep(q.access_const ? std::vector<int64_t>(q.access_const, q.access_const + q.ndim) : std::vector<int64_t>(q.ndim, 0));
    d.sizes = nest->keep(std::vector<int64_t>(q.sizes, q.sizes + q.ndim));
    d.strides = nest->keep(std::vector<int64_t>(q.strides, q.strides + q.ndim));
  }
  std::memset(&nest->root, 0, sizeof nest->root);
  nest->root.n_refs = R;
  nest->root.refs = nest->root_refs.data();
  nest->root.intrinsic = root->intrinsic;
  nest->root.ranges = nest->keep({});
  nest->root.child = &nest->outer;

  // outer and inner levels
  std::vector<int64_t> outer_ranges(n), inner_ranges(n);
  for (int j = 0; j < n; ++j) {
    outer_ranges[j] = (leaf->ranges[j] + tile[j] - 1) / tile[j];
    inner_ranges[j] = tile[j];
  }
  nest->outer_refs.resize(R);
  nest->inner_refs.resize(R);
  for (int r = 0; r < R; ++r) {
    const stripe_refinement_t& q = leaf->refs[r];
    std::vector<int64_t> oc((size_t)q.ndim * n), ok(q.ndim), osz(q.ndim), ic((size_t)q.ndim * inner_vars, 0), ik(q.ndim), isz(q.ndim, 1);
    for (int d = 0; d < q.ndim; ++d) {
      int64_t lo, hi;
      span_of(f, r, d, tile, &lo, &hi);
      for (int j = 0; j < n; ++j) {
        // the tile's origin moves by tile_j per outer step; an index left whole has a single outer step
        oc[(size_t)d * n + j] = tile[j] == leaf->ranges[j] ? 0 : q.access_coeff[(size_t)d * n + j] * tile[j];
        ic[(size_t)d * inner_vars + j] = q.access_coeff[(size_t)d * n + j];
      }
      ok[d] = q.access_const[d] + lo;    // view origin: the lowest coordinate the tile reaches
      osz[d] = hi - lo + 1;              // view size: halo and overflow included
      ik[d] = -lo;                       // inner accesses are relative to the view origin
    }
    std::vector<int64_t> strides(q.strides, q.strides + q.ndim);
    stripe_refinement_t& o = nest->outer_refs[r];
    o = q;
    o.access_coeff = nest->keep(oc);
    o.access_const = nest->keep(ok);
    o.sizes = nest->keep(osz);
    o.strides = nest->keep(strides);
    stripe_refinement_t& i = nest->inner_refs[r];
    i = q;
    i.access_coeff = nest->keep(ic);
    i.access_const = nest->keep(ik);
    i.sizes = nest->keep(isz);
    i.strides = nest->keep(strides);
  }
  std::memset(&nest->outer, 0, sizeof nest->outer);
  nest->outer.n_idx = n;
  nest->outer.ranges = nest->keep(outer_ranges);
  nest->outer.n_refs = R;
  nest->outer.refs = nest->outer_refs.data();
  nest->outer.intrinsic = leaf->intrinsic;
  nest->outer.passed_coeff = nest->keep({});
  nest->outer.passed_const = nest->keep({});
  nest->outer.cons_coeff = nest->keep({});
  nest->outer.cons_const = nest->keep({});
  nest->outer.child = &nest->inner;

  std::vector<int64_t> pc((size_t)n_passed * n, 0), pk(n_passed, 0);
  for (int j = 0; j < n; ++j)
    if (passed_of[j] >= 0) pc[(size_t)passed_of[j] * n + j] = tile[j];       // passed value = tile_j * outer index j
  // constraints: the original rows with index j read as (passed_j + inner j), then one overflow row per ragged index
  std::vector<int64_t> cc, ck;
  for (int q = 0; q < leaf->n_constraints; ++q) {
    std::vector<int64_t> row(inner_vars, 0);
    for (int j = 0; j < n; ++j) {
      const int64_t a = leaf->cons_coeff[(size_t)q * n + j];
      row[j] = a;
      if (passed_of[j] >= 0) row[n + passed_of[j]] = a;
    }
    cc.insert(cc.end(), row.begin(), row.end());
    ck.push_back(leaf->cons_const[q]);
  }
  int n_cons = leaf->n_constraints;
  for (int j = 0; j < n; ++j) {
    if (leaf->ranges[j] % tile[j] == 0) continue;
    std::vector<int64_t> row(inner_vars, 0);
    row[j] = -1;
    row[n + passed_of[j]] = -1;
    cc.insert(cc.end(), row.begin(), row.end());
    ck.push_back(leaf->ranges[j] - 1);      // range_j - 1 - passed_j - inner_j >= 0
    ++n_cons;
  }
  std::memset(&nest->inner, 0, sizeof nest->inner);
  nest->inner.n_idx = n;
  nest->inner.ranges = nest->keep(inner_ranges);
  nest->inner.n_passed = n_passed;
  nest->inner.passed_coeff = nest->keep(pc);
  nest->inner.passed_const = nest->keep(pk);
  nest->inner.n_constraints = n_cons;
  nest->inner.cons_coeff = nest->keep(cc);
  nest->inner.cons_const = nest->keep(ck);
  nest->inner.n_refs = R;
  nest->inner.refs = nest->inner_refs.data();
  nest->inner.intrinsic = leaf->intrinsic;
  nest->inner.child = nullptr;
  *out = &nest->root;
  return STRIPE_OK;
}

void stripe_desc_free(stripe_block_desc_t* desc) {
  delete reinterpret_cast<stripe::OwnedNest*>(desc);
}

}  // extern "C"
