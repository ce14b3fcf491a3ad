/*
 * Stripe block oracle -- TEST INFRASTRUCTURE, not part of the product.
 * See stripe_oracle.h for what it computes and which passages it follows.
 *
 * Written for checking by eye: one loop per index in declaration order, every
 * constraint tested at every point, every access bounds-checked, no tiling,
 * no flattening of the nest, no reordering.
 */
#include "stripe_oracle.h"

#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
  const so_block_t* lvl[SO_MAX_LEVELS];
  int n_levels;
  int n_refs;
  int out_ref;                 /* index of the output refinement */
  int int_mode;                /* output is i32 */
  int agg;                     /* the one non-assign aggregation of the nest, or assign */
  int64_t vars[SO_MAX_LEVELS][SO_MAX_VARS];
  int64_t coord[SO_MAX_LEVELS][SO_MAX_REFS][SO_MAX_DIMS];
  int64_t iters[SO_MAX_LEVELS]; /* number of hull points of one execution of the level */
  int64_t* owner[SO_MAX_LEVELS]; /* per assign level with > 1 iteration: ordinal of last writer */
  const void* const* inputs;
  double* out_f64;
  int64_t* out_i64;
  uint8_t* touched;
  const int64_t* win_lo;
  const int64_t* win_hi;
  int64_t n_points;
  char* err;
  size_t errlen;
} ctx_t;

static int fail(ctx_t* c, int code, const char* fmt, ...) {
  if (c->err && c->errlen) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(c->err, c->errlen, fmt, ap);
    va_end(ap);
  }
  return code;
}

static int n_vars_of(const so_block_t* b) { return b->n_idx + b->n_passed; }

/* Widen a bf16 bit pattern exactly: it is the upper half of an fp32. */
static double widen_bf16(uint16_t h) {
  uint32_t u = ((uint32_t)h) << 16;
  float f;
  memcpy(&f, &u, sizeof f);
  return (double)f;
}

static double load_float(const void* base, int dtype, int64_t addr) {
  if (dtype == SO_BF16) return widen_bf16(((const uint16_t*)base)[addr]);
  return (double)((const float*)base)[addr];
}

static int64_t load_int(const void* base, int dtype, int64_t addr) {
  if (dtype == SO_I8) return (int64_t)((const int8_t*)base)[addr];
  return (int64_t)((const int32_t*)base)[addr];
}

static int fits_i32(int64_t v) { return v >= INT32_MIN && v <= INT32_MAX; }

static int run_level(ctx_t* c, int L);

/* The leaf statement list at one point of the leaf's iteration space. */
static int leaf_statements(ctx_t* c, int L) {
  int64_t addr[SO_MAX_REFS];
  c->n_points++;
  for (int r = 0; r < c->n_refs; ++r) {
    const int ndim = c->lvl[0]->refs[r].ndim;
    addr[r] = 0;
    for (int d = 0; d < ndim; ++d) {
      /* The scalar must lie inside the view of every enclosing level; the
       * root's view is the buffer itself. */
      for (int l = 0; l < L; ++l) {
        int64_t rel = 0;
        for (int m = l + 1; m <= L; ++m) rel += c->coord[m][r][d];
        if (rel < 0 || rel >= c->lvl[l]->refs[r].sizes[d])
          return fail(c, SO_ERR_OUT_OF_BOUNDS,
                      "refinement %lld dim %lld: coordinate %lld outside the enclosing view", (long long)(r), (long long)(d), (long long)(rel));
      }
      for (int l = 0; l <= L; ++l) addr[r] += c->lvl[l]->refs[r].strides[d] * c->coord[l][r][d];
    }
  }

  const so_block_t* leaf = c->lvl[L];
  const int64_t e = addr[c->out_ref];

  /* 'assign' levels: two iterations of one execution of the level may not
   * write the same element (Section 3.2). */
  {
    int64_t ord = 0;
    for (int l = 1; l <= L; ++l) {
      for (int j = 0; j < c->lvl[l]->n_idx; ++j) ord = ord * c->lvl[l]->ranges[j] + c->vars[l][j];
      if (c->owner[l]) {
        const int64_t last = c->owner[l][e];
        if (last >= 0 && last / c->iters[l] == ord / c->iters[l] && last != ord)
          return fail(c, SO_ERR_ASSIGN, "level %lld: element %lld written by two iterations (%lld)", (long long)(l), (long long)(e), (long long)(ord));
        c->owner[l][e] = ord;
      }
    }
  }

  if (c->int_mode) {
    int64_t v;
    const int64_t a = load_int(c->inputs[0], c->lvl[0]->refs[0].dtype, addr[0]);
    if (leaf->intrinsic == SO_INTR_COPY) {
      v = a;
    } else {
      const int64_t b = load_int(c->inputs[1], c->lvl[0]->refs[1].dtype, addr[1]);
      v = (leaf->intrinsic == SO_INTR_MUL) ? a * b : a + b;
      if (leaf->intrinsic == SO_INTR_ADD_RELU && v < 0) v = 0;
    }
    if (!fits_i32(v)) return fail(c, SO_ERR_INT_OVERFLOW, "value %lld at element %lld exceeds int32", (long long)(v), (long long)(e));
    if (!c->touched[e]) {
      c->touched[e] = 1;
      c->out_i64[e] = v;
    } else {
      int64_t acc = c->out_i64[e];
      switch (c->agg) {
        case SO_AGG_ADD: acc = acc + v; break;
        case SO_AGG_MUL: acc = acc * v; break;
        case SO_AGG_MAX: if (v > acc) acc = v; break;
        case SO_AGG_MIN: if (v < acc) acc = v; break;
        default: return fail(c, SO_ERR_ASSIGN, "element %lld written twice under assign", (long long)(e));
      }
      if (!fits_i32(acc)) return fail(c, SO_ERR_INT_OVERFLOW, "partial result %lld at element %lld exceeds int32", (long long)(acc), (long long)(e));
      c->out_i64[e] = acc;
    }
  } else {
    double v;
    const double a = load_float(c->inputs[0], c->lvl[0]->refs[0].dtype, addr[0]);
    if (leaf->intrinsic == SO_INTR_COPY) {
      v = a;
    } else {
      const double b = load_float(c->inputs[1], c->lvl[0]->refs[1].dtype, addr[1]);
      v = (leaf->intrinsic == SO_INTR_MUL) ? a * b : a + b;
      if (leaf->intrinsic == SO_INTR_ADD_RELU && v < 0) v = 0;
    }
    if (!c->touched[e]) {
      c->touched[e] = 1;
      c->out_f64[e] = v;
    } else {
      double acc = c->out_f64[e];
      switch (c->agg) {
        case SO_AGG_ADD: acc = acc + v; break;
        case SO_AGG_MUL: acc = acc * v; break;
        case SO_AGG_MAX: if (v > acc) acc = v; break;
        case SO_AGG_MIN: if (v < acc) acc = v; break;
        default: return fail(c, SO_ERR_ASSIGN, "element %lld written twice under assign", (long long)(e));
      }
      c->out_f64[e] = acc;
    }
  }
  return SO_OK;
}

/* One point of level L: test the constraints, place the views, run the statement. */
static int point(ctx_t* c, int L) {
  const so_block_t* b = c->lvl[L];
  const int nv = n_vars_of(b);
  for (int q = 0; q < b->n_cons; ++q) {
    int64_t s = b->cons_const[q];
    for (int v = 0; v < nv; ++v) s += b->cons_coeff[(size_t)q * nv + v] * c->vars[L][v];
    if (s < 0) return SO_OK; /* outside the polyhedron: nothing runs here */
  }
  for (int r = 0; r < c->n_refs; ++r) {
    const so_ref_t* ref = &b->refs[r];
    for (int d = 0; d < ref->ndim; ++d) {
      int64_t s = ref->access_const[d];
      for (int v = 0; v < nv; ++v) s += ref->access_coeff[(size_t)d * nv + v] * c->vars[L][v];
      c->coord[L][r][d] = s;
    }
  }
  if (b->child) return run_level(c, L + 1);
  return leaf_statements(c, L);
}

/* Loop over index j of level L, then the rest. */
static int loop_index(ctx_t* c, int L, int j) {
  const so_block_t* b = c->lvl[L];
  if (j == b->n_idx) return point(c, L);
  int64_t lo = 0, hi = b->ranges[j];
  if (L == 1 && c->win_lo && c->win_hi) {
    lo = c->win_lo[j];
    hi = c->win_hi[j];
  }
  for (int64_t v = lo; v < hi; ++v) {
    c->vars[L][j] = v;
    const int rc = loop_index(c, L, j + 1);
    if (rc) return rc;
  }
  return SO_OK;
}

/* One execution of level L under the current point of level L-1. */
static int run_level(ctx_t* c, int L) {
  const so_block_t* b = c->lvl[L];
  if (L > 0) {
    const int pnv = n_vars_of(c->lvl[L - 1]);
    for (int p = 0; p < b->n_passed; ++p) {
      int64_t s = b->passed_const ? b->passed_const[p] : 0;
      for (int v = 0; v < pnv; ++v) s += b->passed_coeff[(size_t)p * pnv + v] * c->vars[L - 1][v];
      c->vars[L][b->n_idx + p] = s;
    }
  }
  return loop_index(c, L, 0);
}

static int collect(ctx_t* c, const so_block_t* root) {
  c->n_levels = 0;
  for (const so_block_t* b = root; b; b = b->child) {
    if (c->n_levels == SO_MAX_LEVELS) return fail(c, SO_ERR_BAD_BLOCK, "more than %lld levels", (long long)(SO_MAX_LEVELS));
    c->lvl[c->n_levels++] = b;
  }
  if (c->n_levels < 2) return fail(c, SO_ERR_BAD_BLOCK, "need a declaring root and at least one block");
  if (root->n_idx != 0 || root->n_passed != 0 || root->n_cons != 0)
    return fail(c, SO_ERR_BAD_BLOCK, "the root block declares buffers only: no indexes or constraints");
  c->n_refs = root->n_refs;
  if (c->n_refs < 2 || c->n_refs > SO_MAX_REFS) return fail(c, SO_ERR_BAD_BLOCK, "bad refinement count %lld", (long long)(c->n_refs));
  c->out_ref = c->n_refs - 1;
  c->agg = SO_AGG_ASSIGN;
  for (int l = 0; l < c->n_levels; ++l) {
    const so_block_t* b = c->lvl[l];
    if (b->n_refs != c->n_refs) return fail(c, SO_ERR_BAD_BLOCK, "level %lld: refinement count differs from the root", (long long)(l));
    if (b->n_idx < 0 || b->n_passed < 0 || n_vars_of(b) > SO_MAX_VARS) return fail(c, SO_ERR_BAD_BLOCK, "level %lld: too many variables", (long long)(l));
    c->iters[l] = 1;
    for (int j = 0; j < b->n_idx; ++j) {
      if (b->ranges[j] < 0) return fail(c, SO_ERR_BAD_BLOCK, "level %lld index %lld: negative range", (long long)(l), (long long)(j));
      c->iters[l] *= b->ranges[j];
    }
    for (int r = 0; r < c->n_refs; ++r) {
      const so_ref_t* ref = &b->refs[r];
      const so_ref_t* top = &root->refs[r];
      if (ref->ndim != top->ndim || ref->ndim < 1 || ref->ndim > SO_MAX_DIMS || ref->dtype != top->dtype || ref->dir != top->dir)
        return fail(c, SO_ERR_BAD_BLOCK, "level %lld refinement %lld: shape, type or direction differs from the root", (long long)(l), (long long)(r));
      if (ref->dir != (r == c->out_ref ? SO_DIR_OUT : SO_DIR_IN))
        return fail(c, SO_ERR_BAD_BLOCK, "refinement %lld: inputs come first, the output last", (long long)(r));
      for (int d = 0; d < ref->ndim; ++d)
        if (ref->strides[d] != top->strides[d] || ref->strides[d] < 0 || ref->sizes[d] < 1)
          return fail(c, SO_ERR_BAD_BLOCK, "level %lld refinement %lld dim %lld: a view keeps its parent's (non-negative) strides and has positive sizes", (long long)(l), (long long)(r), (long long)(d));
    }
    /* Each level aggregates with the nest's one operation, or declares with
     * 'assign' that its iterations write disjoint elements. */
    const int a = b->refs[c->out_ref].agg;
    if (a != SO_AGG_ASSIGN) {
      if (c->agg != SO_AGG_ASSIGN && c->agg != a) return fail(c, SO_ERR_BAD_BLOCK, "level %lld: a second aggregation operation in one nest", (long long)(l));
      c->agg = a;
    }
  }
  const so_block_t* leaf = c->lvl[c->n_levels - 1];
  const int n_in = c->n_refs - 1;
  if (leaf->intrinsic == SO_INTR_COPY ? n_in != 1 : n_in != 2) return fail(c, SO_ERR_BAD_BLOCK, "intrinsic %lld does not take %lld inputs", (long long)(leaf->intrinsic), (long long)(n_in));
  const int odt = root->refs[c->out_ref].dtype;
  /* a bf16 output buffer is a float block too: the result is returned in fp64, rounding it to the buffer's type is
     left to whoever compares */
  if (odt != SO_I32 && odt != SO_F32 && odt != SO_BF16) return fail(c, SO_ERR_BAD_BLOCK, "output type must be i32, f32 or bf16");
  c->int_mode = (odt == SO_I32);
  for (int r = 0; r < n_in; ++r) {
    const int dt = root->refs[r].dtype;
    const int is_int = (dt == SO_I8 || dt == SO_I32);
    if (is_int != c->int_mode) return fail(c, SO_ERR_BAD_BLOCK, "input %lld: integer and float buffers mixed", (long long)(r));
  }
  return SO_OK;
}

int64_t so_output_extent(const so_block_t* root) {
  if (!root || root->n_refs < 1) return -1;
  const so_ref_t* o = &root->refs[root->n_refs - 1];
  int64_t hi = 0;
  for (int d = 0; d < o->ndim; ++d) {
    if (o->strides[d] < 0 || o->access_const[d] < 0 || o->sizes[d] < 1) return -1;
    hi += (o->access_const[d] + o->sizes[d] - 1) * o->strides[d];
  }
  return hi + 1;
}

int so_eval(const so_block_t* root, const void* const* inputs, double* out_f64, int64_t* out_i64,
            uint8_t* touched, const int64_t* win_lo, const int64_t* win_hi, int64_t* n_points,
            char* err, size_t errlen) {
  ctx_t* c = (ctx_t*)calloc(1, sizeof(ctx_t));
  if (!c) return SO_ERR_BAD_BLOCK;
  c->err = err;
  c->errlen = errlen;
  if (err && errlen) err[0] = 0;
  int rc = root ? collect(c, root) : SO_ERR_BAD_BLOCK;
  if (rc == SO_OK) {
    if (!inputs || !touched || (c->int_mode ? !out_i64 : !out_f64))
      rc = fail(c, SO_ERR_BAD_BLOCK, "missing input, output or touched array");
  }
  if (rc == SO_OK && so_output_extent(root) < 1) rc = fail(c, SO_ERR_BAD_BLOCK, "bad output declaration");
  if (rc == SO_OK && win_lo && win_hi) {
    for (int j = 0; j < c->lvl[1]->n_idx; ++j)
      if (win_lo[j] < 0 || win_hi[j] > c->lvl[1]->ranges[j])
        rc = fail(c, SO_ERR_BAD_BLOCK, "window of index %lld leaves its range", (long long)j);
  }
  if (rc == SO_OK) {
    const int64_t ext = so_output_extent(root);
    for (int l = 1; l < c->n_levels && rc == SO_OK; ++l) {
      if (c->lvl[l]->refs[c->out_ref].agg == SO_AGG_ASSIGN && c->iters[l] > 1) {
        c->owner[l] = (int64_t*)malloc(sizeof(int64_t) * (size_t)(ext > 0 ? ext : 1));
        if (!c->owner[l]) rc = fail(c, SO_ERR_BAD_BLOCK, "out of memory");
        else for (int64_t i = 0; i < ext; ++i) c->owner[l][i] = -1;
      }
    }
  }
  if (rc == SO_OK) {
    c->inputs = inputs;
    c->out_f64 = out_f64;
    c->out_i64 = out_i64;
    c->touched = touched;
    c->win_lo = win_lo;
    c->win_hi = win_hi;
    rc = run_level(c, 0);
  }
  if (n_points) *n_points = c->n_points;
  for (int l = 0; l < SO_MAX_LEVELS; ++l) free(c->owner[l]);
  free(c);
  return rc;
}
