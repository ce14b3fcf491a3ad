/*
 * Stripe block oracle -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow CPU evaluator of a nested Stripe block, used only by the
 * tests, the smoke check and the benchmark's cpu_baseline leg to judge the
 * GPU library.  It shares no code, header or table with the GPU library and
 * neither includes the other.
 *
 * What it computes (paper, Section 3.1.2, Definition 2, rule 3, with the
 * Stripe restrictions of Section 3.2): every integer point of the iteration
 * space of every nesting level is visited by literal loops; at each point all
 * affine constraints of that level are tested; at the leaf the statement list
 * load / (mul) / store runs, and all values written to one output element are
 * combined with the buffer's aggregation operation.  An element written by
 * exactly one iteration receives that value as is.  An element that no
 * iteration writes is left untouched.
 *
 * Nesting (Section 3.1.3, Section 3.2 "refinements", Figure 5b): a level's
 * refinement gives, per buffer dimension, an affine access in that level's
 * variables.  It is the origin of the view handed to the level's statements,
 * measured from the origin of the view the level itself received.  The
 * absolute coordinate of a scalar access is the sum of the accesses of all
 * levels.  Parent indexes reach a child only as explicitly passed affine
 * functions (Figure 5b: xo = 3*x).
 *
 * Precision: float blocks accumulate in fp64 (bf16/fp32 inputs widen exactly,
 * their product is exact in fp64); integer blocks accumulate in int64 and
 * every partial sum must fit int32, otherwise evaluation fails.
 */
#ifndef STRIPE_ORACLE_H
#define STRIPE_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { SO_DIR_IN = 0, SO_DIR_OUT = 1 };
enum { SO_I8 = 0, SO_I32 = 1, SO_BF16 = 2, SO_F32 = 3 };
enum { SO_AGG_ASSIGN = 0, SO_AGG_ADD = 1, SO_AGG_MAX = 2, SO_AGG_MIN = 3, SO_AGG_MUL = 4 };
enum { SO_INTR_MUL = 0, SO_INTR_COPY = 1, SO_INTR_ADD = 2, SO_INTR_ADD_RELU = 3 /* load, load, add, relu (max with 0), store */ };

enum {
  SO_OK = 0,
  SO_ERR_BAD_BLOCK = 1,     /* malformed description */
  SO_ERR_OUT_OF_BOUNDS = 2, /* an executed access left its buffer or its view */
  SO_ERR_ASSIGN = 3,        /* two iterations of an 'assign' level wrote one element */
  SO_ERR_INT_OVERFLOW = 4   /* an integer partial result does not fit int32 */
};

#define SO_MAX_LEVELS 8
#define SO_MAX_VARS 24
#define SO_MAX_REFS 4
#define SO_MAX_DIMS 8

/* One refinement: a buffer as one level sees it (Section 3.2). */
typedef struct {
  int32_t dir;                 /* SO_DIR_* */
  int32_t dtype;               /* SO_* element type */
  int32_t agg;                 /* SO_AGG_*, meaningful for the output */
  int32_t ndim;
  const int64_t* access_coeff; /* [ndim][n_idx + n_passed], row-major */
  const int64_t* access_const; /* [ndim] */
  const int64_t* sizes;        /* [ndim] extent of the view this level hands on
                                  (root: extent of the buffer; leaf: all 1) */
  const int64_t* strides;      /* [ndim] in elements */
} so_ref_t;

/* One nesting level.  Variables of a level = its own indexes, then its passed
 * parent values.  Level 0 is the declaring root block: no indexes, one
 * iteration (Figure 5, "block []:1"). */
typedef struct so_block {
  int32_t n_idx;
  const int64_t* ranges;       /* [n_idx], index j runs over 0..ranges[j]-1 */
  int32_t n_passed;
  const int64_t* passed_coeff; /* [n_passed][parent n_idx + parent n_passed] */
  const int64_t* passed_const; /* [n_passed] */
  int32_t n_cons;
  const int64_t* cons_coeff;   /* [n_cons][n_idx + n_passed]; row . vars + const >= 0 */
  const int64_t* cons_const;   /* [n_cons] */
  int32_t n_refs;              /* inputs first, the single output last */
  const so_ref_t* refs;
  int32_t intrinsic;           /* SO_INTR_*, leaf only */
  const struct so_block* child; /* NULL at the leaf */
} so_block_t;

/* Number of elements the output buffer must hold (largest address + 1). */
int64_t so_output_extent(const so_block_t* root);

/*
 * Evaluate the block.
 *   inputs   host pointers, one per input refinement, element type as declared
 *   out_f64  accumulator image of the output buffer for float blocks, else NULL
 *   out_i64  the same for integer blocks, else NULL
 *            (so_output_extent() elements; untouched elements keep their value)
 *   touched  so_output_extent() bytes; set to 1 where an iteration wrote
 *   win_lo / win_hi  optional window [lo, hi) per index of level 1 (the first
 *            level below the root); NULL = the whole range.  Restricting an
 *            index that the output does not depend on changes the result.
 *   n_points receives the number of leaf points executed (all constraints met)
 * Returns SO_OK or an SO_ERR_* code; err receives a message.
 */
int so_eval(const so_block_t* root, const void* const* inputs, double* out_f64, int64_t* out_i64,
            uint8_t* touched, const int64_t* win_lo, const int64_t* win_hi, int64_t* n_points,
            char* err, size_t errlen);

#ifdef __cplusplus
}
#endif
#endif
