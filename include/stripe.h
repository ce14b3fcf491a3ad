/*
 * stripe.h -- C ABI of the MI355X (gfx950) executor for one Stripe block.
 *
 * A Stripe block (paper, Section 3.2) is a parallel polyhedral block
 * (Section 3.1.2, Definition 2): a list of indexes with one range each, a
 * list of affine constraints "expr >= 0", a single statement list, and the
 * buffers it reads and writes, each with an aggregation operation.  Blocks
 * nest (Section 3.1.3): a statement may be another block, which sees its
 * parent's buffers only through refinements -- offset, sized and strided
 * views -- and its parent's indexes only as explicitly passed affine values
 * (Figure 5b).  This library evaluates such a nest whose leaf statement list
 * is  load, [load, mul|add,] store  on one GPU.
 *
 * All descriptor memory is HOST memory owned by the caller; create() copies
 * what it needs, so the descriptor may be freed right after it returns.
 * Buffers handed to run() are DEVICE pointers owned by the caller.  No
 * function throws or aborts; every failure is a status code, with detail in
 * stripe_last_error().  Apart from that thread-local string the library keeps
 * no global state; handles are independent of each other.
 */
#ifndef STRIPE_H
#define STRIPE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  STRIPE_OK = 0,
  STRIPE_ERR_NULL = 1,            /* a required pointer argument is NULL */
  STRIPE_ERR_INVALID_DESC = 2,    /* malformed descriptor (counts, ranges, shapes, type mix) */
  STRIPE_ERR_UNSUPPORTED = 3,     /* a legal block this library cannot run (yet) */
  STRIPE_ERR_OUT_OF_BOUNDS = 4,   /* an access inside the polyhedron may leave its buffer or view */
  STRIPE_ERR_ASSIGN_CONFLICT = 5, /* 'assign' level whose iterations are not provably disjoint */
  STRIPE_ERR_HIP = 6,             /* a HIP runtime call failed */
  STRIPE_ERR_NOMEM = 7,           /* out of host or device memory, or a workspace / the static scratch is too small */
  STRIPE_ERR_MISALIGNED = 8       /* a buffer pointer lacks the 16-byte alignment the planned kernel family needs */
} stripe_status_t;

typedef enum { STRIPE_I8 = 0, STRIPE_I32 = 1, STRIPE_BF16 = 2, STRIPE_F32 = 3 } stripe_dtype_t;

/* Aggregation operations (Section 2.1 last sentence; Section 3.2: 'assign'
 * declares that no two iterations write the same element). */
typedef enum {
  STRIPE_AGG_ASSIGN = 0, STRIPE_AGG_ADD = 1, STRIPE_AGG_MAX = 2, STRIPE_AGG_MIN = 3,
  STRIPE_AGG_MUL = 4   /* product; integer products wrap in int32 like any int32 arithmetic here */
} stripe_agg_t;

/* Leaf statement lists (Section 3.2 "intrinsics"; Figure 5, the four statements of the inner block):
 *   MUL : $a = load(in0); $b = load(in1); $o = mul($a,$b); out = store($o)
 *   ADD : the same with add
 *   COPY: $a = load(in0); out = store($a)
 *   ADD_RELU: $a = load(in0); $b = load(in1); $o = relu(add($a,$b)); out = store($o)   (relu(v) = max(v, 0)) */
typedef enum { STRIPE_INTR_MUL = 0, STRIPE_INTR_COPY = 1, STRIPE_INTR_ADD = 2, STRIPE_INTR_ADD_RELU = 3 } stripe_intrinsic_t;

/* TEMP: only at the root of a block with several statements: a buffer the library owns, written by one statement
 * and read by later ones.  The caller passes no pointer for it. */
typedef enum { STRIPE_IN = 0, STRIPE_OUT = 1, STRIPE_TEMP = 2 } stripe_dir_t;

/* Which kernel family runs the block (reported by stripe_block_query). */
typedef enum {
  STRIPE_PATH_AUTO = 0,      /* create: let the planner choose */
  STRIPE_PATH_GENERIC = 1,   /* affine-index contraction, any legal block */
  STRIPE_PATH_MFMA_GEMM = 2, /* nested-tile dense contraction on matrix cores */
  STRIPE_PATH_MFMA_CONV = 3, /* nested-tile convolution-shaped contraction on matrix cores */
  STRIPE_PATH_POOL = 4       /* max aggregation over a window of one input */
} stripe_path_t;

/*
 * One refinement (Section 3.2, "refinements"; Figure 5 "in I[3*x - 1, 4*y - 1, 0]
 * i8(5, 6, 8):(128, 8, 1)"): a buffer as one nesting level sees it.
 *   access_coeff [ndim][n_vars] row-major, access_const [ndim]:
 *       per dimension the affine origin of the view, in this level's variables
 *       (own indexes first, then passed values), measured from the origin of
 *       the view the level itself received.  The absolute coordinate of a
 *       leaf access is the sum over all levels.
 *   sizes [ndim]: extent of the view handed to this level's statements
 *       (root level: the extent of the buffer itself; leaf: all 1).  A view
 *       may hang over the edge of its parent (halo tiles); only accesses that
 *       are executed must fall inside every enclosing view and the buffer.
 *   strides [ndim]: in elements, non-negative, identical at every level.
 *   agg: aggregation of the output at this level; each level carries the
 *       nest's single operation or ASSIGN.  Ignored for inputs.
 */
typedef struct {
  stripe_dir_t dir;
  stripe_dtype_t dtype;
  stripe_agg_t agg;
  int32_t ndim;                /* 1..8 */
  const int64_t* access_coeff;
  const int64_t* access_const;
  const int64_t* sizes;
  const int64_t* strides;
} stripe_refinement_t;

/*
 * One nesting level (Section 3.2 first paragraph; Figure 5).
 * The outermost descriptor is the declaring root block ("block []:1"):
 * n_idx = n_passed = n_constraints = 0, its refinements give the buffers'
 * extents, strides and element types, access_const is the element offset of
 * the origin (normally 0) and access_coeff is unused.  Below it come 1..6
 * block levels; the last one (child == NULL) holds the intrinsic.
 * Every level lists the same buffers in the same order: inputs first (one for
 * COPY, two for MUL/ADD), the single output last.
 * Element types: inputs i8/i32 with an i32 output, or bf16/f32 with an f32
 * or bf16 output (rounded to nearest even on store).  Integer arithmetic is exact two's-complement int32 (operands
 * sign-extended before the multiply); float blocks accumulate in fp32.
 */
typedef struct stripe_block_desc {
  int32_t n_idx;
  const int64_t* ranges;        /* [n_idx]; index j takes 0 .. ranges[j]-1; 0 = empty block */
  int32_t n_passed;
  const int64_t* passed_coeff;  /* [n_passed][parent n_vars]: value = row . parent vars + const */
  const int64_t* passed_const;  /* [n_passed] */
  int32_t n_constraints;
  const int64_t* cons_coeff;    /* [n_constraints][n_vars]: row . vars + const >= 0 */
  const int64_t* cons_const;    /* [n_constraints] */
  int32_t n_refs;
  const stripe_refinement_t* refs;
  stripe_intrinsic_t intrinsic; /* leaf only */
  const struct stripe_block_desc* child;
  /* Statement lists (Section 3.2: a block may hold several statements, executed as if in serial).  Supported
   * at the root only: root->child is the first statement, ->next the following ones (NULL ends the list).
   * A statement of a list names the root refinements it uses, inputs first and its output last, in
   * parent_refs[n_refs]; with a single statement parent_refs may be NULL (same positions).  Root refinements
   * then come in the order: the caller's inputs, temporaries (STRIPE_TEMP), the single output last. */
  const struct stripe_block_desc* next;
  const int32_t* parent_refs;
} stripe_block_desc_t;          /* n_vars of a level = n_idx + n_passed */

typedef struct stripe_block stripe_block_t; /* opaque handle */

/* What the planner decided; algorithmic figures count in-polyhedron points only. */
typedef struct {
  int32_t path;               /* stripe_path_t actually used */
  int32_t n_idx;              /* indexes after flattening and merging */
  int32_t n_out_idx;          /* indexes the output address depends on */
  int32_t n_red_idx;          /* reduction indexes */
  int64_t hull_points;        /* product of the flattened ranges */
  int64_t work_points;        /* points meeting all constraints; -1 if not counted */
  int64_t output_elements;    /* distinct output elements the hull can write */
  int64_t algorithmic_bytes;  /* each input and output element once */
  int32_t tile_m, tile_n, tile_k;   /* workgroup tile of the nested-tile paths, else 0 */
  int32_t frag_m, frag_n, frag_k;   /* matrix-core fragment, else 0 */
  int32_t lds_bytes;
  int32_t workgroup_size;
  int64_t grid;               /* workgroups per launch */
  char kernel[96];            /* name of the kernel variant */
  int64_t workspace_bytes;    /* device workspace the handle's launches use (see stripe_block_set_workspace); 0 = none */
} stripe_block_info_t;

/*
 * Validate, flatten and plan a block (host only, no GPU call).
 * Flattening composes refinement offsets down the nest and substitutes passed
 * values (Section 3.1.3), so a tiled nest and its un-tiled form plan alike.
 * Every access is proven to stay inside its buffer and views for all points
 * of the polyhedron, otherwise STRIPE_ERR_OUT_OF_BOUNDS.
 * On success *out receives a handle the caller must release with
 * stripe_block_destroy().
 */
stripe_status_t stripe_block_create(const stripe_block_desc_t* desc, stripe_block_t** out);

/* As stripe_block_create, but forces a kernel family (STRIPE_PATH_AUTO = planner's
 * choice).  STRIPE_ERR_UNSUPPORTED if the block does not have that family's shape. */
stripe_status_t stripe_block_create_for_path(const stripe_block_desc_t* desc, stripe_path_t path,
                                             stripe_block_t** out);

/*
 * Launch the block on `hip_stream` (a hipStream_t; NULL = the default stream)
 * of the current device.  inputs[i] is the DEVICE pointer of the i-th input
 * refinement's buffer origin, output that of the output buffer; element types
 * and extents as declared at the root.  Output elements no iteration writes
 * keep their contents; written elements are overwritten (prior contents do
 * not enter the aggregation).  A block whose output elements are shared
 * between index tuples through different output indexes (O[x + i]) is run as
 * two launches: the aggregation's identity to every reached element, then an
 * atomic combine.  A statement list runs its statements in order on the
 * stream.
 * Workspace: temporaries of a statement list that are not fused away, and
 * the partial sums of a dense contraction whose reduction index is split
 * over workgroups (Section 2.1: aggregations are associative and commutative,
 * so a reduction may be regrouped; chosen at create for products with few
 * output tiles and a long reduction), live in a device workspace of
 * stripe_block_workspace_size() bytes.  If the caller has handed one over
 * with stripe_block_set_workspace(), run() uses it and never allocates;
 * otherwise the handle allocates it on its first run on a device (the only
 * allocation run() ever makes; that first call then is not purely
 * asynchronous) and frees it on destroy.  Either way two overlapping runs of
 * one handle race on the workspace.  Handles that report 0 bytes never
 * allocate.
 * Alignment: the specialised kernel families move 16 bytes per lane.
 * Whether a block's strides and origins keep that alignment is decided at
 * create (a block that does not runs on the generic kernels, which take
 * any element-aligned pointer); the buffer POINTERS are only seen here, and a
 * pointer that is not 16-byte aligned, handed to a handle planned for a
 * specialised family (path != STRIPE_PATH_GENERIC in stripe_block_query),
 * is refused with STRIPE_ERR_MISALIGNED before anything is launched.
 * Non-finite inputs are outside the contract of the specialised families:
 * they realise constraints by feeding zeros for removed points (0 * Inf is
 * NaN where the definition skips the point) and use IEEE maxNum/minNum for
 * max/min (a NaN operand is ignored).
 * Asynchronous: returns after enqueueing; only launch errors are reported.
 * Calls on different handles may overlap; two overlapping calls that write
 * the same output buffer race.
 */
stripe_status_t stripe_block_run(stripe_block_t* blk, const void* const* inputs, void* output,
                                 void* hip_stream);

/*
 * stripe_block_run for callers that cannot allocate device memory (code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc): the same launches, but the handle's workspace (temporaries of a
 * statement list, partial sums of a split reduction) lives in a fixed array of STRIPE_STATIC_SCRATCH_BYTES that
 * is part of the library's code object (each GPU the library runs on holds its own copy until the process
 * ends) instead of memory the handle allocates on its first run; a workspace set with
 * stripe_block_set_workspace is not used by this call.
 * The call makes no hipMalloc / hipFree and calls no allocating library routine; the caller still passes inputs
 * and output.  If stripe_block_workspace_size() exceeds STRIPE_STATIC_SCRATCH_BYTES the call returns
 * STRIPE_ERR_NOMEM and launches nothing (use stripe_block_run then).  Handles that need no workspace use no
 * scratch at all.
 * Every call on a GPU shares that GPU's array, which keeps the previous call's contents; nothing in it needs to
 * start at zero (every element of a temporary or of a partial-sum image is written before it is read).  Two
 * calls that overlap on one GPU (different streams, or different host threads) and both need a workspace RACE
 * on the array: serialise them on one stream.  The array's device address is looked up on the first call on
 * each device.
 */
#define STRIPE_STATIC_SCRATCH_BYTES (8u << 20)
stripe_status_t stripe_block_run_static(stripe_block_t* blk, const void* const* inputs, void* output, void* hip_stream);

/*
 * The device workspace of a handle (see stripe_block_run).  workspace_size: bytes the handle's launches need, 0
 * if none.  set_workspace: `device_ptr` (256-byte aligned DEVICE memory of at least that many bytes, owned by
 * the caller, valid until replaced or the handle is destroyed) becomes the workspace of every later
 * stripe_block_run, which then never allocates; NULL returns to handle-owned memory.  STRIPE_ERR_NOMEM if
 * `bytes` is too small, STRIPE_ERR_INVALID_DESC if misaligned.  Host only.
 */
stripe_status_t stripe_block_workspace_size(const stripe_block_t* blk, size_t* bytes);
stripe_status_t stripe_block_set_workspace(stripe_block_t* blk, void* device_ptr, size_t bytes);

stripe_status_t stripe_block_query(const stripe_block_t* blk, stripe_block_info_t* info);

void stripe_block_destroy(stripe_block_t* blk);

const char* stripe_status_string(stripe_status_t status);

/* Detail of the last failure on the calling thread ("" if none).  The pointer
 * stays valid until the next failing call on this thread. */
const char* stripe_last_error(void);

/*
 * Bandwidth yardstick: copies n_bytes (a multiple of 16, both pointers
 * 16-byte aligned DEVICE memory) with a plain grid-stride 16-byte-per-lane
 * kernel on `hip_stream`.  Used to scale hardware traffic counters and to
 * state the achievable HBM rate next to the pooling kernels.
 */
stripe_status_t stripe_device_copy(const void* src, void* dst, size_t n_bytes, void* hip_stream);

/*
 * Streaming yardsticks with a chosen read : write mix: `reads` input streams (0, 1, 2 or 4) of n_vectors 16-byte
 * vectors each, laid one after the other from `src`, are added into one output stream of n_vectors vectors at
 * `dst` (write != 0), or only read (write == 0; dst then points at 4 spare bytes).  Streaming loads and stores, four
 * independent vectors per lane and trip, `grid` workgroups of 256 lanes.  DEVICE pointers, 16-byte aligned.  They
 * state what a perfectly regular kernel with the window kernels' 4 : 1 mix reaches on this chip.
 */
stripe_status_t stripe_device_stream(const void* src, void* dst, size_t n_vectors, int reads, int write, int grid, void* hip_stream);

/*
 * Matrix-core yardstick: every wavefront of `grid` workgroups of 256 lanes runs `iters` (even) passes over a
 * 4 x 4 tile of 32 x 32 x 16 bf16 matrix instructions whose operand fragments stay in registers (no LDS or global
 * traffic inside the loop): iters * 16 instructions = iters * 524,288 flop per wavefront, 4 wavefronts per
 * workgroup.  `operands`: DEVICE, 16-byte aligned, 16 * 256 vectors of 8 bf16 (64 KB): vector (s * 8 + f) * 256 + lane
 * is fragment f (0-3: A, 4-7: B) of operand set s (0, 1; the sets alternate from pass to pass) for lane `lane` of
 * the workgroup.  `out`: DEVICE, grid * 256 floats; each receives the sum of its lane's 256 accumulator elements.
 * from_lds != 0: the fragments are parked in LDS and fetched again before every pass (eight 16-byte reads per lane
 * for sixteen instructions, the contraction kernels' ratio) instead of staying in registers.
 * It states what the chip sustains for the contraction kernels' instruction on given operand values, apart from
 * the memory system (Section 3.3's roofline speaks of the compute roof; this measures it).
 */
stripe_status_t stripe_device_mfma(const void* operands, void* out, int iters, int from_lds, int grid, void* hip_stream);

/* ------------------------------------------------------------------------
 * Autotiling (paper Section 3.3, Figures 4 and 5): host-only integer code.
 *
 * All three calls take the FLAT form of a block: the declaring root (no
 * indexes) whose child is the leaf.  A tile gives one size per leaf index,
 * 1 <= tile[j] <= ranges[j]; tile[j] == ranges[j] leaves index j whole.
 *
 * Cost model (Figure 4's caption): cache lines touched per unit of work.
 * For every counted refinement the tile's view is the box its accesses span
 * over one tile, overflow and halo included (constraints remove those
 * accesses at run time but the view still holds them).  Lines of a view =
 * product of its extents, the stride-1 dimension counted in whole lines
 * (views taken as line-aligned); footprint = product of its extents.
 *   cost = tiles * lines_per_tile / work,   tiles = prod ceil(range_j / tile_j),
 * work = product of the ranges of the indexes in `tiled_idx` (the figure
 * counts work in points of the tiled, spatial indexes: with 8 input
 * channels, 16 output channels, lines of 8 elements and a 512-element cap
 * this reproduces its 4.5 for the 3 x 4 tile and 4.666 for 6 x 2; dividing
 * by multiply-accumulates instead scales every cost of a block by one
 * constant).  A tile is inadmissible if its footprint exceeds the cap, or
 * if it violates `multiple_of` / `power_of_two` (Section 3.3: memory cap,
 * multiples of an earlier tensorisation, power-of-two pruning); a size equal
 * to the whole range is always allowed.
 */
typedef struct {
  int64_t line_elems;         /* cache line size in elements, >= 1 */
  int64_t mem_cap_elems;      /* cap on the summed footprints of the counted views, in elements; 0 = no cap */
  uint32_t counted_refs;      /* bit r: refinement r (descriptor order) counts toward lines and footprint */
  uint32_t tiled_idx;         /* bit j: index j may be tiled by the search and counts as work */
  int32_t power_of_two;       /* non-zero: the search tries power-of-two sizes only */
  const int64_t* multiple_of; /* [n_idx] or NULL: tile[j] must be a multiple of multiple_of[j] (entries < 1 = 1) */
} stripe_tile_model_t;

typedef struct {
  int64_t tiles;
  int64_t lines_per_tile;
  int64_t footprint_elems;
  int64_t work;
  double cost;
  int32_t admissible;
} stripe_tile_cost_t;

/* Cost of one given tile.  STRIPE_ERR_INVALID_DESC if root is not a flat form or a size is out of range. */
stripe_status_t stripe_tile_cost(const stripe_block_desc_t* root, const int64_t* tile, const stripe_tile_model_t* model,
                                 stripe_tile_cost_t* out);

/* Exhaustive search over the sizes of the indexes in model->tiled_idx (all others stay whole).
 * best_tile[n_idx] receives the admissible tile of least cost; ties go to fewer tiles, then to the
 * lexicographically larger tile.  STRIPE_ERR_UNSUPPORTED if no tile is admissible or the space
 * exceeds 2^22 candidates. */
stripe_status_t stripe_tile_search(const stripe_block_desc_t* root, const stripe_tile_model_t* model, int64_t* best_tile,
                                   stripe_tile_cost_t* best);

/*
 * The tiling rewrite (Section 3.3; Figure 5a -> 5b): returns a new nest
 * root -> outer block (ranges ceil(range_j / tile_j), refinements with the
 * tile's views: offsets scaled by the tile size, sizes including the halo) ->
 * inner block (ranges tile_j, accesses relative to the view, the original
 * constraints with every tiled index replaced by "passed outer value + inner
 * index", and one overflow constraint per index whose tile does not divide
 * its range).  The result is semantically the input block.  It is HOST
 * memory owned by the caller: release it with stripe_desc_free().
 */
stripe_status_t stripe_block_tile(const stripe_block_desc_t* root, const int64_t* tile, stripe_block_desc_t** out);
void stripe_desc_free(stripe_block_desc_t* desc);

#ifdef __cplusplus
}
#endif
#endif /* STRIPE_H */
