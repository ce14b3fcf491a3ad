// Host-side planner of the Stripe block executor: descriptor -> flat affine
// form -> canonical form -> kernel family and launch parameters.
// Integer arithmetic only; runs once per handle at create time.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "../../include/stripe.h"

namespace stripe {

constexpr int kMaxFlatIdx = 24;  // indexes of all levels together
constexpr int kMaxDims = 8;
constexpr int kMaxRefs = 3;
constexpr int kMaxLevels = 8;    // root + 7

// sum_j c[j] * idx[j] + k over the flat index list
struct Affine {
  int64_t c[kMaxFlatIdx];
  int64_t k;
};

struct FlatRef {
  int dir = 0, dtype = 0, ndim = 0;
  int64_t sizes[kMaxDims] = {};    // extents of the buffer (root level)
  int64_t strides[kMaxDims] = {};
  Affine coord[kMaxDims];          // absolute coordinate of the leaf access, per dimension
  Affine addr;                     // element address from the buffer origin
  int64_t elements = 0;            // product of sizes
};

// 0 <= rel < size must hold at every executed point (a leaf access inside an enclosing view)
struct RangeCheck {
  Affine rel;
  int64_t size;
  int ref, dim, level;
};

struct FlatBlock {
  int n_idx = 0;
  int64_t range[kMaxFlatIdx] = {};
  int level_of[kMaxFlatIdx] = {};   // nesting level that declared the index (1-based; 0 after merging)
  std::vector<Affine> cons;         // each >= 0
  int n_refs = 0;
  FlatRef ref[kMaxRefs];
  std::vector<RangeCheck> checks;   // buffer bounds and view containment
  int agg = STRIPE_AGG_ASSIGN;      // the nest's one aggregation (ASSIGN if every level says assign)
  int level_agg[kMaxLevels] = {};   // output aggregation declared per level
  int n_levels = 0;
  int intrinsic = STRIPE_INTR_MUL;
  bool int_mode = false;
  bool out_bf16 = false;            // float block whose output buffer holds bf16 (rounded on store)
  bool empty = false;               // some range is 0 or the constraints exclude every point
};

struct GemmShape {       // C[b,m,n] (+)= A[b,m,k] * B[b,k,n]   (batch = 1: no batch index)
  int64_t M, N, K;
  int64_t a_m, a_k, b_k, b_n, c_m, c_n;   // element strides
  int64_t a_base, b_base, c_base;
  int64_t batch, a_b, b_b, c_b;           // batch count and element strides of the batch index (every operand moves with it)
};

struct Conv2dShape {     // O[n,y,x,k] (+)= I[n, s*y+d*i-p, s*x+d*j-q, c] * F[i,j,k,c]  (any strides)
  int64_t N, Ho, Wo, Co, R, S, Ci, H, W;
  int64_t stride_y, stride_x, pad_y, pad_x;
  int64_t dil_y, dil_x;                   // dilation: coefficient of the tap indexes i, j in the input access
  int64_t i_n, i_y, i_x, i_c;             // input element strides
  int64_t f_r, f_s, f_k, f_c;             // filter element strides
  int64_t o_n, o_y, o_x, o_k;             // output element strides
  int64_t i_base, f_base, o_base;
};

struct Pool2dShape {     // O[n,y,x,c] = agg over in-bounds taps of I[n, s*y+d*i-p, s*x+d*j-q, c]
  int64_t N, Ho, Wo, C, R, S, H, W;
  int64_t stride_y, stride_x, pad_y, pad_x;
  int64_t dil_y, dil_x;
  int64_t i_n, i_y, i_x, i_c, o_n, o_y, o_x, o_c;
  int64_t i_base, o_base;
  int agg;                 // STRIPE_AGG_MAX, _MIN or _ADD (sum pooling)
  // Weighted windows (MUL intrinsic, sum aggregation, no channel reduction): every tap is multiplied by an element of
  // a second input.  w_mode 0: none (COPY intrinsic); 1: one scalar for all taps (average pooling, the scale as a
  // one-element buffer); 2: a weight per tap and channel, W[i, j, c] (depthwise convolution).
  int w_mode;
  int64_t w_base, w_r, w_s, w_c;
};

// Parameters of the generic affine-index kernel (passed by value as kernel argument).
constexpr int kGenIdx = 8;
constexpr int kGenCons = 8;
struct GenericParams {
  int32_t n_out, n_red, lanes;
  int32_t narrow;                  // 1: offsets, constraint values and the output count all fit in 32 bits
  int32_t out_range[kGenIdx], red_range[kGenIdx];
  int64_t a_out[kGenIdx], b_out[kGenIdx], o_out[kGenIdx];
  int64_t a_red[kGenIdx], b_red[kGenIdx];
  int64_t a_base, b_base, o_base;
  int32_t cons_out[kGenCons][kGenIdx], cons_red[kGenCons][kGenIdx];
  int64_t cons_const[kGenCons];
  int64_t n_outputs;
  uint32_t red_total, inner_range;
  int32_t point4, pad_;            // point4 1: no reduction, no constraints, four consecutive outputs per lane (vector loads and stores)
  int32_t atomic, out_bf16;        // atomic 1: output map not injective on the output indexes -> identity pass + atomic combine
};

// Parameters of the register-tiled generic contraction kernel: every lane owns a 4 x 4 patch of outputs
// (4 values of one index that only the first operand and the output use, times 4 values of one index that only
// the second operand and the output use) and walks the reduction indexes with up to four nested loops.
constexpr int kTiledOuter = 6;
constexpr int kTiledRed = 4;
struct TiledParams {
  int32_t use;                               // 0: this block runs on the plain generic kernel
  int32_t vec;                               // 1 or 4: elements fetched per load along the innermost reduction index
  int32_t n_outer, n_cons;
  int32_t outer_range[kTiledOuter], a_outer[kTiledOuter], b_outer[kTiledOuter], o_outer[kTiledOuter];
  int32_t cons_outer[kGenCons][kTiledOuter];
  int32_t pm_range, pn_range, pm_blocks, pn_blocks;
  int32_t a_pm, o_pm, b_pn, o_pn;
  int32_t cons_pm[kGenCons];
  int32_t red_range[kTiledRed], a_red[kTiledRed], b_red[kTiledRed];   // [0] innermost; no constraint depends on it
  int32_t cons_red[kGenCons][kTiledRed];
  int32_t cons_const[kGenCons];
  int32_t a_base, b_base, o_base;
  int32_t pad_;
  int64_t n_items;                           // lanes: pn_blocks * pm_blocks * prod(outer_range)
};

struct Plan {
  FlatBlock flat;                  // canonical form
  stripe_block_info_t info = {};
  bool noop = false;               // empty iteration space: run() launches nothing
  GenericParams gen = {};
  TiledParams tiled = {};
  GemmShape gemm = {};
  Conv2dShape conv = {};
  Pool2dShape pool = {};
  int in_dtype = 0;
  bool is_gemm = false, is_conv = false, is_pool = false;   // which shape matchers accept the block (gemm / conv / pool filled accordingly)
};

// Each returns STRIPE_OK or an error with `err` filled.
stripe_status_t flatten(const stripe_block_desc_t* root, FlatBlock* out, std::string* err);
stripe_status_t prove_checks(const FlatBlock& fb, std::string* err);
stripe_status_t check_assign_levels(const FlatBlock& fb, std::string* err);
void canonicalize(FlatBlock* fb);
stripe_status_t make_plan(const FlatBlock& canonical, stripe_path_t forced, Plan* plan, std::string* err);

bool match_gemm(const FlatBlock& fb, GemmShape* g);
bool match_conv2d(const FlatBlock& fb, Conv2dShape* c);
bool match_pool2d(const FlatBlock& fb, Pool2dShape* p);

int64_t count_points(const FlatBlock& fb, int64_t enumeration_cap);
void address_form(const FlatBlock& fb, size_t target, std::vector<int64_t>* rng, std::vector<int64_t>* ca, std::vector<int64_t>* cb,
                  std::vector<int64_t>* cc);

// ---- Section 3.3's cost model, usable by the kernel selectors -------------------------------------------------
// A block as the model sees it: index ranges, and per buffer the coefficient of every index in every dimension's
// access plus the dimension's stride (the stride-1 dimension is the one counted in lines).
struct TileRef {
  std::vector<int64_t> coeff;    // [ndim][n_idx] row-major
  std::vector<int64_t> stride;   // [ndim]
};
struct TileProblem {
  std::vector<int64_t> range;
  std::vector<TileRef> refs;
};
void tile_cost_of(const TileProblem& pr, const int64_t* tile, const stripe_tile_model_t& m, stripe_tile_cost_t* c);
bool tile_search_in(const TileProblem& pr, const stripe_tile_model_t& m, const std::vector<std::vector<int64_t>>& cand,
                    std::vector<int64_t>* best_tile, stripe_tile_cost_t* best);

// Parameter sets of that model for the two memory levels of a gfx950 compute unit that the kernel families tile for.
//   register level: a "line" is one 16-byte vector load (four 32-bit registers); the hard cap is the 256 registers a
//     lane can address with two wavefronts per SIMD; below it every data register costs occupancy, which the
//     selectors charge as a factor 1 + registers * kGfx950RegPenalty on the model's cost (fitted to the strip-height
//     measurements of the window kernels: 0.3 % per register);
//   LDS level: lines of 128 bytes; the cap is the CU's 160 KB.
constexpr int64_t kGfx950RegLineBytes = 16, kGfx950RegCapRegs = 256;
constexpr double kGfx950RegPenalty = 0.003;
// window kernels, fitted together with the register penalty: an access served by the CU's L1 costs about a quarter of
// a vector fetched from L2; launches keep at least eight workgroups per CU when the block allows
constexpr double kGfx950L1AccessCost = 0.26;
constexpr int64_t kGfx950MinWorkgroups = 2048;
constexpr int64_t kGfx950LdsLineBytes = 128, kGfx950LdsCapBytes = 160 * 1024;

// Records the calling thread's error detail (what stripe_last_error() returns) and passes the status through.
stripe_status_t api_fail(stripe_status_t st, const std::string& msg);

}  // namespace stripe
