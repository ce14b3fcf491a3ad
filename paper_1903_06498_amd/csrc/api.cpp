// C ABI of the Stripe block executor: see include/stripe.h.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <new>
#include <string>

#include "kernels.hpp"
#include "plan.hpp"

using namespace stripe;

struct stripe_block {
  Plan plan;
  GemmLaunch gemm;
  ConvLaunch conv;
  PoolLaunch pool;
  int n_inputs = 0;
};

namespace {

thread_local std::string g_last_error;

stripe_status_t fail(stripe_status_t st, const std::string& msg) {
  g_last_error = msg;
  return st;
}

}  // namespace

namespace stripe {
stripe_status_t api_fail(stripe_status_t st, const std::string& msg) { return fail(st, msg); }
}  // namespace stripe

extern "C" {

stripe_status_t stripe_block_create_for_path(const stripe_block_desc_t* desc, stripe_path_t path, stripe_block_t** out) {
  if (!desc || !out) return fail(STRIPE_ERR_NULL, "desc or out is NULL");
  *out = nullptr;
  if (path < STRIPE_PATH_AUTO || path > STRIPE_PATH_POOL) return fail(STRIPE_ERR_INVALID_DESC, "unknown path");
  std::string err;
  FlatBlock fb;
  stripe_status_t st = flatten(desc, &fb, &err);
  if (st == STRIPE_OK) st = prove_checks(fb, &err);
  if (st == STRIPE_OK) st = check_assign_levels(fb, &err);
  if (st != STRIPE_OK) return fail(st, err);
  canonicalize(&fb);
  stripe_block* blk = new (std::nothrow) stripe_block();
  if (!blk) return fail(STRIPE_ERR_NOMEM, "out of host memory");
  st = make_plan(fb, path, &blk->plan, &err);
  if (st != STRIPE_OK) {
    delete blk;
    return fail(st, err);
  }
  blk->n_inputs = fb.n_refs - 1;
  Plan& p = blk->plan;
  if (tune_int("generic_i64", 0)) p.gen.narrow = 0;   // test hook: 64-bit index arithmetic in the generic kernel
  if (tune_int("generic_i64", 0) || !tune_int("generic_tiled", 1)) p.tiled.use = 0;
  else if (tune_int("generic_tiled", 1) == 2 && p.tiled.n_items > 0) p.tiled.use = 1;   // test hook: tiled kernel also for small blocks
  if (!p.noop) {
    const bool forced = path != STRIPE_PATH_AUTO;
    bool picked = false;
    switch (p.info.path) {
      case STRIPE_PATH_MFMA_GEMM: picked = gemm_select(p.gemm, p.in_dtype, &blk->gemm, &p.info); break;
      case STRIPE_PATH_MFMA_CONV: picked = conv_select(p.conv, p.in_dtype, &blk->conv, &p.info); break;
      case STRIPE_PATH_POOL: picked = pool_select(p.pool, p.in_dtype, &blk->pool, &p.info); break;
      default: break;
    }
    if (!picked) {
      if (forced && p.info.path != STRIPE_PATH_GENERIC) {
        delete blk;
        return fail(STRIPE_ERR_UNSUPPORTED, "the requested kernel family has no variant for this shape (tile divisibility, layout or element type)");
      }
      if (p.gen.n_outputs < 0) {
        delete blk;
        return fail(STRIPE_ERR_UNSUPPORTED, "no kernel family covers this block");
      }
      generic_info(p, &p.info);
    }
  }
  *out = blk;
  return STRIPE_OK;
}

stripe_status_t stripe_block_create(const stripe_block_desc_t* desc, stripe_block_t** out) {
  return stripe_block_create_for_path(desc, STRIPE_PATH_AUTO, out);
}

stripe_status_t stripe_block_run(stripe_block_t* blk, const void* const* inputs, void* output, void* hip_stream) {
  if (!blk || !inputs || !output) return fail(STRIPE_ERR_NULL, "blk, inputs or output is NULL");
  for (int i = 0; i < blk->n_inputs; ++i)
    if (!inputs[i]) return fail(STRIPE_ERR_NULL, "an input pointer is NULL");
  const Plan& p = blk->plan;
  if (p.noop) return STRIPE_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  const void* in0 = inputs[0];
  const void* in1 = blk->n_inputs > 1 ? inputs[1] : nullptr;
  hipError_t e = hipSuccess;
  switch (p.info.path) {
    case STRIPE_PATH_MFMA_GEMM: e = launch_gemm(p.gemm, blk->gemm, in0, in1, output, s); break;
    case STRIPE_PATH_MFMA_CONV: e = launch_conv(p.conv, blk->conv, in0, in1, output, s); break;
    case STRIPE_PATH_POOL: e = launch_pool(p.pool, blk->pool, in0, output, s); break;
    default: e = launch_generic(p, in0, in1, output, s); break;
  }
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
  return STRIPE_OK;
}

stripe_status_t stripe_block_query(const stripe_block_t* blk, stripe_block_info_t* info) {
  if (!blk || !info) return fail(STRIPE_ERR_NULL, "blk or info is NULL");
  *info = blk->plan.info;
  return STRIPE_OK;
}

void stripe_block_destroy(stripe_block_t* blk) { delete blk; }

const char* stripe_status_string(stripe_status_t status) {
  switch (status) {
    case STRIPE_OK: return "ok";
    case STRIPE_ERR_NULL: return "null pointer argument";
    case STRIPE_ERR_INVALID_DESC: return "invalid block descriptor";
    case STRIPE_ERR_UNSUPPORTED: return "unsupported block";
    case STRIPE_ERR_OUT_OF_BOUNDS: return "access may leave its buffer or view";
    case STRIPE_ERR_ASSIGN_CONFLICT: return "assign aggregation with several writers";
    case STRIPE_ERR_HIP: return "HIP runtime error";
    case STRIPE_ERR_NOMEM: return "out of memory";
  }
  return "unknown status";
}

const char* stripe_last_error(void) { return g_last_error.c_str(); }

stripe_status_t stripe_device_copy(const void* src, void* dst, size_t n_bytes, void* hip_stream) {
  if (!src || !dst) return fail(STRIPE_ERR_NULL, "src or dst is NULL");
  if (n_bytes % 16 || ((uintptr_t)src % 16) || ((uintptr_t)dst % 16))
    return fail(STRIPE_ERR_INVALID_DESC, "copy needs 16-byte aligned pointers and size");
  const hipError_t e = launch_copy(src, dst, n_bytes, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("copy launch failed: ") + hipGetErrorString(e));
  return STRIPE_OK;
}

}  // extern "C"
