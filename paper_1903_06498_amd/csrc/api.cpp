// C ABI of the Stripe block executor: see include/stripe.h.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.hpp"
#include "plan.hpp"

using namespace stripe;

// One statement of a root block's statement list, planned like a block of its own, with the root refinements it
// reads and writes.
struct Stage {
  stripe_block* blk = nullptr;
  int n_in = 0;
  int src[2] = {-1, -1};
  int dst = -1;
};

struct stripe_block {
  Plan plan;
  GemmLaunch gemm;
  ConvLaunch conv;
  PoolLaunch pool;
  int n_inputs = 0;
  // statement lists (empty for a single block): stages in order, and per root refinement either the caller's
  // input number, or the size of a temporary the handle owns (allocated on the first run, per device)
  std::vector<Stage> stages;
  std::vector<int> input_slot;       // root refinement -> index into run()'s inputs, -1 otherwise
  std::vector<int64_t> temp_bytes;   // root refinement -> bytes of the temporary, 0 otherwise
  // Device workspace of the handle's launches: temporaries of a statement list (temp_off), then each stage's own
  // workspace (stage_ws_off); for a single block the partial sums of a split reduction.  Every part starts on a
  // 256-byte boundary.  The memory is the caller's (set_workspace), else the handle's (allocated on the first
  // run on a device), else the library's static scratch array (run_static).
  std::vector<int64_t> temp_off, stage_ws_off;
  int64_t ws_bytes = 0;
  void* caller_ws = nullptr;
  size_t caller_ws_bytes = 0;
  void* owned_ws = nullptr;
  int owned_ws_dev = -1;
  // 1, 2: the two statements run as one convolution kernel with a bias+relu epilogue (fp32 / bf16 output);
  // 3, 4: the same with the dense-contraction kernel
  int fused = 0;
  int64_t fuse_bias_off = 0, fuse_o_m = 0, fuse_o_base = 0;
  ~stripe_block() {
    for (Stage& st : stages) delete st.blk;
    if (owned_ws) (void)hipFree(owned_ws);
  }
};

// Scratch memory of stripe_block_run_static(): one array per GPU, part of the code object, never allocated or
// freed.  In host code the name is only a stand-in for the symbol; the device address of each GPU's copy is
// looked up once per device (static_scratch_of) and only that pointer is ever handed to a kernel.
static __device__ __align__(256) unsigned char scratch[STRIPE_STATIC_SCRATCH_BYTES];

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

namespace {

int64_t round_up_256(int64_t v) { return (v + 255) / 256 * 256; }

stripe_status_t create_single(const stripe_block_desc_t* desc, stripe_path_t path, stripe_block_t** out);

// A root block with a statement list (Section 3.2: statements execute as if in serial): every statement is planned
// as a block of its own over the root buffers it names; temporaries of the root live in memory the handle owns.
stripe_status_t create_program(const stripe_block_desc_t* root, stripe_path_t path, stripe_block_t** out) {
  if (root->n_idx != 0 || root->n_passed != 0 || root->n_constraints != 0 || !root->refs || root->n_refs < 2 || root->n_refs > 16)
    return fail(STRIPE_ERR_INVALID_DESC, "a statement list needs a declaring root block with 2..16 buffers");
  if (path != STRIPE_PATH_AUTO && path != STRIPE_PATH_GENERIC)
    return fail(STRIPE_ERR_UNSUPPORTED, "a kernel family can be forced for single blocks only");
  const int R = root->n_refs;
  stripe_block* prog = new (std::nothrow) stripe_block();
  if (!prog) return fail(STRIPE_ERR_NOMEM, "out of host memory");
  prog->input_slot.assign(R, -1);
  prog->temp_bytes.assign(R, 0);
  std::vector<char> written(R, 0);
  int n_inputs = 0, phase = 0;
  for (int r = 0; r < R; ++r) {
    const stripe_refinement_t& t = root->refs[r];
    const int want = t.dir == STRIPE_IN ? 0 : t.dir == STRIPE_TEMP ? 1 : 2;
    if (want < phase || (r == R - 1) != (t.dir == STRIPE_OUT) || t.ndim < 1 || t.ndim > 8 || !t.sizes || !t.strides || !t.access_const) {
      delete prog;
      return fail(STRIPE_ERR_INVALID_DESC, "root buffers come as inputs, then temporaries, then the single output");
    }
    phase = want;
    if (t.dir == STRIPE_IN) {
      prog->input_slot[r] = n_inputs++;
      written[r] = 1;
    } else if (t.dir == STRIPE_TEMP) {
      if (t.dtype != STRIPE_F32 && t.dtype != STRIPE_I32) {
        delete prog;
        return fail(STRIPE_ERR_UNSUPPORTED, "temporaries hold f32 or i32");
      }
      int64_t extent = 1;
      for (int d = 0; d < t.ndim; ++d) {
        if (t.sizes[d] < 1 || t.strides[d] < 0 || t.access_const[d] < 0 || t.sizes[d] > ((int64_t)1 << 40) || t.strides[d] > ((int64_t)1 << 40)) {
          delete prog;
          return fail(STRIPE_ERR_INVALID_DESC, "bad temporary declaration");
        }
        extent += (t.access_const[d] + t.sizes[d] - 1) * t.strides[d];
      }
      if (extent > ((int64_t)1 << 40)) {
        delete prog;
        return fail(STRIPE_ERR_INVALID_DESC, "temporary too large");
      }
      prog->temp_bytes[r] = extent * 4;
    }
  }
  prog->n_inputs = n_inputs;
  int n_stmt = 0;
  for (const stripe_block_desc_t* st = root->child; st; st = st->next) {
    ++n_stmt;
    if (n_stmt > 8 || st->n_refs < 2 || st->n_refs > 3 || !st->parent_refs || !st->refs) {
      delete prog;
      return fail(STRIPE_ERR_INVALID_DESC, "a statement of a list has 2 or 3 refinements and names their root buffers in parent_refs");
    }
    stripe_refinement_t refs[3];
    Stage stage;
    stage.n_in = st->n_refs - 1;
    for (int i = 0; i < st->n_refs; ++i) {
      const int j = st->parent_refs[i];
      const bool is_out = i == st->n_refs - 1;
      if (j < 0 || j >= R || (is_out ? root->refs[j].dir == STRIPE_IN : !written[j]) || (is_out && st->next == nullptr) != (is_out && j == R - 1)) {
        delete prog;
        return fail(STRIPE_ERR_INVALID_DESC, "a statement reads a buffer nothing wrote yet, writes a caller's input, or the list does not end with the output");
      }
      refs[i] = root->refs[j];
      refs[i].dir = is_out ? STRIPE_OUT : STRIPE_IN;
      if (is_out) stage.dst = j; else stage.src[i] = j;
    }
    written[stage.dst] = 1;
    const bool updates_in_place = stage.dst == stage.src[0] || (stage.n_in > 1 && stage.dst == stage.src[1]);
    stripe_block_desc_t stmt = *st;
    stmt.next = nullptr;
    stmt.parent_refs = nullptr;
    stripe_block_desc_t sub = {};
    sub.n_refs = st->n_refs;
    sub.refs = refs;
    sub.child = &stmt;
    const stripe_status_t rc = create_single(&sub, path, &stage.blk);
    if (rc != STRIPE_OK) {
      delete prog;
      return rc;   // detail already recorded
    }
    if (updates_in_place) {
      // Definition 2 rule 2: an element one iteration writes may not be read by another.  A statement that reads the
      // buffer it writes is only legal as a per-element update: the read and write maps coincide, every index moves
      // the address, and the map is injective (make_plan proved that unless it chose the atomic form).
      const Plan& sp = stage.blk->plan;
      bool ok = !sp.noop && sp.info.n_red_idx == 0 && sp.gen.atomic == 0;
      for (int i = 0; i < stage.n_in && ok; ++i)
        if (stage.src[i] == stage.dst) {
          const Affine &rd = sp.flat.ref[i].addr, &wr = sp.flat.ref[sp.flat.n_refs - 1].addr;
          ok = rd.k == wr.k;
          for (int j = 0; j < sp.flat.n_idx && ok; ++j) ok = rd.c[j] == wr.c[j];
        }
      if (!ok && !sp.noop) {
        delete stage.blk;
        delete prog;
        return fail(STRIPE_ERR_INVALID_DESC, "a statement reads the buffer it writes through a different map (or with a reduction): an element written by "
                                             "one iteration would be read by another");
      }
    }
    prog->stages.push_back(stage);
  }
  // A temporary element that is read but never written has no defined value (the statements run as if in serial and
  // nothing initialises a temporary).  Refused where it can be shown: an upper bound on the elements a statement can
  // write into the temporary (the hull's distinct output elements, one fewer if some output tuple provably has no
  // point inside the polyhedron) against a lower bound on the elements a later constraint-free statement reads.
  for (size_t w = 0; w < prog->stages.size(); ++w) {
    const Stage& ws = prog->stages[w];
    if (root->refs[ws.dst].dir != STRIPE_TEMP) continue;
    const Plan& wp = ws.blk->plan;
    int64_t written_upper = wp.noop ? 0 : wp.info.output_elements;
    if (!wp.noop) {
      const FlatBlock& f = wp.flat;
      const Affine& oaddr = f.ref[f.n_refs - 1].addr;
      for (const Affine& q : f.cons) {
        // the most favourable value of the constraint over everything but the least favourable output tuple
        __int128 worst = q.k;
        for (int j = 0; j < f.n_idx; ++j) {
          const __int128 span = (__int128)q.c[j] * (f.range[j] - 1);
          if (oaddr.c[j]) worst += span < 0 ? span : 0;    // output index: pick the tuple that hurts
          else worst += span > 0 ? span : 0;               // reduction index: pick the point that helps
        }
        if (worst < 0) {
          --written_upper;
          break;
        }
      }
    }
    for (size_t r = w + 1; r < prog->stages.size(); ++r) {
      const Stage& rs = prog->stages[r];
      if (rs.dst == ws.dst) break;                         // rewritten before any further read
      for (int i = 0; i < rs.n_in; ++i) {
        if (rs.src[i] != ws.dst) continue;
        const Plan& rp = rs.blk->plan;
        if (rp.noop || !rp.flat.cons.empty()) continue;
        // distinct elements read: product of the ranges of the indexes that move the address, if that map is
        // injective (strides sorted by magnitude, each exceeding the span of the smaller ones)
        const FlatBlock& f = rp.flat;
        std::vector<std::pair<int64_t, int64_t>> terms;
        for (int j = 0; j < f.n_idx; ++j)
          if (f.ref[i].addr.c[j] && f.range[j] > 1) terms.push_back({f.ref[i].addr.c[j] < 0 ? -f.ref[i].addr.c[j] : f.ref[i].addr.c[j], f.range[j]});
        std::sort(terms.begin(), terms.end());
        __int128 span = 0, count = 1;
        bool injective = true;
        for (const auto& t : terms) {
          if ((__int128)t.first <= span) injective = false;
          span += (__int128)t.first * (t.second - 1);
          count *= t.second;
        }
        if (injective && count > (__int128)written_upper) {
          delete prog;
          return fail(STRIPE_ERR_INVALID_DESC, "a statement reads elements of a temporary that no earlier statement writes (at most " +
                                                   std::to_string((long long)written_upper) + " written, " + std::to_string((long long)count) + " read)");
        }
      }
    }
  }

  // Fusion and scalarisation (Section 2.3): a convolution into a temporary followed by O = relu(T + bias[k]) over
  // the same dense image runs as one kernel whose accumulators are the temporary, which then needs no memory.
  if (prog->stages.size() == 2 && tune_int("fuse", 1)) {
    const Stage &s0 = prog->stages[0], &s1 = prog->stages[1];
    const Plan& c = s0.blk->plan;
    const FlatBlock& e = s1.blk->plan.flat;
    bool ok = c.info.path == STRIPE_PATH_MFMA_CONV && c.in_dtype == STRIPE_BF16 && conv_can_fuse_bias_relu(c.conv, s0.blk->conv) &&
              root->refs[s0.dst].dir == STRIPE_TEMP && s1.n_in == 2 && s1.src[0] == s0.dst && !e.empty && e.intrinsic == STRIPE_INTR_ADD_RELU &&
              e.cons.empty() && e.n_refs == 3 && e.n_idx >= 2 && e.ref[0].dtype == STRIPE_F32 && e.ref[1].dtype == STRIPE_F32;
    if (ok) {
      // the second statement as its address maps see it: one merged pixel index and the channel index
      std::vector<int64_t> rng, ct, cbias, co;
      address_form(e, 2, &rng, &ct, &cbias, &co);
      const int64_t pixels = c.conv.N * c.conv.Ho * c.conv.Wo;
      ok = rng.size() == 2;
      if (ok) {
        const int k = (rng[0] == c.conv.Co && cbias[0] == 1) ? 0 : 1, px = 1 - k;
        ok = rng[k] == c.conv.Co && rng[px] == pixels && ct[k] == 1 && cbias[k] == 1 && co[k] == 1 && ct[px] == c.conv.Co && cbias[px] == 0 &&
             co[px] == c.conv.Co && e.ref[0].addr.k == 0 && e.ref[1].addr.k % 4 == 0 && e.ref[2].addr.k == 0;
      }
      if (ok) {
        prog->fused = e.out_bf16 ? 2 : 1;
        prog->plan.conv = c.conv;
        prog->conv = s0.blk->conv;
        prog->fuse_bias_off = e.ref[1].addr.k;      // element offset of the bias inside its buffer
        prog->temp_bytes[s0.dst] = 0;               // scalarised away
      }
    }
  }
  // The same for a dense contraction C = A * B (or A * B^T) followed by O[m,n] = relu(C[m,n] + bias[n]).
  if (!prog->fused && prog->stages.size() == 2 && tune_int("fuse", 1)) {
    const Stage &s0 = prog->stages[0], &s1 = prog->stages[1];
    const Plan& c = s0.blk->plan;
    const FlatBlock& e = s1.blk->plan.flat;
    bool ok = c.info.path == STRIPE_PATH_MFMA_GEMM && c.in_dtype == STRIPE_BF16 && gemm_can_fuse_bias_relu(c.gemm, s0.blk->gemm) &&
              root->refs[s0.dst].dir == STRIPE_TEMP && s1.n_in == 2 && s1.src[0] == s0.dst && !e.empty && e.intrinsic == STRIPE_INTR_ADD_RELU &&
              e.cons.empty() && e.n_refs == 3 && e.n_idx >= 2 && e.ref[0].dtype == STRIPE_F32 && e.ref[1].dtype == STRIPE_F32;
    if (ok) {
      std::vector<int64_t> rng, ct, cbias, co;
      address_form(e, 2, &rng, &ct, &cbias, &co);
      ok = rng.size() == 2;
      if (ok) {
        const int n = (rng[0] == c.gemm.N && cbias[0] == 1 && ct[0] == 1) ? 0 : 1, m = 1 - n;
        ok = rng[n] == c.gemm.N && rng[m] == c.gemm.M && ct[n] == 1 && cbias[n] == 1 && co[n] == 1 && ct[m] == c.gemm.c_m && cbias[m] == 0 &&
             co[m] >= c.gemm.N && e.ref[0].addr.k == c.gemm.c_base;
        if (ok) {
          prog->fused = e.out_bf16 ? 4 : 3;
          prog->plan.gemm = c.gemm;
          prog->gemm = s0.blk->gemm;
          prog->fuse_bias_off = e.ref[1].addr.k;
          prog->fuse_o_m = co[m];
          prog->fuse_o_base = e.ref[2].addr.k;
          prog->temp_bytes[s0.dst] = 0;
        }
      }
    }
  }
  // what the program as a whole looks like from outside
  stripe_block_info_t& info = prog->plan.info;
  info = prog->stages[0].blk->plan.info;
  info.hull_points = info.work_points = 0;
  info.algorithmic_bytes = 0;
  std::string names;
  for (const Stage& stg : prog->stages) {
    const stripe_block_info_t& si = stg.blk->plan.info;
    info.hull_points += si.hull_points;
    info.work_points = (info.work_points < 0 || si.work_points < 0) ? -1 : info.work_points + si.work_points;
    names += (names.empty() ? "" : " ; ") + std::string(si.kernel);
  }
  info.output_elements = prog->stages.back().blk->plan.info.output_elements;
  for (int r = 0; r < R; ++r)   // every caller-visible buffer once; temporaries are the library's business
    if (root->refs[r].dir != STRIPE_TEMP) {
      int64_t n = 1;
      for (int d = 0; d < root->refs[r].ndim; ++d) n *= root->refs[r].sizes[d];
      info.algorithmic_bytes += n * (root->refs[r].dtype == STRIPE_I8 ? 1 : root->refs[r].dtype == STRIPE_BF16 ? 2 : 4);
    }
  if (prog->fused) names = std::string(prog->stages[0].blk->plan.info.kernel) + (prog->fused == 2 ? "+bias_relu_bf16" : "+bias_relu");
  std::snprintf(info.kernel, sizeof info.kernel, "%s", names.c_str());
  // workspace layout: temporaries that were not scalarised away, then what each stage's own launches need
  prog->temp_off.assign(R, 0);
  prog->ws_bytes = 0;
  for (int r = 0; r < R; ++r)
    if (prog->temp_bytes[r]) {
      prog->temp_off[r] = prog->ws_bytes;
      prog->ws_bytes += round_up_256(prog->temp_bytes[r]);
    }
  prog->stage_ws_off.assign(prog->stages.size(), 0);
  if (!prog->fused)
    for (size_t i = 0; i < prog->stages.size(); ++i) {
      prog->stage_ws_off[i] = prog->ws_bytes;
      prog->ws_bytes += round_up_256(prog->stages[i].blk->ws_bytes);
    }
  info.workspace_bytes = prog->ws_bytes;
  *out = prog;
  return STRIPE_OK;
}

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
std::atomic<unsigned char*> g_scratch_ptr[kMaxDevices];

// Device address of the current GPU's copy of `scratch` (looked up on the first call on that GPU).
stripe_status_t static_scratch_of(int dev, unsigned char** out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(STRIPE_ERR_UNSUPPORTED, "device ordinal beyond the 64 this call keeps scratch pointers for");
  unsigned char* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!p) {
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
    if (!p) {
      void* sym = nullptr;
      const hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch));
      if (e != hipSuccess || !sym) return fail(STRIPE_ERR_HIP, std::string("hipGetSymbolAddress(scratch) failed: ") + hipGetErrorString(e));
      p = (unsigned char*)sym;
      g_scratch_ptr[dev].store(p, std::memory_order_release);
    }
  }
  *out = p;
  return STRIPE_OK;
}

// Where the handle's workspace lives for this run.  use_static: the GPU's static scratch array (no allocation
// ever); otherwise the caller's workspace if one was set, else memory the handle allocates on its first run on a
// device.  A handle that needs no workspace gets NULL.
stripe_status_t resolve_workspace(stripe_block* blk, bool use_static, unsigned char** ws) {
  *ws = nullptr;
  if (blk->ws_bytes == 0) return STRIPE_OK;
  if (use_static && blk->ws_bytes > (int64_t)STRIPE_STATIC_SCRATCH_BYTES)
    return fail(STRIPE_ERR_NOMEM, "the block's workspace needs " + std::to_string((long long)blk->ws_bytes) + " bytes, the static scratch holds " +
                                      std::to_string((long long)STRIPE_STATIC_SCRATCH_BYTES));
  if (!use_static && blk->caller_ws) {
    *ws = (unsigned char*)blk->caller_ws;
    return STRIPE_OK;
  }
  int dev = -1;
  const hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, hipGetErrorString(e));
  if (use_static) return static_scratch_of(dev, ws);
  if (dev != blk->owned_ws_dev) {   // first run (on this device)
    if (blk->owned_ws) (void)hipFree(blk->owned_ws);
    blk->owned_ws = nullptr;
    blk->owned_ws_dev = -1;
    if (hipMalloc(&blk->owned_ws, (size_t)blk->ws_bytes) != hipSuccess) {
      blk->owned_ws = nullptr;
      return fail(STRIPE_ERR_NOMEM, "out of device memory for the handle's workspace");
    }
    blk->owned_ws_dev = dev;
  }
  *ws = (unsigned char*)blk->owned_ws;
  return STRIPE_OK;
}

stripe_status_t run_single(stripe_block* blk, const void* const* inputs, void* output, void* hip_stream, unsigned char* ws);

stripe_status_t run_program(stripe_block* prog, const void* const* inputs, void* output, void* hip_stream, unsigned char* ws) {
  hipError_t e = hipSuccess;
  const int R = (int)prog->input_slot.size();
  if (prog->fused) {
    const Stage &s0 = prog->stages[0], &s1 = prog->stages[1];
    const float* bias = (const float*)inputs[prog->input_slot[s1.src[1]]] + prog->fuse_bias_off;
    const bool conv = prog->fused < 3, out_bf16 = prog->fused == 2 || prog->fused == 4;
    if (((uintptr_t)inputs[prog->input_slot[s0.src[0]]] % 16) || ((uintptr_t)inputs[prog->input_slot[s0.src[1]]] % 16) ||
        ((uintptr_t)bias % (conv ? 16 : 4)) || ((uintptr_t)output % (conv ? 16 : out_bf16 ? 2 : 4)))
      return fail(STRIPE_ERR_MISALIGNED, "the fused matrix-core kernel needs 16-byte aligned operands (convolution: also bias and output)");
    if (prog->fused >= 3)
      e = launch_gemm_bias_relu(prog->plan.gemm, prog->gemm, inputs[prog->input_slot[s0.src[0]]], inputs[prog->input_slot[s0.src[1]]], bias,
                                output, prog->fuse_o_m, prog->fuse_o_base, prog->fused == 4, (hipStream_t)hip_stream);
    else
    e = launch_conv_bias_relu(prog->plan.conv, prog->conv, inputs[prog->input_slot[s0.src[0]]], inputs[prog->input_slot[s0.src[1]]], bias,
                              output, prog->fused == 2, (hipStream_t)hip_stream);
    if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
    return STRIPE_OK;
  }
  auto where = [&](int r) -> const void* {
    if (r == R - 1) return output;
    if (prog->input_slot[r] >= 0) return inputs[prog->input_slot[r]];
    return ws + prog->temp_off[r];
  };
  for (size_t i = 0; i < prog->stages.size(); ++i) {
    const Stage& st = prog->stages[i];
    const void* ins[2] = {where(st.src[0]), st.n_in > 1 ? where(st.src[1]) : nullptr};
    const stripe_status_t rc = run_single(st.blk, ins, const_cast<void*>(where(st.dst)), hip_stream, ws ? ws + prog->stage_ws_off[i] : nullptr);
    if (rc != STRIPE_OK) return rc;
  }
  return STRIPE_OK;
}

stripe_status_t run_single(stripe_block* blk, const void* const* inputs, void* output, void* hip_stream, unsigned char* ws) {
  const Plan& p = blk->plan;
  if (p.noop) return STRIPE_OK;
  hipStream_t s = (hipStream_t)hip_stream;
  const void* in0 = inputs[0];
  const void* in1 = blk->n_inputs > 1 ? inputs[1] : nullptr;
  hipError_t e = hipSuccess;
  const bool out4 = p.info.path == STRIPE_PATH_MFMA_GEMM || (p.info.path == STRIPE_PATH_MFMA_CONV && blk->conv.variant >= kConvIgemmVariant);
  if (p.info.path != STRIPE_PATH_GENERIC && (((uintptr_t)in0 % 16) || (in1 && ((uintptr_t)in1 % 16)) || ((uintptr_t)output % (out4 ? 4 : 16))))
    return fail(STRIPE_ERR_MISALIGNED, "this handle was planned for a kernel family that moves 16 bytes per lane: input pointers (and, except for "
                                       "dense contractions and the general convolution kernel, the output pointer) must be 16-byte aligned");
  switch (p.info.path) {
    case STRIPE_PATH_MFMA_GEMM: e = launch_gemm(p.gemm, blk->gemm, in0, in1, output, ws, s); break;
    case STRIPE_PATH_MFMA_CONV: e = launch_conv(p.conv, blk->conv, in0, in1, output, s); break;
    case STRIPE_PATH_POOL: e = launch_pool(p.pool, blk->pool, in0, in1, output, s); break;
    default: e = launch_generic(p, in0, in1, output, s); break;
  }
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("kernel launch failed: ") + hipGetErrorString(e));
  return STRIPE_OK;
}

stripe_status_t run_any(stripe_block* blk, const void* const* inputs, void* output, void* hip_stream, bool use_static) {
  if (!blk || !inputs || !output) return fail(STRIPE_ERR_NULL, "blk, inputs or output is NULL");
  for (int i = 0; i < blk->n_inputs; ++i)
    if (!inputs[i]) return fail(STRIPE_ERR_NULL, "an input pointer is NULL");
  unsigned char* ws = nullptr;
  const stripe_status_t rc = resolve_workspace(blk, use_static, &ws);
  if (rc != STRIPE_OK) return rc;
  if (!blk->stages.empty()) return run_program(blk, inputs, output, hip_stream, ws);
  return run_single(blk, inputs, output, hip_stream, ws);
}

stripe_status_t create_single(const stripe_block_desc_t* desc, stripe_path_t path, stripe_block_t** out) {
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
  if (tune_int("generic_i64", 0) || !tune_int("generic_point4", 1)) p.gen.point4 = 0;
  if (tune_int("generic_i64", 0) || !tune_int("generic_tiled", 1)) p.tiled.use = 0;
  else if (tune_int("generic_tiled", 1) == 2 && p.tiled.n_items > 0) p.tiled.use = 1;   // test hook: tiled kernel also for small blocks
  if (!p.noop) {
    const bool forced = path != STRIPE_PATH_AUTO;
    bool picked = false;
    // a narrow product runs as a 1x1 convolution on the general convolution kernel, whose 256 x 64 tile it fills
    if (!forced && p.info.path == STRIPE_PATH_MFMA_GEMM) picked = conv_select_narrow_product(p.gemm, p.in_dtype, &p.conv, &blk->conv, &p.info);
    if (!picked) switch (p.info.path) {
      case STRIPE_PATH_MFMA_GEMM: picked = gemm_select(p.gemm, p.in_dtype, &blk->gemm, &p.info); break;
      case STRIPE_PATH_MFMA_CONV: picked = conv_select(p.conv, p.in_dtype, &blk->conv, &p.info); break;
      case STRIPE_PATH_POOL: picked = pool_select(p.pool, p.in_dtype, &blk->pool, &p.info); break;
      default: break;
    }
    // a block both matchers accept (a 1x1 convolution) whose shape the contraction kernels do not cover
    if (!picked && !forced && p.info.path == STRIPE_PATH_MFMA_GEMM && p.is_conv) {
      picked = conv_select(p.conv, p.in_dtype, &blk->conv, &p.info);
      if (!picked) p.info.path = STRIPE_PATH_MFMA_GEMM;
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
    if (p.info.path == STRIPE_PATH_MFMA_GEMM && picked) blk->ws_bytes = blk->gemm.ws_bytes;
  }
  p.info.workspace_bytes = blk->ws_bytes;
  *out = blk;
  return STRIPE_OK;
}

}  // namespace

extern "C" {

stripe_status_t stripe_block_create_for_path(const stripe_block_desc_t* desc, stripe_path_t path, stripe_block_t** out) {
  if (!desc || !out) return fail(STRIPE_ERR_NULL, "desc or out is NULL");
  *out = nullptr;
  if (path < STRIPE_PATH_AUTO || path > STRIPE_PATH_POOL) return fail(STRIPE_ERR_INVALID_DESC, "unknown path");
  if (desc->child && (desc->child->next || desc->child->parent_refs)) return create_program(desc, path, out);
  for (int r = 0; desc->refs && r < desc->n_refs; ++r)
    if (desc->refs[r].dir == STRIPE_TEMP) return fail(STRIPE_ERR_INVALID_DESC, "a temporary needs a statement list that writes and reads it");
  return create_single(desc, path, out);
}

stripe_status_t stripe_block_create(const stripe_block_desc_t* desc, stripe_block_t** out) {
  return stripe_block_create_for_path(desc, STRIPE_PATH_AUTO, out);
}

stripe_status_t stripe_block_run_static(stripe_block_t* blk, const void* const* inputs, void* output, void* hip_stream) {
  return run_any(blk, inputs, output, hip_stream, /*use_static=*/true);
}

stripe_status_t stripe_block_run(stripe_block_t* blk, const void* const* inputs, void* output, void* hip_stream) {
  return run_any(blk, inputs, output, hip_stream, /*use_static=*/false);
}

stripe_status_t stripe_block_workspace_size(const stripe_block_t* blk, size_t* bytes) {
  if (!blk || !bytes) return fail(STRIPE_ERR_NULL, "blk or bytes is NULL");
  *bytes = (size_t)blk->ws_bytes;
  return STRIPE_OK;
}

stripe_status_t stripe_block_set_workspace(stripe_block_t* blk, void* device_ptr, size_t bytes) {
  if (!blk) return fail(STRIPE_ERR_NULL, "blk is NULL");
  if (!device_ptr) {
    blk->caller_ws = nullptr;
    blk->caller_ws_bytes = 0;
    return STRIPE_OK;
  }
  if ((uintptr_t)device_ptr % 256) return fail(STRIPE_ERR_INVALID_DESC, "the workspace must be 256-byte aligned");
  if ((int64_t)bytes < blk->ws_bytes)
    return fail(STRIPE_ERR_NOMEM, "the workspace holds " + std::to_string(bytes) + " bytes, the handle needs " + std::to_string((long long)blk->ws_bytes));
  blk->caller_ws = device_ptr;
  blk->caller_ws_bytes = bytes;
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
    case STRIPE_ERR_MISALIGNED: return "buffer pointer not aligned for the planned kernel family";
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

stripe_status_t stripe_device_stream(const void* src, void* dst, size_t n_vectors, int reads, int write, int grid, void* hip_stream) {
  if (!dst || (reads > 0 && !src)) return fail(STRIPE_ERR_NULL, "src or dst is NULL");
  if ((reads != 0 && reads != 1 && reads != 2 && reads != 4) || (reads == 0 && !write) || (reads == 2 && !write) || grid < 1 || grid > (1 << 20))
    return fail(STRIPE_ERR_INVALID_DESC, "reads is 0, 1, 2 or 4 (0 and 2 only with write); grid is 1 .. 2^20 workgroups");
  if (((uintptr_t)src % 16) || ((uintptr_t)dst % 16)) return fail(STRIPE_ERR_MISALIGNED, "stream yardstick needs 16-byte aligned pointers");
  const hipError_t e = launch_stream(src, dst, n_vectors, reads, write, grid, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("stream launch failed: ") + hipGetErrorString(e));
  return STRIPE_OK;
}

stripe_status_t stripe_device_mfma(const void* operands, void* out, int iters, int from_lds, int grid, void* hip_stream) {
  if (!operands || !out) return fail(STRIPE_ERR_NULL, "operands or out is NULL");
  if (iters < 2 || (iters & 1) || iters > (1 << 24) || grid < 1 || grid > (1 << 20))
    return fail(STRIPE_ERR_INVALID_DESC, "iters is even, 2 .. 2^24; grid is 1 .. 2^20 workgroups");
  if (((uintptr_t)operands % 16) || ((uintptr_t)out % 4)) return fail(STRIPE_ERR_MISALIGNED, "matrix-core yardstick needs 16-byte aligned operands");
  const hipError_t e = launch_mfma_probe(operands, out, iters, grid, from_lds != 0, (hipStream_t)hip_stream);
  if (e != hipSuccess) return fail(STRIPE_ERR_HIP, std::string("matrix-core yardstick launch failed: ") + hipGetErrorString(e));
  return STRIPE_OK;
}

}  // extern "C"
