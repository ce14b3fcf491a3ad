// Generic affine-index contraction kernel (gfx950): evaluates any legal flat
// Stripe block.  Output indexes are spread over the grid, reduction indexes
// are walked inside the kernel; every constraint is an integer affine test
// per point (paper Section 3.2: ranges plus affine constraints); values that
// land on one output element are combined with the aggregation operation
// (Definition 2, rule 3) and elements no point writes are left alone.
//
// Two lane mappings:
//   lanes == 1 : one lane per output element.  The fastest grid index is the
//                output index with the smallest output stride, so stores -- and
//                loads of inputs that follow that index -- coalesce.
//   lanes == 64: one wavefront per output element; the 64 lanes stride through
//                the flattened reduction space (innermost reduction index =
//                smallest input stride, so a wavefront reads consecutive
//                elements) and a cross-lane butterfly finishes the aggregation.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "kernels.hpp"

namespace stripe {
namespace {

template <typename T>
struct Elem;
template <>
struct Elem<int8_t> {
  using Acc = int32_t;
  static __device__ __forceinline__ int32_t load(const void* p, int64_t i) { return (int32_t)((const int8_t*)p)[i]; }
};
template <>
struct Elem<int32_t> {
  using Acc = int32_t;
  static __device__ __forceinline__ int32_t load(const void* p, int64_t i) { return ((const int32_t*)p)[i]; }
};
template <>
struct Elem<uint16_t> {  // bf16 bit pattern: the upper half of an fp32
  using Acc = float;
  static __device__ __forceinline__ float load(const void* p, int64_t i) {
    return __uint_as_float(((uint32_t)((const uint16_t*)p)[i]) << 16);
  }
};
template <>
struct Elem<float> {
  using Acc = float;
  static __device__ __forceinline__ float load(const void* p, int64_t i) { return ((const float*)p)[i]; }
};

// Identity of the aggregation: what an output element holds before the atomic combine pass.
template <int AGG>
__device__ __forceinline__ int32_t identity_of(int32_t) {
  return AGG == STRIPE_AGG_MAX ? (int32_t)0x80000000 : AGG == STRIPE_AGG_MIN ? 0x7fffffff : AGG == STRIPE_AGG_MUL ? 1 : 0;
}
template <int AGG>
__device__ __forceinline__ float identity_of(float) {
  return AGG == STRIPE_AGG_MAX ? -__builtin_huge_valf() : AGG == STRIPE_AGG_MIN ? __builtin_huge_valf() : AGG == STRIPE_AGG_MUL ? 1.f : 0.f;
}

// Atomic aggregation onto one output element.  Integer operations are exact in any order; float sums
// depend on the order (the paper leaves the order of a floating-point aggregation open, Section 3.2);
// float max/min are exact and use a compare-and-swap loop.
template <int AGG>
__device__ __forceinline__ void atomic_combine(int32_t* p, int32_t v) {
  if (AGG == STRIPE_AGG_MUL) {
    int32_t seen = __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
      const int32_t prev = atomicCAS(p, seen, (int32_t)((uint32_t)seen * (uint32_t)v));
      if (prev == seen) break;
      seen = prev;
    }
  } else if (AGG == STRIPE_AGG_MAX) atomicMax(p, v);
  else if (AGG == STRIPE_AGG_MIN) atomicMin(p, v);
  else atomicAdd(p, v);
}
template <int AGG>
__device__ __forceinline__ void atomic_combine(float* p, float v) {
  if (AGG == STRIPE_AGG_MAX || AGG == STRIPE_AGG_MIN) {
    unsigned* u = (unsigned*)p;
    unsigned seen = __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    while (AGG == STRIPE_AGG_MAX ? v > __uint_as_float(seen) : v < __uint_as_float(seen)) {
      const unsigned prev = atomicCAS(u, seen, __float_as_uint(v));
      if (prev == seen) break;
      seen = prev;
    }
  } else if (AGG == STRIPE_AGG_MUL) {
    unsigned* u = (unsigned*)p;
    unsigned seen = __hip_atomic_load(u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    for (;;) {
      const unsigned prev = atomicCAS(u, seen, __float_as_uint(__uint_as_float(seen) * v));
      if (prev == seen) break;
      seen = prev;
    }
  } else {
    atomicAdd(p, v);
  }
}

template <int AGG, typename A>
__device__ __forceinline__ A combine(A acc, A v) {
  if (AGG == STRIPE_AGG_MAX) return v > acc ? v : acc;
  if (AGG == STRIPE_AGG_MIN) return v < acc ? v : acc;
  if (AGG == STRIPE_AGG_MUL) {
    if constexpr (std::is_same<A, int32_t>::value) return (A)((uint32_t)acc * (uint32_t)v);   // wraps, like the atomic form
    else return acc * v;
  }
  return acc + v;
}

// Bits of `m` moved to the position of their butterfly partner at distance d (d a power of two).
__device__ __forceinline__ uint64_t swap_blocks(uint64_t m, int d) {
  const uint64_t low = d == 32 ? 0x00000000ffffffffull : d == 16 ? 0x0000ffff0000ffffull : d == 8 ? 0x00ff00ff00ff00ffull
                     : d == 4 ? 0x0f0f0f0f0f0f0f0full : d == 2 ? 0x3333333333333333ull : 0x5555555555555555ull;
  return ((m & low) << d) | ((m >> d) & low);
}

// pass: 0 = the output map is injective on the output indexes, every lane (or wavefront) owns its element and
// stores it; 1 and 2 = two launches for maps where several output-index tuples share an element: pass 1
// writes the aggregation's identity to every element some point reaches (all writers write the same value),
// pass 2 combines each tuple's partial result onto it atomically.  Elements no point reaches stay untouched.
//
// NARROW: the planner has shown that every element offset, every constraint
// value and the output count fit in 32 bits, so all index arithmetic (and the
// divisions that decode a flat position into indexes) runs in 32-bit.
template <typename TIn, int INTR, int AGG, int LANES, bool NARROW>
__global__ __launch_bounds__(256) void generic_kernel(const GenericParams p, const void* __restrict__ in0,
                                                      const void* __restrict__ in1, void* __restrict__ out, const int pass) {
  using Acc = typename Elem<TIn>::Acc;
  using I = typename std::conditional<NARROW, int32_t, int64_t>::type;    // offsets and constraint values
  using U = typename std::conditional<NARROW, uint32_t, uint64_t>::type;  // flat output position
  const int lane = threadIdx.x & 63;
  U t;
  if (LANES == 1) {
    t = (U)blockIdx.x * 256 + threadIdx.x;
  } else {
    t = (U)blockIdx.x * 4 + (U)__builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));   // uniform per wavefront
  }
  if ((int64_t)t >= p.n_outputs) return;

  I offA = (I)p.a_base, offB = (I)p.b_base, offO = (I)p.o_base;
  I cv[kGenCons];
#pragma unroll
  for (int q = 0; q < kGenCons; ++q) cv[q] = (I)p.cons_const[q];
  for (int j = 0; j < p.n_out; ++j) {
    const U rng = (U)p.out_range[j];
    const U quot = t / rng;
    const I o = (I)(t - quot * rng);
    t = quot;
    offA += (I)p.a_out[j] * o;
    offB += (I)p.b_out[j] * o;
    offO += (I)p.o_out[j] * o;
#pragma unroll
    for (int q = 0; q < kGenCons; ++q) cv[q] += (I)p.cons_out[q][j] * o;
  }

  Acc acc = 0;
  bool touched = false;

  auto visit = [&](I oa, I ob) {
    if (pass == 1) {        // identity pass: only whether the tuple has a point matters
      touched = true;
      return;
    }
    const Acc a = Elem<TIn>::load(in0, oa);
    Acc v = a;
    if (INTR != STRIPE_INTR_COPY) {
      const Acc b = Elem<TIn>::load(in1, ob);
      v = (INTR == STRIPE_INTR_MUL) ? a * b : a + b;
      if (INTR == STRIPE_INTR_ADD_RELU) v = v > (Acc)0 ? v : (Acc)0;
    }
    acc = touched ? combine<AGG, Acc>(acc, v) : v;
    touched = true;
  };

  auto finish = [&](I off) {
    if (std::is_same<Acc, float>::value && p.out_bf16) {   // bf16 output buffer: round to nearest even (never atomic)
      const uint32_t u = __float_as_uint((float)acc);
      ((uint16_t*)out)[off] = (u & 0x7fffffffu) > 0x7f800000u ? (uint16_t)((u >> 16) | 0x40u)       // NaN stays NaN
                                                              : (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
      return;
    }
    Acc* dst = (Acc*)out + off;
    if (pass == 0) *dst = acc;
    else if (pass == 1) *dst = identity_of<AGG>(Acc());
    else atomic_combine<AGG>(dst, acc);
  };

  if (LANES == 1) {
    const uint32_t inner = p.inner_range;
    const uint32_t outer_total = p.red_total / inner;
    for (uint32_t ro = 0; ro < outer_total; ++ro) {
      I oa = offA, ob = offB;
      I cw[kGenCons];
#pragma unroll
      for (int q = 0; q < kGenCons; ++q) cw[q] = cv[q];
      uint32_t rest = ro;
      for (int j = 1; j < p.n_red; ++j) {
        const uint32_t rng = (uint32_t)p.red_range[j];
        const uint32_t quot = rest / rng;
        const I rj = (I)(rest - quot * rng);
        rest = quot;
        oa += (I)p.a_red[j] * rj;
        ob += (I)p.b_red[j] * rj;
#pragma unroll
        for (int q = 0; q < kGenCons; ++q) cw[q] += (I)p.cons_red[q][j] * rj;
      }
      const I sa = (I)p.a_red[0], sb = (I)p.b_red[0];
      for (uint32_t r0 = 0; r0 < inner; ++r0) {
        bool ok = true;
#pragma unroll
        for (int q = 0; q < kGenCons; ++q) {
          ok = ok && (cw[q] >= 0);
          cw[q] += (I)p.cons_red[q][0];
        }
        if (ok) visit(oa, ob);
        oa += sa;
        ob += sb;
      }
    }
    if (touched) finish(offO);
  } else {
    for (uint32_t r = lane; r < p.red_total; r += 64) {
      I oa = offA, ob = offB;
      I cw[kGenCons];
#pragma unroll
      for (int q = 0; q < kGenCons; ++q) cw[q] = cv[q];
      uint32_t rest = r;
      for (int j = 0; j < p.n_red; ++j) {
        const uint32_t rng = (uint32_t)p.red_range[j];
        const uint32_t quot = rest / rng;
        const I rj = (I)(rest - quot * rng);
        rest = quot;
        oa += (I)p.a_red[j] * rj;
        ob += (I)p.b_red[j] * rj;
#pragma unroll
        for (int q = 0; q < kGenCons; ++q) cw[q] += (I)p.cons_red[q][j] * rj;
      }
      bool ok = true;
#pragma unroll
      for (int q = 0; q < kGenCons; ++q) ok = ok && (cw[q] >= 0);
      if (ok) visit(oa, ob);
    }
    // Butterfly over the 64 lanes.  Which lanes hold a value is tracked in a
    // wave-uniform mask, so only the values cross lanes; a lane whose partner
    // saw no point takes nothing from it.
    uint64_t mask = __ballot(touched);
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) {
      const Acc other = __shfl_xor(acc, m, 64);
      const uint64_t partner = swap_blocks(mask, m);
      if ((partner >> lane) & 1) {
        acc = touched ? combine<AGG, Acc>(acc, other) : other;
        touched = true;
      }
      mask |= partner;
    }
    if (lane == 0 && touched) finish(offO);
  }
}

// Pointwise blocks: no reduction, no constraints, every lane computes four consecutive outputs along the fastest
// output index (vector loads where an input follows that index, a broadcast where it does not; one vector store).
template <typename TIn, int INTR>
__global__ __launch_bounds__(256) void generic_point4_kernel(const GenericParams p, const void* __restrict__ in0,
                                                             const void* __restrict__ in1, void* __restrict__ out) {
  using Acc = typename Elem<TIn>::Acc;
  typedef TIn in4 __attribute__((ext_vector_type(4)));
  typedef Acc acc4 __attribute__((ext_vector_type(4)));
  uint32_t t = blockIdx.x * 256u + threadIdx.x;
  if ((int64_t)t >= p.n_outputs / 4) return;
  const uint32_t q0 = (uint32_t)p.out_range[0] / 4u;
  const int o0 = (int)(t % q0) * 4;
  t /= q0;
  int offA = (int)p.a_base + (int)p.a_out[0] * o0, offB = (int)p.b_base + (int)p.b_out[0] * o0, offO = (int)p.o_base + o0;
  for (int j = 1; j < p.n_out; ++j) {
    const uint32_t rng = (uint32_t)p.out_range[j];
    const int o = (int)(t % rng);
    t /= rng;
    offA += (int)p.a_out[j] * o;
    offB += (int)p.b_out[j] * o;
    offO += (int)p.o_out[j] * o;
  }
  auto fetch = [](const void* base, int off, bool follows) {
    in4 r;
    if (follows) {
      r = *(const in4*)((const TIn*)base + off);
    } else {
      const TIn s = ((const TIn*)base)[off];
      r = (in4){s, s, s, s};
    }
    return r;
  };
  auto widen = [](TIn x) -> Acc {
    if constexpr (std::is_same<TIn, uint16_t>::value) return __uint_as_float((uint32_t)x << 16);
    else return (Acc)x;
  };
  const in4 a = fetch(in0, offA, p.a_out[0] == 1);
  in4 b = a;
  if (INTR != STRIPE_INTR_COPY) b = fetch(in1, offB, p.b_out[0] == 1);
  acc4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const Acc x = widen(a[e]), y = widen(b[e]);
    Acc r = INTR == STRIPE_INTR_COPY ? x : INTR == STRIPE_INTR_MUL ? x * y : x + y;
    if (INTR == STRIPE_INTR_ADD_RELU) r = r > (Acc)0 ? r : (Acc)0;
    v[e] = r;
  }
  if (std::is_same<Acc, float>::value && p.out_bf16) {
    typedef __bf16 bf4 __attribute__((ext_vector_type(4)));
    typedef float f4 __attribute__((ext_vector_type(4)));
    *(bf4*)((uint16_t*)out + offO) = __builtin_convertvector((f4){(float)v[0], (float)v[1], (float)v[2], (float)v[3]}, bf4);   // round to nearest even
  } else {
    *(acc4*)((Acc*)out + offO) = v;
  }
}

template <typename TIn, int INTR>
hipError_t launch_point4(const GenericParams& p, const void* a, const void* b, void* o, hipStream_t s) {
  const int64_t grid = (p.n_outputs / 4 + 255) / 256;
  hipLaunchKernelGGL((generic_point4_kernel<TIn, INTR>), dim3((unsigned)grid), dim3(256), 0, s, p, a, b, o);
  return hipGetLastError();
}

template <typename TIn, int INTR, int AGG>
hipError_t launch_lanes(const GenericParams& p, const void* a, const void* b, void* o, hipStream_t s) {
  const int64_t grid = p.lanes == 64 ? (p.n_outputs + 3) / 4 : (p.n_outputs + 255) / 256;
  void (*kernel)(const GenericParams, const void*, const void*, void*, const int) =
      p.lanes == 64 ? (p.narrow ? generic_kernel<TIn, INTR, AGG, 64, true> : generic_kernel<TIn, INTR, AGG, 64, false>)
                    : (p.narrow ? generic_kernel<TIn, INTR, AGG, 1, true> : generic_kernel<TIn, INTR, AGG, 1, false>);
  if (p.atomic) {
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, s, p, a, b, o, 1);
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, s, p, a, b, o, 2);
  } else {
    hipLaunchKernelGGL(kernel, dim3((unsigned)grid), dim3(256), 0, s, p, a, b, o, 0);
  }
  return hipGetLastError();
}

template <typename TIn, int INTR>
hipError_t launch_agg(int agg, const GenericParams& p, const void* a, const void* b, void* o, hipStream_t s) {
  switch (agg) {
    case STRIPE_AGG_MAX: return launch_lanes<TIn, INTR, STRIPE_AGG_MAX>(p, a, b, o, s);
    case STRIPE_AGG_MIN: return launch_lanes<TIn, INTR, STRIPE_AGG_MIN>(p, a, b, o, s);
    case STRIPE_AGG_MUL: return launch_lanes<TIn, INTR, STRIPE_AGG_MUL>(p, a, b, o, s);
    default: return launch_lanes<TIn, INTR, STRIPE_AGG_ADD>(p, a, b, o, s);  // assign: single writer, any op
  }
}

template <typename TIn>
hipError_t launch_intr(int intr, int agg, const GenericParams& p, const void* a, const void* b, void* o, hipStream_t s) {
  // the four-outputs-per-lane form needs the buffers themselves 16-byte aligned
  if (p.point4 && !((uintptr_t)a % 16) && !((uintptr_t)o % 16) && (intr == STRIPE_INTR_COPY || !((uintptr_t)b % 16))) {
    switch (intr) {
      case STRIPE_INTR_COPY: return launch_point4<TIn, STRIPE_INTR_COPY>(p, a, b, o, s);
      case STRIPE_INTR_ADD: return launch_point4<TIn, STRIPE_INTR_ADD>(p, a, b, o, s);
      case STRIPE_INTR_ADD_RELU: return launch_point4<TIn, STRIPE_INTR_ADD_RELU>(p, a, b, o, s);
      default: return launch_point4<TIn, STRIPE_INTR_MUL>(p, a, b, o, s);
    }
  }
  switch (intr) {
    case STRIPE_INTR_COPY: return launch_agg<TIn, STRIPE_INTR_COPY>(agg, p, a, b, o, s);
    case STRIPE_INTR_ADD: return launch_agg<TIn, STRIPE_INTR_ADD>(agg, p, a, b, o, s);
    case STRIPE_INTR_ADD_RELU: return launch_agg<TIn, STRIPE_INTR_ADD_RELU>(agg, p, a, b, o, s);
    default: return launch_agg<TIn, STRIPE_INTR_MUL>(agg, p, a, b, o, s);
  }
}

}  // namespace

hipError_t launch_generic(const Plan& plan, const void* in0, const void* in1, void* out, hipStream_t stream) {
  if (plan.tiled.use) return launch_generic_tiled(plan, in0, in1, out, stream);
  const GenericParams& p = plan.gen;
  if (p.n_outputs <= 0) return hipErrorInvalidValue;
  const int64_t blocks = p.lanes == 64 ? (p.n_outputs + 3) / 4 : (p.n_outputs + 255) / 256;
  if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
  const int intr = plan.flat.intrinsic, agg = plan.flat.agg;
  switch (plan.in_dtype) {
    case STRIPE_I8: return launch_intr<int8_t>(intr, agg, p, in0, in1, out, stream);
    case STRIPE_I32: return launch_intr<int32_t>(intr, agg, p, in0, in1, out, stream);
    case STRIPE_BF16: return launch_intr<uint16_t>(intr, agg, p, in0, in1, out, stream);
    default: return launch_intr<float>(intr, agg, p, in0, in1, out, stream);
  }
}

void generic_info(const Plan& plan, stripe_block_info_t* info) {
  const GenericParams& p = plan.gen;
  info->path = STRIPE_PATH_GENERIC;
  if (plan.tiled.use) {
    info->tile_m = 4; info->tile_n = 4; info->tile_k = plan.tiled.vec;
    info->frag_m = info->frag_n = info->frag_k = 0;
    info->lds_bytes = 0;
    info->workgroup_size = 256;
    info->grid = (plan.tiled.n_items + 255) / 256;
    snprintf(info->kernel, sizeof info->kernel, "generic_tiled_4x4%s", plan.tiled.vec == 4 ? "_v4" : "");
    return;
  }
  info->tile_m = info->tile_n = info->tile_k = 0;
  info->frag_m = info->frag_n = info->frag_k = 0;
  info->lds_bytes = 0;
  info->workgroup_size = 256;
  info->grid = p.lanes == 64 ? (p.n_outputs + 3) / 4 : (p.n_outputs + 255) / 256;
  if (p.point4) {
    info->grid = (p.n_outputs / 4 + 255) / 256;
    snprintf(info->kernel, sizeof info->kernel, "generic_pointwise_x4");
    return;
  }
  snprintf(info->kernel, sizeof info->kernel, "generic_affine_%s%s%s", p.lanes == 64 ? "wave_per_output" : "lane_per_output",
           p.narrow ? "" : "_i64", p.atomic ? "_atomic" : "");
}

// ---------------------------------------------------------------------------
// Bandwidth yardstick: plain 16-byte-per-lane grid-stride copy.
// ---------------------------------------------------------------------------
namespace {
__global__ __launch_bounds__(256) void copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) dst[i] = src[i];
}
}  // namespace

// ---------------------------------------------------------------------------
// Streaming yardsticks: R input streams folded into one output stream (R = 0: write only; write = 0: read only),
// 16 bytes per lane, four independent vectors per lane and trip so that 4 * R loads are in flight per lane,
// streaming (non-temporal) loads and stores, grid chosen by the caller.  They state what a perfectly regular
// kernel with a given read : write mix reaches on this chip, next to the window kernels.
// ---------------------------------------------------------------------------
namespace {
typedef float y_f32x4 __attribute__((ext_vector_type(4)));
template <int R, bool WRITE>
__global__ __launch_bounds__(256) void stream_kernel(const y_f32x4* __restrict__ src, y_f32x4* __restrict__ dst, size_t n16, float* __restrict__ flag) {
  constexpr int U = 4;
  const size_t step = (size_t)gridDim.x * 256;
  y_f32x4 keep = {0.f, 0.f, 0.f, 0.f};
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += step * U) {
    y_f32x4 v[U][R > 0 ? R : 1];
#pragma unroll
    for (int u = 0; u < U; ++u)
#pragma unroll
      for (int r = 0; r < R; ++r) {
        const size_t at = i + u * step;
        v[u][r] = at < n16 ? __builtin_nontemporal_load(src + (size_t)r * n16 + at) : keep;
      }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      y_f32x4 sum = {1.f, 2.f, 3.f, 4.f};
#pragma unroll
      for (int r = 0; r < R; ++r) sum = r ? sum + v[u][r] : v[u][0];
      const size_t at = i + u * step;
      if (WRITE) {
        if (at < n16) __builtin_nontemporal_store(sum, dst + at);
      } else {
        keep += sum;
      }
    }
  }
  if (!WRITE && keep.x + keep.y + keep.z + keep.w == 12345.678f) flag[0] = 1.f;   // keeps the loads alive; practically never true
}
}  // namespace

hipError_t launch_stream(const void* src, void* dst, size_t n16, int reads, int write, int grid, hipStream_t stream) {
  if (n16 == 0) return hipSuccess;
  const dim3 g((unsigned)grid), b(256);
  const y_f32x4* s = (const y_f32x4*)src;
  y_f32x4* d = (y_f32x4*)dst;
  if (reads == 0 && write) hipLaunchKernelGGL((stream_kernel<0, true>), g, b, 0, stream, s, d, n16, (float*)dst);
  else if (reads == 1 && write) hipLaunchKernelGGL((stream_kernel<1, true>), g, b, 0, stream, s, d, n16, (float*)dst);
  else if (reads == 2 && write) hipLaunchKernelGGL((stream_kernel<2, true>), g, b, 0, stream, s, d, n16, (float*)dst);
  else if (reads == 4 && write) hipLaunchKernelGGL((stream_kernel<4, true>), g, b, 0, stream, s, d, n16, (float*)dst);
  else if (reads == 1 && !write) hipLaunchKernelGGL((stream_kernel<1, false>), g, b, 0, stream, s, d, n16, (float*)dst);
  else if (reads == 4 && !write) hipLaunchKernelGGL((stream_kernel<4, false>), g, b, 0, stream, s, d, n16, (float*)dst);
  else return hipErrorInvalidValue;
  return hipGetLastError();
}

hipError_t launch_copy(const void* src, void* dst, size_t n_bytes, hipStream_t stream) {
  const size_t n16 = n_bytes / 16;
  if (n16 == 0) return hipSuccess;
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 256 * 32) blocks = 256 * 32;
  hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, stream, (const uint4*)src, (uint4*)dst, n16);
  return hipGetLastError();
}

}  // namespace stripe
