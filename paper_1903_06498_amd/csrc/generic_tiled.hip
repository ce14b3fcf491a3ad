// Register-tiled generic contraction (gfx950): sum-of-products blocks
//   O[..] += A[..] * B[..]
// with arbitrary affine accesses and constraints, for blocks too irregular
// for the matrix-core families but large enough to deserve operand reuse.
//
// Index roles follow from the three address maps (paper Section 3.2: every
// access is an affine function of the indexes).  One index pm that moves only
// A and the output, and one index pn that moves only B and the output, are
// blocked by 4: a lane owns the 4 x 4 output patch (pm0..pm0+3) x (pn0..pn0+3)
// for one value of every other output index, keeps its 16 partial sums in
// registers and, per reduction point, loads 4 A values and 4 B values for 16
// multiply-adds.  Lanes are numbered pn-block first, so stores and B loads of
// neighbouring lanes touch neighbouring addresses when pn has unit stride.
//
// Constraints (Section 3.2, "expr >= 0") may involve pm, the other output
// indexes and every reduction index except the innermost one, which the
// planner picks free of constraints: a patch row's validity is then fixed
// during the inner loop and is evaluated once per step of the outer reduction
// loops.  A point removed by a constraint contributes a zero first operand;
// a patch row no point reaches is not stored (Definition 2: only written
// elements receive a value).
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace stripe {
namespace {

template <typename T>
struct TElem;
template <>
struct TElem<int8_t> {
  using Acc = int32_t;
  static __device__ __forceinline__ Acc widen(int8_t v) { return (Acc)v; }
};
template <>
struct TElem<int32_t> {
  using Acc = int32_t;
  static __device__ __forceinline__ Acc widen(int32_t v) { return v; }
};
template <>
struct TElem<uint16_t> {   // bf16 bit pattern
  using Acc = float;
  static __device__ __forceinline__ Acc widen(uint16_t v) { return __uint_as_float((uint32_t)v << 16); }
};
template <>
struct TElem<float> {
  using Acc = float;
  static __device__ __forceinline__ Acc widen(float v) { return v; }
};

template <typename T, int VEC>
struct Pack {
  T v[VEC];
};

template <typename T, int VEC>
__device__ __forceinline__ Pack<T, VEC> load_pack(const T* p) {
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  Pack<T, VEC> r;
  if constexpr (VEC == 1) {
    r.v[0] = *p;
  } else {
    const vec_t x = *(const vec_t*)p;
#pragma unroll
    for (int i = 0; i < VEC; ++i) r.v[i] = x[i];
  }
  return r;
}

template <typename T, int VEC>
__global__ __launch_bounds__(256) void generic_tiled_kernel(const TiledParams p, const T* __restrict__ A, const T* __restrict__ B,
                                                            typename TElem<T>::Acc* __restrict__ O) {
  using Acc = typename TElem<T>::Acc;
  int64_t item = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (item >= p.n_items) return;
  uint32_t t = (uint32_t)item;
  const int nb = t % (uint32_t)p.pn_blocks; t /= (uint32_t)p.pn_blocks;
  const int mb = t % (uint32_t)p.pm_blocks; t /= (uint32_t)p.pm_blocks;
  const int m0 = mb * 4, n0 = nb * 4;
  int offA = p.a_base + p.a_pm * m0, offB = p.b_base + p.b_pn * n0, offO = p.o_base + p.o_pm * m0 + p.o_pn * n0;
  int cv[kGenCons];
#pragma unroll
  for (int q = 0; q < kGenCons; ++q) cv[q] = p.cons_const[q] + p.cons_pm[q] * m0;
  for (int j = 0; j < p.n_outer; ++j) {
    const uint32_t rng = (uint32_t)p.outer_range[j];
    const int v = (int)(t % rng);
    t /= rng;
    offA += p.a_outer[j] * v;
    offB += p.b_outer[j] * v;
    offO += p.o_outer[j] * v;
#pragma unroll
    for (int q = 0; q < kGenCons; ++q) cv[q] += p.cons_outer[q][j] * v;
  }
  bool mvalid[4];
  int nstep[4];   // B offset of patch column u; columns past the range re-read the last valid one (never stored)
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    mvalid[u] = m0 + u < p.pm_range;
    nstep[u] = p.b_pn * ((n0 + u < p.pn_range ? n0 + u : p.pn_range - 1) - n0);
  }

  Acc acc[4][4];
  bool touched[4] = {false, false, false, false};
#pragma unroll
  for (int a = 0; a < 4; ++a)
#pragma unroll
    for (int b = 0; b < 4; ++b) acc[a][b] = 0;

  for (int r3 = 0; r3 < p.red_range[3]; ++r3)
    for (int r2 = 0; r2 < p.red_range[2]; ++r2)
      for (int r1 = 0; r1 < p.red_range[1]; ++r1) {
        bool valid[4] = {mvalid[0], mvalid[1], mvalid[2], mvalid[3]};
#pragma unroll
        for (int q = 0; q < kGenCons; ++q) {
          if (q < p.n_cons) {
            const int base = cv[q] + p.cons_red[q][3] * r3 + p.cons_red[q][2] * r2 + p.cons_red[q][1] * r1;
#pragma unroll
            for (int a = 0; a < 4; ++a) valid[a] = valid[a] && (base + p.cons_pm[q] * a >= 0);
          }
        }
        if (!(valid[0] || valid[1] || valid[2] || valid[3])) continue;
        const int safe = valid[0] ? 0 : valid[1] ? 1 : valid[2] ? 2 : 3;   // a row whose addresses are in bounds
        const int ra = offA + p.a_red[3] * r3 + p.a_red[2] * r2 + p.a_red[1] * r1;
        const int rb = offB + p.b_red[3] * r3 + p.b_red[2] * r2 + p.b_red[1] * r1;
        const T* pa[4];
        const T* pb[4];
#pragma unroll
        for (int a = 0; a < 4; ++a) pa[a] = A + ra + p.a_pm * (valid[a] ? a : safe);
#pragma unroll
        for (int b = 0; b < 4; ++b) pb[b] = B + rb + nstep[b];
        const int sa = p.a_red[0], sb = p.b_red[0];
        for (int r0 = 0; r0 < p.red_range[0]; r0 += VEC) {
          Pack<T, VEC> av[4], bv[4];
#pragma unroll
          for (int a = 0; a < 4; ++a) av[a] = load_pack<T, VEC>(pa[a] + sa * r0);
#pragma unroll
          for (int b = 0; b < 4; ++b) bv[b] = load_pack<T, VEC>(pb[b] + sb * r0);
#pragma unroll
          for (int e = 0; e < VEC; ++e) {
            Acc bw[4];
#pragma unroll
            for (int b = 0; b < 4; ++b) bw[b] = TElem<T>::widen(bv[b].v[e]);
#pragma unroll
            for (int a = 0; a < 4; ++a) {
              const Acc aw = valid[a] ? TElem<T>::widen(av[a].v[e]) : (Acc)0;
#pragma unroll
              for (int b = 0; b < 4; ++b) acc[a][b] += aw * bw[b];
            }
          }
        }
#pragma unroll
        for (int a = 0; a < 4; ++a) touched[a] = touched[a] || valid[a];
      }

#pragma unroll
  for (int a = 0; a < 4; ++a) {
    if (!touched[a]) continue;
#pragma unroll
    for (int b = 0; b < 4; ++b)
      if (n0 + b < p.pn_range) O[offO + p.o_pm * a + p.o_pn * b] = acc[a][b];
  }
}

template <typename T>
hipError_t launch_t(const TiledParams& p, int vec, const void* a, const void* b, void* o, hipStream_t s) {
  using Acc = typename TElem<T>::Acc;
  const int64_t grid = (p.n_items + 255) / 256;
  if (vec == 4)
    hipLaunchKernelGGL((generic_tiled_kernel<T, 4>), dim3((unsigned)grid), dim3(256), 0, s, p, (const T*)a, (const T*)b, (Acc*)o);
  else
    hipLaunchKernelGGL((generic_tiled_kernel<T, 1>), dim3((unsigned)grid), dim3(256), 0, s, p, (const T*)a, (const T*)b, (Acc*)o);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_generic_tiled(const Plan& plan, const void* in0, const void* in1, void* out, hipStream_t stream) {
  const TiledParams& p = plan.tiled;
  if (!p.use || p.n_items <= 0 || (p.n_items + 255) / 256 > 0x7fffffffLL) return hipErrorInvalidValue;
  // packed loads need the buffers themselves aligned to four elements; otherwise fall back to single elements
  const size_t elem = plan.in_dtype == STRIPE_I8 ? 1 : plan.in_dtype == STRIPE_BF16 ? 2 : 4;
  int vec = p.vec;
  if (vec == 4 && (((uintptr_t)in0 % (4 * elem)) || ((uintptr_t)in1 % (4 * elem)))) vec = 1;
  switch (plan.in_dtype) {
    case STRIPE_I8: return launch_t<int8_t>(p, vec, in0, in1, out, stream);
    case STRIPE_I32: return launch_t<int32_t>(p, vec, in0, in1, out, stream);
    case STRIPE_BF16: return launch_t<uint16_t>(p, vec, in0, in1, out, stream);
    default: return launch_t<float>(p, vec, in0, in1, out, stream);
  }
}

}  // namespace stripe
