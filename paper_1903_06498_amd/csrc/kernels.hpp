// Launchers of the HIP kernel families (gfx950).  Each *_select() decides on
// the host whether the family covers the shape and fills the launch record
// and the query info; each launch_*() enqueues on the given stream.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdlib>
#include <cstring>

#include "plan.hpp"

namespace stripe {

// Tuning overrides for measurements: STRIPE_TUNE="key=value,key=value" is read
// when a handle is created; without it every family uses its default variant.
inline int tune_int(const char* key, int dflt) {
  const char* s = std::getenv("STRIPE_TUNE");
  if (!s) return dflt;
  const size_t n = std::strlen(key);
  for (const char* f = std::strstr(s, key); f; f = std::strstr(f + 1, key))
    if ((f == s || f[-1] == ',') && f[n] == '=') return std::atoi(f + n + 1);
  return dflt;
}

// ---- generic affine-index contraction (any legal block) -------------------
hipError_t launch_generic(const Plan& plan, const void* in0, const void* in1, void* out, hipStream_t stream);
void generic_info(const Plan& plan, stripe_block_info_t* info);
hipError_t launch_generic_tiled(const Plan& plan, const void* in0, const void* in1, void* out, hipStream_t stream);

// ---- nested-tile dense contraction on matrix cores ------------------------
struct GemmLaunch {
  int variant = -1;
  int t128_waves = 4;   // wavefronts of the 128 x 128-tile kernel: 4 or 8
  int t128_kb = 64;     // bytes of its K tile rows: 64, or 128 where one workgroup per CU covers the product
  int64_t grid = 0;
  int split_k = 1;       // slices of the reduction index, each run as one product of a batch into the workspace
  int64_t ws_bytes = 0;  // workspace launch_gemm needs: split_k images of M x N partial sums
  mutable int lds_enabled_on = -1;  // device on which the kernel's large LDS size has been enabled
};
bool gemm_select(const GemmShape& g, int in_dtype, GemmLaunch* l, stripe_block_info_t* info);
// workspace: device memory of l.ws_bytes (16-byte aligned), may be NULL when that is 0
hipError_t launch_gemm(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, void* c, void* workspace, hipStream_t stream);
// The product fused with a following statement O[m,n] = relu(C[m,n] + bias[n]) (C = the product's output, which then
// never reaches memory): O fp32 or bf16 with row stride o_m and element offset o_base.
bool gemm_can_fuse_bias_relu(const GemmShape& g, const GemmLaunch& l);
hipError_t launch_gemm_bias_relu(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, const void* bias, void* out,
                                 int64_t o_m, int64_t o_base, bool out_bf16, hipStream_t stream);

// ---- nested-tile convolution-shaped contraction on matrix cores -----------
constexpr int kConvIgemmVariant = 300;   // general convolution kernel; 300: 128 x 128 tiles, 301: 256 x 64, 302: 256 x 128
constexpr int kConvGemmVariant = 400;    // large convolutions on the 256 x 256-tile contraction kernel's convolution mode
struct ConvLaunch {
  int variant = -1;
  int64_t grid = 0;
  int in_dtype = 0;       // element type of the operands (general kernel: bf16 or int8)
  mutable int lds_enabled_on = -1;
};
bool conv_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info);
// a dense product with at most 64 columns and K-contiguous operands as a 1 x 1 convolution on the general kernel
bool conv_select_narrow_product(const GemmShape& g, int in_dtype, Conv2dShape* c, ConvLaunch* l, stripe_block_info_t* info);
hipError_t launch_conv(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t stream);
// The 3x3 bf16 kernel fused with a following statement O = relu(T + bias[k]) (T = the convolution's output):
// bias fp32 [64], out fp32 or bf16 in the convolution output's dense layout.
bool conv_can_fuse_bias_relu(const Conv2dShape& c, const ConvLaunch& l);
hipError_t launch_conv_bias_relu(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, const void* bias, void* out,
                                 bool out_bf16, hipStream_t stream);
// general convolution kernel (implicit contraction: any filter extent, stride, dilation, padding, image width;
// bf16 with Ci % 32 == 0 or int8 with Ci % 64 == 0; channels contiguous); conv_select falls back to it
bool conv_igemm_select(const Conv2dShape& c, int in_dtype, bool out_bf16, ConvLaunch* l, stripe_block_info_t* info);
// large bf16 convolutions (at least 128 tiles of 256 pixels x 256 channels, reduction a multiple of four 32-deep K tiles,
// dense output, every pixel written) on the contraction kernel: pixels as rows of A, gathered per filter tap
bool conv_gemm_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info);
hipError_t launch_conv_gemm(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, const void* bias, int epi,
                            hipStream_t st);
// bias != nullptr: the fused form of a following statement O = relu(T + bias[k]) (float blocks only)
hipError_t launch_conv_igemm(const Conv2dShape& c, const ConvLaunch& l, int in_dtype, bool out_bf16, const void* in, const void* flt, void* out,
                             const void* bias, hipStream_t stream);
// strided 7x7 int8 variant (dispatched to by conv_select / launch_conv)
bool conv_i8_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info);
hipError_t launch_conv_i8(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t stream);

// ---- aggregation over a 2-d window without a channel reduction: max / min / sum pooling, scaled sums
// (average pooling), depthwise convolution ------------------------------------
struct PoolLaunch {
  int variant = -1;
  int rows = 0;      // output rows per strip
  int yb = 1;        // strips a workgroup takes side by side, one per 128 lanes (strip kernel)
  int wg = 128;      // lanes per workgroup
  bool lean = false; // strip kernel without selects (32-bit in-row offsets suffice)
  int64_t grid = 0;
};
bool pool_select(const Pool2dShape& p, int dtype, PoolLaunch* l, stripe_block_info_t* info);
// weights: the second input of a weighted window (scale or depthwise weights), NULL for plain pooling
hipError_t launch_pool(const Pool2dShape& p, const PoolLaunch& l, const void* in, const void* weights, void* out, hipStream_t stream);

// ---- bandwidth yardstick ---------------------------------------------------
hipError_t launch_copy(const void* src, void* dst, size_t n_bytes, hipStream_t stream);
// `reads` input streams of n16 16-byte vectors each (0, 1, 2 or 4) folded into one output stream of n16 vectors (write != 0)
// or into nothing (write == 0: dst is a 4-byte flag that is practically never written)
// matrix-core yardstick (gemm.hip): iters (even) passes over a 4 x 4 fragment tile per wavefront, operands resident in
// registers or (lds) fetched again from LDS for every pass
hipError_t launch_mfma_probe(const void* operands, void* out, int iters, int grid, bool lds, hipStream_t stream);
hipError_t launch_stream(const void* src, void* dst, size_t n16, int reads, int write, int grid, hipStream_t stream);

}  // namespace stripe
