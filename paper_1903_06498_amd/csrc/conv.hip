// Nested-tile convolution-shaped contraction on the gfx950 matrix cores.
//
// Block shape (paper Figure 5a, generalised):
//   O[n,y,x,k] = sum over taps (i,j) and channels c of I[n, y+i-p, x+j-p, c] * F[i,j,k,c]
// with the taps that would read outside the image removed from the iteration
// space by affine constraints (Section 3.2).  A removed tap contributes nothing
// to a sum, so the kernel realises the constraints by zero-filling the halo of
// the LDS copy of the image rows: no constraint arithmetic is left in the loop
// (Section 2.3, "Separating Interior and Boundary Tiles").
//
// Nesting (Section 3.1.3), mapped by hand:
//   outer block  -> one workgroup per strip of ROWS output rows of one image,
//   middle block -> the strip's ROWS+2 input rows (with halo) and the whole
//                   3x3x64x64 filter, staged once in LDS (about 139 KB of 160 KB),
//   inner block  -> one wavefront per output row: 2 pixel fragments x 2 channel
//                   fragments of v_mfma_f32_32x32x16_bf16, 36 K steps (9 taps x 64 channels).
// Both LDS arrays hold 128-byte rows (one pixel or one filter row = 64 channels)
// with the 16-byte chunks XOR-swizzled by (row>>1)&7, so the 16-byte fragment
// reads of 32 consecutive pixels / filter rows are bank-conflict free.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

struct ConvParams {
  int32_t N, H, W, strips_per_image, rows, pad_;
  int64_t i_n, i_y, i_x;      // input element strides (channel stride 1)
  int64_t o_n, o_y, o_x;      // output element strides (channel stride 1)
  int64_t i_base, f_base, o_base;
};

constexpr int C_CI = 64, C_CO = 64, C_TAPS = 9;
constexpr int C_FILTER_BYTES = C_TAPS * C_CO * C_CI * 2;   // 73,728
constexpr int C_MAX_ROWS = 7;

__device__ __forceinline__ int swz(int row, int chunk) { return chunk ^ ((row >> 1) & 7); }

// LDS: [filter: 576 rows x 128 B][patch: (rows+2) x (W+2) pixels x 128 B]
__global__ __launch_bounds__(C_MAX_ROWS * 64) void conv3x3_bf16_kernel(const ConvParams p, const uint16_t* __restrict__ I,
                                                                       const uint16_t* __restrict__ F, float* __restrict__ O) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* lf = lds;
  unsigned char* lp = lds + C_FILTER_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6, nthreads = blockDim.x;
  const int n = blockIdx.x / p.strips_per_image;
  const int y0 = (blockIdx.x % p.strips_per_image) * p.rows;   // first output row of the strip
  const int PW = p.W + 2;                                        // patch width in pixels

  // ---- stage the filter (576 rows (tap, k) of 8 chunks) and the image rows
  // y0-1 .. y0+rows with a zero halo.  All global loads of a lane are issued
  // before the first LDS store, so their latencies overlap.
  constexpr int MAXQ = 11;   // ceil(4608 / 448) and ceil(9 * 66 * 8 / 448)
  const u32x4* fg = (const u32x4*)(F + p.f_base);
  const int patch_rows = p.rows + 2;
  const int patch_chunks = patch_rows * PW * 8;
  const uint16_t* ig = I + p.i_base + (int64_t)n * p.i_n;
  u32x4 fv[MAXQ], pv[MAXQ];
#pragma unroll
  for (int u = 0; u < MAXQ; ++u) {
    const int q = t + u * nthreads;
    fv[u] = (u32x4){0u, 0u, 0u, 0u};
    if (q < C_TAPS * C_CO * 8) fv[u] = fg[q];
  }
#pragma unroll
  for (int u = 0; u < MAXQ; ++u) {
    const int q = t + u * nthreads;
    const int pix = q >> 3, c = q & 7;
    const int r = pix / PW, col = pix - r * PW;
    const int y = y0 - 1 + r, x = col - 1;
    pv[u] = (u32x4){0u, 0u, 0u, 0u};
    if (q < patch_chunks && y >= 0 && y < p.H && x >= 0 && x < p.W)
      pv[u] = *(const u32x4*)(ig + (int64_t)y * p.i_y + (int64_t)x * p.i_x + c * 8);
  }
#pragma unroll
  for (int u = 0; u < MAXQ; ++u) {
    const int q = t + u * nthreads;
    const int row = q >> 3, c = q & 7;
    if (q < C_TAPS * C_CO * 8) *(u32x4*)(lf + row * 128 + (swz(row, c) << 4)) = fv[u];
  }
#pragma unroll
  for (int u = 0; u < MAXQ; ++u) {
    const int q = t + u * nthreads;
    const int pix = q >> 3, c = q & 7;
    if (q < patch_chunks) *(u32x4*)(lp + pix * 128 + (swz(pix, c) << 4)) = pv[u];
  }
  __syncthreads();

  // ---- one wavefront per output row ---------------------------------------
  const int y = y0 + wave;
  if (wave >= p.rows || y >= p.H) return;
  const int fr = lane & 31, fh = lane >> 5;
  // pixel fragments: columns 0..31 and 32..63; columns beyond W are clamped (computed, never stored)
  int xa[2];
  xa[0] = fr < p.W ? fr : p.W - 1;
  xa[1] = 32 + fr < p.W ? 32 + fr : p.W - 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int b = 0; b < 2; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.f;

  for (int tap = 0; tap < C_TAPS; ++tap) {
    const int ti = tap / 3, tj = tap - ti * 3;
    // patch pixel of output column x for this tap: row wave + ti, column x + tj   (halo shifts both by one)
    int pa[2];
    pa[0] = (wave + ti) * PW + xa[0] + tj;
    pa[1] = (wave + ti) * PW + xa[1] + tj;
    const int f0 = tap * C_CO + fr;          // filter rows of channel fragment 0; fragment 1 is 32 rows further
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int chunk = 2 * s + fh;
      bf16x8 af[2], bf[2];
      af[0] = *(const bf16x8*)(lp + pa[0] * 128 + (swz(pa[0], chunk) << 4));
      af[1] = *(const bf16x8*)(lp + pa[1] * 128 + (swz(pa[1], chunk) << 4));
      bf[0] = *(const bf16x8*)(lf + f0 * 128 + (swz(f0, chunk) << 4));
      bf[1] = *(const bf16x8*)(lf + (f0 + 32) * 128 + (swz(f0 + 32, chunk) << 4));
#pragma unroll
      for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[a], bf[b], acc[a][b], 0, 0, 0);
    }
  }

  // ---- store: accumulator element v of lane l is pixel 8*(v/4) + 4*(l>>5) + v%4 of its fragment, channel l&31
  float* og = O + p.o_base + (int64_t)n * p.o_n + (int64_t)y * p.o_y + fr;
#pragma unroll
  for (int a = 0; a < 2; ++a)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int x = 32 * a + 8 * (v / 4) + 4 * fh + (v % 4);
      if (x < p.W) {
#pragma unroll
        for (int b = 0; b < 2; ++b) __builtin_nontemporal_store(acc[a][b][v], og + (int64_t)x * p.o_x + 32 * b);
      }
    }
}

int rows_per_strip(const Conv2dShape& c) {
  // most rows such that the patch fits beside the filter in 160 KB and a strip has at most 7 wavefronts
  int rows = C_MAX_ROWS;
  while (rows > 1 && C_FILTER_BYTES + (int64_t)(rows + 2) * (c.W + 2) * 128 > 160 * 1024) --rows;
  return rows;
}

ConvParams make_params(const Conv2dShape& c, int rows) {
  ConvParams p;
  p.N = (int)c.N; p.H = (int)c.H; p.W = (int)c.W;
  p.rows = rows;
  p.strips_per_image = (int)((c.Ho + rows - 1) / rows);
  p.pad_ = 0;
  p.i_n = c.i_n; p.i_y = c.i_y; p.i_x = c.i_x;
  p.o_n = c.o_n; p.o_y = c.o_y; p.o_x = c.o_x;
  p.i_base = c.i_base; p.f_base = c.f_base; p.o_base = c.o_base;
  return p;
}

}  // namespace

bool conv_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info) {
  if (tune_int("conv_mfma", 1) == 0) return false;
  if (in_dtype == STRIPE_I8) return conv_i8_select(c, in_dtype, l, info);
  if (in_dtype != STRIPE_BF16) return false;
  if (c.R != 3 || c.S != 3 || c.stride_y != 1 || c.stride_x != 1 || c.pad_y != 1 || c.pad_x != 1) return false;
  if (c.Ci != C_CI || c.Co != C_CO || c.Ho != c.H || c.Wo != c.W) return false;
  if (c.W > 64 || c.W < 1) return false;
  // channels contiguous; filter laid out [tap][k][c] contiguously; 16-byte global loads
  if (c.i_c != 1 || c.f_c != 1 || c.o_k != 1) return false;
  if (c.f_k != C_CI || c.f_s != C_CO * C_CI || c.f_r != 3 * C_CO * C_CI) return false;
  for (int64_t v : {c.i_n, c.i_y, c.i_x, c.i_base, c.f_base})
    if (v % 8) return false;
  const int rows = rows_per_strip(c);
  // a lane stages at most 11 filter chunks and 11 patch chunks
  if ((int64_t)rows * 64 * 11 < C_TAPS * C_CO * 8 || (int64_t)rows * 64 * 11 < (int64_t)(rows + 2) * (c.W + 2) * 8) return false;
  if (C_FILTER_BYTES + (int64_t)(rows + 2) * (c.W + 2) * 128 > 160 * 1024) return false;
  const int64_t grid = c.N * ((c.Ho + rows - 1) / rows);
  if (grid > 0x7fffffffLL) return false;
  l->variant = rows;
  l->grid = grid;
  info->path = STRIPE_PATH_MFMA_CONV;
  info->tile_m = rows * (int)c.W;   // output pixels per workgroup
  info->tile_n = C_CO;
  info->tile_k = C_TAPS * C_CI;
  info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
  info->lds_bytes = C_FILTER_BYTES + (rows + 2) * ((int)c.W + 2) * 128;
  info->workgroup_size = rows * 64;
  info->grid = grid;
  snprintf(info->kernel, sizeof info->kernel, "conv3x3_bf16_c64k64_strip%d_mfma32x32x16", rows);
  return true;
}

hipError_t launch_conv(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t st) {
  if (l.variant >= 100) return launch_conv_i8(c, l, in, flt, out, st);
  if (((uintptr_t)in % 16) || ((uintptr_t)flt % 16) || ((uintptr_t)out % 4)) return hipErrorInvalidValue;
  const int rows = l.variant;
  const ConvParams p = make_params(c, rows);
  const int lds_bytes = C_FILTER_BYTES + (rows + 2) * ((int)c.W + 2) * 128;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {
    e = hipFuncSetAttribute((const void*)conv3x3_bf16_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(conv3x3_bf16_kernel, dim3((unsigned)l.grid), dim3(rows * 64), lds_bytes, st, p, (const uint16_t*)in,
                     (const uint16_t*)flt, (float*)out);
  return hipGetLastError();
}

}  // namespace stripe
