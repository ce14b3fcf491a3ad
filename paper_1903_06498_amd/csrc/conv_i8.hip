// Strided int8 convolution-shaped contraction on the gfx950 matrix cores,
// exact int32 accumulation:
//   O[n,y,x,k] = sum over taps (i,j) and channels c of I[n, 2y+i-3, 2x+j-3, c] * F[i,j,k,c]
// for a 7x7 filter, 3 input channels, 64 output channels; taps outside the
// image are outside the iteration space (affine constraints, paper Section 3.2)
// and are realised as zero operands, which is exact for integer sums.
//
// With only 3 channels the contraction index (i,j,c) is hostile to matrix
// instructions, so the "microarchitectural transposition / stenciling" of
// Section 2.3 is done explicitly in LDS: for every image row r and output
// column x the 21 bytes I[r, 2x-3 .. 2x+3, 0..2] are laid out as one 32-byte,
// 16-byte-aligned K vector E[r][x] (bytes 21..31 meet zero weights).  One
// v_mfma_i32_16x16x64_i8 then consumes two filter rows (2 x 32 bytes of K) for
// 16 output columns x 16 output channels; the 7 filter rows take 4 K steps (the
// eighth row has zero weights).
//
// Nesting: outer block -> strips of TY output rows of one image, walked by
// persistent workgroups; middle block -> the strip's 2*TY+5 image rows, expanded,
// in LDS; inner block -> one wavefront per output row, 7 x 4 fragments of 16 x 16.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(4))) int i32x4;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;

constexpr int Q_CO = 64, Q_R = 7, Q_S = 7, Q_CI = 3;
constexpr int Q_MAX_WO = 112;                  // 7 column fragments of 16
constexpr int Q_BT_BYTES = 4 * Q_CO * 64;      // filter as K vectors: [K step][k][64 B]

struct I8Params {
  int32_t H, W, Ho, Wo, strips_per_image, raw_row_bytes, total_strips;
  uint32_t chunks_magic, wo_magic;   // ceil(2^32 / d) for d = chunks per raw row and Wo: q / d = umulhi(q, magic) for q < 2^16
  int64_t i_n, i_y;            // input strides in elements (= bytes); pixels and channels are contiguous
  int64_t o_n, o_y, o_x;       // output strides in elements; channels contiguous
  int64_t i_base, f_base, o_base;
};

// Raw chunks of one strip, global -> registers (zero where outside the image or in the row padding).
template <int Q_TY, int RAWQ>
__device__ __forceinline__ void q_load_raw(const I8Params& p, const int8_t* __restrict__ I, int strip, int t, u32x4 (&rv)[RAWQ]) {
  constexpr int Q_ROWS = 2 * Q_TY + 5, NT = Q_TY * 64;
  const int row_chunks = p.raw_row_bytes / 16;          // 16 zero bytes, W*3 data bytes, 16 zero bytes
  const int data_chunks = (p.W * Q_CI) / 16;
  const int n = strip / p.strips_per_image;
  const int y0 = (strip - n * p.strips_per_image) * Q_TY;
  const int8_t* ig = I + p.i_base + (int64_t)n * p.i_n;
#pragma unroll
  for (int u = 0; u < RAWQ; ++u) {
    const int q = t + u * NT;
    const int r = (int)__umulhi((unsigned)q, p.chunks_magic), c = q - r * row_chunks;
    const int y = 2 * y0 - 3 + r;
    rv[u] = (u32x4){0u, 0u, 0u, 0u};
    if (strip < p.total_strips && q < Q_ROWS * row_chunks && c >= 1 && c <= data_chunks && y >= 0 && y < p.H)
      rv[u] = *(const u32x4*)(ig + (int64_t)y * p.i_y + (c - 1) * 16);
  }
}

// Persistent workgroups: each builds the filter's K vectors once, then walks strips
// blockIdx.x, blockIdx.x + gridDim.x, ...  The raw rows of the next strip are fetched
// into registers while the current strip is expanded, multiplied and stored, and the
// stores of a strip (fire and forget) overlap the staging of the next one.
// LDS: [Bt: 16 KB][raw: Q_ROWS x raw_row_bytes][E: Q_ROWS x Wo x 32 B][output transposition: 2 x 4 KB per wavefront]
template <int Q_TY>   // output rows per strip = wavefronts per workgroup
__global__ __launch_bounds__(Q_TY * 64) void conv7x7s2_i8_kernel(const I8Params p, const int8_t* __restrict__ I,
                                                               const int8_t* __restrict__ F, int32_t* __restrict__ O) {
  constexpr int Q_ROWS = 2 * Q_TY + 5;           // image rows a strip touches
  constexpr int NT = Q_TY * 64;
  constexpr int RAWQ = 4, FQ = 5;                 // >= ceil(Q_ROWS*46/NT) and ceil(588/NT) for every strip height
  constexpr int F_BYTES = Q_R * Q_S * Q_CO * Q_CI;   // 9,408 = 588 chunks of 16
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* bt = lds;
  unsigned char* raw = lds + Q_BT_BYTES;
  unsigned char* ex = raw + Q_ROWS * p.raw_row_bytes;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  unsigned char* ot = ex + Q_ROWS * p.Wo * 32 + wave * 8192;   // this wavefront's two output transposition buffers
  const int row_chunks = p.raw_row_bytes / 16;

  // ---- first strip's rows and the filter as it lies in memory (parked where E is built later);
  // all global loads of a lane are issued before the first LDS store so that their latencies overlap
  int strip = blockIdx.x;
  u32x4 rv[RAWQ], fv[FQ];
  q_load_raw<Q_TY, RAWQ>(p, I, strip, t, rv);
  const u32x4* fg = (const u32x4*)(F + p.f_base);
#pragma unroll
  for (int u = 0; u < FQ; ++u) {
    const int q = t + u * NT;
    fv[u] = (u32x4){0u, 0u, 0u, 0u};
    if (q < F_BYTES / 16) fv[u] = fg[q];
  }
#pragma unroll
  for (int u = 0; u < FQ; ++u) {
    const int q = t + u * NT;
    if (q < F_BYTES / 16) *(u32x4*)(ex + q * 16) = fv[u];
  }
  __syncthreads();
  // ---- filter as K vectors: Bt[ks][k][0..31] = F[2ks][*][k][*] (21 B, then zeros), [32..63] = F[2ks+1][...] ----
  for (int q = t; q < 8 * Q_CO; q += NT) {
    const int i = q / Q_CO, k = q - i * Q_CO;           // filter row (7 = the all-zero eighth row), output channel
    unsigned w[8] = {0u, 0u, 0u, 0u, 0u, 0u, 0u, 0u};
    if (i < Q_R) {
#pragma unroll
      for (int b = 0; b < Q_S * Q_CI; ++b) {
        const int j = b / Q_CI, c = b - j * Q_CI;
        const unsigned byte = ex[((i * Q_S + j) * Q_CO + k) * Q_CI + c];
        w[b >> 2] |= byte << (8 * (b & 3));
      }
    }
    unsigned char* dst = bt + ((i >> 1) * Q_CO + k) * 64 + (i & 1) * 32;
    *(u32x4*)dst = (u32x4){w[0], w[1], w[2], w[3]};
    *(u32x4*)(dst + 16) = (u32x4){w[4], w[5], w[6], w[7]};
  }
  __syncthreads();
  // B fragments stay in registers for the workgroup's lifetime: [K step][channel fragment]
  const int fr = lane & 15, kq = lane >> 4;              // fragment row / 16-byte K block of the lane
  i32x4 bfr[4][4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks)
#pragma unroll
    for (int nf = 0; nf < 4; ++nf) bfr[ks][nf] = *(const i32x4*)(bt + (ks * Q_CO + nf * 16 + fr) * 64 + kq * 16);

  for (; strip < p.total_strips; strip += gridDim.x) {
    const int n = strip / p.strips_per_image;
    const int y0 = (strip - n * p.strips_per_image) * Q_TY;
    // ---- this strip's raw rows: registers -> LDS (rows back to back: r*raw_row_bytes + c*16 = q*16)
#pragma unroll
    for (int u = 0; u < RAWQ; ++u) {
      const int q = t + u * NT;
      if (q < Q_ROWS * row_chunks) *(u32x4*)(raw + q * 16) = rv[u];
    }
    __syncthreads();
    // ---- next strip's raw rows: global -> registers, in flight during the rest of this iteration
    q_load_raw<Q_TY, RAWQ>(p, I, strip + gridDim.x, t, rv);

    // ---- expand: E[r][x] = raw[r] bytes 16 + 6x - 9 .. +23 (16 + (2x-3)*3 is where column 2x-3 starts) ----
    for (int q = t; q < Q_ROWS * p.Wo; q += NT) {
      const int r = (int)__umulhi((unsigned)q, p.wo_magic), x = q - r * p.Wo;
      const int start = 6 * x + 7;
      const unsigned* src = (const unsigned*)(raw + r * p.raw_row_bytes + (start & ~3));
      const unsigned sh = start & 3;
      unsigned d[7];
#pragma unroll
      for (int u = 0; u < 7; ++u) d[u] = src[u];
      unsigned e[6];
#pragma unroll
      for (int u = 0; u < 6; ++u) e[u] = __builtin_amdgcn_alignbyte(d[u + 1], d[u], sh);
      e[5] &= 0x000000ffu;                                  // byte 20 is the last of the 21
      // the two 16-byte halves of a vector swap places for every second group of 8 columns (bank spread)
      unsigned char* dst = ex + (r * p.Wo + x) * 32;
      const int flip = ((x >> 3) & 1) * 16;
      *(u32x4*)(dst + flip) = (u32x4){e[0], e[1], e[2], e[3]};
      *(u32x4*)(dst + (16 - flip)) = (u32x4){e[4], e[5], 0u, 0u};
    }
    __syncthreads();

    // ---- one wavefront per output row.  Software pipeline over the row's 16-column fragments: the K vectors
    // of fragment mf+1 are requested before the matrix instructions of fragment mf, and the result tile of
    // fragment mf leaves (LDS read-back + global stores) while fragment mf+1 is multiplied, through two
    // alternating transposition buffers.
    const int y = y0 + wave;
    if (y < p.Ho) {
      const int n_mf = p.Wo / 16;
      int32_t* og = O + p.o_base + (int64_t)n * p.o_n + (int64_t)y * p.o_y;
      // E row of K step ks for this lane: image row 2y + i - 3 relative to the strip's first row; the eighth
      // filter row has zero weights, so any row will do for it
      int erow[4];
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        const int r = 2 * wave + 2 * ks + (kq >> 1);
        erow[ks] = (r < Q_ROWS ? r : Q_ROWS - 1) * p.Wo;
      }
      auto load_a = [&](int mf, i32x4 (&a)[4]) {
        const int x = mf * 16 + fr;
        const int half = ((kq & 1) ^ ((x >> 3) & 1)) * 16;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) a[ks] = *(const i32x4*)(ex + (erow[ks] + x) * 32 + half);
      };
      // a tile leaves: lane (px = 4j + kq, slot fr) reads 16 bytes and stores them; every store instruction
      // writes 4 whole pixels = 1 KB of consecutive addresses when pixels are contiguous
      auto drain = [&](int mf) {
        const unsigned char* buf = ot + (mf & 1) * 4096;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int px = 4 * j + kq;
          const i32x4 v = *(const i32x4*)(buf + px * 256 + ((fr ^ px) << 4));
          *(i32x4*)(og + (int64_t)(mf * 16 + px) * p.o_x + fr * 4) = v;
        }
      };
      i32x4 a_cur[4], a_nxt[4];
      load_a(0, a_cur);
      for (int mf = 0; mf < n_mf; ++mf) {
        if (mf + 1 < n_mf) load_a(mf + 1, a_nxt);
        i32x4 acc[4];
#pragma unroll
        for (int nf = 0; nf < 4; ++nf) acc[nf] = (i32x4){0, 0, 0, 0};
        // filter fragment as the row operand, pixels as the column operand: the result fragment is
        // (channel, pixel) and a lane ends up with 4 consecutive channels of one pixel
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
          for (int nf = 0; nf < 4; ++nf) acc[nf] = __builtin_amdgcn_mfma_i32_16x16x64_i8(bfr[ks][nf], a_cur[ks], acc[nf], 0, 0, 0);
        if (mf > 0) drain(mf - 1);          // written one iteration ago: no wait on LDS
        // accumulator element v of lane l: channel 4*(l>>4) + v of the fragment, pixel l&15 -> 16-byte slots
        // XOR-swizzled with the pixel
        unsigned char* buf = ot + (mf & 1) * 4096;
#pragma unroll
        for (int nf = 0; nf < 4; ++nf) *(i32x4*)(buf + fr * 256 + (((nf * 4 + kq) ^ fr) << 4)) = acc[nf];
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) a_cur[ks] = a_nxt[ks];
      }
      drain(n_mf - 1);
    }
    __syncthreads();   // E and raw are rewritten by the next strip
  }
}

I8Params make_params(const Conv2dShape& c, int Q_TY) {
  I8Params p;
  p.H = (int)c.H; p.W = (int)c.W; p.Ho = (int)c.Ho; p.Wo = (int)c.Wo;
  p.strips_per_image = (int)((c.Ho + Q_TY - 1) / Q_TY);
  p.raw_row_bytes = 16 + (int)c.W * Q_CI + 16;
  p.total_strips = (int)c.N * p.strips_per_image;
  p.chunks_magic = (uint32_t)((((uint64_t)1 << 32) + (p.raw_row_bytes / 16) - 1) / (p.raw_row_bytes / 16));
  p.wo_magic = (uint32_t)((((uint64_t)1 << 32) + p.Wo - 1) / p.Wo);
  p.i_n = c.i_n; p.i_y = c.i_y;
  p.o_n = c.o_n; p.o_y = c.o_y; p.o_x = c.o_x;
  p.i_base = c.i_base; p.f_base = c.f_base; p.o_base = c.o_base;
  return p;
}

int lds_bytes_for(const I8Params& p, int Q_TY) {
  const int Q_ROWS = 2 * Q_TY + 5;
  return Q_BT_BYTES + Q_ROWS * p.raw_row_bytes + Q_ROWS * p.Wo * 32 + Q_TY * 8192;
}

constexpr int kStripChoices[] = {2, 4, 7, 8};

}  // namespace

bool conv_i8_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info) {
  if (c.dil_y != 1 || c.dil_x != 1) return false;
  if (in_dtype != STRIPE_I8) return false;
  if (c.R != Q_R || c.S != Q_S || c.stride_y != 2 || c.stride_x != 2 || c.pad_y != 3 || c.pad_x != 3) return false;
  if (c.Ci != Q_CI || c.Co != Q_CO) return false;
  if (c.W % 32 || c.Wo != c.W / 2 || c.Wo > Q_MAX_WO || c.H % 2 || c.Ho != c.H / 2) return false;   // whole 16-column fragments
  // pixels and channels contiguous in a row, rows 16-byte aligned; filter [i][j][k][c] contiguous
  if (c.i_c != 1 || c.i_x != Q_CI || c.i_y % 16 || c.i_n % 16 || c.i_base % 16) return false;
  if (c.f_c != 1 || c.f_k != Q_CI || c.f_s != Q_CO * Q_CI || c.f_r != Q_S * Q_CO * Q_CI || c.f_base % 16) return false;

  if (c.o_k != 1 || c.o_x % 4 || c.o_y % 4 || c.o_n % 4 || c.o_base % 4) return false;   // 16-byte stores
  int Q_TY = tune_int("conv_i8_rows", 7);
  bool known = false;
  for (int v : kStripChoices) known = known || v == Q_TY;
  if (!known) Q_TY = 7;
  const int Q_ROWS = 2 * Q_TY + 5;
  if (Q_ROWS * (c.W / 2) * 32 < Q_R * Q_S * Q_CO * Q_CI) return false;   // the raw filter is parked in E's space
  const I8Params p = make_params(c, Q_TY);
  if (c.N * (int64_t)p.strips_per_image > 0x7fffffffLL || lds_bytes_for(p, Q_TY) > 160 * 1024) return false;
  // persistent workgroups: as many as fit on the chip at once (LDS-limited), at most one per strip
  const int per_cu = (160 * 1024) / lds_bytes_for(p, Q_TY);
  int64_t grid = (int64_t)tune_int("conv_i8_wg_per_cu", per_cu > 2 ? 2 : per_cu) * 256;
  if (grid > p.total_strips) grid = p.total_strips;
  if (grid < 1) grid = 1;
  if ((int64_t)Q_ROWS * (p.raw_row_bytes / 16) > 4 * Q_TY * 64) return false;   // a lane stages at most 4 row chunks
  l->variant = 100 + Q_TY;
  l->grid = grid;
  info->path = STRIPE_PATH_MFMA_CONV;
  info->tile_m = Q_TY * (int)c.Wo;
  info->tile_n = Q_CO;
  info->tile_k = 4 * 64;
  info->frag_m = 16; info->frag_n = 16; info->frag_k = 64;
  info->lds_bytes = lds_bytes_for(p, Q_TY);
  info->workgroup_size = Q_TY * 64;
  info->grid = grid;
  snprintf(info->kernel, sizeof info->kernel, "conv7x7s2_i8_c3k64_strip%d_mfma16x16x64", Q_TY);
  return true;
}

namespace {

template <int Q_TY>
hipError_t launch_rows(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t st) {
  const I8Params p = make_params(c, Q_TY);
  const int lds_bytes = lds_bytes_for(p, Q_TY);
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {
    e = hipFuncSetAttribute((const void*)conv7x7s2_i8_kernel<Q_TY>, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(conv7x7s2_i8_kernel<Q_TY>, dim3((unsigned)l.grid), dim3(Q_TY * 64), lds_bytes, st, p, (const int8_t*)in,
                     (const int8_t*)flt, (int32_t*)out);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_conv_i8(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t st) {
  if (((uintptr_t)in % 16) || ((uintptr_t)flt % 16) || ((uintptr_t)out % 16)) return hipErrorInvalidValue;
  switch (l.variant - 100) {
    case 2: return launch_rows<2>(c, l, in, flt, out, st);
    case 7: return launch_rows<7>(c, l, in, flt, out, st);
    case 8: return launch_rows<8>(c, l, in, flt, out, st);
    case 4: return launch_rows<4>(c, l, in, flt, out, st);
    default: return launch_rows<7>(c, l, in, flt, out, st);
  }
}

}  // namespace stripe
