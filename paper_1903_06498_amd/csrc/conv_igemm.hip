// Nested-tile convolution on the gfx950 matrix cores for the whole family of dense convolution-shaped blocks
//   O[n,y,x,k] = sum_{i,j,c} I[n, sy*y + dy*i - py, sx*x + dx*j - px, c] * F[i,j,k,c]
// (any filter extent R x S up to 32 x 32, any stride, dilation and padding, any image width, channels contiguous in
// all three tensors; bf16 with Ci a multiple of 32, or int8 with Ci a multiple of 64; any Co).
//
// The nesting of paper Section 3.1.3 (Figure 3's three columns), mapped by hand:
//   outer block  -> one workgroup per tile of TM output pixels x TN output channels; the pixels of a tile are
//                   consecutive in the flattened (n, y, x) order, so a tile may span rows and images;
//   middle block -> the reduction (i, j, c) walked as K tiles of one filter tap x 64 or 128 bytes of channels, staged in a
//                   four-stage LDS ring by LDS-direct loads: the A side gathers each pixel's channels for that tap
//                   straight from the image (the view of Figure 5b, built by address arithmetic instead of a copy),
//                   the B side takes the tap's [k][c] slice of the filter;
//   inner block  -> v_mfma_f32_32x32x16_bf16 / v_mfma_i32_32x32x32_i8 fragments, 64 pixels x 32 or 64 channels per wavefront.
// Constraints (padding) are realised per pixel and tap: a lane whose tap falls outside the image fetches 16 zero
// bytes instead (adding zero is the identity of the sum), so interior and boundary tiles run the same code and no
// per-point test reaches the matrix instructions (Section 2.3: keep the hot loop rectilinear).
// The two tuned kernels (3x3 / 64 channels in conv.hip, 7x7 / 3 channels in conv_i8.hip) stay the fast cases; this
// kernel re-reads each input element once per tap from L2, which they avoid.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 g_bf16x8;
typedef __attribute__((ext_vector_type(16))) float g_f32x16;
typedef __attribute__((ext_vector_type(4))) int g_i32x4;
typedef __attribute__((ext_vector_type(16))) int g_i32x16;

struct IgemmParams {
  int64_t i_n, i_y, i_x;          // element strides; the channel stride is 1 in all three tensors
  int64_t f_r, f_s, f_k;
  int64_t o_n, o_y, o_x;
  int64_t i_base, f_base, o_base;
  int32_t Ho, Wo, H, W, Co;
  int32_t R, S, stride_y, stride_x, pad_y, pad_x, dil_y, dil_x;
  int32_t m_total;                // output pixels N * Ho * Wo
  int32_t tiles_n;                // workgroup tiles along the output channels
  int32_t chunks;                 // channel chunks (one K tile row each: 64 or 128 bytes) per tap
  int32_t k_tiles;                // R * S * chunks
  int32_t out_bf16;               // float blocks: round the result to bf16 on store
  int32_t epi;                    // 1: the fused form of a following statement O = relu(T + bias[k]) (float blocks)
  int32_t vec_out;                // output strides, base and pointer allow one store per four channels
};

// Lanes whose tap lies outside the image fetch these 16 zero bytes instead.
__device__ __attribute__((aligned(16))) unsigned char igemm_zero_chunk[16];

// LDS-direct 16-byte load: lane i of the wavefront lands at lds_off + 16 * i.  Written as assembly because the
// compiler cannot know that a load into one ring stage does not alias the fragment reads of another; the load
// queue depth is managed by hand with s_waitcnt below.  M0 (the wave-uniform LDS destination) is written here and
// nowhere else in this kernel.
__device__ __forceinline__ void g_load_lds16(const void* src, unsigned lds_off) {
  const unsigned uniform_off = __builtin_amdgcn_readfirstlane(lds_off);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(uniform_off) : "memory", "m0");
}

template <bool I8>
__device__ __forceinline__ g_f32x16 g_mma(g_bf16x8 a, g_bf16x8 b, g_f32x16 acc) {
  if constexpr (I8) {
    return __builtin_bit_cast(g_f32x16, __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(g_i32x4, a), __builtin_bit_cast(g_i32x4, b),
                                                                            __builtin_bit_cast(g_i32x16, acc), 0, 0, 0));
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
  }
}

#define G_FENCE() __builtin_amdgcn_sched_barrier(0)

// The variants that leave room for one workgroup per CU only (256 x 128 tiles, 128-byte K tile rows) are used where
// one round of workgroups covers the block anyway: at most one tile per CU; the large tile from 160 tiles on.
constexpr int64_t kIgemmMinBigTiles = 160, kIgemmCus = 256;

template <int N>
__device__ __forceinline__ void g_wait_loads() {   // until at most N of the wavefront's loads are outstanding
  static_assert(N >= 0 && N < 64, "the counter's range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// Tiles of TM pixels x TN channels, eight wavefronts:
//   128 x 128: wavefronts 2 (pixels) x 4 (channels), each 64 x 32;
//   256 x  64: wavefronts 4 x 2, each 64 x 32;
//   256 x 128: wavefronts 4 x 2, each 64 x 64 -- 24 KB staged per 2.1 Mflop of a K tile instead of 16 KB per 1.05,
//              for shapes whose staging rate (the LDS-direct loads fill about 45 bytes per clock and CU) and not
//              the matrix cores bounds the smaller tiles.
// A K tile is one filter tap x KB bytes of channels (64, or 128 where the channel count allows: whole 128-byte
// lines per pixel, half as many requests and barriers per byte).
// LDS: A stages at 0 (TM rows of KB bytes; 16-byte chunk c of row r in slot c ^ ((r >> 2) & 3) for 64-byte rows,
// c ^ ((r >> 1) & 7) for 128-byte rows), B stages behind them (TN rows, same layout); an LDS-direct load fills one
// 1 KB block = 16 or 8 rows.
template <int TM, int TN, bool I8, int KB>
__global__ __launch_bounds__(512, 1) void conv_igemm_kernel(const IgemmParams p, const unsigned char* __restrict__ I,
                                                            const unsigned char* __restrict__ F, void* __restrict__ O,
                                                            const float* __restrict__ bias) {
  static_assert((TM == 128 && TN == 128) || (TM == 256 && (TN == 64 || TN == 128)), "instantiated tiles");
  constexpr int FB = TM * TN / (8 * 64 * 32); // 32-channel fragments of a wavefront's tile (its pixels: always 64)
  constexpr int WN = TN / (32 * FB);          // wavefronts side by side along the channels
  static_assert(KB == 64 || KB == 128, "K tile rows");
  constexpr int RPB = 1024 / KB;              // rows of a 1 KB block
  constexpr int LPR = KB / 16;                // lanes (16-byte chunks) per row
  constexpr int LA = TM / RPB / 8;            // 1 KB A blocks per wavefront and K tile
  constexpr int NBB = TN / RPB;               // B blocks per K tile
  constexpr int LB = NBB > 8 ? NBB / 8 : 1;   // of them per wavefront
  constexpr int LPT = LA + LB;                // loads per wavefront and K tile
  constexpr int KS = KB / 32;                 // matrix-instruction K steps per K tile
  constexpr int A_STAGE = TM * KB, B_STAGE = TN * KB, B0 = 4 * A_STAGE;
  auto key = [](int row) { return KB == 64 ? ((row >> 2) & 3) : ((row >> 1) & 7); };
  constexpr int ES = I8 ? 1 : 2;              // bytes per input element
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6, wn = wv % WN, wm = wv / WN;
  // consecutive hardware workgroup ids go round the 8 XCDs: give each XCD a contiguous run of tiles, channel tiles
  // of one pixel tile next to each other, so the L2 that fetched a pixel tile serves all its channel tiles
  const unsigned grid = gridDim.x, b = blockIdx.x;
  const unsigned logical = (grid % 8u) ? b : (b % 8u) * (grid / 8u) + b / 8u;
  const int tn = (int)(logical % (unsigned)p.tiles_n), tm = (int)(logical / (unsigned)p.tiles_n);

  // ---- A side: the lane's pixel(s), its first byte in the image for tap (0,0), and which taps are inside the image
  const unsigned char* a_base[LA];
  unsigned rmask[LA], cmask[LA];
#pragma unroll
  for (int u = 0; u < LA; ++u) {
    const int row = RPB * (wv + 8 * u) + lane / LPR;
    const int chunk = (lane % LPR) ^ key(row);
    int m = tm * TM + row;
    if (m >= p.m_total) m = p.m_total - 1;    // rows past the end repeat the last pixel; they are never stored
    const int x = m % p.Wo, q = m / p.Wo, y = q % p.Ho, n = q / p.Ho;
    const int iy0 = y * p.stride_y - p.pad_y, ix0 = x * p.stride_x - p.pad_x;
    a_base[u] = I + (p.i_base + (int64_t)n * p.i_n + (int64_t)iy0 * p.i_y + (int64_t)ix0 * p.i_x) * ES + chunk * 16;
    unsigned rm = 0, cm = 0;
    for (int i = 0; i < p.R; ++i) {
      const int yy = iy0 + i * p.dil_y;
      if (yy >= 0 && yy < p.H) rm |= 1u << i;
    }
    for (int j = 0; j < p.S; ++j) {
      const int xx = ix0 + j * p.dil_x;
      if (xx >= 0 && xx < p.W) cm |= 1u << j;
    }
    rmask[u] = rm;
    cmask[u] = cm;
  }
  // ---- B side: the lane's filter row (an output channel; rows past Co repeat the last one, never stored)
  const unsigned char* b_base[LB];
#pragma unroll
  for (int u = 0; u < LB; ++u) {
    const int bb = (wv + 8 * u) % NBB;        // fewer blocks than wavefronts: only wavefronts 0 .. NBB-1 load B (loads_b)
    const int row = RPB * bb + lane / LPR;
    const int chunk = (lane % LPR) ^ key(row);
    int gn = tn * TN + row;
    if (gn >= p.Co) gn = p.Co - 1;
    b_base[u] = F + (p.f_base + (int64_t)gn * p.f_k) * ES + chunk * 16;
  }
  // with fewer B blocks than wavefronts the higher wavefronts issue one load less per K tile; the waits below count accordingly
  const bool loads_b = NBB >= 8 || __builtin_amdgcn_readfirstlane(wv) < NBB;
  // the K tile the next issue() fetches: filter tap (ti, tj), channel chunk tc, and its byte offsets in the image and
  // the filter, advanced by additions (all wave-uniform): next chunk +KB; next filter column: back to chunk 0 and one
  // column on; next filter row: back to column 0 and one row on
  int ti = 0, tj = 0, tc = 0;
  int64_t a_off = 0, b_off = 0;
  const unsigned char* zero_chunk = igemm_zero_chunk;
  asm volatile("" : "+s"(zero_chunk));   // held in registers: the compiler would otherwise re-read its address from memory for every K tile
  const int64_t a_col = (int64_t)p.dil_x * p.i_x * ES - (int64_t)(p.chunks - 1) * KB, b_col = p.f_s * ES - (int64_t)(p.chunks - 1) * KB;
  const int64_t a_row = (int64_t)p.dil_y * p.i_y * ES - (int64_t)(p.S - 1) * p.dil_x * p.i_x * ES - (int64_t)(p.chunks - 1) * KB;
  const int64_t b_row = p.f_r * ES - (int64_t)(p.S - 1) * p.f_s * ES - (int64_t)(p.chunks - 1) * KB;
  auto issue = [&](int stage) {
#pragma unroll
    for (int u = 0; u < LA; ++u) {
      const bool inside = ((rmask[u] >> ti) & (cmask[u] >> tj) & 1u) != 0;
      const void* src = inside ? (const void*)(a_base[u] + a_off) : (const void*)zero_chunk;
      g_load_lds16(src, stage * A_STAGE + (wv + 8 * u) * 1024);
    }
#pragma unroll
    for (int u = 0; u < LB; ++u)
      if (loads_b) g_load_lds16(b_base[u] + b_off, B0 + stage * B_STAGE + ((wv + 8 * u) % NBB) * 1024);
    if (++tc == p.chunks) {
      tc = 0;
      if (++tj == p.S) {
        tj = 0;
        ++ti;
        a_off += a_row;
        b_off += b_row;
      } else {
        a_off += a_col;
        b_off += b_col;
      }
    } else {
      a_off += KB;
      b_off += KB;
    }
  };

  // ---- fragments: lane supplies row (lane & 31) and 16-byte chunk 2 * s + (lane >> 5) of K step s
  const int fr = lane & 31, fh = lane >> 5;
  const unsigned a_fr = (unsigned)((wm * 64 + fr) * KB + ((fh ^ key(fr)) << 4));
  const unsigned b_fr = (unsigned)(B0 + (wn * 32 * FB + fr) * KB + ((fh ^ key(fr)) << 4));
  auto read_frags = [&](int stage, int s, g_bf16x8 (&af)[2], g_bf16x8 (&bf)[FB]) {
#pragma unroll
    for (int q = 0; q < 2; ++q) af[q] = *(const g_bf16x8*)(lds + (a_fr ^ (unsigned)(s << 5)) + stage * A_STAGE + q * 32 * KB);
#pragma unroll
    for (int f = 0; f < FB; ++f) bf[f] = *(const g_bf16x8*)(lds + (b_fr ^ (unsigned)(s << 5)) + stage * B_STAGE + f * 32 * KB);
  };

  g_f32x16 acc[2][FB];
#pragma unroll
  for (int q = 0; q < 2; ++q)
#pragma unroll
    for (int f = 0; f < FB; ++f)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[q][f][v] = 0.f;

  const int k_tiles = p.k_tiles;   // >= 1
  // The ring holds four K tiles.  During iteration kt the wavefronts multiply tile kt from registers and read the
  // fragments of tile kt+1 (a whole tile ahead, so that an LDS read has an iteration to land before the matrix
  // cores need it); tile kt+2 must have landed by the iteration's end, tile kt+3 is in flight, and after the
  // barrier, when nobody reads tile kt any more, its slot takes tile kt+4.
  issue(0);
  if (k_tiles > 1) issue(1);
  if (k_tiles > 2) issue(2);
  if (k_tiles > 3) issue(3);
  if (k_tiles > 3) {                             // tiles 0 and 1 have landed
    if (loads_b) g_wait_loads<2 * LPT>();
    else g_wait_loads<2 * LA>();
  } else if (k_tiles > 2) {
    if (loads_b) g_wait_loads<LPT>();
    else g_wait_loads<LA>();
  }
  else g_wait_loads<0>();
  __syncthreads();
  g_bf16x8 af[2][KS][2], bf[2][KS][FB];          // [tile parity][K step]
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) read_frags(0, ks, af[0][ks], bf[0][ks]);
  __syncthreads();   // (the compiler waits for these reads here, and so knows in the loop that only the reads ahead are outstanding)
  auto iteration = [&](int kt, g_bf16x8 (&ca)[KS][2], g_bf16x8 (&cb)[KS][FB], g_bf16x8 (&na)[KS][2], g_bf16x8 (&nb)[KS][FB]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      G_FENCE();
      // unconditional: behind the last tile this reads a stale ring slot and nobody uses it; under a condition the
      // compiler would make the matrix instructions wait for the reads ahead as well
      read_frags((kt + 1) & 3, ks, na[ks], nb[ks]);
#pragma unroll
      for (int q = 0; q < 2; ++q)
#pragma unroll
        for (int f = 0; f < FB; ++f) acc[q][f] = g_mma<I8>(ca[ks][q], cb[ks][f], acc[q][f]);
    }
    G_FENCE();
    if (kt + 3 >= k_tiles) g_wait_loads<0>();
    else if (loads_b) g_wait_loads<LPT>();       // all but tile kt+3: tile kt+2 has landed
    else g_wait_loads<LA>();
    __syncthreads();
    if (kt + 4 < k_tiles) issue(kt & 3);
    G_FENCE();
  };
  for (int kt = 0; kt < k_tiles; kt += 2) {
    iteration(kt, af[0], bf[0], af[1], bf[1]);
    if (kt + 1 < k_tiles) iteration(kt + 1, af[1], bf[1], af[0], bf[0]);
  }

  // ---- store.  The ring is no longer needed: its first bytes take the output offset of each of the tile's pixels
  // (-1 for rows past the last pixel and for pixels no iteration writes), computed once per pixel instead of once per accumulator element.
  __syncthreads();
  int64_t* out_off = (int64_t*)lds;
  if (t < TM) {
    const int m = tm * TM + t;
    int64_t off = -1;
    if (m < p.m_total) {
      const int x = m % p.Wo, q = m / p.Wo, y = q % p.Ho, n = q / p.Ho;
      // a pixel none of whose taps lies inside the image is written by no iteration: it keeps its contents
      const int iy0 = y * p.stride_y - p.pad_y, ix0 = x * p.stride_x - p.pad_x;
      bool any_row = false, any_col = false;
      for (int i = 0; i < p.R; ++i) any_row |= (iy0 + i * p.dil_y >= 0 && iy0 + i * p.dil_y < p.H);
      for (int j = 0; j < p.S; ++j) any_col |= (ix0 + j * p.dil_x >= 0 && ix0 + j * p.dil_x < p.W);
      if (any_row && any_col) off = p.o_base + (int64_t)n * p.o_n + (int64_t)y * p.o_y + (int64_t)x * p.o_x;
    }
    out_off[t] = off;
  }
  __syncthreads();
  if (p.vec_out) {
    // A fragment (32 pixels x 32 channels) goes through a 4 KB buffer of the wavefront, [pixel][32 channels] with the
    // 16-byte slots swizzled by the pixel, and leaves as one store per pixel and channel quad: eight lanes write
    // the 128 contiguous bytes of a pixel's channels (accumulator element v of lane l is pixel 8*(v/4) + 4*(l>>5) +
    // v%4, channel l&31).  The fused form adds the bias and applies the relu on the way (Section 2.3: the
    // temporary of the two statements never exists in memory).
    unsigned char* buf = lds + TM * 8 + wv * 4096;
    const int sp = lane >> 3, sc = lane & 7;
#pragma unroll
    for (int qf = 0; qf < 2 * FB; ++qf) {
      const int q = qf % 2, f = qf / 2;
      const int k0 = tn * TN + (wn * FB + f) * 32 + sc * 4;   // the lane's four output channels
      float b4[4] = {0.f, 0.f, 0.f, 0.f};
      if (!I8 && p.epi) {
#pragma unroll
        for (int e = 0; e < 4; ++e)
          if (k0 + e < p.Co) b4[e] = bias[k0 + e];
      }
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int pixel = 8 * (v / 4) + 4 * fh + (v % 4);
        *(float*)(buf + pixel * 128 + ((((fr >> 2) ^ (pixel & 7)) << 4) | ((fr & 3) << 2))) = acc[q][f][v];
      }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int pixel = 8 * j + sp;
        typedef __attribute__((ext_vector_type(4))) float f4;
        f4 val = *(const f4*)(buf + pixel * 128 + ((sc ^ sp) << 4));
        const int64_t off = out_off[wm * 64 + 32 * q + pixel];
        if (off < 0 || k0 >= p.Co) continue;
        if (!I8 && p.epi) {
          val.x = __builtin_fmaxf(val.x + b4[0], 0.f);   // relu; a NaN becomes 0
          val.y = __builtin_fmaxf(val.y + b4[1], 0.f);
          val.z = __builtin_fmaxf(val.z + b4[2], 0.f);
          val.w = __builtin_fmaxf(val.w + b4[3], 0.f);
        }
        const float ve[4] = {val.x, val.y, val.z, val.w};
        if (!I8 && p.out_bf16) {
          uint16_t h[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const uint32_t u = __float_as_uint(ve[e]);
            h[e] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);   // round to nearest even
          }
          uint16_t* dst = (uint16_t*)O + off + k0;
          if (k0 + 3 < p.Co) {
            typedef __attribute__((ext_vector_type(2))) unsigned u2;
            const u2 packed = {(unsigned)h[0] | ((unsigned)h[1] << 16), (unsigned)h[2] | ((unsigned)h[3] << 16)};
            __builtin_nontemporal_store(packed, (u2*)dst);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (k0 + e < p.Co) dst[e] = h[e];
          }
        } else {
          float* dst = (float*)O + off + k0;             // int32 results travel as bit patterns
          if (k0 + 3 < p.Co) {
            __builtin_nontemporal_store(val, (f4*)dst);
          } else {
#pragma unroll
            for (int e = 0; e < 4; ++e)
              if (k0 + e < p.Co) __builtin_nontemporal_store(ve[e], dst + e);
          }
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
    return;
  }
#pragma unroll
  for (int qf = 0; qf < 2 * FB; ++qf) {
    const int q = qf % 2, f = qf / 2;
    const int k = tn * TN + (wn * FB + f) * 32 + fr;   // the lane's output channel
    if (k >= p.Co) continue;
    float b1 = 0.f;
    if (!I8 && p.epi) b1 = bias[k];
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int row = wm * 64 + 32 * q + 8 * (v / 4) + (v % 4) + 4 * fh;
      const int64_t off = out_off[row];
      if (off < 0) continue;
      float val = acc[q][f][v];
      if (!I8 && p.epi) val = __builtin_fmaxf(val + b1, 0.f);
      if (!I8 && p.out_bf16) {
        const uint32_t u = __float_as_uint(val);
        ((uint16_t*)O)[off + k] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);   // round to nearest even
      } else {
        __builtin_nontemporal_store(val, (float*)O + off + k);   // int32 results travel as bit patterns
      }
    }
  }
}

}  // namespace

bool conv_igemm_select(const Conv2dShape& c, int in_dtype, bool out_bf16, ConvLaunch* l, stripe_block_info_t* info) {
  if (tune_int("conv_igemm", 1) == 0) return false;
  const bool i8 = in_dtype == STRIPE_I8;
  if (!i8 && in_dtype != STRIPE_BF16) return false;
  const int64_t ck = i8 ? 64 : 32;            // channels per 64-byte K tile row
  const int64_t al = i8 ? 16 : 8;             // elements per 16 bytes
  if (c.i_c != 1 || c.f_c != 1 || c.o_k != 1) return false;
  if (c.Ci < ck || c.Ci % ck || c.Co < 1 || c.R < 1 || c.S < 1 || c.R > 32 || c.S > 32) return false;
  if (c.stride_y < 1 || c.stride_x < 1 || c.dil_y < 1 || c.dil_x < 1 || c.pad_y < 0 || c.pad_x < 0) return false;
  for (int64_t v : {c.i_n, c.i_y, c.i_x, c.i_base, c.f_r, c.f_s, c.f_k, c.f_base})
    if (v % al) return false;                 // 16-byte loads
  for (int64_t v : {c.N, c.Ho, c.Wo, c.H, c.W, c.Co, c.stride_y, c.stride_x, c.pad_y, c.pad_x, c.dil_y, c.dil_x})
    if (v > 0x3fffffff) return false;
  const int64_t m_total = c.N * c.Ho * c.Wo;
  if (m_total < 1 || m_total > 0x7fffffffLL - 512) return false;
  if (c.R * c.S * (c.Ci / ck) > 0x7fffffffLL) return false;
  // Workgroup tile by the cost model of paper Section 3.3 at the LDS level: the block as a contraction over
  // indexes (pixel, channel, reduction); a tile's views are its TM x Kt slice of gathered input and its TN x Kt
  // slice of the filter, Kt = the four K tiles the ring holds; cost = 128-byte lines staged per multiply-accumulate,
  // overflow of ragged tiles included.  A range shorter than the tile is padded to one tile (the kernel computes
  // the padding and discards it) while the work stays the real one.  Candidates are the instantiated tiles; the
  // largest, 256 x 128 with one workgroup per CU, only where its tiles cover most of the chip's 256 CUs and no more
  // (the model has no term for idle CUs or for rounds of workgroups; measured: 196 such tiles beat 392 of 128 x 128,
  // 392 of them lose to 784); ties go to fewer tiles.  STRIPE_TUNE conv_igemm_tn = 64 / 128, conv_igemm_tm =
  // 128 / 256 and conv_igemm_kb = 64 / 128 override the choices.
  int tn = 0, tm = 0;
  {
    const int64_t k_total = c.R * c.S * c.Ci, kt = std::min<int64_t>(4 * ck, k_total);
    stripe_tile_model_t m = {};
    m.line_elems = kGfx950LdsLineBytes / (i8 ? 1 : 2);
    m.mem_cap_elems = kGfx950LdsCapBytes / (i8 ? 1 : 2);
    m.counted_refs = 3u;
    m.tiled_idx = 7u;
    const int forced = tune_int("conv_igemm_tn", 0), forced_tm = tune_int("conv_igemm_tm", 0);
    double best = 0;
    int64_t best_tiles = 0;
    const int cands[3][2] = {{256, 128}, {128, 128}, {256, 64}};
    for (const auto& cd : cands) {
      const int cand = cd[1], cand_tm = cd[0];
      if (cand == 128 && forced_tm && forced_tm != cand_tm) continue;
      const int64_t big_tiles = ((m_total + 255) / 256) * ((c.Co + 127) / 128);
      if (cand_tm == 256 && cand == 128 && forced_tm != 256 && (big_tiles < kIgemmMinBigTiles || big_tiles > kIgemmCus)) continue;
      const int64_t tile[3] = {cand_tm, cand, kt};
      TileProblem pr;
      pr.range = {std::max<int64_t>(m_total, tile[0]), std::max<int64_t>(c.Co, tile[1]), k_total};
      TileRef a, b;
      a.coeff = {1, 0, 0, /**/ 0, 0, 1};
      a.stride = {k_total, 1};
      b.coeff = {0, 1, 0, /**/ 0, 0, 1};
      b.stride = {k_total, 1};
      pr.refs = {a, b};
      stripe_tile_cost_t cost;
      tile_cost_of(pr, tile, m, &cost);
      const double per_real_work = cost.cost * ((double)pr.range[0] / (double)m_total) * ((double)pr.range[1] / (double)c.Co);
      if (forced == cand) {
        tn = cand;
        tm = cand_tm;
        break;
      }
      if (!cost.admissible) continue;
      if (!tn || per_real_work < best || (per_real_work == best && cost.tiles < best_tiles)) {
        tn = cand;
        tm = cand_tm;
        best = per_real_work;
        best_tiles = cost.tiles;
      }
    }
    if (!tn) tn = 128, tm = 128;
  }
  const int64_t tiles_m = (m_total + tm - 1) / tm, tiles_n = (c.Co + tn - 1) / tn;
  if (tiles_m * tiles_n > 0x7fffffffLL) return false;
  // 128-byte K tile rows where a tap's channels are whole 128-byte lines, on the 128 x 128 tile (four such stages of
  // the 256-pixel tiles would not fit the LDS), for blocks of at most one tile per CU (128 KB: one workgroup per CU)
  const int forced_kb = tune_int("conv_igemm_kb", 0);
  const bool kb128 = (c.Ci * (i8 ? 1 : 2)) % 128 == 0 && tm == 128 && (forced_kb ? forced_kb == 128 : tiles_m * tiles_n <= kIgemmCus);
  const int kb = kb128 ? 128 : 64;
  l->variant = kConvIgemmVariant + (tn == 64 ? 1 : tm == 256 ? 2 : 0) + (kb128 ? 4 : 0);
  l->grid = tiles_m * tiles_n;
  info->path = STRIPE_PATH_MFMA_CONV;
  info->tile_m = tm; info->tile_n = tn; info->tile_k = kb / (i8 ? 1 : 2);
  info->frag_m = 32; info->frag_n = 32; info->frag_k = i8 ? 32 : 16;
  info->lds_bytes = 4 * (tm + tn) * kb;
  info->workgroup_size = 512;
  info->grid = l->grid;
  snprintf(info->kernel, sizeof info->kernel, "conv_igemm_%s_%dx%dx%d_mfma32x32x%d_w8_lds_direct%s", i8 ? "i8" : "bf16", tm, tn, kb / (i8 ? 1 : 2),
           i8 ? 32 : 16, (!i8 && out_bf16) ? "_obf16" : "");
  return true;
}

hipError_t launch_conv_igemm(const Conv2dShape& c, const ConvLaunch& l, int in_dtype, bool out_bf16, const void* in, const void* flt, void* out,
                             const void* bias, hipStream_t st) {
  const bool i8 = in_dtype == STRIPE_I8;
  if (((uintptr_t)in % 16) || ((uintptr_t)flt % 16) || ((uintptr_t)out % (out_bf16 ? 2 : 4)) || ((uintptr_t)bias % 4)) return hipErrorInvalidValue;
  if (bias && i8) return hipErrorInvalidValue;
  IgemmParams p;
  p.i_n = c.i_n; p.i_y = c.i_y; p.i_x = c.i_x;
  p.f_r = c.f_r; p.f_s = c.f_s; p.f_k = c.f_k;
  p.o_n = c.o_n; p.o_y = c.o_y; p.o_x = c.o_x;
  p.i_base = c.i_base; p.f_base = c.f_base; p.o_base = c.o_base;
  p.Ho = (int)c.Ho; p.Wo = (int)c.Wo; p.H = (int)c.H; p.W = (int)c.W; p.Co = (int)c.Co;
  p.R = (int)c.R; p.S = (int)c.S;
  p.stride_y = (int)c.stride_y; p.stride_x = (int)c.stride_x; p.pad_y = (int)c.pad_y; p.pad_x = (int)c.pad_x;
  p.dil_y = (int)c.dil_y; p.dil_x = (int)c.dil_x;
  p.m_total = (int)(c.N * c.Ho * c.Wo);
  const int shape = (l.variant - kConvIgemmVariant) & 3, kb = ((l.variant - kConvIgemmVariant) & 4) ? 128 : 64;
  const int tn = shape == 1 ? 64 : 128, tm = shape == 0 ? 128 : 256;
  if (kb == 128 && shape != 0) return hipErrorInvalidValue;
  p.tiles_n = (int)((c.Co + tn - 1) / tn);
  p.chunks = (int)(c.Ci * (i8 ? 1 : 2) / kb);
  p.k_tiles = (int)(c.R * c.S) * p.chunks;
  p.out_bf16 = out_bf16 ? 1 : 0;
  p.epi = bias ? 1 : 0;
  // one store per pixel and four channels where every such group starts on a 16-byte (bf16 output: 8-byte) boundary
  p.vec_out = (c.o_n % 4 == 0 && c.o_y % 4 == 0 && c.o_x % 4 == 0 && c.o_base % 4 == 0 && (uintptr_t)out % (out_bf16 ? 8 : 16) == 0) ? 1 : 0;
  typedef void (*kern_t)(const IgemmParams, const unsigned char*, const unsigned char*, void*, const float*);
  kern_t fn;
  if (kb == 64) {
    fn = tn == 64    ? (i8 ? (kern_t)conv_igemm_kernel<256, 64, true, 64> : (kern_t)conv_igemm_kernel<256, 64, false, 64>)
         : tm == 256 ? (i8 ? (kern_t)conv_igemm_kernel<256, 128, true, 64> : (kern_t)conv_igemm_kernel<256, 128, false, 64>)
                     : (i8 ? (kern_t)conv_igemm_kernel<128, 128, true, 64> : (kern_t)conv_igemm_kernel<128, 128, false, 64>);
  } else {
    fn = i8 ? (kern_t)conv_igemm_kernel<128, 128, true, 128> : (kern_t)conv_igemm_kernel<128, 128, false, 128>;
  }
  const int lds_bytes = 4 * (tm + tn) * kb;   // the ring; the store phase needs tm * 8 + 8 * 4096 of it
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {   // more than 64 KB of dynamic LDS has to be enabled once per device
    e = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(fn, dim3((unsigned)l.grid), dim3(512), lds_bytes, st, p, (const unsigned char*)in, (const unsigned char*)flt, out,
                     (const float*)bias);
  return hipGetLastError();
}

}  // namespace stripe
