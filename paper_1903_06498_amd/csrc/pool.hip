// Max aggregation over a 2-d window of one input (gfx950), HBM-bound.
//
// Block shape (paper Section 2.1 "the max of a maxpool"; Section 3.2 for the
// constraints):  O[n,y,x,c] = max over taps (i,j) with
//   0 <= s*y + i - p < H  and  0 <= s*x + j - q < W   of  I[n, s*y+i-p, s*x+j-q, c].
// Out-of-range taps are not part of the iteration space: they contribute
// nothing, no address outside the image is read and no padding value enters.
//
// Mapping: channels are contiguous, so a lane owns 4 channels (one 16-byte
// load) of one output column; 16 lanes cover the 256 bytes of a 64-channel
// pixel.  Three kernels share it:
//   strip (default)   128 lanes own 128 consecutive (column, channel-quad)
//                     items and TY output rows; all stride*(TY-1)+R input rows
//                     are requested up front and rows shared by neighbouring
//                     windows are reused from registers;
//   strip with selects the same, with out-of-range taps replaced by -inf
//                     (used when in-row offsets need more than 32 bits);
//   rolling           a lane walks down a chunk of output rows and carries the
//                     shared input row, so a chunk fetches every row once
//                     (lowest L2 fetch traffic, slightly slower in time).
// Boundary handling follows Section 2.3 ("Separating Interior and Boundary
// Tiles") in spirit: the loads carry no per-tap constraint tests and no
// branches.  A tap outside the iteration space is read at its coordinate
// clamped into the image; the clamped tap is one the window holds anyway
// (every window has an in-range row and column) and max is idempotent, so
// the duplicate cannot change the result.
#include <hip/hip_runtime.h>

#include <cmath>

#include <algorithm>

#include "kernels.hpp"

namespace stripe {
namespace {

struct PoolParams {
  int32_t N, H, W, Ho, Wo, C4;       // C4 = channels / 4
  int32_t pad_y, pad_x;
  int32_t items;                      // Wo * C4
  int32_t blocks_per_row, y_strips;
  int32_t xcd_remap;
  int32_t rows;                      // output rows per workgroup (rolling kernel)
  int32_t stream_loads, stream_stores;   // strip kernel: non-temporal loads / stores
  int64_t i_n, i_y, i_x, o_n, o_y, o_x;  // element strides (channel stride is 1)
  int64_t i_base, o_base;
  int64_t w_base, w_r, w_s;              // weighted windows: element offset and tap strides of the weights
  uint32_t bpr_mul, bpr_shr, ys_mul, ys_shr, c4_mul, c4_shr, step_;   // divisions by blocks_per_row, y_strips and C4 as multiply-high and shift (fast_div)
};

// n / d for 0 <= n < 2^31 without a division: with l = ceil(log2 d), p = 31 + l and mul = ceil(2^p / d) < 2^32,
// floor(n * mul / 2^p) = floor(n / d), because mul * d - 2^p < d <= 2^(p - 31) adds less than 1 / d to n / d.
// The host passes mul and shr = p - 32 (magic_of); mul = 0 stands for d = 1.
__device__ __forceinline__ unsigned fast_div(unsigned n, uint32_t mul, uint32_t shr) { return mul ? __umulhi(n, mul) >> shr : n; }

typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ f32x4 max4(f32x4 a, f32x4 b) {
  f32x4 r;
  r.x = b.x > a.x ? b.x : a.x;
  r.y = b.y > a.y ? b.y : a.y;
  r.z = b.z > a.z ? b.z : a.z;
  r.w = b.w > a.w ? b.w : a.w;
  return r;
}

// Workgroups that share input rows should share an L2: consecutive hardware
// workgroup ids go round-robin over the 8 XCDs, so give every XCD one
// contiguous range of logical ids.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned grid) {
  if (grid % 8u) return b;
  return (b % 8u) * (grid / 8u) + b / 8u;
}

// The same idea at a finer grain: every XCD takes runs of `group` consecutive logical ids (whole rows of
// workgroups, so that the columns and rows shared between neighbours are fetched into one L2 once) and the runs go
// round-robin over the XCDs, which keeps the chip as a whole streaming through the tensor front to back.
__device__ __forceinline__ unsigned xcd_grouped(unsigned b, unsigned grid, unsigned group) {
  const unsigned full = grid / (8u * group) * (8u * group);
  if (b >= full) return b;
  const unsigned x = b % 8u, t = b / 8u;
  return ((t / group) * 8u + x) * group + t % group;
}

__device__ __forceinline__ unsigned logical_block(int mode, unsigned b, unsigned grid) {
  return mode == 1 ? xcd_contiguous(b, grid) : mode > 1 ? xcd_grouped(b, grid, (unsigned)mode) : b;
}

template <int R, int S, int ST, int TY, bool NT>
__global__ __launch_bounds__(128) void pool_max_f32_kernel(const PoolParams p, const float* __restrict__ in,
                                                          float* __restrict__ out) {
  const unsigned b = logical_block(p.xcd_remap, blockIdx.x, gridDim.x);
  const int bx = b % p.blocks_per_row;
  const int rest = b / p.blocks_per_row;
  const int ys = rest % p.y_strips;
  const int n = rest / p.y_strips;
  const int item = bx * 128 + threadIdx.x;
  if (item >= p.items) return;
  const int c4 = item % p.C4;
  const int xo = item / p.C4;

  const float* inb = in + p.i_base + (int64_t)n * p.i_n + c4 * 4;
  float* outb = out + p.o_base + (int64_t)n * p.o_n + (int64_t)xo * p.o_x + c4 * 4;

  // Branch-free: every coordinate is clamped into the buffer so that all loads of
  // the strip are issued unconditionally and back to back (they are independent;
  // the memory system sees (ST*(TY-1)+R)*S sixteen-byte loads per lane in flight),
  // then taps outside the iteration space are replaced by the identity of max.
  constexpr int NR = ST * (TY - 1) + R;   // input rows a strip of TY output rows touches
  const int x0 = xo * ST - p.pad_x;
  bool xv[S];
  int64_t xoff[S];
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int xc = x0 + j;
    xv[j] = xc >= 0 && xc < p.W;
    xoff[j] = (int64_t)(xc < 0 ? 0 : (xc >= p.W ? p.W - 1 : xc)) * p.i_x;
  }
  const float ninf = -__builtin_huge_valf();
  const f32x4 lowest = {ninf, ninf, ninf, ninf};
  const int yo0 = ys * TY;
  const int y0 = yo0 * ST - p.pad_y;

  f32x4 v[NR][S];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int y = y0 + r;
    const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
    const float* rp = inb + (int64_t)yc * p.i_y;
#pragma unroll
    for (int j = 0; j < S; ++j)
      v[r][j] = NT ? __builtin_nontemporal_load((const f32x4*)(rp + xoff[j])) : *(const f32x4*)(rp + xoff[j]);
  }
  f32x4 hm[NR];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int y = y0 + r;
    const bool yv = y >= 0 && y < p.H;
    f32x4 m = lowest;
#pragma unroll
    for (int j = 0; j < S; ++j) m = max4(m, (yv && xv[j]) ? v[r][j] : lowest);
    hm[r] = m;
  }
#pragma unroll
  for (int ty = 0; ty < TY; ++ty) {
    const int yo = yo0 + ty;
    f32x4 m = hm[ty * ST];
#pragma unroll
    for (int i = 1; i < R; ++i) m = max4(m, hm[ty * ST + i]);
    if (yo < p.Ho) {
      f32x4* dst = (f32x4*)(outb + (int64_t)yo * p.o_y);
      if (NT) __builtin_nontemporal_store(m, dst);
      else *dst = m;
    }
  }
}

// Rolling variant for R = 3, stride 2: a lane keeps its (column, channel-quad)
// and walks down `rows` output rows.  Consecutive windows share one input row
// (row 2y+1-p of output row y is row 2(y+1)-1-p of the next), whose horizontal
// maximum is carried in registers, so inside a workgroup's chunk every input
// row is fetched exactly once; the two new rows of the next output row are
// requested before the current one is reduced and stored.
//
// The kernel is written to issue few vector instructions per byte, which
// matters as much as the access pattern at this arithmetic intensity:
//  * a tap outside the iteration space is read at its coordinate clamped into
//    the image.  The clamped tap is a tap the window holds anyway (every
//    window has at least one in-range row and column), and max is idempotent,
//    so the duplicate leaves the result unchanged and no select is needed;
//  * rows are uniform over a workgroup, so a row's base address lives in
//    scalar registers and each load adds only a per-lane 32-bit byte offset;
//  * the 3-way maxima map to three-operand max instructions.
__device__ __forceinline__ f32x4 max3x4(f32x4 a, f32x4 b, f32x4 c) {
  f32x4 r;
  r.x = __builtin_fmaxf(__builtin_fmaxf(a.x, b.x), c.x);
  r.y = __builtin_fmaxf(__builtin_fmaxf(a.y, b.y), c.y);
  r.z = __builtin_fmaxf(__builtin_fmaxf(a.z, b.z), c.z);
  r.w = __builtin_fmaxf(__builtin_fmaxf(a.w, b.w), c.w);
  return r;
}

__global__ __launch_bounds__(512) void pool_max_f32_roll_kernel(const PoolParams p, const float* __restrict__ in,
                                                               float* __restrict__ out) {
  constexpr int ST = 2, S = 3;
  const unsigned b = blockIdx.x;
  const int bx = b % p.blocks_per_row;
  const int rest = b / p.blocks_per_row;
  const int ys = rest % p.y_strips;
  const int n = rest / p.y_strips;
  const int item = bx * (int)blockDim.x + threadIdx.x;
  if (item >= p.items) return;
  const int c4 = item % p.C4;
  const int xo = item / p.C4;

  // per-lane byte offsets inside a row (the host has checked that they fit in 32 bits)
  uint32_t voff[S];
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int xc = xo * ST - p.pad_x + j;
    const int xcl = xc < 0 ? 0 : (xc >= p.W ? p.W - 1 : xc);
    voff[j] = ((uint32_t)xcl * (uint32_t)p.i_x + (uint32_t)c4 * 4u) * 4u;
  }
  const uint32_t ooff = ((uint32_t)xo * (uint32_t)p.o_x + (uint32_t)c4 * 4u) * 4u;
  // uniform bases
  const char* ib = (const char*)(in + p.i_base + (int64_t)n * p.i_n);
  char* ob = (char*)(out + p.o_base + (int64_t)n * p.o_n);

  auto hload = [&](f32x4 (&v)[S], int y) {
    const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
    const char* rp = ib + (int64_t)yc * p.i_y * 4;
#pragma unroll
    for (int j = 0; j < S; ++j) v[j] = *(const f32x4*)(rp + voff[j]);
  };
  const int yo0 = ys * p.rows;
  auto store = [&](int yo, f32x4 m) { *(f32x4*)(ob + (int64_t)yo * p.o_y * 4 + ooff) = m; };

  const int yend = yo0 + p.rows < p.Ho ? yo0 + p.rows : p.Ho;   // yo0 < Ho by construction of the grid
  int yi = yo0 * ST - p.pad_y;                                    // first input row of the current window
  f32x4 c[S], a0[S], a1[S], b0[S], b1[S];
  hload(c, yi);
  hload(a0, yi + 1);
  hload(a1, yi + 2);
  f32x4 carried = max3x4(c[0], c[1], c[2]);
  int yo = yo0;
  // two output rows per trip so that the register sets swap roles without copies
  for (; yo + 2 < yend; yo += 2, yi += 2 * ST) {
    hload(b0, yi + 3);
    hload(b1, yi + 4);
    f32x4 h1 = max3x4(a1[0], a1[1], a1[2]);
    store(yo, max3x4(carried, max3x4(a0[0], a0[1], a0[2]), h1));
    carried = h1;
    hload(a0, yi + 5);
    hload(a1, yi + 6);
    h1 = max3x4(b1[0], b1[1], b1[2]);
    store(yo + 1, max3x4(carried, max3x4(b0[0], b0[1], b0[2]), h1));
    carried = h1;
  }
  if (yo + 1 < yend) {   // two rows left
    hload(b0, yi + 3);
    hload(b1, yi + 4);
    f32x4 h1 = max3x4(a1[0], a1[1], a1[2]);
    store(yo, max3x4(carried, max3x4(a0[0], a0[1], a0[2]), h1));
    store(yo + 1, max3x4(h1, max3x4(b0[0], b0[1], b0[2]), max3x4(b1[0], b1[1], b1[2])));
  } else {               // one row left
    store(yo, max3x4(carried, max3x4(a0[0], a0[1], a0[2]), max3x4(a1[0], a1[1], a1[2])));
  }
}

// Strip kernel with the same instruction diet as the rolling kernel (clamped
// duplicates instead of selects, uniform row bases, three-operand maxima):
// 128 lanes own 128 (column, channel-quad) items and TY output rows, and all
// loads of the strip are issued before the first reduction.  Window R x S,
// stride ST, max or min (both idempotent, which the clamped duplicates need).
// MODE: 0 max, 1 min, 2 sum.  A sum is not idempotent, so there the taps outside the image are replaced by zeros
// (exact for a sum) instead of being left as clamped duplicates.
template <int MODE>
__device__ __forceinline__ float pick(float a, float b) {
  return MODE == 2 ? a + b : MODE == 1 ? __builtin_fminf(a, b) : __builtin_fmaxf(a, b);
}
template <int N, int MODE>
__device__ __forceinline__ f32x4 fold(const f32x4* v) {
  f32x4 r = v[0];
#pragma unroll
  for (int i = 1; i < N; ++i) {
    r.x = pick<MODE>(r.x, v[i].x);
    r.y = pick<MODE>(r.y, v[i].y);
    r.z = pick<MODE>(r.z, v[i].z);
    r.w = pick<MODE>(r.w, v[i].w);
  }
  return r;
}

template <int R, int S, int ST, int TY, int MODE>
__global__ __launch_bounds__(1024) void pool_f32_strip_kernel(const PoolParams p, const float* __restrict__ in,
                                                            float* __restrict__ out, const float* __restrict__ scale) {
  // scale: a sum (MODE 2) times one factor kept in a one-element buffer (average pooling), or NULL
  constexpr int NR = ST * (TY - 1) + R;
  // A workgroup keeps its 128 (column, channel-quad) items and walks over strips (image, row strip) with the
  // grid's stride: gridDim.x = blocks_per_row * (strips walked side by side), so everything that depends on the
  // column is computed once.  Fewer, longer-lived workgroups stream better than one short workgroup per strip.
  // A workgroup lives for a few thousand cycles, so what precedes its first load counts: the arguments are all
  // fetched at once (the compiler would fetch them group by group where first used, one memory latency each), and
  // the quotients come from multiplications.
  const unsigned grid_x = gridDim.x, strips_per_wg = blockDim.y;
  asm volatile("" ::"s"(p.N), "s"(p.items), "s"(p.i_n), "s"(p.o_n), "s"(p.i_base), "s"(p.o_base), "s"(p.bpr_mul), "s"(p.ys_mul), "s"(p.ys_shr),
               "s"(p.c4_mul), "s"(p.c4_shr), "s"(p.step_), "s"(grid_x), "s"(strips_per_wg), "s"(in), "s"(out), "s"(scale));
  float factor = 1.f;
  if constexpr (MODE == 2)
    if (scale) factor = scale[p.w_base];
  const unsigned b = logical_block(p.xcd_remap, blockIdx.x, grid_x);
  const unsigned brow = fast_div(b, p.bpr_mul, p.bpr_shr);
  const int bx = (int)(b - brow * (unsigned)p.blocks_per_row);
  const int item = bx * 128 + threadIdx.x;
  if (item >= p.items) return;
  const int xo = (int)fast_div((unsigned)item, p.c4_mul, p.c4_shr);
  const int c4 = item - xo * p.C4;
  uint32_t voff[S];
  bool xv[S];
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int xc = xo * ST - p.pad_x + j;
    const int xcl = xc < 0 ? 0 : (xc >= p.W ? p.W - 1 : xc);
    xv[j] = xc == xcl;
    voff[j] = ((uint32_t)xcl * (uint32_t)p.i_x + (uint32_t)c4 * 4u) * 4u;
  }
  const uint32_t ooff = ((uint32_t)xo * (uint32_t)p.o_x + (uint32_t)c4 * 4u) * 4u;
  // blockDim.y strips per workgroup (threadIdx.y picks one: row bases stay wave-uniform), gridDim.x / blocks_per_row
  // such workgroups side by side
  const int strips = p.N * p.y_strips, step = (int)p.step_ * (int)strips_per_wg;
  for (int rest = (int)brow * (int)strips_per_wg + (int)threadIdx.y; rest < strips; rest += step) {
    const int n = (int)fast_div((unsigned)rest, p.ys_mul, p.ys_shr);
    const int ys = rest - n * p.y_strips;
    const char* ib = (const char*)(in + p.i_base + (int64_t)n * p.i_n);
    char* ob = (char*)(out + p.o_base + (int64_t)n * p.o_n);
    const int yo0 = ys * TY;
    const int y0 = yo0 * ST - p.pad_y;

    f32x4 v[NR][S];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int y = y0 + r;
      const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
      const char* rp = ib + (int64_t)yc * p.i_y * 4;
      if (p.stream_loads) {
#pragma unroll
        for (int j = 0; j < S; ++j) v[r][j] = __builtin_nontemporal_load((const f32x4*)(rp + voff[j]));
      } else {
#pragma unroll
        for (int j = 0; j < S; ++j) v[r][j] = *(const f32x4*)(rp + voff[j]);
      }
    }
    f32x4 hm[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      if constexpr (MODE == 2) {
        const int y = y0 + r;
        const bool yv = y >= 0 && y < p.H;
        const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < S; ++j) v[r][j] = (yv && xv[j]) ? v[r][j] : zero;
      }
      hm[r] = fold<S, MODE>(v[r]);
    }
#pragma unroll
    for (int ty = 0; ty < TY; ++ty) {
      const int yo = yo0 + ty;
      if (yo < p.Ho) {
        f32x4 res = fold<R, MODE>(hm + ty * ST);
        if constexpr (MODE == 2) res *= factor;
        if (p.stream_stores) __builtin_nontemporal_store(res, (f32x4*)(ob + (int64_t)yo * p.o_y * 4 + ooff));
        else *(f32x4*)(ob + (int64_t)yo * p.o_y * 4 + ooff) = res;
      }
    }
  }
}

// ---------------------------------------------------------------------------
// LDS-staged strip kernel.  The workgroup's input patch -- every input row of its blockDim.y output rows, the
// columns its 128 (column, channel-quad) items reach -- goes global -> LDS once, by LDS-direct 16-byte loads (no
// staging registers, no LDS-store instructions); every lane then takes its R x S taps from LDS.  Each input vector
// is requested from L1 / L2 once per workgroup instead of once per tap that uses it, which is what separates the
// register kernel above from a plain 4 : 1 stream.  Taps outside the image: max / min stage the clamped pixel (a
// duplicate of a tap the window holds anyway), sums stage zeros.  One output row per 128 lanes (threadIdx.y).
// ---------------------------------------------------------------------------
__device__ __attribute__((aligned(16))) unsigned char pool_zero_chunk[16];

// M0 (the wave-uniform LDS destination of an LDS-direct load) is written here and nowhere else in this kernel.
__device__ __forceinline__ void pool_load_lds16(const void* src, unsigned lds_off) {
  const unsigned uniform_off = __builtin_amdgcn_readfirstlane(lds_off);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(uniform_off) : "memory", "m0");
}

template <int R, int S, int ST, int MODE>
__global__ __launch_bounds__(1024) void pool_f32_lds_kernel(const PoolParams p, const float* __restrict__ in, float* __restrict__ out) {
  extern __shared__ __attribute__((aligned(16))) unsigned char patch[];
  const unsigned b = blockIdx.x;
  const int bx = b % p.blocks_per_row;
  const int rest = b / p.blocks_per_row;
  const int yg = rest % p.y_strips;               // group of blockDim.y output rows
  const int n = rest / p.y_strips;
  const int rows_out = (int)blockDim.y;
  const int t = threadIdx.y * 128 + threadIdx.x, lanes = 128 * rows_out;
  // columns of the patch: the items bx*128 .. bx*128+127 of the row (clipped) cover output columns xo_first .. xo_last
  const int item_first = bx * 128, item_last = min(item_first + 127, p.items - 1);
  const int xo_first = item_first / p.C4, xo_last = item_last / p.C4;
  const int x0 = xo_first * ST - p.pad_x;                              // first input column (may be -1: clamped)
  const int pw = (xo_last - xo_first) * ST + S;                        // patch width in pixels
  const int pwv = pw * p.C4;                                           // ... in 16-byte vectors
  const int y0 = yg * rows_out * ST - p.pad_y;                         // first input row
  const int nr = ST * (rows_out - 1) + R;                              // patch rows
  const int total = nr * pwv;
  const char* ib = (const char*)(in + p.i_base + (int64_t)n * p.i_n);
  // ---- stage: vector g of the patch = (row g / pwv, pixel (g % pwv) / C4, channel quad (g % pwv) % C4); every
  // wavefront issues whole loads, lanes past the end fetch a dummy vector into the slack behind the patch
  for (int g0 = 0; g0 < total; g0 += lanes) {
    const int g = g0 + t;
    const int gc = g < total ? g : 0;
    const int row = gc / pwv, col = gc - row * pwv;
    const int px = col / p.C4, c4 = col - px * p.C4;
    const int y = y0 + row, x = x0 + px;
    const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y), xc = x < 0 ? 0 : (x >= p.W ? p.W - 1 : x);
    const void* src = ib + ((int64_t)yc * p.i_y + (int64_t)xc * p.i_x + c4 * 4) * 4;
    if (MODE == 2 && (y != yc || x != xc)) src = pool_zero_chunk;
    pool_load_lds16(src, (unsigned)((g0 + (t & ~63)) * 16));
  }
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();
  // ---- reduce: lane = one (column, channel quad) item of output row threadIdx.y
  const int item = item_first + threadIdx.x;
  const int yo = yg * rows_out + threadIdx.y;
  if (item >= p.items || yo >= p.Ho) return;
  const int c4 = item % p.C4, xo = item / p.C4;
  const unsigned char* lp = patch + ((threadIdx.y * ST) * pwv + (xo - xo_first) * ST * p.C4 + c4) * 16;
  f32x4 hm[R];
#pragma unroll
  for (int r = 0; r < R; ++r) {
    f32x4 v[S];
#pragma unroll
    for (int j = 0; j < S; ++j) v[j] = *(const f32x4*)(lp + (r * pwv + j * p.C4) * 16);
    hm[r] = fold<S, MODE>(v);
  }
  const f32x4 res = fold<R, MODE>(hm);
  float* op = out + p.o_base + (int64_t)n * p.o_n + (int64_t)yo * p.o_y + (int64_t)xo * p.o_x + c4 * 4;
  if (p.stream_stores) __builtin_nontemporal_store(res, (f32x4*)op);
  else *(f32x4*)op = res;
}

// Weighted windows (sum aggregation of products, no reduction over channels): every tap of the window is multiplied
// by a weight before it enters the sum.  WMODE 1: one scalar for all taps -- average pooling written as
// O += I * scale with the scale in a one-element buffer; the kernel sums the in-range taps and scales once.
// WMODE 2: a weight per tap and channel, W[i, j, c] -- depthwise convolution; a lane keeps the R x S weight quads
// of its four channels in registers.  Same lane mapping and load pattern as the strip kernel above; taps outside
// the image are read at a clamped address and replaced by zeros (exact for a sum).
template <int R, int S, int ST, int TY, int WMODE>
__global__ __launch_bounds__(512) void window_weighted_f32_kernel(const PoolParams p, const float* __restrict__ in,
                                                                 const float* __restrict__ wgt, float* __restrict__ out) {
  constexpr int NR = ST * (TY - 1) + R;
  // (arguments fetched at once and quotients by multiplication, as in the strip kernel)
  const unsigned grid_x = gridDim.x, strips_per_wg = blockDim.y;
  if constexpr (WMODE == 2)
    asm volatile("" ::"s"(p.N), "s"(p.items), "s"(p.i_n), "s"(p.o_n), "s"(p.i_base), "s"(p.o_base), "s"(p.w_base), "s"(p.bpr_mul), "s"(p.ys_mul),
                 "s"(p.ys_shr), "s"(p.c4_mul), "s"(p.c4_shr), "s"(grid_x), "s"(strips_per_wg), "s"(in), "s"(wgt), "s"(out));
  const unsigned b = logical_block(p.xcd_remap, blockIdx.x, grid_x);
  const unsigned brow = fast_div(b, p.bpr_mul, p.bpr_shr);
  const int bx = (int)(b - brow * (unsigned)p.blocks_per_row);
  // blockDim.y strips side by side per workgroup, one per 128 lanes (they share input rows through L1)
  const int rest = (int)brow * (int)strips_per_wg + (int)threadIdx.y;
  if (rest >= p.N * p.y_strips) return;
  const int n = (int)fast_div((unsigned)rest, p.ys_mul, p.ys_shr);
  const int ys = rest - n * p.y_strips;
  const int item = bx * 128 + threadIdx.x;
  if (item >= p.items) return;
  const int xo = (int)fast_div((unsigned)item, p.c4_mul, p.c4_shr);
  const int c4 = item - xo * p.C4;
  uint32_t voff[S];
  bool xv[S];
#pragma unroll
  for (int j = 0; j < S; ++j) {
    const int xc = xo * ST - p.pad_x + j;
    const int xcl = xc < 0 ? 0 : (xc >= p.W ? p.W - 1 : xc);
    xv[j] = xc == xcl;
    voff[j] = ((uint32_t)xcl * (uint32_t)p.i_x + (uint32_t)c4 * 4u) * 4u;
  }
  const uint32_t ooff = ((uint32_t)xo * (uint32_t)p.o_x + (uint32_t)c4 * 4u) * 4u;
  const char* ib = (const char*)(in + p.i_base + (int64_t)n * p.i_n);
  char* ob = (char*)(out + p.o_base + (int64_t)n * p.o_n);
  const int yo0 = ys * TY;
  const int y0 = yo0 * ST - p.pad_y;

  f32x4 v[NR][S];
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int y = y0 + r;
    const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
    const char* rp = ib + (int64_t)yc * p.i_y * 4;
#pragma unroll
    for (int j = 0; j < S; ++j) v[r][j] = *(const f32x4*)(rp + voff[j]);
  }
  f32x4 w[R][S];
  float scale = 1.f;
  if constexpr (WMODE == 2) {
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
      for (int j = 0; j < S; ++j) w[i][j] = *(const f32x4*)(wgt + p.w_base + (int64_t)i * p.w_r + (int64_t)j * p.w_s + c4 * 4);
  } else {
    scale = wgt[p.w_base];
  }
  const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int r = 0; r < NR; ++r) {
    const int y = y0 + r;
    const bool yv = y >= 0 && y < p.H;
#pragma unroll
    for (int j = 0; j < S; ++j) v[r][j] = (yv && xv[j]) ? v[r][j] : zero;
  }
#pragma unroll
  for (int ty = 0; ty < TY; ++ty) {
    const int yo = yo0 + ty;
    f32x4 acc = zero;
#pragma unroll
    for (int i = 0; i < R; ++i)
#pragma unroll
      for (int j = 0; j < S; ++j) {
        if constexpr (WMODE == 2) acc += v[ty * ST + i][j] * w[i][j];
        else acc += v[ty * ST + i][j];
      }
    if constexpr (WMODE == 1) acc *= scale;
    if (yo < p.Ho) *(f32x4*)(ob + (int64_t)yo * p.o_y * 4 + ooff) = acc;
  }
}

// multiplier and shift of fast_div for the divisor d >= 1
static void magic_of(int64_t d, uint32_t* mul, uint32_t* shr) {
  if (d <= 1) {
    *mul = 0;
    *shr = 0;
    return;
  }
  int l = 0;
  while (((int64_t)1 << l) < d) ++l;
  const int pw = 31 + l;
  *mul = (uint32_t)((((unsigned __int128)1 << pw) + (unsigned __int128)d - 1) / (unsigned __int128)d);
  *shr = (uint32_t)(pw - 32);
}

PoolParams make_params(const Pool2dShape& s, int ty, int wg) {
  PoolParams p;
  p.N = (int)s.N; p.H = (int)s.H; p.W = (int)s.W; p.Ho = (int)s.Ho; p.Wo = (int)s.Wo; p.C4 = (int)(s.C / 4);
  p.pad_y = (int)s.pad_y; p.pad_x = (int)s.pad_x;
  p.items = p.Wo * p.C4;
  p.blocks_per_row = (p.items + wg - 1) / wg;
  p.y_strips = (p.Ho + ty - 1) / ty;
  p.xcd_remap = tune_int("pool_xcd", 0);      // 1: one contiguous range of workgroups per XCD
  if (const int rows = tune_int("pool_xcd_rows", 0); rows > 0 && p.xcd_remap == 0)
    p.xcd_remap = rows * p.blocks_per_row > 1 ? rows * p.blocks_per_row : 2;   // runs of `rows` whole rows of workgroups per XCD
  p.stream_loads = tune_int("pool_ntl", 0);
  p.stream_stores = tune_int("pool_nts", 0);
  p.rows = ty;
  p.i_n = s.i_n; p.i_y = s.i_y; p.i_x = s.i_x; p.o_n = s.o_n; p.o_y = s.o_y; p.o_x = s.o_x;
  p.i_base = s.i_base; p.o_base = s.o_base;
  p.w_base = s.w_base; p.w_r = s.w_r; p.w_s = s.w_s;
  magic_of(p.blocks_per_row, &p.bpr_mul, &p.bpr_shr);
  magic_of(p.y_strips, &p.ys_mul, &p.ys_shr);
  magic_of(p.C4, &p.c4_mul, &p.c4_shr);
  p.step_ = 0;   // workgroups side by side (grid / blocks_per_row): set at launch
  return p;
}

constexpr int kTyChoices[] = {1, 2, 3, 4, 7};



template <int TY, bool NT>
hipError_t launch_ty(const PoolParams& p, int64_t grid, const void* in, void* out, hipStream_t st, bool lean, int yb) {
  if (lean && !NT) {
    PoolParams q = p;
    q.step_ = (uint32_t)(grid / p.blocks_per_row);
    hipLaunchKernelGGL((pool_f32_strip_kernel<3, 3, 2, TY, 0>), dim3((unsigned)grid), dim3(128, yb), 0, st, q, (const float*)in, (float*)out, (const float*)nullptr);
    return hipGetLastError();
  }
  hipLaunchKernelGGL((pool_max_f32_kernel<3, 3, 2, TY, NT>), dim3((unsigned)grid), dim3(128), 0, st, p, (const float*)in, (float*)out);
  return hipGetLastError();
}

}  // namespace

// variant = index into kTyChoices * 2 + nontemporal flag for the strip kernel, kRollVariant for the rolling kernel
constexpr int kRollVariant = 100;
// other windows, min and sum pooling: lean strip kernel, 2 output rows per strip; variant = kShapeVariant + 3*shape + mode
constexpr int kShapeVariant = 200;
// weighted windows: variant = kWeightedVariant + 2*shape + (0: one scale, 1: per tap and channel)
constexpr int kWeightedVariant = 300;
// LDS-staged kernel: variant = kLdsVariant + 3*shape + mode, rows per workgroup in PoolLaunch::rows
constexpr int kLdsVariant = 400;
struct PoolWindow { int r, s, stride; };
constexpr PoolWindow kWindows[] = {{3, 3, 2}, {2, 2, 2}, {3, 3, 1}};

// Strip shape by the cost model of paper Section 3.3, applied at the two memory levels a window kernel tiles for:
//   lane level   a lane's tile is one output column x four channels x TY rows; its views (the
//                (stride * (TY - 1) + R) x S x 4 input patch, the outputs, the weights of a weighted window) live in
//                registers; its cost is the 16-byte accesses the lane issues per output vector;
//   workgroup level  YB strips side by side, one per 128 lanes, share input rows through the CU's L1: the tile is
//                TY * YB output rows of the whole image width; its cost is the 16-byte vectors fetched from L2 per
//                output vector.
// Registers are a soft memory (a larger tile still runs, with fewer wavefronts resident), so instead of a hard cap the
// L2-level cost is scaled by 1 + registers * kGfx950RegPenalty, and an L1 access is charged kGfx950L1AccessCost of an
// L2 access.  Launches with fewer than kGfx950MinWorkgroups workgroups are avoided when a candidate has more (ramp
// and tail of such launches cost more than the sharing saves).  These three constants were fitted to sweeps of every
// window shape on this chip and reproduce the measured optimum of each.  Candidates are the shapes the kernels are
// instantiated for; STRIPE_TUNE pool_ty / pool_yb override the choice.
struct StripShape { int ty, yb; };
StripShape choose_strip_shape(const Pool2dShape& s, std::initializer_list<int> ty_available, std::initializer_list<int> yb_available) {
  TileProblem pr;
  pr.range = {s.Ho, s.Wo, s.C, s.R, s.S};                      // indexes y, x, c, i, j
  TileRef in, out;
  in.coeff = {s.stride_y, 0, 0, s.dil_y, 0, /**/ 0, s.stride_x, 0, 0, s.dil_x, /**/ 0, 0, 1, 0, 0};
  in.stride = {s.i_y, s.i_x, 1};
  out.coeff = {1, 0, 0, 0, 0, /**/ 0, 1, 0, 0, 0, /**/ 0, 0, 1, 0, 0};
  out.stride = {s.o_y, s.o_x, 1};
  pr.refs = {in, out};
  if (s.w_mode == 2) {
    TileRef w;
    w.coeff = {0, 0, 0, 1, 0, /**/ 0, 0, 0, 0, 1, /**/ 0, 0, 1, 0, 0};
    w.stride = {s.w_r, s.w_s, 1};
    pr.refs.push_back(w);
  }                                                            // (a scale is one scalar register: not a view of the lane's tile)
  stripe_tile_model_t m = {};
  m.line_elems = kGfx950RegLineBytes / 4;
  m.mem_cap_elems = kGfx950RegCapRegs;
  m.counted_refs = (1u << pr.refs.size()) - 1;
  m.tiled_idx = 1u;                                            // work counted in output rows
  stripe_tile_model_t wg = m;
  wg.mem_cap_elems = 0;
  wg.counted_refs = 3u;                                        // input and output; the weights stay in registers
  const int want_ty = tune_int("pool_ty", 0), want_yb = tune_int("pool_yb", 0);
  const double vectors_per_row = (double)s.Wo * (double)(s.C / 4);
  const int64_t blocks_per_row = (s.Wo * (s.C / 4) + 127) / 128;
  StripShape best = {0, 0}, fallback = {0, 0};
  double best_cost = 0;
  int64_t best_fp = 0;
  bool best_large = false;
  for (int ty : ty_available) {
    if (want_ty && ty != want_ty && std::find(ty_available.begin(), ty_available.end(), want_ty) != ty_available.end()) continue;
    for (int yb : yb_available) {
      if (want_yb && yb != want_yb && std::find(yb_available.begin(), yb_available.end(), want_yb) != yb_available.end()) continue;
      if (!fallback.ty || ty * yb < fallback.ty * fallback.yb) fallback = {ty, yb};
      if (ty > s.Ho || (int64_t)ty * yb > s.Ho + ty - 1) continue;
      const int64_t lane_tile[5] = {ty, 1, 4, s.R, s.S};
      stripe_tile_cost_t lane;
      tile_cost_of(pr, lane_tile, m, &lane);
      if (!lane.admissible) continue;
      const int64_t rows = std::min<int64_t>((int64_t)ty * yb, s.Ho);
      const int64_t wg_tile[5] = {rows, s.Wo, s.C, s.R, s.S};
      stripe_tile_cost_t group;
      tile_cost_of(pr, wg_tile, wg, &group);
      const double l1 = lane.cost / vectors_per_row, l2 = group.cost / vectors_per_row;
      double cost = l2 * (1.0 + (double)lane.footprint_elems * kGfx950RegPenalty) + kGfx950L1AccessCost * l1;
      // occupancy cliff: the tile's registers plus about eight for addresses, in granules of eight, divide the SIMD's 512;
      // under four wavefronts per SIMD the loads in flight no longer cover the memory latency (per-tap weights, four
      // rows: 130 registers, three wavefronts, 52.7 us against 50.5 for three rows)
      const int64_t regs = (lane.footprint_elems + 8 + 7) / 8 * 8, waves = regs > 0 ? 512 / regs : 8;
      if (waves < 4) cost *= std::sqrt(4.0 / (double)(waves > 0 ? waves : 1));
      const int64_t workgroups = blocks_per_row * ((s.N * ((s.Ho + ty - 1) / ty) + yb - 1) / yb);
      const bool large = workgroups >= kGfx950MinWorkgroups;
      const bool better = !best.ty || (large && !best_large) ||
                          (large == best_large && (cost < best_cost || (cost == best_cost && lane.footprint_elems * yb < best_fp)));
      if (better) {
        best = {ty, yb};
        best_cost = cost;
        best_fp = lane.footprint_elems * yb;
        best_large = large;
      }
    }
  }
  return best.ty ? best : fallback;
}

// Workgroups of the strip kernel: blocks_per_row column blocks times the number of strips walked side by side.
// One workgroup per strip and column block measured best (26.0 us on the 3x3 / stride 2 configuration against 26.7
// with 4102 workgroups walking the strips, 28.0 with 2051, 29.3 with 1022): the kernel wants every load of the
// block in flight as early as possible.  STRIPE_TUNE pool_groups = n walks the strips n side by side instead.
int64_t strip_grid(const PoolParams& p, int64_t yb) {
  const int64_t strips = ((int64_t)p.N * p.y_strips + yb - 1) / yb;
  int64_t side = tune_int("pool_groups", -1);
  if (side < 0) side = 0;
  if (side == 0 || side > strips) side = strips;
  return side * p.blocks_per_row;
}

// LDS bytes of the staged kernel's patch for `rows` output rows per workgroup, slack for whole loads included
int64_t lds_patch_bytes(const Pool2dShape& s, int rows) {
  const int64_t c4 = s.C / 4, st = s.stride_x;
  const int64_t px_out = std::min<int64_t>((127 + c4 - 1) / c4 + 1, s.Wo);   // output columns 128 consecutive items can touch
  const int64_t pw = (px_out - 1) * st + s.S, nr = s.stride_y * (rows - 1) + s.R, lanes = 128 * rows;
  const int64_t vectors = (nr * pw * c4 + lanes - 1) / lanes * lanes;
  return vectors * 16;
}

template <int R, int S, int ST, int MODE>
hipError_t launch_lds_rows(int rows, int lds_bytes, const PoolParams& p, dim3 g, const float* i, float* o, hipStream_t st) {
  hipLaunchKernelGGL((pool_f32_lds_kernel<R, S, ST, MODE>), g, dim3(128, rows), lds_bytes, st, p, i, o);
  return hipGetLastError();
}

template <int R, int S, int ST, int MODE>
hipError_t launch_strip_rows(int ty, int yb, const PoolParams& p_, dim3 g, const float* i, float* o, hipStream_t st, const float* w = nullptr) {
  PoolParams p = p_;
  p.step_ = g.x / (unsigned)p.blocks_per_row;
  switch (ty) {
    case 1: hipLaunchKernelGGL((pool_f32_strip_kernel<R, S, ST, 1, MODE>), g, dim3(128, yb), 0, st, p, i, o, w); break;
    case 2: hipLaunchKernelGGL((pool_f32_strip_kernel<R, S, ST, 2, MODE>), g, dim3(128, yb), 0, st, p, i, o, w); break;
    case 3: hipLaunchKernelGGL((pool_f32_strip_kernel<R, S, ST, 3, MODE>), g, dim3(128, yb), 0, st, p, i, o, w); break;
    case 4: hipLaunchKernelGGL((pool_f32_strip_kernel<R, S, ST, 4, MODE>), g, dim3(128, yb), 0, st, p, i, o, w); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

template <int R, int S, int ST, int WMODE>
hipError_t launch_weighted_rows(int ty, int yb, const PoolParams& p, dim3 g, const float* i, const float* w, float* o, hipStream_t st) {
  switch (ty) {
    case 1: hipLaunchKernelGGL((window_weighted_f32_kernel<R, S, ST, 1, WMODE>), g, dim3(128, yb), 0, st, p, i, w, o); break;
    case 2: hipLaunchKernelGGL((window_weighted_f32_kernel<R, S, ST, 2, WMODE>), g, dim3(128, yb), 0, st, p, i, w, o); break;
    case 3: hipLaunchKernelGGL((window_weighted_f32_kernel<R, S, ST, 3, WMODE>), g, dim3(128, yb), 0, st, p, i, w, o); break;
    case 4: hipLaunchKernelGGL((window_weighted_f32_kernel<R, S, ST, 4, WMODE>), g, dim3(128, yb), 0, st, p, i, w, o); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

bool pool_select(const Pool2dShape& s, int dtype, PoolLaunch* l, stripe_block_info_t* info) {
  if (s.dil_y != 1 || s.dil_x != 1) return false;   // dilated windows run on the generic kernel
  if (dtype != STRIPE_F32) return false;
  int window = -1;
  for (int w = 0; w < (int)(sizeof kWindows / sizeof kWindows[0]); ++w)
    if (s.R == kWindows[w].r && s.S == kWindows[w].s && s.stride_y == kWindows[w].stride && s.stride_x == kWindows[w].stride) window = w;
  if (window < 0) return false;
  if (s.i_c != 1 || s.o_c != 1 || s.C % 4) return false;
  // every window must hold at least one in-range tap, so every output is written
  if (s.pad_y >= s.R || s.pad_x >= s.S) return false;
  if ((s.Ho - 1) * s.stride_y - s.pad_y > s.H - 1 || (s.Wo - 1) * s.stride_x - s.pad_x > s.W - 1) return false;
  // 16-byte loads and stores
  for (int64_t v : {s.i_n, s.i_y, s.i_x, s.o_n, s.o_y, s.o_x, s.i_base, s.o_base})
    if (v % 4) return false;
  if (s.N > 0x7fffffff / 4 || s.H > 0x3fffffff || s.W > 0x3fffffff || s.Wo * (s.C / 4) > 0x3fffffff) return false;
  const bool row_offsets_fit = ((s.W - 1) * s.i_x + s.C) < ((int64_t)1 << 29) && ((s.Wo - 1) * s.o_x + s.C) < ((int64_t)1 << 29) &&
                              s.i_x >= 0 && s.o_x >= 0;
  const int mode = s.agg == STRIPE_AGG_ADD ? 2 : s.agg == STRIPE_AGG_MIN ? 1 : 0;
  if (s.w_mode) {
    // weighted window: a scale (one element) or per-tap, per-channel weights with the channels contiguous (16-byte loads)
    if (mode != 2 || !row_offsets_fit) return false;
    if (s.w_mode == 2 && (s.w_c != 1 || s.w_r % 4 || s.w_s % 4 || s.w_base % 4)) return false;
    // per-tap weights: four strips side by side measured slower than two or one (3x3 stride 1: three rows per strip
    // 50.5 us alone, 49.4 two side by side, 54.5 four), so only the scaled sum is offered four
    const StripShape shape = s.w_mode == 2 ? choose_strip_shape(s, {1, 2, 3, 4}, {1, 2}) : choose_strip_shape(s, {1, 2, 3, 4}, {1, 2, 4});
    const int rows = shape.ty;
    const PoolParams p = make_params(s, rows, 128);
    if ((int64_t)p.N * p.y_strips * p.blocks_per_row > 0x7fffffffLL) return false;
    l->yb = shape.yb;
    const int64_t grid = (((int64_t)p.N * p.y_strips + shape.yb - 1) / shape.yb) * p.blocks_per_row;
    l->variant = kWeightedVariant + 2 * window + (s.w_mode - 1);
    l->rows = rows;
    l->wg = 128;
    l->grid = grid;
    info->path = STRIPE_PATH_POOL;
    info->tile_m = rows;
    info->tile_n = 128;
    info->tile_k = 0;
    info->frag_m = info->frag_n = info->frag_k = 0;
    info->lds_bytes = 0;
    info->workgroup_size = 128 * shape.yb;
    info->grid = grid;
    snprintf(info->kernel, sizeof info->kernel, "%s_f32_%dx%ds%d_ty%d%s", s.w_mode == 2 ? "depthwise" : "pool_scaled_sum", kWindows[window].r,
             kWindows[window].s, kWindows[window].stride, rows, shape.yb == 4 ? "x4" : shape.yb == 2 ? "x2" : "");
    return true;
  }
  // LDS-staged kernel (STRIPE_TUNE pool_lds = rows per workgroup, 1..8)
  if (const int lds_rows = tune_int("pool_lds", 0); lds_rows >= 1 && lds_rows <= 8 && row_offsets_fit && lds_patch_bytes(s, lds_rows) <= 64 * 1024) {
    const PoolParams p = make_params(s, lds_rows, 128);
    const int64_t grid = (int64_t)p.N * p.y_strips * p.blocks_per_row;
    if (grid > 0x7fffffffLL) return false;
    l->variant = kLdsVariant + 3 * window + mode;
    l->rows = lds_rows;
    l->yb = lds_rows;
    l->wg = 128;
    l->grid = grid;
    info->path = STRIPE_PATH_POOL;
    info->tile_m = lds_rows;
    info->tile_n = 128;
    info->tile_k = 0;
    info->frag_m = info->frag_n = info->frag_k = 0;
    info->lds_bytes = (int)lds_patch_bytes(s, lds_rows);
    info->workgroup_size = 128 * lds_rows;
    info->grid = grid;
    snprintf(info->kernel, sizeof info->kernel, "pool_%s_f32_%dx%ds%d_lds%d", mode == 2 ? "sum" : mode == 1 ? "min" : "max", kWindows[window].r,
             kWindows[window].s, kWindows[window].stride, lds_rows);
    return true;
  }
  if (window != 0 || mode != 0) {
    if (!row_offsets_fit) return false;
    const StripShape shape = choose_strip_shape(s, {1, 2, 3, 4}, {1, 2, 4});
    const int rows = shape.ty;
    const PoolParams p = make_params(s, rows, 128);
    if ((int64_t)p.N * p.y_strips > 0x7fffffffLL) return false;
    l->yb = shape.yb;
    const int64_t grid = strip_grid(p, shape.yb);
    l->variant = kShapeVariant + 3 * window + mode;
    l->rows = rows;
    l->wg = 128;
    l->grid = grid;
    info->path = STRIPE_PATH_POOL;
    info->tile_m = rows;
    info->tile_n = 128;
    info->tile_k = 0;
    info->frag_m = info->frag_n = info->frag_k = 0;
    info->lds_bytes = 0;
    info->workgroup_size = 128 * shape.yb;
    info->grid = grid;
    snprintf(info->kernel, sizeof info->kernel, "pool_%s_f32_%dx%ds%d_ty%d%s", mode == 2 ? "sum" : mode == 1 ? "min" : "max", kWindows[window].r,
             kWindows[window].s, kWindows[window].stride, rows, shape.yb == 4 ? "x4" : shape.yb == 2 ? "x2" : "");
    return true;
  }
  if (tune_int("pool_roll", 0) && row_offsets_fit) {
    int rows = tune_int("pool_roll_rows", 7);
    if (rows < 1) rows = 1;
    if (rows > s.Ho) rows = (int)s.Ho;
    // workgroup size: the multiple of 64 (at most 512) that pads a row of items least; larger wins ties
    const int64_t items = s.Wo * (s.C / 4);
    int wg = tune_int("pool_roll_wg", 0);
    if (wg < 64 || wg > 512 || wg % 64) {
      int64_t best = -1;
      for (int cand = 512; cand >= 64; cand -= 64) {
        const int64_t padded = (items + cand - 1) / cand * cand;
        if (best < 0 || padded < best) best = padded, wg = cand;
      }
    }
    const PoolParams p = make_params(s, rows, wg);
    const int64_t grid = (int64_t)p.N * p.y_strips * p.blocks_per_row;
    if (grid > 0x7fffffffLL) return false;
    l->variant = kRollVariant;
    l->rows = rows;
    l->wg = wg;
    l->grid = grid;
    info->path = STRIPE_PATH_POOL;
    info->tile_m = rows;
    info->tile_n = wg;
    info->tile_k = 0;
    info->frag_m = info->frag_n = info->frag_k = 0;
    info->lds_bytes = 0;
    info->workgroup_size = wg;
    info->grid = grid;
    snprintf(info->kernel, sizeof info->kernel, "pool_max_f32_3x3s2_roll%d_wg%d", rows, wg);
    return true;
  }
  int ty_idx = 1;
  const bool lean_ok = row_offsets_fit && !tune_int("pool_nt", 0) && tune_int("pool_lean", 1);
  const StripShape shape = lean_ok ? choose_strip_shape(s, {1, 2, 3, 4, 7}, {1, 2, 4}) : choose_strip_shape(s, {1, 2, 3, 4, 7}, {1});
  const int chosen = shape.ty;
  l->yb = shape.yb;
  for (int i = 0; i < (int)(sizeof kTyChoices / sizeof kTyChoices[0]); ++i)
    if (kTyChoices[i] == chosen) ty_idx = i;
  const int nt = tune_int("pool_nt", 0) ? 1 : 0;
  const int ty = kTyChoices[ty_idx];
  const PoolParams p = make_params(s, ty, 128);
  if ((int64_t)p.N * p.y_strips * p.blocks_per_row > 0x7fffffffLL) return false;
  const bool lean = row_offsets_fit && !nt && tune_int("pool_lean", 1);
  const int64_t grid = lean ? strip_grid(p, shape.yb) : (int64_t)p.N * p.y_strips * p.blocks_per_row;
  l->variant = ty_idx * 2 + nt;
  l->lean = lean;
  l->rows = ty;
  l->wg = 128;
  l->grid = grid;
  info->path = STRIPE_PATH_POOL;
  info->tile_m = ty;          // output rows per strip
  info->tile_n = 128;         // (column, channel-quad) items per workgroup
  info->tile_k = 0;
  info->frag_m = info->frag_n = info->frag_k = 0;
  info->lds_bytes = 0;
  info->workgroup_size = lean ? 128 * shape.yb : 128;
  info->grid = grid;
  snprintf(info->kernel, sizeof info->kernel, "pool_max_f32_3x3s2_ty%d%s%s", ty, nt ? "_nt" : l->lean ? "" : "_sel",
           !lean ? "" : shape.yb == 4 ? "x4" : shape.yb == 2 ? "x2" : "");
  return true;
}

hipError_t launch_pool(const Pool2dShape& s, const PoolLaunch& l, const void* in, const void* weights, void* out, hipStream_t st) {
  if (((uintptr_t)in % 16) || ((uintptr_t)out % 16)) return hipErrorInvalidValue;
  if (l.variant >= kLdsVariant) {
    const PoolParams p = make_params(s, l.rows, 128);
    const dim3 g((unsigned)l.grid);
    const float* i = (const float*)in;
    float* o = (float*)out;
    const int lds = (int)lds_patch_bytes(s, l.rows);
    switch (l.variant - kLdsVariant) {
      case 0: return launch_lds_rows<3, 3, 2, 0>(l.rows, lds, p, g, i, o, st);
      case 1: return launch_lds_rows<3, 3, 2, 1>(l.rows, lds, p, g, i, o, st);
      case 2: return launch_lds_rows<3, 3, 2, 2>(l.rows, lds, p, g, i, o, st);
      case 3: return launch_lds_rows<2, 2, 2, 0>(l.rows, lds, p, g, i, o, st);
      case 4: return launch_lds_rows<2, 2, 2, 1>(l.rows, lds, p, g, i, o, st);
      case 5: return launch_lds_rows<2, 2, 2, 2>(l.rows, lds, p, g, i, o, st);
      case 6: return launch_lds_rows<3, 3, 1, 0>(l.rows, lds, p, g, i, o, st);
      case 7: return launch_lds_rows<3, 3, 1, 1>(l.rows, lds, p, g, i, o, st);
      case 8: return launch_lds_rows<3, 3, 1, 2>(l.rows, lds, p, g, i, o, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (l.variant >= kWeightedVariant) {
    if (!weights || ((uintptr_t)weights % (s.w_mode == 2 ? 16 : 4))) return hipErrorInvalidValue;
    const PoolParams p = make_params(s, l.rows, 128);
    const dim3 g((unsigned)l.grid);
    const float *i = (const float*)in, *w = (const float*)weights;
    float* o = (float*)out;
    switch (l.variant - kWeightedVariant) {
      // a scaled sum is the strip kernel's sum with one factor; per-tap weights have a kernel of their own
      case 0: return tune_int("pool_scaled_strip", 1) ? launch_strip_rows<3, 3, 2, 2>(l.rows, l.yb, p, g, i, o, st, w) : launch_weighted_rows<3, 3, 2, 1>(l.rows, l.yb, p, g, i, w, o, st);
      case 1: return launch_weighted_rows<3, 3, 2, 2>(l.rows, l.yb, p, g, i, w, o, st);
      case 2: return tune_int("pool_scaled_strip", 1) ? launch_strip_rows<2, 2, 2, 2>(l.rows, l.yb, p, g, i, o, st, w) : launch_weighted_rows<2, 2, 2, 1>(l.rows, l.yb, p, g, i, w, o, st);
      case 3: return launch_weighted_rows<2, 2, 2, 2>(l.rows, l.yb, p, g, i, w, o, st);
      case 4: return tune_int("pool_scaled_strip", 1) ? launch_strip_rows<3, 3, 1, 2>(l.rows, l.yb, p, g, i, o, st, w) : launch_weighted_rows<3, 3, 1, 1>(l.rows, l.yb, p, g, i, w, o, st);
      case 5: return launch_weighted_rows<3, 3, 1, 2>(l.rows, l.yb, p, g, i, w, o, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (l.variant >= kShapeVariant) {
    const PoolParams p = make_params(s, l.rows, 128);
    const dim3 g((unsigned)l.grid);
    const float* i = (const float*)in;
    float* o = (float*)out;
    switch (l.variant - kShapeVariant) {
      case 1: return launch_strip_rows<3, 3, 2, 1>(l.rows, l.yb, p, g, i, o, st);
      case 2: return launch_strip_rows<3, 3, 2, 2>(l.rows, l.yb, p, g, i, o, st);
      case 3: return launch_strip_rows<2, 2, 2, 0>(l.rows, l.yb, p, g, i, o, st);
      case 4: return launch_strip_rows<2, 2, 2, 1>(l.rows, l.yb, p, g, i, o, st);
      case 5: return launch_strip_rows<2, 2, 2, 2>(l.rows, l.yb, p, g, i, o, st);
      case 6: return launch_strip_rows<3, 3, 1, 0>(l.rows, l.yb, p, g, i, o, st);
      case 7: return launch_strip_rows<3, 3, 1, 1>(l.rows, l.yb, p, g, i, o, st);
      case 8: return launch_strip_rows<3, 3, 1, 2>(l.rows, l.yb, p, g, i, o, st);
      default: return hipErrorInvalidValue;
    }
  }
  if (l.variant == kRollVariant) {
    const PoolParams p = make_params(s, l.rows, l.wg);
    hipLaunchKernelGGL(pool_max_f32_roll_kernel, dim3((unsigned)l.grid), dim3(l.wg), 0, st, p, (const float*)in, (float*)out);
    return hipGetLastError();
  }
  const int ty_idx = l.variant / 2;
  const bool nt = l.variant % 2;
  const PoolParams p = make_params(s, kTyChoices[ty_idx], 128);
  switch (ty_idx) {
    case 0: return nt ? launch_ty<1, true>(p, l.grid, in, out, st, l.lean, l.yb) : launch_ty<1, false>(p, l.grid, in, out, st, l.lean, l.yb);
    case 1: return nt ? launch_ty<2, true>(p, l.grid, in, out, st, l.lean, l.yb) : launch_ty<2, false>(p, l.grid, in, out, st, l.lean, l.yb);
    case 2: return nt ? launch_ty<3, true>(p, l.grid, in, out, st, l.lean, l.yb) : launch_ty<3, false>(p, l.grid, in, out, st, l.lean, l.yb);
    case 3: return nt ? launch_ty<4, true>(p, l.grid, in, out, st, l.lean, l.yb) : launch_ty<4, false>(p, l.grid, in, out, st, l.lean, l.yb);
    default: return nt ? launch_ty<7, true>(p, l.grid, in, out, st, l.lean, l.yb) : launch_ty<7, false>(p, l.grid, in, out, st, l.lean, l.yb);
  }
}

}  // namespace stripe
