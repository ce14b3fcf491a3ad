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
//   outer block  -> one workgroup per strip of 7 output rows of one image,
//   middle block -> the strip's 9 input rows (with halo) and the whole
//                   3x3x64x64 filter in LDS (about 139 KB of 160 KB),
//   inner block  -> 32 x 32 fragments of v_mfma_f32_32x32x16_bf16, 36 K steps
//                   (9 taps x 64 channels) per fragment.
// Both LDS arrays hold 128-byte rows (one pixel or one filter row = 64 channels)
// with the 16-byte chunks XOR-swizzled by (row>>1)&7, so the 16-byte fragment
// reads of 32 consecutive pixels / filter rows are bank-conflict free.
//
// Three kernels, in this order in the file:
//   conv3x3_bf16_kernel     one wavefront per output row (2 x 2 fragments), staged through registers;
//                           the fallback for widths whose buffers leave no room for the second kernel's;
//   conv3x3_bf16_w4_kernel  the default: wavefront = (pixel half, channel half), rows taken in groups so that
//                           pixel fragments are shared between filter rows and finished rows are stored while
//                           others are computed; one or two teams of four wavefronts; staging through registers
//                           or by LDS-direct loads that the first row group meets on the way;
//   conv3x3_bf16_ks_kernel  an alternative with the same footprint: the filter in registers, rows walked from top to
//                           bottom with the image still arriving, the reduction split over two teams.  Measured level
//                           with the row-group kernel, kept selectable (conv_ks=1) and tested.
#include <hip/hip_runtime.h>

#include <type_traits>
#include <utility>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(4))) float f32x4s;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2s;

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

// ---------------------------------------------------------------------------
// Row-group kernel: the same LDS images (filter + haloed strip of 7 output
// rows), but the strip's 7 x 2 x 2 output fragments are divided so that every
// SIMD carries the same number of matrix instructions: a wavefront owns one
// pixel half and one channel half (one 32 x 32 fragment per output row).
// Rows are taken in groups; within a group of n rows, one filter column j and
// one 16-channel K step need the n+2 pixel fragments of the group's input
// rows, read once and used by the three filter rows i (output row r uses
// input row r+i), plus 3 filter fragments, for 3n matrix instructions.  Reads
// of the next (j, K step) are issued before the matrix instructions of the
// current one.  Staging index arithmetic is 32-bit with a reciprocal multiply
// for the division by the patch width: at ~13 us per launch the integer work
// of the staged chunks is not free.
// ---------------------------------------------------------------------------
constexpr int W4_ROWS = 7;

// TEAMS: 1 = four wavefronts, each walks three row groups (3 + 2 + 2 rows); 2 = eight wavefronts, two per SIMD:
// team 0 computes row 0, then rows 1-3, team 1 row 4, then rows 5-6, so that one wavefront's store phase (LDS
// transposition, address arithmetic, stores) runs while the other keeps the SIMD's matrix pipe busy, and the
// first stores leave after a single row's worth of matrix work.
// Source of the halo: lanes whose pixel lies outside the image fetch these 16 zero bytes instead.
__device__ __attribute__((aligned(16))) unsigned char conv_zero_chunk[16];

// LDS-direct 16-byte load: lane i of the wavefront lands at lds_off + 16*i (M0 carries the wave-uniform offset).
// Written as assembly so that the compiler does not drain the load queue before unrelated LDS reads; the waits
// are placed by hand (s_waitcnt vmcnt) where the data is first needed.
// M0 is written here and nowhere else: these kernels index no register array dynamically and use no other
// instruction that reads M0, so the compiler (which treats M0 as reserved and ignores the clobber) keeps no value in it.
__device__ __forceinline__ void c_load_lds16(const void* src, unsigned lds_off) {
  const unsigned uniform_off = __builtin_amdgcn_readfirstlane(lds_off);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(uniform_off) : "memory", "m0");
}

// DMA (needs TEAMS == 2): the strip's rows and the filter go global -> LDS with LDS-direct loads instead of
// through registers, the filter in three slices ordered by filter column j.  The first row group of each team
// starts as soon as the rows and the first slice have landed and meets the other two slices on the way, so the
// first stores leave earlier; no LDS-store instructions and no staging registers are spent.
//
// EPI: what happens to a finished accumulator on its way out.  0: stored as it is.  1 and 2: the fused form of
// a following statement O = relu(T + bias[k]) whose temporary T is this block's output (Section 2.3, fusion and
// scalarisation: T never exists in memory, it lives in the accumulators): bias added, relu applied, stored as
// fp32 (1) or rounded to bf16 (2).  `O` then points at that statement's output buffer.
template <int TEAMS, bool DMA = false, int EPI = 0>
__global__ __launch_bounds__(256 * TEAMS, 1) void conv3x3_bf16_w4_kernel(const ConvParams p, const uint16_t* __restrict__ I,
                                                                        const uint16_t* __restrict__ F, void* __restrict__ O,
                                                                        const float* __restrict__ bias) {
  static_assert(!DMA || TEAMS == 2, "the LDS-direct staging is written for eight wavefronts");
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* lf = lds;
  unsigned char* lp = lds + C_FILTER_BYTES;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int n = blockIdx.x / p.strips_per_image;
  const int y0 = (blockIdx.x - n * p.strips_per_image) * W4_ROWS;
  const int PW = p.W + 2;
  constexpr int PR = W4_ROWS + 2;
  // bytes of the patch image rounded up to whole 1 KB load blocks (DMA); the output transposition buffers follow
  const int patch_bytes = DMA ? ((PR * PW * 128 + 1023) & ~1023) : PR * PW * 128;
  // The fused epilogue's bias values are fetched first, so that they are the oldest entries of the load queue: the
  // hand-placed s_waitcnt of the LDS-direct staging below count the younger loads still in flight.
  f32x4s bias4 = {0.f, 0.f, 0.f, 0.f};               // store phase, fp32 form: the lane's four channels
  f32x4s bias8a = {0.f, 0.f, 0.f, 0.f}, bias8b = {0.f, 0.f, 0.f, 0.f};   // bf16 form: the lane's eight channels
  if constexpr (EPI == 1 || (EPI == 2 && TEAMS != 2)) bias4 = *(const f32x4s*)(bias + (wave & 1) * 32 + (lane & 7) * 4);
  if constexpr (EPI == 2 && TEAMS == 2) {
    bias8a = *(const f32x4s*)(bias + (wave & 1) * 32 + (lane & 3) * 8);
    bias8b = *(const f32x4s*)(bias + (wave & 1) * 32 + (lane & 3) * 8 + 4);
  }
  if constexpr (DMA) {
    // ---- staging by LDS-direct loads: 9 patch blocks, then 3 filter blocks per slice, per wavefront (18 loads)
    const int sub = lane >> 3, slot = lane & 7;
    const char* ig = (const char*)(I + p.i_base + (int64_t)n * p.i_n);
    const int n_blocks = patch_bytes >> 10;
#pragma unroll
    for (int e = 0; e < 9; ++e) {
      const int b = wave + 8 * e;                     // block b = LDS pixels 8b .. 8b+7
      const int pix = b * 8 + sub;
      const int r = (int)__umulhi((unsigned)pix, (unsigned)p.pad_), col = pix - r * PW;   // pad_ carries ceil(2^32 / PW)
      const int y = y0 - 1 + r, x = col - 1;
      const int c = slot ^ ((pix >> 1) & 7);
      const bool inside = r < PR && y >= 0 && y < p.H && x >= 0 && x < p.W;
      const void* src = inside ? (const void*)(ig + (uint32_t)(y * (int)p.i_y + x * (int)p.i_x + c * 8) * 2u) : (const void*)conv_zero_chunk;
      // blocks past the patch (a wavefront issues 9 loads whatever the width, so that the wait counts are the same
      // for all) land in the output transposition area, which nothing reads before it is rewritten
      const unsigned dst = C_FILTER_BYTES + (b < n_blocks ? b * 1024 : patch_bytes + wave * 1024);
      c_load_lds16(b < n_blocks ? src : (const void*)conv_zero_chunk, dst);
    }
    const char* fgb = (const char*)(F + p.f_base);
#pragma unroll
    for (int tj = 0; tj < 3; ++tj)
#pragma unroll
      for (int ti = 0; ti < 3; ++ti) {
        const int row = (ti * 3 + tj) * C_CO + wave * 8 + sub;     // filter row (tap, k)
        const int c = slot ^ ((row >> 1) & 7);
        c_load_lds16(fgb + (row * C_CI + c * 8) * 2, ((ti * 3 + tj) * C_CO + wave * 8) * 128);
      }
    asm volatile("s_waitcnt vmcnt(6)" ::: "memory");   // the wavefront's patch blocks and its share of slice 0
    __syncthreads();
  } else {

  // ---- staging.  Every global load of the lane is in flight before the first LDS store.
  // A lane keeps its 16-byte chunk index c = t&7 and walks pixels: filter rows (t>>3) + 32u (its LDS swizzle
  // key does not depend on u), patch columns (t>>3) + 32*pass of every patch row.  Rows are uniform, so a row's
  // base address is scalar and the loads add one per-lane byte offset; halo pixels and rows outside the image
  // are loaded from a clamped address and replaced by zeros.
  constexpr int NT = 256 * TEAMS;
  constexpr int W4_FQ = C_TAPS * C_CO * 8 / NT;   // filter chunks per lane
  constexpr int PPR = 2 / TEAMS;                  // passes over a patch row: the host admits only (W+2)*8 <= 512
  const int c = t & 7, px = t >> 3;
  const u32x4* fg = (const u32x4*)(F + p.f_base) + t;
  u32x4 fv[W4_FQ], pv[PR][PPR];
#pragma unroll
  for (int u = 0; u < W4_FQ; ++u) fv[u] = fg[u * NT];
  const char* ig = (const char*)(I + p.i_base + (int64_t)n * p.i_n);
  uint32_t goff[PPR];
  bool cvalid[PPR], cwrite[PPR];
#pragma unroll
  for (int k = 0; k < PPR; ++k) {
    const int col = px + (NT / 8) * k, x = col - 1;
    cvalid[k] = x >= 0 && x < p.W;
    cwrite[k] = col < PW;
    const int xc = x < 0 ? 0 : (x >= p.W ? p.W - 1 : x);
    goff[k] = (uint32_t)(xc * (int)p.i_x + c * 8) * 2u;
  }
#pragma unroll
  for (int r = 0; r < PR; ++r) {
    const int y = y0 - 1 + r;
    const int yc = y < 0 ? 0 : (y >= p.H ? p.H - 1 : y);
    const char* rp = ig + (int64_t)yc * p.i_y * 2;
#pragma unroll
    for (int k = 0; k < PPR; ++k) pv[r][k] = *(const u32x4*)(rp + goff[k]);
  }
  {
    unsigned char* dst = lf + px * 128 + ((c ^ ((px >> 1) & 7)) << 4);
#pragma unroll
    for (int u = 0; u < W4_FQ; ++u) *(u32x4*)(dst + u * (NT * 16)) = fv[u];
  }
#pragma unroll
  for (int r = 0; r < PR; ++r) {
    const int y = y0 - 1 + r;
    const bool rvalid = y >= 0 && y < p.H;
#pragma unroll
    for (int k = 0; k < PPR; ++k) {
      const int pix = r * PW + px + (NT / 8) * k;
      const u32x4 zero = {0u, 0u, 0u, 0u};
      const u32x4 v = (rvalid && cvalid[k]) ? pv[r][k] : zero;
      if (cwrite[k]) *(u32x4*)(lp + pix * 128 + (swz(pix, c) << 4)) = v;
    }
  }
  __syncthreads();
  }

  // ---- compute: wavefront = (pixel half mh, channel half nh), 7 rows
  const int team = wave >> 2, mh = (wave >> 1) & 1, nh = wave & 1;
  const int fr = lane & 31, fh = lane >> 5;
  const int xcl = mh * 32 + fr < p.W ? mh * 32 + fr : p.W - 1;   // columns beyond W are computed on a clamped pixel, never stored
  // LDS byte address of a fragment chunk = base ^ (K step << 5): the swizzle key only touches bits 4..6
  const unsigned b_base = (unsigned)((nh * 32 + fr) * 128 + ((fh ^ ((fr >> 1) & 7)) << 4));

  // store phase geometry.  Accumulator element v of lane l is pixel 8*(v/4) + 4*(l>>5) + v%4 of its 32-pixel
  // fragment, channel l&31 of the wavefront's 32.  Each fragment goes through a 4 KB buffer of the wavefront
  // ([pixel][32 channels], behind the patch) and leaves as 16-byte stores: 8 lanes write the 128 contiguous
  // bytes of a pixel's channel half.
  constexpr int OT_BYTES = 4096 / TEAMS;             // a fragment leaves in TEAMS rounds of 32 / TEAMS pixels
  unsigned char* ot = lp + patch_bytes + wave * OT_BYTES;
  const int sp = lane >> 3, sc = lane & 7;          // store phase: pixel sp (+8j) of the fragment, channel quad sc
  constexpr int OB = EPI == 2 ? 2 : 4;               // bytes per output element
  char* og = (char*)O + (p.o_base + (int64_t)n * p.o_n + nh * 32 + sc * 4) * OB;
  unsigned char* wbase[4];     // write address of accumulator elements v = 0..3 (pixel 4*fh + v); + 1 KB per further 8 pixels
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int pixel = 4 * fh + v;
    wbase[v] = ot + pixel * 128 + ((((fr >> 2) ^ pixel) << 4) | ((fr & 3) << 2));   // 16-byte slot = channel quad ^ (pixel & 7)
  }
  uint32_t ooff[4];          // pixel sp + 8j of the fragment
  bool ovalid[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int x = mh * 32 + sp + 8 * j;
    ovalid[j] = x < p.W;
    ooff[j] = (uint32_t)((x < p.W ? x : 0) * (int)p.o_x) * (unsigned)OB;
  }
  // bf16 output: a pixel's 32 channels are 64 bytes, so four lanes (eight channels, 16 bytes each) cover a pixel and
  // one store instruction covers the 16 pixels of a round -- half as many store instructions as the fp32 form
  const int sp2 = lane >> 2, sc2 = lane & 3;
  char* og2 = (char*)O + (p.o_base + (int64_t)n * p.o_n + nh * 32 + sc2 * 8) * 2;
  uint32_t ooff2[2] = {0u, 0u};
  bool ovalid2[2] = {false, false};
  if constexpr (EPI == 2 && TEAMS == 2) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const int x = mh * 32 + 16 * h + sp2;
      ovalid2[h] = x < p.W;
      ooff2[h] = (uint32_t)((x < p.W ? x : 0) * (int)p.o_x) * 2u;
    }
  }

  // Output rows are finished in three groups (3 + 2 + 2 rows) rather than all at the end, so that the stores
  // of a group drain to memory while the next group is being computed.  Within a group of n rows, one filter
  // column j and one 16-channel K step need the n+2 pixel fragments of the group's input rows (read once, used
  // by the three filter rows i: output row r takes input row r+i) and 3 filter fragments for 3n matrix
  // instructions; the fragments of the next (j, K step) are requested before the current ones are consumed.
  auto row_group = [&](auto r0_tag, auto n_tag, auto first_tag) {
    constexpr int R0 = decltype(r0_tag)::value, NR = decltype(n_tag)::value;
    constexpr bool MEET_SLICES = DMA && decltype(first_tag)::value;   // first group of a team under DMA staging
    f32x16 acc[NR];
#pragma unroll
    for (int r = 0; r < NR; ++r)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[r][v] = 0.f;
    bf16x8 a[2][NR + 2], b[2][3];
    unsigned a_base[NR + 2];
    auto set_bases = [&](int tj) {
#pragma unroll
      for (int r = 0; r < NR + 2; ++r) {
        const int pix = (R0 + r) * PW + xcl + tj;
        a_base[r] = (unsigned)(pix * 128 + ((fh ^ ((pix >> 1) & 7)) << 4));
      }
    };
    auto read_frags = [&](int buf, int tj, int s) {   // tj, s: compile-time after unrolling
#pragma unroll
      for (int r = 0; r < NR + 2; ++r) a[buf][r] = *(const bf16x8*)(lp + (a_base[r] ^ (unsigned)(s << 5)));
#pragma unroll
      for (int ti = 0; ti < 3; ++ti)
        b[buf][ti] = *(const bf16x8*)(lf + (ti * 3 + tj) * (C_CO * 128) + (b_base ^ (unsigned)(s << 5)));
    };
    set_bases(0);
    read_frags(0, 0, 0);
#pragma unroll
    for (int it = 0; it < 12; ++it) {       // it = tj * 4 + s
      const int cur = it & 1;
      __builtin_amdgcn_sched_barrier(0);
      if (it + 1 < 12) {
        if (((it + 1) & 3) == 0) {
          if constexpr (MEET_SLICES) {   // the next filter column's slice: this wavefront's share, then everybody's
            if (it + 1 == 4) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");
            else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
            __syncthreads();
          }
          set_bases((it + 1) >> 2);
        }
        read_frags(cur ^ 1, (it + 1) >> 2, (it + 1) & 3);
      }
#pragma unroll
      for (int ti = 0; ti < 3; ++ti)
#pragma unroll
        for (int r = 0; r < NR; ++r)
          acc[r] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[cur][r + ti], b[cur][ti], acc[r], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int r = 0; r < NR; ++r) {
      const int y = y0 + R0 + r;
      if (y < p.H) {                                   // uniform
        char* orow = og + (int64_t)y * p.o_y * OB;
#pragma unroll
        for (int h = 0; h < TEAMS; ++h) {
          constexpr int G = 4 / TEAMS;               // groups of 8 pixels per round
#pragma unroll
          for (int v = h * 4 * G; v < (h + 1) * 4 * G; ++v) *(float*)(wbase[v % 4] + (v / 4 - h * G) * 1024) = acc[r][v];
          __builtin_amdgcn_wave_barrier();
          if constexpr (EPI == 2 && TEAMS == 2) {
            // round h holds pixels 16h .. 16h+15 of the fragment: lane = (pixel sp2, channels 8*sc2 .. +7)
            f32x4s va = *(const f32x4s*)(ot + sp2 * 128 + (((2 * sc2) ^ (sp2 & 7)) << 4));
            f32x4s vb = *(const f32x4s*)(ot + sp2 * 128 + (((2 * sc2 + 1) ^ (sp2 & 7)) << 4));
            va.x = __builtin_fmaxf(va.x + bias8a.x, 0.f);
            va.y = __builtin_fmaxf(va.y + bias8a.y, 0.f);
            va.z = __builtin_fmaxf(va.z + bias8a.z, 0.f);
            va.w = __builtin_fmaxf(va.w + bias8a.w, 0.f);
            vb.x = __builtin_fmaxf(vb.x + bias8b.x, 0.f);
            vb.y = __builtin_fmaxf(vb.y + bias8b.y, 0.f);
            vb.z = __builtin_fmaxf(vb.z + bias8b.z, 0.f);
            vb.w = __builtin_fmaxf(vb.w + bias8b.w, 0.f);
            typedef float f32x2d __attribute__((ext_vector_type(2)));
            typedef __bf16 bf16x2d __attribute__((ext_vector_type(2)));
            const bf16x2d q0 = __builtin_convertvector((f32x2d){va.x, va.y}, bf16x2d), q1 = __builtin_convertvector((f32x2d){va.z, va.w}, bf16x2d);
            const bf16x2d q2 = __builtin_convertvector((f32x2d){vb.x, vb.y}, bf16x2d), q3 = __builtin_convertvector((f32x2d){vb.z, vb.w}, bf16x2d);
            const u32x4 packed = {__builtin_bit_cast(unsigned, q0), __builtin_bit_cast(unsigned, q1), __builtin_bit_cast(unsigned, q2),
                                  __builtin_bit_cast(unsigned, q3)};
            char* orow2 = og2 + (int64_t)y * p.o_y * 2;
            if (ovalid2[h]) __builtin_nontemporal_store(packed, (u32x4*)(orow2 + ooff2[h]));
          } else
#pragma unroll
          for (int j = 0; j < G; ++j) {
            const int pixel = sp + 8 * j;            // within the round; (pixel & 7) == sp either way
            f32x4s v = *(const f32x4s*)(ot + pixel * 128 + ((sc ^ (pixel & 7)) << 4));
            if constexpr (EPI != 0) {
              v.x = __builtin_fmaxf(v.x + bias4.x, 0.f);   // relu; a NaN becomes 0
              v.y = __builtin_fmaxf(v.y + bias4.y, 0.f);
              v.z = __builtin_fmaxf(v.z + bias4.z, 0.f);
              v.w = __builtin_fmaxf(v.w + bias4.w, 0.f);
            }
            if constexpr (EPI == 2) {
              // fp32 -> bf16, round to nearest even, two values per conversion instruction
              typedef float f32x2c __attribute__((ext_vector_type(2)));
              typedef __bf16 bf16x2c __attribute__((ext_vector_type(2)));
              const bf16x2c lo = __builtin_convertvector((f32x2c){v.x, v.y}, bf16x2c), hi = __builtin_convertvector((f32x2c){v.z, v.w}, bf16x2c);
              u32x2s packed = {__builtin_bit_cast(unsigned, lo), __builtin_bit_cast(unsigned, hi)};
              // (a wavefront holds 32 of a pixel's 64 channels, i.e. half a 128-byte line of bf16; plain stores that
              // leave the merging of the halves to L2 were measured slower than these streaming half-line stores)
              if (ovalid[h * G + j]) __builtin_nontemporal_store(packed, (u32x2s*)(orow + ooff[h * G + j]));
            } else {
              if (ovalid[h * G + j]) __builtin_nontemporal_store(v, (f32x4s*)(orow + ooff[h * G + j]));
            }
          }
          __builtin_amdgcn_wave_barrier();
        }
      }
    }
  };
  constexpr std::true_type first{};
  constexpr std::false_type later{};
  if constexpr (TEAMS == 1) {
    row_group(std::integral_constant<int, 0>{}, std::integral_constant<int, 3>{}, first);
    row_group(std::integral_constant<int, 3>{}, std::integral_constant<int, 2>{}, later);
    row_group(std::integral_constant<int, 5>{}, std::integral_constant<int, 2>{}, later);
  } else if (team == 0) {   // a single row first: the sooner the first stores leave, the sooner the write stream starts
    row_group(std::integral_constant<int, 0>{}, std::integral_constant<int, 1>{}, first);
    row_group(std::integral_constant<int, 1>{}, std::integral_constant<int, 3>{}, later);
  } else {
    row_group(std::integral_constant<int, 4>{}, std::integral_constant<int, 1>{}, first);
    row_group(std::integral_constant<int, 5>{}, std::integral_constant<int, 2>{}, later);
  }
}

template <int... Is, class Fn>
__device__ __forceinline__ void conv_static_for(std::integer_sequence<int, Is...>, Fn&& fn) {
  (fn(std::integral_constant<int, Is>{}), ...);
}

// ---------------------------------------------------------------------------
// Rolling rows with the reduction split over two teams.  Wavefront = (team,
// pixel half, channel half); a team takes one half of the 64 input channels,
// so a wavefront keeps 18 filter fragments (9 taps x 2 K steps) in registers,
// walks ALL nine input rows of the strip from top to bottom and holds partial
// sums of its 32 pixels x 32 channels.  Every wavefront executes the same
// instruction stream, which makes three kinds of overlap a matter of placing
// instructions in that stream (it is unrolled at compile time):
//   * image rows are requested (LDS-direct) a few rows ahead of their use,
//     the later ones from inside the compute phase, so the matrix cores start
//     once the filter and the first row have landed instead of after the
//     whole patch;
//   * a finished output row is handed over one input row later: each
//     wavefront keeps the partial sums of half of the fragment's pixels and
//     passes the other half to its partner team through LDS (two 16-byte
//     writes per lane, in the accumulator's own lane layout);
//   * one input row after that it adds the partner's half to its own and
//     stores: in the accumulator layout 32 lanes hold the 32 channels of one
//     pixel, i.e. one whole 128-byte line per pixel and store instruction.
// One workgroup barrier per input row orders all of this (arrival of rows,
// hand-over buffers), two buffers per wavefront alternate between rows.
// ---------------------------------------------------------------------------
template <int EPI>
__global__ __launch_bounds__(512, 1) void conv3x3_bf16_ks_kernel(const ConvParams p, const uint16_t* __restrict__ I,
                                                                 const uint16_t* __restrict__ F, void* __restrict__ O,
                                                                 const float* __restrict__ bias) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  unsigned char* lf = lds;                          // the filter image; afterwards the hand-over buffers
  unsigned char* lp = lds + C_FILTER_BYTES;         // the patch
  const int t = threadIdx.x, lane = t & 63, wave = __builtin_amdgcn_readfirstlane(t >> 6);

  const int n = blockIdx.x / p.strips_per_image;
  const int y0 = (blockIdx.x - n * p.strips_per_image) * W4_ROWS;
  const int PW = p.W + 2;
  constexpr int PR = W4_ROWS + 2;
  const int patch_bytes = (PR * PW * 128 + 1023) & ~1023;
  const int kh = wave >> 2, mh = (wave >> 1) & 1, nh = wave & 1;
  const int fr = lane & 31, fh = lane >> 5;
  // the bias values first: the oldest entries of the load queue, the hand-placed waits below count younger loads
  f32x4s bias4 = {0.f, 0.f, 0.f, 0.f}, bias4b = {0.f, 0.f, 0.f, 0.f};
  if constexpr (EPI == 1) bias4 = *(const f32x4s*)(bias + nh * 32 + (lane & 7) * 4);
  if constexpr (EPI == 2) {
    bias4 = *(const f32x4s*)(bias + nh * 32 + (lane & 3) * 8);
    bias4b = *(const f32x4s*)(bias + nh * 32 + (lane & 3) * 8 + 4);
  }

  // ---- staging by LDS-direct loads: 9 filter blocks per wavefront, then the patch in 9 blocks per wavefront;
  // block e of a wavefront covers LDS pixels 8 (wave + 8e) .. +7, so input row q lies within blocks e <= q
  const int sub = lane >> 3, slot = lane & 7;
  const char* ig = (const char*)(I + p.i_base + (int64_t)n * p.i_n);
  const int n_blocks = patch_bytes >> 10;
  auto load_patch = [&](int e) {
    const int b = wave + 8 * e;
    const int pix = b * 8 + sub;
    const int r = (int)__umulhi((unsigned)pix, (unsigned)p.pad_), col = pix - r * PW;   // pad_ carries ceil(2^32 / PW)
    const int y = y0 - 1 + r, x = col - 1;
    const int c = slot ^ ((pix >> 1) & 7);
    const bool inside = r < PR && y >= 0 && y < p.H && x >= 0 && x < p.W;
    const void* src = inside ? (const void*)(ig + (uint32_t)(y * (int)p.i_y + x * (int)p.i_x + c * 8) * 2u) : (const void*)conv_zero_chunk;
    // a wavefront issues nine loads whatever the width (the waits count them); blocks past the patch land behind it
    const unsigned dst = C_FILTER_BYTES + (b < n_blocks ? b * 1024 : patch_bytes + wave * 1024);
    c_load_lds16(b < n_blocks ? src : (const void*)conv_zero_chunk, dst);
  };
  {
    const char* fgb = (const char*)(F + p.f_base);
#pragma unroll
    for (int tap = 0; tap < C_TAPS; ++tap) {
      const int row = tap * C_CO + wave * 8 + sub;     // filter row (tap, k)
      const int c = slot ^ ((row >> 1) & 7);
      c_load_lds16(fgb + (row * C_CI + c * 8) * 2, (tap * C_CO + wave * 8) * 128);
    }
    load_patch(0);
    load_patch(1);
    load_patch(2);
    asm volatile("s_waitcnt vmcnt(3)" ::: "memory");   // this wavefront's filter blocks
    __syncthreads();                                    // everybody's
  }

  // ---- the filter fragments of this channel half and K half, LDS -> registers
  bf16x8 b[C_TAPS][2];
  {
    const unsigned b_base = (unsigned)((nh * 32 + fr) * 128 + ((fh ^ ((fr >> 1) & 7)) << 4)) ^ (unsigned)(kh << 6);
#pragma unroll
    for (int tap = 0; tap < C_TAPS; ++tap)
#pragma unroll
      for (int s = 0; s < 2; ++s) b[tap][s] = *(const bf16x8*)(lf + tap * (C_CO * 128) + (b_base ^ (unsigned)(s << 5)));
  }
  load_patch(3);
  asm volatile("s_waitcnt vmcnt(3)" ::: "memory");     // block 0 of this wavefront: input row 0
  __syncthreads();

  const int xcl = mh * 32 + fr < p.W ? mh * 32 + fr : p.W - 1;   // columns beyond W are computed on a clamped pixel, never stored
  // hand-over buffers: 2 per wavefront, 4 KB each = one fragment as [pixel][32 channels], 16-byte slots swizzled by
  // the pixel.  Accumulator element v of lane l is pixel 8*(v/4) + 4*(l>>5) + v%4 of the fragment, channel l&31.
  unsigned char* const outbox = lf + wave * 8192;
  const unsigned char* const inbox = lf + (wave ^ 4) * 8192;
  unsigned wofs[4];            // element v goes to wofs[v % 4] + 1024 * (v / 4)
#pragma unroll
  for (int v = 0; v < 4; ++v) {
    const int pixel = 4 * fh + v;
    wofs[v] = (unsigned)(pixel * 128 + ((((fr >> 2) ^ pixel) << 4) | ((fr & 3) << 2)));
  }
  // a team finishes half of the fragment's pixels.  fp32 output: pixels 16 kh + 8 j + sp for j = 0, 1 with lane =
  // (pixel sp, channel quad sc), 16 bytes per lane.  bf16 output: a pixel's 32 channels are 64 bytes, so lane =
  // (pixel sp of 16, eight channels sc): two 16-byte slots per buffer in, 16 bytes out, one store for the 16 pixels.
  const int sp = EPI == 2 ? lane >> 2 : lane >> 3, sc = EPI == 2 ? lane & 3 : lane & 7;
  const unsigned rofs = EPI == 2 ? (unsigned)((16 * kh + sp) * 128 + (((2 * sc) ^ (sp & 7)) << 4))
                                 : (unsigned)((16 * kh + sp) * 128 + ((sc ^ sp) << 4));     // + 1024 j
  const unsigned rofs_b = (unsigned)((16 * kh + sp) * 128 + (((2 * sc + 1) ^ (sp & 7)) << 4));   // bf16: the second slot
  const int xs = mh * 32 + 16 * kh + sp;                                                  // + 8 j
  constexpr int OB = EPI == 2 ? 2 : 4;
  char* const og = (char*)O + (p.o_base + (int64_t)n * p.o_n + nh * 32 + sc * (EPI == 2 ? 8 : 4) + (int64_t)xs * p.o_x) * OB;

  constexpr int STEPS = PR * 6;                       // step = q * 6 + tj * 2 + s
  f32x16 acc[4];                                      // output row r accumulates in acc[r & 3]
  bf16x8 a[3];                                        // pixel fragments, requested two steps ahead
  auto read_a = [&](int step) -> bf16x8 {             // step: a constant at every call
    const int q = step / 6, tj = (step % 6) >> 1, s = step & 1;
    const int pix = q * PW + xcl + tj;
    const unsigned base = (unsigned)(pix * 128 + ((fh ^ ((pix >> 1) & 7)) << 4)) ^ (unsigned)(kh << 6);
    return *(const bf16x8*)(lp + (base ^ (unsigned)(s << 5)));
  };
  // hand-over of output row r (its partial sums are complete): the whole fragment into this wavefront's buffer
  auto hand_over = [&](auto r_tag) {
    constexpr int r = decltype(r_tag)::value;
#pragma unroll
    for (int v = 0; v < 16; ++v) *(float*)(outbox + (r & 1) * 4096 + wofs[v % 4] + (v / 4) * 1024) = acc[r & 3][v];
  };
  // both teams' partial sums of this team's pixels: fetched in one step, added, finished and stored (16 bytes per
  // lane, a pixel's 128 bytes per 8 lanes) in the next, so that the LDS latency passes behind matrix instructions
  f32x4s mine[2], theirs[2];
  auto fetch_row = [&](auto r_tag) {
    constexpr int r = decltype(r_tag)::value;
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const unsigned o = (r & 1) * 4096 + (EPI == 2 ? (j ? rofs_b : rofs) : rofs + j * 1024);
      mine[j] = *(const f32x4s*)(outbox + o);
      theirs[j] = *(const f32x4s*)(inbox + o);
    }
  };
  auto finish_row = [&](auto r_tag) {
    constexpr int r = decltype(r_tag)::value;
    const int y = y0 + r;
    f32x4s v[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      v[j] = (f32x4s){mine[j].x + theirs[j].x, mine[j].y + theirs[j].y, mine[j].z + theirs[j].z, mine[j].w + theirs[j].w};
      if constexpr (EPI != 0) {
        const f32x4s bj = (EPI == 2 && j == 1) ? bias4b : bias4;
        v[j].x = __builtin_fmaxf(v[j].x + bj.x, 0.f);   // relu; a NaN becomes 0
        v[j].y = __builtin_fmaxf(v[j].y + bj.y, 0.f);
        v[j].z = __builtin_fmaxf(v[j].z + bj.z, 0.f);
        v[j].w = __builtin_fmaxf(v[j].w + bj.w, 0.f);
      }
    }
    char* orow = og + (int64_t)y * p.o_y * OB;
    if constexpr (EPI == 2) {
      // fp32 -> bf16, round to nearest even, two values per conversion instruction
      typedef float f32x2c __attribute__((ext_vector_type(2)));
      typedef __bf16 bf16x2c __attribute__((ext_vector_type(2)));
      const bf16x2c q0 = __builtin_convertvector((f32x2c){v[0].x, v[0].y}, bf16x2c), q1 = __builtin_convertvector((f32x2c){v[0].z, v[0].w}, bf16x2c);
      const bf16x2c q2 = __builtin_convertvector((f32x2c){v[1].x, v[1].y}, bf16x2c), q3 = __builtin_convertvector((f32x2c){v[1].z, v[1].w}, bf16x2c);
      const u32x4 packed = {__builtin_bit_cast(unsigned, q0), __builtin_bit_cast(unsigned, q1), __builtin_bit_cast(unsigned, q2),
                            __builtin_bit_cast(unsigned, q3)};
      if (y < p.H && xs < p.W) __builtin_nontemporal_store(packed, (u32x4*)orow);
    } else {
#pragma unroll
      for (int j = 0; j < 2; ++j)
        if (y < p.H && xs + 8 * j < p.W) __builtin_nontemporal_store(v[j], (f32x4s*)(orow + (int64_t)(8 * j) * p.o_x * OB));
    }
  };
  const f32x16 zero16 = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};

  // The two teams' wavefronts share SIMDs pairwise (wavefront w and w + 4), and a wavefront issues in order: while
  // it hands a row over or stores one it feeds no matrix instructions.  The teams therefore do these chores at
  // different steps of an input row (team 0 early, team 1 late), so that one of the two always has matrix work.
  auto run = [&](auto team_tag) {
    constexpr int TEAM = decltype(team_tag)::value;
    constexpr int K_FETCH = TEAM ? 2 : 0, K_FINISH = TEAM ? 5 : 1, K_HAND = TEAM ? 3 : 2;
    a[0] = read_a(0);
    a[1] = read_a(1);
    conv_static_for(std::make_integer_sequence<int, STEPS>{}, [&](auto step_tag) {
      constexpr int step = decltype(step_tag)::value;
      constexpr int q = step / 6, k = step % 6, tj = k >> 1, s = k & 1;
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (k == 4) {
        // the next input row must have landed (everybody's blocks), the hand-over buffers change roles
        if constexpr (q == 0) asm volatile("s_waitcnt vmcnt(3)" ::: "memory");   // blocks 2, 3, 4 may be in flight
        if constexpr (q == 1) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");   // blocks 3 .. 6
        if constexpr (q == 2) asm volatile("s_waitcnt vmcnt(5)" ::: "memory");   // blocks 4 .. 8
        if constexpr (q == 3) asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // all of them, before the first store is issued
        __syncthreads();
      }
      if constexpr (step + 2 < STEPS) a[(step + 2) % 3] = read_a(step + 2);
      if constexpr (q - 2 >= 0 && q - 2 < W4_ROWS) acc[(q - 2) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[step % 3], b[6 + tj][s], acc[(q - 2) & 3], 0, 0, 0);
      if constexpr (q - 1 >= 0 && q - 1 < W4_ROWS) acc[(q - 1) & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[step % 3], b[3 + tj][s], acc[(q - 1) & 3], 0, 0, 0);
      if constexpr (q < W4_ROWS) acc[q & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[step % 3], b[tj][s], k == 0 ? zero16 : acc[q & 3], 0, 0, 0);
      // the later patch blocks, requested from inside the compute phase
      if constexpr (q == 0 && k == 1) load_patch(4);
      if constexpr (q == 1 && k == 1) load_patch(5);
      if constexpr (q == 1 && k == 2) load_patch(6);
      if constexpr (q == 2 && k == 1) load_patch(7);
      if constexpr (q == 2 && k == 2) load_patch(8);
      // output row q-4 was handed over during the previous input row (a barrier ago)
      if constexpr (k == K_FETCH && q >= 4) fetch_row(std::integral_constant<int, q - 4>{});
      if constexpr (k == K_FINISH && q >= 4) finish_row(std::integral_constant<int, q - 4>{});
      // output row q-3 met its last input row (q-1) in the previous six steps; handed over before this row's barrier
      if constexpr (k == K_HAND && q >= 3) hand_over(std::integral_constant<int, q - 3>{});
      __builtin_amdgcn_sched_barrier(0);
    });
    // the last rows: 5 was handed over during input row 8; 6 is complete only now
    fetch_row(std::integral_constant<int, 5>{});
    hand_over(std::integral_constant<int, 6>{});
    finish_row(std::integral_constant<int, 5>{});
    __syncthreads();
    fetch_row(std::integral_constant<int, 6>{});
    finish_row(std::integral_constant<int, 6>{});
  };
  if (kh == 0) run(std::integral_constant<int, 0>{});
  else run(std::integral_constant<int, 1>{});
}

constexpr int W4_LDS_EXTRA = 4 * 4096;   // per-wavefront output transposition buffers

constexpr int kConvW4Variant = 200;

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

static bool conv3x3_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info);

// The tuned kernels for their shapes (3x3 over 64 channels, 7x7 stride 2 over 3 channels), the general kernel otherwise.
bool conv_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info) {
  if (tune_int("conv_mfma", 1) == 0) return false;
  l->in_dtype = in_dtype;
  const bool tuned = tune_int("conv_tuned", 1) != 0;   // 0: measure the general kernel on the tuned kernels' shapes
  if (tuned && in_dtype == STRIPE_I8 && conv_i8_select(c, in_dtype, l, info)) return true;
  if (tuned && in_dtype == STRIPE_BF16 && conv3x3_select(c, in_dtype, l, info)) return true;
  if (conv_gemm_select(c, in_dtype, l, info)) return true;
  return conv_igemm_select(c, in_dtype, false, l, info);
}

// A dense product C[m][n] = sum_k A[m][k] * B[n][k] with at most 64 columns would leave three quarters of the
// contraction kernels' 256-wide tiles (half of the 128-wide ones) to padding.  Seen as a 1 x 1 convolution -- rows of
// A are the pixels, K the input channels, N the output channels -- it fits the general convolution kernel's
// 256 x 64 tile exactly.  Fills *c and picks that kernel, or returns false (then the contraction kernels take it).
bool conv_select_narrow_product(const GemmShape& g, int in_dtype, Conv2dShape* c, ConvLaunch* l, stripe_block_info_t* info) {
  if (tune_int("gemm_narrow_conv", 1) == 0 || tune_int("conv_mfma", 1) == 0) return false;
  if (g.batch != 1 || g.N > 64 || g.M < 64 * 256) return false;   // at least 64 tiles: shorter products keep the contraction kernels and their split reduction
  if (g.a_k != 1 || g.b_k != 1 || g.c_n != 1) return false;   // K contiguous in both operands, N contiguous in the output
  Conv2dShape s = {};
  s.N = 1; s.Ho = 1; s.Wo = g.M; s.H = 1; s.W = g.M; s.Co = g.N; s.Ci = g.K; s.R = 1; s.S = 1;
  s.stride_y = s.stride_x = 1; s.pad_y = s.pad_x = 0; s.dil_y = s.dil_x = 1;
  s.i_n = 0; s.i_y = 0; s.i_x = g.a_m; s.i_c = 1;
  s.f_r = 0; s.f_s = 0; s.f_k = g.b_n; s.f_c = 1;
  s.o_n = 0; s.o_y = 0; s.o_x = g.c_m; s.o_k = 1;
  s.i_base = g.a_base; s.f_base = g.b_base; s.o_base = g.c_base;
  l->in_dtype = in_dtype;
  if (!conv_igemm_select(s, in_dtype, false, l, info)) return false;
  *c = s;
  return true;
}

static bool conv3x3_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info) {
  if (in_dtype != STRIPE_BF16) return false;
  if (c.dil_y != 1 || c.dil_x != 1) return false;
  if (c.R != 3 || c.S != 3 || c.stride_y != 1 || c.stride_x != 1 || c.pad_y != 1 || c.pad_x != 1) return false;
  if (c.Ci != C_CI || c.Co != C_CO || c.Ho != c.H || c.Wo != c.W) return false;
  if (c.W > 64 || c.W < 1) return false;
  // channels contiguous; filter laid out [tap][k][c] contiguously; 16-byte global loads
  if (c.i_c != 1 || c.f_c != 1 || c.o_k != 1) return false;
  if (c.f_k != C_CI || c.f_s != C_CO * C_CI || c.f_r != 3 * C_CO * C_CI) return false;
  for (int64_t v : {c.i_n, c.i_y, c.i_x, c.i_base, c.f_base})
    if (v % 8) return false;
  for (int64_t v : {c.o_n, c.o_y, c.o_x, c.o_base})   // 16-byte stores
    if (v % 4) return false;
  // four-wavefront kernel: strips of 7 rows, 32-bit element offsets inside an image
  const bool offsets_fit = c.i_y >= 0 && c.i_x >= 0 && c.o_x >= 0 && (c.H * c.i_y + c.W * c.i_x + 64) < ((int64_t)1 << 30) &&
                           (c.W * c.o_x + 64) < ((int64_t)1 << 30);
  int w4_lds = C_FILTER_BYTES + (W4_ROWS + 2) * ((int)c.W + 2) * 128 + W4_LDS_EXTRA;
  const int w4_teams = tune_int("conv_w4_teams", 2) == 1 ? 1 : 2;
  const bool w4_dma = w4_teams == 2 && tune_int("conv_dma", 1) != 0;
  if (w4_dma) w4_lds = C_FILTER_BYTES + (((W4_ROWS + 2) * ((int)c.W + 2) * 128 + 1023) & ~1023) + W4_LDS_EXTRA;
  if (tune_int("conv_w4", 1) && offsets_fit && w4_lds <= 160 * 1024 && (c.W + 2) * 8 <= 512) {
    const int64_t grid = c.N * ((c.Ho + W4_ROWS - 1) / W4_ROWS);
    if (grid > 0x7fffffffLL) return false;
    // 1: the rolling-row kernel whose teams split the reduction (measured level with the row-group kernel)
    const bool ks = w4_dma && tune_int("conv_ks", 0) != 0;
    l->variant = kConvW4Variant + (ks ? 4 : w4_dma ? 3 : w4_teams);
    l->grid = grid;
    info->path = STRIPE_PATH_MFMA_CONV;
    info->tile_m = W4_ROWS * (int)c.W;
    info->tile_n = C_CO;
    info->tile_k = C_TAPS * C_CI;
    info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
    info->lds_bytes = w4_lds;
    info->workgroup_size = 256 * w4_teams;
    info->grid = grid;
    snprintf(info->kernel, sizeof info->kernel, "conv3x3_bf16_c64k64_strip7_w%d%s_mfma32x32x16", 4 * w4_teams,
             ks ? "_ksplit" : w4_dma ? "_dma" : "");
    return true;
  }
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

bool conv_can_fuse_bias_relu(const Conv2dShape& c, const ConvLaunch& l) {
  // the fused statement's output shares the layout of the temporary: a dense [n][y][x][k] image
  const bool dense = c.o_x == c.Co && (c.Ho == 1 || c.o_y == c.Wo * c.Co) && (c.N == 1 || c.o_n == c.Ho * c.Wo * c.Co) && c.o_base == 0;
  if (!dense) return false;
  if (l.variant == kConvW4Variant + 3 || l.variant == kConvW4Variant + 4) return true;   // the LDS-direct 3x3 kernels
  if (l.variant >= kConvGemmVariant) return true;   // the contraction kernel's convolution mode: chosen only where every pixel is written
  if (l.variant >= kConvIgemmVariant && l.variant < kConvGemmVariant && l.in_dtype == STRIPE_BF16 && c.Co % 4 == 0) {
    // the general kernel leaves a pixel none of whose taps lies inside the image unwritten: with such a pixel the
    // temporary would hold an undefined element, and the two statements stay apart
    for (int64_t y = 0; y < c.Ho; ++y) {
      bool any = false;
      for (int64_t i = 0; i < c.R && !any; ++i) any = y * c.stride_y - c.pad_y + i * c.dil_y >= 0 && y * c.stride_y - c.pad_y + i * c.dil_y < c.H;
      if (!any) return false;
    }
    for (int64_t x = 0; x < c.Wo; ++x) {
      bool any = false;
      for (int64_t j = 0; j < c.S && !any; ++j) any = x * c.stride_x - c.pad_x + j * c.dil_x >= 0 && x * c.stride_x - c.pad_x + j * c.dil_x < c.W;
      if (!any) return false;
    }
    return true;
  }
  return false;
}

static hipError_t launch_conv_epi(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, const void* bias,
                                  int epi, hipStream_t st);

hipError_t launch_conv_bias_relu(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, const void* bias, void* out,
                                 bool out_bf16, hipStream_t st) {
  if (!conv_can_fuse_bias_relu(c, l) || ((uintptr_t)bias % 16) || ((uintptr_t)out % 16)) return hipErrorInvalidValue;
  return launch_conv_epi(c, l, in, flt, out, bias, out_bf16 ? 2 : 1, st);
}

hipError_t launch_conv(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, hipStream_t st) {
  return launch_conv_epi(c, l, in, flt, out, nullptr, 0, st);
}

static hipError_t launch_conv_epi(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, const void* bias,
                                  int epi, hipStream_t st) {
  if (l.variant >= kConvGemmVariant) return launch_conv_gemm(c, l, in, flt, out, epi ? bias : nullptr, epi, st);
  if (l.variant >= kConvIgemmVariant) return launch_conv_igemm(c, l, l.in_dtype, epi == 2, in, flt, out, epi ? bias : nullptr, st);
  if (l.variant >= 100 && l.variant < kConvW4Variant) return launch_conv_i8(c, l, in, flt, out, st);
  if (((uintptr_t)in % 16) || ((uintptr_t)flt % 16) || ((uintptr_t)out % 16)) return hipErrorInvalidValue;
  if (l.variant > kConvW4Variant) {
    const int mode = l.variant - kConvW4Variant;   // 1: four wavefronts, 2: eight, 3: eight with LDS-direct staging, 4: rolling rows with the reduction split over the teams
    ConvParams pp = make_params(c, W4_ROWS);
    const uint32_t pw = (uint32_t)c.W + 2;
    pp.pad_ = (int32_t)(uint32_t)((((uint64_t)1 << 32) + pw - 1) / pw);   // reciprocal of the patch width, for the LDS-direct staging
    const int patch = (W4_ROWS + 2) * ((int)c.W + 2) * 128;
    const int lds_w4 = C_FILTER_BYTES + (mode >= 3 ? ((patch + 1023) & ~1023) : patch) + W4_LDS_EXTRA;
    typedef void (*kern_t)(const ConvParams, const uint16_t*, const uint16_t*, void*, const float*);
    const kern_t fn = mode == 4 ? (epi == 1 ? (kern_t)conv3x3_bf16_ks_kernel<1> : epi == 2 ? (kern_t)conv3x3_bf16_ks_kernel<2> : (kern_t)conv3x3_bf16_ks_kernel<0>)
                    : (mode == 3 && epi == 1) ? (kern_t)conv3x3_bf16_w4_kernel<2, true, 1>
                    : (mode == 3 && epi == 2) ? (kern_t)conv3x3_bf16_w4_kernel<2, true, 2>
                    : mode == 3 ? (kern_t)conv3x3_bf16_w4_kernel<2, true> : mode == 2 ? (kern_t)conv3x3_bf16_w4_kernel<2, false>
                                                                                      : (kern_t)conv3x3_bf16_w4_kernel<1, false>;
    int dev4 = -1;
    hipError_t e4 = hipGetDevice(&dev4);
    if (e4 != hipSuccess) return e4;
    if (dev4 != l.lds_enabled_on) {
      e4 = hipFuncSetAttribute((const void*)fn, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
      if (e4 != hipSuccess) return e4;
      l.lds_enabled_on = dev4;
    }
    hipLaunchKernelGGL(fn, dim3((unsigned)l.grid), dim3(mode == 1 ? 256 : 512), lds_w4, st, pp, (const uint16_t*)in,
                       (const uint16_t*)flt, out, (const float*)bias);
    return hipGetLastError();
  }
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

