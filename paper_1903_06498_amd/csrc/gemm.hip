// Nested-tile dense contraction on the gfx950 matrix cores:
//   C[m,n] = sum_k A[m,k] * B[k,n],  bf16 inputs, fp32 accumulate and output.
//
// The three nesting levels of the Stripe block (paper Section 3.1.3; Figure 3's
// columns) are mapped by hand:
//   outer block  -> one workgroup per 256 x 256 tile of C (XCD-aware tile order),
//   middle block -> K tiles staged in LDS (ring of 2 or 4 stages),
//   inner block  -> v_mfma_f32_32x32x16_bf16 fragments (v_mfma_i32_32x32x32_i8 in the int8 mode).
// Three kernels, in this order in the file:
//   gemm_bf16_w8_kernel   8 wavefronts, operands staged through registers, B transposed on the way into LDS
//                         (the "microarchitectural transposition" of Section 2.3), K tiles of 64;
//   gemm_bf16_w4_kernel   4 wavefronts of 128 x 128, same staging, deeper software pipeline;
//   gemm_bf16_dma_kernel  the default: LDS-direct loads into a four-stage ring, B kept [k][n] and read with the
//                         transposing LDS read; template modes for a transposed B, ragged M/N and int8.
// All LDS tiles hold K-contiguous rows whose 16-byte chunks are XOR-swizzled with the row number, so fragment
// reads (16 bytes per lane) spread over all banks.
#include <hip/hip_runtime.h>

#include <string>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

struct GemmParams {
  int32_t tiles_m, tiles_n, k_tiles, pad_;
  int32_t M, N;               // used by the variants that accept M, N that are not multiples of the tile
  int64_t a_m, b_k, c_m;      // row strides in elements (a_k = b_n = c_n = 1); for a transposed B ([n][k], k contiguous) b_k holds its row stride
  int64_t a_base, b_base, c_base;
  int64_t a_b, b_b, c_b;      // element distance between two products of a batch (LDS-direct kernel only)
  // Fused following statement O = relu(C + bias[n]) (LDS-direct kernels, float modes): epi 0 = none, 1 = fp32
  // output, 2 = bf16 output; the C pointer and c_m / c_base then describe O.
  const float* bias;
  int32_t epi;
  int32_t vec_c;              // LDS-direct 256-tile kernel: C strides, base and pointer allow one store per row and four columns
  // Convolution mode of the LDS-direct 256-tile kernel (D_CONV): row m of A is output pixel m (flattened n, y, x), the
  // reduction walks filter taps (i, j) and channel chunks of 32; a_base / b_base are the input's and the filter's.
  int32_t cv_Ho, cv_Wo, cv_H, cv_W, cv_sy, cv_sx, cv_py, cv_px, cv_dy, cv_dx, cv_R, cv_S, cv_chunks, cv_pad_;
  int64_t cv_i_n, cv_i_y, cv_i_x, cv_f_r, cv_f_s;   // element strides of the input (image, row, pixel) and of the filter's taps
};

// Fused epilogue of one accumulator value: bias, relu, store as fp32 or bf16 (round to nearest even).
__device__ __forceinline__ void epi_store(const GemmParams& p, float* C, int64_t off, float v, float bias) {
  v = __builtin_fmaxf(v + bias, 0.f);
  if (p.epi == 1) {
    __builtin_nontemporal_store(v, C + off);
  } else {
    const uint32_t u = __float_as_uint(v);
    ((uint16_t*)C)[off] = (uint16_t)((u + 0x7fffu + ((u >> 16) & 1u)) >> 16);
  }
}

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WAVES_M = 2, WAVES_N = 4;            // 8 wavefronts, 512 lanes
constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // 128 x 64 per wavefront
constexpr int FM = WM / 32, FN = WN / 32;          // 4 x 2 fragments of 32 x 32
constexpr int ROW_BYTES = BK * 2;                  // 128
constexpr int A_STAGE = BM * ROW_BYTES;            // 32 KB
constexpr int B_STAGE = BN * ROW_BYTES;            // 32 KB
constexpr int STAGE = A_STAGE + B_STAGE;           // 64 KB, two stages = 128 KB of the 160 KB LDS
constexpr int THREADS = 512;

// Which 16-byte slot of its 128-byte row chunk c of row r lives in.  LDS has 64
// four-byte banks, i.e. two 128-byte rows per bank sweep; a fragment read puts
// 16 consecutive rows of one chunk into one sweep, the B transposition writes
// rows 8 apart.  Keying the swizzle on (row>>1) and (row>>4) separates both.
template <int SWZ>
__device__ __forceinline__ int slot(int row, int c) {
  if (SWZ == 2) return c ^ (((row >> 1) ^ (row >> 4)) & 7);
  return c ^ ((row >> SWZ) & 7);
}

// Tile order: hardware workgroup ids go round-robin over the 8 XCDs; give each
// XCD a contiguous run of logical ids, and make each run of 32 logical ids a
// 4 x 8 patch of C tiles, so the 32 CUs behind one L2 share 4 A panels and 8 B panels.
__device__ __forceinline__ void tile_of(unsigned b, unsigned grid, int tiles_m, int tiles_n, int* tm, int* tn) {
  unsigned l = (grid % 8u) ? b : (b % 8u) * (grid / 8u) + b / 8u;
  if (tiles_m % 4 == 0 && tiles_n % 8 == 0) {
    const unsigned patch = l / 32u, w = l % 32u, per_row = tiles_n / 8;
    *tm = (patch / per_row) * 4 + w / 8u;
    *tn = (patch % per_row) * 8 + w % 8u;
  } else {
    *tm = l / tiles_n;
    *tn = l % tiles_n;
  }
}

template <int SWZ>
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_w8_kernel(const GemmParams p, const uint16_t* __restrict__ A,
                                                               const uint16_t* __restrict__ B, float* __restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  int tm, tn;
  tile_of(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, &tm, &tn);

  // ---- global -> register staging -------------------------------------
  // A tile: 256 rows x 8 chunks of 16 B; lane t takes chunk t&7 of rows (t>>3) + 64*i.
  const int a_c = t & 7, a_r0 = t >> 3;
  const uint16_t* a_g = A + p.a_base + ((int64_t)tm * BM + a_r0) * p.a_m + a_c * 8;
  // B tile: 64 k x 256 n; a lane takes a 4(k) x 8(n) patch.  Within a wavefront 8 lanes
  // step through k quads and 8 through n blocks: global reads are 128-byte row segments
  // and the transposed LDS writes of one instruction spread over all banks.
  const int b_kq = (lane & 7) + 8 * (wave & 1), b_nb = (lane >> 3) + 8 * (wave >> 1);
  const uint16_t* b_g = B + p.b_base + (int64_t)(b_kq * 4) * p.b_k + (int64_t)tn * BN + b_nb * 8;

  u32x4 ra[4], rb[4];
  auto load_tile = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) ra[i] = *(const u32x4*)(a_g + (int64_t)(64 * i) * p.a_m + kt * BK);
#pragma unroll
    for (int i = 0; i < 4; ++i) rb[i] = *(const u32x4*)(b_g + ((int64_t)kt * BK + i) * p.b_k);
  };
  auto store_tile = [&](int stage) {
    unsigned char* la = lds + stage * STAGE;
    unsigned char* lb = la + A_STAGE;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = a_r0 + 64 * i;
      *(u32x4*)(la + row * ROW_BYTES + (slot<SWZ>(row, a_c) << 4)) = ra[i];
    }
    // transpose the 4(k) x 8(n) patch: dword d of rb[i] holds n = 2d (low half) and 2d+1 (high half) at k = i
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      u32x2 even, odd;
      even.x = (rb[0][d] & 0xffffu) | (rb[1][d] << 16);
      even.y = (rb[2][d] & 0xffffu) | (rb[3][d] << 16);
      odd.x = (rb[0][d] >> 16) | (rb[1][d] & 0xffff0000u);
      odd.y = (rb[2][d] >> 16) | (rb[3][d] & 0xffff0000u);
      const int n0 = b_nb * 8 + 2 * d;
      const int kc = b_kq >> 1, half = (b_kq & 1) * 8;
      *(u32x2*)(lb + n0 * ROW_BYTES + (slot<SWZ>(n0, kc) << 4) + half) = even;
      *(u32x2*)(lb + (n0 + 1) * ROW_BYTES + (slot<SWZ>(n0 + 1, kc) << 4) + half) = odd;
    }
  };

  // ---- LDS -> fragment addressing ---------------------------------------
  // Fragment operand layout of the 32x32x16 instruction: lane l supplies row
  // (l & 31) of the 32-row operand and the 8 consecutive k values 8*(l >> 5)..+7.
  const int fr = lane & 31, fh = lane >> 5;
  const int a_row0 = wm * WM + fr;   // + 32*i ; (row >> SWZ) & 7 does not change with i
  const int b_row0 = wn * WN + fr;

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  load_tile(0);
  store_tile(0);
  __syncthreads();

  for (int kt = 0; kt < p.k_tiles; ++kt) {
    const int cur = kt & 1;
    const bool more = kt + 1 < p.k_tiles;
    if (more) load_tile(kt + 1);
    const unsigned char* la = lds + cur * STAGE;
    const unsigned char* lb = la + A_STAGE;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      bf16x8 af[FM], bf[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i) {
        const int row = a_row0 + 32 * i;
        af[i] = *(const bf16x8*)(la + row * ROW_BYTES + (slot<SWZ>(row, 2 * s + fh) << 4));
      }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int row = b_row0 + 32 * j;
        bf[j] = *(const bf16x8*)(lb + row * ROW_BYTES + (slot<SWZ>(row, 2 * s + fh) << 4));
      }
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
    }
    if (more) store_tile(cur ^ 1);
    __syncthreads();
  }

  // ---- epilogue: accumulator element v of lane l is row 8*(v/4) + 4*(l>>5) + v%4, column l&31
  float* c_g = C + p.c_base + ((int64_t)tm * BM + wm * WM + 4 * fh) * p.c_m + (int64_t)tn * BN + wn * WN + fr;
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = 32 * i + 8 * (v / 4) + (v % 4);
        __builtin_nontemporal_store(acc[i][j][v], c_g + (int64_t)r * p.c_m + 32 * j);
      }
}

// ---------------------------------------------------------------------------
// Four-wavefront variant: 2 x 2 wavefronts of 128 x 128 (4 x 4 fragments, 256
// accumulator registers, one wavefront per SIMD).  Per 16 matrix instructions a
// wavefront reads 8 fragments from LDS instead of 12, which is what keeps the
// LDS pipe below saturation.  With a single wavefront per SIMD nothing hides a
// stall, so the K loop is software-pipelined by hand:
//   * global -> register loads run two K tiles ahead (two staging sets),
//   * the register -> LDS stores of the next tile are spread over K steps 0..2,
//   * one barrier before K step 3, after which the first fragments of the next
//     tile are read while step 3's matrix instructions run,
//   * fragments are double-buffered across K steps.
// ---------------------------------------------------------------------------
constexpr int W4_THREADS = 256;

#define SGB(mask, n) __builtin_amdgcn_sched_group_barrier(mask, n, 0)
constexpr int SG_MFMA = 0x008, SG_VMEM_RD = 0x020, SG_DS_RD = 0x100, SG_DS_WR = 0x200, SG_VALU = 0x002;

// LDS map of the four-wavefront kernel: [A stage 0 | A stage 1 | B stage 0 | B stage 1],
// 32 KB each, so that a stage toggle and a 32-row fragment step are immediate
// offsets of the LDS instruction.  Swizzle key (row>>1)&7: it does not change
// when 32 or 64 is added to the row, so one address register serves all
// fragments (and one all store rows) of an operand.
constexpr int W4_A0 = 0, W4_B0 = 2 * A_STAGE, W4_STAGE = A_STAGE;  // B_STAGE == A_STAGE

struct W4Ctx {
  const uint16_t* a_panel;   // uniform: first element of this workgroup's 256-row panel of A
  const uint16_t* b_panel;   // uniform: first element of this workgroup's 256-column panel of B
  unsigned a_off, b_off;     // per-lane element offsets into the panels
  unsigned a_rowstep, b_rowstep;  // uniform: 32 rows of A, 1 row of B, in elements
  unsigned a_st, b_st;       // per-lane LDS byte address of the lane's first store slot (stage 0; b_st includes W4_B0)
  unsigned a_fr, b_fr;       // per-lane LDS byte address of the lane's first fragment chunk (stage 0, K step 0; b_fr includes W4_B0)
};

__device__ __forceinline__ void w4_load_tile(const W4Ctx& c, int kt, unsigned b_kstep, u32x4 (&ga)[8], u32x4 (&gb)[8]) {
  const uint16_t* ap = c.a_panel + kt * BK;
  const uint16_t* bp = c.b_panel + (size_t)kt * b_kstep;
#pragma unroll
  for (int i = 0; i < 8; ++i) ga[i] = *(const u32x4*)((ap + (size_t)i * c.a_rowstep) + c.a_off);  // uniform base + lane offset
#pragma unroll
  for (int i = 0; i < 8; ++i) gb[i] = *(const u32x4*)((bp + (size_t)i * c.b_rowstep) + c.b_off);
}

template <int STAGE_N, int I0, int I1>
__device__ __forceinline__ void w4_store_a(const W4Ctx& c, unsigned char* lds, const u32x4 (&ga)[8]) {
#pragma unroll
  for (int i = I0; i < I1; ++i) *(u32x4*)(lds + c.a_st + (W4_A0 + STAGE_N * W4_STAGE + i * 32 * ROW_BYTES)) = ga[i];
}

// transpose column pair d of the 8(k) x 8(n) patch: dword d of gb[i] holds n = 2d (low) and 2d+1 (high) at k = i.
// Rows 2d and 2d+1 of the patch have swizzle key (key of row 0) ^ d.
template <int STAGE_N, int D0, int D1>
__device__ __forceinline__ void w4_store_b(const W4Ctx& c, unsigned char* lds, const u32x4 (&gb)[8]) {
#pragma unroll
  for (int d = D0; d < D1; ++d) {
    u32x4 even, odd;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      even[j] = (gb[2 * j][d] & 0xffffu) | (gb[2 * j + 1][d] << 16);
      odd[j] = (gb[2 * j][d] >> 16) | (gb[2 * j + 1][d] & 0xffff0000u);
    }
    const unsigned at = (c.b_st ^ (d << 4)) + (STAGE_N * W4_STAGE + 2 * d * ROW_BYTES);   // b_st already holds W4_B0
    *(u32x4*)(lds + at) = even;
    *(u32x4*)(lds + at + ROW_BYTES) = odd;
  }
}

template <int STAGE_N, int S>
__device__ __forceinline__ void w4_read_frags(const W4Ctx& c, const unsigned char* lds, bf16x8 (&af)[4], bf16x8 (&bf)[4]) {
  const unsigned a = c.a_fr ^ (S << 5), b = c.b_fr ^ (S << 5);   // chunk 2*S + half: flips slot bits 1..2
#pragma unroll
  for (int i = 0; i < 4; ++i) af[i] = *(const bf16x8*)(lds + a + (W4_A0 + STAGE_N * W4_STAGE + i * 32 * ROW_BYTES));
#pragma unroll
  for (int j = 0; j < 4; ++j) bf[j] = *(const bf16x8*)(lds + b + (STAGE_N * W4_STAGE + j * 32 * ROW_BYTES));   // b_fr already holds W4_B0
}

__device__ __forceinline__ void w4_mfma16(const bf16x8 (&af)[4], const bf16x8 (&bf)[4], f32x16 (&acc)[4][4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bf[j], acc[i][j], 0, 0, 0);
}

// One K tile.  CUR = LDS stage holding this tile; gl_* = staging set loaded now
// (tile kt+2), gs_* = staging set stored now (tile kt+1, loaded one iteration ago).
template <int CUR, bool HAVE_NEXT, bool HAVE_NEXT2>
__device__ __forceinline__ void w4_iteration(const W4Ctx& c, unsigned char* lds, int kt, unsigned b_kstep,
                                             u32x4 (&gl_a)[8], u32x4 (&gl_b)[8], u32x4 (&gs_a)[8], u32x4 (&gs_b)[8],
                                             bf16x8 (&af)[2][4], bf16x8 (&bf)[2][4], f32x16 (&acc)[4][4]) {
  constexpr int NXT = CUR ^ 1;
  constexpr bool have_next = HAVE_NEXT, have_next2 = HAVE_NEXT2;

  // ---- K step 0: fragments of step 1, loads of tile kt+2, A stores of tile kt+1
  w4_read_frags<CUR, 1>(c, lds, af[1], bf[1]);
  if (have_next2) w4_load_tile(c, kt + 2, b_kstep, gl_a, gl_b);
  w4_mfma16(af[0], bf[0], acc);
  if (have_next) w4_store_a<NXT, 0, 8>(c, lds, gs_a);
#pragma unroll
  for (int r = 0; r < 8; ++r) { SGB(SG_MFMA, 1); SGB(SG_DS_RD, 1); SGB(SG_VMEM_RD, 2); }
#pragma unroll
  for (int r = 0; r < 8; ++r) { SGB(SG_MFMA, 1); SGB(SG_DS_WR, 1); }

  // ---- K step 1: fragments of step 2, B stores (column pairs 0, 1)
  w4_read_frags<CUR, 2>(c, lds, af[0], bf[0]);
  w4_mfma16(af[1], bf[1], acc);
  if (have_next) w4_store_b<NXT, 0, 2>(c, lds, gs_b);
#pragma unroll
  for (int r = 0; r < 8; ++r) { SGB(SG_MFMA, 1); SGB(SG_DS_RD, 1); }
#pragma unroll
  for (int r = 0; r < 4; ++r) { SGB(SG_MFMA, 2); SGB(SG_VALU, 4); SGB(SG_DS_WR, 1); }

  // ---- K step 2: fragments of step 3, B stores (column pairs 2, 3)
  w4_read_frags<CUR, 3>(c, lds, af[1], bf[1]);
  w4_mfma16(af[0], bf[0], acc);
  if (have_next) w4_store_b<NXT, 2, 4>(c, lds, gs_b);
#pragma unroll
  for (int r = 0; r < 8; ++r) { SGB(SG_MFMA, 1); SGB(SG_DS_RD, 1); }
#pragma unroll
  for (int r = 0; r < 4; ++r) { SGB(SG_MFMA, 2); SGB(SG_VALU, 4); SGB(SG_DS_WR, 1); }

  // ---- the next tile is complete in LDS once every wavefront has passed here
  __syncthreads();

  // ---- K step 3: first fragments of the next tile
  if (have_next) w4_read_frags<NXT, 0>(c, lds, af[0], bf[0]);
  w4_mfma16(af[1], bf[1], acc);
#pragma unroll
  for (int r = 0; r < 8; ++r) { SGB(SG_MFMA, 1); SGB(SG_DS_RD, 1); }
  SGB(SG_MFMA, 8);
}

__global__ __launch_bounds__(W4_THREADS, 1) void gemm_bf16_w4_kernel(const GemmParams p, const uint16_t* __restrict__ A,
                                                                     const uint16_t* __restrict__ B, float* __restrict__ C) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  int tm, tn;
  tile_of(blockIdx.x, gridDim.x, p.tiles_m, p.tiles_n, &tm, &tn);

  W4Ctx c;
  // A tile: 256 rows x 8 chunks of 16 B; lane t takes chunk t&7 of rows (t>>3) + 32*i.
  const int a_c = t & 7, a_r0 = t >> 3;
  c.a_panel = A + p.a_base + (int64_t)tm * BM * p.a_m;
  c.a_off = (unsigned)(a_r0 * p.a_m) + a_c * 8;
  c.a_rowstep = (unsigned)(32 * p.a_m);
  c.a_st = a_r0 * ROW_BYTES + ((a_c ^ ((a_r0 >> 1) & 7)) << 4);
  // B tile: 64 k x 256 n; a lane takes the 8(k) x 8(n) patch at k = 8*(lane&7), n = 8*((lane>>3) + 8*wave):
  // global reads are 128-byte row segments, transposed rows are whole 16-byte chunks.
  const int b_kq = lane & 7, b_nb = (lane >> 3) + 8 * wave;
  c.b_panel = B + p.b_base + (int64_t)tn * BN;
  c.b_off = (unsigned)(b_kq * 8 * p.b_k) + b_nb * 8;
  c.b_rowstep = (unsigned)p.b_k;
  c.b_st = W4_B0 + b_nb * 8 * ROW_BYTES + ((b_kq ^ ((b_nb * 4) & 7)) << 4);
  const unsigned b_kstep = (unsigned)(BK * p.b_k);
  // fragments: lane l supplies row (l & 31) and the 8 k values of chunk 2*s + (l >> 5)
  const int fr = lane & 31, fh = lane >> 5;
  c.a_fr = (wm * 128 + fr) * ROW_BYTES + ((fh ^ ((fr >> 1) & 7)) << 4);
  c.b_fr = W4_B0 + (wn * 128 + fr) * ROW_BYTES + ((fh ^ ((fr >> 1) & 7)) << 4);

  u32x4 ga[2][8], gb[2][8];
  bf16x8 af[2][4], bf[2][4];
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // prologue: tile 0 -> LDS stage 0, tile 1 -> staging set 1, first fragments
  w4_load_tile(c, 0, b_kstep, ga[0], gb[0]);
  w4_load_tile(c, 1, b_kstep, ga[1], gb[1]);
  w4_store_a<0, 0, 8>(c, lds, ga[0]);
  w4_store_b<0, 0, 4>(c, lds, gb[0]);
  __syncthreads();
  w4_read_frags<0, 0>(c, lds, af[0], bf[0]);

  // k_tiles is even and >= 2 (checked on the host).  The steady-state loop has no
  // conditions in its body; the last two tiles run as a peeled tail.
  const int last2 = p.k_tiles - 2;
  for (int kt = 0; kt < last2; kt += 2) {
    w4_iteration<0, true, true>(c, lds, kt, b_kstep, ga[0], gb[0], ga[1], gb[1], af, bf, acc);
    w4_iteration<1, true, true>(c, lds, kt + 1, b_kstep, ga[1], gb[1], ga[0], gb[0], af, bf, acc);
  }
  w4_iteration<0, true, false>(c, lds, last2, b_kstep, ga[0], gb[0], ga[1], gb[1], af, bf, acc);
  w4_iteration<1, false, false>(c, lds, last2 + 1, b_kstep, ga[1], gb[1], ga[0], gb[0], af, bf, acc);

  // epilogue: accumulator element v of lane l is row 8*(v/4) + 4*(l>>5) + v%4, column l&31
  float* c_g = C + p.c_base + ((int64_t)tm * BM + wm * 128 + 4 * fh) * p.c_m + (int64_t)tn * BN + wn * 128 + fr;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = 32 * i + 8 * (v / 4) + (v % 4);
        __builtin_nontemporal_store(acc[i][j][v], c_g + (int64_t)r * p.c_m + 32 * j);
      }
}

// ---------------------------------------------------------------------------
// Direct-to-LDS variant (the gfx950 way): both operands go global -> LDS with
// 16-byte-per-lane LDS-direct loads, no staging registers and no LDS store
// instructions; A fragments are read with 16-byte LDS reads, B fragments --
// B is stored as it lies in memory, [k][n] -- with the transposing 8-byte LDS
// read, two per fragment.  K tiles of 32 in a four-stage LDS ring: loads run
// three tiles ahead of the matrix instructions.
//
// LDS map: A stages at 0, 16 KB each (256 rows x 64 B, chunk c of row r in slot
// c ^ ((r>>2)&3)); B stages at 64 KB, 16 KB each (32 k rows x 512 B, chunk c of
// row k in slot c ^ (4*(k&3))).  An LDS-direct load writes 1 KB per wavefront,
// lane i at +16*i, so the swizzle is applied by choosing which global chunk a
// lane fetches.
//
// Transposing read (measured lane layout): within 16 lanes, lane p supplies the
// address of 4 consecutive 16-bit values; lane i receives, for j = 0..3, value
// (i & 3) of the address given by lane (i >> 2) + 4*j.  Lane p = q + 4*j
// therefore points at B[k0 + j][n0 + 4*q .. +3] and lane i gets column n0 + i
// at k0..k0+3.
// ---------------------------------------------------------------------------
constexpr int D_BK = 32, D_STAGES = 4, D_A_STAGE = BM * D_BK * 2, D_B_STAGE = D_BK * BN * 2;
constexpr int D_B0 = D_STAGES * D_A_STAGE;                     // 64 KB
constexpr int D_LDS = D_STAGES * (D_A_STAGE + D_B_STAGE);      // 128 KB
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;

// Convolution mode: lanes whose tap lies outside the image fetch these 16 zero bytes instead.
__device__ __attribute__((aligned(16))) uint16_t d_zero_chunk[8];

struct DCtx {
  const uint16_t* a_src;   // per-lane global address of the lane's first A chunk (tile 0, load 0)
  const uint16_t* b_src;   // per-lane global address of the lane's first B chunk (tile 0, load 0)
  size_t a_step, b_step;   // element distance between two of the lane's loads within a tile
  size_t b_kstep;          // element distance of one K tile in B
  unsigned a_fr;           // LDS byte address of the lane's A fragment chunk (stage 0, K step 0, fragment 0)
  unsigned b_fr[4];        // LDS byte address of the lane's B fragment j (stage 0, K step 0, first read)
  unsigned wave_lds;       // LDS byte offset of this wavefront's 1 KB load slot within a stage
  const uint16_t* a_ptr[4];  // ragged variants: the lane's load addresses one by one (rows clamped into the matrix)
  const uint16_t* b_ptr[4];
  unsigned rmask[4], cmask[4];   // convolution mode: which filter rows / columns of the load's pixel lie inside the image
  const uint16_t* zero;          // convolution mode: 16 zero bytes, fetched for taps outside the image
};

// Convolution mode: the K tile the next issue fetches -- filter tap (ti, tj), channel chunk tc -- and its element
// offsets in the image and in the filter, advanced by additions (all wave-uniform).
struct DWalk {
  int ti, tj, tc;
  int64_t a_off, b_off;
  int64_t a_col, a_row, b_col, b_row;   // what a step to the next filter column / row adds (the chunk walk undone)
  int S, chunks;
  __device__ __forceinline__ void advance() {
    if (++tc == chunks) {
      tc = 0;
      if (++tj == S) {
        tj = 0;
        ++ti;
        a_off += a_row;
        b_off += b_row;
      } else {
        a_off += a_col;
        b_off += b_col;
      }
    } else {
      a_off += D_BK;
      b_off += D_BK;
    }
  }
};

// MODE bit 0: B is stored transposed, [n][k] with k contiguous (C = A * B^T as Linear layers and 1x1 convolutions
// have it); its tile then lies in LDS exactly like A's and a fragment is one 16-byte read.
// MODE bit 1: M and N need not be multiples of 256: loads of rows (or column chunks) past the edge are redirected
// to the last valid one -- they only feed accumulators that are never stored -- and the stores are predicated.
// MODE bit 2: the operands are int8 with int32 accumulation (v_mfma_i32_32x32x32_i8).  Only the matrix instruction
// changes: a tile row is 64 bytes either way (64 int8 or 32 bf16 values), a fragment chunk is 16 bytes either way,
// and the 32 x 32 result layout is the same, so the host hands the int8 matrices over as 16-bit matrices of half
// the width (strides and bases in 2-byte units) and the accumulators are kept as bit patterns in the same registers.
// Needs D_BT: with k contiguous in both operands no transposition of bytes is required.
constexpr int D_BT = 1, D_RAGGED = 2, D_I8 = 4, D_CONV = 8;   // D_CONV: see GemmParams; needs D_BT and D_RAGGED
typedef __attribute__((ext_vector_type(4))) int d_i32x4;
typedef __attribute__((ext_vector_type(16))) int d_i32x16;

template <int MODE>
__device__ __forceinline__ f32x16 d_mma(bf16x8 a, bf16x8 b, f32x16 acc) {
  if constexpr (MODE & D_I8) {
    return __builtin_bit_cast(f32x16, __builtin_amdgcn_mfma_i32_32x32x32_i8(__builtin_bit_cast(d_i32x4, a), __builtin_bit_cast(d_i32x4, b),
                                                                           __builtin_bit_cast(d_i32x16, acc), 0, 0, 0));
  } else {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc, 0, 0, 0);
  }
}

// The LDS-direct loads are written as assembly on purpose: the compiler cannot
// tell that a load into one ring stage does not alias the fragment reads of
// another and would drain the whole load queue before every LDS read.  Here the
// queue depth is managed by hand with the s_waitcnt in d_tile().  M0 carries
// the wave-uniform LDS destination (lane i lands at +16*i).
// M0 is written here and nowhere else: these kernels index no register array dynamically and use no other
// instruction that reads M0, so the compiler (which treats M0 as reserved and ignores the clobber) keeps no value in it.
__device__ __forceinline__ void d_load_lds16(const uint16_t* src, unsigned lds_off) {
  const unsigned uniform_off = __builtin_amdgcn_readfirstlane(lds_off);
  asm volatile("s_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, off" : : "v"(src), "s"(uniform_off) : "memory", "m0");
}

// A fragment q of K step S of a stage: rows 32q.. of the wavefront's 128 rows, one 16-byte read.
template <int STAGE_N, int S, int Q>
__device__ __forceinline__ void d_read_a(const DCtx& c, const unsigned char* lds, bf16x8 (&af)[4]) {
  af[Q] = *(const bf16x8*)(lds + (c.a_fr ^ (S << 5)) + (STAGE_N * D_A_STAGE + Q * 32 * 64));
}
// B fragment q of K step S of a stage: columns 32q.. of the wavefront's columns, two transposing 8-byte reads.
template <int STAGE_N, int S, int Q, int FN, int MODE = 0>
__device__ __forceinline__ void d_read_b(const DCtx& c, const unsigned char* lds, bf16x8 (&bf)[FN]) {
  if constexpr (MODE & D_BT) {
    bf[Q] = *(const bf16x8*)(lds + (c.b_fr[Q] ^ (S << 5)) + STAGE_N * D_B_STAGE);
    return;
  }
  typedef __attribute__((address_space(3))) s16x4* lptr;
  const unsigned char* p = lds + c.b_fr[Q] + (STAGE_N * D_B_STAGE + S * 16 * 512);
  const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)p);
  const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(p + 4 * 512));
  bf[Q] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}
// Fragment reads of a K step, spread over the four instruction groups that precede their first use.
// The first matrix instruction of the next step needs every B fragment and A fragment 0, so those are
// read first; the last group reads nothing, so that neither the barrier that follows group 3 (it waits
// for the wavefront's outstanding LDS reads) nor the first group of the next step meets a read that has
// only just been issued.
template <int SCHED, int STAGE_N, int S, int Q, int FN, int MODE = 0>
__device__ __forceinline__ void d_read_group(const DCtx& c, const unsigned char* lds, bf16x8 (&af)[4], bf16x8 (&bf)[FN]) {
  if constexpr (SCHED == 0) {   // plain order: group Q reads A fragment Q and B fragment Q
    d_read_a<STAGE_N, S, Q>(c, lds, af);
    if constexpr (Q < FN) d_read_b<STAGE_N, S, Q, FN, MODE>(c, lds, bf);
  } else if constexpr (FN == 4) {
    if constexpr (Q == 0) { d_read_b<STAGE_N, S, 0, FN, MODE>(c, lds, bf); d_read_b<STAGE_N, S, 1, FN, MODE>(c, lds, bf); }
    if constexpr (Q == 1) { d_read_b<STAGE_N, S, 2, FN, MODE>(c, lds, bf); d_read_b<STAGE_N, S, 3, FN, MODE>(c, lds, bf); d_read_a<STAGE_N, S, 0>(c, lds, af); }
    if constexpr (Q == 2) { d_read_a<STAGE_N, S, 1>(c, lds, af); d_read_a<STAGE_N, S, 2>(c, lds, af); d_read_a<STAGE_N, S, 3>(c, lds, af); }
  } else {
    if constexpr (Q == 0) { d_read_b<STAGE_N, S, 0, FN, MODE>(c, lds, bf); d_read_b<STAGE_N, S, 1, FN, MODE>(c, lds, bf); d_read_a<STAGE_N, S, 0>(c, lds, af); }
    if constexpr (Q == 1) { d_read_a<STAGE_N, S, 1>(c, lds, af); d_read_a<STAGE_N, S, 2>(c, lds, af); }
    if constexpr (Q == 2) { d_read_a<STAGE_N, S, 3>(c, lds, af); }
  }
}
template <int STAGE_N, int S, int FN, int MODE = 0>
__device__ __forceinline__ void d_read_frags(const DCtx& c, const unsigned char* lds, bf16x8 (&af)[4], bf16x8 (&bf)[FN]) {
  d_read_group<0, STAGE_N, S, 0, FN, MODE>(c, lds, af, bf);
  d_read_group<0, STAGE_N, S, 1, FN, MODE>(c, lds, af, bf);
  d_read_group<0, STAGE_N, S, 2, FN, MODE>(c, lds, af, bf);
  d_read_group<0, STAGE_N, S, 3, FN, MODE>(c, lds, af, bf);
}

// SERP: odd rows run backwards, so that one operand stays in place between any two consecutive instructions
template <int Q, int FN, int MODE = 0, bool SERP = false>
__device__ __forceinline__ void d_mfma_row(const bf16x8 (&af)[4], const bf16x8 (&bf)[FN], f32x16 (&acc)[4][FN]) {
#pragma unroll
  for (int j = 0; j < FN; ++j) {
    const int jj = (SERP && (Q & 1)) ? FN - 1 - j : j;
    acc[Q][jj] = d_mma<MODE>(af[Q], bf[jj], acc[Q][jj]);
  }
}

// matrix instructions J0 .. J1-1 of accumulator row Q
template <int Q, int J0, int J1, int FN, int MODE = 0, bool SERP = false>
__device__ __forceinline__ void d_mfma_part(const bf16x8 (&af)[4], const bf16x8 (&bf)[FN], f32x16 (&acc)[4][FN]) {
#pragma unroll
  for (int j = J0; j < J1; ++j) {
    const int jj = (SERP && (Q & 1)) ? FN - 1 - j : j;
    acc[Q][jj] = d_mma<MODE>(af[Q], bf[jj], acc[Q][jj]);
  }
}

#define D_FENCE() __builtin_amdgcn_sched_barrier(0)

// LDS-direct loads number G*PER .. G*PER+PER-1 of a tile (PER per group); loads 0..LPT/2-1 are A, the rest B
// a, b: the lane's first A and B address of the tile (plain variants) or the tile's K offset in elements cast into
// a pointer-sized integer (ragged variants, which add it to the per-load addresses).
template <int LD, int WAVES, int G, int MODE = 0>
__device__ __forceinline__ void d_issue_group(const DCtx& c, const uint16_t* a, const uint16_t* b, size_t a_koff = 0, size_t b_koff = 0, int ti = 0,
                                              int tj = 0) {
  constexpr int LPT = 32 / WAVES, HALF = LPT / 2, PER = LPT / 4 > 0 ? LPT / 4 : 1;
#pragma unroll
  for (int e = 0; e < PER; ++e) {
    const int u = G * PER + e;
    if constexpr (MODE & D_CONV) {
      if (u < HALF) {
        const bool inside = ((c.rmask[u < 4 ? u : 0] >> ti) & (c.cmask[u < 4 ? u : 0] >> tj) & 1u) != 0;
        d_load_lds16(inside ? c.a_ptr[u < 4 ? u : 0] + a_koff : c.zero, LD * D_A_STAGE + u * (1024 * WAVES) + c.wave_lds);
      } else if (u < LPT) {
        d_load_lds16(c.b_ptr[u - HALF] + b_koff, D_B0 + LD * D_B_STAGE + (u - HALF) * (1024 * WAVES) + c.wave_lds);
      }
    } else if constexpr (MODE & D_RAGGED) {
      if (u < HALF) d_load_lds16(c.a_ptr[u] + a_koff, LD * D_A_STAGE + u * (1024 * WAVES) + c.wave_lds);
      else if (u < LPT) d_load_lds16(c.b_ptr[u - HALF] + b_koff, D_B0 + LD * D_B_STAGE + (u - HALF) * (1024 * WAVES) + c.wave_lds);
    } else {
      if (u < HALF) d_load_lds16(a + u * c.a_step, LD * D_A_STAGE + u * (1024 * WAVES) + c.wave_lds);
      else if (u < LPT) d_load_lds16(b + (u - HALF) * c.b_step, D_B0 + LD * D_B_STAGE + (u - HALF) * (1024 * WAVES) + c.wave_lds);
    }
  }
}

template <int PENDING>
__device__ __forceinline__ void d_wait_loads() {
  if (PENDING == 8) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");
  else if (PENDING == 4) asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
}

// One K tile of the ring, as eight groups of matrix instructions.  The
// scheduler may not move anything across a fence, so every group carries the
// LDS reads (and, in the second half, the LDS-direct loads) written next to it:
//   groups 0-3: K step 0 of this tile  + fragment reads of K step 1,
//   barrier   : tile kt+1 complete in LDS (its loads were issued two tiles ago),
//   groups 4-7: K step 1 of this tile  + fragment reads of K step 0 of tile kt+1
//               + the loads of tile kt+3.
// ISSUE: start the loads of tile kt+3 (after the barrier).  PENDING: how many
// younger loads (those of tile kt+2) may still be in flight when tile kt+1 must
// have landed.
template <int WAVES, int SCHED, int STAGE_N, bool ISSUE, int PENDING, bool NEXT_FRAGS, int MODE = 0>
__device__ __forceinline__ void d_tile(const DCtx& c, unsigned char* lds, int kt, bf16x8 (&af)[2][4],
                                       bf16x8 (&bf)[2][WAVES == 4 ? 4 : 2], f32x16 (&acc)[4][WAVES == 4 ? 4 : 2], DWalk* walk = nullptr) {
  constexpr int FN = WAVES == 4 ? 4 : 2;
  constexpr int NXT = (STAGE_N + 1) % D_STAGES;
  constexpr int LD = (STAGE_N + 3) % D_STAGES;
  const uint16_t* a = c.a_src + (size_t)(kt + 3) * D_BK;
  const uint16_t* b = c.b_src + (size_t)(kt + 3) * c.b_kstep;
  size_t a_koff = (size_t)(kt + 3) * D_BK, b_koff = (size_t)(kt + 3) * c.b_kstep;
  int ti = 0, tj = 0;
  if constexpr ((MODE & D_CONV) != 0) {   // tile kt+3 is the walk's next tile
    a_koff = (size_t)walk->a_off;
    b_koff = (size_t)walk->b_off;
    ti = walk->ti;
    tj = walk->tj;
    if (ISSUE) walk->advance();
  }
  D_FENCE();
  d_mfma_row<0, FN, MODE, SCHED == 1>(af[0], bf[0], acc); d_read_group<SCHED, STAGE_N, 1, 0, FN, MODE>(c, lds, af[1], bf[1]); D_FENCE();
  d_mfma_row<1, FN, MODE, SCHED == 1>(af[0], bf[0], acc); d_read_group<SCHED, STAGE_N, 1, 1, FN, MODE>(c, lds, af[1], bf[1]); D_FENCE();
  d_mfma_row<2, FN, MODE, SCHED == 1>(af[0], bf[0], acc); d_read_group<SCHED, STAGE_N, 1, 2, FN, MODE>(c, lds, af[1], bf[1]); D_FENCE();
  // the barrier sits before the group's last matrix instruction, which then covers the barrier's latency
  constexpr int EARLY = SCHED == 2 ? FN - 1 : FN;   // matrix instructions of group 3 issued before the barrier
  d_mfma_part<3, 0, EARLY, FN, MODE, SCHED == 1>(af[0], bf[0], acc);
  if constexpr (SCHED == 0) d_read_group<SCHED, STAGE_N, 1, 3, FN, MODE>(c, lds, af[1], bf[1]);
  D_FENCE();
  d_wait_loads<PENDING>();
  __syncthreads();
  D_FENCE();
  d_mfma_part<3, EARLY, FN, FN, MODE, SCHED == 1>(af[0], bf[0], acc);
  d_mfma_row<0, FN, MODE, SCHED == 1>(af[1], bf[1], acc);
  if (NEXT_FRAGS) d_read_group<SCHED, NXT, 0, 0, FN, MODE>(c, lds, af[0], bf[0]);
  if (ISSUE) d_issue_group<LD, WAVES, 0, MODE>(c, a, b, a_koff, b_koff, ti, tj);
  D_FENCE();
  d_mfma_row<1, FN, MODE, SCHED == 1>(af[1], bf[1], acc);
  if (NEXT_FRAGS) d_read_group<SCHED, NXT, 0, 1, FN, MODE>(c, lds, af[0], bf[0]);
  if (ISSUE) d_issue_group<LD, WAVES, 1, MODE>(c, a, b, a_koff, b_koff, ti, tj);
  D_FENCE();
  d_mfma_row<2, FN, MODE, SCHED == 1>(af[1], bf[1], acc);
  if (NEXT_FRAGS) d_read_group<SCHED, NXT, 0, 2, FN, MODE>(c, lds, af[0], bf[0]);
  if (ISSUE) d_issue_group<LD, WAVES, 2, MODE>(c, a, b, a_koff, b_koff, ti, tj);
  D_FENCE();
  d_mfma_row<3, FN, MODE, SCHED == 1>(af[1], bf[1], acc);
  if (NEXT_FRAGS) d_read_group<SCHED, NXT, 0, 3, FN, MODE>(c, lds, af[0], bf[0]);
  if (ISSUE) d_issue_group<LD, WAVES, 3, MODE>(c, a, b, a_koff, b_koff, ti, tj);
  D_FENCE();
}

template <int WAVES, int SCHED, int MODE = 0>
__global__ __launch_bounds__(WAVES * 64, 1) void gemm_bf16_dma_kernel(const GemmParams p, const uint16_t* __restrict__ A,
                                                                      const uint16_t* __restrict__ B, float* __restrict__ C) {
  constexpr int FN = WAVES == 4 ? 4 : 2;        // 32-column fragments per wavefront
  constexpr int WN_WAVES = WAVES / 2;           // wavefronts side by side along n
  constexpr int LPT = 32 / WAVES;               // LDS-direct loads per lane and tile
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int wm = wave / WN_WAVES, wn = wave % WN_WAVES;
  int tm, tn;
  // a batch of products: consecutive groups of tiles_m * tiles_n workgroups take consecutive batch entries
  const unsigned tiles = (unsigned)(p.tiles_m * p.tiles_n), batch = blockIdx.x / tiles;
  A += (int64_t)batch * p.a_b;
  B += (int64_t)batch * p.b_b;
  C += (int64_t)batch * p.c_b;
  tile_of(blockIdx.x - batch * tiles, tiles, p.tiles_m, p.tiles_n, &tm, &tn);

  DCtx c;
  // A loads: load u of wavefront w fills LDS rows 16*(WAVES*u+w) .. +15 of the stage (1 KB): lane -> row + lane/4, slot lane&3
  {
    const int row = 16 * wave + (lane >> 2);           // + 16*WAVES*u
    const int chunk = (lane & 3) ^ ((row >> 2) & 3);   // (row>>2)&3 does not change with u
    c.a_src = A + p.a_base + ((int64_t)tm * BM + row) * p.a_m + chunk * 8;
    c.a_step = (size_t)(16 * WAVES) * p.a_m;
  }
  if constexpr (MODE & D_BT) {
    // transposed B: rows are n, loaded and laid out like A's rows
    const int row = 16 * wave + (lane >> 2);
    const int chunk = (lane & 3) ^ ((row >> 2) & 3);
    c.b_src = B + p.b_base + ((int64_t)tn * BN + row) * p.b_k + chunk * 8;
    c.b_step = (size_t)(16 * WAVES) * p.b_k;
    c.b_kstep = (size_t)D_BK;
  } else {
    // B loads: load u of wavefront w fills k rows 2*(WAVES*u+w), +1: lane -> k = 2*(WAVES*u+w) + lane/32, slot lane&31
    const int k = 2 * wave + (lane >> 5);               // + 2*WAVES*u ; k&3 does not change with u
    const int chunk = (lane & 31) ^ (4 * (k & 3));
    c.b_src = B + p.b_base + (int64_t)k * p.b_k + (int64_t)tn * BN + chunk * 8;
    c.b_step = (size_t)(2 * WAVES) * p.b_k;
    c.b_kstep = (size_t)D_BK * p.b_k;
  }
  if constexpr (MODE & D_RAGGED) {
    // one address per load, with the row (or, for a row-major B, the 8-column chunk) clamped into the matrix
    constexpr int HALF_LOADS = 16 / WAVES;
#pragma unroll
    for (int u = 0; u < HALF_LOADS; ++u) {
      const int row = 16 * wave + (lane >> 2) + 16 * WAVES * u;
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      const int64_t gm = (int64_t)tm * BM + row;
      c.a_ptr[u] = A + p.a_base + (gm < p.M ? gm : p.M - 1) * p.a_m + chunk * 8;
      if constexpr (MODE & D_BT) {
        const int64_t gn = (int64_t)tn * BN + row;
        c.b_ptr[u] = B + p.b_base + (gn < p.N ? gn : p.N - 1) * p.b_k + chunk * 8;
      } else {
        const int k = 2 * wave + (lane >> 5) + 2 * WAVES * u;
        const int bchunk = (lane & 31) ^ (4 * (k & 3));
        const int64_t gn = (int64_t)tn * BN + bchunk * 8;
        c.b_ptr[u] = B + p.b_base + (int64_t)k * p.b_k + (gn + 8 <= p.N ? gn : p.N - 8);
      }
    }
  }
  DWalk walk = {};
  if constexpr ((MODE & D_CONV) != 0) {
    static_assert((MODE & D_BT) && (MODE & D_RAGGED) && WAVES == 4, "the convolution mode builds on the transposed-B, ragged, four-wavefront form");
    // Row m of A is output pixel m = (n, y, x): the load's address for filter tap (0, 0) and the masks of the taps
    // inside the image; rows past the last pixel repeat it (they feed accumulators that are never stored).
    const uint16_t* zero = d_zero_chunk;
    asm volatile("" : "+s"(zero));   // held in registers (else its address is re-read from memory before every load)
    c.zero = zero;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int row = 16 * wave + (lane >> 2) + 64 * u;
      const int chunk = (lane & 3) ^ ((row >> 2) & 3);
      int64_t gm = (int64_t)tm * BM + row;
      if (gm >= p.M) gm = p.M - 1;
      const int m = (int)gm, x = m % p.cv_Wo, q = m / p.cv_Wo, y = q % p.cv_Ho, n = q / p.cv_Ho;
      const int iy0 = y * p.cv_sy - p.cv_py, ix0 = x * p.cv_sx - p.cv_px;
      c.a_ptr[u] = A + p.a_base + (int64_t)n * p.cv_i_n + (int64_t)iy0 * p.cv_i_y + (int64_t)ix0 * p.cv_i_x + chunk * 8;
      unsigned rm = 0, cm = 0;
      for (int i = 0; i < p.cv_R; ++i) {
        const int yy = iy0 + i * p.cv_dy;
        if (yy >= 0 && yy < p.cv_H) rm |= 1u << i;
      }
      for (int j = 0; j < p.cv_S; ++j) {
        const int xx = ix0 + j * p.cv_dx;
        if (xx >= 0 && xx < p.cv_W) cm |= 1u << j;
      }
      c.rmask[u] = rm;
      c.cmask[u] = cm;
    }
    walk.S = p.cv_S;
    walk.chunks = p.cv_chunks;
    walk.a_col = (int64_t)p.cv_dx * p.cv_i_x - (int64_t)(p.cv_chunks - 1) * D_BK;
    walk.b_col = p.cv_f_s - (int64_t)(p.cv_chunks - 1) * D_BK;
    walk.a_row = (int64_t)p.cv_dy * p.cv_i_y - (int64_t)(p.cv_S - 1) * p.cv_dx * p.cv_i_x - (int64_t)(p.cv_chunks - 1) * D_BK;
    walk.b_row = p.cv_f_r - (int64_t)(p.cv_S - 1) * p.cv_f_s - (int64_t)(p.cv_chunks - 1) * D_BK;
  }
  c.wave_lds = wave * 1024;
  // A fragments: lane supplies row (lane&31) (+32*i) and chunk 2*s + (lane>>5)
  {
    const int fr = lane & 31, fh = lane >> 5;
    c.a_fr = (wm * 128 + fr) * 64 + ((fh ^ ((fr >> 2) & 3)) << 4);
  }
  if constexpr (MODE & D_BT) {
    const int fr = lane & 31, fh = lane >> 5;
#pragma unroll
    for (int j = 0; j < 4; ++j)
      c.b_fr[j] = D_B0 + (wn * 32 * FN + 32 * (j < FN ? j : 0) + fr) * 64 + ((fh ^ ((fr >> 2) & 3)) << 4);
  } else
  // B fragments: 16-lane group g, lane p in it: k = 8*(g>>1) + (p>>2) (+16*s, +4 second read),
  // columns wn*32*FN + 32*j + 16*(g&1) + 4*(p&3) .. +3
  {
    const int g = lane >> 4, pl = lane & 15;
    const int k = 8 * (g >> 1) + (pl >> 2);
    const int low2 = 2 * (g & 1) + ((pl & 3) >> 1);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int chunk = (wn * 4 * FN + 4 * (j < FN ? j : 0) + low2) ^ (4 * (k & 3));
      c.b_fr[j] = D_B0 + k * 512 + chunk * 16 + (pl & 1) * 8;
    }
  }

  bf16x8 af[2][4], bf[2][FN];
  f32x16 acc[4][FN];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  // prologue: tiles 0, 1, 2 in flight, wait for tile 0   (k_tiles is a multiple of 4, checked on the host)
  if constexpr ((MODE & D_CONV) != 0) {
    const uint16_t* a = nullptr;
    const uint16_t* b = nullptr;
    d_issue_group<0, WAVES, 0, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<0, WAVES, 1, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    d_issue_group<0, WAVES, 2, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<0, WAVES, 3, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    walk.advance();
    d_issue_group<1, WAVES, 0, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<1, WAVES, 1, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    d_issue_group<1, WAVES, 2, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<1, WAVES, 3, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    walk.advance();
    d_issue_group<2, WAVES, 0, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<2, WAVES, 1, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    d_issue_group<2, WAVES, 2, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj); d_issue_group<2, WAVES, 3, MODE>(c, a, b, (size_t)walk.a_off, (size_t)walk.b_off, walk.ti, walk.tj);
    walk.advance();   // the walk now stands at tile 3, the first one the loop issues
  } else {
    const uint16_t* a = c.a_src;
    const uint16_t* b = c.b_src;
    size_t ak = 0, bk = 0;
    d_issue_group<0, WAVES, 0, MODE>(c, a, b, ak, bk); d_issue_group<0, WAVES, 1, MODE>(c, a, b, ak, bk); d_issue_group<0, WAVES, 2, MODE>(c, a, b, ak, bk); d_issue_group<0, WAVES, 3, MODE>(c, a, b, ak, bk);
    a += D_BK; b += c.b_kstep; ak += D_BK; bk += c.b_kstep;
    d_issue_group<1, WAVES, 0, MODE>(c, a, b, ak, bk); d_issue_group<1, WAVES, 1, MODE>(c, a, b, ak, bk); d_issue_group<1, WAVES, 2, MODE>(c, a, b, ak, bk); d_issue_group<1, WAVES, 3, MODE>(c, a, b, ak, bk);
    a += D_BK; b += c.b_kstep; ak += D_BK; bk += c.b_kstep;
    d_issue_group<2, WAVES, 0, MODE>(c, a, b, ak, bk); d_issue_group<2, WAVES, 1, MODE>(c, a, b, ak, bk); d_issue_group<2, WAVES, 2, MODE>(c, a, b, ak, bk); d_issue_group<2, WAVES, 3, MODE>(c, a, b, ak, bk);
  }
  d_wait_loads<2 * LPT>();
  __syncthreads();
  d_read_frags<0, 0, FN, MODE>(c, lds, af[0], bf[0]);

  const int last4 = p.k_tiles - 4;
  for (int kt = 0; kt < last4; kt += 4) {
    d_tile<WAVES, SCHED, 0, true, LPT, true, MODE>(c, lds, kt, af, bf, acc, &walk);
    d_tile<WAVES, SCHED, 1, true, LPT, true, MODE>(c, lds, kt + 1, af, bf, acc, &walk);
    d_tile<WAVES, SCHED, 2, true, LPT, true, MODE>(c, lds, kt + 2, af, bf, acc, &walk);
    d_tile<WAVES, SCHED, 3, true, LPT, true, MODE>(c, lds, kt + 3, af, bf, acc, &walk);
  }
  d_tile<WAVES, SCHED, 0, true, LPT, true, MODE>(c, lds, last4, af, bf, acc, &walk);        // issues the last tile's loads
  d_tile<WAVES, SCHED, 1, false, LPT, true, MODE>(c, lds, last4 + 1, af, bf, acc, &walk);
  d_tile<WAVES, SCHED, 2, false, 0, true, MODE>(c, lds, last4 + 2, af, bf, acc, &walk);
  d_tile<WAVES, SCHED, 3, false, 0, false, MODE>(c, lds, last4 + 3, af, bf, acc, &walk);

  const int fr = lane & 31, fh = lane >> 5;
  if constexpr (!(MODE & D_RAGGED)) {
    if (p.vec_c) {   // uniform branch
      // A 4-byte store per lane costs the address unit as much as a 16-byte one, and a wavefront holds 256 values
      // per lane: each fragment (32 x 32) goes through a 4 KB buffer of the wavefront in the idle ring, [row][32
      // columns] with the 16-byte slots swizzled by the row, and leaves as one store per row and four columns --
      // eight lanes write a row's 128 contiguous bytes.  (Accumulator element v of lane l is row 8*(v/4) +
      // 4*(l>>5) + v%4 of the fragment, column l&31.)  The fused form adds the bias and applies the relu on the way.
      __syncthreads();   // every wavefront is done with the ring
      unsigned char* buf = lds + wave * 4096;
      const int sp = lane >> 3, sc = lane & 7;
      const bool fused = !(MODE & D_I8) && p.epi;
      float b4[FN][4];
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) b4[j][e] = fused ? p.bias[(int64_t)tn * BN + wn * 32 * FN + 32 * j + sc * 4 + e] : 0.f;
      const int64_t off0 = p.c_base + ((int64_t)tm * BM + wm * 128 + sp) * p.c_m + (int64_t)tn * BN + wn * 32 * FN + sc * 4;
      unsigned wofs[4];
#pragma unroll
      for (int v = 0; v < 4; ++v) {
        const int row = 4 * fh + v;
        wofs[v] = (unsigned)(row * 128 + ((((fr >> 2) ^ row) << 4) | ((fr & 3) << 2)));
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j) {
#pragma unroll
          for (int v = 0; v < 16; ++v) *(float*)(buf + wofs[v % 4] + (v / 4) * 1024) = acc[i][j][v];
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int r8 = 0; r8 < 4; ++r8) {
            typedef __attribute__((ext_vector_type(4))) float f4;
            f4 val = *(const f4*)(buf + (8 * r8 + sp) * 128 + ((sc ^ sp) << 4));
            const int64_t off = off0 + (int64_t)(32 * i + 8 * r8) * p.c_m + 32 * j;
            if (fused) {
              val.x = __builtin_fmaxf(val.x + b4[j][0], 0.f);
              val.y = __builtin_fmaxf(val.y + b4[j][1], 0.f);
              val.z = __builtin_fmaxf(val.z + b4[j][2], 0.f);
              val.w = __builtin_fmaxf(val.w + b4[j][3], 0.f);
            }
            if (fused && p.epi == 2) {
              const float ve[4] = {val.x, val.y, val.z, val.w};
              unsigned h[4];
#pragma unroll
              for (int e = 0; e < 4; ++e) {
                const uint32_t u = __float_as_uint(ve[e]);
                h[e] = (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;   // round to nearest even
              }
              const u32x2 packed = {h[0] | (h[1] << 16), h[2] | (h[3] << 16)};
              __builtin_nontemporal_store(packed, (u32x2*)((uint16_t*)C + off));
            } else {
              __builtin_nontemporal_store(val, (f4*)(C + off));
            }
          }
          __builtin_amdgcn_wave_barrier();
        }
      return;
    }
  }
  if (!(MODE & D_I8) && p.epi) {   // the fused form of a following relu(C + bias) statement; uniform branch
    const int64_t off0 = p.c_base + ((int64_t)tm * BM + wm * 128 + 4 * fh) * p.c_m + (int64_t)tn * BN + wn * 32 * FN + fr;
    float bj[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int64_t gn = (int64_t)tn * BN + wn * 32 * FN + fr + 32 * j;
      bj[j] = p.bias[(MODE & D_RAGGED) ? (gn < p.N ? gn : p.N - 1) : gn];
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const int r = 32 * i + 8 * (v / 4) + (v % 4);
          const int64_t gm = (int64_t)tm * BM + wm * 128 + 4 * fh + r, gn = (int64_t)tn * BN + wn * 32 * FN + fr + 32 * j;
          if (!(MODE & D_RAGGED) || (gm < p.M && gn < p.N)) epi_store(p, C, off0 + (int64_t)r * p.c_m + 32 * j, acc[i][j][v], bj[j]);
        }
    return;
  }
  float* c_g = C + p.c_base + ((int64_t)tm * BM + wm * 128 + 4 * fh) * p.c_m + (int64_t)tn * BN + wn * 32 * FN + fr;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int r = 32 * i + 8 * (v / 4) + (v % 4);
        if constexpr (MODE & D_RAGGED) {
          const int64_t gm = (int64_t)tm * BM + wm * 128 + 4 * fh + r, gn = (int64_t)tn * BN + wn * 32 * FN + fr + 32 * j;
          if (gm < p.M && gn < p.N) __builtin_nontemporal_store(acc[i][j][v], c_g + (int64_t)r * p.c_m + 32 * j);
        } else {
          __builtin_nontemporal_store(acc[i][j][v], c_g + (int64_t)r * p.c_m + 32 * j);
        }
      }
}

// ---------------------------------------------------------------------------
// 128 x 128 tiles for products with fewer 256 x 256 tiles than the chip has
// CUs (a 2048^3 product has 64): four times as many workgroups, each four
// wavefronts side by side along n (128 rows x 32 columns per wavefront: four A
// fragments, one B fragment, four matrix instructions per 16-deep K step).
// Same staging as the large-tile kernel -- LDS-direct loads into a four-stage
// ring of 32-deep K tiles, A rows swizzled by (row>>2)&3, B kept [k][n] in
// 256-byte rows swizzled by 4*(k&3) and read with the transposing LDS read --
// at half the bytes per tile (8 KB + 8 KB), so two workgroups fit on a CU.
// M and N multiples of 128, K a multiple of 128 (256 for int8).  MODE as in the large-tile kernel: D_BT for a
// transposed B (its tile then lies in LDS like A's), D_I8 for int8 operands with int32 accumulation.
// ---------------------------------------------------------------------------
constexpr int T_BM = 128, T_BN = 128;
constexpr int t128_lds_bytes(int kb) { return D_STAGES * (T_BM + T_BN) * kb; }   // 64 KB, or 128 KB with 128-byte K tile rows

template <int N>
__device__ __forceinline__ void t_wait_loads() {   // until at most N of the wavefront's loads are outstanding
  static_assert(N >= 0 && N < 64, "the counter's range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// W8: eight wavefronts (2 along m x 4 along n, 64 x 32 each) instead of four (128 x 32 each): two wavefronts per
// SIMD, so that one's waits (LDS latency, barrier) are covered by the other's matrix instructions.
// KB: bytes of a K tile row of A (and of a transposed B): 64, or 128 -- K tiles of 64 instead of 32 deep, half as
// many barriers per matrix instruction, whole 128-byte lines per row -- where one workgroup per CU covers the
// product anyway (the ring then takes 128 KB).
template <int MODE, int W8 = 0, int KB = 64>
__global__ __launch_bounds__(256 * (1 + W8), 1) void gemm_bf16_t128_kernel(const GemmParams p, const uint16_t* __restrict__ A,
                                                                         const uint16_t* __restrict__ B, float* __restrict__ C) {
  static_assert(KB == 64 || KB == 128, "K tile rows");
  constexpr int NW = 4 * (1 + W8);          // wavefronts
  constexpr int NF = 4 / (1 + W8);          // A fragments (32 rows each) per wavefront
  constexpr int BKE = KB / 2;               // depth of a K tile in 16-bit elements
  constexpr int T_A_STAGE = T_BM * KB, T_B_STAGE = T_BN * KB, T_B0 = D_STAGES * T_A_STAGE;
  constexpr int LPW = T_A_STAGE / 1024 / NW;   // 1 KB load blocks per wavefront, per operand and K tile
  constexpr int LPT = 2 * LPW;                 // loads per wavefront and K tile
  constexpr int KS = KB / 32;                  // matrix-instruction K steps per K tile
  constexpr int RPB = 1024 / KB, LPR = KB / 16;   // rows of a 1 KB block of A, lanes per row
  auto key = [](int row) { return KB == 64 ? ((row >> 2) & 3) : ((row >> 1) & 7); };
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  typedef __attribute__((address_space(3))) s16x4* lptr;
  const int t = threadIdx.x, lane = t & 63, wv = t >> 6, wn = wv & 3, wm = wv >> 2;
  const unsigned tiles = (unsigned)(p.tiles_m * p.tiles_n), batch = blockIdx.x / tiles;
  A += (int64_t)batch * p.a_b;
  B += (int64_t)batch * p.b_b;
  C += (int64_t)batch * p.c_b;
  const unsigned tile = blockIdx.x - batch * tiles;
  const int tm = (int)(tile / (unsigned)p.tiles_n), tn = (int)(tile % (unsigned)p.tiles_n);

  // loads: block wv (+ NW*u) of each operand's 8 blocks of 1 KB per K tile
  const uint16_t* a_src;
  const uint16_t* b_src;
  {
    const int row = RPB * wv + lane / LPR;              // + RPB*NW*u
    const int chunk = (lane % LPR) ^ key(row);
    a_src = A + p.a_base + ((int64_t)tm * T_BM + row) * p.a_m + chunk * 8;
    if constexpr (MODE & D_BT) {
      b_src = B + p.b_base + ((int64_t)tn * T_BN + row) * p.b_k + chunk * 8;
    } else {
      const int k = 4 * wv + (lane >> 4);                 // + 4*NW*u ; k&3 == lane>>4
      const int bchunk = (lane & 15) ^ (4 * (k & 3));
      b_src = B + p.b_base + (int64_t)k * p.b_k + (int64_t)tn * T_BN + bchunk * 8;
    }
  }
  const size_t a_step = (size_t)(RPB * NW) * p.a_m, b_step = (MODE & D_BT) ? (size_t)(RPB * NW) * p.b_k : (size_t)(4 * NW) * p.b_k,
               b_kstep = (MODE & D_BT) ? (size_t)BKE : (size_t)BKE * p.b_k;
  const unsigned wave_lds = wv * 1024;
  auto issue = [&](int stage, int kt) {
    const uint16_t* a = a_src + (size_t)kt * BKE;
    const uint16_t* b = b_src + (size_t)kt * b_kstep;
#pragma unroll
    for (int u = 0; u < LPW; ++u) d_load_lds16(a + u * a_step, stage * T_A_STAGE + u * (NW * 1024) + wave_lds);
#pragma unroll
    for (int u = 0; u < LPW; ++u) d_load_lds16(b + u * b_step, T_B0 + stage * T_B_STAGE + u * (NW * 1024) + wave_lds);
  };
  // fragment addresses
  const int fr = lane & 31, fh = lane >> 5;
  const unsigned a_fr = (unsigned)((wm * 64 * W8 + fr) * KB + ((fh ^ key(fr)) << 4));
  unsigned b_fr;
  {
    const int g = lane >> 4, pl = lane & 15;
    const int k = 8 * (g >> 1) + (pl >> 2);
    const int low2 = 2 * (g & 1) + ((pl & 3) >> 1);
    b_fr = (unsigned)(T_B0 + k * 256 + (((wn * 4 + low2) ^ (4 * (k & 3))) << 4) + (pl & 1) * 8);
    if constexpr (MODE & D_BT) b_fr = (unsigned)(T_B0 + (wn * 32 + fr) * KB + ((fh ^ key(fr)) << 4));
  }
  auto read_frags = [&](int stage, int s, bf16x8 (&af)[NF], bf16x8& bf) {
#pragma unroll
    for (int q = 0; q < NF; ++q) af[q] = *(const bf16x8*)(lds + (a_fr ^ (unsigned)(s << 5)) + stage * T_A_STAGE + q * 32 * KB);
    if constexpr (MODE & D_BT) {
      bf = *(const bf16x8*)(lds + (b_fr ^ (unsigned)(s << 5)) + stage * T_B_STAGE);
    } else {
      const unsigned char* pb = lds + b_fr + stage * T_B_STAGE + s * 16 * 256;
      const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)pb);
      const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lptr)(pb + 4 * 256));
      bf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
    }
  };

  f32x16 acc[NF];
#pragma unroll
  for (int q = 0; q < NF; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[q][v] = 0.f;

  const int k_tiles = p.k_tiles;   // at least 2 (host)
  // The ring holds four K tiles.  During iteration kt the wavefronts multiply tile kt from registers and read the
  // fragments of tile kt+1 (a whole tile ahead, so that an LDS read has an iteration to land before the matrix
  // cores need it); tile kt+2 must have landed by the iteration's end, tile kt+3 is in flight, and after the
  // barrier, when nobody reads tile kt any more, its slot takes tile kt+4.
  issue(0, 0);
  issue(1, 1);
  if (k_tiles > 2) issue(2, 2);
  if (k_tiles > 3) issue(3, 3);
  if (k_tiles > 3) t_wait_loads<2 * LPT>();      // tiles 0 and 1 have landed
  else if (k_tiles > 2) t_wait_loads<LPT>();
  else t_wait_loads<0>();
  __syncthreads();
  bf16x8 af[2][KS][NF], bf[2][KS];               // [tile parity][K step]
#pragma unroll
  for (int ks = 0; ks < KS; ++ks) read_frags(0, ks, af[0][ks], bf[0][ks]);
  __syncthreads();   // (the compiler waits for these reads here, and so knows in the loop that only the reads ahead are outstanding)
  auto iteration = [&](int kt, bf16x8 (&ca)[KS][NF], bf16x8 (&cb)[KS], bf16x8 (&na)[KS][NF], bf16x8 (&nb)[KS]) {
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      D_FENCE();
      // unconditional: behind the last tile this reads a stale ring slot and nobody uses it; under a condition the
      // compiler would make the matrix instructions wait for the reads ahead as well
      read_frags((kt + 1) & 3, ks, na[ks], nb[ks]);
#pragma unroll
      for (int q = 0; q < NF; ++q) acc[q] = d_mma<MODE>(ca[ks][q], cb[ks], acc[q]);
    }
    D_FENCE();
    if (kt + 3 < k_tiles) t_wait_loads<LPT>();   // all but tile kt+3: tile kt+2 has landed
    else t_wait_loads<0>();
    __syncthreads();
    if (kt + 4 < k_tiles) issue(kt & 3, kt + 4);
    D_FENCE();
  };
  for (int kt = 0; kt < k_tiles; kt += 2) {
    iteration(kt, af[0], bf[0], af[1], bf[1]);
    if (kt + 1 < k_tiles) iteration(kt + 1, af[1], bf[1], af[0], bf[0]);
  }

  if (!(MODE & D_I8) && p.epi) {   // fused relu(C + bias)
    const int64_t off0 = p.c_base + ((int64_t)tm * T_BM + wm * 64 * W8 + 4 * fh) * p.c_m + (int64_t)tn * T_BN + wn * 32 + fr;
    const float bn = p.bias[(int64_t)tn * T_BN + wn * 32 + fr];
#pragma unroll
    for (int q = 0; q < NF; ++q)
#pragma unroll
      for (int v = 0; v < 16; ++v) epi_store(p, C, off0 + (int64_t)(32 * q + 8 * (v / 4) + (v % 4)) * p.c_m, acc[q][v], bn);
    return;
  }
  float* c_g = C + p.c_base + ((int64_t)tm * T_BM + wm * 64 * W8 + 4 * fh) * p.c_m + (int64_t)tn * T_BN + wn * 32 + fr;
#pragma unroll
  for (int q = 0; q < NF; ++q)
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const int r = 32 * q + 8 * (v / 4) + (v % 4);
      __builtin_nontemporal_store(acc[q][v], c_g + (int64_t)r * p.c_m);
    }
}

// ---------------------------------------------------------------------------
// Split reduction (Section 2.1, last paragraph; Definition 2 rule 3: an aggregation may be regrouped because the
// operation is associative and commutative).  A product with few output tiles and a long reduction index is run
// as S products over K / S each -- the batch mechanism of the kernels above, every slice writing its own M x N
// image of partial sums into a workspace -- and this kernel adds the S images in a fixed order, so the result does
// not depend on scheduling: integer sums are exact, float sums are reproducible from run to run.
// Where the output is small (few items, many slices) a thread per item would add its S values one after the other
// from a handful of workgroups, bound by the latency of the loads; then G threads share an item, each adding a run
// of consecutive slices, and the G sums meet in LDS, again in slice order.
// ---------------------------------------------------------------------------
template <typename T, int VEC>
__global__ __launch_bounds__(256) void splitk_reduce_kernel(const T* __restrict__ part, T* __restrict__ C, int64_t M, int64_t N, int64_t c_m,
                                                            int64_t c_base, int S, int G) {
  typedef T vec_t __attribute__((ext_vector_type(VEC)));
  __shared__ vec_t partial[256];
  const int64_t per_row = N / VEC, total = M * per_row, image = M * N;
  const int items = 256 / G;                      // items of a workgroup; G is a power of two, at most 16
  const int grp = (int)threadIdx.x / items, it = (int)threadIdx.x % items;
  const int run = (S + G - 1) / G, first = grp * run, last = first + run < S ? first + run : S;
  for (int64_t base = (int64_t)blockIdx.x * items; base < total; base += (int64_t)gridDim.x * items) {
    const int64_t e = base + it;
    const bool valid = e < total;
    const int64_t m = valid ? e / per_row : 0, n = valid ? (e - m * per_row) * VEC : 0;
    const T* src = part + m * N + n;
    vec_t acc = {};
    if (valid) {
      int sl = first;
      for (; sl + 8 <= last; sl += 8) {   // eight loads in flight, added in slice order
        vec_t v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = __builtin_nontemporal_load((const vec_t*)(src + (int64_t)(sl + u) * image));
#pragma unroll
        for (int u = 0; u < 8; ++u) acc += v[u];
      }
      for (; sl < last; ++sl) acc += __builtin_nontemporal_load((const vec_t*)(src + (int64_t)sl * image));
    }
    if (G > 1) {
      partial[threadIdx.x] = acc;
      __syncthreads();
      if (grp == 0)
        for (int q = 1; q < G; ++q) acc += partial[q * items + it];
      __syncthreads();
    }
    if (valid && grp == 0) *(vec_t*)(C + c_base + m * c_m + n) = acc;
  }
}

GemmParams make_params(const GemmShape& g, bool i8 = false) {
  GemmParams p;
  p.tiles_m = (int)((g.M + BM - 1) / BM);
  p.tiles_n = (int)((g.N + BN - 1) / BN);
  p.M = (int)g.M;
  p.N = (int)g.N;
  p.k_tiles = (int)(g.K / BK);
  p.pad_ = 0;
  p.a_m = g.a_m; p.c_m = g.c_m;
  p.b_k = (g.b_k == 1 && g.b_n != 1) ? g.b_n : g.b_k;   // row stride of B as stored: [n][k] (transposed) or [k][n]
  if (i8) {   // int8 operands seen as 16-bit matrices of half the width (see D_I8)
    p.a_m /= 2;
    p.b_k /= 2;
  }
  p.a_base = i8 ? g.a_base / 2 : g.a_base;
  p.b_base = i8 ? g.b_base / 2 : g.b_base;
  p.c_base = g.c_base;
  p.a_b = i8 ? g.a_b / 2 : g.a_b;
  p.b_b = i8 ? g.b_b / 2 : g.b_b;
  p.c_b = g.c_b;
  p.bias = nullptr;
  p.epi = 0;
  p.vec_c = 0;
  return p;
}

}  // namespace

static bool gemm_select_one(const GemmShape& g, int in_dtype, GemmLaunch* l, stripe_block_info_t* info);

// How many slices of the reduction index a single product is cut into (1 = not split).  Only the LDS-direct
// kernels walk a batch; a slice must be whole passes through their four-stage ring.  The choice minimises a small
// time model calibrated on this chip: workgroups run in rounds of one per CU, a round costs the slice's K tiles
// times the measured time per tile, and splitting adds a second launch plus writing and re-reading S images of
// partial sums.  A split has to beat the unsplit launch by a fifth to be taken.
// STRIPE_TUNE gemm_splitk: 0 or 1 = never, n > 1 = n slices if legal.
static int choose_split_k(const GemmShape& g, int in_dtype, const GemmLaunch& l) {
  if (g.batch > 1 || l.variant < 20) return 1;
  const bool i8 = in_dtype == STRIPE_I8;
  const int64_t ring = i8 ? 256 : D_BK * D_STAGES;
  const int forced = tune_int("gemm_splitk", -1);
  if (forced == 0 || forced == 1) return 1;
  auto legal = [&](int64_t s) {
    return s >= 2 && g.K % (s * ring) == 0 && s * l.grid <= 0x7fffffffLL && s * g.M * g.N * 4 <= ((int64_t)1 << 31);
  };
  if (forced > 1) return legal(forced) ? forced : 1;
  if (g.K < 16 * ring) return 1;   // short reductions: a second launch costs more than the idle CUs
  const double us_per_tile = l.variant >= 50 ? 0.30 : 0.85;   // one K tile (32 deep; int8: 64) of a 128- / 256-wide workgroup tile
  const double k_tile = i8 ? 64.0 : (double)D_BK;
  auto model_us = [&](int64_t s) {
    const double rounds = (double)((l.grid * s + 255) / 256);
    double t = 3.0 + rounds * ((double)g.K / (double)s / k_tile) * us_per_tile;
    if (s > 1) t += 2.5 + (double)s * (double)g.M * (double)g.N * 8.0 / 2.0e6;   // second launch; partial sums out and back at an effective 2 TB/s
    return t;
  };
  int64_t best = 1;
  double best_t = model_us(1) * 0.8;
  for (int64_t s = 2; s <= g.K / ring && s <= 1024; ++s)
    if (legal(s) && model_us(s) < best_t) {
      best = s;
      best_t = model_us(s);
    }
  return (int)best;
}

bool gemm_select(const GemmShape& g, int in_dtype, GemmLaunch* l, stripe_block_info_t* info) {
  if (!gemm_select_one(g, in_dtype, l, info)) return false;
  l->split_k = choose_split_k(g, in_dtype, *l);
  l->ws_bytes = 0;
  l->t128_kb = 64;
  if (l->variant >= 50 && l->t128_waves == 8) {
    // 128-byte K tile rows (a 128 KB ring: one workgroup per CU) where one round of workgroups covers the product anyway
    const int64_t final_grid = l->grid * (l->split_k > 1 ? l->split_k : 1) * (g.batch > 1 ? g.batch : 1);
    const int forced = tune_int("gemm_t128_kb", 0);
    if (forced ? forced == 128 : final_grid <= 256) {
      l->t128_kb = 128;
      info->tile_k *= 2;
      info->lds_bytes = t128_lds_bytes(128);
      char* at = strstr(info->kernel, in_dtype == STRIPE_I8 ? "128x128x64_" : "128x128x32_");
      if (at) {   // the K tile's depth in the name: 32 -> 64 elements (int8: 64 -> 128; one character longer)
        std::string name(info->kernel, at);
        name += in_dtype == STRIPE_I8 ? "128x128x128_" : "128x128x64_";
        name += at + 11;
        snprintf(info->kernel, sizeof info->kernel, "%s", name.c_str());
      }
    }
  }
  if (l->split_k > 1) {
    l->ws_bytes = (int64_t)l->split_k * g.M * g.N * 4;
    l->grid *= l->split_k;
    info->grid = l->grid;
    const size_t n = strlen(info->kernel);
    snprintf(info->kernel + n, sizeof info->kernel - n, "_splitk%d", l->split_k);
  }
  if (g.batch > 1) {
    // a batch of products: only the LDS-direct kernel walks the batch index; batch strides keep the 16-byte alignment
    const int64_t align = in_dtype == STRIPE_I8 ? 16 : 8;
    if (l->variant < 20 || g.a_b % align || g.b_b % align || g.batch > 0x7fffffffLL / l->grid) return false;
    l->grid *= g.batch;
    info->grid = l->grid;
    const size_t n = strlen(info->kernel);
    snprintf(info->kernel + n, sizeof info->kernel - n, "_batch");
  }
  return true;
}

static bool gemm_select_one(const GemmShape& g, int in_dtype, GemmLaunch* l, stripe_block_info_t* info) {
  if (in_dtype == STRIPE_I8) {
    // int8 x int8 -> int32 with both operands k-contiguous (C = A * B^T); K tiles of 64 bytes, four in flight
    if (g.a_k != 1 || g.c_n != 1 || g.b_k != 1 || g.b_n == 1 || tune_int("gemm_dma", 1) == 0) return false;
    if (g.K % 256 || g.K < 256 || g.M < 1 || g.N < 8 || g.M > 0x7fffffff || g.N > 0x7fffffff) return false;
    if (g.a_m % 16 || g.b_n % 16 || g.a_base % 16 || g.b_base % 16) return false;   // 16-byte global loads
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    if (tiles_m > 32767 || tiles_n > 32767) return false;
    const bool ragged = (g.M % BM || g.N % BN);
    if (tiles_m * tiles_n * (g.batch > 1 ? g.batch : 1) <= 128 && g.M % T_BM == 0 && g.N % T_BN == 0 && tune_int("gemm_t128", 1) != 0 &&
        g.M / T_BM <= 32767 && g.N / T_BN <= 32767) {
      l->variant = 52;
      l->t128_waves = tune_int("gemm_t128_waves", 8) == 4 ? 4 : 8;
      l->grid = (g.M / T_BM) * (g.N / T_BN);
      info->path = STRIPE_PATH_MFMA_GEMM;
      info->tile_m = T_BM; info->tile_n = T_BN; info->tile_k = 64;
      info->frag_m = 32; info->frag_n = 32; info->frag_k = 32;
      info->lds_bytes = t128_lds_bytes(64);
      info->workgroup_size = 64 * l->t128_waves;
      info->grid = l->grid;
      snprintf(info->kernel, sizeof info->kernel, "gemm_i8_128x128x64_mfma32x32x32_w%d_lds_direct_bt", l->t128_waves);
      return true;
    }
    l->variant = 40 + (ragged ? D_RAGGED : 0);
    l->grid = tiles_m * tiles_n;
    info->path = STRIPE_PATH_MFMA_GEMM;
    info->tile_m = BM; info->tile_n = BN; info->tile_k = 64;
    info->frag_m = 32; info->frag_n = 32; info->frag_k = 32;
    info->lds_bytes = D_LDS;
    info->workgroup_size = 256;
    info->grid = l->grid;
    snprintf(info->kernel, sizeof info->kernel, "gemm_i8_256x256x64_mfma32x32x32_w4_lds_direct_bt%s", ragged ? "_ragged" : "");
    return true;
  }
  if (in_dtype != STRIPE_BF16) return false;
  if (g.a_k != 1 || g.c_n != 1) return false;
  // B row-major ([k][n], n contiguous) or transposed ([n][k], k contiguous); the LDS-direct kernel also takes
  // M and N that are not multiples of the tile (row-major B then needs whole 8-column chunks)
  const bool bt = g.b_k == 1 && g.b_n != 1;
  if (!bt && g.b_n != 1) return false;
  const int64_t b_row = bt ? g.b_n : g.b_k;
  const bool dma_shape = g.K % (D_BK * D_STAGES) == 0 && g.K >= D_BK * D_STAGES && tune_int("gemm_dma", 1) != 0;
  const bool ragged = (g.M % BM || g.N % BN);
  // few large tiles: 128 x 128 tiles put four times as many workgroups on the chip
  const int64_t big_tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN) * (g.batch > 1 ? g.batch : 1);
  if (dma_shape && big_tiles <= 128 && g.M % T_BM == 0 && g.N % T_BN == 0 && tune_int("gemm_t128", 1) != 0 &&
      g.a_m % 8 == 0 && b_row % 8 == 0 && g.a_base % 8 == 0 && g.b_base % 8 == 0 && g.M / T_BM <= 32767 && g.N / T_BN <= 32767) {
    l->variant = bt ? 51 : 50;
    l->t128_waves = tune_int("gemm_t128_waves", 8) == 4 ? 4 : 8;
    l->grid = (g.M / T_BM) * (g.N / T_BN);
    info->path = STRIPE_PATH_MFMA_GEMM;
    info->tile_m = T_BM; info->tile_n = T_BN; info->tile_k = D_BK;
    info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
    info->lds_bytes = t128_lds_bytes(64);
    info->workgroup_size = 64 * l->t128_waves;
    info->grid = l->grid;
    snprintf(info->kernel, sizeof info->kernel, "gemm_bf16_128x128x32_mfma32x32x16_w%d_lds_direct%s", l->t128_waves, bt ? "_bt" : "");
    return true;
  }
  if (bt || ragged) {
    if (!dma_shape || g.M < 1 || g.N < 8 || (!bt && g.N % 8) || g.M > 0x7fffffff || g.N > 0x7fffffff) return false;
    if (g.a_m % 8 || b_row % 8 || g.a_base % 8 || g.b_base % 8) return false;
    const int64_t tiles_m = (g.M + BM - 1) / BM, tiles_n = (g.N + BN - 1) / BN;
    if (tiles_m > 32767 || tiles_n > 32767) return false;
    l->variant = 30 + (bt ? D_BT : 0) + (ragged ? D_RAGGED : 0);
    l->grid = tiles_m * tiles_n;
    info->path = STRIPE_PATH_MFMA_GEMM;
    info->tile_m = BM; info->tile_n = BN; info->tile_k = D_BK;
    info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
    info->lds_bytes = D_LDS;
    info->workgroup_size = 256;
    info->grid = l->grid;
    snprintf(info->kernel, sizeof info->kernel, "gemm_bf16_256x256x32_mfma32x32x16_w4_lds_direct%s%s", bt ? "_bt" : "", ragged ? "_ragged" : "");
    return true;
  }
  if (g.M % BM || g.N % BN || g.K % BK || g.K < BK) return false;
  if (g.a_m % 8 || g.b_k % 8 || g.a_base % 8 || g.b_base % 8) return false;  // 16-byte global loads
  if (g.M / BM > 32767 || g.N / BN > 32767 || g.K / BK > 0x7fffffff / BK) return false;
  int swz = tune_int("gemm_swz", 2);
  if (swz < 0 || swz > 2) swz = 2;
  int waves = tune_int("gemm_waves", 4) == 8 ? 8 : 4;
  if ((g.K / BK) % 2) waves = 8;   // the four-wavefront pipeline consumes K tiles in pairs
  const bool dma = tune_int("gemm_dma", 1) != 0 && g.K % (D_BK * D_STAGES) == 0 && g.K >= D_BK * D_STAGES;
  const int dma_waves = tune_int("gemm_dma_waves", 4) == 8 ? 8 : 4;
  // 0: plain read order, 1: reads ahead of use and odd accumulator rows backwards (one operand stays between consecutive
  // matrix instructions: 114.3 -> 113.7 us on 4096^3, four alternating pairs), 2: reads ahead and the barrier before the last
  // instruction of its group, 3: reads ahead only
  int sched = tune_int("gemm_sched", 1);
  if (sched < 0 || sched > 3 || dma_waves == 8) sched = 1;
  l->variant = dma ? (dma_waves == 8 ? 21 : sched == 0 ? 22 : sched == 2 ? 23 : sched == 3 ? 24 : 20) : (waves == 8 ? 10 : 0) + swz;
  l->grid = (g.M / BM) * (g.N / BN);
  info->path = STRIPE_PATH_MFMA_GEMM;
  info->tile_m = BM; info->tile_n = BN; info->tile_k = dma ? D_BK : BK;
  info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
  info->lds_bytes = dma ? D_LDS : 2 * STAGE;
  info->workgroup_size = dma ? dma_waves * 64 : (waves == 8 ? THREADS : W4_THREADS);
  info->grid = l->grid;
  if (dma) snprintf(info->kernel, sizeof info->kernel, "gemm_bf16_256x256x32_mfma32x32x16_w%d_lds_direct%s", dma_waves,
                    sched == 0 ? "_s0" : sched == 2 ? "_s2" : sched == 3 ? "_s3" : "");
  else snprintf(info->kernel, sizeof info->kernel, "gemm_bf16_256x256x64_mfma32x32x16_w%d_swz%d", waves, swz);
  return true;
}

static hipError_t launch_gemm_epi(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, void* c, const float* bias, int epi,
                                  int64_t o_m, int64_t o_base, hipStream_t st);

bool gemm_can_fuse_bias_relu(const GemmShape& g, const GemmLaunch& l) {
  // the LDS-direct kernels in their float modes, one product (no batch, reduction not split)
  return g.batch <= 1 && l.split_k <= 1 && ((l.variant >= 20 && l.variant < 40) || l.variant == 50 || l.variant == 51);
}

hipError_t launch_gemm_bias_relu(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, const void* bias, void* out,
                                 int64_t o_m, int64_t o_base, bool out_bf16, hipStream_t st) {
  if (!gemm_can_fuse_bias_relu(g, l) || !bias || ((uintptr_t)bias % 4) || ((uintptr_t)out % (out_bf16 ? 2 : 4))) return hipErrorInvalidValue;
  return launch_gemm_epi(g, l, a, b, out, (const float*)bias, out_bf16 ? 2 : 1, o_m, o_base, st);
}

hipError_t launch_gemm(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, void* c, void* workspace, hipStream_t st) {
  if (l.split_k <= 1) return launch_gemm_epi(g, l, a, b, c, nullptr, 0, g.c_m, g.c_base, st);
  // S slices of the reduction index as a batch of S products into the workspace, then their sum into C
  if (!workspace || ((uintptr_t)workspace % 16) || ((uintptr_t)c % 4)) return hipErrorInvalidValue;
  const bool bt = g.b_k == 1 && g.b_n != 1;
  GemmShape slice = g;
  slice.K = g.K / l.split_k;
  slice.batch = l.split_k;
  slice.a_b = slice.K;                                  // A is k-contiguous
  slice.b_b = bt ? slice.K : slice.K * g.b_k;
  slice.c_b = g.M * g.N;
  const hipError_t e = launch_gemm_epi(slice, l, a, b, workspace, nullptr, 0, g.N, 0, st);
  if (e != hipSuccess) return e;
  const bool i8 = (l.variant >= 40 && l.variant < 50) || l.variant == 52;
  const bool vec4 = g.N % 4 == 0 && g.c_m % 4 == 0 && g.c_base % 4 == 0 && ((uintptr_t)c % 16) == 0;
  const int64_t items = g.M * (vec4 ? g.N / 4 : g.N);
  int G = 1;                                            // threads per item: enough workgroups to fill the chip
  while (G < 16 && 2 * G <= l.split_k && items * G < 1024 * 256) G *= 2;
  G = tune_int("gemm_reduce_g", G);
  if (G < 1 || G > 16 || (G & (G - 1))) return hipErrorInvalidValue;
  const int64_t wgs = (items * G + 255) / 256;
  const unsigned blocks = (unsigned)(wgs < 8192 ? wgs : 8192);
  if (i8) {
    if (vec4) hipLaunchKernelGGL((splitk_reduce_kernel<int, 4>), dim3(blocks), dim3(256), 0, st, (const int*)workspace, (int*)c, g.M, g.N, g.c_m, g.c_base, l.split_k, G);
    else hipLaunchKernelGGL((splitk_reduce_kernel<int, 1>), dim3(blocks), dim3(256), 0, st, (const int*)workspace, (int*)c, g.M, g.N, g.c_m, g.c_base, l.split_k, G);
  } else {
    if (vec4) hipLaunchKernelGGL((splitk_reduce_kernel<float, 4>), dim3(blocks), dim3(256), 0, st, (const float*)workspace, (float*)c, g.M, g.N, g.c_m, g.c_base, l.split_k, G);
    else hipLaunchKernelGGL((splitk_reduce_kernel<float, 1>), dim3(blocks), dim3(256), 0, st, (const float*)workspace, (float*)c, g.M, g.N, g.c_m, g.c_base, l.split_k, G);
  }
  return hipGetLastError();
}

static hipError_t launch_gemm_epi(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, void* c, const float* bias, int epi,
                                  int64_t o_m, int64_t o_base, hipStream_t st) {
  if (((uintptr_t)a % 16) || ((uintptr_t)b % 16) || ((uintptr_t)c % (epi == 2 ? 2 : 4))) return hipErrorInvalidValue;
  const bool i8 = (l.variant >= 40 && l.variant < 50) || l.variant == 52;
  const GemmParams p = make_params(g, i8);
  const bool t128_w8 = l.variant >= 50 && l.t128_waves == 8, t128_kb128 = t128_w8 && l.t128_kb == 128;
  void (*kernel)(const GemmParams, const uint16_t*, const uint16_t*, float*) = nullptr;
  switch (l.variant) {
    case 0: case 1: case 2: kernel = gemm_bf16_w4_kernel; break;
    case 20: kernel = gemm_bf16_dma_kernel<4, 1>; break;
    case 21: kernel = gemm_bf16_dma_kernel<8, 1>; break;
    case 22: kernel = gemm_bf16_dma_kernel<4, 0>; break;
    case 23: kernel = gemm_bf16_dma_kernel<4, 2>; break;
    case 24: kernel = gemm_bf16_dma_kernel<4, 3>; break;
    case 30 + D_BT: kernel = gemm_bf16_dma_kernel<4, 1, D_BT>; break;
    case 30 + D_RAGGED: kernel = gemm_bf16_dma_kernel<4, 1, D_RAGGED>; break;
    case 30 + D_BT + D_RAGGED: kernel = gemm_bf16_dma_kernel<4, 1, D_BT + D_RAGGED>; break;
    case 50: kernel = t128_kb128 ? gemm_bf16_t128_kernel<0, 1, 128> : t128_w8 ? gemm_bf16_t128_kernel<0, 1> : gemm_bf16_t128_kernel<0, 0>; break;
    case 51: kernel = t128_kb128 ? gemm_bf16_t128_kernel<D_BT, 1, 128> : t128_w8 ? gemm_bf16_t128_kernel<D_BT, 1> : gemm_bf16_t128_kernel<D_BT, 0>; break;
    case 52: kernel = t128_kb128 ? gemm_bf16_t128_kernel<D_BT + D_I8, 1, 128> : t128_w8 ? gemm_bf16_t128_kernel<D_BT + D_I8, 1> : gemm_bf16_t128_kernel<D_BT + D_I8, 0>; break;
    case 40: kernel = gemm_bf16_dma_kernel<4, 1, D_BT + D_I8>; break;
    case 40 + D_RAGGED: kernel = gemm_bf16_dma_kernel<4, 1, D_BT + D_RAGGED + D_I8>; break;
    case 10: kernel = gemm_bf16_w8_kernel<0>; break;
    case 11: kernel = gemm_bf16_w8_kernel<1>; break;
    default: kernel = gemm_bf16_w8_kernel<2>; break;
  }
  const int threads = (l.variant == 21 || (l.variant >= 10 && l.variant < 20) || t128_w8) ? THREADS : W4_THREADS;
  const int lds_bytes = l.variant >= 50 ? t128_lds_bytes(l.t128_kb) : l.variant >= 20 ? D_LDS : 2 * STAGE;
  GemmParams pk = p;
  if (l.variant >= 20) pk.k_tiles = (int)(g.K / ((i8 ? 64 : D_BK) * (t128_kb128 ? 2 : 1)));
  pk.bias = bias;
  pk.epi = epi;
  pk.c_m = o_m;
  pk.c_base = o_base;
  // 16-byte stores through LDS where the store phase is bound by its instructions: the fused forms (measured on
  // 4096^3: bf16 output 121.0 -> 117.5 us; the plain fp32 product is bound by the 67 MB it writes, 112.1 us with
  // 4-byte stores, 112.9 with these).  STRIPE_TUNE gemm_epi16 = 0: never, 1: also for plain products.
  const int epi16 = tune_int("gemm_epi16", -1);
  pk.vec_c = (l.variant >= 20 && l.variant < 50 && (epi16 == 1 || (epi16 != 0 && epi != 0)) && o_m % 4 == 0 && o_base % 4 == 0 &&
              g.c_b % 4 == 0 && (uintptr_t)c % (epi == 2 ? 8 : 16) == 0)
                 ? 1
                 : 0;
  if (l.variant >= 50) {
    pk.tiles_m = (int)(g.M / T_BM);
    pk.tiles_n = (int)(g.N / T_BN);
  }
  // more than 64 KB of dynamic LDS has to be enabled once per device
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {
    e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)l.grid), dim3(threads), lds_bytes, st, pk, (const uint16_t*)a,
                     (const uint16_t*)b, (float*)c);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Convolutions on the 256 x 256-tile kernel (its D_CONV mode): the nesting of paper Section 3.1.3 with the output
// pixels (flattened n, y, x) as the rows of A and the filter taps and channel chunks as the K walk -- Figure 5b's
// view by address arithmetic, as in the general convolution kernel, but with this kernel's 128 x 128 register tiles
// and schedule.  For convolutions large enough to fill the chip with such tiles.
// ---------------------------------------------------------------------------
bool conv_gemm_select(const Conv2dShape& c, int in_dtype, ConvLaunch* l, stripe_block_info_t* info) {
  const int mode = tune_int("conv_gemm", 1);   // 0: never, 2: whatever the tile count and the padding of the channel tile
  if (mode == 0 || in_dtype != STRIPE_BF16 || tune_int("gemm_dma", 1) == 0) return false;
  if (c.i_c != 1 || c.f_c != 1 || c.o_k != 1) return false;
  if (c.Ci % D_BK || c.R < 1 || c.S < 1 || c.R > 32 || c.S > 32 || c.Co < 8) return false;
  const int64_t k_tiles = c.R * c.S * (c.Ci / D_BK);
  if (k_tiles % D_STAGES || k_tiles < D_STAGES || k_tiles > 0x7fffffffLL) return false;
  if (c.stride_y < 1 || c.stride_x < 1 || c.dil_y < 1 || c.dil_x < 1 || c.pad_y < 0 || c.pad_x < 0) return false;
  for (int64_t v : {c.i_n, c.i_y, c.i_x, c.i_base, c.f_r, c.f_s, c.f_k, c.f_base})
    if (v % 8) return false;                   // 16-byte loads
  for (int64_t v : {c.N, c.Ho, c.Wo, c.H, c.W, c.Co, c.stride_y, c.stride_x, c.pad_y, c.pad_x, c.dil_y, c.dil_x})
    if (v > 0x3fffffff) return false;
  // pixel m = (n * Ho + y) * Wo + x at o_base + m * o_x: the output as a row-major matrix (strides of one-element indexes do not matter)
  if ((c.Ho > 1 && c.o_y != c.Wo * c.o_x) || (c.N > 1 && c.o_n != c.Ho * c.Wo * c.o_x)) return false;
  const int64_t m_total = c.N * c.Ho * c.Wo;
  if (m_total < 1 || m_total > 0x7fffffffLL - 512) return false;
  // every pixel has a tap inside the image in each direction, so every row of the output matrix is stored
  auto all_have_tap = [](int64_t outs, int64_t stride, int64_t pad, int64_t dil, int64_t taps, int64_t extent) {
    if (outs > ((int64_t)1 << 20)) return false;
    for (int64_t o = 0; o < outs; ++o) {
      bool any = false;
      for (int64_t i = 0; i < taps && !any; ++i) {
        const int64_t v = o * stride - pad + i * dil;
        any = v >= 0 && v < extent;
      }
      if (!any) return false;
    }
    return true;
  };
  if (!all_have_tap(c.Ho, c.stride_y, c.pad_y, c.dil_y, c.R, c.H) || !all_have_tap(c.Wo, c.stride_x, c.pad_x, c.dil_x, c.S, c.W)) return false;
  const int64_t tiles_m = (m_total + BM - 1) / BM, tiles_n = (c.Co + BN - 1) / BN;
  if (tiles_m > 32767 || tiles_n > 32767) return false;
  if (mode != 2 && (tiles_m * tiles_n < 128 || (tiles_n * BN - c.Co) * 4 > tiles_n * BN)) return false;   // fill the chip; at most a quarter of the channel tiles padding
  l->variant = kConvGemmVariant;
  l->in_dtype = in_dtype;
  l->grid = tiles_m * tiles_n;
  info->path = STRIPE_PATH_MFMA_CONV;
  info->tile_m = BM; info->tile_n = BN; info->tile_k = D_BK;
  info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
  info->lds_bytes = D_LDS;
  info->workgroup_size = 256;
  info->grid = l->grid;
  snprintf(info->kernel, sizeof info->kernel, "conv_gemm_bf16_256x256x32_mfma32x32x16_w4_lds_direct");
  return true;
}

// bias / epi: the fused form of a following statement O = relu(T + bias[k]); epi 1 = fp32 output, 2 = bf16 output (out then is O)
hipError_t launch_conv_gemm(const Conv2dShape& c, const ConvLaunch& l, const void* in, const void* flt, void* out, const void* bias, int epi,
                            hipStream_t st) {
  if (((uintptr_t)in % 16) || ((uintptr_t)flt % 16) || ((uintptr_t)out % (epi == 2 ? 2 : 4)) || ((uintptr_t)bias % 4) || (epi && !bias)) return hipErrorInvalidValue;
  GemmParams p = {};
  const int64_t m_total = c.N * c.Ho * c.Wo;
  p.tiles_m = (int)((m_total + BM - 1) / BM);
  p.tiles_n = (int)((c.Co + BN - 1) / BN);
  p.k_tiles = (int)(c.R * c.S * (c.Ci / D_BK));
  p.M = (int)m_total;
  p.N = (int)c.Co;
  p.a_m = 0; p.b_k = c.f_k; p.c_m = c.o_x;
  p.a_base = c.i_base; p.b_base = c.f_base; p.c_base = c.o_base;
  p.bias = (const float*)bias; p.epi = epi; p.vec_c = 0;
  p.cv_Ho = (int)c.Ho; p.cv_Wo = (int)c.Wo; p.cv_H = (int)c.H; p.cv_W = (int)c.W;
  p.cv_sy = (int)c.stride_y; p.cv_sx = (int)c.stride_x; p.cv_py = (int)c.pad_y; p.cv_px = (int)c.pad_x;
  p.cv_dy = (int)c.dil_y; p.cv_dx = (int)c.dil_x; p.cv_R = (int)c.R; p.cv_S = (int)c.S; p.cv_chunks = (int)(c.Ci / D_BK);
  p.cv_i_n = c.i_n; p.cv_i_y = c.i_y; p.cv_i_x = c.i_x; p.cv_f_r = c.f_r; p.cv_f_s = c.f_s;
  void (*kernel)(const GemmParams, const uint16_t*, const uint16_t*, float*) = gemm_bf16_dma_kernel<4, 1, D_BT + D_RAGGED + D_CONV>;
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {   // more than 64 KB of dynamic LDS has to be enabled once per device
    e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, D_LDS);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)l.grid), dim3(W4_THREADS), D_LDS, st, p, (const uint16_t*)in, (const uint16_t*)flt, (float*)out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------
// Matrix-core yardstick: the 4 x 4 fragment tile of the 256-tile kernel's wavefront with both operands resident in
// registers -- no LDS, no global traffic inside the loop.  Two sets of 4 + 4 operand fragments (loaded once from
// `operands`) take turns, so that the operands of consecutive matrix instructions differ as they do in the real
// kernel; what the loop reaches is the rate the chip sustains for this instruction on these operand values.
// ---------------------------------------------------------------------------
namespace {
// LDS: the operand fragments are fetched again from LDS before every pass (eight 16-byte reads per lane for sixteen
// matrix instructions, the real kernel's ratio), one pass ahead of their use.
template <bool LDS>
__global__ __launch_bounds__(256, 1) void mfma_probe_kernel(const bf16x8* __restrict__ operands, float* __restrict__ out, int iters) {
  __shared__ bf16x8 frag[LDS ? 16 * 256 : 1];
  const int t = threadIdx.x;
  bf16x8 a[2][4], b[2][4];
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      a[s][i] = operands[((s * 8 + i) * 256) + t];
      b[s][i] = operands[((s * 8 + 4 + i) * 256) + t];
      if constexpr (LDS) {
        frag[(s * 8 + i) * 256 + t] = a[s][i];
        frag[(s * 8 + 4 + i) * 256 + t] = b[s][i];
      }
    }
  if constexpr (LDS) __syncthreads();
  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
  for (int it = 0; it < iters; it += 2) {
#pragma unroll
    for (int s = 0; s < 2; ++s) {
      if constexpr (LDS) {   // the other set's fragments for the next pass (a lane reads what it wrote: no barrier needed)
        __builtin_amdgcn_sched_barrier(0);
        asm volatile("" ::: "memory");   // the fragments are fetched again, not kept from the previous pass
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          a[s ^ 1][i] = frag[((s ^ 1) * 8 + i) * 256 + t];
          b[s ^ 1][i] = frag[((s ^ 1) * 8 + 4 + i) * 256 + t];
        }
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int jj = (i & 1) ? 3 - j : j;   // the order of the real kernel: one operand stays between consecutive instructions
          acc[i][jj] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[s][i], b[s][jj], acc[i][jj], 0, 0, 0);
        }
      if constexpr (LDS) __builtin_amdgcn_sched_barrier(0);
    }
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) sum += acc[i][j][v];
  out[(size_t)blockIdx.x * 256 + t] = sum;
}
}  // namespace

hipError_t launch_mfma_probe(const void* operands, void* out, int iters, int grid, bool lds, hipStream_t st) {
  if (lds) hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16x8*)operands, (float*)out, iters);
  else hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3((unsigned)grid), dim3(256), 0, st, (const bf16x8*)operands, (float*)out, iters);
  return hipGetLastError();
}

}  // namespace stripe
