// Nested-tile dense contraction on the gfx950 matrix cores:
//   C[m,n] = sum_k A[m,k] * B[k,n],  bf16 inputs, fp32 accumulate and output.
//
// The three nesting levels of the Stripe block (paper Section 3.1.3; Figure 3's
// columns) are mapped by hand:
//   outer block  -> one workgroup per BM x BN tile of C (XCD-aware tile order),
//   middle block -> K tiles of BK staged in LDS, double-buffered,
//   inner block  -> v_mfma_f32_32x32x16_bf16 fragments, 4 x 2 per wavefront.
// The "microarchitectural transposition" the matrix core needs (Section 2.3) is
// done on the way into LDS: both operands are stored K-contiguous per row
// (A as [m][k], B transposed to [n][k]) in 128-byte rows whose 16-byte chunks
// are XOR-swizzled with the row number, so fragment reads (16 bytes per lane)
// spread over all banks.
#include <hip/hip_runtime.h>

#include "kernels.hpp"

namespace stripe {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) unsigned u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned u32x2;

struct GemmParams {
  int32_t tiles_m, tiles_n, k_tiles, pad_;
  int64_t a_m, b_k, c_m;      // row strides in elements (a_k = b_n = c_n = 1)
  int64_t a_base, b_base, c_base;
};

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int WAVES_M = 2, WAVES_N = 4;            // 8 wavefronts, 512 lanes
constexpr int WM = BM / WAVES_M, WN = BN / WAVES_N;  // 128 x 64 per wavefront
constexpr int FM = WM / 32, FN = WN / 32;          // 4 x 2 fragments of 32 x 32
constexpr int ROW_BYTES = BK * 2;                  // 128
constexpr int A_STAGE = BM * ROW_BYTES;            // 32 KB
constexpr int B_STAGE = BN * ROW_BYTES;            // 32 KB
constexpr int STAGE = A_STAGE + B_STAGE;           // 64 KB, two stages = 128 KB of the 160 KB LDS
constexpr int THREADS = 512;

// Which 16-byte slot of its 128-byte row chunk c of row r lives in.
template <int SWZ>
__device__ __forceinline__ int slot(int row, int c) {
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
__global__ __launch_bounds__(THREADS, 1) void gemm_bf16_kernel(const GemmParams p, const uint16_t* __restrict__ A,
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
  // B tile: 64 k x 256 n; lane t takes the 4(k) x 8(n) patch at k = 4*(t>>5), n = 8*(t&31).
  const int b_nb = t & 31, b_kq = t >> 5;
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

GemmParams make_params(const GemmShape& g) {
  GemmParams p;
  p.tiles_m = (int)(g.M / BM);
  p.tiles_n = (int)(g.N / BN);
  p.k_tiles = (int)(g.K / BK);
  p.pad_ = 0;
  p.a_m = g.a_m; p.b_k = g.b_k; p.c_m = g.c_m;
  p.a_base = g.a_base; p.b_base = g.b_base; p.c_base = g.c_base;
  return p;
}

}  // namespace

bool gemm_select(const GemmShape& g, int in_dtype, GemmLaunch* l, stripe_block_info_t* info) {
  if (in_dtype != STRIPE_BF16) return false;
  if (g.a_k != 1 || g.b_n != 1 || g.c_n != 1) return false;
  if (g.M % BM || g.N % BN || g.K % BK || g.K < BK) return false;
  if (g.a_m % 8 || g.b_k % 8 || g.a_base % 8 || g.b_base % 8) return false;  // 16-byte global loads
  if (g.M / BM > 32767 || g.N / BN > 32767 || g.K / BK > 0x7fffffff / BK) return false;
  l->variant = tune_int("gemm_swz", 1) ? 1 : 0;
  l->grid = (g.M / BM) * (g.N / BN);
  info->path = STRIPE_PATH_MFMA_GEMM;
  info->tile_m = BM; info->tile_n = BN; info->tile_k = BK;
  info->frag_m = 32; info->frag_n = 32; info->frag_k = 16;
  info->lds_bytes = 2 * STAGE;
  info->workgroup_size = THREADS;
  info->grid = l->grid;
  snprintf(info->kernel, sizeof info->kernel, "gemm_bf16_256x256x64_mfma32x32x16_swz%d", l->variant);
  return true;
}

hipError_t launch_gemm(const GemmShape& g, const GemmLaunch& l, const void* a, const void* b, void* c, hipStream_t st) {
  if (((uintptr_t)a % 16) || ((uintptr_t)b % 16) || ((uintptr_t)c % 4)) return hipErrorInvalidValue;
  const GemmParams p = make_params(g);
  auto kernel = l.variant == 1 ? gemm_bf16_kernel<1> : gemm_bf16_kernel<0>;
  // more than 64 KB of dynamic LDS has to be enabled once per device
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev != l.lds_enabled_on) {
    e = hipFuncSetAttribute((const void*)kernel, hipFuncAttributeMaxDynamicSharedMemorySize, 2 * STAGE);
    if (e != hipSuccess) return e;
    l.lds_enabled_on = dev;
  }
  hipLaunchKernelGGL(kernel, dim3((unsigned)l.grid), dim3(THREADS), 2 * STAGE, st, p, (const uint16_t*)a,
                     (const uint16_t*)b, (float*)c);
  return hipGetLastError();
}

}  // namespace stripe
