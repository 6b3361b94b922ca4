// bf16 MFMA matrix product  C[M, N] = A[M, K] . W[N, K]^T  with fused epilogues.
//
// Both operands are K-contiguous, so a lane's 8 consecutive k values are one 16-byte
// load and map directly onto the v_mfma_f32_32x32x16_bf16 operand registers.
//
// * Workgroup tile BM x BN x 64.  The 256 x 256 tile runs 8 waves (two per SIMD: one wave
//   alone cannot keep a matrix core issuing back to back), each owning 128 x 64.
// * LDS tiles are [row][64 bf16] with the 16-byte chunks XOR-swizzled by (row >> 1) & 7:
//   LDS serves a 16-byte-per-lane read 16 lanes at a time over 64 banks, and this
//   swizzle makes any 16 consecutive rows of one logical chunk hit 16 distinct bank groups.
// * Two LDS stages, one barrier per k-step, global loads for step k+1 in flight while step
//   k is multiplied.
// * The product is formed transposed (W fragment as the MFMA row operand), so a lane ends
//   up with four consecutive output columns of one token row per register quad.  The
//   epilogue adds bias, applies GELU / residual, converts, stages the 32 x TN block of a
//   wave through LDS and writes rows back with 16 bytes per lane.
// * Workgroup ids are dealt round-robin to the 8 XCDs; each XCD walks its own range of
//   row blocks in 8 x 4 tile groups so the tiles in flight on one XCD share A and W
//   slices in that XCD's L2.
#include "common.h"

namespace vitenc {

namespace {

constexpr int BK = 64;  // bf16 elements per k-step = 128 bytes = 8 chunks of 16 bytes
constexpr int GROUP_M = 8, GROUP_N = 4;

__device__ __forceinline__ uint32_t lds_off(int row, int chunk) {
  return (uint32_t)(row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
}

// One k-step of a row-major tile: thread t moves 16-byte chunk (t & 7) of row (t >> 3) (+ NT/8 per pass).
template <int LOADS, int NT>
__device__ __forceinline__ void tile_load(u32x4 (&r)[LOADS], const bf16_t* base, int ld, int tid, int kt) {
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int idx = tid + i * NT, row = idx >> 3, ch = idx & 7;
    r[i] = *(const u32x4*)(base + (size_t)row * ld + kt * BK + ch * 8);
  }
}
template <int LOADS, int NT>
__device__ __forceinline__ void tile_store(const u32x4 (&r)[LOADS], unsigned char* lds, int tid) {
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int idx = tid + i * NT, row = idx >> 3, ch = idx & 7;
    *(u32x4*)(lds + lds_off(row, ch)) = r[i];
  }
}

template <int BM, int BN, int WM, int WN, int EPI>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(const GemmArgs a, int tiles_m, int tiles_n,
                                                               int mt_per_xcd, int n_bands) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;  // per-wave tile
  constexpr int FM = TM / 32, FN = TN / 32;  // 32x32 MFMA blocks per wave
  constexpr int A_LOADS = BM * 8 / NT, B_LOADS = BN * 8 / NT;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");
  constexpr int STAGE_BF16 = TN * 2 + 16, STAGE_F32 = TN * 4 + 16;  // bytes per staged row (padded)
  static_assert(WM * WN * 32 * STAGE_F32 <= 2 * (BM + BN) * 128, "epilogue staging must fit in the tile buffers");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* sA = smem;                 // 2 stages x BM x 128 B
  unsigned char* sB = smem + 2 * BM * 128;  // 2 stages x BN x 128 B

  // ---- tile assignment (see header comment)
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int blk = q / (GROUP_M * GROUP_N), r = q - blk * (GROUP_M * GROUP_N);
  const int mb = blk / n_bands, nb = blk - mb * n_bands;
  const int m_local = mb * GROUP_M + r / GROUP_N;
  const int tile_m = xcd * mt_per_xcd + m_local, tile_n = nb * GROUP_N + (r % GROUP_N);
  if (m_local >= mt_per_xcd || tile_m >= tiles_m || tile_n >= tiles_n) return;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;
  const int lrow = lane & 31, lk = lane >> 5;

  const bf16_t* A = (const bf16_t*)a.A + (size_t)m0 * a.lda;
  const bf16_t* W = (const bf16_t*)a.W + (size_t)n0 * a.ldw;

  u32x4 ra[A_LOADS], rb[B_LOADS];
  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

  const int KT = a.K / BK;
  tile_load<A_LOADS, NT>(ra, A, a.lda, tid, 0);
  tile_load<B_LOADS, NT>(rb, W, a.ldw, tid, 0);
  tile_store<A_LOADS, NT>(ra, sA, tid);
  tile_store<B_LOADS, NT>(rb, sB, tid);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < KT) {
      tile_load<A_LOADS, NT>(ra, A, a.lda, tid, kt + 1);
      tile_load<B_LOADS, NT>(rb, W, a.ldw, tid, kt + 1);
    }
    const unsigned char* pa = sA + stage * BM * 128;
    const unsigned char* pb = sB + stage * BN * 128;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      bf16x8 fa[FM], fb[FN];
#pragma unroll
      for (int i = 0; i < FM; ++i)
        fa[i] = *(const bf16x8*)(pa + lds_off(wm * TM + i * 32 + lrow, ks * 2 + lk));
#pragma unroll
      for (int j = 0; j < FN; ++j)
        fb[j] = *(const bf16x8*)(pb + lds_off(wn * TN + j * 32 + lrow, ks * 2 + lk));
#pragma unroll
      for (int i = 0; i < FM; ++i)
#pragma unroll
        for (int j = 0; j < FN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      tile_store<A_LOADS, NT>(ra, sA + (stage ^ 1) * BM * 128, tid);
      tile_store<B_LOADS, NT>(rb, sB + (stage ^ 1) * BN * 128, tid);
    }
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j] is the transposed block: lane holds token row
  // m0 + wm*TM + 32i + lrow; register 4jj + e holds output column n0 + wn*TN + 32j + 8jj + 4lk + e.
  const int ncol0 = n0 + wn * TN;  // first column of this wave
  f32x4 bias[FN][4];
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) bias[j][jj] = *(const f32x4*)(a.bias + ncol0 + j * 32 + jj * 8 + lk * 4);

  if constexpr (EPI == EPI_PATCH) {
    // rows are (tile, patch); the residual stream row is tile*T + cls + patch and the position row is added
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = m0 + wm * TM + i * 32 + lrow;
      if (row >= a.M) continue;
      const int tile = row / a.patches, tok = a.cls + (row - tile * a.patches);
      float* xr = a.resid + ((size_t)tile * a.tokens + tok) * a.ldo;
      const float* pr = a.pos + (size_t)tok * a.ldo;
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          const int col = ncol0 + j * 32 + jj * 8 + lk * 4;
          if (col < a.N) {
            const f32x4 p = *(const f32x4*)(pr + col);
            f32x4 v;
#pragma unroll
            for (int e = 0; e < 4; ++e) v[e] = acc[i][j][jj * 4 + e] + bias[j][jj][e] + p[e];
            *(f32x4*)(xr + col) = v;
          }
        }
    }
  } else if constexpr (EPI == EPI_BIAS_RESIDUAL) {
    unsigned char* st = smem + wave * 32 * STAGE_F32;  // this wave's private staging rows
    constexpr int LPR = TN / 4;                        // lanes per staged row (16 bytes each)
    constexpr int RPI = 64 / LPR;                      // rows per pass
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = acc[i][j][jj * 4 + e] + bias[j][jj][e];
          *(f32x4*)(st + lrow * STAGE_F32 + (j * 32 + jj * 8 + lk * 4) * 4) = v;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 32 / RPI; ++p) {
        const int sr = p * RPI + lane / LPR, sc = (lane % LPR) * 4;
        const int row = m0 + wm * TM + i * 32 + sr, col = ncol0 + sc;
        const f32x4 v = *(const f32x4*)(st + sr * STAGE_F32 + sc * 4);
        if (row < a.M && col < a.N) {
          float* xp = a.resid + (size_t)row * a.ldo + col;
          f32x4 x = *(const f32x4*)xp;
          x += v;
          *(f32x4*)xp = x;
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  } else {  // EPI_BIAS, EPI_BIAS_GELU: bf16 output
    unsigned char* st = smem + wave * 32 * STAGE_BF16;
    constexpr int LPR = TN / 8;  // lanes per staged row (16 bytes = 8 bf16 each)
    constexpr int RPI = 64 / LPR;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = acc[i][j][jj * 4 + e] + bias[j][jj][e];
            if constexpr (EPI == EPI_BIAS_GELU) v[e] = gelu_fast(v[e]);
          }
          const u32x2 pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
          *(u32x2*)(st + lrow * STAGE_BF16 + (j * 32 + jj * 8 + lk * 4) * 2) = pk;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 32 / RPI; ++p) {
        const int sr = p * RPI + lane / LPR, sc = (lane % LPR) * 8;
        const int row = m0 + wm * TM + i * 32 + sr, col = ncol0 + sc;
        const u32x4 v = *(const u32x4*)(st + sr * STAGE_BF16 + sc * 2);
        if (row < a.M && col < a.N) *(u32x4*)((bf16_t*)a.out + (size_t)row * a.ldo + col) = v;
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t s) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int mt_per_xcd = (tiles_m + 7) / 8;
  const int n_bands = (tiles_n + GROUP_N - 1) / GROUP_N;
  const int m_blocks = (mt_per_xcd + GROUP_M - 1) / GROUP_M;
  const long grid = 8L * m_blocks * n_bands * GROUP_M * GROUP_N;
  if (grid > 0x7fffffffL) return hipErrorInvalidValue;
  const size_t smem = 2 * (BM + BN) * 128;
  dim3 block(WM * WN * 64);
#define VIT_LAUNCH(EPI)                                                                                              \
  do {                                                                                                               \
    auto kfn = gemm_bf16_kernel<BM, BN, WM, WN, EPI>;                                                                \
    static bool attr_set = false; /* raising the dynamic LDS limit is needed once per kernel */                      \
    if (!attr_set) {                                                                                                 \
      hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);   \
      if (e != hipSuccess) return e;                                                                                 \
      attr_set = true;                                                                                               \
    }                                                                                                                \
    hipLaunchKernelGGL(kfn, dim3((unsigned)grid), block, smem, s, a, tiles_m, tiles_n, mt_per_xcd, n_bands);         \
  } while (0)
  switch (a.epilogue) {
    case EPI_BIAS: VIT_LAUNCH(EPI_BIAS); break;
    case EPI_BIAS_GELU: VIT_LAUNCH(EPI_BIAS_GELU); break;
    case EPI_BIAS_RESIDUAL: VIT_LAUNCH(EPI_BIAS_RESIDUAL); break;
    case EPI_PATCH: VIT_LAUNCH(EPI_PATCH); break;
    default: return hipErrorInvalidValue;
  }
#undef VIT_LAUNCH
  return hipGetLastError();
}

}  // namespace

int gemm_row_pad() { return 256; }

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  // 16-byte epilogue accesses need 8-element aligned columns and leading dimensions
  if (a.K <= 0 || a.K % BK != 0 || a.lda % 8 != 0 || a.ldw % 8 != 0 || a.ldo % 8 != 0 || a.N % 8 != 0)
    return hipErrorInvalidValue;
  // Large tiles need enough of them to fill 256 compute units.
  const long big_tiles = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (big_tiles >= 512) return launch_cfg<256, 256, 2, 4>(a, s);
  return launch_cfg<128, 128, 2, 2>(a, s);
}

}  // namespace vitenc
