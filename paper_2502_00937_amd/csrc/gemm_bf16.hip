// bf16 MFMA matrix product  C[M, N] = A[M, K] . W[N, K]^T  with fused epilogues.
//
// Both operands are K-contiguous, so a lane's 8 consecutive k values are one 16-byte
// load and map directly onto the v_mfma_f32_32x32x16_bf16 operand registers.
// Workgroup tile BM x BN x 64, staged through LDS with an XOR swizzle of the 16-byte
// chunks (chunk ^ (row & 7)) so that both the 16-byte tile writes and the MFMA
// fragment reads are bank-conflict free; two LDS stages, one barrier per k-step,
// global loads for step k+1 in flight while step k is multiplied.
#include "common.h"

namespace vitenc {

namespace {

constexpr int BK = 64;  // bf16 elements per k-step = 128 bytes = 8 chunks of 16 bytes

__device__ inline uint32_t lds_off(int row, int chunk) { return (uint32_t)(row * 128 + ((chunk ^ (row & 7)) << 4)); }

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

template <int BM, int BN, int WM, int WN, int EPI, typename OutT>
__global__ __launch_bounds__(WM* WN * 64) void gemm_bf16_kernel(const GemmArgs a, int tiles_n, int total_tiles) {
  constexpr int NT = WM * WN * 64;
  constexpr int TM = BM / WM, TN = BN / WN;  // per-wave tile
  constexpr int FM = TM / 32, FN = TN / 32;  // 32x32 MFMA blocks per wave
  constexpr int A_LOADS = BM * 8 / NT, B_LOADS = BN * 8 / NT;
  static_assert(BM * 8 % NT == 0 && BN * 8 % NT == 0, "tile/threads mismatch");

  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* sA = smem;                  // 2 stages x BM x 128 B
  unsigned char* sB = smem + 2 * BM * 128;   // 2 stages x BN x 128 B

  // Workgroups are dealt round-robin to the 8 XCDs; give each XCD a contiguous run of
  // logical tiles (n fastest) so tiles sharing an A row block meet in one L2.
  int pid = blockIdx.x;
  int per_xcd = (total_tiles + 7) >> 3;
  int logical = (pid & 7) * per_xcd + (pid >> 3);
  if (logical >= total_tiles) return;
  const int tile_m = logical / tiles_n, tile_n = logical - tile_m * tiles_n;
  const int m0 = tile_m * BM, n0 = tile_n * BN;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave / WN, wn = wave % WN;

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

  const int lrow = lane & 31, lk = lane >> 5;
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
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    if (kt + 1 < KT) {
      tile_store<A_LOADS, NT>(ra, sA + (stage ^ 1) * BM * 128, tid);
      tile_store<B_LOADS, NT>(rb, sB + (stage ^ 1) * BN * 128, tid);
    }
    __syncthreads();
  }

  // C layout of the 32x32 MFMA: lane holds column lane%32; register v holds row
  // 8*(v/4) + 4*(lane/32) + v%4.
#pragma unroll
  for (int i = 0; i < FM; ++i) {
#pragma unroll
    for (int j = 0; j < FN; ++j) {
      const int col = n0 + wn * TN + j * 32 + lrow;
      if (col >= a.N) continue;
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int row = m0 + wm * TM + i * 32 + 8 * (v >> 2) + 4 * lk + (v & 3);
        if (row < a.M) epilogue_store<EPI, OutT>(a, row, col, acc[i][j][v]);
      }
    }
  }
}

template <int BM, int BN, int WM, int WN>
hipError_t launch_cfg(const GemmArgs& a, hipStream_t s) {
  const int tiles_m = (a.M + BM - 1) / BM, tiles_n = (a.N + BN - 1) / BN;
  const int total = tiles_m * tiles_n;
  const int grid = ((total + 7) / 8) * 8;
  const size_t smem = 2 * (BM + BN) * 128;
  dim3 block(WM * WN * 64);
#define VIT_LAUNCH(EPI, OutT)                                                                             \
  do {                                                                                                    \
    auto kfn = gemm_bf16_kernel<BM, BN, WM, WN, EPI, OutT>;                                               \
    static bool attr_set = false; /* raising the dynamic LDS limit is needed once per kernel */           \
    if (!attr_set) {                                                                                      \
      hipError_t e = hipFuncSetAttribute((const void*)kfn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem); \
      if (e != hipSuccess) return e;                                                                      \
      attr_set = true;                                                                                    \
    }                                                                                                     \
    hipLaunchKernelGGL(kfn, dim3(grid), block, smem, s, a, tiles_n, total);                               \
  } while (0)
  switch (a.epilogue) {
    case EPI_BIAS: VIT_LAUNCH(EPI_BIAS, bf16_t); break;
    case EPI_BIAS_GELU: VIT_LAUNCH(EPI_BIAS_GELU, bf16_t); break;
    case EPI_BIAS_RESIDUAL: VIT_LAUNCH(EPI_BIAS_RESIDUAL, bf16_t); break;
    case EPI_PATCH: VIT_LAUNCH(EPI_PATCH, bf16_t); break;
    default: return hipErrorInvalidValue;
  }
#undef VIT_LAUNCH
  return hipGetLastError();
}

}  // namespace

int gemm_row_pad() { return 256; }

hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.K <= 0 || a.K % BK != 0 || a.lda % 8 != 0 || a.ldw % 8 != 0) return hipErrorInvalidValue;
  // Large tiles need enough of them to fill 256 compute units.
  const long big_tiles = (long)((a.M + 255) / 256) * ((a.N + 255) / 256);
  if (big_tiles >= 512) return launch_cfg<256, 256, 2, 2>(a, s);
  return launch_cfg<128, 128, 2, 2>(a, s);
}

}  // namespace vitenc
