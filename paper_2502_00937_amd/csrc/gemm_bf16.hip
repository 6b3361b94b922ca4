// bf16 MFMA matrix product  C[M, N] = A[M, K] . W[N, K]^T  with fused epilogues.
//
// Both operands are K-contiguous, so a lane's 8 consecutive k values are one 16-byte
// load and map directly onto the v_mfma_f32_32x32x16_bf16 operand registers.
//
// Two kernels share the fragment layout and the epilogues; both move their operands global -> LDS
// directly (global_load_lds_dwordx4) and are described where they are defined:
// * gemm_bf16_ring_kernel (below 384 tiles of 256 x 256, and short last rounds of the large kernel): one 128 x 128
//   (or 64 x 128) tile per workgroup, eight
//   waves of 64 x 32, a ring of four (or two) 64-wide k-stages;
// * gemm_bf16_dma_kernel (everything large): persistent, 256 x 256 tiles, eight waves of 128 x 64,
//   two 64-wide k-stages.
// * LDS tiles are [row][64 bf16] with the 16-byte chunks XOR-swizzled by (row >> 1) & 7:
//   LDS serves a 16-byte-per-lane read 16 lanes at a time over 64 banks, and this
//   swizzle makes any 16 consecutive rows of one logical chunk hit 16 distinct bank groups.
// * The product is formed transposed (W fragment as the MFMA row operand), so a lane ends
//   up with four consecutive output columns of one token row per register quad.  The
//   epilogue adds bias, applies GELU / residual, converts, stages the 32 x TN block of a
//   wave through LDS and writes rows back with 16 bytes per lane.
// * Workgroup ids are dealt round-robin to the 8 XCDs; each XCD walks its own range of
//   row blocks in 8 x 4 tile groups so the tiles in flight on one XCD share A and W
//   slices in that XCD's L2.
#include <type_traits>

#include "common.h"

namespace vitenc {

namespace {

constexpr int BK = 64;  // bf16 elements per k-step = 128 bytes = 8 chunks of 16 bytes
constexpr int GROUP_M = 8, GROUP_N = 4;

// Epilogue of one wave.  acc[i][j] is a transposed 32x32 block: the lane holds token row
// row0 + 32i + (lane & 31); register 4jj + e holds output column ncol0 + 32j + 8jj + 4(lane >> 5) + e.
// `smem` is free LDS (all waves are past their last tile read); each wave stages its own rows.
template <int EPI, int FM, int FN>
__device__ __forceinline__ void wave_epilogue(const GemmArgs& a, f32x16 (&acc)[FM][FN], unsigned char* smem, int row0,
                                              int ncol0, int wave, int lane) {
  constexpr int TN = FN * 32;
  constexpr int STAGE_BF16 = TN * 2 + 16, STAGE_F32 = TN * 4 + 16;  // bytes per staged row (padded)
  const int lrow = lane & 31, lk = lane >> 5;
  f32x4 bias[FN][4];
#pragma unroll
  for (int j = 0; j < FN; ++j)
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) bias[j][jj] = *(const f32x4*)(a.bias + ncol0 + j * 32 + jj * 8 + lk * 4);

  if constexpr (EPI == EPI_PATCH) {
    // rows are (tile, patch); the residual stream row is tile*T + cls + patch and the position row is added
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      const int row = row0 + i * 32 + lrow;
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
        const int row = row0 + i * 32 + sr, col = ncol0 + sc;
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
    float cs[FN][4];  // scale of each accumulator quad: the query columns' (see GemmArgs::q_cols), 1/2 ahead of GELU; the bias is scaled with it
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        cs[j][jj] = EPI == EPI_BIAS_GELU ? 0.5f : ncol0 + j * 32 + jj * 8 + lk * 4 < a.q_cols ? a.q_scale : 1.0f;
        bias[j][jj] *= cs[j][jj];
      }
    unsigned char* st = smem + wave * 32 * STAGE_BF16;
    constexpr int LPR = TN / 8;  // lanes per staged row (16 bytes = 8 bf16 each)
    constexpr int RPI = 64 / LPR;
    // EPI_BIAS_HEADS: heads of 64 or 128 columns stored one after the other, so the wave's TN columns lie inside
    // one head: a row stride and the offset of column ncol0, both wave-uniform
    const int hm_blk = EPI == EPI_BIAS_HEADS ? ncol0 / a.hm_dh : 0;
    const int rs = EPI == EPI_BIAS_HEADS ? a.hm_dh : a.ldo;
    const size_t col0_off =
        EPI == EPI_BIAS_HEADS ? (size_t)hm_blk * a.hm_rows * a.hm_dh + (ncol0 - hm_blk * a.hm_dh) : (size_t)ncol0;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = fmaf(acc[i][j][jj * 4 + e], cs[j][jj], bias[j][jj][e]);
            if constexpr (EPI == EPI_BIAS_GELU) v[e] = gelu_fast_half(v[e]);
          }
          const u32x2 pk = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
          *(u32x2*)(st + lrow * STAGE_BF16 + (j * 32 + jj * 8 + lk * 4) * 2) = pk;
        }
      __builtin_amdgcn_wave_barrier();
#pragma unroll
      for (int p = 0; p < 32 / RPI; ++p) {
        const int sr = p * RPI + lane / LPR, sc = (lane % LPR) * 8;
        const int row = row0 + i * 32 + sr, col = ncol0 + sc;
        const u32x4 v = *(const u32x4*)(st + sr * STAGE_BF16 + sc * 2);
        if (row < a.M && col < a.N) *(u32x4*)((bf16_t*)a.out + (size_t)row * rs + col0_off + sc) = v;
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Large-problem kernel: persistent, 256 x 256 tile, eight waves (two per SIMD), 128 x 64 per wave.
//
// The memory system, not the matrix cores, sets the pace of this product on gfx950.  A compute
// unit's L1 is filled in whole 128-byte lines: a probe that reads L2-resident rows in 64-byte
// pieces gets 70 GB/s per unit, in 128-byte pieces 135 GB/s.  A 256 x 256 tile needs 32 KiB per
// 32 k-values, which at full MFMA rate is 60 GB/s: affordable only when every line is asked for
// once.  Hence 64-wide k-stages (one 128-byte line per row) and the biggest tile the accumulators
// allow.
//
// * One workgroup per compute unit walks a list of tiles.  Operand tiles go global -> LDS directly
//   (global_load_lds_dwordx4: each lane supplies its own global offset, the wave writes 1 KiB of
//   consecutive LDS = 8 rows) through two 64-wide k-stages of 64 KiB.  The stream of stages does
//   not stop at tile boundaries, so the next tile's first stages land while the current tile
//   finishes and its epilogue runs; no launch gap, no cold prologue per tile.
// * A stage is multiplied in four 16-wide sub-steps, each reading the next sub-step's fragments
//   while its own MFMAs run.  Before the last sub-step one wait + barrier establishes both that
//   the other stage has landed and that nobody reads this stage's LDS any more; the last sub-step
//   then reads the other stage's first fragments and issues the loads that refill this stage, one
//   after each MFMA (a wave that issued them back to back would sit in the memory pipeline's
//   back-pressure while the matrix core runs dry).
// * LDS rows are 128 bytes; the 16-byte chunk index is XORed with (row >> 1) & 7, which the lane
//   achieves by choosing which global chunk it loads, so any 16 consecutive rows of one logical
//   chunk fall on 16 distinct 16-byte bank groups of the 64 banks.
// * Tile order: the tile grid is cut into (8-row-block x 4-column-band) groups of 32 tiles, one per
//   compute unit of an XCD (a remainder of one or two tile columns is cut into 32 x 1 or 16 x 2
//   groups); consecutive groups along N go to consecutive XCDs, so the XCDs working at the same
//   time share A rows (first fetch fills the memory-side cache for the others) and the 32 units of
//   one XCD share both operands in its L2.
// * Epilogue staging has its own 18 KiB of LDS (16 rows x 144 bytes per wave).
constexpr int D_BM = 256, D_BN = 256, D_BK = 64, D_ST = 2;
constexpr int D_ROW = D_BK * 2;                       // bytes per LDS row
constexpr int D_STAGE_BYTES = (D_BM + D_BN) * D_ROW;  // 64 KiB
constexpr int D_STAGING_ROW = 144, D_STAGING_BYTES = 8 * 16 * D_STAGING_ROW;
constexpr int D_LDS_BYTES = D_ST * D_STAGE_BYTES + D_STAGING_BYTES;  // 146 KiB of the 160 KiB
constexpr int D_GROUP_M = 8, D_GROUP_N = 4;
constexpr int D_LOADS = 8;  // direct-to-LDS instructions per wave and stage (4 for A, 4 for W), 8 rows each

typedef const __attribute__((address_space(1))) void* gptr_t;
typedef __attribute__((address_space(3))) void* lptr_t;

// Epilogue of one wave of the persistent kernel: same register layout as wave_epilogue, but staged
// 16 rows at a time through the wave's private 16 x 144-byte LDS rows (`st`).
template <int EPI, bool STREAM_OUT, bool FULL>
__device__ __forceinline__ void wave_epilogue_p(const GemmArgs& a, f32x16 (&acc)[4][2], unsigned char* st, int row0,
                                                int ncol0, int lane) {
  constexpr int FM = 4, FN = 2;
  const int lrow = lane & 31, lk = lane >> 5;
  f32x4 bias[FN][4];  // per accumulator quad (the fp32 paths add their bias after the LDS round trip instead)
  if constexpr (EPI == EPI_BIAS || EPI == EPI_BIAS_GELU || EPI == EPI_BIAS_HEADS) {
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) bias[j][jj] = *(const f32x4*)(a.bias + ncol0 + j * 32 + jj * 8 + lk * 4);
  }

  if constexpr (EPI == EPI_PATCH) {
    // rows are (tile, patch); the residual stream row is tile * T + cls + patch, and that token's position row is
    // added.  Staged like the residual epilogue below (16 rows x 32 fp32 columns per piece, read back as 8 lanes
    // per row), so that the stream is written and the position table read in whole 128-byte row pieces; the row
    // mapping of a 32-row block is worked out once and serves both of its column blocks.
    const int sr0 = lane >> 3, sc = (lane & 7) * 4;
    f32x4 brow[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) brow[j] = *(const f32x4*)(a.bias + ncol0 + j * 32 + sc);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      size_t dst_off[2][2], pos_off[2][2];  // [half][pass], in elements, of this lane's row
      bool ok[2][2];
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const int row = row0 + i * 32 + half * 16 + p * 8 + sr0;
          ok[half][p] = FULL || row < a.M;
          const int rr = ok[half][p] ? row : 0;
          const int tile = rr / a.patches, tok = a.cls + (rr - tile * a.patches);
          dst_off[half][p] = ((size_t)tile * a.tokens + tok) * a.ldo;
          pos_off[half][p] = (size_t)tok * a.ldo;
        }
#pragma unroll
      for (int j = 0; j < FN; ++j) {
        const int col = ncol0 + j * 32 + sc;
        const bool col_ok = FULL || col < a.N;
        f32x4 posv[2][2];
#pragma unroll
        for (int half = 0; half < 2; ++half)
#pragma unroll
          for (int p = 0; p < 2; ++p)
            posv[half][p] = ok[half][p] && col_ok ? *(const f32x4*)(a.pos + pos_off[half][p] + col) : f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int half = 0; half < 2; ++half) {
          if ((lrow >> 4) == half) {
#pragma unroll
            for (int jj = 0; jj < 4; ++jj) {
              const f32x4 v = {acc[i][j][jj * 4], acc[i][j][jj * 4 + 1], acc[i][j][jj * 4 + 2], acc[i][j][jj * 4 + 3]};
              *(f32x4*)(st + (lrow & 15) * D_STAGING_ROW + (jj * 8 + lk * 4) * 4) = v;
            }
          }
          __builtin_amdgcn_wave_barrier();
#pragma unroll
          for (int p = 0; p < 2; ++p) {
            const f32x4 t = *(const f32x4*)(st + (p * 8 + sr0) * D_STAGING_ROW + sc * 4);
            if (ok[half][p] && col_ok) *(f32x4*)(a.resid + dst_off[half][p] + col) = posv[half][p] + (t + brow[j]);
          }
          __builtin_amdgcn_wave_barrier();
        }
      }
    }
  } else if constexpr (EPI == EPI_BIAS_RESIDUAL) {
    // Pieces of 16 rows x 32 fp32 columns (128 bytes + pad per staged row); a piece is read back
    // as 8 lanes per row, 8 rows per pass, and the bias is added there (one float4 per lane and column
    // block instead of one per accumulator quad).  The residual values of a 32 x 32 unit are loaded one
    // unit ahead; two, three and up to five units ahead (the registers of the next tile's first fragments
    // are free here, see the kernel) measured the same or slower: the epilogue is not bound by the latency
    // of these loads.  Addresses are a wave-uniform base (scalar arithmetic) plus a per-lane byte offset
    // that never changes; FULL tiles (all but the last row block and a ragged last column) carry no bounds
    // test.
    const int sr0 = lane >> 3, sc = (lane & 7) * 4;
    const uint32_t lane_off = (uint32_t)(sr0 * a.ldo + sc) * 4u;
    unsigned char* const tile_base = (unsigned char*)a.resid + ((size_t)row0 * a.ldo + ncol0) * 4;
    const int row_lim = a.M - row0 - sr0, col_lim = a.N - ncol0 - sc;  // valid: row offset < row_lim, col offset < col_lim
    auto x_ptr = [&](int i, int j, int half, int p) {
      return (float*)(tile_base + ((size_t)(i * 32 + half * 16 + p * 8) * a.ldo + j * 32) * 4 + lane_off);
    };
    auto x_ok = [&](int i, int j, int half, int p) {
      return FULL || (i * 32 + half * 16 + p * 8 < row_lim && j * 32 < col_lim);
    };
    f32x4 brow[FN];
#pragma unroll
    for (int j = 0; j < FN; ++j) brow[j] = *(const f32x4*)(a.bias + ncol0 + j * 32 + sc);
    f32x4 xin[2][2][2];  // [buffer][half][pass] of one unit
    auto load_unit = [&](int u, int buf) {  // unit u = i * FN + j
      const int i = u / FN, j = u % FN;
#pragma unroll
      for (int half = 0; half < 2; ++half)
#pragma unroll
        for (int p = 0; p < 2; ++p)
          xin[buf][half][p] = x_ok(i, j, half, p) ? *(const f32x4*)x_ptr(i, j, half, p) : f32x4{0.f, 0.f, 0.f, 0.f};
    };
    load_unit(0, 0);
#pragma unroll
    for (int u = 0; u < FM * FN; ++u) {
      const int i = u / FN, j = u % FN;
      if (u + 1 < FM * FN) load_unit(u + 1, (u + 1) & 1);
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if ((lrow >> 4) == half) {
#pragma unroll
          for (int jj = 0; jj < 4; ++jj) {
            const f32x4 v = {acc[i][j][jj * 4], acc[i][j][jj * 4 + 1], acc[i][j][jj * 4 + 2], acc[i][j][jj * 4 + 3]};
            *(f32x4*)(st + (lrow & 15) * D_STAGING_ROW + (jj * 8 + lk * 4) * 4) = v;
          }
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < 2; ++p) {
          const f32x4 t = *(const f32x4*)(st + (p * 8 + sr0) * D_STAGING_ROW + sc * 4);
          if (x_ok(i, j, half, p)) *(f32x4*)x_ptr(i, j, half, p) = xin[u & 1][half][p] + (t + brow[j]);
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
  } else {  // EPI_BIAS, EPI_BIAS_GELU: bf16 output, pieces of 16 rows x 64 columns (128 bytes + pad)
    // (storing the 8-byte register quads directly was measured slower than this LDS round trip)
    // Store addresses: wave-uniform base (scalar arithmetic) + a per-lane byte offset that never changes.
    float cs[FN][4];  // scale of each accumulator quad: the query columns' (see GemmArgs::q_cols), 1/2 ahead of GELU; the bias is scaled with it
#pragma unroll
    for (int j = 0; j < FN; ++j)
#pragma unroll
      for (int jj = 0; jj < 4; ++jj) {
        cs[j][jj] = EPI == EPI_BIAS_GELU ? 0.5f : ncol0 + j * 32 + jj * 8 + lk * 4 < a.q_cols ? a.q_scale : 1.0f;
        bias[j][jj] *= cs[j][jj];
      }
    const int sc = (lane & 7) * 8;
    // EPI_BIAS_HEADS: heads of 64 or 128 columns stored one after the other, so the wave's 64 columns lie inside one
    // head: its rows are hm_dh elements apart and (row0, ncol0) sits at a wave-uniform address of its own
    const int rs = EPI == EPI_BIAS_HEADS ? a.hm_dh : a.ldo;
    const uint32_t lane_off = (uint32_t)((lane >> 3) * rs + sc) * 2u;
    const int hm_blk = EPI == EPI_BIAS_HEADS ? ncol0 / a.hm_dh : 0;
    unsigned char* const tile_base =
        (unsigned char*)a.out + (EPI == EPI_BIAS_HEADS ? ((size_t)hm_blk * a.hm_rows + row0) * a.hm_dh + (ncol0 - hm_blk * a.hm_dh)
                                                       : (size_t)row0 * a.ldo + ncol0) * 2;
    const int row_lim = a.M - row0 - (lane >> 3);
    const bool col_ok = ncol0 + sc < a.N;
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      u32x2 pk[FN][4];  // all lanes convert once; the two half-wave passes below only move data
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          float v[4];
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            v[e] = fmaf(acc[i][j][jj * 4 + e], cs[j][jj], bias[j][jj][e]);
            if constexpr (EPI == EPI_BIAS_GELU) v[e] = gelu_fast_half(v[e]);
          }
          pk[j][jj] = u32x2{pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        }
#pragma unroll
      for (int half = 0; half < 2; ++half) {
        if ((lrow >> 4) == half) {
#pragma unroll
          for (int j = 0; j < FN; ++j)
#pragma unroll
            for (int jj = 0; jj < 4; ++jj)
              *(u32x2*)(st + (lrow & 15) * D_STAGING_ROW + (j * 32 + jj * 8 + lk * 4) * 2) = pk[j][jj];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int p = 0; p < 2; ++p) {  // 8 lanes per row (8 bf16 each), 8 rows per pass
          const int sr = p * 8 + (lane >> 3);
          const u32x4 t = *(const u32x4*)(st + sr * D_STAGING_ROW + sc * 2);
          if (FULL || (i * 32 + half * 16 + p * 8 < row_lim && col_ok)) {
            u32x4* dst = (u32x4*)(tile_base + (size_t)(i * 32 + half * 16 + p * 8) * rs * 2 + lane_off);
            // STREAM_OUT: the output is larger than the memory-side cache; it passes through once and
            // would only displace the operands, so it is stored non-temporally (-1 % on the large encode
            // step).  Smaller outputs are what the next kernel finds in that cache; there the hint costs
            // 2-5 %.  (A compile-time flag: a run-time choice between the two stores gets merged into one
            // plain store.)  Whole 128-byte row pieces only: on the attention kernel's 8-byte stores the
            // hint cost 10 %.
            if constexpr (STREAM_OUT) __builtin_nontemporal_store(t, dst);
            else *dst = t;
          }
        }
        __builtin_amdgcn_wave_barrier();
      }
    }
  }
}

template <int EPI, bool STREAM_OUT>
__global__ __launch_bounds__(512) void gemm_bf16_dma_kernel(const GemmArgs a, int tiles_m, int tiles_n, int n_bands,
                                                            int groups_full, int narrow_w, int n_groups) {
  constexpr int FM = 4, FN = 2, TM = 128, TN = 64;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  unsigned char* staging = smem + D_ST * D_STAGE_BYTES;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform: keeps addresses in scalar registers
  const int wm = wave >> 2, wn = wave & 3;
  const int lrow = lane & 31, lk = lane >> 5;

  // ---- tile list of this workgroup: groups xcd, xcd + 8, ...; inside a group the unit's slot picks the tile
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;  // slot in [0, 32)
  const int sm = slot / D_GROUP_N, sn = slot % D_GROUP_N;
  auto tile_of = [&](int g, int& tm, int& tn) {  // false when the slot has no tile in group g
    if (g < groups_full) {  // 8 x 4 groups over the full-width column bands
      const int mblk = g / n_bands, band = g - mblk * n_bands;
      tm = mblk * D_GROUP_M + sm;
      tn = band * D_GROUP_N + sn;
    } else {  // the last one or two tile columns: 32 x 1 or 16 x 2 groups, so no slot idles
      tm = (g - groups_full) * (32 / narrow_w) + slot / narrow_w;
      tn = n_bands * D_GROUP_N + slot % narrow_w;
    }
    const bool ok = tm < tiles_m && tn < tiles_n;
    if (a.reverse) tm = tiles_m - 1 - tm;
    return ok;
  };
  auto next_group = [&](int g) {  // first group >= g (stride 8) in which this slot has a tile, or n_groups
    int tm, tn;
    while (g < n_groups && !tile_of(g, tm, tn)) g += 8;
    return g < n_groups ? g : n_groups;
  };

  // ---- loader addressing: one instruction fills 8 tile rows of 128 bytes (lane -> row lane/8, LDS
  //      chunk lane%8); wave w moves rows [32w, 32w + 32) of both operand tiles.  An address is a
  //      wave-uniform 64-bit base (scalar registers) plus a per-lane 32-bit byte offset that never
  //      changes.  The logical chunk that lands in LDS chunk c of row r is c ^ ((r >> 1) & 7); for
  //      row 32w + 8i + lane/8 that is (4 * (i & 1) + lane/16) & 7: two offset variants per operand.
  const int ld_row = wave * 32 + (lane >> 3);
  const int ld_chunk = (lane & 7) ^ (lane >> 4);
  const uint32_t offA0 = (uint32_t)(ld_row * a.lda + ld_chunk * 8) * 2u;
  const uint32_t offA1 = (uint32_t)(ld_row * a.lda + (ld_chunk ^ 4) * 8) * 2u;
  const uint32_t offW0 = (uint32_t)(ld_row * a.ldw + ld_chunk * 8) * 2u;
  const uint32_t offW1 = (uint32_t)(ld_row * a.ldw + (ld_chunk ^ 4) * 8) * 2u;
  const size_t a_step = (size_t)16 * a.lda, w_step = (size_t)16 * a.ldw;  // bytes per 8 rows
  const unsigned char *baseA = nullptr, *baseW = nullptr;  // load cursor: uniform tile bases at k = 0
  int g_l = next_group(xcd), kt_l = 0;
  auto set_load_tile = [&]() {
    int tm, tn;
    if (g_l < n_groups && tile_of(g_l, tm, tn)) {
      baseA = (const unsigned char*)a.A + (size_t)tm * D_BM * a.lda * 2;
      baseW = (const unsigned char*)a.W + (size_t)tn * D_BN * a.ldw * 2;
    }
  };
  set_load_tile();
  // One direct-to-LDS instruction.  It is written as inline assembly so that the compiler's
  // wait-count insertion, which cannot know that the stage written here is never one being read,
  // does not fence every surrounding LDS read; completion is tracked by hand (sync_stage).  M0 holds
  // the LDS destination of lane 0.
  auto dma16 = [&](const unsigned char* gbase, uint32_t goff, unsigned char* lptr) {
    // low 32 bits of a generic LDS pointer = LDS offset; wave-uniform by construction
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lptr);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(goff), "s"(gbase)
                 : "memory", "m0");
  };
  // instruction i of stage slot `st` at the load cursor: i in [0,4) -> A rows 8i.., [4,8) -> W rows 8(i-4)..
  auto issue_load = [&](int st, int i) {
    unsigned char* base = smem + st * D_STAGE_BYTES;
    if (i < 4)
      dma16(baseA + i * a_step + kt_l * D_ROW, (i & 1) ? offA1 : offA0, base + (wave * 32 + i * 8) * D_ROW);
    else
      dma16(baseW + (i - 4) * w_step + kt_l * D_ROW, (i & 1) ? offW1 : offW0,
            base + D_BM * D_ROW + (wave * 32 + (i - 4) * 8) * D_ROW);
  };
  const int KT = a.K / D_BK;
  auto advance_load_cursor = [&]() {
    if (++kt_l == KT) {
      kt_l = 0;
      g_l = next_group(g_l + 8);
      set_load_tile();
    }
  };

  // ---- fragment addressing: row*128 + ((2ks + lk) ^ ((row >> 1) & 7)) * 16, row = 32-aligned base + lrow;
  //      with pos0 = lk ^ sw the chunk of sub-step ks is pos0 ^ 2ks, i.e. the byte offset XOR (ks << 5)
  const int sw = (lrow >> 1) & 7;
  const uint32_t fa_off = (uint32_t)((wm * TM + lrow) * D_ROW + ((lk ^ sw) << 4));
  const uint32_t fb_off = (uint32_t)(D_BM * D_ROW + (wn * TN + lrow) * D_ROW + ((lk ^ sw) << 4));

  f32x16 acc[FM][FN];
  bf16x8 fa0[FM], fb0[FN], fa1[FM], fb1[FN];  // fragments of even / odd sub-steps

  auto rd_a = [&](int st, int ks, int i) {
    return *(const bf16x8*)(smem + st * D_STAGE_BYTES + (fa_off ^ (uint32_t)(ks << 5)) + i * 32 * D_ROW);
  };
  auto rd_b = [&](int st, int ks, int j) {
    return *(const bf16x8*)(smem + st * D_STAGE_BYTES + (fb_off ^ (uint32_t)(ks << 5)) + j * 32 * D_ROW);
  };
  auto mm = [&](int i, const bf16x8& x, const bf16x8 (&w)[FN]) {
#pragma unroll
    for (int j = 0; j < FN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(w[j], x, acc[i][j], 0, 0, 0);
  };

  // ---- how many k-stages this workgroup will load in total
  int n_my_tiles = 0;
  for (int g = next_group(xcd); g < n_groups; g = next_group(g + 8)) ++n_my_tiles;
  const int total_stages = n_my_tiles * KT;
  int issued = 0, consumed = 0;  // k-stages issued to the ring / multiplied so far
  int st_c = 0;                  // ring slot of the stage being multiplied

  // Every load this wave has issued has landed and every LDS read it has issued is complete; then
  // meet the other waves.  (The vector-memory counter also counts the epilogue's stores.)
  auto sync_stage = [&]() {
    __builtin_amdgcn_s_waitcnt(0x0070);  // vmcnt(0) lgkmcnt(0)
    __builtin_amdgcn_s_barrier();
  };

  // One sub-step that multiplies fragment set (x, w) while reading sub-step `ks` of stage `st`
  // into (nx, nw); with `late` set, load instructions late0 .. late0 + 3 of the stage being
  // prefetched follow the four MFMA pairs.  sched_barrier(0) fences keep each group's instructions
  // together in this order.
  auto sub_step = [&](int st, int ks, const bf16x8 (&x)[FM], const bf16x8 (&w)[FN], bf16x8 (&nx)[FM],
                      bf16x8 (&nw)[FN], bool late, int late0) {
    nw[0] = rd_b(st, ks, 0); nw[1] = rd_b(st, ks, 1);
    nx[0] = rd_a(st, ks, 0);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      mm(i, x[i], w);
      if (i + 1 < FM) nx[i + 1] = rd_a(st, ks, i + 1);
      if (late) issue_load(st ^ 1, late0 + i);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // One 64-wide k-stage.  On entry fa0 / fb0 hold the fragments of its sub-step 0.
  //   sub-steps 0..2: MFMAs of sub-step j while the fragments of sub-step j + 1 are read;
  //   sync:           the other stage has landed for every wave and this stage's LDS is dead;
  //   sub-step 3:     its MFMAs while sub-step 0 of the other stage is read and the first four loads
  //                   of the stage after that go into the slot this stage just freed, one per MFMA
  //                   pair; the other four follow in sub-step 0 of the next stage (eight in a row
  //                   would queue up in the memory pipeline and hold back the MFMAs behind them).
  bool pend = false;  // the second half of a stage's loads is still to be issued
  // AHEAD = false (a tile's last stage in the residual kernel): the next tile's first fragments are not read
  // here but after the epilogue, which needs their registers for residual values in flight.
  auto k_stage = [&](auto load_tag, auto next_tag, const bool AHEAD) {
    constexpr bool LOAD = decltype(load_tag)::value, NEXT = decltype(next_tag)::value;
    const int sn = st_c ^ 1;
    sub_step(st_c, 1, fa0, fb0, fa1, fb1, pend, 4);
    if (pend) { advance_load_cursor(); pend = false; }
    sub_step(st_c, 2, fa1, fb1, fa0, fb0, false, 0);
    // the last fragments of this stage are read up front so that they are complete at the barrier
    fb1[0] = rd_b(st_c, 3, 0); fb1[1] = rd_b(st_c, 3, 1);
#pragma unroll
    for (int i = 0; i < FM; ++i) fa1[i] = rd_a(st_c, 3, i);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < FM; ++i) mm(i, fa0[i], fb0);
    __builtin_amdgcn_sched_barrier(0);
    if (NEXT) sync_stage();
    __builtin_amdgcn_sched_barrier(0);
    if (NEXT && AHEAD) { fb0[0] = rd_b(sn, 0, 0); fb0[1] = rd_b(sn, 0, 1); fa0[0] = rd_a(sn, 0, 0); }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < FM; ++i) {
      mm(i, fa1[i], fb1);
      if (NEXT && AHEAD && i < FM - 1) fa0[i + 1] = rd_a(sn, 0, i + 1);
      if (LOAD) issue_load(st_c, i);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (LOAD) { pend = true; ++issued; }
    ++consumed;
    st_c = sn;
  };

  // ---- prologue: fill both stages, wait for them, read the first fragments
  for (int i = 0; i < D_ST && issued < total_stages; ++i) {
#pragma unroll
    for (int j = 0; j < D_LOADS; ++j) issue_load(i, j);
    advance_load_cursor();
    ++issued;
  }
  if (total_stages > 0) {
    sync_stage();
    fb0[0] = rd_b(0, 0, 0); fb0[1] = rd_b(0, 0, 1);
#pragma unroll
    for (int i = 0; i < FM; ++i) fa0[i] = rd_a(0, 0, i);
  }

  int stamp_i = 0;  // measurement aid: tiles of this workgroup stamped so far
  for (int g_c = next_group(xcd); g_c < n_groups; g_c = next_group(g_c + 8)) {
    int tm, tn;
    tile_of(g_c, tm, tn);
    // measurement aid (off unless the host asked for it): constant-rate clock at the tile's start, after its
    // k-loop and after its epilogue, and the shader clocks the tile took
    unsigned long long stamp_t0 = 0, stamp_t1 = 0, stamp_c0 = 0;
    if (a.tile_stamps) { stamp_t0 = wall_clock64(); stamp_c0 = __builtin_readcyclecounter(); }
    const int row0 = tm * D_BM + wm * TM, ncol0 = tn * D_BN + wn * TN;
#pragma unroll
    for (int i = 0; i < FM; ++i)
#pragma unroll
      for (int j = 0; j < FN; ++j)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    // stages that still prefetch one; then (only at the end of the list) a stage that only reads
    // ahead; then the very last stage of the list, which has nothing after it
    const int n_ld = min(KT, total_stages - issued);
    const int n_nx = min(KT, total_stages - 1 - consumed);
    constexpr bool RESID = EPI == EPI_BIAS_RESIDUAL;
    const std::true_type T{};
    const std::false_type F{};
    // (wave-uniform run-time flag: a compile-time variant of the last stage would merge three copies of the
    //  accumulators' live ranges and spill)
    for (int kt = 0; kt < n_ld; ++kt) k_stage(T, T, !RESID || kt != KT - 1);
    for (int kt = n_ld; kt < n_nx; ++kt) k_stage(F, T, !RESID || kt != KT - 1);
    for (int kt = max(n_ld, n_nx); kt < KT; ++kt) k_stage(F, F, true);
    if constexpr (RESID) {  // the fragment registers are dead across the epilogue: say so
#pragma unroll
      for (int i = 0; i < FM; ++i) fa0[i] = bf16x8{};
      fb0[0] = bf16x8{}; fb0[1] = bf16x8{};
    }
    asm volatile("" ::: "memory");  // keep the epilogue's loads below the k-loop
    if (a.tile_stamps) stamp_t1 = wall_clock64();
    // a wave's 128 x 64 block lies wholly inside the matrix for all but the last row block / a ragged last column
    if (row0 + TM <= a.M && ncol0 + TN <= a.N)
      wave_epilogue_p<EPI, STREAM_OUT, true>(a, acc, staging + wave * 16 * D_STAGING_ROW, row0, ncol0, lane);
    else
      wave_epilogue_p<EPI, STREAM_OUT, false>(a, acc, staging + wave * 16 * D_STAGING_ROW, row0, ncol0, lane);
    if constexpr (RESID) {  // the next tile's first fragments (its first stage landed before the last sync)
      if (consumed < total_stages) {
        fb0[0] = rd_b(st_c, 0, 0); fb0[1] = rd_b(st_c, 0, 1);
#pragma unroll
        for (int i = 0; i < FM; ++i) fa0[i] = rd_a(st_c, 0, i);
      }
    }
    if (a.tile_stamps) {
      asm volatile("" ::: "memory");
      const unsigned long long stamp_t2 = wall_clock64();
      if (tid == 0 && stamp_i < kTileStampSlots) {
        unsigned long long* d = a.tile_stamps + ((size_t)blockIdx.x * kTileStampSlots + stamp_i) * 4;
        d[0] = stamp_t0; d[1] = stamp_t1; d[2] = stamp_t2;
        d[3] = __builtin_readcyclecounter() - stamp_c0 + 1;  // never 0: marks the slot as written
      }
      ++stamp_i;
    }
  }
}

// ---------------------------------------------------------------------------------------------
// Small-problem kernel (fewer than 384 tiles of 256 x 256; also the short last round of a large product that is
// one column band wide, see launch_gemm_bf16): one 128 x 128 tile per workgroup, eight
// waves of 64 x 32 (two per SIMD), operands global -> LDS directly into a ring of R_NS 64-wide
// k-stages (32 KiB each).  One wait + barrier per stage establishes that the stage has landed for
// every wave and that the slot refilled next is dead; all fragments of a stage are read before
// its MFMAs start (registers are plentiful here).
// * R_NS = 4 when there are no more tiles than compute units: a workgroup is then alone on its
//   unit and nothing but its own instruction order hides latency, so the loads run three stages
//   ahead.
// * R_NS = 2 (64 KiB) beyond that when it needs fewer rounds (see launch_ring): two workgroups share a unit
//   and cover each other's waits, and a grid of 1.2 or 1.7 rounds no longer costs 2.
// (The register-staged predecessor spent 2 800 clocks per k-stage on 512 clocks of MFMA work: LDS
// writes, their waits and un-overlapped fragment reads.)
// * BM = 64 (a 64 x 128 tile, waves of 32 x 32, 24 KiB stages) for the very smallest products, one or two
//   images: twice the workgroups on the idle units, and a k-stage that is a third shorter because it
//   moves a third less through LDS (a single image's fc2 is a chain of 64 stages on 40 units otherwise).
//   A token's k-steps are added in the same order in every variant.
constexpr int R_BN = 128;
constexpr int ring_stage_bytes(int bm) { return (bm + R_BN) * D_ROW; }  // 32 KiB (BM = 128) or 24 KiB

template <int EPI, int R_NS, int BM>
__global__ __launch_bounds__(512) void gemm_bf16_ring_kernel(const GemmArgs a, int tiles_m, int tiles_n,
                                                             int mt_per_xcd, int n_bands) {
  static_assert(BM == 128 || BM == 64, "tile heights: 128 or 64 rows");
  constexpr int R_BM = BM, R_STAGE_BYTES = ring_stage_bytes(BM);
  constexpr int FM = BM / 64, FN = 1, TM = BM / 2, TN = 32;
  constexpr int LOADS = BM == 128 ? 4 : 3;  // direct-to-LDS instructions per wave and stage
  static_assert(8 * 32 * (TN * 4 + 16) <= R_NS * R_STAGE_BYTES, "epilogue staging must fit in the ring");
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];

  // ---- tile assignment: workgroup ids are dealt round-robin to the 8 XCDs; each XCD walks its own range of
  //      row blocks in 8 x 4 tile groups so the tiles in flight on one XCD share A and W slices in its L2
  const int xcd = blockIdx.x & 7, q = blockIdx.x >> 3;
  const int blk = q / (GROUP_M * GROUP_N), r = q - blk * (GROUP_M * GROUP_N);
  const int mb = blk / n_bands, nb = blk - mb * n_bands;
  const int m_local = mb * GROUP_M + r / GROUP_N;
  const int tile_m = xcd * mt_per_xcd + m_local, tile_n = nb * GROUP_N + (r % GROUP_N);
  if (m_local >= mt_per_xcd || tile_m >= tiles_m || tile_n >= tiles_n) return;
  const int m0 = tile_m * R_BM, n0 = tile_n * R_BN;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 2, wn = wave & 3;
  const int lrow = lane & 31, lk = lane >> 5;

  // ---- loader: an instruction fills 8 rows of 128 bytes; wave w moves rows [16w, 16w + 16) of a 128-row
  //      operand tile (two instructions) or rows [8w, 8w + 8) of the 64-row A tile (one).  The chunk that
  //      lands in LDS chunk c of row r is c ^ ((r >> 1) & 7).
  const int ld_row = wave * 16 + (lane >> 3);
  const int ld_chunk = (lane & 7) ^ (lane >> 4);
  const int a_row = BM == 128 ? ld_row : wave * 8 + (lane >> 3);
  const int a_chunk = BM == 128 ? ld_chunk : ld_chunk ^ (4 * (wave & 1));
  const uint32_t offA0 = (uint32_t)(a_row * a.lda + a_chunk * 8) * 2u;
  const uint32_t offA1 = (uint32_t)((ld_row + 8) * a.lda + (ld_chunk ^ 4) * 8) * 2u;  // BM = 128 only
  const uint32_t offW0 = (uint32_t)(ld_row * a.ldw + ld_chunk * 8) * 2u;
  const uint32_t offW1 = (uint32_t)((ld_row + 8) * a.ldw + (ld_chunk ^ 4) * 8) * 2u;
  const unsigned char* const baseA = (const unsigned char*)a.A + (size_t)m0 * a.lda * 2;
  const unsigned char* const baseW = (const unsigned char*)a.W + (size_t)n0 * a.ldw * 2;
  auto dma16 = [&](const unsigned char* gbase, uint32_t goff, unsigned char* lptr) {
    const uint32_t lds_addr = __builtin_amdgcn_readfirstlane((uint32_t)(uintptr_t)lptr);
    asm volatile("s_mov_b32 m0, %0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(goff), "s"(gbase)
                 : "memory", "m0");
  };
  auto issue_stage = [&](int slot, int kt) {  // LOADS instructions per wave
    unsigned char* stage = smem + slot * R_STAGE_BYTES;
    const unsigned char* ga = baseA + kt * D_ROW;
    const unsigned char* gw = baseW + kt * D_ROW;
    if constexpr (BM == 128) {
      dma16(ga, offA0, stage + wave * 16 * D_ROW);
      dma16(ga, offA1, stage + wave * 16 * D_ROW + 8 * D_ROW);
    } else {
      dma16(ga, offA0, stage + wave * 8 * D_ROW);
    }
    dma16(gw, offW0, stage + R_BM * D_ROW + wave * 16 * D_ROW);
    dma16(gw, offW1, stage + R_BM * D_ROW + wave * 16 * D_ROW + 8 * D_ROW);
  };

  const int sw = (lrow >> 1) & 7;
  const uint32_t fa_off = (uint32_t)((wm * TM + lrow) * D_ROW + ((lk ^ sw) << 4));
  const uint32_t fb_off = (uint32_t)(R_BM * D_ROW + (wn * TN + lrow) * D_ROW + ((lk ^ sw) << 4));

  f32x16 acc[FM][FN];
#pragma unroll
  for (int i = 0; i < FM; ++i)
#pragma unroll
    for (int v = 0; v < 16; ++v) acc[i][0][v] = 0.f;

  const int KT = a.K / D_BK;
  // The tail re-reads the last k-stage into slots nobody uses any more, so that every stage issues
  // the same four loads and the wait below can count them.
#pragma unroll
  for (int s = 0; s < R_NS - 1; ++s) issue_stage(s, min(s, KT - 1));

  bf16x8 fa[4][FM], fb[4];  // all four sub-steps of a stage are read up front: registers are plentiful here
  for (int kt = 0; kt < KT; ++kt) {
    const int slot = kt & (R_NS - 1);
    // this wave's loads of stage kt have landed (those of the two later stages may be in flight) and
    // its LDS reads of stage kt - 1 are complete; then meet the other waves
    __builtin_amdgcn_s_waitcnt(0x0070 | (LOADS * (R_NS - 2)));
    __builtin_amdgcn_s_barrier();
    issue_stage((kt + R_NS - 1) & (R_NS - 1), min(kt + R_NS - 1, KT - 1));
    const unsigned char* st = smem + slot * R_STAGE_BYTES;
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
#pragma unroll
      for (int i = 0; i < FM; ++i) fa[ks][i] = *(const bf16x8*)(st + (fa_off ^ (uint32_t)(ks << 5)) + i * 32 * D_ROW);
      fb[ks] = *(const bf16x8*)(st + (fb_off ^ (uint32_t)(ks << 5)));
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks)
#pragma unroll
      for (int i = 0; i < FM; ++i)
        acc[i][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[ks], fa[ks][i], acc[i][0], 0, 0, 0);
    __builtin_amdgcn_sched_barrier(0);
  }
  // the trailing loads still write LDS, which the epilogue reuses
  __builtin_amdgcn_s_waitcnt(0x0070);
  __builtin_amdgcn_s_barrier();
  wave_epilogue<EPI, FM, FN>(a, acc, smem, m0 + wm * TM, n0 + wn * TN, wave, lane);
}

hipError_t launch_ring(const GemmArgs& a, hipStream_t s) {
  const int tiles_n = (a.N + R_BN - 1) / R_BN;
  // At most 96 tiles of 128 x 128 (the N = 1024 products of one or two images): 64-row tiles, still fewer
  // workgroups than units.  Measured at 577 and 1154 rows: 40 and 80 tiles gain 30-45 %, 120 tiles (QKV of
  // one image) lose 15 %.  Products of at most eight tile columns (N <= 1024) keep gaining up to one 64-row tile
  // per unit (three images: 112 tiles of 128 rows, 224 of 64: out-proj and fc2 18-22 % faster), and again where
  // the 128-row tiles are a few more than the units and their second workgroups leave most units with one: there
  // three 64-row workgroups with two-stage rings share a unit in a single round of up to 768 tiles (eight images,
  // 296 tiles of 128 rows: 7 %).
  const long tiles128 = (long)((a.M + 127) / 128) * tiles_n, tiles64 = (long)((a.M + 63) / 64) * tiles_n;
  const bool narrow = tiles_n <= 8;
  const bool half3 = narrow && tiles128 > 256 && tiles64 <= 768;  // three two-stage workgroups of 64 rows per unit
  const bool half = tiles128 <= 96 || (narrow && tiles64 <= 256) || half3;
  const int bm = half ? 64 : 128;
  const int tiles_m = (a.M + bm - 1) / bm;
  const int mt_per_xcd = (tiles_m + 7) / 8;
  const int n_bands = (tiles_n + GROUP_N - 1) / GROUP_N;
  const int m_blocks = (mt_per_xcd + GROUP_M - 1) / GROUP_M;
  const long grid = 8L * m_blocks * n_bands * GROUP_M * GROUP_N;
  if (grid > 0x7fffffffL) return hipErrorInvalidValue;
  // Up to one tile per compute unit: the four-stage ring, whose loads run three stages ahead.  Beyond that either
  // two-stage rings (64 KiB), two workgroups to a unit covering each other's waits, in rounds of 512 tiles, or the
  // four-stage ring in rounds of 256: a k-stage of a workgroup takes 0.95 us when it shares its unit and 0.58 us
  // when it has it alone (measured on the N = 1024 products), so whichever needs fewer rounds by that measure.
  const long n_tiles = (long)tiles_m * tiles_n;
  const bool two = !half && n_tiles > 256 && ((n_tiles + 511) / 512) * 95 < ((n_tiles + 255) / 256) * 58;
#define VIT_LAUNCH_NS(EPI, NS, BM)                                                                                   \
  do {                                                                                                               \
    auto kfn = gemm_bf16_ring_kernel<EPI, NS, BM>;                                                                   \
    constexpr int lds = NS * ring_stage_bytes(BM);                                                                   \
    static LdsLimitOnce lds_limit;                                                                                   \
    if (hipError_t e = lds_limit.ensure((const void*)kfn, lds); e != hipSuccess) return e;                           \
    hipLaunchKernelGGL(kfn, dim3((unsigned)grid), dim3(512), lds, s, a, tiles_m, tiles_n, mt_per_xcd, n_bands);      \
  } while (0)
#define VIT_LAUNCH(EPI)            \
  do {                             \
    if (half3)                     \
      VIT_LAUNCH_NS(EPI, 2, 64);   \
    else if (half)                 \
      VIT_LAUNCH_NS(EPI, 4, 64);   \
    else if (two)                  \
      VIT_LAUNCH_NS(EPI, 2, 128);  \
    else                           \
      VIT_LAUNCH_NS(EPI, 4, 128);  \
  } while (0)
  switch (a.epilogue) {
    case EPI_BIAS: VIT_LAUNCH(EPI_BIAS); break;
    case EPI_BIAS_HEADS: VIT_LAUNCH(EPI_BIAS_HEADS); break;
    case EPI_BIAS_GELU: VIT_LAUNCH(EPI_BIAS_GELU); break;
    case EPI_BIAS_RESIDUAL: VIT_LAUNCH(EPI_BIAS_RESIDUAL); break;
    case EPI_PATCH: VIT_LAUNCH(EPI_PATCH); break;
    default: return hipErrorInvalidValue;
  }
#undef VIT_LAUNCH
#undef VIT_LAUNCH_NS
  return hipGetLastError();
}

hipError_t launch_dma(const GemmArgs& a, hipStream_t s) {
  const int tiles_m = (a.M + D_BM - 1) / D_BM, tiles_n = (a.N + D_BN - 1) / D_BN;
  // column bands of four tiles; a remainder of one or two tile columns gets its own group shape
  // (a remainder of three is a band with one idle column)
  const int rem = tiles_n % D_GROUP_N;
  const int narrow_w = rem == 3 ? 0 : rem;
  const int n_bands = tiles_n / D_GROUP_N + (rem == 3 ? 1 : 0);
  const int groups_full = ((tiles_m + D_GROUP_M - 1) / D_GROUP_M) * n_bands;
  const int groups_narrow = narrow_w ? (tiles_m + 32 / narrow_w - 1) / (32 / narrow_w) : 0;
  const int n_groups = groups_full + groups_narrow;
  // compute units of the current device, looked up once per device
  static std::atomic<int> cu_of_device[64];
  int dev = 0;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
  int n_cu = cu_of_device[dev].load(std::memory_order_relaxed);
  if (n_cu == 0) {
    if (hipError_t e = hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev); e != hipSuccess) return e;
    cu_of_device[dev].store(n_cu, std::memory_order_relaxed);
  }
  // one workgroup per compute unit: 8 XCDs x 32 slots.  The unit count is a performance assumption only (the
  // workgroups never wait for each other); a device with fewer units takes the small-tile kernel instead.
  const int grid = 8 * D_GROUP_M * D_GROUP_N;
  if (n_cu < grid) return launch_ring(a, s);
#define VIT_LAUNCH(EPI, STREAM)                                                                                      \
  do {                                                                                                               \
    auto kfn = gemm_bf16_dma_kernel<EPI, STREAM>;                                                                    \
    static LdsLimitOnce lds_limit;                                                                                   \
    if (hipError_t e = lds_limit.ensure((const void*)kfn, D_LDS_BYTES); e != hipSuccess) return e;                   \
    hipLaunchKernelGGL(kfn, dim3(grid), dim3(512), D_LDS_BYTES, s, a, tiles_m, tiles_n, n_bands, groups_full,        \
                       narrow_w, n_groups);                                                                          \
  } while (0)
  switch (a.epilogue) {
    case EPI_BIAS:
      if (a.stream_out) VIT_LAUNCH(EPI_BIAS, true);
      else VIT_LAUNCH(EPI_BIAS, false);
      break;
    case EPI_BIAS_HEADS:
      if (a.stream_out) VIT_LAUNCH(EPI_BIAS_HEADS, true);
      else VIT_LAUNCH(EPI_BIAS_HEADS, false);
      break;
    case EPI_BIAS_GELU:
      if (a.stream_out) VIT_LAUNCH(EPI_BIAS_GELU, true);
      else VIT_LAUNCH(EPI_BIAS_GELU, false);
      break;
    case EPI_BIAS_RESIDUAL: VIT_LAUNCH(EPI_BIAS_RESIDUAL, false); break;
    case EPI_PATCH: VIT_LAUNCH(EPI_PATCH, false); break;
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
  // head-by-head output: heads of 64 or 128 columns (a wave's column block never straddles two)
  if (a.epilogue == EPI_BIAS_HEADS && (a.hm_dh <= 0 || a.hm_dh % 64 != 0 || a.hm_rows < (size_t)a.M)) return hipErrorInvalidValue;
  const int tiles_m = (a.M + 255) / 256, tiles_n = (a.N + 255) / 256;
  const long big_tiles = (long)tiles_m * tiles_n;
  // A product one column band wide (1, 2 or 4 tile columns) is walked in rounds of 256 / tiles_n row blocks, one
  // tile per compute unit.  When the last round holds at most 128 tiles, half or more of the units would sit out a
  // whole tile time: those row blocks go to the small-tile kernel in a second launch instead (at most 512 tiles of
  // 128 x 128: one round of two workgroups per unit), also when that leaves the persistent kernel a single round
  // (a product of 257 to 383 tiles, which as a whole would be too small for it).  Measured on the N = 1024
  // products at 24 to 64 images: a limit of 64 tiles leaves 3 % on the table at 36 to 40 and at 64 images, a
  // limit of 192 loses 5 % at 48.  Both kernels give a row the same bits, so where the cut falls does not show
  // in the result.  The cut is made at the end the walk reaches last.
  if (a.epilogue != EPI_PATCH && (tiles_n == 1 || tiles_n == 2 || tiles_n == 4)) {
    const int per_round = 256 / tiles_n;
    const int tail_blocks = tiles_m % per_round;
    if (tail_blocks > 0 && tiles_m > per_round && tail_blocks * tiles_n <= 128) {
      const int cut = a.reverse ? tail_blocks * 256 : (tiles_m - tail_blocks) * 256;  // first row of the upper part
      auto rows_from = [&](int row0, int rows) {
        GemmArgs b = a;
        b.M = rows;
        b.A = (const unsigned char*)a.A + (size_t)row0 * a.lda * 2;
        if (a.out) b.out = (unsigned char*)a.out + (size_t)row0 * (a.epilogue == EPI_BIAS_HEADS ? a.hm_dh : a.ldo) * 2;  // a row's stride
        if (a.resid) b.resid = a.resid + (size_t)row0 * a.ldo;
        return b;
      };
      const GemmArgs lower = rows_from(0, cut), upper = rows_from(cut, a.M - cut);
      if (hipError_t e = launch_dma(a.reverse ? upper : lower, s); e != hipSuccess) return e;
      return launch_ring(a.reverse ? lower : upper, s);
    }
  }
  // The persistent 256 x 256 kernel pays off from about one and a half tiles per compute unit
  // (measured crossover between 300 and 440 tiles on the encoder's shapes); below that its last,
  // partly filled round costs more than the smaller tiles' extra operand traffic.
  if (big_tiles < 384) return launch_ring(a, s);
  return launch_dma(a, s);
}

}  // namespace vitenc
