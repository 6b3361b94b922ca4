// Memory-bound row kernels: LayerNorm (fp32 residual stream -> matrix operand), patch
// gather, CLS rows, padding fill.  All are HBM-bound; each element is read once and
// written once with 16-byte accesses where the layout allows.
#include "common.h"

namespace vitenc {

namespace {

__device__ inline float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// One wave per token row.  Two passes over registers: mean, then biased variance of the
// centred values (no E[x^2] - mean^2 cancellation).  Columns D..out_cols-1 of the output
// are written as zero so the row can feed a K-padded matrix product.
// NORMALIZE = 0 turns the kernel into a plain fp32 -> OutT conversion.
template <typename OutT, int MAXV, int NORMALIZE, bool STREAM_IN>
__global__ __launch_bounds__(256) void layernorm_kernel(const float* __restrict__ x, int ldx, OutT* __restrict__ out,
                                                        int ldo, int out_cols, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, float eps, int rows, int D,
                                                        int reverse) {
  const int lane = threadIdx.x & 63;
  int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= rows) return;
  if (reverse) row = rows - 1 - row;
  const float* xr = x + (size_t)row * ldx;
  f32x4 v[MAXV];
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c < D) {
      // STREAM_IN: x is larger than the memory-side cache; it is read once here and non-temporally, so that
      // it does not displace operands (-1 % on the large encode step).  A small x sits in L2, where the hint
      // costs 2-5 %.  (Compile-time: a run-time choice between the two loads gets merged into one plain load.)
      if constexpr (STREAM_IN) v[i] = __builtin_nontemporal_load((const f32x4*)(xr + c));
      else v[i] = *(const f32x4*)(xr + c);
      s += (v[i][0] + v[i][1]) + (v[i][2] + v[i][3]);
    } else {
      v[i] = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
  float mean = 0.f, rstd = 1.f;
  if (NORMALIZE) {
    mean = wave_sum(s) / (float)D;
    float q = 0.f;
#pragma unroll
    for (int i = 0; i < MAXV; ++i) {
      const int c = (i * 64 + lane) * 4;
      if (c < D) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float d = v[i][e] - mean;
          q += d * d;
        }
      }
    }
    rstd = rsqrtf(wave_sum(q) / (float)D + eps);
  }
  OutT* orow = out + (size_t)row * ldo;
#pragma unroll
  for (int i = 0; i < MAXV; ++i) {
    const int c = (i * 64 + lane) * 4;
    if (c >= out_cols) continue;
    float y[4] = {0.f, 0.f, 0.f, 0.f};
    if (c < D) {
      if (NORMALIZE) {
        const f32x4 g = *(const f32x4*)(gamma + c), b = *(const f32x4*)(beta + c);
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = (v[i][e] - mean) * rstd * g[e] + b[e];
      } else {
#pragma unroll
        for (int e = 0; e < 4; ++e) y[e] = v[i][e];
      }
    }
    if constexpr (sizeof(OutT) == 2) {
      u32x2 pk = {pack_bf16x2(y[0], y[1]), pack_bf16x2(y[2], y[3])};
      *(u32x2*)(orow + c) = pk;
    } else {
      *(f32x4*)(orow + c) = f32x4{y[0], y[1], y[2], y[3]};
    }
  }
}

// patches[(tile*g*g + gy*g + gx), c*p*p + py*p + px] = pixels[tile, c, gy*p+py, gx*p+px];
// columns K..Kpad-1 are zero.  One thread per output element, column fastest (coalesced writes;
// reads are runs of p contiguous pixels).
template <typename OutT>
__global__ __launch_bounds__(256) void patch_gather_kernel(const float* __restrict__ px, OutT* __restrict__ out, int ld,
                                                           long total, int C, int S, int p, int g, int K, int Kpad) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= total) return;
  const int col = (int)(idx % Kpad);
  const long row = idx / Kpad;
  float v = 0.f;
  if (col < K) {
    const int P = g * g;
    const long tile = row / P;
    const int pi = (int)(row - tile * P), gy = pi / g, gx = pi - gy * g;
    const int c = col / (p * p), r = col - c * p * p, py = r / p, pxx = r - py * p;
    v = px[((tile * C + c) * S + (gy * p + py)) * (long)S + gx * p + pxx];
  }
  Elem<OutT>::store(out + row * ld + col, v);
}

// The same gather for image sides that are a multiple of 4, one workgroup per strip of patches (one tile, one
// patch row gy: g patches): the strip's C * p image rows are read once, 16 bytes per lane and coalesced (an image
// row is contiguous across the strip's patches), scattered into an LDS image of the strip's g output rows, and
// written out in 16-byte pieces with the padding columns zero.  Every pixel is read once and every output byte
// written once with full-width accesses; the element-per-thread form above read 3.2 times the pixel bytes.
template <typename OutT>
__global__ __launch_bounds__(256) void patch_gather_strip_kernel(const float* __restrict__ px, OutT* __restrict__ out,
                                                                 int ld, int C, int S, int p, int g, int K, int Kpad) {
  extern __shared__ __attribute__((aligned(16))) unsigned char strip_raw[];
  OutT* strip = (OutT*)strip_raw;  // [g][Kpad]
  const int tid = threadIdx.x;
  const long tile = blockIdx.x / g;
  const int gy = blockIdx.x - (int)tile * g;
  // padding columns K .. Kpad - 1 of every row
  const int padc = Kpad - K;
  for (int it = tid; it < g * padc; it += 256) strip[(it / padc) * Kpad + K + it % padc] = (OutT)0;
  // image rows r = c * p + py, one wave per row at a time, 4 pixels per lane; pixels past the last whole patch
  // are dropped.  x / p by a float reciprocal (exact for x < 2^20 with the half added).
  const int quads = S >> 2, used = g * p;
  const float inv_p = 1.0f / (float)p;
  const float* base = px + ((tile * C) * S + (long)gy * p) * S;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  for (int r = wave; r < C * p; r += 4) {
    const int c = r / p, py = r - c * p;  // wave-uniform
    const float* row = base + ((long)c * S + py) * S;
    OutT* drow = strip + r * p;
    for (int q = lane; q < quads; q += 64) {
      const f32x4 v = *(const f32x4*)(row + q * 4);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const int x = q * 4 + e;
        if (x < used) {
          const int gx = (int)(((float)x + 0.5f) * inv_p), pxx = x - gx * p;
          OutT* dst = drow + gx * Kpad + pxx;
          if constexpr (sizeof(OutT) == 2) *dst = f32_to_bf16(v[e]);
          else *dst = v[e];
        }
      }
    }
  }
  __syncthreads();
  const int chunks = Kpad * (int)sizeof(OutT) / 16;  // 16-byte pieces per output row
  unsigned char* orow = (unsigned char*)(out + (tile * g * g + (long)gy * g) * ld);
  for (int it = tid; it < g * chunks; it += 256) {
    const int row = it / chunks, ch = it - row * chunks;
    *(u32x4*)(orow + (long)row * ld * sizeof(OutT) + ch * 16) = *(const u32x4*)(strip_raw + ((long)row * Kpad * sizeof(OutT)) + ch * 16);
  }
}

// x[tile*T, :] = cls + pos[0, :]
__global__ __launch_bounds__(256) void cls_rows_kernel(float* __restrict__ x, int ldx, const float* __restrict__ cls,
                                                       const float* __restrict__ pos, int n_tiles, int T, int D) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= (long)n_tiles * D) return;
  const int c = (int)(idx % D);
  const long tile = idx / D;
  x[tile * T * ldx + c] = cls[c] + pos[c];
}

template <typename T>
__global__ __launch_bounds__(256) void fill_zero_cols_kernel(T* buf, int ld, long rows, int col0, int ncols) {
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= rows * ncols) return;
  buf[(idx / ncols) * ld + col0 + (int)(idx % ncols)] = (T)0;
}

// Token down-sampling: every m x m block of neighbouring patch tokens of a tile becomes one token whose
// channels are the block's tokens one after the other, (dy, dx) row-major; the CLS row is dropped.
// One thread moves 16 bytes; src rows are [tile*T + cls + y*g + x], dst rows [tile*(g/m)^2 + y2*(g/m) + x2].
__global__ __launch_bounds__(256) void token_merge_kernel(const unsigned char* __restrict__ src, long src_ld_bytes,
                                                          unsigned char* __restrict__ dst, long dst_ld_bytes,
                                                          long n_out, int T, int cls, int g, int m, int row_chunks,
                                                          int pad_chunks) {
  const int chunks = m * m * row_chunks + pad_chunks;  // 16-byte chunks per output row, padding included
  const long idx = (long)blockIdx.x * 256 + threadIdx.x;
  if (idx >= n_out * chunks) return;
  const long r = idx / chunks;
  const int c = (int)(idx - r * chunks);
  u32x4 v = {0u, 0u, 0u, 0u};
  if (c < m * m * row_chunks) {
    const int gm = g / m, pm = gm * gm;
    const long tile = r / pm;
    const int o = (int)(r - tile * pm), y2 = o / gm, x2 = o - y2 * gm;
    const int q = c / row_chunks, k = c - q * row_chunks, dy = q / m, dx = q - dy * m;
    const long srow = tile * T + cls + (long)(y2 * m + dy) * g + (x2 * m + dx);
    v = *(const u32x4*)(src + srow * src_ld_bytes + (long)k * 16);
  }
  *(u32x4*)(dst + r * dst_ld_bytes + (long)c * 16) = v;
}

template <typename OutT, int NORMALIZE>
hipError_t ln_dispatch(const float* x, int ldx, void* out, int ldo, int out_cols, const float* gamma, const float* beta,
                       float eps, int rows, int D, int reverse, int stream_in, hipStream_t s) {
  const dim3 grid((rows + 3) / 4), block(256);
  const int need = (out_cols + 255) / 256;  // float4 slots per lane
#define VIT_LN_S(MAXV, STREAM)                                                                                    \
  hipLaunchKernelGGL((layernorm_kernel<OutT, MAXV, NORMALIZE, STREAM>), grid, block, 0, s, x, ldx, (OutT*)out, ldo, \
                     out_cols, gamma, beta, eps, rows, D, reverse)
#define VIT_LN(MAXV)                        \
  do {                                      \
    if (stream_in) VIT_LN_S(MAXV, true);    \
    else VIT_LN_S(MAXV, false);             \
  } while (0)
  if (need <= 1) VIT_LN(1);
  else if (need <= 2) VIT_LN(2);
  else if (need <= 4) VIT_LN(4);
  else if (need <= 5) VIT_LN(5);
  else if (need <= 8) VIT_LN(8);
  else if (need <= 16) VIT_LN(16);
  else return hipErrorInvalidValue;
#undef VIT_LN
#undef VIT_LN_S
  return hipGetLastError();
}

}  // namespace

hipError_t launch_layernorm(const float* x, int ldx, void* out, int ldo, int out_cols, const float* gamma,
                            const float* beta, float eps, int rows, int D, int normalize, int out_bf16, int reverse,
                            int stream_in, hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  if (D % 4 != 0 || out_cols % 4 != 0 || ldx % 4 != 0 || ldo % 4 != 0 || out_cols < D) return hipErrorInvalidValue;
  if (out_bf16) {
    return normalize ? ln_dispatch<bf16_t, 1>(x, ldx, out, ldo, out_cols, gamma, beta, eps, rows, D, reverse, stream_in, s)
                     : ln_dispatch<bf16_t, 0>(x, ldx, out, ldo, out_cols, gamma, beta, eps, rows, D, reverse, stream_in, s);
  }
  return normalize ? ln_dispatch<float, 1>(x, ldx, out, ldo, out_cols, gamma, beta, eps, rows, D, reverse, stream_in, s)
                   : ln_dispatch<float, 0>(x, ldx, out, ldo, out_cols, gamma, beta, eps, rows, D, reverse, stream_in, s);
}

hipError_t launch_patch_gather(const float* pixels, void* patches, int ld, int n_tiles, int C, int S, int p, int g,
                               int Kpad, int out_bf16, hipStream_t s) {
  const long total = (long)n_tiles * g * g * Kpad;
  if (total <= 0) return hipSuccess;
  const int K = C * p * p;
  // strip form: whole float4s per image row, 16-byte output pieces, a strip that fits 64 KiB of LDS
  const size_t es = out_bf16 ? 2 : 4, strip_bytes = (size_t)g * Kpad * es;
  if (S % 4 == 0 && (Kpad * es) % 16 == 0 && ((size_t)ld * es) % 16 == 0 && strip_bytes <= 64 * 1024 &&
      (long)n_tiles * g <= 0x7fffffffL) {
    const dim3 sgrid((unsigned)(n_tiles * g)), sblock(256);
    if (out_bf16) {
      static LdsLimitOnce lim;
      if (hipError_t e = lim.ensure((const void*)patch_gather_strip_kernel<bf16_t>, 64 * 1024); e != hipSuccess) return e;
      hipLaunchKernelGGL(patch_gather_strip_kernel<bf16_t>, sgrid, sblock, strip_bytes, s, pixels, (bf16_t*)patches, ld, C, S,
                         p, g, K, Kpad);
    } else {
      static LdsLimitOnce lim;
      if (hipError_t e = lim.ensure((const void*)patch_gather_strip_kernel<float>, 64 * 1024); e != hipSuccess) return e;
      hipLaunchKernelGGL(patch_gather_strip_kernel<float>, sgrid, sblock, strip_bytes, s, pixels, (float*)patches, ld, C, S, p,
                         g, K, Kpad);
    }
    return hipGetLastError();
  }
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (out_bf16)
    hipLaunchKernelGGL(patch_gather_kernel<bf16_t>, grid, block, 0, s, pixels, (bf16_t*)patches, ld, total, C, S, p, g,
                       K, Kpad);
  else
    hipLaunchKernelGGL(patch_gather_kernel<float>, grid, block, 0, s, pixels, (float*)patches, ld, total, C, S, p, g, K,
                       Kpad);
  return hipGetLastError();
}

hipError_t launch_cls_rows(float* x, int ldx, const float* cls, const float* pos, int n_tiles, int T, int D,
                           hipStream_t s) {
  const long total = (long)n_tiles * D;
  if (total <= 0) return hipSuccess;
  hipLaunchKernelGGL(cls_rows_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, x, ldx, cls, pos, n_tiles,
                     T, D);
  return hipGetLastError();
}

hipError_t launch_token_merge(const void* src, int src_ld, void* dst, int dst_ld, int n_tiles, int T, int cls, int g,
                              int m, int D, int elem_bytes, hipStream_t s) {
  const long n_out = (long)n_tiles * (g / m) * (g / m);
  if (n_out <= 0) return hipSuccess;
  // 16-byte moves: the channel count and both leading dimensions must be whole chunks
  if (m < 1 || g % m != 0 || ((long)D * elem_bytes) % 16 != 0 || ((long)src_ld * elem_bytes) % 16 != 0 ||
      ((long)dst_ld * elem_bytes) % 16 != 0 || dst_ld < m * m * D)
    return hipErrorInvalidValue;
  const int row_chunks = D * elem_bytes / 16;
  const int pad_chunks = (dst_ld - m * m * D) * elem_bytes / 16;
  const long total = n_out * (m * m * row_chunks + pad_chunks);
  const long blocks = (total + 255) / 256;
  if (blocks > 0x7fffffffL) return hipErrorInvalidValue;
  hipLaunchKernelGGL(token_merge_kernel, dim3((unsigned)blocks), dim3(256), 0, s, (const unsigned char*)src,
                     (long)src_ld * elem_bytes, (unsigned char*)dst, (long)dst_ld * elem_bytes, n_out, T, cls, g, m,
                     row_chunks, pad_chunks);
  return hipGetLastError();
}

hipError_t launch_fill_zero_cols(void* buf, int ld, int rows, int col0, int col1, int elem_bytes, hipStream_t s) {
  const int ncols = col1 - col0;
  const long total = (long)rows * ncols;
  if (total <= 0) return hipSuccess;
  const dim3 grid((unsigned)((total + 255) / 256)), block(256);
  if (elem_bytes == 2)
    hipLaunchKernelGGL(fill_zero_cols_kernel<bf16_t>, grid, block, 0, s, (bf16_t*)buf, ld, (long)rows, col0, ncols);
  else
    hipLaunchKernelGGL(fill_zero_cols_kernel<float>, grid, block, 0, s, (float*)buf, ld, (long)rows, col0, ncols);
  return hipGetLastError();
}

}  // namespace vitenc
