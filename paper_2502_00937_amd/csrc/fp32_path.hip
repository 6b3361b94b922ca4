// fp32 arithmetic mode: plain FMA matrix product and attention.  This mode exists for
// exact-arithmetic parity runs on small encoders; it is not the throughput path.
#include "common.h"

namespace vitenc {

namespace {

// C[M, N] = A[M, K] . W[N, K]^T, 64x64 tile, 16-wide k-steps, 4x4 outputs per thread.
// Operand rows are padded by the host so tile loads never leave the buffers.
template <int EPI>
__global__ __launch_bounds__(256) void gemm_f32_kernel(const GemmArgs a) {
  __shared__ float sA[16][68];
  __shared__ float sB[16][68];
  const int tid = threadIdx.x;
  const int m0 = blockIdx.y * 64, n0 = blockIdx.x * 64;
  const float* A = (const float*)a.A + (size_t)m0 * a.lda;
  const float* W = (const float*)a.W + (size_t)n0 * a.ldw;
  const int lrow = tid >> 2, lk = (tid & 3) * 4;
  const int tx = tid & 15, ty = tid >> 4;  // thread computes rows ty*4.., cols tx + 16*j
  float acc[4][4] = {};
  for (int k0 = 0; k0 < a.K; k0 += 16) {
    const f32x4 va = *(const f32x4*)(A + (size_t)lrow * a.lda + k0 + lk);
    const f32x4 vb = *(const f32x4*)(W + (size_t)lrow * a.ldw + k0 + lk);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      sA[lk + e][lrow] = va[e];
      sB[lk + e][lrow] = vb[e];
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 16; ++k) {
      float ra[4], rb[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) ra[i] = sA[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) rb[j] = sB[k][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(ra[i], rb[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty * 4 + i;
    if (row >= a.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx + 16 * j;
      if (col < a.N) epilogue_store<EPI, float>(a, row, col, acc[i][j]);
    }
  }
}

// One workgroup = 64 query rows x one head; 4 adjacent lanes share a query row, each owning a
// quarter of the head dimension.  Keys/values are staged in LDS 64 at a time; softmax is the
// running-max / running-sum form, all in fp32.
constexpr int F32_BK = 64, F32_DQ_MAX = 32;  // (the 64 query rows are what attention_q_block reports for fp32)

__global__ __launch_bounds__(256) void attention_f32_kernel(const AttnArgs a) {
  extern __shared__ float smem_f[];
  const int dhp = a.dh_pad, dq = dhp >> 2;
  float* sK = smem_f;               // [64][dhp + 4]
  float* sV = smem_f + F32_BK * (dhp + 4);
  const int ldk = dhp + 4;
  const AttnWork w = a.work[blockIdx.x];
  const int head = blockIdx.y;
  const int tid = threadIdx.x, qi = tid >> 2, part = tid & 3;
  const int seg_end = w.seg_start + w.seg_len;
  const int qrow = w.q0 + qi;
  const bool qvalid = qrow < seg_end;
  const float* base = (const float*)a.qkv;
  const int qoff = head * dhp, koff = (a.heads + head) * dhp, voff = (2 * a.heads + head) * dhp;
  float q[F32_DQ_MAX], o[F32_DQ_MAX];
  const float scale = 1.0f / sqrtf((float)a.dh);
#pragma unroll
  for (int i = 0; i < F32_DQ_MAX; ++i) {
    o[i] = 0.f;
    q[i] = (i < dq && qvalid) ? base[(size_t)qrow * a.ld_qkv + qoff + part * dq + i] * scale : 0.f;
  }
  float m = -INFINITY, l = 0.f;
  for (int k0 = 0; k0 < w.seg_len; k0 += F32_BK) {
    const int nk = min(F32_BK, w.seg_len - k0);
    for (int idx = tid; idx < nk * dhp; idx += 256) {
      const int r = idx / dhp, c = idx - r * dhp;
      const size_t g = (size_t)(w.seg_start + k0 + r) * a.ld_qkv;
      sK[r * ldk + c] = base[g + koff + c];
      sV[r * ldk + c] = base[g + voff + c];
    }
    __syncthreads();
    for (int j = 0; j < nk; ++j) {
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < F32_DQ_MAX; ++i)
        if (i < dq) s = fmaf(q[i], sK[j * ldk + part * dq + i], s);
      s += __shfl_xor(s, 1, 64);
      s += __shfl_xor(s, 2, 64);
      const float mn = fmaxf(m, s);
      const float corr = expf(m - mn), p = expf(s - mn);  // the library's exp: this mode is for exact-arithmetic parity
      l = l * corr + p;
      m = mn;
#pragma unroll
      for (int i = 0; i < F32_DQ_MAX; ++i)
        if (i < dq) o[i] = fmaf(p, sV[j * ldk + part * dq + i], o[i] * corr);
    }
    __syncthreads();
  }
  if (qvalid) {
    const float inv = 1.0f / l;
    float* out = (float*)a.out + (size_t)qrow * a.ld_o + head * dhp + part * dq;
#pragma unroll
    for (int i = 0; i < F32_DQ_MAX; ++i)
      if (i < dq) out[i] = o[i] * inv;
  }
}

}  // namespace

hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s) {
  if (a.M <= 0 || a.N <= 0) return hipSuccess;
  if (a.K <= 0 || a.K % 16 != 0 || a.lda % 4 != 0 || a.ldw % 4 != 0) return hipErrorInvalidValue;
  const dim3 grid((a.N + 63) / 64, (a.M + 63) / 64), block(256);
  switch (a.epilogue) {
    case EPI_BIAS: hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS>, grid, block, 0, s, a); break;
    case EPI_BIAS_GELU: hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_GELU>, grid, block, 0, s, a); break;
    case EPI_BIAS_RESIDUAL: hipLaunchKernelGGL(gemm_f32_kernel<EPI_BIAS_RESIDUAL>, grid, block, 0, s, a); break;
    case EPI_PATCH: hipLaunchKernelGGL(gemm_f32_kernel<EPI_PATCH>, grid, block, 0, s, a); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

hipError_t launch_attention_f32(const AttnArgs& a, hipStream_t s) {
  if (a.n_work <= 0) return hipSuccess;
  if (a.dh_pad % 4 != 0 || a.dh_pad > 4 * F32_DQ_MAX) return hipErrorInvalidValue;
  const size_t smem = 2 * F32_BK * (a.dh_pad + 4) * sizeof(float);
  hipError_t e = hipFuncSetAttribute((const void*)attention_f32_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                     (int)(2 * F32_BK * (4 * F32_DQ_MAX + 4) * sizeof(float)));
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(attention_f32_kernel, dim3(a.n_work, a.heads), dim3(256), smem, s, a);
  return hipGetLastError();
}

}  // namespace vitenc
