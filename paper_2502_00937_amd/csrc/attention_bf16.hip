// Variable-length flash attention on bf16 MFMA.  A work item is a block of query rows of
// one segment (a tile, or all tiles of an image); keys never come from outside the
// segment, so no padding or masking crosses images.
//
// Everything is computed transposed so that a lane owns one query for the whole kernel:
//   S^T[key, q]  = K[key, :] . Q[q, :]       (A = K tile from LDS, B = Q^T held in registers)
//   O^T[d, q]   += V^T[d, key] . P^T[key, q] (A = V^T tile from LDS, B = P^T straight from the
//                                             S^T accumulator registers)
// With the 32x32 MFMA accumulator layout (lane = column q, registers = rows) the softmax
// statistics of a query are per-lane scalars, the row maximum needs one exchange with lane^32,
// and the P^T operand of the second product is the accumulator of the first, converted in
// place: registers 8s..8s+7 of an S^T block are exactly the 8 k-values lane group g feeds
// to k-step s, provided V^T is read in the same key order (keys 16s + 8jj + 4g + i).
#include "common.h"

namespace vitenc {

namespace {

constexpr int AQ = 128;   // query rows per workgroup (4 waves x 32)
constexpr int AKV = 64;   // keys per LDS tile

template <int DHP>
struct AttnShape {
  static constexpr int KS = DHP / 16;               // k-steps of the S^T product
  static constexpr int DB = (DHP + 31) / 32;        // 32-row blocks of O^T
  static constexpr int NCH = DHP / 8;               // 16-byte chunks per K/V row
  static constexpr int K_STRIDE = DHP * 2 + 16;     // bytes per K row in LDS (padding kills bank conflicts)
  static constexpr int VT_STRIDE = AKV * 2 + 8;     // bytes per V^T row in LDS
  static constexpr int K_BYTES = AKV * K_STRIDE;
  static constexpr int VT_BYTES = DB * 32 * VT_STRIDE;
};

template <int DHP>
__global__ __launch_bounds__(256) void attention_bf16_kernel(const AttnArgs a, float scale_log2) {
  using Sh = AttnShape<DHP>;
  __shared__ __attribute__((aligned(16))) unsigned char sK[Sh::K_BYTES];
  __shared__ __attribute__((aligned(16))) unsigned char sVt[Sh::VT_BYTES];

  const AttnWork w = a.work[blockIdx.x];
  const int head = blockIdx.y;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int lq = lane & 31, g = lane >> 5;
  const bf16_t* base = (const bf16_t*)a.qkv;
  const int qoff = head * DHP, koff = (a.heads + head) * DHP, voff = (2 * a.heads + head) * DHP;
  const int seg_end = w.seg_start + w.seg_len;
  const int qrow = w.q0 + wave * 32 + lq;
  const int qload = min(qrow, seg_end - 1);  // rows past the segment end compute on a copy of its last row

  // Q^T fragments: lane holds d = 16*ks + 8*g .. +8 of its query row.
  bf16x8 qf[Sh::KS];
#pragma unroll
  for (int ks = 0; ks < Sh::KS; ++ks)
    qf[ks] = *(const bf16x8*)(base + (size_t)qload * a.ld_qkv + qoff + ks * 16 + g * 8);

  f32x16 o[Sh::DB];
#pragma unroll
  for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
    for (int v = 0; v < 16; ++v) o[b][v] = 0.f;
  float m = -INFINITY, l = 0.f;

  constexpr int K_ITEMS = AKV * Sh::NCH;          // 16-byte chunks of the K tile
  constexpr int V_ITEMS = (AKV / 2) * Sh::NCH;    // (key pair, chunk) items of the V tile
  constexpr int K_PER = (K_ITEMS + 255) / 256, V_PER = (V_ITEMS + 255) / 256;

  for (int k0 = 0; k0 < w.seg_len; k0 += AKV) {
    // ---- global -> registers (rows past the segment end are clamped to its last row; their
    //      logits are masked below, the clamped values only need to be finite)
    u32x4 rk[K_PER], rv0[V_PER], rv1[V_PER];
#pragma unroll
    for (int i = 0; i < K_PER; ++i) {
      const int it = tid + i * 256;
      if (it < K_ITEMS) {
        const int key = it / Sh::NCH, ch = it - key * Sh::NCH;
        const int row = min(w.seg_start + k0 + key, seg_end - 1);
        rk[i] = *(const u32x4*)(base + (size_t)row * a.ld_qkv + koff + ch * 8);
      }
    }
#pragma unroll
    for (int i = 0; i < V_PER; ++i) {
      const int it = tid + i * 256;
      if (it < V_ITEMS) {
        const int ch = it >> 5, kp = it & 31;
        const int r0 = min(w.seg_start + k0 + 2 * kp, seg_end - 1);
        const int r1 = min(w.seg_start + k0 + 2 * kp + 1, seg_end - 1);
        rv0[i] = *(const u32x4*)(base + (size_t)r0 * a.ld_qkv + voff + ch * 8);
        rv1[i] = *(const u32x4*)(base + (size_t)r1 * a.ld_qkv + voff + ch * 8);
      }
    }
    __syncthreads();  // everyone finished reading the previous tile
#pragma unroll
    for (int i = 0; i < K_PER; ++i) {
      const int it = tid + i * 256;
      if (it < K_ITEMS) {
        const int key = it / Sh::NCH, ch = it - key * Sh::NCH;
        *(u32x4*)(sK + key * Sh::K_STRIDE + ch * 16) = rk[i];
      }
    }
#pragma unroll
    for (int i = 0; i < V_PER; ++i) {
      const int it = tid + i * 256;
      if (it < V_ITEMS) {
        const int ch = it >> 5, kp = it & 31;
        // transpose on the way in: V^T[d][2kp], V^T[d][2kp+1] packed into one 32-bit word
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const uint32_t x0 = rv0[i][e], x1 = rv1[i][e];
          const uint32_t lo = (x0 & 0xFFFFu) | (x1 << 16);
          const uint32_t hi = (x0 >> 16) | (x1 & 0xFFFF0000u);
          *(uint32_t*)(sVt + (ch * 8 + 2 * e) * Sh::VT_STRIDE + kp * 4) = lo;
          *(uint32_t*)(sVt + (ch * 8 + 2 * e + 1) * Sh::VT_STRIDE + kp * 4) = hi;
        }
      }
    }
    __syncthreads();

    // ---- S^T = K . Q^T for the two 32-key blocks of the tile
    f32x16 st[2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
#pragma unroll
      for (int v = 0; v < 16; ++v) st[kb][v] = 0.f;
#pragma unroll
      for (int ks = 0; ks < Sh::KS; ++ks) {
        const bf16x8 kf = *(const bf16x8*)(sK + (kb * 32 + lq) * Sh::K_STRIDE + (ks * 2 + g) * 16);
        st[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], st[kb], 0, 0, 0);
      }
    }
    // ---- scale, mask keys past the segment end, running max
    const int remaining = w.seg_len - k0;  // valid keys in this tile (may exceed AKV)
    float mx = -INFINITY;
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int key = kb * 32 + 8 * (v >> 2) + 4 * g + (v & 3);
        float s = st[kb][v] * scale_log2;
        s = key < remaining ? s : -INFINITY;
        st[kb][v] = s;
        mx = fmaxf(mx, s);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m, mx);
    const float corr = __builtin_amdgcn_exp2f(m - m_new);
    m = m_new;
    float psum = 0.f;
    bf16x8 pf[2][2];
#pragma unroll
    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2)
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float p = __builtin_amdgcn_exp2f(st[kb][s2 * 8 + e] - m_new);
          psum += p;
          pf[kb][s2][e] = (__bf16)p;
        }
    l = l * corr + psum;
#pragma unroll
    for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[b][v] *= corr;
    // ---- O^T += V^T . P^T
#pragma unroll
    for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int s2 = 0; s2 < 2; ++s2) {
          const unsigned char* p = sVt + (b * 32 + lq) * Sh::VT_STRIDE + (kb * 32 + s2 * 16 + 4 * g) * 2;
          const u32x2 lo = *(const u32x2*)p, hi = *(const u32x2*)(p + 16);
          const u32x4 packed = {lo[0], lo[1], hi[0], hi[1]};
          o[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, packed), pf[kb][s2], o[b], 0, 0, 0);
        }
  }

  // ---- normalise and store: lane owns query qrow; registers 4j..4j+3 of block b are
  //      d = 32b + 8j + 4g .. +3, four consecutive columns -> one 8-byte store
  l += __shfl_xor(l, 32, 64);
  if (qrow < seg_end) {
    const float inv = 1.0f / l;
    bf16_t* orow = (bf16_t*)a.out + (size_t)qrow * a.ld_o + head * DHP;
#pragma unroll
    for (int b = 0; b < Sh::DB; ++b)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int d = b * 32 + 8 * j + 4 * g;
        if (d < DHP) {
          const u32x2 pk = {pack_bf16x2(o[b][4 * j] * inv, o[b][4 * j + 1] * inv),
                            pack_bf16x2(o[b][4 * j + 2] * inv, o[b][4 * j + 3] * inv)};
          *(u32x2*)(orow + d) = pk;
        }
      }
  }
}

}  // namespace

int attention_q_block(int dtype_bf16) { return dtype_bf16 ? AQ : 64; }

hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s) {
  if (a.n_work <= 0) return hipSuccess;
  if (a.ld_qkv % 8 != 0 || a.ld_o % 4 != 0) return hipErrorInvalidValue;
  const float scale_log2 = 1.4426950408889634f / sqrtf((float)a.dh);
  const dim3 grid(a.n_work, a.heads), block(256);
  switch (a.dh_pad) {
    case 64: hipLaunchKernelGGL(attention_bf16_kernel<64>, grid, block, 0, s, a, scale_log2); break;
    case 80: hipLaunchKernelGGL(attention_bf16_kernel<80>, grid, block, 0, s, a, scale_log2); break;
    case 96: hipLaunchKernelGGL(attention_bf16_kernel<96>, grid, block, 0, s, a, scale_log2); break;
    case 128: hipLaunchKernelGGL(attention_bf16_kernel<128>, grid, block, 0, s, a, scale_log2); break;
    default: return hipErrorInvalidValue;
  }
  return hipGetLastError();
}

}  // namespace vitenc
