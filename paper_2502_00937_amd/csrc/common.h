// Shared device helpers and the launcher interface between the host plan and the kernels.
// gfx950 only: wave64, MFMA with 8-element bf16 operands.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

namespace vitenc {

// A kernel's dynamic-LDS limit is an attribute of (kernel, device): raised once for each device a launcher
// runs on, with that device current.  One object per kernel instantiation; safe to call from several threads.
struct LdsLimitOnce {
  std::atomic<uint64_t> done{0};
  hipError_t ensure(const void* fn, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    const uint64_t bit = 1ull << dev;
    if (done.load(std::memory_order_acquire) & bit) return hipSuccess;
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return e;
    done.fetch_or(bit, std::memory_order_release);
    return hipSuccess;
  }
};

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

typedef uint16_t bf16_t;  // storage type of a bfloat16 value in global memory

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

// fp32 -> bf16, round to nearest even; NaN stays NaN.  On the device this is the hardware
// conversion (v_cvt_pk_bf16_f32), on the host the integer form of the same rounding.
__host__ __device__ inline bf16_t f32_to_bf16(float f) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __builtin_bit_cast(bf16_t, (__bf16)f);
#else
  union { float f; uint32_t u; } v;
  v.f = f;
  if ((v.u & 0x7FFFFFFFu) > 0x7F800000u) return (bf16_t)((v.u >> 16) | 0x40u);
  v.u += 0x7FFFu + ((v.u >> 16) & 1u);
  return (bf16_t)(v.u >> 16);
#endif
}
__host__ __device__ inline float bf16_to_f32(bf16_t h) {
  union { float f; uint32_t u; } v;
  v.u = ((uint32_t)h) << 16;
  return v.f;
}
// two fp32 -> packed pair of bf16 (low half = a)
__device__ inline uint32_t pack_bf16x2(float a, float b) {
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}

// Element-type traits for the two arithmetic modes.
template <typename T> struct Elem;
template <> struct Elem<float> {
  __device__ static inline float load(const float* p) { return *p; }
  __device__ static inline void store(float* p, float v) { *p = v; }
};
template <> struct Elem<bf16_t> {
  __device__ static inline float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static inline void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// Exact-form GELU z/2 (1 + erf(z / sqrt 2)).
__device__ inline float gelu_erf(float z) { return 0.5f * z * (1.0f + erff(z * 0.70710678118654752440f)); }

// GELU for the bf16 path, z/2 * (1 + erf(z / sqrt 2)), without transcendental instructions, taking HALF its
// argument (the epilogue forms h = z / 2 with the multiply-add that adds the bias): with t = min(|h|, 2),
// erf(sqrt 2 h) ~ t * Q(t^2), Q a degree-6 minimax polynomial (weighted for the error of the product below)
// constrained to 2 * Q(4) = 1 - 2e-6, so the value never exceeds 1 and large |z| give z resp. 0 to 3e-6 relative.
// |error of the result| <= 1.9e-4 for |z| <= 50, largest near |z| = 3.9, where the bf16 output's own rounding
// step is 1.6e-2.  The epilogue that applies it is bound by its VALU instructions: this form costs 10 of them
// after the bias multiply-add; the rational approximation on exp2 / rcp cost 14 plus two quarter-rate ones.
__device__ inline float gelu_fast_half(float h) {
  const float t = fminf(fabsf(h), 2.0f);
  const float u = t * t;
  float p = fmaf(3.698568902e-04f, u, -6.504944063e-03f);
  p = fmaf(p, u, 4.889602571e-02f);
  p = fmaf(p, u, -2.078860937e-01f);
  p = fmaf(p, u, 5.608358441e-01f);
  p = fmaf(p, u, -1.032848863e+00f);
  p = fmaf(p, u, 1.591477259e+00f);
  const float e = t * p;          // erf(|z| / sqrt 2), in [0, 1)
  return fmaf(fabsf(h), e, h);    // (z + |z| erf) / 2
}

// ---- epilogues of the matrix products ---------------------------------------------------
enum Epilogue {
  EPI_BIAS = 0,           // out[r, c] = acc + bias[c]                         (activation type)
  EPI_BIAS_GELU = 1,      // out[r, c] = gelu(acc + bias[c])                   (activation type)
  EPI_BIAS_RESIDUAL = 2,  // resid[r, c] += acc + bias[c]                      (fp32, in place)
  EPI_PATCH = 3,          // resid[tile*T + cls + patch, c] = acc + bias[c] + pos[cls + patch, c]
  EPI_BIAS_HEADS = 4      // bf16 only: EPI_BIAS with the output laid out head by head (GemmArgs::hm_dh)
};

struct GemmArgs {
  const void* A;      // [M_pad, lda] activations, K contiguous
  const void* W;      // [N_pad, ldw] weights, K contiguous (zero padded)
  const float* bias;  // [N_pad]
  void* out;          // activation-type output (EPI_BIAS, EPI_BIAS_GELU)
  float* resid;       // fp32 residual stream (EPI_BIAS_RESIDUAL, EPI_PATCH)
  const float* pos;   // [T, ld_resid] position table (EPI_PATCH)
  int M;              // valid rows
  int N;              // valid output columns (stores are masked beyond)
  int K;              // padded contraction length, multiple of 64
  int lda, ldw, ldo;  // leading dimensions in elements (ldo: of out or resid)
  int patches;        // EPI_PATCH: patches per tile P
  int tokens;         // EPI_PATCH: tokens per tile T
  int cls;            // EPI_PATCH: 1 if a CLS row precedes the patches
  int epilogue;
  int reverse;        // 1: walk the row blocks from the last to the first (see vit_encode_packed)
  unsigned long long* tile_stamps;  // measurement aid, normally null: [256 workgroups][kTileStampSlots][4] words written
                                    // by the persistent kernel per tile (see vit_profile_tiles_read)
  int q_cols;         // EPI_BIAS, EPI_BIAS_HEADS: output columns [0, q_cols) are multiplied by q_scale after the bias (0: none);
  float q_scale;      //   the QKV product hands the attention kernel its queries times log2(e) / sqrt(head dim)
  int stream_out;     // 1: the bf16 output exceeds the memory-side cache; the persistent kernel stores it non-temporally
  int hm_dh;          // EPI_BIAS_HEADS: 64 or 128; the output is laid out head by head, column c of row r at
  size_t hm_rows;     //   ((c / hm_dh) * hm_rows + r) * hm_dh + c % hm_dh (every head's rows contiguous: what the
                      //   attention kernel reads); ldo is not used
};

// Applies one epilogue to a single accumulator; the caller guarantees row < M and col < N.
template <int EPI, typename OutT>
__device__ __forceinline__ void epilogue_store(const GemmArgs& a, int row, int col, float acc) {
  float v = acc + a.bias[col];
  if constexpr (EPI == EPI_BIAS) {
    Elem<OutT>::store((OutT*)a.out + (size_t)row * a.ldo + col, v);
  } else if constexpr (EPI == EPI_BIAS_GELU) {
    Elem<OutT>::store((OutT*)a.out + (size_t)row * a.ldo + col, gelu_erf(v));
  } else if constexpr (EPI == EPI_BIAS_RESIDUAL) {
    float* p = a.resid + (size_t)row * a.ldo + col;
    *p += v;
  } else {  // EPI_PATCH
    int tile = row / a.patches;
    int tok = a.cls + (row - tile * a.patches);
    a.resid[((size_t)tile * a.tokens + tok) * a.ldo + col] = v + a.pos[(size_t)tok * a.ldo + col];
  }
}

constexpr int kTileStampSlots = 64;  // tiles per workgroup whose phases are recorded

// Attention work item: one block of query rows inside one segment.
struct AttnWork {
  int32_t q0;         // first query row (global token row)
  int32_t seg_start;  // first key row of the segment
  int32_t seg_len;    // number of keys in the segment
};

struct AttnArgs {
  const void* qkv;  // qkv_rows == 0: [rows, ld_qkv], Q heads, then K heads, then V heads, each head dh_pad wide;
                    // else (bf16 path, head dims 64 and 128) the same 3 * heads column blocks laid out one after
                    // the other, each [qkv_rows, dh_pad] (GemmArgs::hm_dh): a head's keys are consecutive rows
  size_t qkv_rows;  // rows of each head's block, or 0
  void* out;        // [rows, ld_o]: head h at columns h*dh_pad
  const AttnWork* work;
  int n_work;
  int heads;
  int dh;      // true head dim (for the logit scale)
  int dh_pad;  // padded head dim used in memory
  int ld_qkv, ld_o;
  int reverse;  // 1: walk the work list from the last item to the first
};

// ---- launchers (defined in the .hip files) ----------------------------------------------
// bf16 MFMA path
hipError_t launch_gemm_bf16(const GemmArgs& a, hipStream_t s);
hipError_t launch_attention_bf16(const AttnArgs& a, hipStream_t s);
// fp32 path
hipError_t launch_gemm_f32(const GemmArgs& a, hipStream_t s);
hipError_t launch_attention_f32(const AttnArgs& a, hipStream_t s);
// shared, templated on activation type inside
hipError_t launch_layernorm(const float* x, int ldx, void* out, int ldo, int out_cols, const float* gamma,
                            const float* beta, float eps, int rows, int D, int normalize, int out_bf16, int reverse,
                            int stream_in, hipStream_t s);  // stream_in: x exceeds the memory-side cache, read it non-temporally
hipError_t launch_patch_gather(const float* pixels, void* patches, int ld, int n_tiles, int C, int S, int p, int g,
                               int Kpad, int out_bf16, hipStream_t s);
hipError_t launch_cls_rows(float* x, int ldx, const float* cls, const float* pos, int n_tiles, int T, int D,
                           hipStream_t s);
hipError_t launch_fill_zero_cols(void* buf, int ld, int rows, int col0, int col1, int elem_bytes, hipStream_t s);
// dst[tile*(g/m)^2 + y2*(g/m) + x2, (dy*m + dx)*D + c] = src[tile*T + cls + (y2*m + dy)*g + x2*m + dx, c];
// columns [m*m*D, dst_ld) of dst are zeroed
hipError_t launch_token_merge(const void* src, int src_ld, void* dst, int dst_ld, int n_tiles, int T, int cls, int g,
                              int m, int D, int elem_bytes, hipStream_t s);

int attention_q_block(int dtype_bf16, int dh_pad);  // query rows per work item for each path and head dim
int gemm_row_pad();                     // row padding every activation buffer must have

}  // namespace vitenc
