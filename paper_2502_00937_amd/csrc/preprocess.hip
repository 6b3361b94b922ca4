// Image preprocessing on the GPU (paper Sec. 2, "Image Preprocessing": resize, rescale, normalise,
// segment into tiles): one 8-bit interleaved image in, the encoder's fp32 [tile, C, S, S] pixels out.
// Bound by HBM: C bytes read per source pixel (the four taps of neighbouring outputs share cache
// lines), 4C bytes written per output pixel.
#include "../../include/vitenc.h"

#include <hip/hip_runtime.h>

#include <cmath>

namespace vitenc {
vit_status_t set_error(vit_status_t st, const char* fmt, ...);  // vitenc_api.hip: message for vit_last_error()
}
using vitenc::set_error;

namespace {

struct PrepArgs {
  const unsigned char* img;
  float* out;
  int H, W, C, S, rows, cols, thumb;
  float scale[4], shift[4];  // out = tap * scale[c] + shift[c]: 1/(255 std) and -mean/std
};

// Source taps of output coordinate o on an axis resized from n_in to n_out pixels (pixel centres at
// half-integers, coordinate clamped below at 0, last pixel repeated above).
__device__ __forceinline__ void taps(int o, float ratio, int n_in, int& i0, int& i1, float& w) {
  float src = ((float)o + 0.5f) * ratio - 0.5f;
  src = fmaxf(src, 0.f);
  i0 = min((int)src, n_in - 1);
  i1 = min(i0 + 1, n_in - 1);
  w = src - (float)i0;
}

// One thread per output pixel (x fastest, so a wave writes 256 contiguous bytes per channel plane);
// grid.y = tile index, the thumbnail (if any) is the last one.
__global__ __launch_bounds__(256) void preprocess_kernel(const PrepArgs a) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx >= a.S * a.S) return;
  const int y = idx / a.S, x = idx - y * a.S;
  const int tile = blockIdx.y, n_grid = a.rows * a.cols;
  int oy, ox, out_h, out_w;
  if (tile < n_grid) {  // a tile of the (rows*S) x (cols*S) canvas
    const int ty = tile / a.cols, tx = tile - ty * a.cols;
    oy = ty * a.S + y; ox = tx * a.S + x;
    out_h = a.rows * a.S; out_w = a.cols * a.S;
  } else {  // the whole image at S x S
    oy = y; ox = x;
    out_h = a.S; out_w = a.S;
  }
  int y0, y1, x0, x1;
  float wy, wx;
  taps(oy, (float)a.H / (float)out_h, a.H, y0, y1, wy);
  taps(ox, (float)a.W / (float)out_w, a.W, x0, x1, wx);
  const unsigned char* r0 = a.img + (size_t)y0 * a.W * a.C;
  const unsigned char* r1 = a.img + (size_t)y1 * a.W * a.C;
  float* o = a.out + ((size_t)tile * a.C * a.S + y) * a.S + x;
  for (int c = 0; c < a.C; ++c) {
    const float p00 = r0[x0 * a.C + c], p01 = r0[x1 * a.C + c], p10 = r1[x0 * a.C + c], p11 = r1[x1 * a.C + c];
    const float top = p00 + (p01 - p00) * wx, bot = p10 + (p11 - p10) * wx;
    o[(size_t)c * a.S * a.S] = (top + (bot - top) * wy) * a.scale[c] + a.shift[c];
  }
}

}  // namespace

extern "C" vit_status_t vit_preprocess_tiles(const uint8_t* image, int32_t height, int32_t width, int32_t channels,
                                             int32_t tile_size, int32_t grid_rows, int32_t grid_cols,
                                             int32_t thumbnail, const float* mean, const float* std_,
                                             float* out_pixels, size_t out_capacity_bytes, void* stream) {
  if (!image || !mean || !std_ || !out_pixels) return set_error(VIT_EINVAL, "vit_preprocess_tiles: NULL argument");
  if (height <= 0 || width <= 0 || channels <= 0 || channels > 4 || tile_size <= 0 || grid_rows <= 0 || grid_cols <= 0)
    return set_error(VIT_EINVAL, "vit_preprocess_tiles: sizes must be positive and channels <= 4");
  if ((int64_t)grid_rows * grid_cols + 1 > 65535 || (int64_t)tile_size * tile_size > (int64_t)1 << 30 ||
      (int64_t)height * width * channels > (int64_t)1 << 40 || (int64_t)width * channels > INT32_MAX)
    return set_error(VIT_EINVAL, "vit_preprocess_tiles: at most 65534 tiles of at most 2^30 pixels, image rows below 2^31 bytes");
  PrepArgs a;
  for (int c = 0; c < channels; ++c) {
    if (!(std_[c] > 0.f) || !std::isfinite(std_[c]) || !std::isfinite(mean[c]))
      return set_error(VIT_EINVAL, "vit_preprocess_tiles: std must be positive, mean and std finite");
    a.scale[c] = 1.0f / (255.0f * std_[c]);
    a.shift[c] = -mean[c] / std_[c];
  }
  const int n_tiles = grid_rows * grid_cols + (thumbnail ? 1 : 0);
  const size_t need = (size_t)n_tiles * channels * tile_size * tile_size * sizeof(float);
  if (out_capacity_bytes < need)
    return set_error(VIT_ECAPACITY, "vit_preprocess_tiles: out_pixels holds %zu bytes, %zu needed", out_capacity_bytes, need);
  a.img = image; a.out = out_pixels;
  a.H = height; a.W = width; a.C = channels; a.S = tile_size; a.rows = grid_rows; a.cols = grid_cols;
  a.thumb = thumbnail ? 1 : 0;
  const dim3 grid((unsigned)(((int64_t)tile_size * tile_size + 255) / 256), (unsigned)n_tiles);
  hipLaunchKernelGGL(preprocess_kernel, grid, dim3(256), 0, (hipStream_t)stream, a);
  const hipError_t e = hipGetLastError();
  if (e != hipSuccess) return set_error(VIT_EDEVICE, "vit_preprocess_tiles: launch: %s", hipGetErrorString(e));
  return VIT_OK;
}
