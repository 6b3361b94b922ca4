// C ABI of the packed ViT encoder: validation, weight re-layout, segment planning,
// workspace carving and the launch sequence.  No arithmetic of the encoder happens on the
// host; every step runs in the kernels of this library.
#include "../../include/vitenc.h"

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <vector>

#include "common.h"

using namespace vitenc;

namespace {

thread_local char g_err[512] = "";

vit_status_t fail(vit_status_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}

}  // namespace

namespace vitenc {
// the same per-thread message buffer for the other translation units of the library
vit_status_t set_error(vit_status_t st, const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
  return st;
}
}  // namespace vitenc

namespace {

#define HIP_TRY(expr)                                                                       \
  do {                                                                                      \
    hipError_t e_ = (expr);                                                                 \
    if (e_ != hipSuccess) return fail(VIT_EDEVICE, "%s: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }

// Shapes derived from a config (all in elements).
struct Dims {
  int S, p, C, g, P, T, Kp, Kp_pad;
  int D, H, dh, dhp, M;
  int Dp, QKVN, Op, Mp;
  int L, L_loc;
  int proj_layers, proj_dims[2], proj0_ld;
  int out_dim;
  int bf16;  // 1: bf16 operands, 0: fp32
  int es;    // bytes per activation element
  float eps;
  int has_cls, final_ln;
  int merge;     // token down-sampling factor (1 = none)
  int T_out;     // output tokens per tile
  int pin, pin_ld;  // inputs of the first projector layer (merge^2 * D) and its padded leading dimension
};

bool derive(const vit_config_t* c, Dims* d, const char** why) {
  *why = "";
  if (!c) { *why = "cfg is NULL"; return false; }
  if (c->image_size <= 0 || c->patch_size <= 0 || c->channels <= 0 || c->patch_size > c->image_size) {
    *why = "image_size, patch_size, channels must be positive and patch_size <= image_size";
    return false;
  }
  // bounds that keep every derived count (tokens per tile, patch vector length, T * D) inside 32 bits
  if (c->channels > 16 || c->patch_size > 256 || c->image_size / c->patch_size > 512) {
    *why = "channels <= 16, patch_size <= 256 and floor(image_size / patch_size) <= 512";
    return false;
  }
  if (c->hidden <= 0 || c->heads <= 0 || c->hidden % c->heads != 0) { *why = "hidden must be a positive multiple of heads"; return false; }
  const int dh = c->hidden / c->heads;
  if (dh % 8 != 0 || dh > 128) { *why = "head dim must be a multiple of 8 and <= 128"; return false; }
  if (c->mlp <= 0 || c->mlp % 8 != 0 || c->mlp > 65536) { *why = "mlp must be a positive multiple of 8, at most 65536"; return false; }
  if (c->layers_local < 0 || c->layers_global < 0 || c->layers_local > 1024 || c->layers_global > 1024) {
    *why = "layer counts must be in [0, 1024]";
    return false;
  }
  if (c->has_cls != 0 && c->has_cls != 1) { *why = "has_cls must be 0 or 1"; return false; }
  if (c->final_ln != 0 && c->final_ln != 1) { *why = "final_ln must be 0 or 1"; return false; }
  if (!(c->ln_eps >= 0.f) || !std::isfinite(c->ln_eps)) { *why = "ln_eps must be finite and >= 0"; return false; }
  if (c->proj_layers < 0 || c->proj_layers > 2) { *why = "proj_layers must be 0, 1 or 2"; return false; }
  for (int i = 0; i < c->proj_layers; ++i)
    if (c->proj_dims[i] <= 0 || c->proj_dims[i] % 8 != 0 || c->proj_dims[i] > 65536) {
      *why = "proj_dims must be positive multiples of 8, at most 65536";
      return false;
    }
  if (c->dtype != VIT_DTYPE_FP32 && c->dtype != VIT_DTYPE_BF16) { *why = "dtype must be VIT_DTYPE_FP32 or VIT_DTYPE_BF16"; return false; }
  if (c->hidden > 4096) { *why = "hidden must be <= 4096"; return false; }
  if (c->token_merge < 0 || c->token_merge > 8) { *why = "token_merge must be in [0, 8]"; return false; }
  if (c->token_merge > 1 && (c->image_size / c->patch_size) % c->token_merge != 0) {
    *why = "floor(image_size / patch_size) must be a multiple of token_merge";
    return false;
  }

  d->S = c->image_size; d->p = c->patch_size; d->C = c->channels;
  d->g = d->S / d->p; d->P = d->g * d->g; d->T = d->P + c->has_cls;
  d->Kp = d->C * d->p * d->p; d->Kp_pad = (int)round_up(d->Kp, 64);
  d->D = c->hidden; d->H = c->heads; d->dh = dh; d->M = c->mlp;
  // head dims the attention kernels take as they are; every other one is stored padded to the next of these
  // (zero weight rows / columns), with the true head dim in the logit scale
  d->dhp = dh <= 64 ? 64 : dh == 72 ? 72 : dh <= 80 ? 80 : dh <= 96 ? 96 : 128;
  d->Dp = (int)round_up(d->D, 64);
  d->QKVN = 3 * d->H * d->dhp;
  d->Op = (int)round_up(d->H * d->dhp, 64);
  d->Mp = (int)round_up(d->M, 64);
  d->L_loc = c->layers_local; d->L = c->layers_local + c->layers_global;
  d->proj_layers = c->proj_layers;
  d->proj_dims[0] = c->proj_dims[0]; d->proj_dims[1] = c->proj_dims[1];
  d->proj0_ld = c->proj_layers == 2 ? (int)round_up(c->proj_dims[0], 64) : 0;
  d->merge = c->token_merge > 1 ? c->token_merge : 1;
  d->T_out = d->merge > 1 ? (d->g / d->merge) * (d->g / d->merge) : d->T;
  d->pin = d->merge * d->merge * d->D;
  d->pin_ld = d->merge > 1 ? (int)round_up(d->pin, 64) : d->Dp;
  d->out_dim = c->proj_layers ? c->proj_dims[c->proj_layers - 1] : d->pin;
  d->bf16 = c->dtype == VIT_DTYPE_BF16; d->es = d->bf16 ? 2 : 4;
  d->eps = c->ln_eps; d->has_cls = c->has_cls; d->final_ln = c->final_ln;
  return true;
}

size_t weight_count(const Dims& d) {
  size_t D = d.D, M = d.M, n = 0;
  n += D * d.Kp + D + (d.has_cls ? D : 0) + (size_t)d.T * D;
  n += (size_t)d.L * (2 * D + 3 * D * D + 3 * D + D * D + D + 2 * D + M * D + M + D * M + D);
  if (d.final_ln) n += 2 * D;
  size_t in = d.pin;
  for (int i = 0; i < d.proj_layers; ++i) { n += (size_t)d.proj_dims[i] * in + d.proj_dims[i]; in = d.proj_dims[i]; }
  return n;
}

// One matrix product's device-side weights.
struct Linear {
  const void* W = nullptr;   // [rows_pad, K] activation element type
  const float* bias = nullptr;
  int N = 0;                 // columns written
  int K = 0;                 // padded contraction length = leading dimension of W
};

struct Layer {
  const float *ln1_g, *ln1_b, *ln2_g, *ln2_b;
  Linear qkv, wo, w1, w2;
};

// Builds the device image of all weights in host memory, then uploads it in one copy.
struct Arena {
  std::vector<unsigned char> host;
  size_t reserve(size_t bytes) {
    size_t off = (host.size() + 255) / 256 * 256;
    host.resize(off + bytes, 0);
    return off;
  }
};

struct StageSlot {
  void* host = nullptr;
  size_t cap = 0;
  hipEvent_t done = nullptr;
  bool used = false;
};

struct ProfRec { int family; hipEvent_t start, stop; };

// One cached launch sequence of vit_encode_packed_graph.  The kernels' pointer arguments are part of a graph, so the
// key holds the three device buffers beside the batch shape.
struct GraphEntry {
  const void* pixels = nullptr;
  void* out = nullptr;
  void* workspace = nullptr;
  std::vector<int32_t> tile_offsets;  // n_images + 1
  hipGraphExec_t exec = nullptr;      // null until the key has been seen a second time
  uint64_t used = 0;
};
constexpr size_t kMaxGraphs = 8;

constexpr size_t kStampWordsPerFamily = (size_t)256 * kTileStampSlots * 4;

}  // namespace

struct vit_encoder {
  vit_config_t cfg;
  Dims d;
  int device = 0;
  unsigned char* dev_weights = nullptr;
  size_t dev_weight_bytes = 0;
  unsigned char* scratch = nullptr;  // this device's copy of the static scratch array (vit_encode_packed_static)
  hipError_t scratch_error = hipSuccess;
  unsigned long long* tile_stamps = nullptr;  // pinned [VIT_PROF_COUNT][256][kTileStampSlots][4], vit_profile_tiles_*
  Linear patch, proj[2];
  const float *cls = nullptr, *pos = nullptr, *lnf_g = nullptr, *lnf_b = nullptr;
  std::vector<Layer> layers;
  StageSlot stage[4];
  int next_stage = 0;
  bool profiling = false;
  std::vector<ProfRec> prof;
  std::vector<hipEvent_t> free_events;
  double prof_ms[VIT_PROF_COUNT] = {};
  int64_t prof_n[VIT_PROF_COUNT] = {};
  // vit_encode_packed_graph: launch sequences captured per (buffers, batch shape), least recently used replaced
  std::vector<GraphEntry> graphs;
  uint64_t graph_tick = 0;
  hipStream_t capture_stream = nullptr;
};

namespace {

// Copies src[rows, cols] (fp32, row-major) into the arena as [rows_pad, ld] of the activation
// element type, mapping source (row, col) through row_map / col_map (nullptr = identity).
size_t put_matrix(Arena& ar, const Dims& d, const float* src, int rows, int cols, int rows_pad, int ld,
                  const std::vector<int>* row_map, const std::vector<int>* col_map) {
  const size_t off = ar.reserve((size_t)rows_pad * ld * d.es);
  for (int r = 0; r < rows; ++r) {
    const int rr = row_map ? (*row_map)[r] : r;
    unsigned char* dst = ar.host.data() + off + (size_t)rr * ld * d.es;
    const float* s = src + (size_t)r * cols;
    if (d.bf16) {
      bf16_t* o = (bf16_t*)dst;
      if (col_map) for (int c = 0; c < cols; ++c) o[(*col_map)[c]] = f32_to_bf16(s[c]);
      else for (int c = 0; c < cols; ++c) o[c] = f32_to_bf16(s[c]);
    } else {
      float* o = (float*)dst;
      if (col_map) for (int c = 0; c < cols; ++c) o[(*col_map)[c]] = s[c];
      else memcpy(o, s, (size_t)cols * 4);
    }
  }
  return off;
}

size_t put_vector(Arena& ar, const float* src, int n, int n_pad, const std::vector<int>* map) {
  const size_t off = ar.reserve((size_t)n_pad * 4);
  float* o = (float*)(ar.host.data() + off);
  for (int i = 0; i < n; ++i) o[map ? (*map)[i] : i] = src[i];
  return off;
}

struct PendingLinear { Linear* dst; size_t w_off, b_off; };
struct PendingPtr { const float** dst; size_t off; };

hipEvent_t get_event(vit_encoder* e) {
  if (!e->free_events.empty()) {
    hipEvent_t ev = e->free_events.back();
    e->free_events.pop_back();
    return ev;
  }
  hipEvent_t ev = nullptr;
  if (hipEventCreate(&ev) != hipSuccess) return nullptr;
  return ev;
}

struct ProfScope {
  vit_encoder* e;
  hipStream_t s;
  int family;
  hipEvent_t start = nullptr, stop = nullptr;
  ProfScope(vit_encoder* e_, hipStream_t s_, int family_, bool on = true) : e(e_), s(s_), family(family_) {
    if (!on || !e->profiling) return;
    start = get_event(e);
    stop = get_event(e);
    if (start && stop) (void)hipEventRecord(start, s);
  }
  ~ProfScope() {
    if (!start || !stop) {  // an event could not be created: the launch goes untimed, nothing is kept
      if (start) (void)hipEventDestroy(start);
      if (stop) (void)hipEventDestroy(stop);
      return;
    }
    if (!e->profiling) return;
    (void)hipEventRecord(stop, s);
    try {
      e->prof.push_back({family, start, stop});
    } catch (...) {  // out of host memory: this one launch goes untimed
      (void)hipEventDestroy(start);
      (void)hipEventDestroy(stop);
    }
  }
};

// ---- the allocation-free entry point's device memory -------------------------------------------
// One array per GPU the library runs on, held until the process ends.  Every vit_encode_packed_static
// call on a GPU carves its workspace out of that GPU's copy.
constexpr size_t kStaticScratchBytes = VIT_STATIC_SCRATCH_BYTES;
constexpr int kStaticMaxImages = VIT_STATIC_MAX_IMAGES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// In host code `scratch` is only a handle for the symbol; the array's address on a device comes from
// hipGetSymbolAddress with that device current, looked up once per device and kept here.
std::atomic<unsigned char*> g_scratch_ptr[64];

hipError_t scratch_of_current_device(int device, unsigned char** out) {
  *out = nullptr;
  if (device < 0 || device >= 64) return hipErrorInvalidDevice;
  unsigned char* p = g_scratch_ptr[device].load(std::memory_order_acquire);
  if (!p) {
    void* sym = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)); e != hipSuccess) return e;
    if (!sym) return hipErrorInvalidSymbol;
    p = (unsigned char*)sym;
    g_scratch_ptr[device].store(p, std::memory_order_release);
  }
  *out = p;
  return hipSuccess;
}

// Attention work lists written on the device from tile offsets that travel as a kernel argument (no
// staging buffer, no copy).  Same order as the host-built lists: query blocks of tile 0, tile 1, ...;
// then, for global layers, query blocks of image 0, image 1, ...
struct TileOffsetsArg { int32_t v[kStaticMaxImages + 1]; };

__global__ __launch_bounds__(256) void attn_work_kernel(const TileOffsetsArg to, int n_images, int T, int bq,
                                                        AttnWork* __restrict__ loc, AttnWork* __restrict__ glob) {
  const int n_tiles = to.v[n_images];
  const int nb = (T + bq - 1) / bq;
  for (int idx = threadIdx.x; idx < n_tiles * nb; idx += 256) {
    const int t = idx / nb, j = idx - t * nb;
    loc[idx] = AttnWork{t * T + j * bq, t * T, T};
  }
  if (!glob) return;
  for (int i = threadIdx.x; i < n_images; i += 256) {
    int first = 0;
    for (int k = 0; k < i; ++k) first += ((to.v[k + 1] - to.v[k]) * T + bq - 1) / bq;
    const int start = to.v[i] * T, len = (to.v[i + 1] - to.v[i]) * T;
    for (int q = 0, n = 0; q < len; q += bq, ++n) glob[first + n] = AttnWork{start + q, start, len};
  }
}

// Register-only MFMA loop: eight independent 32x32 accumulators per wave, no memory traffic inside the
// loop.  What it sustains is the matrix cores' practical ceiling on this device: the clock the chip
// holds under full MFMA load times the issue rate.  That clock depends on the operand DATA (the chip
// is power-limited and random mantissas toggle far more of the multiplier array than constants do:
// about 1.75 PFLOP/s against 2.48 measured), so the operands are four fragments per matrix of
// caller-supplied values, here seeded uniform [-1, 1), as a matrix product of real activations has.
__global__ __launch_bounds__(256) void mfma_ceiling_kernel(const u32x4* __restrict__ frag, float* out, int iters) {
  bf16x8 a[4], b[4];
  for (int i = 0; i < 4; ++i) {
    a[i] = __builtin_bit_cast(bf16x8, frag[(threadIdx.x * 8 + i) & 4095]);
    b[i] = __builtin_bit_cast(bf16x8, frag[(threadIdx.x * 8 + 4 + i) & 4095]);
  }
  f32x16 acc[8];
  for (int j = 0; j < 8; ++j)
    for (int v = 0; v < 16; ++v) acc[j][v] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[j & 3], b[(j >> 1) & 3], acc[j], 0, 0, 0);
  }
  float sum = 0.f;
  for (int j = 0; j < 8; ++j)
    for (int v = 0; v < 16; ++v) sum += acc[j][v];
  if (sum == 123.456f) out[threadIdx.x] = sum;  // keeps the loop alive; never true in practice
}

}  // namespace

extern "C" {

const char* vit_last_error(void) { return g_err; }

size_t vit_weight_count(const vit_config_t* cfg) {
  Dims d;
  const char* why;
  if (!derive(cfg, &d, &why)) return 0;
  return weight_count(d);
}

vit_status_t vit_encoder_create(const vit_config_t* cfg, const float* weights, size_t n_weights, int device,
                                vit_encoder_t** out) {
  if (out) *out = nullptr;
  if (!cfg || !weights || !out) return fail(VIT_EINVAL, "vit_encoder_create: NULL argument");
  Dims d;
  const char* why;
  if (!derive(cfg, &d, &why)) return fail(VIT_EINVAL, "vit_encoder_create: invalid config: %s", why);
  if (n_weights != weight_count(d))
    return fail(VIT_EINVAL, "vit_encoder_create: n_weights = %zu but the config needs %zu", n_weights, weight_count(d));
  int ndev = 0;
  HIP_TRY(hipGetDeviceCount(&ndev));
  if (device < 0 || device >= ndev) return fail(VIT_EINVAL, "vit_encoder_create: device %d of %d", device, ndev);
  HIP_TRY(hipSetDevice(device));

  vit_encoder* e = new (std::nothrow) vit_encoder();
  if (!e) return fail(VIT_ENOMEM, "vit_encoder_create: out of host memory");
  e->cfg = *cfg;
  e->d = d;
  e->device = device;

  Arena ar;
  std::vector<PendingLinear> plin;
  std::vector<PendingPtr> pptr;
  try {
    e->layers.resize(d.L);
    // one allocation for the host image of the weights (padding adds a few per cent; a short estimate
    // only means the vector grows): a 6B-class encoder is 11 GB here, and growing by doubling would
    // hold three times that for a moment
    ar.host.reserve((size_t)((double)weight_count(d) * d.es * 1.1) + ((size_t)64 << 20));
    const float* w = weights;
    auto take = [&](size_t n) { const float* p = w; w += n; return p; };
    auto add_linear = [&](Linear* dst, const float* W, const float* b, int rows, int cols, int N, int K,
                          const std::vector<int>* row_map, const std::vector<int>* col_map) {
      const int rows_pad = (int)round_up(N, 256);
      const size_t wo = put_matrix(ar, d, W, rows, cols, rows_pad, K, row_map, col_map);
      const size_t bo = put_vector(ar, b, rows, rows_pad, row_map);
      dst->N = N;
      dst->K = K;
      plin.push_back({dst, wo, bo});
    };
    auto add_vec = [&](const float** dst, const float* v, int n) { pptr.push_back({dst, put_vector(ar, v, n, n, nullptr)}); };

    // head-padded orderings: source row s*D + h*dh + j -> (s*H + h)*dhp + j; source col h*dh + j -> h*dhp + j
    std::vector<int> qkv_rows(3 * d.D), o_cols(d.D);
    for (int s = 0; s < 3; ++s)
      for (int h = 0; h < d.H; ++h)
        for (int j = 0; j < d.dh; ++j) qkv_rows[s * d.D + h * d.dh + j] = (s * d.H + h) * d.dhp + j;
    for (int h = 0; h < d.H; ++h)
      for (int j = 0; j < d.dh; ++j) o_cols[h * d.dh + j] = h * d.dhp + j;

    const float* pw = take((size_t)d.D * d.Kp);
    const float* pb = take(d.D);
    add_linear(&e->patch, pw, pb, d.D, d.Kp, d.D, d.Kp_pad, nullptr, nullptr);
    if (d.has_cls) add_vec(&e->cls, take(d.D), d.D);
    add_vec(&e->pos, take((size_t)d.T * d.D), d.T * d.D);
    for (int l = 0; l < d.L; ++l) {
      Layer& L = e->layers[l];
      add_vec(&L.ln1_g, take(d.D), d.D);
      add_vec(&L.ln1_b, take(d.D), d.D);
      const float* wq = take((size_t)3 * d.D * d.D);
      const float* bq = take(3 * d.D);
      add_linear(&L.qkv, wq, bq, 3 * d.D, d.D, d.QKVN, d.Dp, &qkv_rows, nullptr);
      const float* wo = take((size_t)d.D * d.D);
      const float* bo = take(d.D);
      add_linear(&L.wo, wo, bo, d.D, d.D, d.D, d.Op, nullptr, &o_cols);
      add_vec(&L.ln2_g, take(d.D), d.D);
      add_vec(&L.ln2_b, take(d.D), d.D);
      const float* w1 = take((size_t)d.M * d.D);
      const float* b1 = take(d.M);
      add_linear(&L.w1, w1, b1, d.M, d.D, d.Mp, d.Dp, nullptr, nullptr);
      const float* w2 = take((size_t)d.D * d.M);
      const float* b2 = take(d.D);
      add_linear(&L.w2, w2, b2, d.D, d.M, d.D, d.Mp, nullptr, nullptr);
    }
    if (d.final_ln) {
      add_vec(&e->lnf_g, take(d.D), d.D);
      add_vec(&e->lnf_b, take(d.D), d.D);
    }
    int in = d.pin, in_ld = d.pin_ld;
    for (int i = 0; i < d.proj_layers; ++i) {
      const int dout = d.proj_dims[i];
      const float* W = take((size_t)dout * in);
      const float* b = take(dout);
      const bool last = i == d.proj_layers - 1;
      add_linear(&e->proj[i], W, b, dout, in, last ? dout : d.proj0_ld, in_ld, nullptr, nullptr);
      in = dout;
      in_ld = d.proj0_ld;
    }
  } catch (...) {  // bad_alloc, or length_error from a size no vector can hold
    delete e;
    return fail(VIT_ENOMEM, "vit_encoder_create: out of host memory while laying out weights");
  }

  e->dev_weight_bytes = ar.host.size();
  hipError_t he = hipMalloc((void**)&e->dev_weights, e->dev_weight_bytes);
  if (he != hipSuccess) {
    delete e;
    return fail(he == hipErrorOutOfMemory ? VIT_ENOMEM : VIT_EDEVICE, "vit_encoder_create: hipMalloc(%zu): %s",
                ar.host.size(), hipGetErrorString(he));
  }
  he = hipMemcpy(e->dev_weights, ar.host.data(), e->dev_weight_bytes, hipMemcpyHostToDevice);
  if (he != hipSuccess) {
    (void)hipFree(e->dev_weights);
    delete e;
    return fail(VIT_EDEVICE, "vit_encoder_create: weight upload: %s", hipGetErrorString(he));
  }
  for (auto& p : plin) {
    p.dst->W = e->dev_weights + p.w_off;
    p.dst->bias = (const float*)(e->dev_weights + p.b_off);
  }
  for (auto& p : pptr) *p.dst = (const float*)(e->dev_weights + p.off);
  // the static scratch array's address on this device (which is current here); a failure only disables
  // vit_encode_packed_static, which then reports it
  e->scratch_error = scratch_of_current_device(device, &e->scratch);
  *out = e;
  return VIT_OK;
}

void vit_encoder_destroy(vit_encoder_t* e) {
  if (!e) return;
  (void)hipSetDevice(e->device);
  if (e->tile_stamps) (void)hipHostFree(e->tile_stamps);
  for (auto& g : e->graphs)
    if (g.exec) (void)hipGraphExecDestroy(g.exec);
  if (e->capture_stream) (void)hipStreamDestroy(e->capture_stream);
  for (auto& r : e->prof) { (void)hipEventDestroy(r.start); (void)hipEventDestroy(r.stop); }
  for (auto ev : e->free_events) (void)hipEventDestroy(ev);
  for (auto& s : e->stage) {
    if (s.done) { (void)hipEventSynchronize(s.done); (void)hipEventDestroy(s.done); }
    if (s.host) (void)hipHostFree(s.host);
  }
  if (e->dev_weights) (void)hipFree(e->dev_weights);
  delete e;
}

}  // extern "C"

namespace {

// Workspace carving, shared by query and encode.
struct Workspace {
  int64_t n_tok, Mpad, patch_rows_pad, max_work;
  int64_t n_out, out_pad;
  size_t off_x, off_h, off_qkv, off_o, off_u, off_tables, off_merge, table_bytes, total;
};

void plan_workspace(const Dims& d, int64_t n_tiles, Workspace* w) {
  const int64_t pad = gemm_row_pad();
  w->n_tok = n_tiles * d.T;
  w->Mpad = round_up(std::max<int64_t>(w->n_tok, 1), pad);
  w->patch_rows_pad = round_up(std::max<int64_t>(n_tiles * d.P, 1), pad);
  const int bq = attention_q_block(d.bf16, d.dhp);
  w->max_work = n_tiles * ((d.T + bq - 1) / bq);
  size_t off = 0;
  auto carve = [&](size_t bytes) { size_t o = off; off += (bytes + 255) / 256 * 256; return o; };
  w->off_x = carve((size_t)w->Mpad * d.D * 4);
  w->off_h = carve((size_t)w->Mpad * d.Dp * d.es);
  w->off_qkv = carve((size_t)w->Mpad * d.QKVN * d.es);
  w->off_o = carve((size_t)w->Mpad * d.Op * d.es);
  size_t u_elems = (size_t)w->Mpad * std::max(d.Mp, d.proj0_ld);
  u_elems = std::max(u_elems, (size_t)w->patch_rows_pad * d.Kp_pad);
  w->off_u = carve(u_elems * d.es);
  w->table_bytes = (size_t)(d.L > d.L_loc ? 2 : 1) * w->max_work * sizeof(AttnWork);
  w->off_tables = carve(w->table_bytes);
  w->n_out = n_tiles * d.T_out;
  w->out_pad = round_up(std::max<int64_t>(w->n_out, 1), pad);
  // down-sampled rows ahead of the projector (with no projector they go straight to the output)
  w->off_merge = carve(d.merge > 1 && d.proj_layers > 0 ? (size_t)w->out_pad * d.pin_ld * d.es : 0);
  w->total = off;
}

}  // namespace

extern "C" {

vit_status_t vit_encoder_query(const vit_encoder_t* e, int32_t n_tiles, int32_t n_images, int64_t* n_tokens,
                               int32_t* out_dim, size_t* out_bytes, size_t* workspace_bytes) {
  if (!e) return fail(VIT_EINVAL, "vit_encoder_query: NULL encoder");
  if (n_tiles < 0 || n_images < 0 || n_images > n_tiles || (n_tiles > 0 && n_images == 0))
    return fail(VIT_EINVAL, "vit_encoder_query: need 0 <= n_images <= n_tiles and n_images >= 1 when n_tiles > 0");
  if ((int64_t)n_tiles * e->d.T > (int64_t)INT32_MAX - 1024)
    return fail(VIT_EINVAL, "vit_encoder_query: n_tiles * tokens_per_tile exceeds the 2^31 row limit");
  Workspace w;
  plan_workspace(e->d, n_tiles, &w);
  if (n_tokens) *n_tokens = w.n_out;
  if (out_dim) *out_dim = e->d.out_dim;
  if (out_bytes) *out_bytes = (size_t)w.n_out * e->d.out_dim * e->d.es;
  if (workspace_bytes) *workspace_bytes = n_tiles ? w.total : 0;
  return VIT_OK;
}

// The encode path behind the entry points.
struct EncodeMode {
  bool static_scratch = false;  // the workspace is the calling device's static array (wording of the capacity error)
  bool device_tables = false;   // the attention work lists are written by a kernel from the tile offsets (at most
                                // kStaticMaxImages images); nothing is allocated and nothing but kernels is queued:
                                // no pinned staging, no copy, no events (per-kernel timing is off for such a call)
  bool host_only = false;       // validate, fill request_token_offsets, report the image count; launch nothing
};
static vit_status_t encode_impl(const char* fn, vit_encoder_t* e, const float* pixels, const int32_t* images_per_request,
                                int32_t n_requests, const int32_t* tile_offsets, void* out_tokens,
                                size_t out_capacity_bytes, int64_t* request_token_offsets, void* workspace,
                                size_t workspace_bytes, void* stream, const EncodeMode mode,
                                int64_t* n_images_out = nullptr) {
  const bool static_scratch = mode.static_scratch;
  if (!e) return fail(VIT_EINVAL, "%s: NULL encoder", fn);
  if (n_requests < 0) return fail(VIT_EINVAL, "%s: n_requests < 0", fn);
  if (n_requests > 0 && !images_per_request) return fail(VIT_EINVAL, "%s: images_per_request is NULL", fn);
  if (!tile_offsets) return fail(VIT_EINVAL, "%s: tile_offsets is NULL", fn);
  const Dims& d = e->d;
  int64_t n_images = 0;
  for (int r = 0; r < n_requests; ++r) {
    if (images_per_request[r] < 0) return fail(VIT_EINVAL, "%s: images_per_request[%d] < 0", fn, r);
    n_images += images_per_request[r];
  }
  if (n_images > INT32_MAX) return fail(VIT_EINVAL, "%s: too many images", fn);
  if (tile_offsets[0] != 0) return fail(VIT_EINVAL, "%s: tile_offsets[0] must be 0", fn);
  for (int64_t i = 0; i < n_images; ++i)
    if (tile_offsets[i + 1] <= tile_offsets[i])
      return fail(VIT_EINVAL, "%s: image %lld has no tiles (tile_offsets must increase)", fn, (long long)i);
  const int64_t n_tiles = tile_offsets[n_images];
  if (n_images_out) *n_images_out = n_images;
  if (n_tiles * d.T > (int64_t)INT32_MAX - 1024) return fail(VIT_EINVAL, "%s: more than 2^31 token rows", fn);
  if (request_token_offsets) {
    int64_t img = 0;
    request_token_offsets[0] = 0;
    for (int r = 0; r < n_requests; ++r) {
      img += images_per_request[r];
      request_token_offsets[r + 1] = (int64_t)tile_offsets[img] * d.T_out;
    }
  }
  if (n_tiles == 0) return VIT_OK;
  if (!pixels || !out_tokens || !workspace) return fail(VIT_EINVAL, "%s: NULL device buffer", fn);
  if (((uintptr_t)workspace & 255) || ((uintptr_t)out_tokens & 15) || ((uintptr_t)pixels & 15))
    return fail(VIT_EINVAL, "%s: workspace must be 256-byte aligned, pixels and out_tokens 16-byte aligned", fn);

  Workspace w;
  plan_workspace(d, n_tiles, &w);
  const size_t out_need = (size_t)w.n_out * d.out_dim * d.es;
  if (out_capacity_bytes < out_need)
    return fail(VIT_ECAPACITY, "%s: out_tokens holds %zu bytes, %zu needed", fn, out_capacity_bytes, out_need);
  if (workspace_bytes < w.total)
    return fail(VIT_ECAPACITY, static_scratch ? "%s: the static scratch array holds %zu bytes, this batch needs %zu"
                                              : "%s: workspace holds %zu bytes, %zu needed",
                fn, workspace_bytes, w.total);
  if (mode.device_tables && n_images > kStaticMaxImages)
    return fail(VIT_ECAPACITY, "%s: %lld images, at most %d per call", fn, (long long)n_images, kStaticMaxImages);
  if (mode.host_only) return VIT_OK;

  HIP_TRY(hipSetDevice(e->device));
  hipStream_t s = (hipStream_t)stream;
  unsigned char* ws = (unsigned char*)workspace;
  float* x = (float*)(ws + w.off_x);
  void* h = ws + w.off_h;
  void* qkv = ws + w.off_qkv;
  void* o = ws + w.off_o;
  void* u = ws + w.off_u;
  AttnWork* tables = (AttnWork*)(ws + w.off_tables);
  const int n_tok = (int)w.n_tok;

  // ---- segment planning: blocks of query rows per tile (local layers) and per image (global layers)
  const int bq = attention_q_block(d.bf16, d.dhp);
  const bool has_global = d.L > d.L_loc;
  const bool timing = !mode.device_tables;  // events are created on demand: not in a call that may not allocate
  int n_local = 0, n_global = 0;
  if (mode.device_tables) {
    // the lists' lengths on the host (launch sizes), their contents by a kernel from the offsets themselves
    n_local = (int)(n_tiles * ((d.T + bq - 1) / bq));
    TileOffsetsArg to;
    memset(&to, 0, sizeof(to));
    for (int64_t i = 0; i <= n_images; ++i) to.v[i] = tile_offsets[i];
    if (has_global)
      for (int64_t i = 0; i < n_images; ++i) n_global += ((tile_offsets[i + 1] - tile_offsets[i]) * d.T + bq - 1) / bq;
    hipLaunchKernelGGL(attn_work_kernel, dim3(1), dim3(256), 0, s, to, (int)n_images, d.T, bq, tables,
                       has_global ? tables + w.max_work : (AttnWork*)nullptr);
    HIP_TRY(hipGetLastError());
  } else {
    StageSlot& slot = e->stage[e->next_stage];
    e->next_stage = (e->next_stage + 1) % 4;
    if (slot.used) HIP_TRY(hipEventSynchronize(slot.done));
    if (slot.cap < w.table_bytes) {
      if (slot.host) HIP_TRY(hipHostFree(slot.host));
      slot.host = nullptr;
      slot.cap = 0;
      HIP_TRY(hipHostMalloc(&slot.host, w.table_bytes, hipHostMallocDefault));
      slot.cap = w.table_bytes;
    }
    if (!slot.done) HIP_TRY(hipEventCreateWithFlags(&slot.done, hipEventDisableTiming));
    AttnWork* loc = (AttnWork*)slot.host;
    for (int64_t t = 0; t < n_tiles; ++t)
      for (int q = 0; q < d.T; q += bq) loc[n_local++] = {(int32_t)(t * d.T + q), (int32_t)(t * d.T), d.T};
    AttnWork* glob = loc + w.max_work;
    if (has_global)
      for (int64_t i = 0; i < n_images; ++i) {
        const int start = tile_offsets[i] * d.T, len = (tile_offsets[i + 1] - tile_offsets[i]) * d.T;
        for (int q = 0; q < len; q += bq) glob[n_global++] = {start + q, start, len};
      }
    HIP_TRY(hipMemcpyAsync(tables, slot.host, w.table_bytes, hipMemcpyHostToDevice, s));
    HIP_TRY(hipEventRecord(slot.done, s));
    slot.used = true;
  }

  // Streams larger than the 256 MB memory-side cache get non-temporal hints: they cannot be found there by
  // the next kernel anyway and would only displace operands; smaller ones are left to the caches.
  constexpr size_t kCacheBytes = (size_t)256 << 20;
  // Every kernel of the chain walks the token rows in the direction opposite to its producer:
  // what a kernel wrote last is still in the 256 MB memory-side cache when its consumer starts there.
  int reverse = 0;
  auto gemm = [&](int family, const Linear& lin, const void* A, int lda, int M, int epi, void* out, int ldo,
                  float* resid) -> hipError_t {
    GemmArgs a;
    memset(&a, 0, sizeof(a));
    a.A = A; a.W = lin.W; a.bias = lin.bias; a.out = out; a.resid = resid; a.pos = e->pos;
    a.M = M; a.N = lin.N; a.K = lin.K; a.lda = lda; a.ldw = lin.K; a.ldo = ldo;
    a.patches = d.P; a.tokens = d.T; a.cls = d.has_cls; a.epilogue = epi;
    a.reverse = reverse;
    reverse ^= 1;
    a.stream_out = (size_t)M * lin.N * d.es > kCacheBytes;
    if (family == VIT_PROF_GEMM_QKV && d.bf16) {
      // the bf16 attention kernel takes its queries in units of log2: exp2(q . k) is the softmax weight
      a.q_cols = d.H * d.dhp;
      a.q_scale = 1.4426950408889634f / sqrtf((float)d.dh);
      // and, for head dims whose rows are whole 128-byte lines, reads every head's rows back to back: the product's
      // 3 * H column blocks are stored one after the other, so a K or V tile is one contiguous block and not 64
      // pieces a whole row of the product apart (an odd number of lines between the rows instead, which spreads
      // them over the sets of a compute unit's L1 just as well, was measured to give nothing: it is the contiguity)
      if (d.dhp % 64 == 0) {
        a.epilogue = EPI_BIAS_HEADS;
        a.hm_dh = d.dhp;
        a.hm_rows = w.Mpad;
      }
    }
    a.tile_stamps = e->tile_stamps && timing ? e->tile_stamps + (size_t)family * kStampWordsPerFamily : nullptr;
    ProfScope ps(e, s, family, timing);
    return d.bf16 ? launch_gemm_bf16(a, s) : launch_gemm_f32(a, s);
  };
  auto layernorm = [&](const float* g_, const float* b_, int normalize, void* out, int ldo, int out_cols) -> hipError_t {
    ProfScope ps(e, s, VIT_PROF_LAYERNORM, timing);
    const int rev = reverse;
    reverse ^= 1;
    return launch_layernorm(x, d.D, out, ldo, out_cols, g_, b_, d.eps, n_tok, d.D, normalize, d.bf16, rev,
                            (size_t)n_tok * d.D * 4 > kCacheBytes, s);
  };

  // ---- patch embedding: gather -> matrix product with (+bias, +pos, row remap) epilogue; CLS rows
  {
    ProfScope ps(e, s, VIT_PROF_PATCHIFY, timing);
    HIP_TRY(launch_patch_gather(pixels, u, d.Kp_pad, (int)n_tiles, d.C, d.S, d.p, d.g, d.Kp_pad, d.bf16, s));
    if (d.has_cls) HIP_TRY(launch_cls_rows(x, d.D, e->cls, e->pos, (int)n_tiles, d.T, d.D, s));
  }
  HIP_TRY(gemm(VIT_PROF_GEMM_PATCH, e->patch, u, d.Kp_pad, (int)(n_tiles * d.P), EPI_PATCH, nullptr, d.D, x));
  if (d.Op > d.H * d.dhp) HIP_TRY(launch_fill_zero_cols(o, d.Op, n_tok, d.H * d.dhp, d.Op, d.es, s));

  // ---- transformer blocks
  for (int l = 0; l < d.L; ++l) {
    const Layer& L = e->layers[l];
    HIP_TRY(layernorm(L.ln1_g, L.ln1_b, 1, h, d.Dp, d.Dp));
    HIP_TRY(gemm(VIT_PROF_GEMM_QKV, L.qkv, h, d.Dp, n_tok, EPI_BIAS, qkv, d.QKVN, nullptr));
    {
      const bool global = l >= d.L_loc;
      AttnArgs a;
      a.qkv = qkv; a.out = o; a.qkv_rows = d.bf16 && d.dhp % 64 == 0 ? (size_t)w.Mpad : 0;
      a.work = global ? tables + w.max_work : tables;
      a.n_work = global ? n_global : n_local;
      a.heads = d.H; a.dh = d.dh; a.dh_pad = d.dhp; a.ld_qkv = d.QKVN; a.ld_o = d.Op;
      a.reverse = reverse;
      reverse ^= 1;
      ProfScope ps(e, s, VIT_PROF_ATTENTION, timing);
      HIP_TRY(d.bf16 ? launch_attention_bf16(a, s) : launch_attention_f32(a, s));
    }
    HIP_TRY(gemm(VIT_PROF_GEMM_OUT, L.wo, o, d.Op, n_tok, EPI_BIAS_RESIDUAL, nullptr, d.D, x));
    HIP_TRY(layernorm(L.ln2_g, L.ln2_b, 1, h, d.Dp, d.Dp));
    HIP_TRY(gemm(VIT_PROF_GEMM_FC1, L.w1, h, d.Dp, n_tok, EPI_BIAS_GELU, u, d.Mp, nullptr));
    HIP_TRY(gemm(VIT_PROF_GEMM_FC2, L.w2, u, d.Mp, n_tok, EPI_BIAS_RESIDUAL, nullptr, d.D, x));
  }

  // ---- final LayerNorm, token down-sampling and projector
  if (d.merge == 1) {
    if (d.proj_layers == 0) {
      HIP_TRY(layernorm(e->lnf_g, e->lnf_b, d.final_ln, out_tokens, d.D, d.D));
    } else {
      HIP_TRY(layernorm(e->lnf_g, e->lnf_b, d.final_ln, h, d.Dp, d.Dp));
    }
  } else {
    // normalised rows -> h, then m x m neighbours side by side: straight into the output, or into the
    // projector's operand buffer
    HIP_TRY(layernorm(e->lnf_g, e->lnf_b, d.final_ln, h, d.Dp, d.Dp));
    void* dst = d.proj_layers == 0 ? out_tokens : (void*)(ws + w.off_merge);
    const int dst_ld = d.proj_layers == 0 ? d.pin : d.pin_ld;
    ProfScope ps(e, s, VIT_PROF_PATCHIFY, timing);
    HIP_TRY(launch_token_merge(h, d.Dp, dst, dst_ld, (int)n_tiles, d.T, d.has_cls, d.g, d.merge, d.D, d.es, s));
  }
  if (d.proj_layers > 0) {
    const void* pin = d.merge == 1 ? h : (const void*)(ws + w.off_merge);
    const int n_out = (int)w.n_out;
    if (d.proj_layers == 1) {
      HIP_TRY(gemm(VIT_PROF_GEMM_PROJ, e->proj[0], pin, d.pin_ld, n_out, EPI_BIAS, out_tokens, d.out_dim, nullptr));
    } else {
      HIP_TRY(gemm(VIT_PROF_GEMM_PROJ, e->proj[0], pin, d.pin_ld, n_out, EPI_BIAS_GELU, u, d.proj0_ld, nullptr));
      HIP_TRY(gemm(VIT_PROF_GEMM_PROJ, e->proj[1], u, d.proj0_ld, n_out, EPI_BIAS, out_tokens, d.out_dim, nullptr));
    }
  }
  return VIT_OK;
}

vit_status_t vit_encode_packed(vit_encoder_t* e, const float* pixels, const int32_t* images_per_request,
                               int32_t n_requests, const int32_t* tile_offsets, void* out_tokens,
                               size_t out_capacity_bytes, int64_t* request_token_offsets, void* workspace,
                               size_t workspace_bytes, void* stream) {
  return encode_impl("vit_encode_packed", e, pixels, images_per_request, n_requests, tile_offsets, out_tokens,
                     out_capacity_bytes, request_token_offsets, workspace, workspace_bytes, stream, EncodeMode{});
}

vit_status_t vit_encode_packed_static(vit_encoder_t* e, const float* pixels, const int32_t* images_per_request,
                                      int32_t n_requests, const int32_t* tile_offsets, void* out_tokens,
                                      size_t out_capacity_bytes, int64_t* request_token_offsets, void* stream) {
  if (!e) return fail(VIT_EINVAL, "vit_encode_packed_static: NULL encoder");
  if (!e->scratch)
    return fail(VIT_EDEVICE, "vit_encode_packed_static: the static scratch array has no address on device %d: %s",
                e->device, hipGetErrorString(e->scratch_error));
  EncodeMode mode;
  mode.static_scratch = mode.device_tables = true;
  return encode_impl("vit_encode_packed_static", e, pixels, images_per_request, n_requests, tile_offsets, out_tokens,
                     out_capacity_bytes, request_token_offsets, e->scratch, kStaticScratchBytes, stream, mode);
}

vit_status_t vit_encode_packed_graph(vit_encoder_t* e, const float* pixels, const int32_t* images_per_request,
                                     int32_t n_requests, const int32_t* tile_offsets, void* out_tokens,
                                     size_t out_capacity_bytes, int64_t* request_token_offsets, void* workspace,
                                     size_t workspace_bytes, void* stream) {
  const char* fn = "vit_encode_packed_graph";
  // every check of the plain call, the host-side result and the image count; nothing launched yet
  EncodeMode check;
  check.host_only = true;
  int64_t n_images = 0;
  if (vit_status_t st = encode_impl(fn, e, pixels, images_per_request, n_requests, tile_offsets, out_tokens,
                                    out_capacity_bytes, request_token_offsets, workspace, workspace_bytes, stream, check,
                                    &n_images);
      st != VIT_OK)
    return st;
  if (tile_offsets[n_images] == 0) return VIT_OK;
  auto eager = [&](bool device_tables) {
    EncodeMode m;
    m.device_tables = device_tables;
    return encode_impl(fn, e, pixels, images_per_request, n_requests, tile_offsets, out_tokens, out_capacity_bytes,
                       request_token_offsets, workspace, workspace_bytes, stream, m);
  };
  // a graph holds nothing but kernels: batches whose work lists cannot be built on the device run as they are
  if (n_images > kStaticMaxImages) return eager(false);

  GraphEntry* hit = nullptr;
  for (auto& g : e->graphs)
    if (g.pixels == pixels && g.out == out_tokens && g.workspace == workspace &&
        g.tile_offsets.size() == (size_t)n_images + 1 &&
        std::equal(g.tile_offsets.begin(), g.tile_offsets.end(), tile_offsets)) {
      hit = &g;
      break;
    }
  if (!hit) {
    // first sight of these buffers and this shape: run it as it is (which also leaves every kernel's launch
    // attributes set) and remember the key; the least recently used entry makes room
    try {
      if (e->graphs.size() < kMaxGraphs) {
        e->graphs.emplace_back();
        hit = &e->graphs.back();
      } else {
        hit = &*std::min_element(e->graphs.begin(), e->graphs.end(),
                                 [](const GraphEntry& a, const GraphEntry& b) { return a.used < b.used; });
        if (hit->exec) (void)hipGraphExecDestroy(hit->exec);
        hit->exec = nullptr;
      }
      hit->tile_offsets.assign(tile_offsets, tile_offsets + n_images + 1);
    } catch (...) {
      if (hit) hit->tile_offsets.clear(), hit->pixels = nullptr;
      return eager(true);  // no memory for the key: the call itself does not need it
    }
    hit->pixels = pixels; hit->out = out_tokens; hit->workspace = workspace;
    hit->used = ++e->graph_tick;
    return eager(true);
  }
  hit->used = ++e->graph_tick;
  HIP_TRY(hipSetDevice(e->device));
  if (!hit->exec) {
    // second sight: record the launch sequence on a stream of the library's own (the caller's may be the legacy
    // default stream, which cannot be captured) and keep the executable graph
    if (!e->capture_stream) HIP_TRY(hipStreamCreateWithFlags(&e->capture_stream, hipStreamNonBlocking));
    HIP_TRY(hipStreamBeginCapture(e->capture_stream, hipStreamCaptureModeThreadLocal));
    EncodeMode m;
    m.device_tables = true;
    const vit_status_t st = encode_impl(fn, e, pixels, images_per_request, n_requests, tile_offsets, out_tokens,
                                        out_capacity_bytes, request_token_offsets, workspace, workspace_bytes,
                                        e->capture_stream, m);
    hipGraph_t graph = nullptr;
    const hipError_t end = hipStreamEndCapture(e->capture_stream, &graph);
    hipGraphExec_t exec = nullptr;
    hipError_t inst = hipErrorUnknown;
    if (st == VIT_OK && end == hipSuccess && graph) inst = hipGraphInstantiate(&exec, graph, nullptr, nullptr, 0);
    if (graph) (void)hipGraphDestroy(graph);
    if (inst != hipSuccess) {  // nothing ran during the capture: run the call as it is
      (void)hipGetLastError();
      return eager(true);
    }
    hit->exec = exec;
  }
  HIP_TRY(hipGraphLaunch(hit->exec, (hipStream_t)stream));
  return VIT_OK;
}

vit_status_t vit_profile_enable(vit_encoder_t* e, int enable) {
  if (!e) return fail(VIT_EINVAL, "vit_profile_enable: NULL encoder");
  HIP_TRY(hipSetDevice(e->device));
  try {
    e->free_events.reserve(e->free_events.size() + 2 * e->prof.size());
  } catch (...) {
    return fail(VIT_ENOMEM, "vit_profile_enable: out of host memory");
  }
  for (auto& r : e->prof) {
    HIP_TRY(hipEventSynchronize(r.stop));
    e->free_events.push_back(r.start);
    e->free_events.push_back(r.stop);
  }
  e->prof.clear();
  for (int i = 0; i < VIT_PROF_COUNT; ++i) { e->prof_ms[i] = 0; e->prof_n[i] = 0; }
  e->profiling = enable != 0;
  return VIT_OK;
}

vit_status_t vit_profile_read(vit_encoder_t* e, double* ms, int64_t* launches) {
  if (!e || !ms || !launches) return fail(VIT_EINVAL, "vit_profile_read: NULL argument");
  HIP_TRY(hipSetDevice(e->device));
  try {
    e->free_events.reserve(e->free_events.size() + 2 * e->prof.size());
  } catch (...) {
    return fail(VIT_ENOMEM, "vit_profile_read: out of host memory");
  }
  for (auto& r : e->prof) {
    HIP_TRY(hipEventSynchronize(r.stop));
    float t = 0.f;
    HIP_TRY(hipEventElapsedTime(&t, r.start, r.stop));
    e->prof_ms[r.family] += t;
    e->prof_n[r.family] += 1;
    e->free_events.push_back(r.start);
    e->free_events.push_back(r.stop);
  }
  e->prof.clear();
  for (int i = 0; i < VIT_PROF_COUNT; ++i) { ms[i] = e->prof_ms[i]; launches[i] = e->prof_n[i]; }
  return VIT_OK;
}

vit_status_t vit_profile_tiles_enable(vit_encoder_t* e, int enable) {
  if (!e) return fail(VIT_EINVAL, "vit_profile_tiles_enable: NULL encoder");
  HIP_TRY(hipSetDevice(e->device));
  HIP_TRY(hipDeviceSynchronize());  // no kernel may still be writing stamps
  const size_t bytes = (size_t)VIT_PROF_COUNT * kStampWordsPerFamily * sizeof(unsigned long long);
  if (enable) {
    if (!e->tile_stamps) HIP_TRY(hipHostMalloc((void**)&e->tile_stamps, bytes, hipHostMallocDefault));
    memset(e->tile_stamps, 0, bytes);
  } else if (e->tile_stamps) {
    HIP_TRY(hipHostFree(e->tile_stamps));
    e->tile_stamps = nullptr;
  }
  return VIT_OK;
}

vit_status_t vit_profile_tiles_read(vit_encoder_t* e, double* main_loop_us, double* epilogue_us, double* clock_mhz,
                                    int64_t* tiles) {
  if (!e || !main_loop_us || !epilogue_us || !clock_mhz || !tiles)
    return fail(VIT_EINVAL, "vit_profile_tiles_read: NULL argument");
  if (!e->tile_stamps) return fail(VIT_EINVAL, "vit_profile_tiles_read: not enabled");
  HIP_TRY(hipSetDevice(e->device));
  HIP_TRY(hipDeviceSynchronize());
  int rate_khz = 0;  // of the constant-rate clock the kernel reads
  HIP_TRY(hipDeviceGetAttribute(&rate_khz, hipDeviceAttributeWallClockRate, e->device));
  if (rate_khz <= 0) return fail(VIT_EDEVICE, "vit_profile_tiles_read: the device reports no wall-clock rate");
  const double us_per_tick = 1e3 / (double)rate_khz;
  for (int f = 0; f < VIT_PROF_COUNT; ++f) {
    const unsigned long long* D = e->tile_stamps + (size_t)f * kStampWordsPerFamily;
    double main_t = 0, epi_t = 0, cycles = 0;
    int64_t n = 0;
    for (size_t r = 0; r < (size_t)256 * kTileStampSlots; ++r) {
      const unsigned long long* d = D + r * 4;
      if (!d[3]) continue;
      main_t += (double)(d[1] - d[0]);
      epi_t += (double)(d[2] - d[1]);
      cycles += (double)(d[3] - 1);
      ++n;
    }
    tiles[f] = n;
    main_loop_us[f] = n ? main_t / n * us_per_tick : 0.0;
    epilogue_us[f] = n ? epi_t / n * us_per_tick : 0.0;
    clock_mhz[f] = main_t + epi_t > 0 ? cycles / ((main_t + epi_t) * us_per_tick) : 0.0;
  }
  return VIT_OK;
}

vit_status_t vit_mfma_ceiling(int device, double seconds, int32_t random_operands, double* tflops) {
  if (!tflops || !(seconds > 0.0) || seconds > 2.0) return fail(VIT_EINVAL, "vit_mfma_ceiling: bad argument");
  HIP_TRY(hipSetDevice(device));
  int n_cu = 0;
  HIP_TRY(hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, device));
  // 4096 fragments of 8 bf16: seeded uniform [-1, 1) (xorshift32) or the constant 1/128
  std::vector<uint16_t> host(4096 * 8);
  uint32_t rs = 0x9E3779B9u;
  for (auto& v : host) {
    rs ^= rs << 13; rs ^= rs >> 17; rs ^= rs << 5;
    v = random_operands ? f32_to_bf16((float)(rs >> 8) * (2.0f / 16777216.0f) - 1.0f) : (uint16_t)0x3C00;
  }
  unsigned char* dev = nullptr;
  HIP_TRY(hipMalloc((void**)&dev, host.size() * 2 + 1024));
  hipError_t err = hipMemcpy(dev, host.data(), host.size() * 2, hipMemcpyHostToDevice);
  float* out = (float*)(dev + host.size() * 2);
  hipEvent_t e0 = nullptr, e1 = nullptr;
  if (err == hipSuccess) err = hipEventCreate(&e0);
  if (err == hipSuccess) err = hipEventCreate(&e1);
  const int grid = 2 * n_cu;  // 4 waves per workgroup, 2 workgroups per unit: two waves per SIMD
  const double flop_per_iter = (double)grid * 4 * 8 * 2.0 * 32 * 32 * 16;
  double best = 0.0;
  int iters = 20000;  // about 5 ms; the second launch is sized from the first to last `seconds`
  for (int rep = 0; rep < 2 && err == hipSuccess; ++rep) {
    err = hipEventRecord(e0, 0);
    if (err != hipSuccess) break;
    hipLaunchKernelGGL(mfma_ceiling_kernel, dim3(grid), dim3(256), 0, 0, (const u32x4*)dev, out, iters);
    err = hipGetLastError();
    if (err == hipSuccess) err = hipEventRecord(e1, 0);
    if (err == hipSuccess) err = hipEventSynchronize(e1);
    float ms = 0.f;
    if (err == hipSuccess) err = hipEventElapsedTime(&ms, e0, e1);
    if (err != hipSuccess || ms <= 0.f) break;
    best = flop_per_iter * iters / (ms * 1e-3) / 1e12;
    const double want = (double)iters * (seconds * 1e3 / ms);
    iters = (int)(want < 1000.0 ? 1000.0 : want > 4.0e6 ? 4.0e6 : want);
  }
  if (e0) (void)hipEventDestroy(e0);
  if (e1) (void)hipEventDestroy(e1);
  (void)hipFree(dev);
  if (err != hipSuccess) return fail(VIT_EDEVICE, "vit_mfma_ceiling: %s", hipGetErrorString(err));
  *tflops = best;
  return VIT_OK;
}

}  // extern "C"
