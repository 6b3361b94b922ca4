// Pull-style hand-off of finished image tokens (paper Sec. 4.3, "Image Token Transfer").
//
// A producer (an encoder launch) publishes where the tokens of one image of a request lie in device
// memory and records an event on its stream; nothing is copied then.  When every image of the
// request has been published the consumer, which by now knows where the request will run, pulls:
// the copies of all images, in image order, are queued on the consumer's stream behind the
// producers' events (many-to-one aggregation, transfer deferred until the request is complete).
// On one GPU the pull is a device-to-device copy; the same table would carry peer pointers.
// Host plumbing only: no arithmetic of the encoder happens here.
#include "../../include/vitenc.h"

#include <hip/hip_runtime.h>

#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

namespace vitenc {
vit_status_t set_error(vit_status_t st, const char* fmt, ...);  // vitenc_api.hip: message for vit_last_error()
}
using vitenc::set_error;

namespace {
struct Piece {
  const void* ptr = nullptr;
  size_t bytes = 0;
  hipEvent_t ready = nullptr;
  bool published = false;
};
struct Request {
  std::vector<Piece> pieces;
  int published = 0;
  size_t total = 0;
};
}  // namespace

struct vit_handoff {
  int device = 0;
  std::mutex mu;
  std::unordered_map<int64_t, Request> requests;
};

namespace {
void drop(Request& r) {
  for (auto& p : r.pieces)
    if (p.ready) (void)hipEventDestroy(p.ready);
}
}  // namespace

extern "C" {

vit_status_t vit_handoff_create(int device, vit_handoff_t** out) {
  if (!out || device < 0) return set_error(VIT_EINVAL, "vit_handoff_create: bad argument");
  vit_handoff_t* h = new (std::nothrow) vit_handoff_t;
  if (!h) return set_error(VIT_ENOMEM, "vit_handoff_create: out of host memory");
  h->device = device;
  *out = h;
  return VIT_OK;
}

void vit_handoff_destroy(vit_handoff_t* h) {
  if (!h) return;
  for (auto& kv : h->requests) drop(kv.second);
  delete h;
}

vit_status_t vit_handoff_expect(vit_handoff_t* h, int64_t request_id, int32_t n_images) {
  if (!h || n_images <= 0 || n_images > 65536)
    return set_error(VIT_EINVAL, "vit_handoff_expect: need a handle and 1 <= n_images <= 65536");
  std::lock_guard<std::mutex> lock(h->mu);
  if (h->requests.count(request_id)) return set_error(VIT_EINVAL, "vit_handoff_expect: request %lld is already known", (long long)request_id);
  try {
    h->requests[request_id].pieces.resize((size_t)n_images);
  } catch (...) {  // out of host memory: nothing of the request stays behind
    h->requests.erase(request_id);
    return set_error(VIT_ENOMEM, "vit_handoff_expect: out of host memory for %d images", n_images);
  }
  return VIT_OK;
}

vit_status_t vit_handoff_publish(vit_handoff_t* h, int64_t request_id, int32_t image_index, const void* tokens,
                                 size_t bytes, void* stream) {
  if (!h || !tokens || bytes == 0) return set_error(VIT_EINVAL, "vit_handoff_publish: bad argument");
  std::lock_guard<std::mutex> lock(h->mu);
  auto it = h->requests.find(request_id);
  if (it == h->requests.end()) return set_error(VIT_EINVAL, "vit_handoff_publish: unknown request %lld", (long long)request_id);
  Request& r = it->second;
  if (image_index < 0 || (size_t)image_index >= r.pieces.size())
    return set_error(VIT_EINVAL, "vit_handoff_publish: image %d outside the %zu images expected", image_index, r.pieces.size());
  Piece& p = r.pieces[(size_t)image_index];
  if (p.published) return set_error(VIT_EINVAL, "vit_handoff_publish: image %d was already published", image_index);
  hipError_t e = hipSetDevice(h->device);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&p.ready, hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventRecord(p.ready, (hipStream_t)stream);
  if (e != hipSuccess) {
    if (p.ready) (void)hipEventDestroy(p.ready);
    p.ready = nullptr;
    return set_error(VIT_EDEVICE, "vit_handoff_publish: %s", hipGetErrorString(e));
  }
  p.ptr = tokens;
  p.bytes = bytes;
  p.published = true;
  r.published += 1;
  r.total += bytes;
  return VIT_OK;
}

int32_t vit_handoff_complete(vit_handoff_t* h, int64_t request_id, size_t* total_bytes) {
  if (!h) return 0;
  std::lock_guard<std::mutex> lock(h->mu);
  auto it = h->requests.find(request_id);
  if (it == h->requests.end()) return 0;
  if (total_bytes) *total_bytes = it->second.total;
  return it->second.published == (int)it->second.pieces.size() ? 1 : 0;
}

vit_status_t vit_handoff_pull(vit_handoff_t* h, int64_t request_id, void* dst, size_t capacity, void* stream,
                              size_t* bytes) {
  if (!h || !dst) return set_error(VIT_EINVAL, "vit_handoff_pull: bad argument");
  std::lock_guard<std::mutex> lock(h->mu);
  auto it = h->requests.find(request_id);
  if (it == h->requests.end()) return set_error(VIT_EINVAL, "vit_handoff_pull: unknown request %lld", (long long)request_id);
  Request& r = it->second;
  if (r.published != (int)r.pieces.size())
    return set_error(VIT_ENOTREADY, "vit_handoff_pull: %d of %zu images published", r.published, r.pieces.size());
  if (r.total > capacity) return set_error(VIT_ECAPACITY, "vit_handoff_pull: %zu bytes needed, %zu given", r.total, capacity);
  hipError_t e = hipSetDevice(h->device);
  size_t off = 0;
  for (size_t i = 0; i < r.pieces.size() && e == hipSuccess; ++i) {
    const Piece& p = r.pieces[i];
    e = hipStreamWaitEvent((hipStream_t)stream, p.ready, 0);
    if (e == hipSuccess)
      e = hipMemcpyAsync((char*)dst + off, p.ptr, p.bytes, hipMemcpyDeviceToDevice, (hipStream_t)stream);
    off += p.bytes;
  }
  if (e != hipSuccess) return set_error(VIT_EDEVICE, "vit_handoff_pull: %s", hipGetErrorString(e));
  if (bytes) *bytes = r.total;
  return VIT_OK;
}

vit_status_t vit_handoff_release(vit_handoff_t* h, int64_t request_id) {
  if (!h) return set_error(VIT_EINVAL, "vit_handoff_release: NULL handle");
  std::lock_guard<std::mutex> lock(h->mu);
  auto it = h->requests.find(request_id);
  if (it == h->requests.end()) return set_error(VIT_EINVAL, "vit_handoff_release: unknown request %lld", (long long)request_id);
  drop(it->second);
  h->requests.erase(it);
  return VIT_OK;
}

}  // extern "C"
