// Host side of the C ABI: argument validation and launch set-up.  Nothing here touches device memory.
#include <hip/hip_runtime.h>

#include <mutex>

#include "kvlinc_internal.h"

namespace {

// Scratch of kvlinc_decode_attention_noalloc: part of the device image, one copy per GPU.  The name below is a host-side
// stand-in, not a device address: host code only ever uses the address hipGetSymbolAddress returns for the current
// device, looked up once per device.
static __device__ __align__(256) unsigned char scratch[KVLINC_STATIC_SCRATCH_BYTES];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mutex;

int scratch_of_current_device(void** ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return KVLINC_EHIP;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return KVLINC_EHIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return KVLINC_OK;
}

inline bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }
inline bool bad_ptr(const void* p, uintptr_t a) { return p == nullptr || !aligned(p, a); }

}  // namespace

extern "C" {

int kvlinc_version(void) { return 100; }

const char* kvlinc_strerror(int code) {
  switch (code) {
    case KVLINC_OK: return "ok";
    case KVLINC_EINVAL: return "invalid argument (NULL or misaligned pointer, unsupported shape or parameter)";
    case KVLINC_EWORKSPACE: return "workspace too small or misaligned";
    case KVLINC_EHIP: return "HIP call failed";
    case KVLINC_ESCRATCH: return "the launch needs more scratch than the library's static buffer holds";
    default: return "unknown kvlinc error code";
  }
}

int kvlinc_cache_validate(const kvlinc_cache* c) {
  if (c == nullptr) return KVLINC_EINVAL;
  if (c->B < 1 || c->H_q < 1 || c->H_kv < 1) return KVLINC_EINVAL;
  if (c->d != kvlinc::kHeadDim || c->G != kvlinc::kGroup || c->D != kvlinc::kRank || (c->bits != 2 && c->bits != 4)) return KVLINC_EINVAL;
  if (c->R < 4 || c->R > kvlinc::kGroup || c->R % 4 != 0) return KVLINC_EINVAL;
  if (c->H_q % c->H_kv != 0 || c->H_q / c->H_kv > kvlinc::kMaxGq) return KVLINC_EINVAL;
  if (c->max_groups < 1 || c->max_groups > (1ll << 24)) return KVLINC_EINVAL;
  if ((long long)c->B * c->H_kv > (1ll << 24)) return KVLINC_EINVAL;
  if (bad_ptr(c->groups, 16)) return KVLINC_EINVAL;
  if (bad_ptr(c->k_res, 16) || bad_ptr(c->v_res, 16)) return KVLINC_EINVAL;
  if (bad_ptr(c->n_quant, 4) || bad_ptr(c->n_res, 4) || bad_ptr(c->status, 4) || bad_ptr(c->split_done, 4))
    return KVLINC_EINVAL;
  const int n_corr = (c->S16 != nullptr) + (c->P != nullptr) + (c->Wq != nullptr) + (c->Wk != nullptr);
  if (n_corr != 0 && n_corr != 4) return KVLINC_EINVAL;
  if (n_corr == 0 && c->S != nullptr) return KVLINC_EINVAL;  // the fp32 master copy is an option of the correction
  if (n_corr == 4 && (!aligned(c->S, 16) || !aligned(c->S16, 16) || !aligned(c->P, 16) || !aligned(c->Wq, 16) ||
                      !aligned(c->Wk, 16)))
    return KVLINC_EINVAL;
  if ((c->flags & ~(KVLINC_FLAG_ALG1_LITERAL | KVLINC_FLAG_SLIDING_VALUES)) != 0) return KVLINC_EINVAL;
  if ((c->flags & KVLINC_FLAG_SLIDING_VALUES) != 0 && c->R != kvlinc::kGroup) return KVLINC_EINVAL;
  return KVLINC_OK;
}

int kvlinc_append_quantize(const kvlinc_cache* cache, const kvlinc_half* k_new, const kvlinc_half* v_new,
                           const int32_t* n_new, int32_t T, int32_t keep_residual, void* stream) {
  const int rc = kvlinc_cache_validate(cache);
  if (rc != KVLINC_OK) return rc;
  if (bad_ptr(k_new, 16) || bad_ptr(v_new, 16)) return KVLINC_EINVAL;
  if (n_new != nullptr && !aligned(n_new, 4)) return KVLINC_EINVAL;
  if (T < 1 || T > (1 << 24)) return KVLINC_EINVAL;
  if (keep_residual < 0 || keep_residual > cache->R) return KVLINC_EINVAL;
  if (keep_residual == 0 && cache->R != kvlinc::kGroup) return KVLINC_EINVAL;
  if (keep_residual != 0 && (cache->flags & KVLINC_FLAG_SLIDING_VALUES) != 0) return KVLINC_EINVAL;
  return kvlinc::launch_append(*cache, k_new, v_new, n_new, T, keep_residual, static_cast<hipStream_t>(stream));
}

size_t kvlinc_decode_workspace_bytes(const kvlinc_cache* cache, int32_t max_context) {
  if (kvlinc_cache_validate(cache) != KVLINC_OK) return 0;
  return kvlinc::decode_workspace_floats(*cache, kvlinc::decode_splits(*cache, max_context).most) * sizeof(float);
}

static int decode_checked(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, void* workspace,
                          size_t workspace_bytes, int32_t max_context, void* stream, void* start, void* stop) {
  const int rc = kvlinc_cache_validate(cache);
  if (rc != KVLINC_OK) return rc;
  if (bad_ptr(q, 16) || bad_ptr(out, 16)) return KVLINC_EINVAL;
  if ((start == nullptr) != (stop == nullptr)) return KVLINC_EINVAL;
  if (bad_ptr(workspace, 16) || workspace_bytes < kvlinc_decode_workspace_bytes(cache, max_context))
    return KVLINC_EWORKSPACE;
  return kvlinc::launch_decode(*cache, q, out, static_cast<float*>(workspace), kvlinc::decode_splits(*cache, max_context),
                               static_cast<hipStream_t>(stream), static_cast<hipEvent_t>(start),
                               static_cast<hipEvent_t>(stop));
}

int kvlinc_decode_attention(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, void* workspace,
                            size_t workspace_bytes, int32_t max_context, void* stream) {
  return decode_checked(cache, q, out, workspace, workspace_bytes, max_context, stream, nullptr, nullptr);
}

int kvlinc_decode_attention_timed(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out, void* workspace,
                                  size_t workspace_bytes, int32_t max_context, void* stream, void* start_event,
                                  void* stop_event) {
  if (start_event == nullptr || stop_event == nullptr) return KVLINC_EINVAL;
  return decode_checked(cache, q, out, workspace, workspace_bytes, max_context, stream, start_event, stop_event);
}

int kvlinc_decode_attention_noalloc(const kvlinc_cache* cache, const kvlinc_half* q, kvlinc_half* out,
                                    int32_t max_context, void* stream) {
  const int rc = kvlinc_cache_validate(cache);
  if (rc != KVLINC_OK) return rc;
  if (bad_ptr(q, 16) || bad_ptr(out, 16)) return KVLINC_EINVAL;
  const size_t need = kvlinc_decode_workspace_bytes(cache, max_context);
  if (need > (size_t)KVLINC_STATIC_SCRATCH_BYTES) return KVLINC_ESCRATCH;
  void* ws = nullptr;
  const int rs = scratch_of_current_device(&ws);
  if (rs != KVLINC_OK) return rs;
  return kvlinc::launch_decode(*cache, q, out, static_cast<float*>(ws), kvlinc::decode_splits(*cache, max_context),
                               static_cast<hipStream_t>(stream), nullptr, nullptr);
}

}  // extern "C"
