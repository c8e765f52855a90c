// C-ABI entry points of libkvra: argument checks, then the kernel launchers.
#include "kvra_internal.h"

namespace {

// Largest element count the kernels index with 32-bit arithmetic inside one tensor row block.
constexpr int64_t kMaxTokens = int64_t(1) << 24;   // 16M tokens per call
constexpr int kMaxHeads = 1024;

int check_heads(int n_q_heads, int n_kv_heads, int head_dim) {
  if (n_q_heads < 1 || n_kv_heads < 1) return KVRA_EINVAL;
  if (n_q_heads % n_kv_heads != 0) return KVRA_EINVAL;
  if (head_dim != 64 && head_dim != 128) return KVRA_EUNSUPPORTED;
  if (n_q_heads > kMaxHeads) return KVRA_EUNSUPPORTED;
  return KVRA_OK;
}

}  // namespace

extern "C" const char* kvra_strerror(int code) {
  switch (code) {
    case KVRA_OK: return "ok";
    case KVRA_EINVAL: return "invalid argument";
    case KVRA_EUNSUPPORTED: return "unsupported shape (head_dim must be 64 or 128)";
    case KVRA_ERANGE: return "prefix_len + chunk_len exceeds cache capacity";
    case KVRA_ELAUNCH: return "HIP launch or allocation failed";
    case KVRA_ENODEVICE: return "no usable gfx950 device";
    default: return "unknown error";
  }
}

extern "C" int kvra_version(void) { return 100; }

extern "C" int kvra_append_kv(const void* k_in, const void* v_in, void* q_inout,
                              void* k_cache, void* v_cache,
                              int64_t prefix_len, int64_t chunk_len, int64_t capacity,
                              int n_q_heads, int n_kv_heads, int head_dim,
                              float rope_base, void* stream) {
  if (k_in == nullptr || v_in == nullptr || k_cache == nullptr || v_cache == nullptr) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0 || capacity < 1) return KVRA_EINVAL;
  if (!(rope_base == rope_base)) return KVRA_EINVAL;  // NaN
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  if (prefix_len + chunk_len > capacity) return KVRA_ERANGE;
  return kvra::launch_append_kv(k_in, v_in, q_inout, k_cache, v_cache, prefix_len, chunk_len,
                                n_q_heads, n_kv_heads, head_dim, rope_base,
                                static_cast<hipStream_t>(stream));
}

extern "C" int kvra_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                               int64_t prefix_len, int64_t chunk_len,
                               int n_q_heads, int n_kv_heads, int head_dim,
                               float scale, void* out, void* stream) {
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0) return KVRA_EINVAL;
  if (!(scale > 0.0f) || !(scale < INFINITY)) return KVRA_EINVAL;
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  return kvra::launch_chunk_attn(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads,
                                 head_dim, scale, out, static_cast<hipStream_t>(stream));
}
