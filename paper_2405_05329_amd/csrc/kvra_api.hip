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
    case KVRA_ESCRATCH: return "launch needs more scratch than the fixed buffer of kvra_chunk_attn_noalloc holds";
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

namespace {

int chunk_attn_checked(const void* q, const void* k_cache, const void* v_cache,
                       int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                       float scale, void* out, void* stream, bool static_scratch_only) {
  if (q == nullptr || k_cache == nullptr || v_cache == nullptr || out == nullptr) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0) return KVRA_EINVAL;
  if (!(scale > 0.0f) || !(scale < INFINITY)) return KVRA_EINVAL;
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  return kvra::launch_chunk_attn(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads,
                                 head_dim, scale, out, static_cast<hipStream_t>(stream), static_scratch_only);
}

}  // namespace

extern "C" int kvra_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                               int64_t prefix_len, int64_t chunk_len,
                               int n_q_heads, int n_kv_heads, int head_dim,
                               float scale, void* out, void* stream) {
  return chunk_attn_checked(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim,
                            scale, out, stream, false);
}

extern "C" int kvra_chunk_attn_noalloc(const void* q, const void* k_cache, const void* v_cache,
                                       int64_t prefix_len, int64_t chunk_len,
                                       int n_q_heads, int n_kv_heads, int head_dim,
                                       float scale, void* out, void* stream) {
  return chunk_attn_checked(q, k_cache, v_cache, prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim,
                            scale, out, stream, true);
}

extern "C" int64_t kvra_chunk_attn_noalloc_scratch_bytes(void) { return kvra::attn_static_scratch_bytes(); }

extern "C" int kvra_chunk_attn_plan(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads,
                                    int head_dim, int n_cus, kvra_attn_plan* plan) {
  if (plan == nullptr || n_cus < 1) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0) return KVRA_EINVAL;
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  kvra::AttnPlan p;
  rc = kvra::plan_chunk_attn(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus, true, &p);
  if (rc != KVRA_OK) return rc;
  plan->row_tiles = p.row_tiles;
  plan->rows_per_tile = p.rows_per_tile;
  plan->key_tile = p.key_tile;
  plan->groups = p.groups;
  plan->slots = p.slots;
  plan->units = p.units;
  plan->rounds = p.rounds;
  plan->head_steps = p.head_steps;
  plan->cut_units = p.cut;
  plan->segments = p.segments;
  plan->steps_per_slot = p.steps_per_slot;
  plan->partial_pieces = p.partial_pieces;
  plan->gangs = p.gangs;
  plan->gang_heads = p.gang_heads;
  plan->scratch_bytes = kvra::attn_partial_bytes(128) * p.scratch_slots;
  return KVRA_OK;
}

extern "C" int kvra_chunk_attn_pieces(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads,
                                      int head_dim, int n_cus, int32_t* records, int64_t capacity,
                                      int64_t* count_out) {
  if (n_cus < 1 || capacity < 0 || (records == nullptr && capacity > 0)) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0) return KVRA_EINVAL;
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  return kvra::list_chunk_attn_pieces(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, n_cus, records,
                                      capacity, count_out);
}

// ---------------------------------------------------------------- decoder layer around the attention
namespace {

constexpr int64_t kMaxOperandBytes = int64_t(1) << 32;   // per-lane byte offsets are 32-bit

int check_linear(int64_t m, int64_t n, int64_t k) {
  if (m < 1 || n < 1 || k < 1) return KVRA_EINVAL;
  if (n % 32 != 0 || k % 64 != 0) return KVRA_EUNSUPPORTED;
  if (m > kMaxTokens || n > (int64_t(1) << 24)) return KVRA_EUNSUPPORTED;
  if (m * k * 2 >= kMaxOperandBytes || n * k * 2 >= kMaxOperandBytes) return KVRA_EUNSUPPORTED;
  return KVRA_OK;
}

int64_t align256(int64_t b) { return (b + 255) / 256 * 256; }

}  // namespace

extern "C" int kvra_rms_norm(const void* x, const void* gain, void* y, int64_t rows, int hidden, float eps,
                             void* stream) {
  if (x == nullptr || gain == nullptr || y == nullptr || rows < 1 || hidden < 1) return KVRA_EINVAL;
  if (!(eps >= 0.0f) || !(eps < INFINITY)) return KVRA_EINVAL;
  if (hidden % 8 != 0 || hidden > kvra::rms_norm_max_hidden() || rows > kMaxTokens) return KVRA_EUNSUPPORTED;
  return kvra::launch_rms_norm(x, gain, y, rows, hidden, eps, static_cast<hipStream_t>(stream));
}

extern "C" int kvra_linear(const void* x, const void* w, const void* w2, const void* residual, void* out,
                           int64_t m, int64_t n, int64_t k, void* stream) {
  if (x == nullptr || w == nullptr || out == nullptr) return KVRA_EINVAL;
  if (w2 != nullptr && residual != nullptr) return KVRA_EINVAL;
  int rc = check_linear(m, n, k);
  if (rc != KVRA_OK) return rc;
  void* outs[1] = {out};
  const int cols[1] = {static_cast<int>(n)};
  return kvra::launch_linear(x, w, w2, residual, outs, cols, 1, m, n, k, static_cast<hipStream_t>(stream));
}

extern "C" int kvra_qkv_proj(const void* x, const void* wqkv, void* q_out, void* k_out, void* v_out,
                             int64_t m, int n_q_heads, int n_kv_heads, int head_dim, int64_t k, void* stream) {
  if (x == nullptr || wqkv == nullptr || q_out == nullptr || k_out == nullptr || v_out == nullptr) return KVRA_EINVAL;
  int rc = check_heads(n_q_heads, n_kv_heads, head_dim);
  if (rc != KVRA_OK) return rc;
  const int64_t n = static_cast<int64_t>(n_q_heads + 2 * n_kv_heads) * head_dim;
  rc = check_linear(m, n, k);
  if (rc != KVRA_OK) return rc;
  void* outs[3] = {q_out, k_out, v_out};
  const int cols[3] = {n_q_heads * head_dim, n_kv_heads * head_dim, n_kv_heads * head_dim};
  return kvra::launch_linear(x, wqkv, nullptr, nullptr, outs, cols, 3, m, n, k, static_cast<hipStream_t>(stream));
}

namespace {

int check_layer(const kvra_layer* L) {
  if (L == nullptr) return KVRA_EINVAL;
  if (L->norm1 == nullptr || L->wqkv == nullptr || L->wo == nullptr || L->norm2 == nullptr ||
      L->w_gate == nullptr || L->w_up == nullptr || L->w_down == nullptr)
    return KVRA_EINVAL;
  if (L->hidden < 1 || L->ffn < 1) return KVRA_EINVAL;
  int rc = check_heads(L->n_q_heads, L->n_kv_heads, L->head_dim);
  if (rc != KVRA_OK) return rc;
  if (L->hidden % 64 != 0 || L->ffn % 64 != 0 || L->hidden > kvra::rms_norm_max_hidden()) return KVRA_EUNSUPPORTED;
  if (!(L->scale > 0.0f) || !(L->scale < INFINITY) || !(L->rms_eps >= 0.0f) || !(L->rms_eps < INFINITY)) return KVRA_EINVAL;
  if (!(L->rope_base == L->rope_base)) return KVRA_EINVAL;
  return KVRA_OK;
}

struct LayerWorkspace {
  int64_t h, q, k, v, attn, x2, act, total;   // byte offsets
};

LayerWorkspace layer_workspace(const kvra_layer* L, int64_t c) {
  const int64_t hd = static_cast<int64_t>(L->n_q_heads) * L->head_dim;
  const int64_t kvd = static_cast<int64_t>(L->n_kv_heads) * L->head_dim;
  LayerWorkspace w;
  int64_t at = 0;
  w.h = at;    at += align256(c * L->hidden * 2);
  w.q = at;    at += align256(c * hd * 2);
  w.k = at;    at += align256(c * kvd * 2);
  w.v = at;    at += align256(c * kvd * 2);
  w.attn = at; at += align256(c * hd * 2);
  w.x2 = at;   at += align256(c * L->hidden * 2);
  w.act = at;  at += align256(c * L->ffn * 2);
  w.total = at;
  return w;
}

}  // namespace

extern "C" int64_t kvra_layer_workspace_bytes(const kvra_layer* layer, int64_t chunk_len) {
  if (check_layer(layer) != KVRA_OK || chunk_len < 1 || chunk_len > kMaxTokens) return -1;
  return layer_workspace(layer, chunk_len).total;
}

extern "C" int kvra_layer_chunk(const kvra_layer* L, const void* x, void* y, void* k_cache, void* v_cache,
                                int64_t prefix_len, int64_t chunk_len, int64_t capacity,
                                void* workspace, int64_t workspace_bytes, void* stream) {
  int rc = check_layer(L);
  if (rc != KVRA_OK) return rc;
  if (x == nullptr || y == nullptr || k_cache == nullptr || v_cache == nullptr || workspace == nullptr) return KVRA_EINVAL;
  if (chunk_len < 1 || prefix_len < 0 || capacity < 1) return KVRA_EINVAL;
  if (chunk_len > kMaxTokens || prefix_len > kMaxTokens) return KVRA_EUNSUPPORTED;
  if (prefix_len + chunk_len > capacity) return KVRA_ERANGE;
  const int64_t c = chunk_len;
  const LayerWorkspace w = layer_workspace(L, c);
  if (workspace_bytes < w.total) return KVRA_EINVAL;
  if (reinterpret_cast<uintptr_t>(workspace) % 256 != 0) return KVRA_EINVAL;
  const int64_t hd = static_cast<int64_t>(L->n_q_heads) * L->head_dim;
  const int64_t qkv_rows = hd + 2 * static_cast<int64_t>(L->n_kv_heads) * L->head_dim;
  // every shape check up front, so that nothing is enqueued when a later step would be refused
  if ((rc = check_linear(c, qkv_rows, L->hidden)) != KVRA_OK) return rc;
  if ((rc = check_linear(c, L->hidden, hd)) != KVRA_OK) return rc;
  if ((rc = check_linear(c, 2 * static_cast<int64_t>(L->ffn), L->hidden)) != KVRA_OK) return rc;
  if ((rc = check_linear(c, L->hidden, L->ffn)) != KVRA_OK) return rc;
  char* ws = static_cast<char*>(workspace);
  void *h = ws + w.h, *q = ws + w.q, *k = ws + w.k, *v = ws + w.v, *attn = ws + w.attn, *x2 = ws + w.x2, *act = ws + w.act;
  if ((rc = kvra_rms_norm(x, L->norm1, h, c, L->hidden, L->rms_eps, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_qkv_proj(h, L->wqkv, q, k, v, c, L->n_q_heads, L->n_kv_heads, L->head_dim, L->hidden, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_append_kv(k, v, q, k_cache, v_cache, prefix_len, c, capacity, L->n_q_heads, L->n_kv_heads,
                           L->head_dim, L->rope_base, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_chunk_attn(q, k_cache, v_cache, prefix_len, c, L->n_q_heads, L->n_kv_heads, L->head_dim,
                            L->scale, attn, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_linear(attn, L->wo, nullptr, x, x2, c, L->hidden, hd, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_rms_norm(x2, L->norm2, h, c, L->hidden, L->rms_eps, stream)) != KVRA_OK) return rc;
  if ((rc = kvra_linear(h, L->w_gate, L->w_up, nullptr, act, c, L->ffn, L->hidden, stream)) != KVRA_OK) return rc;
  return kvra_linear(act, L->w_down, nullptr, x2, y, c, L->hidden, L->ffn, stream);
}
