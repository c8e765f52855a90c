// Internal declarations shared by the translation units of libkvra (not installed).
#ifndef KVRA_INTERNAL_H
#define KVRA_INTERNAL_H

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "kvra.h"

namespace kvra {

int launch_append_kv(const void* k_in, const void* v_in, void* q_inout, void* k_cache, void* v_cache,
                     int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                     float rope_base, hipStream_t stream);

int launch_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                      int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                      float scale, void* out, hipStream_t stream, bool static_scratch_only);
int64_t attn_static_scratch_bytes();   // size of the fixed scratch array kvra_chunk_attn_noalloc uses

// Launch shape of kvra_chunk_attn for a device with `cus` compute units (pure host arithmetic).
struct AttnPlan {
  int row_tiles;       // row tiles per kv head
  int rows_per_tile;   // virtual rows (token * group + head in group) per workgroup, <= 256
  int key_tile;        // keys per tile step
  int whole_units;     // (kv head, row tile) units that run as one workgroup
  int split_units;     // units cut into `segments` key segments, one workgroup each, merged by the fix-up kernel
  int segments;        // 1 = no key-split
};
int64_t attn_partial_bytes(int head_dim);   // scratch bytes per (split unit, key segment)
int plan_chunk_attn(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                    int cus, bool scratch_available, AttnPlan* plan);

// out[m, n_out] = x[m, k] . w[n_out, k]^T (+ residual), or silu(x . w^T) * (x . w2^T) when w2 is given.
// The n_out output columns are split over n_seg (1..3) dense matrices of seg_cols[s] columns each.
int launch_linear(const void* x, const void* w, const void* w2, const void* residual,
                  void* const* out, const int* seg_cols, int n_seg,
                  int64_t m, int64_t n_out, int64_t k, hipStream_t stream);

int launch_rms_norm(const void* x, const void* gain, void* y, int64_t rows, int hidden, float eps,
                    hipStream_t stream);
int rms_norm_max_hidden();

// Launch with the runtime's own status as the result.  (hipGetLastError would also pick up
// stale, unrelated codes that other users of the runtime in this thread left behind.)
template <typename Args>
inline int launch_kernel(void (*kernel)(Args), dim3 grid, dim3 block, Args& args, hipStream_t stream,
                         unsigned dynamic_lds_bytes = 0) {
  if (dynamic_lds_bytes > 64 * 1024) {
    // more than 64 KiB of dynamic LDS has to be granted per kernel (once per device is enough,
    // the call is cheap and idempotent)
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                            static_cast<int>(dynamic_lds_bytes)) != hipSuccess)
      return KVRA_ELAUNCH;
  }
  void* params[] = {static_cast<void*>(&args)};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void*>(kernel), grid, block, params,
                                       dynamic_lds_bytes, stream);
  return e == hipSuccess ? KVRA_OK : KVRA_ELAUNCH;
}

}  // namespace kvra

#endif
