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
//
// Units.  A unit is one kv head x one tile of rows_per_tile query rows walked over the key tiles it can
// see (`steps` of them).  The kv heads are dealt to `groups` groups (8 = one per XCD when the head count
// and the CU count allow, else 1); every group has the same list of units, longest first, and `slots`
// persistent workgroups, one per CU.
//
// Schedule of a slot.  Round 0: slot c runs unit c - only its first head_steps key tiles if it is one of
// the `cut` longest units (cutting is considered while there are fewer than two complete rounds).  Rounds
// 1 .. rounds-1: whole units (round k, slot c: unit k * slots + c, every second round in reverse slot order
// so that long and short units add up alike).  What is left over - the tails of the cut units, then the
// units beyond the complete rounds - forms `segments` key ranges laid end to end; slot c takes the part of
// that line from (fill_seg[c], fill_off[c]) to (fill_seg[c+1], fill_off[c+1]), chosen so that all slots
// finish together.  A piece that is not a whole unit leaves its un-normalised result in the scratch; the
// piece of a unit that finishes last merges them.
constexpr int kMaxSlots = 256;
struct AttnPlan {
  int row_tiles;       // row tiles per kv head
  int rows_per_tile;   // virtual rows (token * group + head in group) per workgroup, <= 256
  int key_tile;        // keys per tile step
  int groups;
  int slots;           // per group, <= kMaxSlots
  int units;           // per group
  int rounds;
  int head_steps;      // 0 = no unit is cut
  int cut;             // units 0 .. cut-1 of the first round stop after head_steps key tiles
  int segments;
  int gangs;           // gang mode: gangs of filler slots per group (0: the line of segments is shared out evenly)
  int gang_heads;      // gang mode: heads per gang slot
  int steps_per_slot;  // planned tile steps (plus the per-piece allowance) of the busiest slot
  int partial_pieces;  // pieces (all groups) that go through the scratch
  int scratch_slots;   // partial-result slots the launch may touch (all groups)
  unsigned fill_seg[kMaxSlots + 1];
  unsigned fill_off[kMaxSlots + 1];
};
int64_t attn_partial_bytes(int head_dim);   // scratch bytes per partial-result slot
int64_t attn_counter_bytes();               // scratch bytes of the merge counters, behind the slots
int plan_chunk_attn(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                    int cus, bool scratch_available, AttnPlan* plan);
// Every piece of the launch as kPieceRecordInts ints: workgroup, kv head, row tile, first key tile, end key
// tile, key tiles of the unit, partial-result slot (-1: whole unit), pieces the merge of its unit reads,
// whether its own slot is among them, merge counter (-1: none).
constexpr int kPieceRecordInts = 10;
int list_chunk_attn_pieces(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                           int cus, int32_t* records, int64_t capacity, int64_t* count_out);

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
