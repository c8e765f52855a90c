/*
 * libkvra - single-GPU hot path of KV-Runahead (chunked prefill with a KV-cache) for gfx950.
 *
 * The prompt of length C is cut into consecutive chunks c_0..c_{p-1} (Sec. 3).  The worker of
 * chunk i appends its K,V behind the cache built from chunks 0..i-1 and attends its queries
 * to prefix+chunk keys; only the diagonal block needs the causal mask (Sec. 4.1, Fig. 2, Fig. 5,
 * App. C listing).  On one GPU the chunks run as successive launches on one stream.
 *
 * Conventions shared by all entry points
 *   - Plain C ABI.  Every `void*` tensor argument is a DEVICE pointer owned by the caller; the
 *     library never frees or keeps it.  bf16 = the upper 16 bits of an IEEE float32.
 *   - Tensors are dense, token-major: [tokens, heads, head_dim], head_dim contiguous.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  GPU entry points
 *     only enqueue work on it and return; they never synchronise.
 *   - Return value: KVRA_OK, or a negative code; on error nothing was enqueued.
 *   - head_dim must be 64 or 128; n_q_heads must be a multiple of n_kv_heads; query head h
 *     reads key/value head h / (n_q_heads / n_kv_heads).
 *   - The only state the library keeps is one scratch buffer per device (about 100 MB, hipMalloc'ed
 *     by the first kvra_chunk_attn call on that device that is allowed to allocate, kept until the
 *     process ends).  It holds the partial results and merge counters of row tiles that
 *     kvra_chunk_attn cuts along the keys, which it does whenever the (kv head, 256-row tile) units
 *     of a call do not divide evenly over the device's CUs - e.g. a short chunk behind a long
 *     prefix, or 160 units on 256 CUs.  While there is no buffer - the allocation failed, or
 *     `stream` is being captured into a graph, where allocating is illegal - a call runs whole
 *     units only (same results up to rounding order, slower on such shapes) and the next call
 *     tries again; to have cut units inside a captured graph, make one kvra_chunk_attn call on the
 *     device before the capture starts, or use kvra_chunk_attn_noalloc.  The buffer belongs to the
 *     device that is current when the call is made, which must be the device of `stream`
 *     (KVRA_EINVAL if `stream` is known to belong to another device).
 *     Two calls that cut units (kvra_layer_chunk included) and overlap in time on one device, from
 *     different streams, share the buffer and race: not supported, not detected.
 */
#ifndef KVRA_H
#define KVRA_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  KVRA_OK = 0,
  KVRA_EINVAL = -1,       /* null pointer, non-positive size, heads not divisible, bad scale   */
  KVRA_EUNSUPPORTED = -2, /* head_dim other than 64 / 128, or a size beyond the 32-bit tiling   */
  KVRA_ERANGE = -3,       /* prefix_len + chunk_len exceeds the cache capacity                  */
  KVRA_ELAUNCH = -4,      /* the HIP runtime refused the launch                                  */
  KVRA_ENODEVICE = -5,    /* no usable gfx950 device                                            */
  KVRA_ESCRATCH = -6      /* kvra_chunk_attn_noalloc: the launch needs more scratch than it owns */
};

/* Human-readable text for a return code (static storage, never NULL). */
const char* kvra_strerror(int code);

/* Library version as major*10000 + minor*100 + patch. */
int kvra_version(void);

/*
 * Cache population of one chunk: the "K = cat(cache.K, K); V = cat(cache.V, V)" step of the
 * attention block (App. C listing; Sec. 4.3 asks for the cache to be physically contiguous).
 * Rotary position embedding is applied on the way (the paper's models, Sec. 5, are rotary;
 * half-split pairing: component i pairs with i + head_dim/2 and turns by
 * position * rope_base^(-2i/head_dim), position = prefix_len + row).
 *
 *   k_in    [chunk_len, n_kv_heads, head_dim] bf16, un-rotated            (device, read)
 *   v_in    [chunk_len, n_kv_heads, head_dim] bf16                        (device, read)
 *   q_inout [chunk_len, n_q_heads,  head_dim] bf16 or NULL; rotated in place (device, read/write)
 *   k_cache, v_cache [capacity, n_kv_heads, head_dim] bf16; rows [prefix_len, prefix_len+chunk_len)
 *           are written, every other row is left untouched               (device, write)
 *   rope_base  e.g. 10000; <= 0 turns the rotation off (K and Q are copied / left as they are)
 *
 * Angles are formed in fp64, the rotation in fp32, results rounded to nearest-even bf16.
 * V is copied bit for bit.  Errors: KVRA_EINVAL, KVRA_EUNSUPPORTED, KVRA_ERANGE, KVRA_ELAUNCH.
 */
int kvra_append_kv(const void* k_in, const void* v_in, void* q_inout,
                   void* k_cache, void* v_cache,
                   int64_t prefix_len, int64_t chunk_len, int64_t capacity,
                   int n_q_heads, int n_kv_heads, int head_dim,
                   float rope_base, void* stream);

/*
 * Attention of one chunk against prefix+chunk keys: softmax(scale * Q K^T + mask) V with the
 * mask -inf above the diagonal (Fig. 1(b); Sec. 4.1; App. C listing, weights and output steps).
 * The query in chunk row r sits at absolute position prefix_len + r and sees cache rows
 * 0 .. prefix_len + r inclusive.  Tiles wholly above the diagonal are never issued.
 *
 *   q        [chunk_len, n_q_heads, head_dim] bf16, already rotated       (device, read)
 *   k_cache, v_cache  token-major caches, rows [0, prefix_len+chunk_len) valid (device, read)
 *   scale    multiplies Q K^T before the softmax (1/sqrt(head_dim) by convention); finite, > 0
 *   out      [chunk_len, n_q_heads, head_dim] bf16                        (device, write)
 *
 * bf16 MFMA products with fp32 accumulation, fp32 online softmax, P rounded to bf16 before P V.
 * scale (times log2 e) is multiplied into Q before the score product and that Q rounded to bf16.
 * Errors: KVRA_EINVAL, KVRA_EUNSUPPORTED, KVRA_ELAUNCH.
 */
int kvra_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                    int64_t prefix_len, int64_t chunk_len,
                    int n_q_heads, int n_kv_heads, int head_dim,
                    float scale, void* out, void* stream);

/*
 * kvra_chunk_attn for callers that cannot allocate device memory: code that runs under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels, same
 * launch plan and therefore the same results bit for bit; it calls no hipMalloc / hipFree and no
 * allocating library routine.  The partial results and counters of cut units go to a fixed array in the
 * library's device image instead of the allocated buffer: kvra_chunk_attn_noalloc_scratch_bytes()
 * bytes (99 MiB = 768 partial-result slots, three per compute unit of a 256-CU device), which every
 * GPU the library is loaded on holds until the process ends.  Its device address is looked up on the
 * first call on each device (hipGetSymbolAddress, no allocation).
 *   - A call whose launch plan (kvra_chunk_attn_plan with the device's CU count) needs more than
 *     that - possible only on a device with more than 256 CUs - returns KVRA_ESCRATCH and enqueues
 *     nothing.  KVRA_ENODEVICE: the array's address could not be obtained.
 *   - Calls need no clearing in between: a partial-result slot is written in full before the piece
 *     that merges its row tile reads it, and the merge counters (zero when the library is loaded)
 *     are set back to zero by every merge.  The other contents after a call are scratch.
 *   - All calls on one GPU share the array: two calls that overlap in time on one device (different
 *     streams, or two graphs replayed concurrently) race.  Calls on one stream are ordered and safe.
 */
int kvra_chunk_attn_noalloc(const void* q, const void* k_cache, const void* v_cache,
                            int64_t prefix_len, int64_t chunk_len,
                            int n_q_heads, int n_kv_heads, int head_dim,
                            float scale, void* out, void* stream);
int64_t kvra_chunk_attn_noalloc_scratch_bytes(void);

/*
 * How kvra_chunk_attn lays the chunk's trapezoid of (query, key) pairs (Fig. 2(c), Sec. 4.1) onto a device
 * with `n_cus` compute units.  Host arithmetic only: nothing is launched or allocated, and no device
 * needs to be present.
 *   A unit is one kv head x one tile of `rows_per_tile` query rows (row = token * group + head in group)
 * walked over all the key tiles it can see.  The kv heads are dealt to `groups` groups (8, one per XCD,
 * when the head count and n_cus are multiples of 8; else 1); each group has `units` units, longest first,
 * and `slots` persistent workgroups, one per compute unit: the launch has groups * slots workgroups.
 *   In round 0 slot c runs unit c, but only its first `head_steps` key tiles if it is one of the `cut_units`
 * longest units (units are cut while there are fewer than two complete rounds).  Rounds 1 .. rounds-1 are
 * whole units.  The rest - the tails of the cut units, then the units beyond the complete rounds - is
 * `segments` key ranges laid end to end and shared out among the slots so that all finish together after
 * about `steps_per_slot` tile steps (eight of which per piece are the allowance for starting and finishing it).
 * `partial_pieces` pieces (over all groups) are not whole units: they leave their un-normalised results in
 * the scratch (`scratch_bytes` = the partial-result slots the launch may touch x 132 KiB), and the piece
 * of a unit that finishes last merges them inside the kernel.
 *   Gang mode (`gangs` > 0): when a group has fewer units than slots, every unit is cut and at least
 * `row_tiles` slots have no unit of their own, the tails are not shared out piecemeal: the free slots form
 * `gangs` gangs of `row_tiles` slots, gang slot r runs the tail of row tile r of `gang_heads` heads one after
 * the other, and the row tiles of a head then read the same keys at the same time (K/V comes from HBM once,
 * every such unit has exactly two pieces); the gangs take the first gangs * gang_heads heads of the group, and
 * free slots that fit no gang share the tails of the other heads as above, or stay idle if there is none.  Taken
 * while it ends at most a tenth later, in tile steps, than the evenly shared plan.
 *   kvra_chunk_attn takes this plan with the CU count of the current device; while it has no scratch (see
 * the conventions at the top) it takes the plan in which no unit is cut.
 * Errors: KVRA_EINVAL (plan NULL, n_cus < 1, sizes as for kvra_chunk_attn), KVRA_EUNSUPPORTED.
 */
typedef struct kvra_attn_plan {
  int row_tiles;        /* row tiles per kv head */
  int rows_per_tile;    /* multiple of 32, <= 256 */
  int key_tile;         /* keys per tile step: 64 at head_dim 128, 128 at head_dim 64 */
  int groups;
  int slots;            /* per group */
  int units;            /* per group */
  int rounds;
  int head_steps;
  int cut_units;
  int segments;
  int steps_per_slot;
  int partial_pieces;
  int gangs;            /* gang mode: gangs of row_tiles slots per group that run the tails in step; else 0 */
  int gang_heads;       /* gang mode: heads (tails) per gang slot */
  int64_t scratch_bytes;
} kvra_attn_plan;
int kvra_chunk_attn_plan(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads,
                         int head_dim, int n_cus, kvra_attn_plan* plan);

/*
 * The pieces of that plan, one record of 10 ints each, workgroup by workgroup in the order each
 * workgroup runs them (host arithmetic only; the kernel walks the same list with the same code):
 *   [0] workgroup id  [1] kv head  [2] row tile  [3] first key tile  [4] end key tile (exclusive)
 *   [5] key tiles of the whole unit  [6] partial-result slot in the scratch, -1 for a whole unit
 *   [7] number of pieces the merge of this unit reads, 0 for a whole unit  [8] 1 if this piece's slot is
 *   among them  [9] index of the unit's merge counter, -1 for a whole unit
 *   records    host array of capacity * 10 ints, or NULL with capacity 0 to ask for the count only
 *   count_out  number of pieces of the launch (may exceed capacity; only `capacity` records are written)
 * Errors: as kvra_chunk_attn_plan; KVRA_EINVAL for a negative capacity or NULL records with capacity > 0.
 */
int kvra_chunk_attn_pieces(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads,
                           int head_dim, int n_cus, int32_t* records, int64_t capacity, int64_t* count_out);

/*
 * Context-level load balancing (Sec. 4.2), host only.  Picks boundaries 0 = b_0 < b_1 < ... <
 * b_n = context_len, all multiples of `granularity`, that minimise the largest per-chunk cost
 * max_i cost(b_i, b_{i+1} - b_i): with one worker per chunk and many layers the slowest worker
 * sets the time to first token.  The search is exact over the grid (dynamic programme over
 * O(n_chunks * (context_len/granularity)^2) cost evaluations); among partitions of equal makespan
 * the lexicographically smallest boundary vector is returned.
 *
 *   cost   called on the host with (prefix_len, chunk_len, user); any unit; NULL selects the
 *          analytic causal-work model chunk_len * (2*prefix_len + chunk_len)
 *   boundaries_out  host array of n_chunks + 1 entries
 *   makespan_out    host double or NULL
 *
 * Errors (KVRA_EINVAL): n_chunks < 1, granularity < 1, context_len not a multiple of granularity,
 * context_len < n_chunks * granularity, NULL boundaries_out, a cost that returns NaN.
 */
typedef double (*kvra_cost_fn)(int64_t prefix_len, int64_t chunk_len, void* user);

int kvra_balance(int64_t context_len, int n_chunks, int64_t granularity,
                 kvra_cost_fn cost, void* user,
                 int64_t* boundaries_out, double* makespan_out);

/* Even partitioning (the KVR-E variant of Sec. 5): b_k = granularity * round(k*C/(n*granularity)).
 * Same argument checks as kvra_balance. */
int kvra_equal_split(int64_t context_len, int n_chunks, int64_t granularity, int64_t* boundaries_out);

/* Largest per-chunk cost of a given partition (same cost convention as kvra_balance).
 * boundaries: host array of n_chunks + 1 strictly rising entries starting at 0. */
int kvra_makespan(const int64_t* boundaries, int n_chunks, kvra_cost_fn cost, void* user,
                  double* makespan_out);

/*
 * Time to first token of the chain of processes p_0 -> p_1 -> ... (Sec. 4 overview and Fig. 5(b):
 * every process runs every layer on its own chunk and must wait, in each layer, for the KV-cache of
 * its precedent, which makes the later processes lag by layers), with one process per chunk and
 * `n_layers` identical layers.  Per layer, process i first spends before_attn(prefix_i, c_i) (norm,
 * projections, rotation, append); its cache is complete when that is done and the cache of process
 * i-1 has arrived, handoff(prefix_{i-1}, c_{i-1}) after that one was complete (NULL: no transfer
 * time); then it attends for attn(prefix_i, c_i) plus whatever follows in the layer, and starts
 * the next layer.  The result is the time at which the last process leaves the last layer.
 * Host only.  All three callbacks get the same `user`; costs must be >= 0.
 * Errors (KVRA_EINVAL): NULL boundaries / ttft_out / before_attn / attn, n_chunks < 1,
 * n_layers < 1, boundaries not strictly rising from 0, a negative or NaN cost.
 */
int kvra_chain_ttft(const int64_t* boundaries, int n_chunks, int n_layers,
                    kvra_cost_fn before_attn, kvra_cost_fn attn, kvra_cost_fn handoff,
                    void* user, double* ttft_out);

/*
 * One-dimensional search for two processes (Sec. 4.2, the two-partition panel of the search
 * figure): the first process's cost grows and the second's shrinks as the interior boundary moves
 * right, so the crossing is found by bisection in O(log(context_len/granularity)) cost
 * evaluations and the better of the two grid points around it is returned (ties: the smaller
 * boundary).  Exact when cost(0, c) is non-decreasing and cost(b, C - b) non-increasing in the
 * boundary; otherwise still a valid partition.
 *   boundaries_out   host array of 3 entries;  makespan_out, evaluations_out   host scalars or NULL
 * Errors (KVRA_EINVAL): as kvra_balance with n_chunks = 2.
 */
int kvra_search_two_way(int64_t context_len, int64_t granularity, kvra_cost_fn cost, void* user,
                        int64_t* boundaries_out, double* makespan_out, int64_t* evaluations_out);

/*
 * Hierarchical grid search (Sec. 4.2, search figure panels with strides 8/4/2; appendix on lookup
 * table generation: five values per boundary and level).  Level by level every interior boundary
 * is tried at its current value + {-2,-1,0,1,2} * stride; of all 5^(n_chunks-1) combinations that
 * are strictly rising inside (0, context_len) the one with the smallest makespan (ties: the
 * lexicographically smallest) becomes the centre of the next level, whose stride is half as
 * large.  The first stride is the largest granularity * 2^k with 2 * stride < context_len /
 * n_chunks; the last is `granularity`.  A heuristic: its reach is limited to about two first
 * strides around the starting point.
 *   start            host array of n_chunks + 1 entries (a valid partition on the grid), or NULL for
 *                    the even split
 *   boundaries_out   host array of n_chunks + 1 entries (never worse than `start`)
 *   makespan_out, evaluations_out (number of cost callbacks made)   host scalars or NULL
 * Errors (KVRA_EINVAL): as kvra_balance; `start` not a partition of context_len on the grid.
 */
int kvra_search_grid(int64_t context_len, int n_chunks, int64_t granularity, const int64_t* start,
                     kvra_cost_fn cost, void* user, int64_t* boundaries_out, double* makespan_out,
                     int64_t* evaluations_out);

/*
 * The hierarchical grid search with the objective left to the caller, as in the paper, whose search
 * runs on the measured time to first token of the whole chain (Sec. 4.2): same levels, strides,
 * candidates and tie-break as kvra_search_grid, but `objective` is called once per feasible
 * combination (up to 5^(n_chunks-1) per level; n_chunks <= 10) with a host array of n_chunks + 1
 * boundaries.  kvra_chain_ttft over fitted per-chunk costs is one such objective.
 *   value_out, evaluations_out   host scalars or NULL
 * Errors: KVRA_EINVAL as kvra_search_grid, NULL objective, an objective that returns NaN;
 * KVRA_EUNSUPPORTED for n_chunks > 10.
 */
typedef double (*kvra_partition_fn)(const int64_t* boundaries, int n_chunks, void* user);

int kvra_search_grid_objective(int64_t context_len, int n_chunks, int64_t granularity, const int64_t* start,
                               kvra_partition_fn objective, void* user, int64_t* boundaries_out,
                               double* value_out, int64_t* evaluations_out);

/*
 * Predicted partitioning from two lookup-table entries (KVR-P; Sec. 4.2, and the partitioning
 * paragraph of Sec. 5 that interpolates 8k and 12k entries for a 10k context).  The cumulative
 * ratios b_k / length of the two entries are blended linearly in context_len (clamped to the
 * nearer entry outside [len_lo, len_hi]), scaled by context_len and rounded to the nearest
 * multiple of `granularity` (halves up); colliding boundaries are pushed one granule apart.
 *   bounds_lo, bounds_hi   host arrays of n_chunks + 1 strictly rising entries, 0 .. len_lo / len_hi
 *   boundaries_out         host array of n_chunks + 1 entries
 * Errors (KVRA_EINVAL): bad grid, len_hi < len_lo, entries that are not partitions of their length.
 */
int kvra_interpolate(int64_t context_len, int n_chunks, int64_t granularity,
                     int64_t len_lo, const int64_t* bounds_lo,
                     int64_t len_hi, const int64_t* bounds_hi, int64_t* boundaries_out);

/*
 * Prediction from a whole lookup table (the partitioning table of the overview figure): picks the
 * two entries that bracket context_len (the nearest single entry outside the table's range) and
 * applies kvra_interpolate.
 *   entry_lens     host array [n_entries], any order
 *   entry_bounds   host array [n_entries][n_chunks + 1], row e partitions entry_lens[e]
 */
int kvra_table_predict(int64_t context_len, int n_chunks, int64_t granularity, int n_entries,
                       const int64_t* entry_lens, const int64_t* entry_bounds, int64_t* boundaries_out);

/*
 * ---- The decoder layer a process runs around its attention block --------------------------------
 * Every process runs each layer on its own chunk (Sec. 4.1); the App. C listing shows the q/k/v
 * projections before and the output projection after the attention.  Normalisation and MLP are not
 * written out in the paper; they follow the LLaMA architecture of the models in Sec. 5: pre-norm
 * RMSNorm, no biases, SwiGLU MLP, two residual connections.  All tensors are dense bf16 device
 * memory; arithmetic is fp32 (MFMA accumulation, norms, activation) with one rounding to bf16 per
 * stored tensor.
 */

/* y[t, :] = x[t, :] / sqrt(mean_j x[t, j]^2 + eps) * gain.   x, y: [rows, hidden]; gain: [hidden].
 * hidden must be a multiple of 8 and at most 8192 (KVRA_EUNSUPPORTED otherwise). */
int kvra_rms_norm(const void* x, const void* gain, void* y, int64_t rows, int hidden, float eps, void* stream);

/*
 * Linear layer without bias on the matrix cores: out[m, n] = sum_j x[m, j] * w[n, j]
 * (weights stored [out_features, in_features]).
 *   residual != NULL   out = x.w^T + residual            (residual: [m, n]; may alias out)
 *   w2 != NULL         out = silu(x.w^T) * (x.w2^T)      (the SwiGLU gate and up projections in one pass)
 * residual and w2 exclude each other (KVRA_EINVAL).  m is free; n must be a multiple of 32 and k of
 * 64, and x and w must each stay below 4 GiB (KVRA_EUNSUPPORTED).
 */
int kvra_linear(const void* x, const void* w, const void* w2, const void* residual, void* out,
                int64_t m, int64_t n, int64_t k, void* stream);

/*
 * The three projections of the App. C listing in one launch.  wqkv: [(n_q_heads + 2 n_kv_heads) *
 * head_dim, k], query rows first, then key rows, then value rows.  q_out [m, n_q_heads, head_dim],
 * k_out, v_out [m, n_kv_heads, head_dim] are the dense tensors kvra_append_kv takes (un-rotated).
 */
int kvra_qkv_proj(const void* x, const void* wqkv, void* q_out, void* k_out, void* v_out,
                  int64_t m, int n_q_heads, int n_kv_heads, int head_dim, int64_t k, void* stream);

typedef struct {
  int hidden, ffn, n_q_heads, n_kv_heads, head_dim;
  float rms_eps;       /* 1e-6 for the LLaMA shapes                                    */
  float rope_base;     /* <= 0 disables the rotary embedding                             */
  float scale;         /* softmax scale, 1/sqrt(head_dim) by convention                  */
  const void* norm1;   /* [hidden]                                                       */
  const void* wqkv;    /* [(n_q_heads + 2 n_kv_heads) head_dim, hidden]                  */
  const void* wo;      /* [hidden, n_q_heads head_dim]                                   */
  const void* norm2;   /* [hidden]                                                       */
  const void* w_gate;  /* [ffn, hidden]                                                  */
  const void* w_up;    /* [ffn, hidden]                                                  */
  const void* w_down;  /* [hidden, ffn]                                                  */
} kvra_layer;

/* Bytes of device workspace kvra_layer_chunk needs for a chunk of this length (-1: bad layer). */
int64_t kvra_layer_workspace_bytes(const kvra_layer* layer, int64_t chunk_len);

/*
 * One layer over one chunk: RMSNorm, q/k/v projections, kvra_append_kv (rotary embedding + cache
 * rows [prefix_len, prefix_len + chunk_len)), kvra_chunk_attn, output projection + residual,
 * RMSNorm, SwiGLU MLP + residual; eight launches on `stream`.
 *   x, y        [chunk_len, hidden]; y may not alias x
 *   workspace   caller-owned device memory, 256-byte aligned, at least
 *               kvra_layer_workspace_bytes(layer, chunk_len); contents are scratch
 * Errors: as the calls it is made of; KVRA_EINVAL for a short or misaligned workspace.  hidden and
 * ffn must be multiples of 64.
 */
int kvra_layer_chunk(const kvra_layer* layer, const void* x, void* y, void* k_cache, void* v_cache,
                     int64_t prefix_len, int64_t chunk_len, int64_t capacity,
                     void* workspace, int64_t workspace_bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* KVRA_H */
