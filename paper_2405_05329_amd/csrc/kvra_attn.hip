// kvra_chunk_attn: flash-style tiled causal attention of one chunk against prefix+chunk keys
// (Sec. 4.1, Fig. 5(b); App. C listing, weights and output steps) for gfx950.
//
// Orientation.  Each wave owns 32 query rows and computes the TRANSPOSED score tile
//   S^T[key, query] = K_tile . Q^T        (v_mfma_f32_32x32x16_bf16, A = K from LDS, B = Q in VGPRs)
// so that one lane holds 32 scores of a single query: row max / row sum are in-lane reductions
// plus one exchange between the two lane halves.  The accumulator layout of S^T is, register
// for register, the B-operand layout of the second product
//   O^T[d, query] += V_tile^T . P^T       (A = V^T via ds_read_b64_tr_b16, B = P in VGPRs)
// so P never visits LDS.
//
// Rows.  With grouped queries (G = n_q_heads / n_kv_heads > 1) the G heads that share a KV head
// are folded into the row index: virtual row v = token * G + head_in_group.  One K/V tile in LDS
// then serves several query heads, and the diagonal band (the only masked part) stays one key
// tile wide whatever G is.
//
// Schedule.  A workgroup is 8 waves = two groups of 4 (one wave of each group per SIMD).  Per key
// tile a wave runs an MFMA block (P.V of the previous tile, then K.Q^T of this one: 32 MFMAs at
// d = 128) and a VALU block (softmax of this tile, staging of future K/V tiles).  While one group
// keeps the matrix pipe busy its SIMD partner does the exponentials on the vector ALU
// ("ping-pong").  At d = 64 there is a workgroup barrier after each block and the second group
// starts one barrier late.  At d = 128 there is one barrier per tile step: the first group runs
// [MFMA block, VALU block, barrier], the second [VALU block of the previous tile, MFMA block,
// barrier]; the barrier puts the groups back into opposite phases, and in between a group that is
// done with its vector work starts on the matrix pipe at once instead of waiting for its partner.
//
// Softmax arithmetic.  scale * log2(e) is folded into the Q fragment (one more bf16 rounding of
// Q, of the size the rotation already made) and the score accumulators start at minus the row's
// exponent reference m, so the MFMAs hand back  s = scale log2(e) q.k - m  and a weight is one
// exp2 away.  No row maximum is formed on the way (see kSumLimit).  Every instruction of the VALU
// block costs issue time the matrix pipe of the partner wave waits for, scalar ones included, and
// v_dot2c_f32_bf16 queues behind the partner's MFMAs: the block is kept to exp2, add and convert.
//
// Launch shape.  A unit is one 256-row tile of one kv head against all the key tiles it sees.  A launch is
// one persistent kernel, one workgroup per compute unit, that walks a schedule made on the host
// (plan_chunk_attn): the workgroups form groups (one per XCD, each with its own kv heads), a slot of a
// group runs whole units of the complete rounds and then its share of what does not fill a round - leftover
// units and, when there is at most one complete round, the tails of the first round's units cut at a common
// length - so that every slot ends up with the same number of tile steps.  A piece that is not a whole unit
// leaves its un-normalised (O, m, l) in a scratch slot with device-coherent stores and adds its tile steps
// to the unit's counter; the piece that completes the count merges the unit's partial results in a fixed
// order (the usual log-sum-exp merge) and writes the rows.  No workgroup waits for another one.  Where a
// group's free slots can form gangs of one slot per row tile, the tails of a head are run side by side by a
// gang instead (gang mode, see plan_chunk_attn), so that they share the K/V stream as the heads do.
#include "kvra_internal.h"

#include <algorithm>
#include <mutex>
#include <type_traits>
#include <vector>

namespace kvra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kWaves = 8;              // waves per workgroup
constexpr int kThreads = 64 * kWaves;
// keys per tile: 64 at head_dim 128; 128 at head_dim 64, where a 64-key tile holds too little MFMA
// work (16 per wave) to carry the two barriers of a tile step
constexpr int key_tile(int D) { return D == 64 ? 128 : 64; }
constexpr int kStages = 3;             // LDS ring depth for K and for V tiles
// barriers per tile step: one at head_dim 128 (measured +4..5 %), two at head_dim 64 (one: -4 %)
constexpr bool one_barrier(int D) { return D == 128; }
constexpr float kSumLimit = 1048576.0f; // a lane's partial row sum over one tile beyond which the reference is moved
constexpr float kNoKeyYet = -1e30f;    // exponent reference of a row before its first visible key

struct AttnArgs {
  const __bf16* q;
  const __bf16* k;
  const __bf16* v;
  __bf16* out;
  int prefix;
  int chunk;
  int H;
  int Hkv;
  int G;
  int nq_tiles;      // row tiles per kv head
  int rows_per_wg;   // virtual rows per workgroup: 32 * (active waves), <= 256
  float c_log2;      // scale * log2(e): softmax runs in base 2
  int bn;            // keys per tile, key_tile(head_dim)
  // schedule (see AttnPlan): the launch has groups * slots persistent workgroups
  int groups;
  int slots;
  int units;         // per group
  int rounds;
  int head_steps;
  int cut;
  int segments;
  int gangs;         // 0, or (gang mode) the gangs of filler slots per group: see plan_chunk_attn
  int gang_heads;    // heads each gang slot works through, one tail after the other
  float* scratch;    // partial results: slots_per_group() slots per group; nullptr when nothing is cut
  int* counters;     // key tiles merged so far, one per (group, segment); all zero between launches
#ifdef KVRA_TRACE
  unsigned long long* trace;   // kTraceWords words per piece, kTracePieces pieces per workgroup, or nullptr
#endif
  unsigned fill_seg[kMaxSlots + 1];
  unsigned fill_off[kMaxSlots + 1];
};

#ifdef KVRA_TRACE
// Timeline build (python -m paper_2405_05329_amd.build --trace): every workgroup leaves time stamps of the
// constant 100 MHz clock - entry, first tile step, last tile step done, exit - with the compute unit it
// ran on, its number of tile steps and the shader-clock cycle counter at both ends of the tile loop, for the
// accounting of where a launch's time goes.
constexpr int kTraceWords = 10;
constexpr int kTracePieces = 8;   // pieces of a workgroup that leave stamps
__device__ __forceinline__ void trace_stamp(unsigned long long* rec, int word) {
  if (rec != nullptr && threadIdx.x == 0) {
    rec[word] = wall_clock64();
    // around the tile loop also the shader-clock cycle counter: cycles / time = the clock the loop ran at
    if (word == 1 || word == 2) rec[7 + word] = clock64();
  }
}
#define KVRA_TRACE_STAMP(rec, word) trace_stamp(rec, word)
#else
#define KVRA_TRACE_STAMP(rec, word)
#endif

// Units of a group, longest row tiles first: unit j of group x is kv head x + groups * (j % hp),
// hp = heads per group, row tile nq_tiles - 1 - j / hp.  With 8 groups, workgroup ids go round-robin
// over the XCDs, so group x = workgroup id % 8 lives on one XCD and that XCD's L2 holds the K/V
// stream of its own heads only.
__host__ __device__ __forceinline__ void unit_of(const AttnArgs& a, int x, int j, int* g, int* qt) {
  const int hp = a.Hkv / a.groups;
#ifdef KVRA_HEADS_CONTIGUOUS
  *g = x * hp + (j % hp);
#else
  *g = x + a.groups * (j % hp);
#endif
  *qt = a.nq_tiles - 1 - j / hp;
}
__host__ __device__ __forceinline__ int unit_steps(const AttnArgs& a, int qt) {
  const int rows = a.chunk * a.G;
  const int row_hi = (qt + 1) * a.rows_per_wg < rows ? (qt + 1) * a.rows_per_wg : rows;   // exclusive, in virtual rows
  return (a.prefix + (row_hi - 1) / a.G) / a.bn + 1;                                      // key tiles the row tile walks
}

// Gang mode (a.gangs > 0; every unit of the group is cut, the line of segments is their tails and nothing
// else): the line is not in unit order but gang by gang, row tile by row tile, head by head, so that the
// a.gang_heads tails a gang slot takes are consecutive and the slots of a gang - one per row tile - work
// on the same head at the same time.  Segment s of the line <-> unit j of the group:
// (the gangs take the first gangs * gang_heads heads of the group; the tails of the other heads follow in
// the line head by head, row tile by row tile, for the free slots that fit no gang)
__host__ __device__ __forceinline__ int seg_to_unit(const AttnArgs& a, int s) {
  if (a.gangs == 0) return s;
  const int hp = a.Hkv / a.groups, R = a.nq_tiles, k = a.gang_heads, gang_segments = a.gangs * R * k;
  if (s >= gang_segments) return ((s - gang_segments) % R) * hp + a.gangs * k + (s - gang_segments) / R;
  const int g = s / (R * k), rank = (s % (R * k)) / k, i = s % k;
  return rank * hp + g + a.gangs * i;
}
__host__ __device__ __forceinline__ int unit_to_seg(const AttnArgs& a, int j) {
  if (a.gangs == 0) return j;
  const int hp = a.Hkv / a.groups, R = a.nq_tiles, k = a.gang_heads;
  const int head = j % hp, rank = j / hp;
  if (head >= a.gangs * k) return a.gangs * R * k + (head - a.gangs * k) * R + rank;
  return ((head % a.gangs) * R + rank) * k + head / a.gangs;
}
// Partial-result slots of a group: id c + s for the piece of segment s that slot c runs (both only grow
// along the line of segments, so the sum is unique), and slots + segments + s for the head of unit s.
__host__ __device__ __forceinline__ int slots_per_group(const AttnArgs& a) { return a.slots + 2 * a.segments; }

// One piece of work: key tiles [jt0, jt1) of a unit.
struct Piece {
  int g, qt;         // kv head, row tile
  int jt0, jt1;
  int n;             // key tiles of the whole unit
  int seg;           // segment the unit belongs to (pieces that are not the whole unit), else -1
  int slot;          // partial-result slot within the group, -1 for a whole unit
};

// The pieces of slot c of group x, in the order the slot runs them (the same code on the device, where
// the kernel walks them, and on the host, where kvra_chunk_attn_pieces lists them).
struct PieceWalker {
  int x, c, seg, off, seg_end, off_end, round;
  __host__ __device__ PieceWalker(const AttnArgs& a, int group, int slot)
      : x(group), c(slot), seg(static_cast<int>(a.fill_seg[slot])), off(static_cast<int>(a.fill_off[slot])),
        seg_end(static_cast<int>(a.fill_seg[slot + 1])), off_end(static_cast<int>(a.fill_off[slot + 1])), round(0) {}
  __host__ __device__ bool next(const AttnArgs& a, Piece* pc) {
    const int P = a.slots;
    if (round == 0 && c < a.units) {
      // first round: unit c, cut after head_steps key tiles if it is one of the `cut` longest units
      ++round;
      unit_of(a, x, c, &pc->g, &pc->qt);
      pc->n = unit_steps(a, pc->qt);
      pc->jt0 = 0;
      const bool is_cut = c < a.cut;
      pc->jt1 = is_cut ? a.head_steps : pc->n;
      pc->seg = is_cut ? unit_to_seg(a, c) : -1;
      pc->slot = is_cut ? P + a.segments + c : -1;
      return true;
    }
    if (round > 0 && round < a.rounds) {
      const int j = round * P + ((round & 1) ? P - 1 - c : c);
      ++round;
      unit_of(a, x, j, &pc->g, &pc->qt);
      pc->n = unit_steps(a, pc->qt);
      pc->jt0 = 0;
      pc->jt1 = pc->n;
      pc->seg = -1;
      pc->slot = -1;
      return true;
    }
    if (seg < seg_end || (seg == seg_end && off < off_end)) {
      round = a.rounds + 1;
      // the unit behind segment `seg` and where the segment starts inside it: the tails of the cut units
      // come first, then the units beyond the complete rounds
      const int j = seg < a.cut ? seg_to_unit(a, seg) : a.rounds * P + seg - a.cut;
      const int first = seg < a.cut ? a.head_steps : 0;
      unit_of(a, x, j, &pc->g, &pc->qt);
      pc->n = unit_steps(a, pc->qt);
      pc->jt0 = first + off;
      pc->jt1 = seg < seg_end ? pc->n : first + off_end;
      const bool whole = pc->jt0 == 0 && pc->jt1 == pc->n;
      pc->seg = whole ? -1 : seg;
      pc->slot = whole ? -1 : c + seg;
      if (seg < seg_end) { ++seg; off = 0; }
      else off = off_end;
      return true;
    }
    return false;
  }
};

// The partial-result slots (within the group) of all pieces of segment s, in the fixed order of the merge:
// the head (if the segment is the tail of a cut unit), then the slots whose share of the line of segments
// meets this segment.
template <typename F>
__host__ __device__ __forceinline__ void for_each_piece_of_segment(const AttnArgs& a, int s, F&& fn) {
  if (s < a.cut) fn(a.slots + a.segments + seg_to_unit(a, s));
  for (int c = 0; c < a.slots; ++c) {
    const unsigned s0 = a.fill_seg[c], o0 = a.fill_off[c], s1 = a.fill_seg[c + 1], o1 = a.fill_off[c + 1];
    const bool nonempty = s0 < s1 || (s0 == s1 && o0 < o1);
    const bool meets = static_cast<int>(s0) <= s && (static_cast<int>(s1) > s || (static_cast<int>(s1) == s && o1 > 0));
    if (nonempty && meets) fn(c + s);
  }
}

constexpr int kPartialFloats(int D) { return kWaves * (D / 32 * 16 + 2) * 64; }   // per scratch slot

// A store that is visible to the whole device once it has been acknowledged, and a load that sees such
// stores (they go past whatever a non-coherent cache level holds).
__device__ __forceinline__ void store_coherent(float* p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float load_coherent(const float* p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

__device__ __forceinline__ float other_half(float x) {
  // value held by lane ^ 32
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

// 64 lanes x 16 bytes from global memory straight into 1 KiB of consecutive LDS starting at
// lds_byte_addr (lane l lands at +16 l).  Global address = uniform base + per-lane byte offset.
// Written as inline assembly on purpose: the compiler guards every LDS-direct load it knows about
// with a full vmcnt(0) wait (it cannot tell the ring slots apart), which would serialise the
// prefetch; here completion is awaited by hand, once per block, with s_waitcnt vmcnt(n).
__device__ __forceinline__ void lds_dma16(const void* uniform_base, unsigned lane_byte_off, unsigned lds_byte_addr) {
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_off), "s"(uniform_base), "s"(lds_byte_addr)
               : "memory", "m0");
}

// The same under a wave-uniform switch: with on_mask = 0 the instruction is issued with no lanes
// enabled and moves nothing (no branch around it, so that it can sit in straight-line code).
__device__ __forceinline__ void lds_dma16_if(unsigned long long on_mask, const void* uniform_base,
                                             unsigned lane_byte_off, unsigned lds_byte_addr) {
  unsigned long long saved;
  asm volatile("s_mov_b32 m0, %3\n\ts_and_saveexec_b64 %0, %4\n\tglobal_load_lds_dwordx4 %1, %2\n\ts_mov_b64 exec, %0"
               : "=&s"(saved)
               : "v"(lane_byte_off), "s"(uniform_base), "s"(lds_byte_addr), "s"(on_mask)
               : "memory", "m0", "scc");
}

// One piece of work: the queries of row tile pc.qt of kv head pc.g against key tiles [pc.jt0, pc.jt1).
// pc.slot < 0: the piece covers all the keys the tile needs, O / l goes to a.out.  Otherwise the
// un-normalised state (O, m, l per lane) goes to the piece's partial-result slot of group x, and the piece
// of the unit that gets there last merges all of them (in a fixed order, so that the result does not depend
// on which one that was) and writes the output.
template <int D>
__device__ __forceinline__ void attend(const AttnArgs& a, u32x4* smem, int* last_flag, const int x, const Piece& pc
#ifdef KVRA_TRACE
                                       , unsigned long long* trace_rec
#endif
                                       ) {
  const int g = pc.g, qt = pc.qt, jt0 = pc.jt0, jt1 = pc.jt1;
  constexpr int BN = key_tile(D);
  constexpr int MB = BN / 32;              // 32-key blocks of a tile
  constexpr int CPR = D / 8;               // 16-byte pieces per K/V row
  constexpr int KS = D / 16;               // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;               // 32-row blocks of O^T
  constexpr int RPB = 256 / (D * 2);       // rows per 256-byte LDS bank span
  constexpr int TILE = BN * CPR;           // 16-byte pieces per tile
  constexpr int LOADS = TILE / kThreads;   // pieces each thread moves per tile
  constexpr int PF = 4;                    // LDS operand reads kept in flight ahead of the MFMAs
  // One workgroup barrier per tile step instead of two (see "Schedule" at the top of the file).
  constexpr bool ONE_BARRIER = one_barrier(D);
  static_assert(TILE % kThreads == 0, "tile must split evenly over the workgroup");

  // smem: K ring then V ring, kStages tiles each
  auto ldsK = [&](int b) -> u32x4* { return smem + b * TILE; };
  auto ldsV = [&](int b) -> u32x4* { return smem + (kStages + b) * TILE; };

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction
  const int n = lane & 31, kg = lane >> 5;
  const int phase = wave >> 2;             // 0: first group, 1: second group (one barrier late)

  const int VR = a.chunk * a.G;            // virtual rows of this kv head
  const int total = a.prefix + a.chunk;    // valid cache rows
  const int row_lo = qt * a.rows_per_wg;
  const int row_hi = min(row_lo + a.rows_per_wg, VR);   // exclusive
  const int v0 = row_lo + wave * 32;
  const bool wave_active = v0 < row_hi;
  int vr = v0 + n;
  const bool row_valid = vr < row_hi;
  if (!row_valid) vr = row_hi - 1;
  const int r = vr / a.G;
  const int h = g * a.G + (vr - r * a.G);
  const int qpos = a.prefix + r;
  const int wmin = a.prefix + min(v0, row_hi - 1) / a.G;        // wave-uniform
  const int wmax = a.prefix + min(v0 + 31, row_hi - 1) / a.G;   // wave-uniform
  const int nt = jt1 - jt0;                                     // key tiles this fragment walks
  // key tiles of the fragment this wave needs (its rows see keys up to wmax)
  const int jw = wave_active ? min(max(wmax / BN + 1 - jt0, 0), nt) : 0;

  // Q fragment: B operand of S^T, lane (n, kg) holds Q[row n][16 ks + 8 kg .. +7], times
  // scale * log2(e) (rounded to bf16 again)
  bf16x8 qf[KS];
  {
    const __bf16* qrow = a.q + (static_cast<long long>(r) * a.H + h) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const bf16x8 raw = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * kg);
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[ks][e] = static_cast<__bf16>(static_cast<float>(raw[e]) * a.c_log2);
    }
  }

  // ---- global -> LDS staging of K/V tiles (LDS-direct loads, no registers in between) ---------
  // One wave instruction moves 64 x 16 bytes into 1 KiB of consecutive LDS; lane l lands at
  // base + 16 l.  Piece p of a tile = (row p / CPR, slot p % CPR); the XOR swizzles that keep the
  // MFMA operand reads free of bank conflicts are applied on the global side: the lane that owns
  // slot (row, slot) fetches column piece  slot ^ f(row)  of that row.
  //   K is read 16 bytes per lane down 16+ consecutive rows of one column piece;
  //   V is read (transposing) 8 bytes per lane over 4 consecutive rows x 64 bytes.
  int ld_row[LOADS];
  unsigned ld_kcc[LOADS], ld_vcc[LOADS], koff[LOADS], voff[LOADS];
  const unsigned row_stride = static_cast<unsigned>(a.Hkv) * D;   // elements between cache rows
#pragma unroll
  for (int i = 0; i < LOADS; ++i) {
    const int p = (i * kWaves + wave) * 64 + lane;
    ld_row[i] = p / CPR;
    const int slot = p % CPR;
    ld_kcc[i] = static_cast<unsigned>(slot ^ ((ld_row[i] / RPB) % CPR)) * 8;
    ld_vcc[i] = static_cast<unsigned>(slot ^ (4 * ((ld_row[i] / RPB) % (D / 32)))) * 8;
    koff[i] = 2u * (static_cast<unsigned>(ld_row[i]) * row_stride + ld_kcc[i]);   // bytes
    voff[i] = 2u * (static_cast<unsigned>(ld_row[i]) * row_stride + ld_vcc[i]);
  }
  // offsets for the one tile that straddles the end of the cache: rows past the end repeat the last valid row
  unsigned koff_last[LOADS], voff_last[LOADS];
  {
    const int lim_last = (total - 1) % BN;
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      koff_last[i] = 2u * (static_cast<unsigned>(min(ld_row[i], lim_last)) * row_stride + ld_kcc[i]);
      voff_last[i] = 2u * (static_cast<unsigned>(min(ld_row[i], lim_last)) * row_stride + ld_vcc[i]);
    }
  }
  const __bf16* kbase = a.k + static_cast<long long>(g) * D;
  const __bf16* vbase = a.v + static_cast<long long>(g) * D;

  // tile kt of K (or V) -> ring slot buf; rows past the end of the cache repeat the last valid row
  auto dma_tile = [&](const __bf16* head_base, const unsigned (&off)[LOADS], const unsigned (&cc)[LOADS],
                      int kt, u32x4* dst) {
    const __bf16* base = head_base + static_cast<long long>(jt0 + kt) * BN * row_stride;
    const int lim = total - 1 - (jt0 + kt) * BN;
    if (lim >= BN - 1) {   // whole tile inside the cache: the precomputed offsets (a real branch, wave-uniform)
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
            (lds_void*)(dst + (i * kWaves + wave) * 64)));
        lds_dma16(base, off[i], lds_addr);
      }
    } else {
#pragma unroll
      for (int i = 0; i < LOADS; ++i) {
        const unsigned o32 = 2u * (static_cast<unsigned>(min(ld_row[i], lim)) * row_stride + cc[i]);
        const unsigned lds_addr = static_cast<unsigned>(reinterpret_cast<uintptr_t>(
            (lds_void*)(dst + (i * kWaves + wave) * 64)));
        lds_dma16(base, o32, lds_addr);
      }
    }
  };
  // staging step s moves K tile s+1 and V tile s; returns the number of loads it issued
  auto stage = [&](int s) -> int {
    int cnt = 0;
    if (s + 1 < nt) { dma_tile(kbase, koff, ld_kcc, s + 1, ldsK((s + 1) % kStages)); cnt += LOADS; }
    if (s < nt) { dma_tile(vbase, voff, ld_vcc, s, ldsV(s % kStages)); cnt += LOADS; }
    return cnt;
  };

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
  // exponent reference of the row (in base-2 score units); trails the running max by a bounded
  // amount (see kSumLimit).  kNoKeyYet marks a row that has not met a visible key yet (possible
  // when a fragment starts beyond the row's last key): its scores are formed against 0 and its
  // first visible keys send the wave through the exact path, which sets the reference.
  float m = kNoKeyYet;
  float l = 0.0f;        // running row sum of this lane's half of the keys
  // start value of the score accumulators: minus the exponent reference (0 while the row has none),
  // so that the MFMAs deliver  s c - m  directly (c is folded into the Q fragment)
  f32x16 sref;
#pragma unroll
  for (int e = 0; e < 16; ++e) sref[e] = 0.0f;

  // lane-constant parts of the LDS read addresses
  const int k_sw = (n / RPB) % CPR;                       // K swizzle of row 32 mb + n
  const int vi = lane & 15, vmh = (lane >> 4) & 1;        // position inside the 16-lane transpose block
  const int v_row0 = 4 * kg + (vi >> 2);                  // + 32 mb + 16 s + 8 e
  const int v_sw = 4 * ((v_row0 / RPB) % (D / 32));
  const int v_cc0 = 2 * vmh + ((vi & 3) >> 1);            // + 4 db
  const int v_sub = (vi & 1) * 4;                         // element offset inside the 16-byte piece

  // Staging state of the tile loop.  At tile step j this wave (st = j + phase) sends off its pieces of
  // K tile st + 2 and V tile st + 1: two running pointers, advanced by one tile per step, and the
  // LDS byte addresses of the ring slots in the order this wave meets them (slot_k[r] is where the K
  // tile goes at a step with j % kStages == r; the V tile of that step goes to slot_v[r]).
  const long long tile_elems = static_cast<long long>(BN) * row_stride;
  const __bf16* kp = kbase + (jt0 + 2 + phase) * tile_elems;
  const __bf16* vp = vbase + (jt0 + 1 + phase) * tile_elems;
  const int kt_ragged = (total % BN != 0) ? (total - 1) / BN - jt0 : -1;   // the tile that straddles the end
  unsigned slot_k[kStages], slot_v[kStages];
#pragma unroll
  for (int r = 0; r < kStages; ++r) {
    slot_k[r] = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)(ldsK((r + 2 + phase) % kStages) + wave * 64)));
    slot_v[r] = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)(ldsV((r + 1 + phase) % kStages) + wave * 64)));
  }

  // ---- prologue: K tiles 0..2 and V tiles 0..1 on their way into LDS -----------------------------
  // the first MFMA block multiplies a zero P by the ring slot "before" V tile 0: make it finite
  for (int i = tid; i < TILE; i += kThreads) ldsV(kStages - 1)[i] = u32x4{0u, 0u, 0u, 0u};
  dma_tile(kbase, koff, ld_kcc, 0, ldsK(0));
  stage(0);
  stage(1);
  // every load so far (the Q fragment included) is drained here: a load left pending across the
  // loop entry would make the compiler guard the loop's MFMAs with vmcnt waits
  __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0)
  __syncthreads();
  if (!ONE_BARRIER && phase == 1) __syncthreads();   // second group runs one barrier behind the first
  KVRA_TRACE_STAMP(trace_rec, 1);

  f32x16 s[MB];
  bf16x8 pf[MB][2];
#pragma unroll
  for (int mb = 0; mb < MB; ++mb)
#pragma unroll
    for (int si = 0; si < 2; ++si)
#pragma unroll
      for (int e = 0; e < 8; ++e) pf[mb][si][e] = static_cast<__bf16>(0.0f);

  // steps whose staging needs no bookkeeping (see the VALU block): K tile st + 2 and V tile st + 1 both exist
  // and neither straddles the end of the cache
  const int bulk_lo = 1 - phase;
  const int bulk_hi = min(nt - 2, kt_ragged >= 0 ? kt_ragged - 2 : nt) - phase;

  // One tile step; RS = j % kStages is a compile-time value so that every LDS operand address is
  // a loop-invariant per-lane register plus an immediate.
  auto tile_step = [&](const int j, auto rs_tag) {
    constexpr int RS = decltype(rs_tag)::value;
    // ================= MFMA block =================
    // P.V of tile j-1 followed by K.Q^T of tile j as ONE software-pipelined stream of operand reads
    // and MFMAs: the LDS read of op i + PF is issued before the MFMA of op i, and the compiler is
    // told not to move anything across the steps.  The block runs whole for j <= jw: at j = 0 the
    // P fragment is zero and the "previous" V slot was zero-filled, at j = jw the scores it forms
    // are never looked at (the price is one tile's worth of MFMAs per wave, the gain is a single
    // straight-line block).
    if (j <= jw) {
      const short* Vb = reinterpret_cast<const short*>(ldsV((RS + kStages - 1) % kStages));
      const bf16x8* Kb = reinterpret_cast<const bf16x8*>(ldsK(RS));
      // contraction slot 4e + t of P.V step (mb, si) is key 32 mb + 16 si + 8 e + 4 kg + t on both operands
      auto vread = [&](int idx) -> bf16x8 {
        const int mb = idx / (2 * DB), si = (idx / DB) % 2, db = idx % DB;
        s16x8 vf;
#pragma unroll
        for (int e = 0; e < 2; ++e) {
          const int row = 32 * mb + 16 * si + 8 * e + v_row0;
          const int slot = (4 * db + v_cc0) ^ v_sw;
          const short* p = Vb + (row * CPR + slot) * 8 + v_sub;
          const s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
          vf[4 * e + 0] = t[0]; vf[4 * e + 1] = t[1]; vf[4 * e + 2] = t[2]; vf[4 * e + 3] = t[3];
        }
        return __builtin_bit_cast(bf16x8, vf);
      };
      auto kread = [&](int idx) -> bf16x8 {
        const int ks = idx / MB, mb = idx % MB;
        return Kb[(32 * mb + n) * CPR + ((2 * ks + kg) ^ k_sw)];
      };
      constexpr int N0 = 2 * MB * DB, N = N0 + MB * KS;
      auto frag = [&](int i) -> bf16x8 { return (i < N0) ? vread(i) : kread(i - N0); };
      bf16x8 fq[PF];
#pragma unroll
      for (int i = 0; i < PF; ++i) fq[i] = frag(i);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < N; ++i) {
        const bf16x8 cur = fq[i % PF];
        if (i + PF < N) fq[i % PF] = frag(i + PF);
        if (i < N0) {
          const int mb = i / (2 * DB), si = (i / DB) % 2, db = i % DB;
          o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, pf[mb][si], o[db], 0, 0, 0);
        } else
        {
          const int q = i - N0;
          s[q % MB] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(cur, qf[q / MB], q < MB ? sref : s[q % MB], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    if (!ONE_BARRIER || phase == 1) __syncthreads();

    // ================= VALU block =================
    // staging: this wave's step is j + phase (the late group is one tile ahead in tile numbers);
    // tiles K(st+2), V(st+1) start their trip now and are awaited one period later
    const int st = j + phase;
    // The 2 LOADS loads are handed out one at a time and spread over the softmax below.  A tile
    // beyond the fragment is "loaded" with no lane enabled: no branch, so the loads can sit in
    // straight-line code.  The ragged last tile of the cache takes the clamped offsets.
    // At head_dim 64, where this block is the longer of the two, only the steps near either end of the piece
    // work any of this out: in the bulk of the steps, [bulk_lo, bulk_hi), both tiles exist and neither is
    // the ragged one (a wave-uniform branch around scalar work: every scalar instruction of this block is
    // issue time the matrix pipe waits for; measured +1.5 % at head_dim 64, -1 % at 128, where it stays out).
    bool k_on = true, v_on = true, k_rag = false, v_rag = false;
    if (D != 64 || j < bulk_lo || j >= bulk_hi) {
      k_on = st >= 1 && st + 2 < nt;
      v_on = st >= 1 && st + 1 < nt;
      k_rag = st + 2 == kt_ragged;
      v_rag = st + 1 == kt_ragged;
    }
    const int issued = (k_on ? LOADS : 0) + (v_on ? LOADS : 0);
    const unsigned long long k_mask = __builtin_amdgcn_ballot_w64(k_on), v_mask = __builtin_amdgcn_ballot_w64(v_on);
    auto stage_piece = [&](int idx) __attribute__((always_inline)) {
      __builtin_amdgcn_sched_barrier(0);
      if (idx < LOADS)
        lds_dma16_if(k_mask, kp, k_rag ? koff_last[idx] : koff[idx], slot_k[RS] + idx * (kWaves * 64 * 16));
      else
        lds_dma16_if(v_mask, vp, v_rag ? voff_last[idx - LOADS] : voff[idx - LOADS],
                     slot_v[RS] + (idx - LOADS) * (kWaves * 64 * 16));
      __builtin_amdgcn_sched_barrier(0);
    };
    if (j >= jw) {
#pragma unroll
      for (int idx = 0; idx < 2 * LOADS; ++idx) stage_piece(idx);
    }
    if (j < jw) {
      // register e of block mb is key  j*BN + 32 mb + 8 (e/4) + 4 kg + e%4  of query n
      if ((jt0 + j) * BN + BN - 1 > wmin) {
        int rel = qpos - (jt0 + j) * BN - 4 * kg;   // largest still-visible key offset (minus 4 kg)
        // opaque to the optimiser: otherwise the 32 compares below become 32 loop-carried
        // counters that are kept up to date (and kept in registers) on every tile
        asm volatile("" : "+v"(rel));
        const float ninf = -INFINITY;
        // compare and select one element at a time through vcc (written out: left to itself the
        // compiler keeps all 32 lane masks alive in scalar registers, which spills others)
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            float x = s[mb][e];
            asm volatile("v_cmp_gt_i32 vcc, %1, %2\n\tv_cndmask_b32 %0, %0, %3, vcc"
                         : "+v"(x)
                         : "n"(32 * mb + 8 * (e / 4) + (e % 4)), "v"(rel), "v"(ninf)
                         : "vcc");
            s[mb][e] = x;
          }
      }
      // ---- online softmax (base 2) with a lazily moved exponent reference -------------------
      // weights of this tile: p = exp2(s) against the reference in force (MOVED: exp2(s - delta)
      // against one that was just raised by delta), rounded to bf16 in pairs for the P.V product;
      // the row sum adds the unrounded values.  Returns this lane's part of the row sum.  The first
      // pass also carries the staging loads, one every few exponentials.
      auto weights = [&](auto moved_tag, const float delta) __attribute__((always_inline)) -> float {
        constexpr bool MOVED = decltype(moved_tag)::value;
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        float sum0 = 0.0f, sum1 = 0.0f;
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int e = 0; e < 16; e += 2) {
            if constexpr (!MOVED) {
              constexpr int PAIRS = MB * 8, EVERY = PAIRS / (2 * LOADS);
              const int pair = mb * 8 + e / 2;
              if (pair % EVERY == 0) stage_piece(pair / EVERY);
            }
            const float p0 = __builtin_amdgcn_exp2f(MOVED ? s[mb][e] - delta : s[mb][e]);
            const float p1 = __builtin_amdgcn_exp2f(MOVED ? s[mb][e + 1] - delta : s[mb][e + 1]);
            const bf16x2 pp = {static_cast<__bf16>(p0), static_cast<__bf16>(p1)};
            if ((e / 2) % 2) sum1 += p0 + p1;
            else sum0 += p0 + p1;
            pf[mb][e / 8][e % 8] = pp[0];
            pf[mb][e / 8][e % 8 + 1] = pp[1];
          }
        return sum0 + sum1;
      };
      // Optimistic pass: no row maximum is formed.  As long as the scores stay within reach of m the
      // weights are modest; a lane whose partial sum gets out of hand, or whose row has no reference
      // yet, sends the whole wave through the exact path: row maximum, m, l, O and the accumulator
      // start value re-based to it, weights formed again.
      float psum = weights(std::false_type{}, 0.0f);
      const bool unset = m == kNoKeyYet;
      if (__builtin_amdgcn_ballot_w64(!(psum < kSumLimit) || unset) != 0) {
        float tmax = s[0][0];   // relative to the reference in force
#pragma unroll
        for (int mb = 0; mb < MB; ++mb)
#pragma unroll
          for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[mb][e]);
        tmax = fmaxf(tmax, other_half(tmax));
        // a row without reference takes its maximum as one, once it has met a visible key
        const bool seen = tmax > -INFINITY;
        const float delta = unset ? (seen ? tmax : 0.0f) : fmaxf(tmax, 0.0f);
        const float alpha = unset ? 1.0f : __builtin_amdgcn_exp2f(-delta);
        if (unset) { if (seen) m = tmax; }
        else m += delta;
        l *= alpha;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
#pragma unroll
        for (int e = 0; e < 16; ++e) sref[e] -= delta;
        psum = weights(std::true_type{}, delta);
      }
      l += psum;
    }
    kp += tile_elems;
    vp += tile_elems;
    // everything issued before this block (tiles K(st+1), V(st)) must have landed before the barrier
    if (issued == 2 * LOADS) __builtin_amdgcn_s_waitcnt(0x0F70 | (2 * LOADS));
    else if (issued == LOADS) __builtin_amdgcn_s_waitcnt(0x0F70 | LOADS);
    else __builtin_amdgcn_s_waitcnt(0x0F70);
    if (!ONE_BARRIER || phase == 0) __syncthreads();
  };
  for (int j0 = 0; j0 <= nt; j0 += kStages) {
    tile_step(j0, std::integral_constant<int, 0>{});
    if (j0 + 1 <= nt) tile_step(j0 + 1, std::integral_constant<int, 1>{});
    if (j0 + 2 <= nt) tile_step(j0 + 2, std::integral_constant<int, 2>{});
  }
  static_assert(kStages == 3, "the unrolled loop above is written for a ring of three");
  if (!ONE_BARRIER && phase == 0) __syncthreads();   // both groups execute the same number of barriers
  KVRA_TRACE_STAMP(trace_rec, 2);

  // ---- epilogue: O / l, bf16, store -----------------------------------------------------------
  if (pc.slot >= 0) {
    // [wave][register][lane]: every store is 256 consecutive bytes per wave.  The pieces of a unit are
    // handed from workgroup to workgroup without a fence (a device-scope fence writes back and invalidates
    // the whole L2 of the XCD: tens of microseconds, and the K/V stream the other workgroups share is
    // gone): the partial results are written with device-coherent stores, the wave waits until all of
    // them have been acknowledged, and only then, after a workgroup barrier, are the unit's key tiles
    // added to its counter; the piece that completes the count reads the others with device-coherent loads.
    constexpr int WAVE_FLOATS = (DB * 16 + 2) * 64;
    float* group_slots = a.scratch + static_cast<long long>(x) * slots_per_group(a) * kPartialFloats(D);
    int* counter = a.counters + x * kMaxSlots + pc.seg;
    // A piece looks at the unit's counter first: if every other piece has already been counted, it is the
    // one that merges, nobody will read its partial result, and the store and the wait for it are left out
    // (in a unit of two pieces, whichever comes second).  The others' results are visible then: each was
    // acknowledged before its count was added.  A look that comes too early only costs the round trip.
    bool all_others_counted = false;
    {
      if (tid == 0) {
        const int seen = __hip_atomic_load(counter, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        *last_flag = (seen + nt == pc.n) ? 1 : 0;
      }
      __syncthreads();
      all_others_counted = *last_flag != 0;
      __syncthreads();                     // the flag is written again below
    }
    if (!all_others_counted) {
      float* p = group_slots + static_cast<long long>(pc.slot) * kPartialFloats(D) + wave * WAVE_FLOATS + lane;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) store_coherent(p + (db * 16 + e) * 64, o[db][e]);
      store_coherent(p + (DB * 16) * 64, m);
      store_coherent(p + (DB * 16 + 1) * 64, l);
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      if (tid == 0) {
        const int before = atomicAdd(counter, nt);
        *last_flag = (before + nt == pc.n) ? 1 : 0;
      }
      __syncthreads();
      const bool last = *last_flag != 0;
      __syncthreads();                     // the flag may be rewritten by the next piece
      if (!last) return;
    }
    if (tid == 0) *counter = 0;            // ready for the next launch
    // The unit's pieces in their fixed order (the head if the segment is the tail of a cut unit, then the
    // slots whose share of the line of segments meets it), merged one after the other into (O, m, l)
    // starting from nothing: the result does not depend on which piece happened to be the last.
    // Which slots: every lane tests four slots of the table, the wave votes.
    // This piece's own partial result is not read back: what it stored is what its registers hold, so taking
    // it from there when its turn in the order comes gives the same bits and saves one of the unit's reads.
    const float* mine = group_slots + wave * WAVE_FLOATS + lane;
    f32x16 own_o[DB];
#pragma unroll
    for (int db = 0; db < DB; ++db) own_o[db] = o[db];
    const float own_m = m, own_l = l;
    m = kNoKeyYet;
    l = 0.0f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
    auto merge_in = [&](int slot) {
      const float* p = mine + static_cast<long long>(slot) * kPartialFloats(D);
      float po[DB * 16];
      float pm, pl;
      if (slot == pc.slot) {
#pragma unroll
        for (int i = 0; i < DB * 16; ++i) po[i] = own_o[i / 16][i % 16];
        pm = own_m;
        pl = own_l;
      } else {
#pragma unroll
        for (int i = 0; i < DB * 16; ++i) po[i] = load_coherent(p + i * 64);
        pm = load_coherent(p + (DB * 16) * 64);
        pl = load_coherent(p + (DB * 16 + 1) * 64);
      }
      const float mn = fmaxf(m, pm);
      const float wa = __builtin_amdgcn_exp2f(m - mn), wb = __builtin_amdgcn_exp2f(pm - mn);
      m = mn;
      l = fmaf(pl, wb, l * wa);
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] = fmaf(po[db * 16 + e], wb, o[db][e] * wa);
    };
    if (pc.seg < a.cut) merge_in(a.slots + a.segments + seg_to_unit(a, pc.seg));
    static_assert(kMaxSlots <= 256, "four votes of 64 lanes cover the table");
    for (int k = 0; k < 4; ++k) {
      const int c = 64 * k + lane;
      bool meets = false;
      if (c < a.slots) {
        const unsigned s0 = a.fill_seg[c], o0 = a.fill_off[c], s1 = a.fill_seg[c + 1], o1 = a.fill_off[c + 1];
        const bool nonempty = s0 < s1 || (s0 == s1 && o0 < o1);
        meets = nonempty && static_cast<int>(s0) <= pc.seg &&
                (static_cast<int>(s1) > pc.seg || (static_cast<int>(s1) == pc.seg && o1 > 0));
      }
      unsigned long long votes = __builtin_amdgcn_ballot_w64(meets);
      while (votes != 0) {
        const int c_meet = 64 * k + __builtin_ctzll(votes);
        votes &= votes - 1;
        merge_in(c_meet + pc.seg);
      }
      if (64 * (k + 1) >= a.slots) break;
    }
  }
  const float lsum = l + other_half(l);
  if (wave_active && row_valid) {
    const float inv = 1.0f / lsum;
    __bf16* orow = a.out + (static_cast<long long>(r) * a.H + h) * D;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 w;
#pragma unroll
        for (int t = 0; t < 4; ++t) w[t] = static_cast<__bf16>(o[db][4 * r4 + t] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * r4 + 4 * kg) = w;
      }
  }
}

// Persistent workgroups: workgroup id -> (group x, slot c); the slot walks its pieces in the order of the
// schedule (whole units of the complete rounds, or the head of its own unit; then its share of the line
// of segments).
template <int D>
__global__ __launch_bounds__(kThreads, 1) void chunk_attn_kernel(AttnArgs a) {
#ifdef KVRA_TRACE
  const unsigned long long t_entry = wall_clock64();   // before the first read of the arguments
#endif
  extern __shared__ u32x4 smem[];
  __shared__ int last_flag;
  const int x = blockIdx.x % a.groups, c = blockIdx.x / a.groups;
  PieceWalker walker(a, x, c);
#ifdef KVRA_TRACE
  int ordinal = 0;
#endif
  Piece pc;
  while (walker.next(a, &pc)) {
#ifdef KVRA_TRACE
    unsigned long long* rec = (a.trace != nullptr && ordinal < kTracePieces)
        ? a.trace + (static_cast<long long>(blockIdx.x) * kTracePieces + ordinal) * kTraceWords : nullptr;
    ++ordinal;
    KVRA_TRACE_STAMP(rec, 0);
    attend<D>(a, smem, &last_flag, x, pc, rec);
    KVRA_TRACE_STAMP(rec, 3);
    if (rec != nullptr && threadIdx.x == 0) {
      unsigned hw, xcc;
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_HW_ID)" : "=s"(hw));
      asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
      rec[4] = (static_cast<unsigned long long>(xcc) << 32) | hw;
      // tile steps; for the workgroup's first piece also the time from kernel entry to the piece's start
      // (reading the arguments and the schedule tables), in clock ticks, in the upper half
      rec[5] = static_cast<unsigned long long>(pc.jt1 - pc.jt0) | (ordinal == 1 ? (rec[0] - t_entry) << 32 : 0ull);
      rec[6] = (static_cast<unsigned long long>(static_cast<unsigned>(pc.g)) << 32) | static_cast<unsigned>(pc.qt);
      rec[7] = (static_cast<unsigned long long>(static_cast<unsigned>(pc.slot + 1)) << 32) | static_cast<unsigned>(pc.jt0);
    }
#else
    attend<D>(a, smem, &last_flag, x, pc);
#endif
  }
}

namespace {

// Scratch of the merge path: partial-result slots (three per CU cover every schedule: a group touches at
// most slots + 2 * segments of them, segments < slots) followed by the merge counters.  The allocated one
// is per device, taken on first use and kept until the process ends.
constexpr int kSlotsPerCu = 3;
constexpr int kCounterInts = 8 * kMaxSlots;
constexpr int kMaxDevices = 16;
float* g_scratch[kMaxDevices] = {};
int g_cus[kMaxDevices] = {};
std::mutex g_scratch_mutex;

// Compute units of the current device (0 if it cannot be asked); cached per device.
int device_cus(int dev) {
  if (g_cus[dev] == 0) {
    int cus = 0;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus >= 8) g_cus[dev] = cus;
  }
  return g_cus[dev];
}

// The allocated scratch of the current device, or nullptr (the caller then launches without cutting
// units).  A failed attempt is not remembered: a call made while `stream` is being captured (an
// allocation would be illegal there) or while memory is short runs uncut, and a later call tries again.
float* device_scratch(hipStream_t stream, int* cus_out, int64_t* slots_out) {
  *cus_out = 0;
  *slots_out = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  const int cus = device_cus(dev);
  *cus_out = cus;
  if (cus <= 0) return nullptr;
  const int64_t slots = static_cast<int64_t>(kSlotsPerCu) * cus;
  *slots_out = slots;
  if (g_scratch[dev] == nullptr) {
    hipStreamCaptureStatus capturing = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(stream, &capturing) != hipSuccess) {
      (void)hipGetLastError();
      return nullptr;
    }
    if (capturing != hipStreamCaptureStatusNone) return nullptr;
    const size_t slot_bytes = static_cast<size_t>(slots) * kPartialFloats(128) * sizeof(float);
    void* p = nullptr;
    if (hipMalloc(&p, slot_bytes + kCounterInts * sizeof(int)) != hipSuccess) {
      (void)hipGetLastError();   // leave no sticky error behind; the uncut launch needs no scratch
      return nullptr;
    }
    // the counters start at zero and every merge puts its counter back to zero
    if (hipMemset(static_cast<char*>(p) + slot_bytes, 0, kCounterInts * sizeof(int)) != hipSuccess) {
      (void)hipGetLastError();
      (void)hipFree(p);
      return nullptr;
    }
    g_scratch[dev] = static_cast<float*>(p);
  }
  return g_scratch[dev];
}

}  // namespace

// ---- scratch of kvra_chunk_attn_noalloc: a fixed array in the library's device image ------------
// kStaticSlots partial-result slots = 3 per CU of a 256-CU device (what the allocating path takes
// there, so that both entry points cut a launch the same way), then the merge counters (zero like
// every static array, and put back to zero by every merge).  Every device the library runs on
// holds its own copy at its own address for the life of the process.  In host code the array's
// name is only a handle for hipGetSymbolAddress: the device address is asked for once per device,
// with that device current, and that pointer is what the kernels get.
constexpr int kStaticSlots = 768;
static __device__ __align__(256) float scratch[static_cast<size_t>(kStaticSlots) * kPartialFloats(128) + kCounterInts];

namespace {

float* g_static_scratch[kMaxDevices] = {};

// Device address of `scratch` on the current device (nullptr on failure); no allocation.
float* static_scratch(int* cus_out) {
  *cus_out = 0;
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  *cus_out = device_cus(dev);
  if (g_static_scratch[dev] == nullptr) {
    void* p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) {
      (void)hipGetLastError();
      return nullptr;
    }
    g_static_scratch[dev] = static_cast<float*>(p);
  }
  return g_static_scratch[dev];
}

// ---- the schedule (host arithmetic) --------------------------------------------------------------
#ifndef KVRA_ALLOWANCE
#define KVRA_ALLOWANCE 8
#endif
#ifndef KVRA_MINPIECE
#define KVRA_MINPIECE 8
#endif
#ifndef KVRA_CUT_ROUNDS
#define KVRA_CUT_ROUNDS 1
#endif
constexpr int kPieceAllowance = KVRA_ALLOWANCE;   // what starting and finishing a piece costs, in tile steps
constexpr int kMinPiece = KVRA_MINPIECE;          // no piece shorter than this many tile steps is cut off a unit
#ifndef KVRA_GANG_SLACK
#define KVRA_GANG_SLACK 110
#endif
constexpr int kGangSlackPercent = KVRA_GANG_SLACK;   // gang mode may finish this much later (percent of the evenly shared plan); 0 = never

// Shares the line of segments out to the slots so that every slot's load (what it already has plus its
// share plus one allowance per share) stays within `target`; returns whether the whole line was placed.
// seg_len[s]: length of segment s, the first cut_tails of them tails of cut units; load[c]: tile steps
// (with allowances) slot c runs before its share.
// Cuts never leave less than kMinPiece steps of a segment on either side; with whole_segments_only no
// segment is cut at all.
bool share_out(const std::vector<int>& seg_len, const std::vector<int64_t>& load, int64_t target,
               bool whole_segments_only, int cut_tails, unsigned* fill_seg, unsigned* fill_off, int* partial_pieces) {
  const int P = static_cast<int>(load.size()), S = static_cast<int>(seg_len.size());
  int seg = 0, off = 0, partial = 0;
  for (int c = 0; c < P; ++c) {
    fill_seg[c] = static_cast<unsigned>(seg);
    fill_off[c] = static_cast<unsigned>(off);
    int64_t room = target - load[c];
    while (seg < S) {
      room -= kPieceAllowance;                       // every piece of the share pays the allowance
      if (room <= 0) break;
      const int left = seg_len[seg] - off;           // what is left of this segment
      if (room >= left || (!whole_segments_only && left - room < kMinPiece && room + kMinPiece > left)) {
        // take the rest of the segment (going over the target by less than kMinPiece is allowed)
        if (off > 0 || seg < cut_tails) ++partial;   // (the tail of a cut unit is never a whole unit)
        room -= left;
        ++seg;
        off = 0;
      } else {
        if (whole_segments_only || room < kMinPiece) break;
        off += static_cast<int>(room);
        ++partial;
        break;
      }
    }
  }
  fill_seg[P] = static_cast<unsigned>(seg);
  fill_off[P] = static_cast<unsigned>(off);
  *partial_pieces = partial;
  return seg == S;
}

}  // namespace

int64_t attn_partial_bytes(int head_dim) {
  return static_cast<int64_t>(head_dim == 128 ? kPartialFloats(128) : kPartialFloats(64)) * sizeof(float);
}
int64_t attn_counter_bytes() { return static_cast<int64_t>(kCounterInts) * sizeof(int); }

int plan_chunk_attn(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                    int cus, bool scratch_available, AttnPlan* plan) {
  const int G = n_q_heads / n_kv_heads;
  const int64_t vrows = chunk_len * G;
  if (vrows > (int64_t(1) << 30) || prefix_len + chunk_len > (int64_t(1) << 30)) return KVRA_EUNSUPPORTED;
  // spread the 32-row wave slices evenly over the row tiles (e.g. 34 slices -> 5 tiles of 7)
  const int64_t slices = (vrows + 31) / 32;
  const int64_t tiles = (slices + kWaves - 1) / kWaves;
  const int64_t slices_per_tile = (slices + tiles - 1) / tiles;
  if (tiles * n_kv_heads > 0x3FFFFFFF) return KVRA_EUNSUPPORTED;
  const int bn = key_tile(head_dim);
  const int rows_per_tile = static_cast<int>(32 * slices_per_tile);
  const int R = static_cast<int>(tiles);
  if (cus < 1) cus = 1;
  const int groups = (n_kv_heads % 8 == 0 && cus % 8 == 0) ? 8 : 1;
  const int P = std::min(cus / groups, kMaxSlots);
  const int hp = n_kv_heads / groups;
  const int64_t U64 = static_cast<int64_t>(R) * hp;
  const int U = static_cast<int>(U64);
  auto steps_of_tile = [&](int qt) -> int {
    const int64_t row_hi = std::min<int64_t>(static_cast<int64_t>(qt + 1) * rows_per_tile, vrows);
    return static_cast<int>((prefix_len + (row_hi - 1) / G) / bn + 1);
  };
  auto steps_of_unit = [&](int j) -> int { return steps_of_tile(R - 1 - j / hp); };

  plan->row_tiles = R;
  plan->rows_per_tile = rows_per_tile;
  plan->key_tile = bn;
  plan->groups = groups;
  plan->slots = P;
  plan->units = U;
  plan->rounds = U / P;
  std::vector<int> n(U);
  for (int j = 0; j < U; ++j) n[j] = steps_of_unit(j);
  const int first_round = std::min(U, P);         // units of the first round: unit c on slot c
  // Cutting the first round's units pays while a slot runs at most one more unit after it; with more
  // rounds the reverse order of every second round evens the loads out and the leftover units do the rest.
  const bool may_cut = scratch_available && plan->rounds <= KVRA_CUT_ROUNDS && n[0] >= 2 * kMinPiece;
  // load of every slot from the rounds after the first (every second round in reverse slot order)
  std::vector<int64_t> later(P, 0), load(P, 0);
  for (int k = 1; k < plan->rounds; ++k)
    for (int c = 0; c < P; ++c) later[c] += n[k * P + ((k & 1) ? P - 1 - c : c)] + kPieceAllowance;
  std::vector<int> seg_len;
  int partial = 0, cut = 0;
  // For a finishing time `target`: cut the first round's units at head = target - allowance (if allowed),
  // line up their tails and the leftover units, share the line out; true if everything fits.
  auto fits = [&](int64_t target) -> bool {
    const int64_t head = target - kPieceAllowance;
    seg_len.clear();
    cut = 0;
    if (may_cut)
      while (cut < first_round && n[cut] >= head + kMinPiece && head >= kMinPiece) {
        seg_len.push_back(n[cut] - static_cast<int>(head));
        ++cut;
      }
    for (int j = std::max(plan->rounds, 1) * P; j < U; ++j) seg_len.push_back(n[j]);
    for (int c = 0; c < P; ++c)
      load[c] = later[c] + (c < first_round ? (c < cut ? head : n[c]) + kPieceAllowance : 0);
    // (a unit whose tail would be shorter than the minimum piece stays whole and may overshoot by that much)
    for (int c = 0; c < P; ++c)
      if (load[c] >= target + (c < first_round && may_cut ? kMinPiece : 1)) return false;
    return share_out(seg_len, load, target, !scratch_available, cut, plan->fill_seg, plan->fill_off, &partial);
  };
  int64_t total = 0;
  for (int j = 0; j < U; ++j) total += n[j] + kPieceAllowance;
  int64_t lo = 0, hi = total + kPieceAllowance + 1;           // everything on one slot: always enough
  while (lo + 1 < hi) {                                       // smallest finishing time that fits
    const int64_t mid = (lo + hi) / 2;
    if (fits(mid)) hi = mid;
    else lo = mid;
  }
  fits(hi);
  plan->head_steps = cut > 0 ? static_cast<int>(hi - kPieceAllowance) : 0;
  plan->cut = cut;
  plan->segments = static_cast<int>(seg_len.size());
  plan->steps_per_slot = static_cast<int>(hi);
  partial += cut;                                             // the heads of the cut units
  plan->partial_pieces = partial * groups;
  plan->scratch_slots = partial > 0 ? (P + 2 * plan->segments) * groups : 0;
  plan->gangs = 0;
  plan->gang_heads = 0;
  // Gang mode.  When the group has fewer units than slots, every unit is cut and at least one row tile's worth
  // of slots has no unit of its own, the tails can be run in step instead of being handed out piecemeal: the
  // free slots form gangs of R (one slot per row tile), a gang works through its heads one after the other,
  // and the R tails of a head then read the same keys at the same time, as the heads of the units do - their
  // K/V comes from HBM once instead of R times - and every such tail stays whole (two pieces per unit to
  // merge, no more).  Free slots that fit no gang take the tails of the heads the gangs leave over, shared out
  // evenly among them as before, or stay idle if the gangs take every head.  The price is balance (a gang slot
  // carries whole tails, idle slots carry nothing): the mode is taken while the common finishing time stays
  // within kGangSlack of the evenly shared plan's, with the number of gangs and of heads per gang slot that
  // finish earliest.
  if (may_cut && plan->rounds == 0 && U == R * hp && P - U >= R) {
    const int F = P - U;
    std::vector<int> spare_len;
    std::vector<int64_t> spare_load;
    std::vector<unsigned> sp_seg(kMaxSlots + 1), sp_off(kMaxSlots + 1);
    int spare_partial = 0;
    // smallest finishing time of ng gangs with k heads per gang slot (0: impossible); leaves the spare slots'
    // share tables in sp_seg / sp_off
    auto gang_target = [&](int ng, int k) -> int64_t {
      const int spare_heads = hp - ng * k, spare_slots = F - ng * R;
      if (spare_heads < 0 || (spare_heads > 0 && spare_slots < 1)) return 0;
      for (int64_t target = kMinPiece + kPieceAllowance; target <= n[0] + kPieceAllowance; ++target) {
        const int64_t head = target - kPieceAllowance;
        bool ok = head >= kMinPiece;
        for (int j = 0; ok && j < U; ++j) ok = n[j] >= head + kMinPiece;   // every unit cut, with a tail worth a piece
        for (int g = 0; ok && g < ng; ++g)
          for (int rank = 0; ok && rank < R; ++rank) {
            int64_t load = 0;
            for (int i = 0; i < k; ++i) load += n[rank * hp + g + ng * i] - head + kPieceAllowance;
            ok = load <= target;
          }
        if (ok && spare_heads > 0) {
          spare_len.clear();
          for (int h = ng * k; h < hp; ++h)
            for (int rank = 0; rank < R; ++rank) spare_len.push_back(n[rank * hp + h] - static_cast<int>(head));
          spare_load.assign(spare_slots, 0);
          ok = share_out(spare_len, spare_load, target, false, static_cast<int>(spare_len.size()), sp_seg.data(),
                         sp_off.data(), &spare_partial);
        }
        if (ok) return target;
      }
      return 0;
    };
    int best_ng = 0, best_k = 0;
    int64_t best_t = 0;
    for (int ng = std::min(F / R, hp); ng >= 1; --ng)
      for (int k = 1; ng * k <= hp; ++k) {
        const int64_t t = gang_target(ng, k);
        if (t > 0 && (best_t == 0 || t < best_t || (t == best_t && ng * k > best_ng * best_k))) {
          best_t = t;
          best_ng = ng;
          best_k = k;
        }
      }
    if (best_t > 0 && best_t * 100 <= static_cast<int64_t>(plan->steps_per_slot) * kGangSlackPercent) {
      const int ng = best_ng, k = best_k, gang_segments = ng * R * k, spare_slots = F - ng * R;
      spare_partial = 0;
      (void)gang_target(ng, k);                              // (fills the spare slots' tables again)
      plan->gangs = ng;
      plan->gang_heads = k;
      plan->head_steps = static_cast<int>(best_t - kPieceAllowance);
      plan->cut = U;
      plan->segments = U;
      plan->steps_per_slot = static_cast<int>(best_t);
      for (int c = 0; c <= P; ++c) {
        const int m = c - U;                                 // filler slot number: gang slots first, then spare ones
        if (m <= 0) {
          plan->fill_seg[c] = 0;
          plan->fill_off[c] = 0;
        } else if (m <= ng * R) {
          plan->fill_seg[c] = static_cast<unsigned>(m * k);
          plan->fill_off[c] = 0;
        } else if (ng * k < hp) {
          plan->fill_seg[c] = static_cast<unsigned>(gang_segments) + sp_seg[std::min(m - ng * R, spare_slots)];
          plan->fill_off[c] = sp_off[std::min(m - ng * R, spare_slots)];
        } else {
          plan->fill_seg[c] = static_cast<unsigned>(U);
          plan->fill_off[c] = 0;
        }
      }
      plan->partial_pieces = (U + gang_segments + (ng * k < hp ? spare_partial : 0)) * groups;
      plan->scratch_slots = (P + 2 * plan->segments) * groups;
    }
  }
  return KVRA_OK;
}

int64_t attn_static_scratch_bytes() { return static_cast<int64_t>(kStaticSlots) * kPartialFloats(128) * sizeof(float); }

#ifdef KVRA_TRACE
namespace {
unsigned long long* g_trace_buf = nullptr;
long long g_trace_groups = 0;
}  // namespace
#endif

namespace {

// The shape and schedule fields of the kernel arguments.
void schedule_args(const AttnPlan& plan, int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads,
                   AttnArgs* a) {
  a->prefix = static_cast<int>(prefix_len);
  a->chunk = static_cast<int>(chunk_len);
  a->H = n_q_heads;
  a->Hkv = n_kv_heads;
  a->G = n_q_heads / n_kv_heads;
  a->nq_tiles = plan.row_tiles;
  a->rows_per_wg = plan.rows_per_tile;
  a->bn = plan.key_tile;
  a->groups = plan.groups;
  a->slots = plan.slots;
  a->units = plan.units;
  a->rounds = plan.rounds;
  a->head_steps = plan.head_steps;
  a->cut = plan.cut;
  a->gangs = plan.gangs;
  a->gang_heads = plan.gang_heads;
  a->segments = plan.segments;
  for (int c = 0; c <= plan.slots; ++c) {
    a->fill_seg[c] = plan.fill_seg[c];
    a->fill_off[c] = plan.fill_off[c];
  }
}

}  // namespace

int list_chunk_attn_pieces(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                           int cus, int32_t* records, int64_t capacity, int64_t* count_out) {
  AttnPlan plan;
  const int rc = plan_chunk_attn(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, cus, true, &plan);
  if (rc != KVRA_OK) return rc;
  AttnArgs a;
  schedule_args(plan, prefix_len, chunk_len, n_q_heads, n_kv_heads, &a);
  int64_t count = 0;
  for (int wg = 0; wg < plan.groups * plan.slots; ++wg) {
    const int x = wg % plan.groups, c = wg / plan.groups;
    PieceWalker walker(a, x, c);
    Piece pc;
    while (walker.next(a, &pc)) {
      if (count < capacity && records != nullptr) {
        int listed = 0, found = 0;
        if (pc.slot >= 0)
          for_each_piece_of_segment(a, pc.seg, [&](int slot) { ++listed; found += slot == pc.slot; });
        int32_t* r = records + count * kPieceRecordInts;
        r[0] = wg;
        r[1] = pc.g;
        r[2] = pc.qt;
        r[3] = pc.jt0;
        r[4] = pc.jt1;
        r[5] = pc.n;
        r[6] = pc.slot >= 0 ? x * slots_per_group(a) + pc.slot : -1;
        r[7] = listed;
        r[8] = found;
        r[9] = pc.slot >= 0 ? x * kMaxSlots + pc.seg : -1;
      }
      ++count;
    }
  }
  if (count_out != nullptr) *count_out = count;
  return KVRA_OK;
}

namespace {

// The schedules of the last few distinct shapes: a prefill loop calls with the same handful of
// (prefix, chunk) pairs layer after layer, and working a schedule out takes tens of microseconds.
struct PlanCacheEntry {
  int64_t prefix_len, chunk_len;
  int n_q_heads, n_kv_heads, head_dim, cus, scratch_available;
  bool valid;
  AttnPlan plan;
};
constexpr int kPlanCacheEntries = 32;
PlanCacheEntry g_plan_cache[kPlanCacheEntries] = {};
int g_plan_cache_next = 0;
std::mutex g_plan_cache_mutex;

int cached_plan(int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim, int cus,
                bool scratch_available, AttnPlan* plan) {
  std::lock_guard<std::mutex> lock(g_plan_cache_mutex);
  for (const PlanCacheEntry& e : g_plan_cache)
    if (e.valid && e.prefix_len == prefix_len && e.chunk_len == chunk_len && e.n_q_heads == n_q_heads &&
        e.n_kv_heads == n_kv_heads && e.head_dim == head_dim && e.cus == cus &&
        e.scratch_available == static_cast<int>(scratch_available)) {
      *plan = e.plan;
      return KVRA_OK;
    }
  const int rc = plan_chunk_attn(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, cus, scratch_available, plan);
  if (rc != KVRA_OK) return rc;
  PlanCacheEntry& e = g_plan_cache[g_plan_cache_next];
  g_plan_cache_next = (g_plan_cache_next + 1) % kPlanCacheEntries;
  e = PlanCacheEntry{prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, cus, static_cast<int>(scratch_available), true, *plan};
  return KVRA_OK;
}

}  // namespace

int launch_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                      int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                      float scale, void* out, hipStream_t stream, bool static_scratch_only) {
  // the scratch buffer is looked up by the current device: a stream of another device would get the wrong one
  if (stream != nullptr) {
    hipDevice_t stream_dev = 0;
    int cur = 0;
    if (hipStreamGetDevice(stream, &stream_dev) == hipSuccess && hipGetDevice(&cur) == hipSuccess) {
      if (static_cast<int>(stream_dev) != cur) return KVRA_EINVAL;
    } else {
      (void)hipGetLastError();   // could not be asked: go on as before
    }
  }
  int cus = 0;
  int64_t slots_owned = kStaticSlots;
  float* scratch_ptr = static_scratch_only ? static_scratch(&cus) : device_scratch(stream, &cus, &slots_owned);
  if (static_scratch_only && scratch_ptr == nullptr) return KVRA_ENODEVICE;
  AttnPlan plan;
  const int rc0 = cached_plan(prefix_len, chunk_len, n_q_heads, n_kv_heads, head_dim, cus, scratch_ptr != nullptr, &plan);
  if (rc0 != KVRA_OK) return rc0;
  if (plan.scratch_slots > slots_owned) return KVRA_ESCRATCH;   // only the fixed array can be too small
  AttnArgs a;
  schedule_args(plan, prefix_len, chunk_len, n_q_heads, n_kv_heads, &a);
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k_cache);
  a.v = static_cast<const __bf16*>(v_cache);
  a.out = static_cast<__bf16*>(out);
  a.c_log2 = scale * 1.4426950408889634f;
  a.scratch = plan.partial_pieces > 0 ? scratch_ptr : nullptr;
  a.counters = scratch_ptr != nullptr
      ? reinterpret_cast<int*>(scratch_ptr + static_cast<size_t>(slots_owned) * kPartialFloats(128)) : nullptr;
  const int workgroups = plan.groups * plan.slots;
#ifdef KVRA_TRACE
  a.trace = workgroups <= g_trace_groups ? g_trace_buf : nullptr;
#endif
  const unsigned smem = 2u * kStages * static_cast<unsigned>(a.bn) * static_cast<unsigned>(head_dim) * 2u;   // K ring + V ring
  const dim3 b3(kThreads);
  const dim3 g_main(static_cast<unsigned>(workgroups));
  return head_dim == 128 ? launch_kernel(chunk_attn_kernel<128>, g_main, b3, a, stream, smem)
                         : launch_kernel(chunk_attn_kernel<64>, g_main, b3, a, stream, smem);
}

}  // namespace kvra

#ifdef KVRA_TRACE
// Timeline build only: the device buffer (8 words of 8 bytes per piece) that the next kvra_chunk_attn
// launches stamp (8 pieces per workgroup); a launch with more workgroups than `workgroups` leaves no stamps.
// NULL detaches.
extern "C" int kvra_trace_attach(void* device_buffer, long long workgroups) {
  kvra::g_trace_buf = static_cast<unsigned long long*>(device_buffer);
  kvra::g_trace_groups = device_buffer != nullptr ? workgroups : 0;
  return KVRA_OK;
}
#endif
