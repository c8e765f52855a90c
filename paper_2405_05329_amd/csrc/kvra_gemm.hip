// Linear layers of the decoder layer a KV-Runahead process runs around its attention block
// (App. C listing: q/k/v projections before, output projection after the attention; the SwiGLU MLP
// of the LLaMA models of Sec. 5) for gfx950:  out[m, n] = sum_k x[m, k] * w[n, k], bf16 in, fp32
// accumulate, bf16 out, with three fused epilogues (plain / + residual / silu(gate) * up).
//
// Orientation.  Both operands are contiguous along k, which is exactly what the two register
// operands of v_mfma_f32_32x32x16_bf16 want (lane (r, kg) holds 8 consecutive k of row r).  The
// weight rows go to the A side and the token rows to the B side, i.e. the kernel forms the
// TRANSPOSED tile out^T[n, m]: in the 32x32 accumulator layout a lane then owns one token and
// groups of 4 consecutive n, so the epilogue stores 8-byte bf16x4 pieces of an output row.
//
// Tiling.  Workgroup = 8 waves, tile = 256 weight rows x 256 tokens, k in steps of 64 through a
// two-slot LDS ring filled by LDS-direct loads (no registers in between); 4 x 2 waves, each wave
// 64 weight rows x 128 tokens = 2 x 4 accumulator blocks.  One workgroup barrier per k step: it
// publishes the slot that landed and frees the other one for the next load.
#include "kvra_internal.h"

#include <type_traits>

namespace kvra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) void lds_void;

constexpr int kGemmThreads = 512;
constexpr int kTileN = 256;    // weight rows per workgroup tile
constexpr int kTileM = 256;    // tokens per workgroup tile
constexpr int kTileK = 64;     // k per LDS slot
// Waves (the last ones of the workgroup, one per SIMD) that issue the global -> LDS loads.  The 64
// loads of a k step keep the vector memory pipe busy for about 1000 cycles (64 bytes per clock) and
// a wave sits in its share of them until they are accepted; with every wave issuing 8 loads after
// the barrier no MFMA starts for the first 500 cycles of a step.  With four issuers their SIMD
// partners compute at once and have the matrix pipe to themselves meanwhile: +2.5 to 5 %.
constexpr int kIssuers = 4;
constexpr int kSlotBytes = (kTileN + kTileM) * kTileK * 2;   // 64 KiB: weight tile then token tile

struct OutSegment {
  __bf16* ptr;   // dense [m, width] matrix that receives output columns [first, end)
  int end;       // one past the last output column of this segment
  int first;
  int ld;        // row stride of ptr in elements
};

struct GemmArgs {
  const __bf16* x;     // [m, k]
  const __bf16* w;     // [rows, k]
  const __bf16* w2;    // dual mode: second weight [rows, k]; else null
  const __bf16* res;   // residual [m, seg[0].ld] or null (single segment only)
  OutSegment seg[3];
  int n_seg;
  int m;
  int n;               // weight rows walked: rows, or 2 * rows in dual mode (32-row blocks alternate w / w2)
  int k;
  int tiles_n, tiles_m;
  int dual;
};

__device__ __forceinline__ void gemm_lds_dma16(const void* uniform_base, unsigned lane_byte_off, unsigned lds_byte_addr) {
  // 64 lanes x 16 bytes -> 1 KiB of consecutive LDS (lane l lands at +16 l); inline assembly so that
  // completion can be awaited by hand with s_waitcnt vmcnt(n) instead of a full drain per load
  asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
               :
               : "v"(lane_byte_off), "s"(uniform_base), "s"(lds_byte_addr)
               : "memory", "m0");
}

__global__ __launch_bounds__(kGemmThreads, 1) void linear_kernel(GemmArgs a) {
  extern __shared__ u32x4 smem[];
  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int r32 = lane & 31, kg = lane >> 5;
  const int wn = wave & 3, wm = wave >> 2;

  // workgroup -> tile.  Workgroup ids go round-robin over the 8 XCDs; each XCD takes a contiguous
  // run of the tile order "bands of 4 weight tiles, token tiles inside a band, weight tile
  // fastest", so that the 32 workgroups an XCD runs together share 4 weight tiles and 8 token
  // tiles in its L2.
  int tn, tm;
  {
    const int total = a.tiles_n * a.tiles_m;
    const int per = (total + 7) >> 3;
    const int t = (blockIdx.x & 7) * per + (blockIdx.x >> 3);
    if (t >= total) return;   // whole workgroup leaves before any barrier
    const int band = t / (4 * a.tiles_m);
    const int width = min(4, a.tiles_n - 4 * band);
    const int within = t - band * 4 * a.tiles_m;
    tm = within / width;
    tn = 4 * band + within % width;
  }
  const int n0 = tn * kTileN, m0 = tm * kTileM;

  // ---- global -> LDS staging -----------------------------------------------------------------
  // A 256 x 64 bf16 tile is 2048 pieces of 16 bytes = 32 wave loads, NL per issuing wave and operand.
  // Piece p = (row p / 8, slot p % 8); the lane that owns (row, slot) fetches column piece
  // slot ^ ((row / 2) % 8) so that the operand reads below (16 rows of one column piece per
  // quarter wave) spread over all banks.  Rows past the end of a matrix repeat its last row.
  constexpr int NL = 32 / kIssuers;   // loads per issuing wave and operand
  const bool issuer = wave >= 8 - kIssuers;
  const int iw = wave - (8 - kIssuers);
  unsigned woff[NL], xoff[NL];
  const __bf16* wsrc[NL];
#pragma unroll
  for (int i = 0; i < NL; ++i) {
    const int p = (i * kIssuers + (issuer ? iw : 0)) * 64 + lane;
    const int row = p >> 3, slot = p & 7;
    const unsigned piece = static_cast<unsigned>(slot ^ ((row >> 1) & 7));
    int vrow = min(n0 + row, a.n - 1);                       // row in the walked order
    int wrow = vrow;
    const __bf16* src = a.w;
    if (a.dual) {                                            // 32-row blocks alternate between the two weights
      const int blk = vrow >> 5;
      wrow = ((blk >> 1) << 5) + (vrow & 31);
      // 8-row groups never straddle a 32-row block, so the choice is uniform per load
      if (__builtin_amdgcn_readfirstlane(blk & 1)) src = a.w2;
    }
    wsrc[i] = src;
    woff[i] = 2u * (static_cast<unsigned>(wrow) * static_cast<unsigned>(a.k) + 8u * piece);
    const int xrow = min(m0 + row, a.m - 1);
    xoff[i] = 2u * (static_cast<unsigned>(xrow) * static_cast<unsigned>(a.k) + 8u * piece);
  }
  const unsigned lds0 = static_cast<unsigned>(reinterpret_cast<uintptr_t>((lds_void*)smem));
  auto dma_slot = [&](int kt, int slot) __attribute__((always_inline)) {
    const long long kofs = static_cast<long long>(kt) * kTileK;
    if (!issuer) return;
#pragma unroll
    for (int i = 0; i < NL; ++i) {
      const unsigned dst = lds0 + slot * kSlotBytes + (i * kIssuers + iw) * 1024;
      gemm_lds_dma16(wsrc[i] + kofs, woff[i], dst);
      gemm_lds_dma16(a.x + kofs, xoff[i], dst + kTileN * kTileK * 2);
    }
  };

  f32x16 acc[2][4];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb)
#pragma unroll
    for (int mb = 0; mb < 4; ++mb)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[nb][mb][e] = 0.0f;

  const int sw = (r32 >> 1) & 7;   // swizzle of the rows this lane reads (tile rows are multiples of 32 apart)
  // one k step of 64 on LDS slot S: operand reads of contraction step ks + 1 are issued before the
  // MFMAs of step ks
  auto compute = [&](auto slot_tag) __attribute__((always_inline)) {
    constexpr int S = decltype(slot_tag)::value;
    const bf16x8* Wt = reinterpret_cast<const bf16x8*>(smem) + S * (kSlotBytes / 16);
    const bf16x8* Xt = Wt + kTileN * kTileK / 8;
    auto wread = [&](int nb, int ks) -> bf16x8 { return Wt[(64 * wn + 32 * nb + r32) * 8 + ((2 * ks + kg) ^ sw)]; };
    auto xread = [&](int mb, int ks) -> bf16x8 { return Xt[(128 * wm + 32 * mb + r32) * 8 + ((2 * ks + kg) ^ sw)]; };
    bf16x8 fw[2][2], fx[2][4];
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) fw[0][nb] = wread(nb, 0);
#pragma unroll
    for (int mb = 0; mb < 4; ++mb) fx[0][mb] = xread(mb, 0);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      if (ks + 1 < 4) {
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) fw[(ks + 1) & 1][nb] = wread(nb, ks + 1);
#pragma unroll
        for (int mb = 0; mb < 4; ++mb) fx[(ks + 1) & 1][mb] = xread(mb, ks + 1);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int mb = 0; mb < 4; ++mb)
#pragma unroll
        for (int nb = 0; nb < 2; ++nb)
          acc[nb][mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fw[ks & 1][nb], fx[ks & 1][mb], acc[nb][mb], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  const int KT = a.k / kTileK;
  dma_slot(0, 0);
  for (int kt = 0; kt < KT; kt += 2) {
    __builtin_amdgcn_s_waitcnt(0x0F70);   // vmcnt(0): this wave's part of tile kt has landed
    __syncthreads();                      // ... everybody's has, and slot 1 is no longer being read
    if (kt + 1 < KT) dma_slot(kt + 1, 1);
    compute(std::integral_constant<int, 0>{});
    if (kt + 1 < KT) {
      __builtin_amdgcn_s_waitcnt(0x0F70);
      __syncthreads();
      if (kt + 2 < KT) dma_slot(kt + 2, 0);
      compute(std::integral_constant<int, 1>{});
    }
  }

  // ---- epilogue ------------------------------------------------------------------------------
  // register e of block (nb, mb): weight row 64 wn + 32 nb + 8 (e/4) + 4 kg + e%4, token
  // 128 wm + 32 mb + r32 (tile-relative)
  if (a.dual) {
    // blocks nb = 0 / 1 are the gate / up rows of the same 32 output columns
    const int col0 = (n0 >> 1) + 32 * wn;
    if (n0 + 64 * wn < a.n) {
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const int tok = m0 + 128 * wm + 32 * mb + r32;
        if (tok < a.m) {
          __bf16* orow = a.seg[0].ptr + static_cast<long long>(tok) * a.seg[0].ld + col0 + 4 * kg;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            bf16x4 o4;
#pragma unroll
            for (int t = 0; t < 4; ++t) {
              const float g = acc[0][mb][4 * q + t], u = acc[1][mb][4 * q + t];
              o4[t] = static_cast<__bf16>(g * __builtin_amdgcn_rcpf(1.0f + __expf(-g)) * u);
            }
            *reinterpret_cast<bf16x4*>(orow + 8 * q) = o4;
          }
        }
      }
    }
  } else {
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int nblk = n0 + 64 * wn + 32 * nb;   // first output column of this 32-wide block
      if (nblk >= a.n) continue;
      // segment that holds this block (segment edges are multiples of 32)
      int s = 0;
      if (a.n_seg > 1 && nblk >= a.seg[0].end) s = 1;
      if (a.n_seg > 2 && nblk >= a.seg[1].end) s = 2;
      __bf16* obase = a.seg[s].ptr;
      const int ld = a.seg[s].ld, col0 = nblk - a.seg[s].first + 4 * kg;
#pragma unroll
      for (int mb = 0; mb < 4; ++mb) {
        const int tok = m0 + 128 * wm + 32 * mb + r32;
        if (tok < a.m) {
          __bf16* orow = obase + static_cast<long long>(tok) * ld + col0;
          const __bf16* rrow = a.res ? a.res + static_cast<long long>(tok) * ld + col0 : nullptr;
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            bf16x4 o4;
            if (rrow != nullptr) {
              const bf16x4 r4 = *reinterpret_cast<const bf16x4*>(rrow + 8 * q);
#pragma unroll
              for (int t = 0; t < 4; ++t) o4[t] = static_cast<__bf16>(acc[nb][mb][4 * q + t] + static_cast<float>(r4[t]));
            } else {
#pragma unroll
              for (int t = 0; t < 4; ++t) o4[t] = static_cast<__bf16>(acc[nb][mb][4 * q + t]);
            }
            *reinterpret_cast<bf16x4*>(orow + 8 * q) = o4;
          }
        }
      }
    }
  }
}

int launch_linear(const void* x, const void* w, const void* w2, const void* residual,
                  void* const* out, const int* seg_cols, int n_seg,
                  int64_t m, int64_t n_out, int64_t k, hipStream_t stream) {
  GemmArgs a;
  a.x = static_cast<const __bf16*>(x);
  a.w = static_cast<const __bf16*>(w);
  a.w2 = static_cast<const __bf16*>(w2);
  a.res = static_cast<const __bf16*>(residual);
  a.n_seg = n_seg;
  int first = 0;
  for (int s = 0; s < 3; ++s) {
    if (s < n_seg) {
      a.seg[s].ptr = static_cast<__bf16*>(out[s]);
      a.seg[s].first = first;
      a.seg[s].end = first + seg_cols[s];
      a.seg[s].ld = seg_cols[s];
      first += seg_cols[s];
    } else {
      a.seg[s] = OutSegment{nullptr, 0, 0, 0};
    }
  }
  a.dual = w2 != nullptr ? 1 : 0;
  a.m = static_cast<int>(m);
  a.n = static_cast<int>(a.dual ? 2 * n_out : n_out);
  a.k = static_cast<int>(k);
  a.tiles_n = (a.n + kTileN - 1) / kTileN;
  a.tiles_m = (a.m + kTileM - 1) / kTileM;
  const int total = a.tiles_n * a.tiles_m;
  const unsigned grid = 8u * static_cast<unsigned>((total + 7) / 8);
  return launch_kernel(linear_kernel, dim3(grid), dim3(kGemmThreads), a, stream, 2 * kSlotBytes);
}

// ---- RMSNorm ------------------------------------------------------------------------------------
// y[t, :] = x[t, :] / sqrt(mean(x[t, :]^2) + eps) * gain, fp32 arithmetic, one workgroup per token.
// HBM-bound: every element is read once and written once with 16-byte accesses.
struct NormArgs {
  const __bf16* x;
  const __bf16* gain;
  __bf16* y;
  int rows;
  int hidden;
  float eps;
};

constexpr int kNormThreads = 256;
constexpr int kNormMaxPieces = 4;   // 16-byte pieces a thread keeps in registers: hidden <= 8192

__global__ __launch_bounds__(kNormThreads) void rms_norm_kernel(NormArgs a) {
  __shared__ float part[kNormThreads / 64];
  const int tid = threadIdx.x;
  const int pieces = a.hidden / 8;
  const bf16x8* xr = reinterpret_cast<const bf16x8*>(a.x + static_cast<long long>(blockIdx.x) * a.hidden);
  bf16x8 v[kNormMaxPieces];
  float ss = 0.0f;
#pragma unroll
  for (int i = 0; i < kNormMaxPieces; ++i) {
    const int p = tid + i * kNormThreads;
    if (p < pieces) {
      v[i] = xr[p];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float f = static_cast<float>(v[i][e]);
        ss = fmaf(f, f, ss);
      }
    }
  }
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
  if ((tid & 63) == 0) part[tid >> 6] = ss;
  __syncthreads();
  float tot = 0.0f;
#pragma unroll
  for (int w = 0; w < kNormThreads / 64; ++w) tot += part[w];
  const float rinv = 1.0f / sqrtf(tot / static_cast<float>(a.hidden) + a.eps);
  const bf16x8* gr = reinterpret_cast<const bf16x8*>(a.gain);
  bf16x8* yr = reinterpret_cast<bf16x8*>(a.y + static_cast<long long>(blockIdx.x) * a.hidden);
#pragma unroll
  for (int i = 0; i < kNormMaxPieces; ++i) {
    const int p = tid + i * kNormThreads;
    if (p < pieces) {
      const bf16x8 g = gr[p];
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 8; ++e) o[e] = static_cast<__bf16>(static_cast<float>(v[i][e]) * rinv * static_cast<float>(g[e]));
      yr[p] = o;
    }
  }
}

int launch_rms_norm(const void* x, const void* gain, void* y, int64_t rows, int hidden, float eps, hipStream_t stream) {
  NormArgs a;
  a.x = static_cast<const __bf16*>(x);
  a.gain = static_cast<const __bf16*>(gain);
  a.y = static_cast<__bf16*>(y);
  a.rows = static_cast<int>(rows);
  a.hidden = hidden;
  a.eps = eps;
  return launch_kernel(rms_norm_kernel, dim3(static_cast<unsigned>(rows)), dim3(kNormThreads), a, stream);
}

int rms_norm_max_hidden() { return kNormThreads * kNormMaxPieces * 8; }

}  // namespace kvra
