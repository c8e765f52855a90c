// kvra_append_kv: rotary embedding + KV-cache population of one chunk (App. C listing, cache
// concatenation step; Sec. 4.3 contiguity).  HBM-bound streaming kernel: every byte of K, V
// (and Q) is read once and written once with 128-bit accesses.
#include "kvra_internal.h"

namespace kvra {

typedef unsigned short u16x8 __attribute__((ext_vector_type(8)));

struct AppendArgs {
  const unsigned short* k_in;
  const unsigned short* v_in;
  unsigned short* q;        // may be null
  unsigned short* k_cache;
  unsigned short* v_cache;
  long long prefix_len;
  int chunk_len;
  int n_q_heads;
  int n_kv_heads;
  int use_rope;
  double inv_freq[64];      // base^(-2i/d), i < d/2, formed on the host in fp64
};

__device__ __forceinline__ float bf16_to_f32(unsigned short b) {
  return __uint_as_float(static_cast<unsigned int>(b) << 16);
}

__device__ __forceinline__ unsigned short f32_to_bf16_rne(float x) {
  // round to nearest, ties to even, on the bit pattern; a NaN stays a (quiet) NaN instead of
  // being carried into an infinity or a zero by the rounding increment
  unsigned int u = __float_as_uint(x);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return static_cast<unsigned short>((u >> 16) | 0x0040u);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return static_cast<unsigned short>(u >> 16);
}

// One workgroup serves TOK consecutive tokens (TOK * D/2 <= 256).  Phase 1: TOK * D/2 threads form
// cos/sin of (prefix + row) * inv_freq[i] in fp64 and park them in LDS as fp32.  Phase 2: all
// threads stream "pair units" (a 16-byte piece of the low half of a head row and its partner in
// the high half) for K and Q, and plain 16-byte pieces for V.  Long chunks use the largest TOK
// (every thread busy in phase 1); short chunks use fewer tokens per workgroup so that the launch
// still puts several workgroups on every CU.
template <int D, int TOK>
__global__ __launch_bounds__(256) void append_kv_kernel(AppendArgs a) {
  constexpr int HALF = D / 2;
  static_assert(TOK * HALF <= 256, "one thread per (token, frequency) in phase 1");
  constexpr int PAIRS = D / 16;            // pair units per head row
  constexpr int CHUNKS = D / 8;            // 16-byte pieces per head row
  __shared__ float cs[TOK][HALF];
  __shared__ float sn[TOK][HALF];

  const int tid = threadIdx.x;
  const int tok0 = blockIdx.x * TOK;
  const int ntok = min(TOK, a.chunk_len - tok0);

  const int Hkv = a.n_kv_heads, H = a.n_q_heads;

  // ---- V: bit-exact copy, issued first: it needs no angles, and its traffic overlaps the
  // fp64 sincos below -------------------------------------------------------------------
  {
    const int per_tok = Hkv * CHUNKS;
    const int total = ntok * per_tok;
    const u16x8* src = reinterpret_cast<const u16x8*>(a.v_in) + static_cast<long long>(tok0) * per_tok;
    u16x8* dst = reinterpret_cast<u16x8*>(a.v_cache) + (a.prefix_len + tok0) * per_tok;
#pragma unroll 4
    for (int u = tid; u < total; u += 256) dst[u] = src[u];
  }

  if (a.use_rope) {
    const int t = tid / HALF, i = tid % HALF;
    if (t < ntok) {
      const double phi = static_cast<double>(a.prefix_len + tok0 + t) * a.inv_freq[i];
      double s, c;
      sincos(phi, &s, &c);
      cs[t][i] = static_cast<float>(c);
      sn[t][i] = static_cast<float>(s);
    }
    __syncthreads();
  }

  // ---- K: rotate (or copy) into the cache --------------------------------------------
  {
    const int per_tok = Hkv * PAIRS;
    const int total = ntok * per_tok;
#pragma unroll 2
    for (int u = tid; u < total; u += 256) {
      const int t = u / per_tok;
      const int rem = u - t * per_tok;
      const int head = rem / PAIRS;
      const int j = rem - head * PAIRS;
      const long long src_row = (static_cast<long long>(tok0 + t) * Hkv + head) * D;
      const long long dst_row = ((a.prefix_len + tok0 + t) * Hkv + head) * D;
      const u16x8 lo = *reinterpret_cast<const u16x8*>(a.k_in + src_row + 8 * j);
      const u16x8 hi = *reinterpret_cast<const u16x8*>(a.k_in + src_row + HALF + 8 * j);
      u16x8 olo = lo, ohi = hi;
      if (a.use_rope) {
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const float c = cs[t][8 * j + e], s = sn[t][8 * j + e];
          const float x0 = bf16_to_f32(lo[e]), x1 = bf16_to_f32(hi[e]);
          olo[e] = f32_to_bf16_rne(fmaf(x0, c, -(x1 * s)));
          ohi[e] = f32_to_bf16_rne(fmaf(x1, c, x0 * s));
        }
      }
      *reinterpret_cast<u16x8*>(a.k_cache + dst_row + 8 * j) = olo;
      *reinterpret_cast<u16x8*>(a.k_cache + dst_row + HALF + 8 * j) = ohi;
    }
  }

  // ---- Q: rotate in place -------------------------------------------------------------
  if (a.q != nullptr && a.use_rope) {
    const int per_tok = H * PAIRS;
    const int total = ntok * per_tok;
#pragma unroll 2
    for (int u = tid; u < total; u += 256) {
      const int t = u / per_tok;
      const int rem = u - t * per_tok;
      const int head = rem / PAIRS;
      const int j = rem - head * PAIRS;
      unsigned short* row = a.q + (static_cast<long long>(tok0 + t) * H + head) * D;
      const u16x8 lo = *reinterpret_cast<const u16x8*>(row + 8 * j);
      const u16x8 hi = *reinterpret_cast<const u16x8*>(row + HALF + 8 * j);
      u16x8 olo, ohi;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float c = cs[t][8 * j + e], s = sn[t][8 * j + e];
        const float x0 = bf16_to_f32(lo[e]), x1 = bf16_to_f32(hi[e]);
        olo[e] = f32_to_bf16_rne(fmaf(x0, c, -(x1 * s)));
        ohi[e] = f32_to_bf16_rne(fmaf(x1, c, x0 * s));
      }
      *reinterpret_cast<u16x8*>(row + 8 * j) = olo;
      *reinterpret_cast<u16x8*>(row + HALF + 8 * j) = ohi;
    }
  }
}

int launch_append_kv(const void* k_in, const void* v_in, void* q_inout, void* k_cache, void* v_cache,
                     int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                     float rope_base, hipStream_t stream) {
  AppendArgs a;
  a.k_in = static_cast<const unsigned short*>(k_in);
  a.v_in = static_cast<const unsigned short*>(v_in);
  a.q = static_cast<unsigned short*>(q_inout);
  a.k_cache = static_cast<unsigned short*>(k_cache);
  a.v_cache = static_cast<unsigned short*>(v_cache);
  a.prefix_len = prefix_len;
  a.chunk_len = static_cast<int>(chunk_len);
  a.n_q_heads = n_q_heads;
  a.n_kv_heads = n_kv_heads;
  a.use_rope = rope_base > 0.0f ? 1 : 0;
  for (int i = 0; i < 64; ++i) a.inv_freq[i] = 0.0;
  if (a.use_rope) {
    for (int i = 0; i < head_dim / 2; ++i)
      a.inv_freq[i] = std::pow(static_cast<double>(rope_base), -2.0 * i / head_dim);
  }
  // tokens per workgroup: the most that phase 1 can serve, halved until the grid holds about
  // eight workgroups per CU (256 CUs) or one token per workgroup is reached
  int tok = 256 / (head_dim / 2);
  while (tok > 1 && (chunk_len + tok - 1) / tok < 2048) tok >>= 1;
  const unsigned grid = static_cast<unsigned>((chunk_len + tok - 1) / tok);
  const dim3 g(grid), b(256);
  if (head_dim == 128) {
    if (tok == 4) return launch_kernel(append_kv_kernel<128, 4>, g, b, a, stream);
    if (tok == 2) return launch_kernel(append_kv_kernel<128, 2>, g, b, a, stream);
    return launch_kernel(append_kv_kernel<128, 1>, g, b, a, stream);
  }
  if (tok == 8) return launch_kernel(append_kv_kernel<64, 8>, g, b, a, stream);
  if (tok == 4) return launch_kernel(append_kv_kernel<64, 4>, g, b, a, stream);
  if (tok == 2) return launch_kernel(append_kv_kernel<64, 2>, g, b, a, stream);
  return launch_kernel(append_kv_kernel<64, 1>, g, b, a, stream);
}

}  // namespace kvra
