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
#include "kvra_internal.h"

namespace kvra {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef short s16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;

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
  int nq_tiles;
  float c_log2;   // scale * log2(e): softmax runs in base 2
};

__device__ __forceinline__ float other_half(float x) {
  // value held by lane ^ 32
  auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float((threadIdx.x & 32) ? r[0] : r[1]);
}

template <int D, int NW>
__global__ __launch_bounds__(64 * NW, 2) void chunk_attn_kernel(AttnArgs a) {
  constexpr int BM = 32 * NW;              // virtual rows per workgroup
  constexpr int BN = 64;                   // keys per tile
  constexpr int CPR = D / 8;               // 16-byte pieces per K/V row
  constexpr int KS = D / 16;               // contraction steps of S^T = K Q^T
  constexpr int DB = D / 32;               // 32-row blocks of O^T
  constexpr int RPB = 256 / (D * 2);       // rows per 256-byte LDS bank span
  constexpr int TILE = BN * CPR;           // 16-byte pieces per tile
  constexpr int LOADS = TILE / (64 * NW);  // pieces each thread moves per tile
  static_assert(TILE % (64 * NW) == 0, "tile must split evenly over the workgroup");

  __shared__ u32x4 ldsK[2][TILE];
  __shared__ u32x4 ldsV[2][TILE];

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n = lane & 31, kg = lane >> 5;

  // workgroup -> (kv head, row tile): longest row tiles first; with Hkv a multiple of 8 the
  // heads are dealt to the 8 XCDs (workgroup ids go round-robin over XCDs) so that each
  // XCD's L2 holds the K/V stream of its own heads only.
  int g, qt;
  {
    const int bid = blockIdx.x;
    if ((a.Hkv & 7) == 0) {
      const int xcd = bid & 7, j = bid >> 3, hp = a.Hkv >> 3;
      g = xcd + 8 * (j % hp);
      qt = a.nq_tiles - 1 - j / hp;
    } else {
      g = bid % a.Hkv;
      qt = a.nq_tiles - 1 - bid / a.Hkv;
    }
  }

  const int VR = a.chunk * a.G;            // virtual rows of this kv head
  const int total = a.prefix + a.chunk;    // valid cache rows
  const int v0 = qt * BM + wave * 32;
  const bool wave_active = v0 < VR;
  int vr = v0 + n;
  const bool row_valid = vr < VR;
  if (!row_valid) vr = VR - 1;
  const int r = vr / a.G;
  const int h = g * a.G + (vr - r * a.G);
  const int qpos = a.prefix + r;
  const int wmin = a.prefix + min(v0, VR - 1) / a.G;        // wave-uniform
  const int wmax = a.prefix + min(v0 + 31, VR - 1) / a.G;   // wave-uniform
  const int kmax = a.prefix + min(qt * BM + BM - 1, VR - 1) / a.G;
  const int nt = kmax / BN + 1;            // key tiles this workgroup walks

  // Q fragment: B operand of S^T, lane (n, kg) holds Q[row n][16 ks + 8 kg .. +7]
  bf16x8 qf[KS];
  {
    const __bf16* qrow = a.q + (static_cast<long long>(r) * a.H + h) * D;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) qf[ks] = *reinterpret_cast<const bf16x8*>(qrow + 16 * ks + 8 * kg);
  }

  // ---- global -> register -> LDS staging of K/V tiles -------------------------------------
  u32x4 kr[LOADS], vr4[LOADS];
  auto gload = [&](int kt) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int cid = tid + i * 64 * NW;
      const int row = cid / CPR, cc = cid % CPR;
      const int key = min(kt * BN + row, total - 1);   // rows past the end repeat the last valid row
      const long long off = (static_cast<long long>(key) * a.Hkv + g) * D + cc * 8;
      kr[i] = *reinterpret_cast<const u32x4*>(a.k + off);
      vr4[i] = *reinterpret_cast<const u32x4*>(a.v + off);
    }
  };
  auto lstore = [&](int buf) {
#pragma unroll
    for (int i = 0; i < LOADS; ++i) {
      const int cid = tid + i * 64 * NW;
      const int row = cid / CPR, cc = cid % CPR;
      // XOR swizzles keep the MFMA operand reads below free of bank conflicts:
      //   K is read 16 bytes per lane down 16+ consecutive rows of one column piece;
      //   V is read (transposing) 8 bytes per lane over 4 consecutive rows x 64 bytes.
      const int kslot = cc ^ ((row / RPB) % CPR);
      const int vslot = cc ^ (4 * ((row / RPB) % (D / 32)));
      ldsK[buf][row * CPR + kslot] = kr[i];
      ldsV[buf][row * CPR + vslot] = vr4[i];
    }
  };

  f32x16 o[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int e = 0; e < 16; ++e) o[db][e] = 0.0f;
  float m = -INFINITY;   // running row max, already multiplied by c_log2
  float l = 0.0f;        // running row sum of this lane's half of the keys
  const float c = a.c_log2;

  // lane-constant parts of the LDS read addresses
  const int k_sw = (n / RPB) % CPR;                       // K swizzle of row 32 mb + n
  const int vi = lane & 15, vmh = (lane >> 4) & 1;        // position inside the 16-lane transpose block
  const int v_row0 = 4 * kg + (vi >> 2);                  // + 32 mb + 16 s + 8 e
  const int v_sw = 4 * ((v_row0 / RPB) % (D / 32));
  const int v_cc0 = 2 * vmh + ((vi & 3) >> 1);            // + 4 db
  const int v_sub = (vi & 1) * 4;                         // element offset inside the 16-byte piece

  gload(0);
  lstore(0);
  __syncthreads();

  for (int kt = 0; kt < nt; ++kt) {
    const int buf = kt & 1;
    if (kt + 1 < nt) gload(kt + 1);

    if (wave_active && kt * BN <= wmax) {
      // ---- S^T = K Q^T ---------------------------------------------------------------------
      f32x16 s[2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) s[mb][e] = 0.0f;
      const bf16x8* Kb = reinterpret_cast<const bf16x8*>(ldsK[buf]);
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
        for (int mb = 0; mb < 2; ++mb) {
          const int row = 32 * mb + n;
          const bf16x8 kf = Kb[row * CPR + ((2 * ks + kg) ^ k_sw)];
          s[mb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[ks], s[mb], 0, 0, 0);
        }
      }
      // register e of block mb is key  kt*BN + 32 mb + 8 (e/4) + 4 kg + e%4  of query n
      if (kt * BN + BN - 1 > wmin) {
        const int rel = qpos - kt * BN - 4 * kg;   // key offset (within tile, minus 4kg) still visible
#pragma unroll
        for (int mb = 0; mb < 2; ++mb)
#pragma unroll
          for (int e = 0; e < 16; ++e)
            if (32 * mb + 8 * (e / 4) + (e % 4) > rel) s[mb][e] = -INFINITY;
      }
      // ---- online softmax (base 2) ---------------------------------------------------------
      float tmax = s[0][0];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) tmax = fmaxf(tmax, s[mb][e]);
      tmax = fmaxf(tmax, other_half(tmax));
      const float mnew = fmaxf(m, tmax * c);
      const float alpha = __builtin_amdgcn_exp2f(m - mnew);
      float psum = 0.0f;
      bf16x8 pf[2][2];
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const float p = __builtin_amdgcn_exp2f(fmaf(s[mb][e], c, -mnew));
          psum += p;
          pf[mb][e / 8][e % 8] = static_cast<__bf16>(p);
        }
      l = fmaf(l, alpha, psum);
      m = mnew;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int e = 0; e < 16; ++e) o[db][e] *= alpha;
      // ---- O^T += V^T P^T ------------------------------------------------------------------
      // contraction slot 4e + j of step (mb, si) is key 32 mb + 16 si + 8 e + 4 kg + j on both operands
      const short* Vb = reinterpret_cast<const short*>(ldsV[buf]);
#pragma unroll
      for (int mb = 0; mb < 2; ++mb)
#pragma unroll
        for (int si = 0; si < 2; ++si)
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            s16x8 vf;
#pragma unroll
            for (int e = 0; e < 2; ++e) {
              const int row = 32 * mb + 16 * si + 8 * e + v_row0;
              const int slot = (4 * db + v_cc0) ^ v_sw;
              const short* p = Vb + (row * CPR + slot) * 8 + v_sub;
              const s16x4 t = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4*)p);
              vf[4 * e + 0] = t[0]; vf[4 * e + 1] = t[1]; vf[4 * e + 2] = t[2]; vf[4 * e + 3] = t[3];
            }
            o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, vf), pf[mb][si], o[db], 0, 0, 0);
          }
    }

    if (kt + 1 < nt) lstore(buf ^ 1);
    __syncthreads();
  }

  // ---- epilogue: O / l, bf16, store -----------------------------------------------------------
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
        for (int j = 0; j < 4; ++j) w[j] = static_cast<__bf16>(o[db][4 * r4 + j] * inv);
        *reinterpret_cast<bf16x4*>(orow + 32 * db + 8 * r4 + 4 * kg) = w;
      }
  }
}

int launch_chunk_attn(const void* q, const void* k_cache, const void* v_cache,
                      int64_t prefix_len, int64_t chunk_len, int n_q_heads, int n_kv_heads, int head_dim,
                      float scale, void* out, hipStream_t stream) {
  constexpr int NW = 4;
  constexpr int BM = 32 * NW;
  const int G = n_q_heads / n_kv_heads;
  const int64_t vrows = chunk_len * G;
  if (vrows > (int64_t(1) << 30) || prefix_len + chunk_len > (int64_t(1) << 30)) return KVRA_EUNSUPPORTED;
  AttnArgs a;
  a.q = static_cast<const __bf16*>(q);
  a.k = static_cast<const __bf16*>(k_cache);
  a.v = static_cast<const __bf16*>(v_cache);
  a.out = static_cast<__bf16*>(out);
  a.prefix = static_cast<int>(prefix_len);
  a.chunk = static_cast<int>(chunk_len);
  a.H = n_q_heads;
  a.Hkv = n_kv_heads;
  a.G = G;
  a.nq_tiles = static_cast<int>((vrows + BM - 1) / BM);
  a.c_log2 = scale * 1.4426950408889634f;
  const int64_t grid = static_cast<int64_t>(a.nq_tiles) * n_kv_heads;
  if (grid > 0x7FFFFFFF) return KVRA_EUNSUPPORTED;
  const dim3 g3(static_cast<unsigned>(grid)), b3(64 * NW);
  if (head_dim == 128) return launch_kernel(chunk_attn_kernel<128, NW>, g3, b3, a, stream);
  return launch_kernel(chunk_attn_kernel<64, NW>, g3, b3, a, stream);
}

}  // namespace kvra
