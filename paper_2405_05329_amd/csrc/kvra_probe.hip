// Matrix-pipe probe: what a loop of nothing but v_mfma_f32_32x32x16_bf16 on register operands delivers on
// this chip, as a function of how many compute units are busy and of the operand data.  Not part of the
// product path: a yardstick for reading the roofline fractions of the attention and linear kernels (the
// published 2.5 PFLOP/s assumes 2.4 GHz on every matrix pipe at once; the clock under load is managed).
// Built as its own small library (python -m paper_2405_05329_amd.build --probe), driven by probe.py.
#include <hip/hip_runtime.h>

#include <cstdint>

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

// Every wave: 4 accumulators, 4 A and 4 B fragments (lane-wise 16 bytes each from `operands`), `iters`
// rounds of 16 MFMAs (every A with every B, so consecutive MFMAs see different operands and independent
// accumulators).  96 KiB of dynamic LDS per workgroup keeps it to one workgroup per compute unit.
__global__ __launch_bounds__(512, 1) void probe_mfma_kernel(const bf16x8* operands, float* sink, int iters,
                                                            unsigned long long* stamps) {
  extern __shared__ char lds[];
  const unsigned long long t0 = wall_clock64();
  const unsigned long long c0 = clock64();
  const int lane = threadIdx.x & 63;
  bf16x8 a[4], b[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    a[i] = operands[i * 64 + lane];
    b[i] = operands[(4 + i) * 64 + lane];
  }
  f32x16 acc[4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
  // (four rounds per trip: a 16-instruction loop body was found to run a third slower with two waves per SIMD
  // in one build than in the next, with identical instructions - instruction fetch at the loop's edges)
  for (int it = 0; it < iters / 4; ++it) {
#pragma unroll
    for (int u = 0; u < 4; ++u)
#pragma unroll
      for (int j = 0; j < 4; ++j)
#pragma unroll
        for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[(i + j) & 3], b[i], acc[i], 0, 0, 0);
  }
  float r = 0.0f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int e = 0; e < 16; ++e) r += acc[i][e];
  if (iters < 0) lds[threadIdx.x] = 0;   // (never true: keeps the LDS allocation referenced)
  sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = r;
  // per wave: XCD it ran on, start and end of the constant 100 MHz clock, cycles of the shader clock
  if (stamps != nullptr && lane == 0) {
    unsigned xcc;
    asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(xcc));
    unsigned long long* rec = stamps + 4 * (static_cast<size_t>(blockIdx.x) * (blockDim.x / 64) + threadIdx.x / 64);
    rec[0] = xcc & 0xF;
    rec[1] = t0;
    rec[2] = wall_clock64();
    rec[3] = clock64() - c0;
  }
}

// VALU issue probe: waves 4-7 of every workgroup (one per SIMD) run a stream of independent VALU instructions
// - fused multiply-adds, or exponentials each followed by one - and time it with the shader-clock cycle counter,
// while waves 0-3, their SIMD partners, are idle or issue MFMAs back to back.  cycles: one word per timed wave.
__global__ __launch_bounds__(512, 1) void probe_valu_kernel(const bf16x8* operands, float* sink, unsigned long long* cycles,
                                                            int valu_rounds, int with_mfma, int with_exp) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  float r = 0.0f;
  if (wave < 4) {
    if (with_mfma) {
      const bf16x8 a = operands[lane], b = operands[64 + lane];
      f32x16 acc[4];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
      // enough MFMAs to outlast the timed waves: 64 VALU instructions take at most ~700 cycles, 16 MFMAs 512
      for (int it = 0; it < 2 * valu_rounds; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int i = 0; i < 4; ++i) acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, acc[i], 0, 0, 0);
      }
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) r += acc[i][e];
    }
  } else {
    float x[8];
#pragma unroll
    for (int i = 0; i < 8; ++i) x[i] = threadIdx.x * 0.001f + i;
    __builtin_amdgcn_s_sleep(20);   // let the partners get going
    const unsigned long long c0 = clock64();
    if (with_exp) {
      for (int it = 0; it < valu_rounds; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u)
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = fmaf(__builtin_amdgcn_exp2f(x[i]), 0.0f, 0.5f);
      }
    } else {
      for (int it = 0; it < valu_rounds; ++it) {
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
          for (int i = 0; i < 8; ++i) x[i] = fmaf(x[i], 0.999f, 0.5f);
      }
    }
    const unsigned long long c1 = clock64();
#pragma unroll
    for (int i = 0; i < 8; ++i) r += x[i];
    if (lane == 0) cycles[blockIdx.x * 4 + (wave - 4)] = c1 - c0;
  }
  sink[static_cast<size_t>(blockIdx.x) * blockDim.x + threadIdx.x] = r;
}

// One wave that writes the 100 MHz clock: put before and after another kernel on the same stream, it tells how
// long the stream takes to get from one kernel into the next.
__global__ void probe_stamp_kernel(unsigned long long* out) {
  const unsigned long long t = wall_clock64();
  if (threadIdx.x == 0) out[0] = t;
}

}  // namespace

// out: device, one 64-bit word, receives the 100 MHz clock read by a one-wave kernel launched on `stream`.
extern "C" int kvra_probe_stamp(void* out, void* stream) {
  if (out == nullptr) return -1;
  hipLaunchKernelGGL(probe_stamp_kernel, dim3(1), dim3(64), 0, static_cast<hipStream_t>(stream),
                     static_cast<unsigned long long*>(out));
  return static_cast<int>(hipGetLastError());
}

// operands: device, 8 x 64 x 16 bytes (4 A and 4 B fragments per lane, bf16); sink: device,
// workgroups * 64 * waves floats; stamps: device, 4 * workgroups * waves 64-bit words (XCD, start, end, shader-clock cycles per wave),
// or NULL.  waves in 1..8 (waves per workgroup: 4 = one per SIMD, 8 = two).
// iters: rounds of 16 MFMAs per wave, a multiple of 4.  One workgroup per compute unit.  Returns 0, or -1 on bad arguments, or the HIP error code of the launch.
extern "C" int kvra_probe_mfma(const void* operands, void* sink, int workgroups, int waves, int iters, void* stamps,
                               void* stream) {
  if (operands == nullptr || sink == nullptr || workgroups < 1 || waves < 1 || waves > 8 || iters < 4 || iters % 4 != 0) return -1;
  static bool attr_set = false;
  if (!attr_set) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(probe_mfma_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 96 * 1024);
    if (e != hipSuccess) return static_cast<int>(e);
    attr_set = true;
  }
  hipLaunchKernelGGL(probe_mfma_kernel, dim3(workgroups), dim3(64 * waves), 96 * 1024, static_cast<hipStream_t>(stream),
                     static_cast<const bf16x8*>(operands), static_cast<float*>(sink), iters,
                     static_cast<unsigned long long*>(stamps));
  return static_cast<int>(hipGetLastError());
}

// VALU issue probe on `workgroups` compute units: every timed wave issues valu_rounds * 64 VALU instructions
// (64 multiply-adds, or 32 exponentials and 32 multiply-adds).  cycles: device, 4 * workgroups 64-bit words.
extern "C" int kvra_probe_valu(const void* operands, void* sink, void* cycles, int workgroups, int valu_rounds,
                               int with_mfma, int with_exp, void* stream) {
  if (operands == nullptr || sink == nullptr || cycles == nullptr || workgroups < 1 || valu_rounds < 1) return -1;
  hipLaunchKernelGGL(probe_valu_kernel, dim3(workgroups), dim3(512), 0, static_cast<hipStream_t>(stream),
                     static_cast<const bf16x8*>(operands), static_cast<float*>(sink),
                     static_cast<unsigned long long*>(cycles), valu_rounds, with_mfma, with_exp);
  return static_cast<int>(hipGetLastError());
}
