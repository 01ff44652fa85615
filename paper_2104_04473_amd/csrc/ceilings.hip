// Measured ceilings of the machine, for reading roofline fractions against something the chip was seen
// to do: a register-resident MFMA loop (no memory traffic at all) and a plain 16-byte-per-lane copy.
#include "common.h"

namespace ptdp {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8_t;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16_t;

// 8 waves per workgroup, 8 independent 32x32 accumulators per wave.  RANDOM = false: two operand
// registers of small integers that never change (few toggling bits).  RANDOM = true: four A and four B
// operand sets of hash-derived values spread like N(0,1) samples in bf16, rotated so that consecutive
// instructions see different operands, as in a real GEMM.
template <bool RANDOM>
__global__ void __launch_bounds__(512) mfma_ceiling_kernel(float* sink, int iters) {
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (RANDOM) {
        const uint64_t r = mix64(kGolden * (uint64_t)(((blockIdx.x * 512 + threadIdx.x) * 4 + s) * 8 + i + 1));
        // sum of four 16-bit uniforms, centred: roughly normal with unit-order spread
        const float u = (float)(r & 0xffff) + (float)((r >> 16) & 0xffff) + (float)((r >> 32) & 0xffff) + (float)(r >> 48);
        a[s][i] = (__bf16)((u - 131070.f) * (1.f / 37837.f));
        b[s][i] = (__bf16)((float)((r >> 7) & 0xffff) * (1.f / 18918.f) - 1.732f);
      } else {
        a[s][i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[s][i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
      }
    }
  f32x16_t acc[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 8; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[RANDOM ? (j & 3) : 0], b[RANDOM ? ((j >> 1) & 3) : 0], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 8; ++j)
#pragma unroll
    for (int r = 0; r < 16; ++r) s += acc[j][r];
  if (s == 123.456f) sink[0] = s;   // keeps the loop alive without a store on the usual path
}

// The same loop on v_mfma_f32_16x16x32_bf16: 32 independent 16x16 accumulators per wave, half the FLOPs per
// instruction, so 4 * iters rounds give the FLOP count of the kernel above.
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4_t;
__global__ void __launch_bounds__(512) mfma16_ceiling_kernel(float* sink, int iters, int random) {
  bf16x8_t a[4], b[4];
#pragma unroll
  for (int s = 0; s < 4; ++s)
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      if (random) {
        const uint64_t r = mix64(kGolden * (uint64_t)(((blockIdx.x * 512 + threadIdx.x) * 4 + s) * 8 + i + 1));
        const float u = (float)(r & 0xffff) + (float)((r >> 16) & 0xffff) + (float)((r >> 32) & 0xffff) + (float)(r >> 48);
        a[s][i] = (__bf16)((u - 131070.f) * (1.f / 37837.f));
        b[s][i] = (__bf16)((float)((r >> 7) & 0xffff) * (1.f / 18918.f) - 1.732f);
      } else {
        a[s][i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[s][i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
      }
    }
  f32x4_t acc[32];
#pragma unroll
  for (int j = 0; j < 32; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) acc[j][r] = 0.f;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int j = 0; j < 32; ++j)
      acc[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[random ? (j & 3) : 0], b[random ? ((j >> 1) & 3) : 0], acc[j], 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int j = 0; j < 32; ++j)
#pragma unroll
    for (int r = 0; r < 4; ++r) s += acc[j][r];
  if (s == 123.456f) sink[0] = s;
}

// Each workgroup copies one contiguous run, four 16-byte loads per lane in flight, non-temporal accesses: the
// fastest of the forms tried (a grid-wide stride with one access per lane in flight reaches 4.6 TB/s, this 5.5).
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__global__ void __launch_bounds__(256) copy_ceiling_kernel(const u32x4_t* __restrict__ src, u32x4_t* __restrict__ dst, size_t n) {
  const size_t per = (n + gridDim.x - 1) / gridDim.x;
  const size_t b0 = (size_t)blockIdx.x * per, b1 = min(n, b0 + per);
  size_t i = b0 + threadIdx.x;
  for (; i + 3 * 256 < b1; i += 4 * 256) {
    u32x4_t v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = __builtin_nontemporal_load(src + i + u * 256);
#pragma unroll
    for (int u = 0; u < 4; ++u) __builtin_nontemporal_store(v[u], dst + i + u * 256);
  }
  for (; i < b1; i += 256) dst[i] = src[i];
}

}  // namespace ptdp

using namespace ptdp;

extern "C" {

int ptdp_ceiling_mfma(float* sink, int workgroups, int iters, int random_operands, double* flops, void* stream) {
  if (!sink || !flops) return PTDP_E_NULL_PTR;
  if (workgroups <= 0 || iters <= 0) return PTDP_E_INVALID_ARG;
  *flops = 2.0 * 32 * 32 * 16 * 8.0 * iters * 8.0 * workgroups;
  if (random_operands & 2) {   // 16x16x32: 32 accumulators x (iters / 2) rounds = the same FLOP count
    hipLaunchKernelGGL(mfma16_ceiling_kernel, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, sink, iters / 2,
                       random_operands & 1);
    *flops = 2.0 * 16 * 16 * 32 * 32.0 * (iters / 2) * 8.0 * workgroups;
    return hipGetLastError() == hipSuccess ? PTDP_OK : PTDP_E_HIP;
  }
  if (random_operands)
    hipLaunchKernelGGL(mfma_ceiling_kernel<true>, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, sink, iters);
  else
    hipLaunchKernelGGL(mfma_ceiling_kernel<false>, dim3(workgroups), dim3(512), 0, (hipStream_t)stream, sink, iters);
  return hipGetLastError() == hipSuccess ? PTDP_OK : PTDP_E_HIP;
}

int ptdp_ceiling_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst) return PTDP_E_NULL_PTR;
  if (bytes % 16 != 0 || ((uintptr_t)src & 15) || ((uintptr_t)dst & 15)) return PTDP_E_INVALID_ARG;
  if (bytes == 0) return PTDP_OK;
  hipLaunchKernelGGL(copy_ceiling_kernel, dim3(256 * 16), dim3(256), 0, (hipStream_t)stream, (const u32x4_t*)src, (u32x4_t*)dst,
                     bytes / 16);
  return hipGetLastError() == hipSuccess ? PTDP_OK : PTDP_E_HIP;
}

}  // extern "C"
