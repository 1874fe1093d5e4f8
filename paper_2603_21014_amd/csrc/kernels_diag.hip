// Diagnostic kernel, not part of the training step: the MFMA instruction stream of the bf16
// contraction kernel (8 wavefronts per workgroup, one workgroup per CU, 32
// v_mfma_f32_32x32x16_bf16 per K step and wave on 4x2 accumulators) with its operands held in
// registers -- no LDS, no global memory.  Its rate is the ceiling the matrix cores reach on this
// board for a given operand content: the bf16 MFMA rate is limited by board power, and the power an
// MFMA draws depends on how many operand bits toggle, so the loop is run on all-zero operands and on
// pseudo-random ones.  Wave 0 of workgroup 0 brackets its loop with the shader-cycle counter and the
// constant-rate counter, which gives the shader clock the loop ran at.
#include "common.h"

namespace clt {
namespace {

typedef __bf16 bf16x8_t __attribute__((ext_vector_type(8)));
typedef float f32x16_t __attribute__((ext_vector_type(16)));
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ uint32_t mix(uint32_t h) {
  h ^= h >> 16; h *= 0x7feb352du; h ^= h >> 15; h *= 0x846ca68bu; h ^= h >> 16;
  return h;
}
// two bf16 values in (-2, 2) with random sign, exponent in {-2..0} and mantissa
__device__ __forceinline__ uint32_t rand_bf16x2(uint32_t h) {
  const uint32_t lo = (h & 0x807fu) | ((125u + (h >> 8) % 3u) << 7);
  const uint32_t g = mix(h);
  const uint32_t hi = (g & 0x807fu) | ((125u + (g >> 8) % 3u) << 7);
  return lo | (hi << 16);
}

__global__ __launch_bounds__(512) void mfma_loop_kernel(int iters, int random_operands, unsigned long long* out) {
  const uint32_t t = blockIdx.x * 512u + threadIdx.x;
  u32x4 fa[2][4], fb[2][2];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int c = 0; c < 4; ++c) fa[b][i][c] = random_operands ? rand_bf16x2(mix(t * 64u + b * 32u + i * 4u + c)) : 0u;
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int c = 0; c < 4; ++c) fb[b][j][c] = random_operands ? rand_bf16x2(mix(t * 64u + 16u + b * 32u + j * 4u + c)) : 0u;
  }
  f32x16_t acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;
  const long long c0 = clock64(), w0 = wall_clock64();
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < 4; ++s) {         // the four 16-wide slices of one K step of 64
      const int b = s & 1;
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fa[b][i]),
                                                              __builtin_bit_cast(bf16x8_t, fb[b][j]), acc[i][j], 0, 0, 0);
    }
    // keeps the operand registers from being folded into constants and the loop from being unrolled away
    asm volatile("" : "+v"(fa[0][0]), "+v"(fb[0][0]));
  }
  const long long c1 = clock64(), w1 = wall_clock64();
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) sum += acc[i][j][r];
  if (t == 0) {
    out[0] = (unsigned long long)(c1 - c0);
    out[1] = (unsigned long long)(w1 - w0);
  }
  if (sum == 1.2345678e-30f) out[2] = t;   // never true in practice; makes the accumulators observable
}

}  // namespace

hipError_t launch_mfma_loop(hipStream_t s, int workgroups, int iters, int random_operands, unsigned long long* out) {
  hipLaunchKernelGGL(mfma_loop_kernel, dim3(workgroups), dim3(512), 0, s, iters, random_operands, out);
  return hipGetLastError();
}

}  // namespace clt
