// ceiling_kernel.h -- measurement aid, not part of the method: what the matrix pipes of this chip sustain when
// nothing else runs.  The kernel issues the same instruction the contractions use (v_mfma_f32_16x16x32_bf16), in the
// same wave shape (8 wavefronts per workgroup, one workgroup per CU, 8 x 4 accumulator blocks per wavefront, 32
// MFMAs per k-step) from registers only: no LDS, no global loads, no barriers.  Under that load the chip runs below
// its nominal clock (it is power-limited), so this rate -- not the published peak -- is the ceiling a real kernel,
// which also has to move its operands, can approach.
#pragma once
#include "gemm_nt.h"

namespace llamarl {

constexpr int CEILING_KSTEPS_PER_ITER = 2;   // two k-steps with alternating operand registers, as in a K slab

__global__ __launch_bounds__(NTHREADS) void k_mfma_ceiling(int iters, float* sink) {
  // operands with random sign and mantissa bits and exponents spread over eight binades (what hidden states and
  // head weights look like to the datapath: its power draw depends on the bits it toggles)
  bf16x8_t a[2][MB], b[2][NB];
  uint32_t h = (uint32_t)(blockIdx.x * NTHREADS + threadIdx.x) * 2654435761u + 12345u;
  auto next_bf16 = [&h](int exp_hi) {
    h = h * 1664525u + 1013904223u;
    const uint32_t r = h >> 8;
    const uint32_t bits = ((r & 1u) << 15) | ((uint32_t)(exp_hi - (int)((r >> 1) & 7u)) << 7) | ((r >> 4) & 0x7fu);
    return __builtin_bit_cast(__bf16, (uint16_t)bits);
  };
#pragma unroll
  for (int s = 0; s < 2; ++s) {
#pragma unroll
    for (int i = 0; i < MB; ++i)
#pragma unroll
      for (int e = 0; e < 8; ++e) a[s][i][e] = next_bf16(127);     // |a| in [2^-7, 2)
#pragma unroll
    for (int j = 0; j < NB; ++j)
#pragma unroll
      for (int e = 0; e < 8; ++e) b[s][j][e] = next_bf16(121);     // |b| in [2^-13, 2^-5)
  }
  f32x4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int s = 0; s < CEILING_KSTEPS_PER_ITER; ++s)
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j) mma(a[s][i], b[s][j], acc[i][j]);
    asm volatile("" ::: "memory");            // keep the loop a loop
  }
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) t += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  if (t == 12345.678f) sink[0] = t;           // never true in practice; keeps the accumulators alive
}

}  // namespace llamarl
