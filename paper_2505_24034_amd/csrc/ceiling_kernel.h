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

// ---- the same loop with the operand traffic of the contraction kernels added back, piece by piece ---------------
// What a K-contiguous main loop does per k-step besides its 32 MFMAs: twelve ds_read_b128 fragment reads, and (every
// other k-step) this thread's eight LDS-direct loads of the next 64 KB slab.  This kernel runs exactly that, in the
// main loop's slot order, with either piece switched on by TRAFFIC (bit 0: fragment reads, bit 1: slab loads), and
// with no barrier and no wait: nothing here can stall the matrix pipes for long, so what the rate loses against
// TRAFFIC = 0 is what the added traffic costs in clock -- the chip holds its power, not its frequency.
// Operands: two panels of 256 rows x CEILING_PANEL_K bf16 at `panels` (4 MiB, stays in L2); the k offset of the slab
// loads wraps inside a row.  Values computed are meaningless (slabs are overwritten while they are read); every
// access is in bounds and every wavefront runs the same `iters` iterations.
constexpr int CEILING_PANEL_K = 4096;                                        // elements per panel row (8 KB)
constexpr size_t CEILING_PANEL_BYTES = (size_t)2 * BM * CEILING_PANEL_K * 2;   // both panels

__device__ __forceinline__ void ceiling_k_step(bf16x8_t (&a)[MB], const bf16x8_t (&bc)[NB], bf16x8_t (&bn)[NB],
                                               f32x4_t (&acc)[MB][NB], const char* pa_cur, const char* pa_nxt,
                                               const char* pb_nxt, const SlabLoader<BF16>& la,
                                               const SlabLoader<BF16>& lb, char* dst, int k0, int wave, int lane,
                                               const bool READS, const bool LOADS) {   // both flags are constants once inlined
  // slot table of k_step (gemm_nt.h): a[7] of this k-step at slot 0; the next k-step's a[0], a[1] at slots 8, 9,
  // a[2..6] at slots 12, 16, .., 28, its B fragments at slots 10, 14, 18, 22; slab loads at the odd slots 11 .. 25
#pragma unroll
  for (int t = 0; t < MB * NB; ++t) {
    const int ib = t >> 2, jb = snake_col(t);
    mma(a[ib], bc[jb], acc[ib][jb]);
    LLAMARL_FENCE();
    if (READS) {
      if (t == 0) a[7] = *reinterpret_cast<const bf16x8_t*>(pa_cur + 7 * BLOCK_BYTES);
      if (t == 8) a[0] = *reinterpret_cast<const bf16x8_t*>(pa_nxt);
      if (t == 9) a[1] = *reinterpret_cast<const bf16x8_t*>(pa_nxt + BLOCK_BYTES);
      if (t >= 12 && (t & 3) == 0) a[ib - 1] = *reinterpret_cast<const bf16x8_t*>(pa_nxt + (ib - 1) * BLOCK_BYTES);
      if (t >= 10 && t <= 22 && (t & 3) == 2)
        bn[(t - 10) >> 2] = *reinterpret_cast<const bf16x8_t*>(pb_nxt + ((t - 10) >> 2) * BLOCK_BYTES);
      LLAMARL_FENCE();
    }
    if (LOADS && t >= 11 && t <= 25 && (t & 1) == 1) {
      const int n = (t - 11) >> 1;
      if (n < 4) la.issue_one(dst, n, k0, CEILING_PANEL_K, wave, lane, false);
      else lb.issue_one(dst + SLAB_A_BYTES, n - 4, k0, CEILING_PANEL_K, wave, lane, false);
      LLAMARL_FENCE();
    }
  }
}

// READS, LOADS: constants of the four kernels below once this is inlined into them
__device__ __forceinline__ void ceiling_traffic_loop(int iters, float* sink, const void* panels, char* smem,
                                                     const bool READS, const bool LOADS) {
  const int lane = threadIdx.x & 63, wave = wave_id();
  const int wm = wave / WAVES_N, wn = wave % WAVES_N;
  SlabLoader<BF16> la, lb;
  la.init(panels, CEILING_PANEL_K, BM, wave, lane);
  lb.init(reinterpret_cast<const char*>(panels) + (size_t)BM * CEILING_PANEL_K * 2, CEILING_PANEL_K, BN, wave, lane);
  // both stages start with panel data (every variant: the registers then hold the caller's operand values)
#pragma unroll
  for (int s = 0; s < 2; ++s)
#pragma unroll
    for (int n = 0; n < 4; ++n) {
      la.issue_one(smem + s * STAGE_BYTES, n, s * 64, CEILING_PANEL_K, wave, lane, false);
      lb.issue_one(smem + s * STAGE_BYTES + SLAB_A_BYTES, n, s * 64, CEILING_PANEL_K, wave, lane, false);
    }
  wait_vmcnt0();
  __syncthreads();
  // fragment addresses of TileGemm::run
  const int g = lane >> 4, l16 = lane & 15, sw = swizzle(l16);
  int a_addr[2], b_addr[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks) {
    a_addr[ks] = (wm * WAVE_M + l16) * SLAB_ROW_BYTES + (((4 * ks + g) ^ sw) * 16);
    b_addr[ks] = SLAB_A_BYTES + (wn * WAVE_N + l16) * SLAB_ROW_BYTES + (((4 * ks + g) ^ sw) * 16);
  }
  bf16x8_t a[MB], b0[NB], b1[NB];
#pragma unroll
  for (int i = 0; i < MB; ++i) a[i] = *reinterpret_cast<const bf16x8_t*>(smem + a_addr[0] + i * BLOCK_BYTES);
#pragma unroll
  for (int j = 0; j < NB; ++j) {
    b0[j] = *reinterpret_cast<const bf16x8_t*>(smem + b_addr[0] + j * BLOCK_BYTES);
    b1[j] = *reinterpret_cast<const bf16x8_t*>(smem + b_addr[1] + j * BLOCK_BYTES);
  }
  f32x4_t acc[MB][NB];
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) acc[i][j] = f32x4_t{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
    char* cur = smem + (it & 1) * STAGE_BYTES;
    const char* nxt = smem + ((it + 1) & 1) * STAGE_BYTES;
    const int k0 = (it * 64) & (CEILING_PANEL_K - 1);
    LLAMARL_FENCE();
    ceiling_k_step(a, b0, b1, acc, cur + a_addr[0], cur + a_addr[1], cur + b_addr[1], la, lb, cur, k0, wave,
                          lane, READS, false);
    ceiling_k_step(a, b1, b0, acc, cur + a_addr[1], nxt + a_addr[0], nxt + b_addr[0], la, lb, cur, k0, wave,
                          lane, READS, LOADS);
  }
  wait_vmcnt0();              // no LDS-direct load may be in flight when the workgroup gives its LDS back
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < MB; ++i)
#pragma unroll
    for (int j = 0; j < NB; ++j) t += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  if (t == 12345.678f) sink[0] = t;           // never true in practice; keeps the accumulators alive
}

// plain kernels, one per combination (dynamic LDS: MAINLOOP_LDS_BYTES, two 64 KB stages)
#define LLAMARL_CEILING_TRAFFIC_KERNEL(NAME, READS, LOADS)                                           \
  __global__ __launch_bounds__(NTHREADS) void NAME(int iters, float* sink, const void* panels) {    \
    extern __shared__ __attribute__((aligned(1024))) char smem[];                                   \
    ceiling_traffic_loop(iters, sink, panels, smem, READS, LOADS);                                  \
  }
LLAMARL_CEILING_TRAFFIC_KERNEL(k_mfma_ceiling_schedule, false, false)
LLAMARL_CEILING_TRAFFIC_KERNEL(k_mfma_ceiling_lds_reads, true, false)
LLAMARL_CEILING_TRAFFIC_KERNEL(k_mfma_ceiling_slab_loads, false, true)
LLAMARL_CEILING_TRAFFIC_KERNEL(k_mfma_ceiling_reads_and_loads, true, true)
#undef LLAMARL_CEILING_TRAFFIC_KERNEL

}  // namespace llamarl
