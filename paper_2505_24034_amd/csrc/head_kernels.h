// head_kernels.h -- the four contractions of the path and their fused epilogues.
//
//   k_fwd_partials   logits tile -> per-(row, vocab tile) online-softmax partial (max, sum of exp) and the
//                    target logit: the [N,V] logits never leave the accumulators (paper Sec. 6: log pi(y_t|.))
//   k_merge_logp     partials -> lse[t], logp[t]
//   k_bwd_dz         recomputed logits tile -> dz = g * coef * (onehot - softmax), written in both orientations
//   k_gemm_store     plain C = A B^T with a store epilogue (dH and dW)
//   k_transpose      [R,C] -> [C,R] with zero padding (W^T and H^T panels for the two backward contractions)
#pragma once
#include "gemm_nt.h"

namespace llamarl {

constexpr int EPI_LDS_HEADER = 4096;                 // per-row scalars live in the first 4 KB
constexpr int STAGE_LD = 264;                        // bf16 staging tile row stride (elements): 528 B = 33 chunks
constexpr int EPI_STAGE_BYTES = BM * STAGE_LD * 2;   // 135168
constexpr int DZ_LDS_BYTES = EPI_LDS_HEADER + EPI_STAGE_BYTES;   // 139264 <= 160 KB

__device__ __forceinline__ float half_wave_max(float v) {   // over the 32 lanes that share lane/32
  v = fmaxf(v, __shfl_xor(v, 1));
  v = fmaxf(v, __shfl_xor(v, 2));
  v = fmaxf(v, __shfl_xor(v, 4));
  v = fmaxf(v, __shfl_xor(v, 8));
  v = fmaxf(v, __shfl_xor(v, 16));
  return v;
}
__device__ __forceinline__ float half_wave_sum(float v) {
  v += __shfl_xor(v, 1);
  v += __shfl_xor(v, 2);
  v += __shfl_xor(v, 4);
  v += __shfl_xor(v, 8);
  v += __shfl_xor(v, 16);
  return v;
}

struct FwdArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  int64_t N, d, V;
  int tiles_m, tiles_n;
  int64_t n_pad;        // row stride of the partial arrays
  float* part_m;        // [tiles_n][n_pad] running max of the tile's logits
  float* part_s;        // [tiles_n][n_pad] sum of exp(logit - max)
  float* zt;            // [n_pad] target logit, written by the one tile that holds column y_t
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_fwd_partials(FwdArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn;
  tile_coords(a.tiles_m, a.tiles_n, tm, tn);
  const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
  const int rowsA = (int)min((int64_t)BM, a.N - row0);
  const int rowsB = (int)min((int64_t)BN, a.V - col0);
  typedef typename TT::store_t st;
  f32x16_t acc[TM][TN];
  gemm_nt_mainloop<TT>((const st*)a.H + row0 * a.d, a.d, rowsA, (const st*)a.W + col0 * a.d, a.d, rowsB, a.d, smem,
                       acc);

  const int tid = threadIdx.x;
  LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
  __syncthreads();
  int* s_tgt = reinterpret_cast<int*>(smem);                 // [256]
  float* s_m = reinterpret_cast<float*>(smem + 1024);        // [WAVES_N][256]
  float* s_s = s_m + WAVES_N * BM;                           // [WAVES_N][256]
  if (tid < BM) s_tgt[tid] = (tid < rowsA) ? a.targets[row0 + tid] : -1;
  __syncthreads();

  const int wave_col0 = lp.wn * WAVE_N;                      // first column of this wave inside the tile
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rib = lp.row(i, r);
      float v[TN];
      float m = -INFINITY;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        v[j] = (lp.col(j) < rowsB) ? acc[i][j][r] : -INFINITY;
        m = fmaxf(m, v[j]);
      }
      m = half_wave_max(m);
      const float m_safe = (m == -INFINITY) ? 0.f : m;
      float s = 0.f;
#pragma unroll
      for (int j = 0; j < TN; ++j) s += __expf(v[j] - m_safe);   // exp(-inf) = 0 for padded columns
      s = half_wave_sum(s);
      // target logit: at most one lane of one wave of one tile owns column y_t of this row
      const int t = s_tgt[rib] - (int)col0 - wave_col0;
      if (t >= 0 && t < WAVE_N && (t & 31) == (lp.lane & 31) && rib < rowsA && t + wave_col0 < rowsB) {
        float z = acc[i][0][r];
#pragma unroll
        for (int j = 1; j < TN; ++j)
          if ((t >> 5) == j) z = acc[i][j][r];
        a.zt[row0 + rib] = z;
      }
      if ((lp.lane & 31) == 0) {
        s_m[lp.wn * BM + rib] = m;
        s_s[lp.wn * BM + rib] = s;
      }
    }
  }
  __syncthreads();
  if (tid < rowsA) {
    float M = -INFINITY;
#pragma unroll
    for (int w = 0; w < WAVES_N; ++w) M = fmaxf(M, s_m[w * BM + tid]);
    const float M_safe = (M == -INFINITY) ? 0.f : M;
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < WAVES_N; ++w) S += s_s[w * BM + tid] * __expf(s_m[w * BM + tid] - M_safe);
    a.part_m[(int64_t)tn * a.n_pad + row0 + tid] = M;
    a.part_s[(int64_t)tn * a.n_pad + row0 + tid] = S;
  }
}

// lse[t] = log sum over vocab tiles; logp[t] = z[t,y_t] - lse[t]; masked / bad-target rows -> 0 (a select).
__global__ void k_merge_logp(const float* part_m, const float* part_s, const float* zt, const int32_t* targets,
                             const uint8_t* mask, int64_t N, int64_t V, int tiles_n, int64_t n_pad, float* logp,
                             float* lse) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= N) return;
  const int y = targets[t];
  const bool valid = (mask == nullptr || mask[t] != 0) && y >= 0 && (int64_t)y < V;
  if (!valid) {
    logp[t] = 0.f;
    lse[t] = 0.f;
    return;
  }
  float M = -INFINITY;
  for (int j = 0; j < tiles_n; ++j) M = fmaxf(M, part_m[(int64_t)j * n_pad + t]);
  float S = 0.f;
  for (int j = 0; j < tiles_n; ++j) S += part_s[(int64_t)j * n_pad + t] * expf(part_m[(int64_t)j * n_pad + t] - M);
  const float l = M + logf(S);
  lse[t] = l;
  logp[t] = zt[t] - l;
}

struct DzArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  const float* lse;
  const float* coef;
  float g;
  int64_t N, d, V;
  int tiles_m, tiles_n;
  void* dz;     // [N][ldz]   (type of H/W); columns V..ldz-1 written as zero
  int64_t ldz;
  void* dzt;    // [V][ldzt]; columns N..ldzt-1 written as zero
  int64_t ldzt;
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_bwd_dz(DzArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn;
  tile_coords(a.tiles_m, a.tiles_n, tm, tn);
  const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
  const int rowsA = (int)min((int64_t)BM, a.N - row0);
  const int rowsB = (int)min((int64_t)BN, a.V - col0);
  typedef typename TT::store_t st;
  f32x16_t acc[TM][TN];
  gemm_nt_mainloop<TT>((const st*)a.H + row0 * a.d, a.d, rowsA, (const st*)a.W + col0 * a.d, a.d, rowsB, a.d, smem,
                       acc);

  const int tid = threadIdx.x;
  LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
  __syncthreads();
  int* s_tgt = reinterpret_cast<int*>(smem);                 // [256]
  float* s_lse = reinterpret_cast<float*>(smem + 1024);      // [256]
  float* s_cg = reinterpret_cast<float*>(smem + 2048);       // [256]
  if (tid < BM) {
    const bool in = tid < rowsA;
    const float c = in ? a.g * a.coef[row0 + tid] : 0.f;
    s_tgt[tid] = in ? a.targets[row0 + tid] : -1;
    s_cg[tid] = c;
    s_lse[tid] = (c != 0.f) ? a.lse[row0 + tid] : 0.f;
  }
  __syncthreads();

  // dz in place of the logits
#pragma unroll
  for (int i = 0; i < TM; ++i) {
    __builtin_amdgcn_sched_barrier(0);   // keep the unrolled blocks apart: bounds live registers
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int rib = lp.row(i, r);
      const float c = s_cg[rib], l = s_lse[rib];
      const int t = s_tgt[rib] - (int)col0;
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int cib = lp.col(j);
        const float p = __expf(acc[i][j][r] - l);
        const float dzv = c * (((cib == t) ? 1.f : 0.f) - p);
        acc[i][j][r] = (c != 0.f && cib < rowsB) ? dzv : 0.f;   // select: masked rows / padded columns are 0
      }
    }
  }

  // how far the zero padding of each orientation reaches inside this tile
  const int dz_cols = (int)min((int64_t)BN, a.ldz - col0);     // dz[row][col]: rows < N, cols < ldz
  const int dzt_cols = (int)min((int64_t)BM, a.ldzt - row0);   // dzt[col][row]: cols < V, rows < ldzt

  if constexpr (sizeof(st) == 2) {
    uint16_t* stage = reinterpret_cast<uint16_t*>(smem + EPI_LDS_HEADER);
    // orientation 1: stage[row][col]
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int r = 0; r < 16; ++r) stage[lp.row(i, r) * STAGE_LD + lp.col(j)] = float_to_bf16_bits(acc[i][j][r]);
      }
    __syncthreads();
    uint16_t* dz = reinterpret_cast<uint16_t*>(a.dz);
    for (int q = tid; q < BM * (BN / 8); q += NTHREADS) {
      const int row = q >> 5, ch = q & 31;
      if (row < rowsA && ch * 8 < dz_cols) {
        const uint4 v = *reinterpret_cast<const uint4*>(stage + row * STAGE_LD + ch * 8);
        *reinterpret_cast<uint4*>(dz + (row0 + row) * a.ldz + col0 + ch * 8) = v;
      }
    }
    __syncthreads();
    // orientation 2: stage[col][row]; a lane holds 4 consecutive rows of one column
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 pk;
          pk.x = (uint32_t)float_to_bf16_bits(acc[i][j][q4 * 4 + 0]) |
                 ((uint32_t)float_to_bf16_bits(acc[i][j][q4 * 4 + 1]) << 16);
          pk.y = (uint32_t)float_to_bf16_bits(acc[i][j][q4 * 4 + 2]) |
                 ((uint32_t)float_to_bf16_bits(acc[i][j][q4 * 4 + 3]) << 16);
          *reinterpret_cast<uint2*>(stage + lp.col(j) * STAGE_LD + lp.row(i, q4 * 4)) = pk;
        }
      }
    __syncthreads();
    uint16_t* dzt = reinterpret_cast<uint16_t*>(a.dzt);
    for (int q = tid; q < BN * (BM / 8); q += NTHREADS) {
      const int col = q >> 5, ch = q & 31;
      if (col < rowsB && ch * 8 < dzt_cols) {
        const uint4 v = *reinterpret_cast<const uint4*>(stage + col * STAGE_LD + ch * 8);
        *reinterpret_cast<uint4*>(dzt + (col0 + col) * a.ldzt + row0 + ch * 8) = v;
      }
    }
  } else {
    float* dz = reinterpret_cast<float*>(a.dz);
    float* dzt = reinterpret_cast<float*>(a.dzt);
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int rib = lp.row(i, r), cib = lp.col(j);
          if (rib < rowsA && cib < dz_cols) dz[(row0 + rib) * a.ldz + col0 + cib] = acc[i][j][r];
          if (cib < rowsB && rib < dzt_cols) dzt[(col0 + cib) * a.ldzt + row0 + rib] = acc[i][j][r];
        }
  }
}

struct StoreArgs {
  const void* A;
  int64_t lda;
  const void* B;
  int64_t ldb;
  int64_t M, Nn, K;
  int tiles_m, tiles_n;
  void* C;
  int64_t ldc;
  int c_is_f32;
  int accumulate;
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_gemm_store(StoreArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tm, tn;
  tile_coords(a.tiles_m, a.tiles_n, tm, tn);
  const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
  const int rowsA = (int)min((int64_t)BM, a.M - row0);
  const int rowsB = (int)min((int64_t)BN, a.Nn - col0);
  typedef typename TT::store_t st;
  f32x16_t acc[TM][TN];
  gemm_nt_mainloop<TT>((const st*)a.A + row0 * a.lda, a.lda, rowsA, (const st*)a.B + col0 * a.ldb, a.ldb, rowsB, a.K,
                       smem, acc);
  const int tid = threadIdx.x;
  LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int rib = lp.row(i, r), cib = lp.col(j);
        if (rib < rowsA && cib < rowsB) {
          const int64_t idx = (row0 + rib) * a.ldc + col0 + cib;
          float v = acc[i][j][r];
          if (a.c_is_f32) {
            float* C = reinterpret_cast<float*>(a.C);
            if (a.accumulate) v += C[idx];
            C[idx] = v;
          } else {
            uint16_t* C = reinterpret_cast<uint16_t*>(a.C);
            if (a.accumulate) v += bf16_bits_to_float(C[idx]);
            C[idx] = float_to_bf16_bits(v);
          }
        }
      }
}

// out[c][r] = keep(r) ? in[r][c] : 0 for r < R, c < C; out[c][r] = 0 for R <= r < ld_out.
// keep(r) = (row_gate == nullptr || row_gate[r] != 0): rows whose gradient weight is zero must not leak NaNs.
template <typename ST>
__global__ void k_transpose(const ST* in, int64_t R, int64_t C, int64_t ld_in, ST* out, int64_t ld_out,
                            const float* row_gate) {
  __shared__ ST tile[64][65];
  const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;     // 256 threads: 64 x 4
  for (int rr = ty; rr < 64; rr += 4) {
    const int64_t r = r0 + rr, c = c0 + tx;
    ST v = 0;
    if (r < R && c < C && (row_gate == nullptr || row_gate[r] != 0.f)) v = in[r * ld_in + c];
    tile[rr][tx] = v;
  }
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 4) {
    const int64_t c = c0 + cc, r = r0 + tx;
    if (c < C && r < ld_out) out[c * ld_out + r] = tile[tx][cc];
  }
}

}  // namespace llamarl
