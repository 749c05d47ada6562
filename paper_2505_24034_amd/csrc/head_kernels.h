// head_kernels.h -- the four contractions of the path and their fused epilogues.
//
//   k_fwd_partials   logits tile -> per-(vocab tile, token) online-softmax partial (max, sum of exp) and the
//                    target logit: the [N,V] logits never leave the accumulators (paper Sec. 6: log pi(y_t|.))
//   k_merge_logp     partials -> lse[t], logp[t]
//   k_bwd_dz         recomputed logits tile -> dz = g * coef * (onehot - softmax), written in both orientations
//   k_gemm_store     plain C = A B^T with a store epilogue (dH and dW)
//   k_transpose      [R,C] -> [C,R] with zero padding (W^T and H^T panels for the two backward contractions)
//
// In the two logits kernels the MFMA "row" operand is W (vocab) and the "column" operand is H (tokens): an
// accumulator lane then holds ONE token (column = lane % 32) and 16 vocab entries per 32x32 block, so the
// softmax reductions over the vocabulary run inside the lane's own registers, with a single cross-lane step.
#pragma once
#include "gemm_nt.h"

namespace llamarl {

constexpr int STAGE_LD = 264;                        // bf16 staging tile row stride (elements): 528 B = 33 chunks
constexpr int EPI_STAGE_BYTES = BM * STAGE_LD * 2;   // 135168 <= 160 KB
constexpr int DZ_LDS_BYTES = EPI_STAGE_BYTES > MAINLOOP_LDS_BYTES ? EPI_STAGE_BYTES : MAINLOOP_LDS_BYTES;
constexpr float LOG2E = 1.4426950408889634f;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // v_cvt_pk_bf16_f32: round to nearest even
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

struct FwdArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  int64_t N, d, V;
  int tiles_v, tiles_t;   // tiles over the vocabulary (MFMA rows) and over the tokens (MFMA columns)
  int64_t n_pad;          // row stride of the partial arrays
  float* part_m;          // [tiles_v][n_pad] max of the tile's logits of a token
  float* part_s;          // [tiles_v][n_pad] sum of exp(logit - max)
  float* zt;              // [n_pad] target logit, written by the one tile that holds vocab row y_t
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_fwd_partials(FwdArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tv, tt;
  tile_coords(a.tiles_v, a.tiles_t, tv, tt);
  const int64_t v0 = (int64_t)tv * BM, t0 = (int64_t)tt * BN;
  const int rowsV = (int)min((int64_t)BM, a.V - v0);
  const int rowsT = (int)min((int64_t)BN, a.N - t0);
  typedef typename TT::store_t st;
  f32x16_t acc[TM][TN];
  gemm_nt_mainloop<TT>((const st*)a.W + v0 * a.d, a.d, rowsV, (const st*)a.H + t0 * a.d, a.d, rowsT, a.d, smem, acc);

  const int tid = threadIdx.x;
  LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
  __syncthreads();
  float* s_m = reinterpret_cast<float*>(smem);     // [2 waves along the vocabulary][256 tokens]
  float* s_s = s_m + 2 * BN;

#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int tok = lp.col(j);
    const int y = (tok < rowsT) ? a.targets[t0 + tok] : -1;
    const int yrow = y - (int)v0;                    // vocab row of the target inside this tile (if 0 <= . < rowsV)
    float m = -INFINITY, zy = 0.f;
    bool mine = false;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int vr = lp.row(i, r);
        const float z = acc[i][j][r];
        if (vr < rowsV) m = fmaxf(m, z);
        if (vr == yrow) { zy = z; mine = true; }
      }
    m = fmaxf(m, __shfl_xor(m, 32));
    const float mb = (m == -INFINITY) ? 0.f : m * LOG2E;
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float e = exp2f(fmaf(acc[i][j][r], LOG2E, -mb));
        s += (lp.row(i, r) < rowsV) ? e : 0.f;
      }
    s += __shfl_xor(s, 32);
    if (mine && y >= 0 && yrow < rowsV && tok < rowsT) a.zt[t0 + tok] = zy;
    if ((lp.lane >> 5) == 0) {
      s_m[lp.wm * BN + tok] = m;
      s_s[lp.wm * BN + tok] = s;
    }
  }
  __syncthreads();
  if (tid < rowsT) {
    const float m0 = s_m[tid], m1 = s_m[BN + tid];
    const float M = fmaxf(m0, m1);
    const float Mb = (M == -INFINITY) ? 0.f : M;
    const float S = s_s[tid] * __expf(m0 - Mb) + s_s[BN + tid] * __expf(m1 - Mb);
    a.part_m[(int64_t)tv * a.n_pad + t0 + tid] = M;
    a.part_s[(int64_t)tv * a.n_pad + t0 + tid] = S;
  }
}

// lse[t] = log sum over vocab tiles; logp[t] = z[t,y_t] - lse[t]; masked / bad-target rows -> 0 (a select).
// 256 threads = 64 tokens x 4 slices of the vocab-tile list.
__global__ __launch_bounds__(256) void k_merge_logp(const float* part_m, const float* part_s, const float* zt,
                                                     const int32_t* targets, const uint8_t* mask, int64_t N,
                                                     int64_t V, int tiles_v, int64_t n_pad, float* logp,
                                                     float* lse) {
  __shared__ float s_M[4][64], s_S[4][64];
  const int tok = threadIdx.x & 63, sl = threadIdx.x >> 6;
  const int64_t t = (int64_t)blockIdx.x * 64 + tok;
  float M = -INFINITY, S = 0.f;
  if (t < N) {
    for (int j = sl; j < tiles_v; j += 4) {
      const float m = part_m[(int64_t)j * n_pad + t], s = part_s[(int64_t)j * n_pad + t];
      if (m > M) {
        S = S * __expf(M - m) + s;      // exp(-inf) = 0 on the first tile
        M = m;
      } else if (m != -INFINITY) {
        S += s * __expf(m - M);
      }
    }
  }
  s_M[sl][tok] = M;
  s_S[sl][tok] = S;
  __syncthreads();
  if (sl == 0 && t < N) {
    const int y = targets[t];
    const bool valid = (mask == nullptr || mask[t] != 0) && y >= 0 && (int64_t)y < V;
    float l = 0.f, lp = 0.f;
    if (valid) {
      float Mx = s_M[0][tok];
#pragma unroll
      for (int q = 1; q < 4; ++q) Mx = fmaxf(Mx, s_M[q][tok]);
      float Sx = 0.f;
#pragma unroll
      for (int q = 0; q < 4; ++q) Sx += (s_M[q][tok] == -INFINITY) ? 0.f : s_S[q][tok] * expf(s_M[q][tok] - Mx);
      l = Mx + logf(Sx);
      lp = zt[t] - l;
    }
    lse[t] = l;
    logp[t] = lp;
  }
}

struct DzArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  const float* lse;
  const float* coef;
  float g;
  int64_t N, d, V;
  int tiles_v, tiles_t;
  void* dz;     // [N][ldz]  token-major (type of H/W); columns V..ldz-1 written as zero
  int64_t ldz;
  void* dzt;    // [V][ldzt] vocab-major; columns N..ldzt-1 written as zero
  int64_t ldzt;
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_bwd_dz(DzArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  int tv, tt;
  tile_coords(a.tiles_v, a.tiles_t, tv, tt);
  const int64_t v0 = (int64_t)tv * BM, t0 = (int64_t)tt * BN;
  const int rowsV = (int)min((int64_t)BM, a.V - v0);
  const int rowsT = (int)min((int64_t)BN, a.N - t0);
  typedef typename TT::store_t st;
  f32x16_t acc[TM][TN];
  gemm_nt_mainloop<TT>((const st*)a.W + v0 * a.d, a.d, rowsV, (const st*)a.H + t0 * a.d, a.d, rowsT, a.d, smem, acc);

  const int tid = threadIdx.x;
  LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};

  // dz in place of the logits; per-token scalars live in registers (one token per lane and j)
#pragma unroll
  for (int j = 0; j < TN; ++j) {
    const int tok = lp.col(j);
    const bool in = tok < rowsT;
    const float c = in ? a.g * a.coef[t0 + tok] : 0.f;
    const float lb = (c != 0.f) ? a.lse[t0 + tok] * LOG2E : 0.f;
    const int yrow = (in ? a.targets[t0 + tok] : -1) - (int)v0;
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int vr = lp.row(i, r);
        const float p = exp2f(fmaf(acc[i][j][r], LOG2E, -lb));
        const float dzv = c * (((vr == yrow) ? 1.f : 0.f) - p);
        acc[i][j][r] = (c != 0.f && vr < rowsV) ? dzv : 0.f;   // select: masked tokens / padded vocab rows are 0
      }
  }

  // how far the zero padding of each orientation reaches inside this tile
  const int dzt_cols = (int)min((int64_t)BN, a.ldzt - t0);   // dzt[vocab][token]: vocab < V, token < ldzt
  const int dz_cols = (int)min((int64_t)BM, a.ldz - v0);     // dz[token][vocab]:  token < N, vocab < ldz

  if constexpr (sizeof(st) == 2) {
    // bf16: pack pairs of consecutive vocab rows first (the fp32 values die here), then stage each orientation
    // through LDS so that global stores are full 16-byte chunks of contiguous rows.
    uint32_t pk[TM][TN][8];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int p = 0; p < 8; ++p) pk[i][j][p] = pack_bf16(acc[i][j][2 * p], acc[i][j][2 * p + 1]);
    __syncthreads();                                         // main-loop LDS reads are over: reuse smem
    uint16_t* stage = reinterpret_cast<uint16_t*>(smem);
    // token-major: stage[token][vocab]; a lane holds 4 consecutive vocab rows of one token = 8 bytes
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
          uint2 v;
          v.x = pk[i][j][2 * q4];
          v.y = pk[i][j][2 * q4 + 1];
          *reinterpret_cast<uint2*>(stage + lp.col(j) * STAGE_LD + lp.row(i, q4 * 4)) = v;
        }
    __syncthreads();
    uint16_t* dz = reinterpret_cast<uint16_t*>(a.dz);
    for (int q = tid; q < BN * (BM / 8); q += NTHREADS) {
      const int tok = q >> 5, ch = q & 31;
      if (tok < rowsT && ch * 8 < dz_cols) {
        const uint4 v = *reinterpret_cast<const uint4*>(stage + tok * STAGE_LD + ch * 8);
        *reinterpret_cast<uint4*>(dz + (t0 + tok) * a.ldz + v0 + ch * 8) = v;
      }
    }
    __syncthreads();
    // vocab-major: stage[vocab][token]; lanes of a half-wave hold 32 consecutive tokens
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
#pragma unroll
        for (int p = 0; p < 8; ++p) {
          stage[lp.row(i, 2 * p) * STAGE_LD + lp.col(j)] = (uint16_t)(pk[i][j][p] & 0xffffu);
          stage[lp.row(i, 2 * p + 1) * STAGE_LD + lp.col(j)] = (uint16_t)(pk[i][j][p] >> 16);
        }
    __syncthreads();
    uint16_t* dzt = reinterpret_cast<uint16_t*>(a.dzt);
    for (int q = tid; q < BM * (BN / 8); q += NTHREADS) {
      const int vr = q >> 5, ch = q & 31;
      if (vr < rowsV && ch * 8 < dzt_cols) {
        const uint4 v = *reinterpret_cast<const uint4*>(stage + vr * STAGE_LD + ch * 8);
        *reinterpret_cast<uint4*>(dzt + (v0 + vr) * a.ldzt + t0 + ch * 8) = v;
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
          const int vr = lp.row(i, r), tok = lp.col(j);
          if (tok < rowsT && vr < dz_cols) dz[(t0 + tok) * a.ldz + v0 + vr] = acc[i][j][r];
          if (vr < rowsV && tok < dzt_cols) dzt[(v0 + vr) * a.ldzt + t0 + tok] = acc[i][j][r];
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
