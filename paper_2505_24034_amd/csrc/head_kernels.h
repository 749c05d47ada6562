// head_kernels.h -- the four contractions of the path and their fused epilogues.
//
//   k_fwd_partials   logits tile -> per-(vocab tile, token) online-softmax partial (max, sum of exp) and the
//                    target logit: the [N,V] logits never leave the accumulators (paper Sec. 6: log pi(y_t|.))
//   k_merge_logp     partials -> lse[t], logp[t]
//   k_bwd_dz         recomputed logits tile -> dz = g * coef * (onehot - softmax), written in both orientations
//   k_gemm_store     plain contraction with a store epilogue: dW = dz^T H (K-contiguous operands) and
//                    dH = dz W (k-major operands: dz^T as written, W as the caller holds it; bf16)
//   k_transpose      [R,C] -> [C,R] with zero padding and row gather (H^T panel of the active tokens; fp32: W^T too)
//   k_compact_rows   ascending list of active token rows; k_zero_inactive_rows, k_reduce_tail: small helpers
//
// In the two logits kernels the MFMA "row" operand is W (vocab) and the "column" operand is H (tokens): an
// accumulator lane then holds ONE token per column block (column = lane % 16) and 4 vocab entries per 16x16
// block, 32 per token over the wave's 8 row blocks, so the softmax reductions over the vocabulary run inside the
// lane's own registers and finish with two cross-lane steps (lane groups l/16 hold different rows).
#pragma once
#include "gemm_nt.h"
#include "gemm_tn.h"

#include <type_traits>

namespace llamarl {

constexpr float LOG2E = 1.4426950408889634f;

// Row pitch (elements) of the two panels that live in list-position space, dz^T [V][.] and H^T [d][.]: the number
// of active rows rounded up to 64, made an ODD multiple of 64.  It is derived on the device from the active count,
// so the panels are as narrow as the batch's valid tokens allow (the k-major dH contraction walks one row pitch per
// k: a pitch sized for all N rows spreads every 64-row slab over 2 MiB of address space), and an odd multiple of
// 128 bytes never lines rows up on a power-of-two stride.  The workspace is sized for packed_pitch(N).
__host__ __device__ __forceinline__ int64_t packed_pitch(int64_t n_rows) {
  const int64_t p = (n_rows + 63) / 64;
  return ((p & 1) ? p : p + 1) * 64;
}
// Patch rows (TileSchedule::init).  Measured at the Llama-3-8B shape with patches dealt round-robin over the XCDs:
// logits kernels 4 and 8 tie (2: +1 %); dW 8 (4: +1.6 %, 2: +5 %); dH: see PATCH_ROWS_KMAJOR.
constexpr int STORE_LOAD_SLOT = 9;      // first slab-load slot of the K-contiguous store contraction (see k_step)
constexpr int PATCH_ROWS_LOGITS = 4;
constexpr int PATCH_ROWS_STORE = 8;
// dH on k-major operands, whole tiles of K = V, when the output is at most 16 tiles wide (d <= 4096): 16 x 2
// patches (8 x 4: +0.8 %, 4 x 8: +1.7 %).  Wider outputs (d = 8192, 16384) keep 8 x 4 (16 x 2: +2 - 3 % there).
constexpr int PATCH_ROWS_KMAJOR = 16;

typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef unsigned int u32x2_t __attribute__((ext_vector_type(2)));
// v_exp_f32 without the denormal-range fix-up of exp2f(): arguments here are <= 0 up to rounding, results that
// underflow are exact zeros in the sums they feed.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {   // v_cvt_pk_bf16_f32: round to nearest even
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Combine a value over the four lane groups l/16 (lanes l, l^16, l^32, l^48) without going through the LDS pipe:
// v_permlane16_swap / v_permlane32_swap of a register with a copy of itself leave "my 16-lane row's partner" and
// "my half's partner" next to the own value.
__device__ __forceinline__ float rows_max(float x) {
  const auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(p[0]), __uint_as_float(p[1]));
  const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
  const auto p = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(p[0]) + __uint_as_float(p[1]);
  const auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(q[0]) + __uint_as_float(q[1]);
}

struct FwdArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  int64_t N, d, V;        // V: rows of W as passed (the whole vocabulary, or a shard's slice of it)
  int64_t v_off;          // vocabulary index of row 0 of W (0 unless W is a slice): targets are global indices
  int tiles_v, tiles_t;   // tiles over the vocabulary (MFMA rows) and over the tokens (MFMA columns)
  int64_t n_pad;          // row stride of the partial arrays
  float* part_m;          // [tiles_v][n_pad] max of the tile's logits of a token
  float* part_s;          // [tiles_v][n_pad] sum of exp(logit - max)
  float* zt;              // [n_pad] target logit, written by the one tile that holds vocab row y_t
  const int32_t* rows;    // [n_act] active token rows, ascending: position p of the compacted list is token rows[p]
  const int32_t* n_act;   // device scalar
};  // partials and zt are indexed by compacted position, not by token

// The logits kernels gather their column operand (H rows) through the active-row list.  The list entries a lane
// needs for a tile are loaded in ONE batch, branch-free (indices clamped into the list), before the barrier that
// ends the previous tile; the compiler otherwise serialises them, each behind its own s_waitcnt, and puts them
// between the barrier and the slab requests.
template <bool QUAD, typename Args>
__device__ __forceinline__ void gather_rows(const TileSchedule& sch, const Args& a, int id, int n_act, int (&grow)[4]) {
  int tv, tt;
  sch.coords(id, tv, tt);
  const int lane = threadIdx.x & 63, wave = wave_id();
#pragma unroll
  for (int it = 0; it < 4; ++it) {
    const int p = tt * BN + SlabLoader<BF16>::lane_tile_row<QUAD>(it, wave, lane);
    grow[it] = a.rows[min(p, n_act - 1)];
  }
}
// both operand streams of tile `id` (rows = W tile, columns = gathered H rows), first two slabs
template <typename TT, bool QUAD, typename Args>
__device__ __forceinline__ void logits_fetch(TileGemm<TT>& g, const TileSchedule& sch, const Args& a, int id, int n_act,
                                             const int (&grow)[4], char* smem) {
  typedef typename TT::store_t st;
  int tv, tt;
  sch.coords(id, tv, tt);
  g.template prefetch_gathered<QUAD>((const st*)a.W + (int64_t)tv * BM * a.d, a.d,
                                     (int)min((int64_t)BM, a.V - (int64_t)tv * BM), a.H, a.d,
                                     (int)min((int64_t)BN, (int64_t)n_act - (int64_t)tt * BN), a.d, smem, grow, a.N);
}

constexpr int FWD_LDS_BYTES = MAINLOOP_LDS_BYTES + 2 * 2 * BN * 4;   // + per-token (max, sum) of the two wave rows

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_fwd_partials(FwdArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  typedef typename TT::store_t st;
  const int n_act = *a.n_act;
  TileSchedule sch;
  sch.init(a.tiles_v, (n_act + BN - 1) / BN, PATCH_ROWS_LOGITS);        // token tiles that hold active rows only
  if (!sch.has_tile()) return;                       // block-uniform
  float* s_m = reinterpret_cast<float*>(smem + MAINLOOP_LDS_BYTES);   // [2 waves along the vocabulary][256 tokens]
  float* s_s = s_m + 2 * BN;                                          // outside the slab buffers: see prefetch below

  TileGemm<TT> g;
  int id = sch.take();
  int grow[4];
  gather_rows<false>(sch, a, id, n_act, grow);
  logits_fetch<TT, false>(g, sch, a, id, n_act, grow, smem);
  while (true) {
    f32x4_t acc[MB][NB];
    g.run(smem, acc);
    // The lane's position is rebuilt from an opaque copy of the thread id after every main loop: otherwise all the
    // per-lane constants of the epilogue stay live through the loop, are spilled, and every reload waits (vmcnt) for
    // the slab requests of the next tile as well.
    int tid = threadIdx.x;
    asm volatile("" : "+v"(tid));
    const LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
    int tv, tt;
    sch.coords(id, tv, tt);
    const int64_t v0 = (int64_t)tv * BM, t0 = (int64_t)tt * BN;
    const int rowsV = (int)min((int64_t)BM, a.V - v0);
    const int rowsT = (int)min((int64_t)BN, (int64_t)n_act - t0);
    const bool more = sch.has_tile();
    // every global load of the tile boundary in two batches: list entries (this tile's tokens, the next tile's
    // gather rows), then the targets they point to -- all issued before the slab requests below, so that waiting
    // for them later does not mean waiting for those
    const int nid = more ? sch.take() : id;
    gather_rows<false>(sch, a, nid, n_act, grow);
    int ytok[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) ytok[j] = a.rows[min((int)t0 + lp.col(j), n_act - 1)];
#pragma unroll
    for (int j = 0; j < NB; ++j) ytok[j] = a.targets[ytok[j]];
    LLAMARL_FENCE();
    wait_vmcnt0();                                   // see below
    __syncthreads();                                 // every wave is done reading the slab buffers
    if (more) {                                      // start the next tile's first slabs; the epilogue hides them
      id = nid;
      logits_fetch<TT, false>(g, sch, a, id, n_act, grow, smem);
    }
    // From here to the next main loop nothing may wait on vmcnt: the counter is in order, so a wait for any load
    // (or spill reload) issued before the slab requests turns into a wait for the requests themselves, and the
    // epilogue would start only when the slabs have arrived.  Hence the explicit wait above.
    LLAMARL_FENCE();

    if (rowsV < BM) {   // last vocab tile only (block-uniform): rows past V must not enter the softmax
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r)
            if (lp.row(i, r) >= rowsV) acc[i][j][r] = -INFINITY;
    }
    const int lane_row0 = lp.row(0, 0);              // rows of this lane: lane_row0 + 16 ib + r
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int tok = lp.col(j);
      const int y = (tok < rowsT) ? ytok[j] - (int)a.v_off : -1;   // row of W that is the target (negative: none)
      const int yrow = y - (int)v0;                  // vocab row of the target inside this tile (if 0 <= . < rowsV)
      const int yrel = yrow - lane_row0;             // ... relative to this lane's first row
      float m = -INFINITY;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) m = fmaxf(m, acc[i][j][r]);
      m = rows_max(m);                               // the four lane groups hold different rows of the same token
      const float mb = (m == -INFINITY) ? 0.f : m * LOG2E;
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) s += fast_exp2(fmaf(acc[i][j][r], LOG2E, -mb));   // exp2(-inf) = 0
      s = rows_sum(s);
      // target logit: one lane of one wave of one vocab tile owns row y_t of a token; most waves own none
      const bool mine = y >= 0 && yrow < rowsV && tok < rowsT && yrel >= 0 && yrel < WAVE_M && (yrel & 12) == 0;
      if (__any(mine)) {                             // wave-uniform
        float zy = 0.f;
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r) zy = (yrel == i * 16 + r) ? acc[i][j][r] : zy;
        if (mine) a.zt[t0 + tok] = zy;
      }
      if ((lp.lane >> 4) == 0) {
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
    if (!more) break;
  }
}

// lse[t] = log sum over vocab tiles; logp[t] = z[t,y_t] - lse[t], for the active tokens (the compaction pass
// already wrote 0 for masked / bad-target rows).  HBM-bound (8 bytes per token and vocab tile): a block of 1024
// threads takes 32 list positions x 32 slices of the vocab tiles, so a row of 32 lanes reads one 128-byte line and
// there are enough loads in flight to stream.
constexpr int MERGE_TOKENS = 32, MERGE_SLICES = 32;
struct MergeArgs {
  const float* part_m;
  const float* part_s;
  const float* zt;
  const int32_t* rows;
  const int32_t* n_act;
  int tiles_v;
  int64_t n_pad;
  float* out0;            // full vocabulary: logp           shard: m   (max of the shard's logits)
  float* out1;            //                  lse                   s   (sum of exp(z - m) over the shard)
  float* out2;            //                  unused                zt  (target logit if the shard owns it, else 0)
  const int32_t* targets; // shard only
  int64_t v_off, V;       // shard only: its vocabulary range is [v_off, v_off + V)
};
// PARTIAL: W is a shard of a vocabulary-parallel head; the per-token (m, s, zt) are what the shards would
// all-reduce (paper Sec. 8.2, Table 3: trainer model parallelism 8-32), see k_merge_shards.
template <bool PARTIAL>
__global__ __launch_bounds__(MERGE_TOKENS * MERGE_SLICES) void k_merge_logp(MergeArgs a) {
  __shared__ float s_M[MERGE_SLICES][MERGE_TOKENS], s_S[MERGE_SLICES][MERGE_TOKENS];
  const int tok = threadIdx.x % MERGE_TOKENS, sl = threadIdx.x / MERGE_TOKENS;
  const int64_t p = (int64_t)blockIdx.x * MERGE_TOKENS + tok;
  const int64_t n = *a.n_act;
  if ((int64_t)blockIdx.x * MERGE_TOKENS >= n) return;        // block-uniform
  float M = -INFINITY, S = 0.f;
  if (p < n) {
    for (int j = sl; j < a.tiles_v; j += MERGE_SLICES) {
      const float m = a.part_m[(int64_t)j * a.n_pad + p], s = a.part_s[(int64_t)j * a.n_pad + p];
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
  if (sl == 0 && p < n) {
    float Mx = s_M[0][tok];
    for (int q = 1; q < MERGE_SLICES; ++q) Mx = fmaxf(Mx, s_M[q][tok]);
    float Sx = 0.f;
    for (int q = 0; q < MERGE_SLICES; ++q) Sx += (s_M[q][tok] == -INFINITY) ? 0.f : s_S[q][tok] * expf(s_M[q][tok] - Mx);
    const int64_t t = a.rows[p];
    if constexpr (PARTIAL) {
      const int64_t y = (int64_t)a.targets[t] - a.v_off;
      a.out0[t] = Mx;
      a.out1[t] = Sx;
      a.out2[t] = (y >= 0 && y < a.V) ? a.zt[p] : 0.f;
    } else {
      const float l = Mx + logf(Sx);
      a.out1[t] = l;
      a.out0[t] = a.zt[p] - l;
    }
  }
}

// The all-reduce of a vocabulary-parallel head, done here for shards that ran one after another on one GPU:
//   M = max_p m_p,  lse = M + log sum_p s_p exp(m_p - M),  logp = sum_p zt_p - lse        (m, s, zt: [shards][N])
// Rows whose every m_p is -inf (masked / bad target in every shard) get logp = lse = 0.  Shards are summed in
// ascending order: deterministic.
__global__ __launch_bounds__(256) void k_merge_shards(const float* m, const float* s, const float* zt, int shards,
                                                       int64_t N, float* logp, float* lse) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= N) return;
  float M = -INFINITY;
  for (int p = 0; p < shards; ++p) M = fmaxf(M, m[(int64_t)p * N + t]);
  float l = 0.f, lp = 0.f;
  if (M != -INFINITY) {
    float S = 0.f, Z = 0.f;
    for (int p = 0; p < shards; ++p) {
      const float mp = m[(int64_t)p * N + t];
      S += (mp == -INFINITY) ? 0.f : s[(int64_t)p * N + t] * expf(mp - M);
      Z += zt[(int64_t)p * N + t];
    }
    l = M + logf(S);
    lp = Z - l;
  }
  lse[t] = l;
  logp[t] = lp;
}

// Active-row list.  mode 0 (forward): row t is active if mask[t] != 0 (mask == nullptr: always) and its target
// is inside [0,V); inactive rows get out0 = out1 = 0 (logp, lse) here.  mode 2 (forward of a shard): the same
// list, inactive rows get (out0, out1, out2) = (-inf, 0, 0), the shard's (m, s, zt).  mode 1 (backward): active
// if coef[t] != 0.
// The list is ascending, so every later kernel is deterministic.  Block b owns rows [b, b+1) * COMPACT_BLOCK_ROWS:
// it first counts the active rows in front of its range by evaluating the predicate over them (5 bytes a row,
// served by L2 -- cheaper than a second launch or a cross-block wait for the batch sizes of a trainer step), then
// scans its own rows in order.  The last block stores the total.
constexpr int COMPACT_THREADS = 1024;
constexpr int COMPACT_BLOCK_ROWS = 4 * COMPACT_THREADS;

__device__ __forceinline__ bool row_active(int mode, const uint8_t* mask, const int32_t* targets, int64_t V,
                                           const float* coef, int64_t t) {
  if (mode == 1) return coef[t] != 0.f;
  const int y = targets[t];
  return (mask == nullptr || mask[t] != 0) && y >= 0 && (int64_t)y < V;
}

__global__ __launch_bounds__(COMPACT_THREADS) void k_compact_rows(int mode, const uint8_t* mask, const int32_t* targets,
                                                                   int64_t V, const float* coef, int64_t N,
                                                                   int32_t* rows, int32_t* n_act, float* out0,
                                                                   float* out1, float* out2) {
  __shared__ int s_wave[COMPACT_THREADS / 64];
  __shared__ int s_base;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int64_t first = (int64_t)blockIdx.x * COMPACT_BLOCK_ROWS;
  int before_block = 0;
  for (int64_t t = tid; t < first; t += COMPACT_THREADS) before_block += row_active(mode, mask, targets, V, coef, t) ? 1 : 0;
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) before_block += __shfl_xor(before_block, o);
  if (lane == 0) s_wave[wave] = before_block;
  __syncthreads();
  if (tid == 0) {
    int tot = 0;
    for (int w = 0; w < COMPACT_THREADS / 64; ++w) tot += s_wave[w];
    s_base = tot;
  }
  __syncthreads();
  for (int64_t start = first; start < min(N, first + COMPACT_BLOCK_ROWS); start += COMPACT_THREADS) {
    const int64_t t = start + tid;
    bool act = false;
    if (t < N) {
      act = row_active(mode, mask, targets, V, coef, t);
      if (mode != 1 && !act) {
        out0[t] = (mode == 2) ? -INFINITY : 0.f;
        out1[t] = 0.f;
        if (mode == 2) out2[t] = 0.f;
      }
    }
    const unsigned long long b = __ballot(act);
    const int before = __popcll(b & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wave] = __popcll(b);
    __syncthreads();
    int off = s_base;
    for (int w = 0; w < wave; ++w) off += s_wave[w];
    if (act) rows[off + before] = (int32_t)t;
    __syncthreads();
    if (tid == 0) {
      int tot = 0;
      for (int w = 0; w < COMPACT_THREADS / 64; ++w) tot += s_wave[w];
      s_base += tot;
    }
    __syncthreads();
  }
  if (tid == 0 && blockIdx.x == gridDim.x - 1) *n_act = s_base;
}

// dH rows of inactive tokens (coef == 0) are exactly zero; the dH contraction only writes the active ones.
template <typename ST>
__global__ __launch_bounds__(256) void k_zero_inactive_rows(ST* dH, const float* coef, int64_t N, int64_t d) {
  const int64_t t = blockIdx.x;
  if (coef[t] != 0.f) return;
  uint4* p = reinterpret_cast<uint4*>(dH + t * d);
  const int64_t n16 = d * (int64_t)sizeof(ST) / 16;
  for (int64_t i = threadIdx.x; i < n16; i += 256) p[i] = make_uint4(0, 0, 0, 0);
}

struct DzArgs {
  const void* H;
  const void* W;
  const int32_t* targets;
  const float* lse;
  const float* coef;
  float g;
  int64_t N, d, V;
  int64_t v_off;          // vocabulary index of row 0 of W (0 unless W is a shard's slice); lse is always global
  int tiles_v, tiles_t;
  void* dz;     // [N][ldz]  token-major (type of H/W); columns V..ldz-1 written as zero
  int64_t ldz;
  void* dzt;    // [V][packed_pitch(n_act)] vocab-major; columns past the active rows written as zero
  const int32_t* rows;    // active token rows (coef != 0), ascending; dz / dzt are indexed by list position
  const int32_t* n_act;
};

template <typename TT>
__global__ __launch_bounds__(NTHREADS) void k_bwd_dz(DzArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  typedef typename TT::store_t st;
  const int n_act = *a.n_act;
  const int64_t ldzt = packed_pitch(n_act);
  TileSchedule sch;
  sch.init(a.tiles_v, (n_act + BN - 1) / BN, PATCH_ROWS_LOGITS);
  if (!sch.has_tile()) return;                       // block-uniform: no active token at all
  // bf16: token columns are fetched quad-interleaved (a lane's four column blocks are neighbouring tokens), so the
  // vocab-major dz^T leaves straight from registers, 8 bytes per lane and whole 128-byte lines per 16 lanes.
  constexpr bool QUAD = sizeof(st) == 2;
  TileGemm<TT> g;
  int id = sch.take();
  int grow[4];
  gather_rows<QUAD>(sch, a, id, n_act, grow);
  logits_fetch<TT, QUAD>(g, sch, a, id, n_act, grow, smem);
  while (true) {
    f32x4_t acc[MB][NB];
    g.run(smem, acc);
    int tid = threadIdx.x;                           // opaque per tile: see k_fwd_partials
    asm volatile("" : "+v"(tid));
    const LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
    int tv, tt;
    sch.coords(id, tv, tt);
    const bool more = sch.has_tile();
    const int64_t v0 = (int64_t)tv * BM, t0 = (int64_t)tt * BN;
    const int rowsV = (int)min((int64_t)BM, a.V - v0);
    const int rowsT = (int)min((int64_t)BN, (int64_t)n_act - t0);
    // every global load of the tile boundary in two batches (list entries, then what they point to), all issued
    // before the slab requests below
    const int nid = more ? sch.take() : id;
    gather_rows<QUAD>(sch, a, nid, n_act, grow);
    int trow[NB];
    float tcoef[NB], tlse[NB];
    int ttgt[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j) trow[j] = a.rows[min((int)t0 + (QUAD ? lp.col_quad() + j : lp.col(j)), n_act - 1)];
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      tcoef[j] = a.coef[trow[j]];
      tlse[j] = a.lse[trow[j]];
      ttgt[j] = a.targets[trow[j]];
    }
    LLAMARL_FENCE();
    wait_vmcnt0();                                   // nothing may wait on vmcnt after the slab requests: see k_fwd_partials
    __syncthreads();                                 // every wave is done reading the slab buffers
    if (more) {                                      // the epilogue uses no LDS: fetch the next tile under it
      id = nid;
      logits_fetch<TT, QUAD>(g, sch, a, id, n_act, grow, smem);
    }
    LLAMARL_FENCE();

    // dz in place of the logits; per-token scalars live in registers (one token per lane and j)
    const int lane_row0 = lp.row(0, 0);
#pragma unroll
    for (int j = 0; j < NB; ++j) {
      const int tok = QUAD ? lp.col_quad() + j : lp.col(j);
      const bool in = tok < rowsT;
      const float c = in ? a.g * tcoef[j] : 0.f;
      const float lb = (c != 0.f) ? tlse[j] * LOG2E : 0.f;
      const int yrel = (in ? ttgt[j] - (int)a.v_off : -1) - (int)v0 - lane_row0;   // far out of range: another shard's
      const bool live = c != 0.f;                            // select: a masked token's row is exactly 0
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const float p = fast_exp2(fmaf(acc[i][j][r], LOG2E, -lb));
          acc[i][j][r] = live ? -c * p : 0.f;
        }
      // + coef at the target's own vocab row: one lane of one wave of one vocab tile per token
      const bool mine = live && yrel >= 0 && yrel < WAVE_M && (yrel & 12) == 0;
      if (__any(mine)) {                                     // wave-uniform
#pragma unroll
        for (int i = 0; i < MB; ++i)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[i][j][r] += (mine && yrel == i * 16 + r) ? c : 0.f;
      }
    }

    // how far the zero padding of each orientation reaches inside this tile
    const int dzt_cols = (int)min((int64_t)BN, ldzt - t0);   // dzt[vocab][token]: vocab < V, token < ldzt
    if constexpr (QUAD) {
      // bf16: only the vocab-major orientation exists (both gradient contractions read it).  ldzt is a multiple
      // of 64, so a token quad is never cut by the padding limit.
      // Uniform 64-bit tile base + 32-bit lane offset, made opaque once per tile so that the 32 row offsets are
      // not hoisted out of the persistent loop into scratch memory (a 256-row panel of dz^T is < 2 GiB).
      char* tile_base = reinterpret_cast<char*>(a.dzt) + (v0 * ldzt + t0) * 2;
      const uint32_t ld_b = (uint32_t)ldzt * 2u;
      uint32_t lane_off = (uint32_t)lane_row0 * ld_b + (uint32_t)lp.col_quad() * 2u;
      asm volatile("" : "+v"(lane_off));
      const bool in_cols = lp.col_quad() < dzt_cols;
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        LLAMARL_FENCE();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const int rel = i * 16 + r;
          if (lane_row0 + rel < rowsV && in_cols) {
            // non-temporal: dz^T is gigabytes that the gradient contractions stream later; written normally it
            // pushes the H and W panels this kernel re-reads out of the Infinity Cache (-5 % kernel time at
            // 21 k active rows, where the active H rows alone are 174 MB; neutral at 8.6 k)
            const u32x2_t v = {pack_bf16(acc[i][0][r], acc[i][1][r]), pack_bf16(acc[i][2][r], acc[i][3][r])};
            __builtin_nontemporal_store(v, reinterpret_cast<u32x2_t*>(tile_base + (lane_off + (uint32_t)rel * ld_b)));
          }
        }
      }
    } else {
      const int dz_cols = (int)min((int64_t)BM, a.ldz - v0);   // dz[token][vocab]:  token < N, vocab < ldz
      float* dz = reinterpret_cast<float*>(a.dz);
      float* dzt = reinterpret_cast<float*>(a.dzt);
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int vr = lp.row(i, r), tok = lp.col(j);
            const float v = (vr < rowsV) ? acc[i][j][r] : 0.f;   // padded vocab rows of the token-major copy are 0
            if (tok < rowsT && vr < dz_cols) dz[(t0 + tok) * a.ldz + v0 + vr] = v;
            if (vr < rowsV && tok < dzt_cols) dzt[(v0 + vr) * ldzt + t0 + tok] = v;
          }
    }
    if (!more) break;
  }
}

struct StoreArgs {
  const void* A;
  int64_t lda;
  const void* B;
  int64_t ldb;
  int64_t M, Nn, K;
  int tiles_n;
  void* C;
  int64_t ldc;
  int c_is_f32;
  int accumulate;
  const int32_t* m_count;   // non-null: M = *m_count (device scalar)
  const int32_t* k_count;   // non-null: K = *k_count rounded up to 64 (the operands are zero-padded that far)
  const int32_t* c_rows;    // non-null: output row r goes to row c_rows[r] of C
  const int32_t* pitch_count;  // non-null: operands flagged below have the row pitch packed_pitch(*pitch_count)
  int packed_a, packed_b;   // A / B is such a panel (lda / ldb are then ignored)
  int group_m;              // rows of a 32-tile patch (see TileSchedule)
  int max_splits;           // the tiles of the last, partial round may be split this many ways along K (1: never)
  float* part;              // [splits][tail tiles][BM x BN] fp32 partial products of split tiles
  int32_t* plan_out;        // [4] {whole, rem, splits, tiles_m}: what k_reduce_tail has to finish
};

// Work list of a store contraction.  T tiles on a persistent grid of G workgroups: the first floor(T / G) * G tiles
// are contracted whole, one per workgroup and round, and stored in their final form.  The rem = T mod G tiles left
// would occupy only rem of the G workgroups for a whole tile time; instead each is split along K (at most
// max_splits ways, at least four K slabs each) so that the parts fill the grid in a few short rounds, leave fp32
// partial products in the workspace, and k_reduce_tail adds them in split order.  This is what keeps a
// contraction with few output tiles and a long K (dH: 34 x 16 tiles, K = V) on all CUs without a split-K round trip
// for every tile, and what trims the last round of dW (8016 tiles on 256 CUs).  The assignment is fixed by the
// sizes alone: results stay bitwise reproducible.
constexpr int STORE_TAIL_ROUNDS = 4;      // rounds of split parts at the end of a store contraction, at most
struct StorePlan {
  int tiles_m, tiles_n, group_m;
  int whole, rem, splits, n_items;
  int next, stride;
  __device__ __forceinline__ void init(int tiles_m_, int tiles_n_, int group_m_, int nk, int max_splits) {
    tiles_m = tiles_m_;
    tiles_n = tiles_n_;
    group_m = group_m_;
    const int T = tiles_m * tiles_n, G = gridDim.x;
    whole = T / G * G;
    rem = T - whole;
    // split factor of the tail: the one that makes the tail shortest -- ceil(rem s / G) rounds of 1 / s tile time
    // each -- among those that keep four K slabs per part and at most STORE_TAIL_ROUNDS rounds of parts (each part
    // leaves a 256 KB block in the workspace); the smallest such factor on ties
    int best = 1, best_num = 1, best_den = 1;          // tail time best_num / best_den, in tile times
    for (int sp = 2; sp <= max_splits && rem > 0; ++sp) {
      const int rounds = (rem * sp + G - 1) / G;
      if (nk / sp < 4 || rounds > STORE_TAIL_ROUNDS) break;
      if (rounds * best_den < best_num * sp) {
        best = sp;
        best_num = rounds;
        best_den = sp;
      }
    }
    splits = best;
    n_items = whole + rem * splits;
    // 32 consecutive items per XCD and round (see TileSchedule): workgroup b sits on XCD b % 8
    const int b = blockIdx.x;
    next = (G & 7) == 0 ? (b & 7) * (G >> 3) + (b >> 3) : b;
    stride = G;
  }
  __device__ __forceinline__ bool has_item() const { return next < n_items; }
  __device__ __forceinline__ int take() {
    const int it = next;
    next += stride;
    return it;
  }
  // item -> tile id, K split and number of splits; tail items are split-major, so the 32 items an XCD holds in
  // the last round are neighbouring tiles of one K range and share operand panels like whole tiles do
  __device__ __forceinline__ void decode(int item, int& tile, int& split, int& nsplit) const {
    if (item < whole) {
      tile = item;
      split = 0;
      nsplit = 1;
    } else {
      const int j = item - whole;
      split = j / rem;
      tile = whole + (j - split * rem);
      nsplit = splits;
    }
  }
  __device__ __forceinline__ void coords(int id, int& tm, int& tn) const {   // as TileSchedule::coords
    const int per_group = group_m * tiles_n;
    const int g = id / per_group;
    const int first_m = g * group_m;
    const int gsize = min(tiles_m - first_m, group_m);
    const int in_g = id - g * per_group;
    tm = first_m + in_g % gsize;
    tn = in_g / gsize;
  }
};

template <typename TT>
struct StoreTile {     // what one work item of k_gemm_store contracts and where it goes
  int64_t row0, col0, k_lo, k_len;
  int rowsA, rowsB, split, nsplit, tail_index;
  __device__ __forceinline__ void set(const StoreArgs& a, const StorePlan& plan, int64_t M, int64_t K, int item) {
    constexpr int BK = 8 * TT::EPC;
    int tile, tm, tn;
    plan.decode(item, tile, split, nsplit);
    plan.coords(tile, tm, tn);
    tail_index = tile - plan.whole;
    row0 = (int64_t)tm * BM;
    col0 = (int64_t)tn * BN;
    rowsA = (int)min((int64_t)BM, M - row0);
    rowsB = (int)min((int64_t)BN, a.Nn - col0);
    const int nk = (int)((K + BK - 1) / BK);         // 32-bit: slabs per contraction fit an int by far
    k_lo = (int64_t)(nk * split / nsplit) * BK;
    k_len = min(K, (int64_t)(nk * (split + 1) / nsplit) * BK) - k_lo;
  }
};

template <typename TT>
__device__ __forceinline__ StoreTile<TT> store_tile_of(const StorePlan& plan, const StoreArgs& a, int item, int64_t M,
                                                       int64_t K) {
  StoreTile<TT> t;
  t.set(a, plan, M, K, item);
  return t;
}
template <typename TT>
__device__ __forceinline__ void store_fetch(TileGemm<TT, STORE_LOAD_SLOT>& g, const StorePlan& plan, const StoreArgs& a,
                                            int item, int64_t M, int64_t K, char* smem) {
  typedef typename TT::store_t st;
  const StoreTile<TT> t = store_tile_of<TT>(plan, a, item, M, K);
  if (t.k_len > 0)
    g.template prefetch<false, true>((const st*)a.A + t.row0 * a.lda + t.k_lo, a.lda, t.rowsA,
                               (const st*)a.B + t.col0 * a.ldb + t.k_lo, a.ldb, t.rowsB, t.k_len, smem);
}
// k-major operands: A is At [K][lda] (output rows are its columns), B is Bt [K][ldb]
__device__ __forceinline__ void store_fetch(TileGemmTN& g, const StorePlan& plan, const StoreArgs& a, int item, int64_t M,
                                            int64_t K, char* smem) {
  const StoreTile<BF16> t = store_tile_of<BF16>(plan, a, item, M, K);
  if (t.k_len > 0)
    g.prefetch((const uint16_t*)a.A + t.k_lo * a.lda + t.row0, a.lda, t.row0,
               (const uint16_t*)a.B + t.k_lo * a.ldb + t.col0, a.ldb, t.col0, (int)t.k_len, smem);
}

// One output element group in its final form.  MODE: 1 fp32, 2 fp32 accumulate, 3 bf16, 4 bf16 accumulate.
template <int MODE>
__device__ __forceinline__ void store_final4(char* q, float v0, float v1, float v2, float v3) {
  if (MODE <= 2) {
    float4* f = reinterpret_cast<float4*>(q);
    if (MODE == 2) {
      const float4 old = *f;
      v0 += old.x; v1 += old.y; v2 += old.z; v3 += old.w;
    }
    *f = make_float4(v0, v1, v2, v3);
  } else {
    uint2* h = reinterpret_cast<uint2*>(q);
    if (MODE == 4) {
      const uint2 old = *h;
      v0 += bf16_bits_to_float((uint16_t)(old.x & 0xffffu));
      v1 += bf16_bits_to_float((uint16_t)(old.x >> 16));
      v2 += bf16_bits_to_float((uint16_t)(old.y & 0xffffu));
      v3 += bf16_bits_to_float((uint16_t)(old.y >> 16));
    }
    uint2 o;
    o.x = pack_bf16(v0, v1);
    o.y = pack_bf16(v2, v3);
    *h = o;
  }
}
template <int MODE>
__device__ __forceinline__ void store_final1(char* q, float v) {
  if (MODE <= 2) {
    float* f = reinterpret_cast<float*>(q);
    if (MODE == 2) v += *f;
    *f = v;
  } else {
    uint16_t* h = reinterpret_cast<uint16_t*>(q);
    if (MODE == 4) v += bf16_bits_to_float(*h);
    *h = float_to_bf16_bits(v);
  }
}

// MODE (compile time): the final form of the output, see store_final4.  Split tiles of the last round leave fp32
// partial products instead (k_reduce_tail finishes them in the same MODE).
template <typename TT, bool KMAJOR, int MODE>
__global__ __launch_bounds__(NTHREADS) void k_gemm_store(StoreArgs a) {
  extern __shared__ __attribute__((aligned(1024))) char smem[];
  typedef typename TT::store_t st;
  constexpr int BK = 8 * TT::EPC;
  const int64_t M = a.m_count ? (int64_t)*a.m_count : a.M;
  const int64_t K = a.k_count ? ((int64_t)*a.k_count + 63) / 64 * 64 : a.K;
  // a later pass of a chunked backward that found no active rows: nothing to add to what the output holds
  if ((MODE == 2 || MODE == 4) && a.k_count != nullptr && K == 0) {
    if (blockIdx.x == 0 && threadIdx.x == 0) {
      a.plan_out[0] = 0; a.plan_out[1] = 0; a.plan_out[2] = 1; a.plan_out[3] = 0;
    }
    return;
  }
  if (a.pitch_count != nullptr) {                    // kernel arguments are a private copy
    const int64_t pp = packed_pitch(*a.pitch_count);
    if (a.packed_a) a.lda = pp;
    if (a.packed_b) a.ldb = pp;
  }
  const int tiles_m = (int)((M + BM - 1) / BM);
  StorePlan plan;
  plan.init(tiles_m, a.tiles_n, a.group_m, (int)((K + BK - 1) / BK), a.max_splits);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    a.plan_out[0] = plan.whole; a.plan_out[1] = plan.rem; a.plan_out[2] = plan.splits; a.plan_out[3] = tiles_m;
  }
  if (!plan.has_item()) return;                      // block-uniform
  typename std::conditional<KMAJOR, TileGemmTN, TileGemm<TT, STORE_LOAD_SLOT>>::type g;
  int id = plan.take();
  store_fetch(g, plan, a, id, M, K, smem);
  while (true) {
    f32x4_t acc[MB][NB];
    const int cur_id = id;
    if (store_tile_of<TT>(plan, a, cur_id, M, K).k_len > 0) {
      g.run(smem, acc);
    } else {                                         // nothing to contract: the product is zero
#pragma unroll
      for (int i = 0; i < MB; ++i)
#pragma unroll
        for (int j = 0; j < NB; ++j)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[i][j][r] = 0.f;
    }
    const bool more = plan.has_item();
    wait_vmcnt0();                                   // nothing may wait on vmcnt after the slab requests: see k_fwd_partials
    __syncthreads();                                 // every wave is done reading the slab buffers
    if (more) {                                      // the store epilogue uses no LDS: fetch the next tile under it
      id = plan.take();
      store_fetch(g, plan, a, id, M, K, smem);
    }
    LLAMARL_FENCE();

    const StoreTile<TT> cur = store_tile_of<TT>(plan, a, cur_id, M, K);
    int tid = threadIdx.x;                           // opaque per tile: see k_fwd_partials (a spilled per-lane constant
    asm volatile("" : "+v"(tid));                    // reloaded here would wait for the slab requests above)
    const LanePos lp{(tid >> 6) / WAVES_N, (tid >> 6) % WAVES_N, tid & 63};
    // Store epilogue, one 16-row block at a time (fences keep the unrolled blocks from piling up address registers).
    // Addresses are a uniform 64-bit tile base plus a 32-bit per-lane byte offset (a 256-row panel is < 2 GiB).
    // The offset passes through an empty asm once per tile: otherwise the 32 row offsets of a lane, which do not
    // depend on the tile, are hoisted out of the persistent loop and live in scratch memory.
    const int row_l = lp.row(0, 0);                                // lane's first row; (ib, r) adds 16 ib + r
    if (cur.nsplit > 1) {
      // a split tile of the last round (block-uniform): the whole 256 x 256 fp32 block goes to the workspace,
      // rows and columns past the matrix edge included (they hold zeros or values nobody reads)
      char* blk = reinterpret_cast<char*>(a.part + ((int64_t)cur.split * plan.rem + cur.tail_index) * (BM * BN));
      uint32_t lane_off = (uint32_t)row_l * (BN * 4) + (uint32_t)(KMAJOR ? lp.col(0) : lp.col_quad()) * 4u;
      asm volatile("" : "+v"(lane_off));
#pragma unroll
      for (int i = 0; i < MB; ++i) {
        LLAMARL_FENCE();
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          char* q = blk + (lane_off + (uint32_t)(i * 16 + r) * (BN * 4));
          if constexpr (!KMAJOR) {
            *reinterpret_cast<float4*>(q) = make_float4(acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]);
          } else {
#pragma unroll
            for (int j = 0; j < NB; ++j) reinterpret_cast<float*>(q)[j * 16] = acc[i][j][r];
          }
        }
      }
    } else {
      constexpr int esz = (MODE >= 3) ? 2 : 4;
      char* Cb = reinterpret_cast<char*>(a.C);
      const bool scatter = a.c_rows != nullptr;
      const uint32_t ldc_b = (uint32_t)a.ldc * esz;
      char* tile_base = Cb + (cur.row0 * a.ldc + cur.col0) * esz;
      if constexpr (!KMAJOR) {
        // K-contiguous operands are fetched quad-interleaved: a lane's four column blocks are neighbouring columns
        // c .. c+3, stored as one unit; 16 lanes cover 64 consecutive columns of a row -- whole 128-byte lines for
        // bf16 with no cross-lane traffic (stores that split a line over lanes of different rows measured ~0.5 ms
        // per GB slower).  The number of columns is a multiple of 4 (checked on the host): a quad is never cut.
        const int c = lp.col_quad();
        const bool in_cols = c < cur.rowsB;
        uint32_t lane_off = (uint32_t)row_l * ldc_b + (uint32_t)c * esz;
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          LLAMARL_FENCE();
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int rel = i * 16 + r;
            const int rib = row_l + rel;
            if (rib < cur.rowsA && in_cols) {
              char* q = scatter ? Cb + ((int64_t)a.c_rows[cur.row0 + rib] * a.ldc + cur.col0 + c) * esz
                                : tile_base + (lane_off + (uint32_t)rel * ldc_b);
              store_final4<MODE>(q, acc[i][0][r], acc[i][1][r], acc[i][2][r], acc[i][3][r]);
            }
          }
        }
      } else {
        // k-major operands keep the plain column order: one element per lane and column block
        uint32_t lane_off = (uint32_t)row_l * ldc_b + (uint32_t)lp.col(0) * esz;
        asm volatile("" : "+v"(lane_off));
#pragma unroll
        for (int i = 0; i < MB; ++i) {
          LLAMARL_FENCE();
#pragma unroll
          for (int r = 0; r < 4; ++r) {
            const int rel = i * 16 + r;
            const int rib = row_l + rel;
            if (rib < cur.rowsA) {
              char* rowq = scatter ? Cb + ((int64_t)a.c_rows[cur.row0 + rib] * a.ldc + cur.col0 + lp.col(0)) * esz
                                   : tile_base + (lane_off + (uint32_t)rel * ldc_b);
#pragma unroll
              for (int j = 0; j < NB; ++j)
                if (lp.col(j) < cur.rowsB) store_final1<MODE>(rowq + j * 16 * esz, acc[i][j][r]);
            }
          }
        }
      }
    }
    if (!more) break;
  }
}

// Finishes the split tiles of a store contraction's last round: C tile = sum over splits (ascending) of the fp32
// partial blocks, stored in the contraction's MODE (dtype, accumulate, row scatter).  One block per (tail tile,
// stripe of 32 rows); the plan is the one k_gemm_store wrote.
constexpr int TAIL_STRIPE_ROWS = 32;
template <int MODE>
__global__ __launch_bounds__(256) void k_reduce_tail(StoreArgs a) {
  const int whole = a.plan_out[0], rem = a.plan_out[1], splits = a.plan_out[2], tiles_m = a.plan_out[3];
  const int j = blockIdx.x;
  if (splits <= 1 || j >= rem) return;               // block-uniform
  const int64_t M = a.m_count ? (int64_t)*a.m_count : a.M;
  StorePlan plan;
  plan.tiles_m = tiles_m;
  plan.tiles_n = a.tiles_n;
  plan.group_m = a.group_m;
  int tm, tn;
  plan.coords(whole + j, tm, tn);
  const int64_t row0 = (int64_t)tm * BM, col0 = (int64_t)tn * BN;
  const int rowsA = (int)min((int64_t)BM, M - row0), rowsB = (int)min((int64_t)BN, a.Nn - col0);
  constexpr int esz = (MODE >= 3) ? 2 : 4;
  char* Cb = reinterpret_cast<char*>(a.C);
  const int c = (threadIdx.x & 63) * 4;              // 64 threads x 4 columns = one 256-column row
  const int r_in = threadIdx.x >> 6;                 // 4 rows at a time
  for (int rr = r_in; rr < TAIL_STRIPE_ROWS; rr += 4) {
    const int row = blockIdx.y * TAIL_STRIPE_ROWS + rr;
    if (row >= rowsA || c >= rowsB) continue;
    const float* p = a.part + (int64_t)j * (BM * BN) + row * BN + c;
    float4 s = *reinterpret_cast<const float4*>(p);
    for (int q = 1; q < splits; ++q) {
      const float4 v = *reinterpret_cast<const float4*>(p + (int64_t)q * rem * (BM * BN));
      s.x += v.x; s.y += v.y; s.z += v.z; s.w += v.w;
    }
    const int64_t orow = a.c_rows ? (int64_t)a.c_rows[row0 + row] : row0 + row;
    store_final4<MODE>(Cb + (orow * a.ldc + col0 + c) * esz, s.x, s.y, s.z, s.w);
  }
}

// out[c][p] = in[src(p)][c] for p < R, c < C; out[c][p] = 0 for R <= p < ld_out.
// rows == nullptr: src(p) = p and R is the host value.  Otherwise src(p) = rows[p], R = *r_count, the row pitch of
// `out` is packed_pitch(R) (ld_out is the pitch the buffer was sized for) and only the first R rounded up to 64
// columns of `out` are written (the contraction that reads it stops there).
template <typename ST>
__global__ __launch_bounds__(256) void k_transpose(const ST* in, int64_t R, int64_t C, int64_t ld_in, ST* out,
                                                    int64_t ld_out, const int32_t* rows, const int32_t* r_count) {
  if (rows != nullptr) {
    R = *r_count;
    ld_out = packed_pitch(R);
  }
  const int64_t r0 = (int64_t)blockIdx.x * 64, c0 = (int64_t)blockIdx.y * 64;
  if (rows != nullptr && r0 >= R) return;                     // block-uniform
  if constexpr (sizeof(ST) == 2) {
    // 16-bit elements, whole 16-byte chunks along both matrices' rows (block-uniform test): 16-byte loads and
    // stores, eight elements a thread, the transposition through LDS in between
    if (C % 8 == 0 && ld_in % 8 == 0 && ld_out % 8 == 0 && (reinterpret_cast<uintptr_t>(in) & 15) == 0 &&
        (reinterpret_cast<uintptr_t>(out) & 15) == 0) {
      __shared__ __attribute__((aligned(16))) uint16_t t16[64][72];
      const int q = threadIdx.x & 7, line = threadIdx.x >> 3;   // 8 chunks x 32 lines, two rounds
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int rr = line + 32 * h;
        const int64_t r = r0 + rr, c = c0 + q * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < R && c < C)
          v = *reinterpret_cast<const uint4*>(reinterpret_cast<const uint16_t*>(in) +
                                              (rows ? (int64_t)rows[r] : r) * ld_in + c);
        *reinterpret_cast<uint4*>(&t16[rr][q * 8]) = v;
      }
      __syncthreads();
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int cc = line + 32 * h;
        const int64_t c = c0 + cc, r = r0 + q * 8;
        if (c < C && r < ld_out) {
          uint32_t w[4];
#pragma unroll
          for (int j = 0; j < 4; ++j)
            w[j] = (uint32_t)t16[q * 8 + 2 * j][cc] | ((uint32_t)t16[q * 8 + 2 * j + 1][cc] << 16);
          *reinterpret_cast<uint4*>(reinterpret_cast<uint16_t*>(out) + c * ld_out + r) = make_uint4(w[0], w[1], w[2], w[3]);
        }
      }
      return;
    }
  }
  __shared__ ST tile[64][65];
  const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;     // 256 threads: 64 x 4
  for (int rr = ty; rr < 64; rr += 4) {
    const int64_t r = r0 + rr, c = c0 + tx;
    ST v = 0;
    if (r < R && c < C) v = in[(rows ? (int64_t)rows[r] : r) * ld_in + c];
    tile[rr][tx] = v;
  }
  __syncthreads();
  for (int cc = ty; cc < 64; cc += 4) {
    const int64_t c = c0 + cc, r = r0 + tx;
    if (c < C && r < ld_out) out[c * ld_out + r] = tile[tx][cc];
  }
}

}  // namespace llamarl
