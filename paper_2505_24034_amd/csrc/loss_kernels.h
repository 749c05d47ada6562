// loss_kernels.h -- the streaming part of the path: importance ratio, clip, advantage weighting and the
// masked sequence / batch means (paper Sec. 6 display equation; App. A for the PPO mode).
// HBM-bound: ~21 bytes per token in, 4 out.  Two launches: per-generation lengths, then the tokens.  Reductions
// use wavefront shuffles, then one fixed-order cross-block sum in fp64 (run by whichever block finishes last), so
// results are bitwise reproducible.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace llamarl {

constexpr int LOSS_THREADS = 256;
constexpr int LOSS_ITEMS = 4;                                 // tokens per thread
constexpr int LOSS_BLOCK_TOKENS = LOSS_THREADS * LOSS_ITEMS;  // 1024
constexpr int LOSS_MAX_BLOCKS = 512;                          // k_loss_tokens strides over the batch beyond this
constexpr int LOSS_NSUM = 5;                                  // loss, sum r, clipped count, sum delta, valid count

struct LossArgs {
  const float* logp;
  const float* mu_logp;
  const float* adv;
  const uint8_t* mask;
  const int32_t* targets;
  int64_t V;
  int64_t B, T;
  int adv_per_token;
  float rho;
  int clip_mode;
  float eps_lo, eps_hi;
  int norm_mode;
  int32_t* seq_len;    // [B] valid tokens per generation
  int32_t* seq_bad;    // [B] unmasked tokens with an out-of-range target
  double* partials;    // [nblocks][LOSS_NSUM]
  int nblocks;
  unsigned int* ticket;  // blocks of k_loss_tokens that have stored their partials (zeroed by k_seq_lengths)
  float* coef;
  float* loss;
  float* stats;
};

__device__ __forceinline__ bool token_valid(const LossArgs& a, int64_t t, bool* bad) {
  const bool m = (a.mask == nullptr) || (a.mask[t] != 0);
  bool b = false;
  if (m && a.targets != nullptr) {
    const int y = a.targets[t];
    b = (y < 0) || ((int64_t)y >= a.V);
  }
  *bad = b;
  return m && !b;
}

template <typename V>
__device__ __forceinline__ V wave_sum(V v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o);
  return v;
}

// one block per generation: valid-token count and bad-target count
constexpr int SEQ_THREADS = 1024;
__global__ __launch_bounds__(SEQ_THREADS) void k_seq_lengths(LossArgs a) {
  const int b = blockIdx.x;
  int cnt = 0, nbad = 0;
  for (int64_t t = threadIdx.x; t < a.T; t += SEQ_THREADS) {
    bool bad;
    cnt += token_valid(a, (int64_t)b * a.T + t, &bad) ? 1 : 0;
    nbad += bad ? 1 : 0;
  }
  cnt = wave_sum(cnt);
  nbad = wave_sum(nbad);
  __shared__ int s_c[SEQ_THREADS / 64], s_b[SEQ_THREADS / 64];
  if ((threadIdx.x & 63) == 0) {
    s_c[threadIdx.x >> 6] = cnt;
    s_b[threadIdx.x >> 6] = nbad;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    int c = 0, d = 0;
    for (int w = 0; w < SEQ_THREADS / 64; ++w) {
      c += s_c[w];
      d += s_b[w];
    }
    a.seq_len[b] = c;
    a.seq_bad[b] = d;
    if (b == 0) *a.ticket = 0u;
  }
}

// coef[t] and per-block partial sums; the block that finishes last adds the partials up in a fixed order (by
// block index, whichever block it is), so loss and statistics are bitwise reproducible without a third launch.
__global__ __launch_bounds__(LOSS_THREADS) void k_loss_tokens(LossArgs a) {
  __shared__ long long s_red[2][LOSS_THREADS / 64];
  __shared__ double s_sum[LOSS_NSUM + 1][LOSS_THREADS / 64];
  __shared__ bool s_last;
  // every block re-derives the batch normaliser from the B per-generation counts (B is small)
  long long nv = 0, bv = 0;
  for (int64_t b = threadIdx.x; b < a.B; b += LOSS_THREADS) {
    const int l = a.seq_len[b];
    nv += l;
    bv += (l > 0) ? 1 : 0;
  }
  nv = wave_sum(nv);
  bv = wave_sum(bv);
  if ((threadIdx.x & 63) == 0) {
    s_red[0][threadIdx.x >> 6] = nv;
    s_red[1][threadIdx.x >> 6] = bv;
  }
  __syncthreads();
  nv = 0;
  bv = 0;
  for (int w = 0; w < LOSS_THREADS / 64; ++w) {
    nv += s_red[0][w];
    bv += s_red[1][w];
  }
  const float n_valid = (float)(nv > 0 ? nv : 1);
  const float b_valid = (float)(bv > 0 ? bv : 1);

  // a thread owns LOSS_ITEMS consecutive tokens: 16-byte loads of logp, mu_logp, targets (and of a per-token
  // advantage), 4 bytes of mask, one 16-byte store of coef -- every array starts 16-byte aligned and t0 is a
  // multiple of LOSS_ITEMS.  The last, partial group of the batch goes token by token.
  static_assert(LOSS_ITEMS == 4, "vector width of the token loop");
  double acc[LOSS_NSUM] = {0, 0, 0, 0, 0};
  const int64_t N = a.B * a.T;
  for (int64_t chunk = blockIdx.x; chunk * LOSS_BLOCK_TOKENS < N; chunk += gridDim.x) {
    const int64_t t0 = chunk * LOSS_BLOCK_TOKENS + (int64_t)threadIdx.x * LOSS_ITEMS;
    if (t0 >= N) break;
    const bool whole = t0 + LOSS_ITEMS <= N;
    float lp4[4], mu4[4], ad4[4];
    int tg4[4];
    uint8_t mk4[4];
    if (whole) {
      const float4 l = *reinterpret_cast<const float4*>(a.logp + t0);
      const float4 m = *reinterpret_cast<const float4*>(a.mu_logp + t0);
      lp4[0] = l.x; lp4[1] = l.y; lp4[2] = l.z; lp4[3] = l.w;
      mu4[0] = m.x; mu4[1] = m.y; mu4[2] = m.z; mu4[3] = m.w;
      if (a.mask != nullptr) {
        const uchar4 k = *reinterpret_cast<const uchar4*>(a.mask + t0);
        mk4[0] = k.x; mk4[1] = k.y; mk4[2] = k.z; mk4[3] = k.w;
      }
      if (a.targets != nullptr) {
        const int4 y = *reinterpret_cast<const int4*>(a.targets + t0);
        tg4[0] = y.x; tg4[1] = y.y; tg4[2] = y.z; tg4[3] = y.w;
      }
      if (a.adv_per_token) {
        const float4 v = *reinterpret_cast<const float4*>(a.adv + t0);
        ad4[0] = v.x; ad4[1] = v.y; ad4[2] = v.z; ad4[3] = v.w;
      }
    } else {
#pragma unroll
      for (int i = 0; i < LOSS_ITEMS; ++i) {
        const int64_t t = min(t0 + i, N - 1);
        lp4[i] = a.logp[t];
        mu4[i] = a.mu_logp[t];
        mk4[i] = a.mask != nullptr ? a.mask[t] : (uint8_t)1;
        tg4[i] = a.targets != nullptr ? a.targets[t] : 0;
        ad4[i] = a.adv_per_token ? a.adv[t] : 0.f;
      }
    }
    int64_t b = t0 / a.T;                         // generation of the first token; later ones step over the edge
    int64_t in_b = t0 - b * a.T;
    float c4[4];
#pragma unroll
    for (int i = 0; i < LOSS_ITEMS; ++i) {
      while (in_b >= a.T) {
        in_b -= a.T;
        ++b;
      }
      ++in_b;
      c4[i] = 0.f;
      if (t0 + i >= N) continue;
      const bool m = (a.mask == nullptr) || (mk4[i] != 0);
      const bool bad = m && a.targets != nullptr && (tg4[i] < 0 || (int64_t)tg4[i] >= a.V);
      if (!m || bad) continue;
      const float lp = lp4[i];
      const float delta = lp - mu4[i];
      const float r = expf(delta);
      const float A = a.adv_per_token ? ad4[i] : a.adv[b];
      float Z;
      if (a.norm_mode == 0) Z = n_valid;
      else if (a.norm_mode == 1) Z = b_valid * (float)max(a.seq_len[b], 1);
      else Z = (float)a.B;
      bool clipped;
      float term, c;
      if (a.clip_mode == 0) {
        const float w = fminf(r, a.rho);          // one-sided clip from above; w is a constant weight
        c = -(w * A) / Z;
        clipped = r > a.rho;
        term = c * lp;
      } else {
        const float rc = fminf(fmaxf(r, 1.f - a.eps_lo), 1.f + a.eps_hi);
        const float u = r * A, k = rc * A;
        const bool active = u <= k;               // the unclipped term is the min: gradient flows through r
        c = active ? -(A * r) / Z : 0.f;
        clipped = !active;
        term = -fminf(u, k) / Z;
      }
      c4[i] = c;
      acc[0] += (double)term;
      acc[1] += (double)r;
      acc[2] += clipped ? 1.0 : 0.0;
      acc[3] += (double)delta;
      acc[4] += 1.0;
    }
    if (whole) {
      *reinterpret_cast<float4*>(a.coef + t0) = make_float4(c4[0], c4[1], c4[2], c4[3]);
    } else {
#pragma unroll
      for (int i = 0; i < LOSS_ITEMS; ++i)
        if (t0 + i < N) a.coef[t0 + i] = c4[i];
    }
  }
#pragma unroll
  for (int q = 0; q < LOSS_NSUM; ++q) {
    const double v = wave_sum(acc[q]);
    if ((threadIdx.x & 63) == 0) s_sum[q][threadIdx.x >> 6] = v;
  }
  __syncthreads();
  if (threadIdx.x < LOSS_NSUM) {
    double v = 0;
    for (int w = 0; w < LOSS_THREADS / 64; ++w) v += s_sum[threadIdx.x][w];
    a.partials[(int64_t)blockIdx.x * LOSS_NSUM + threadIdx.x] = v;
  }
  // publish the partials, then take a ticket: the block that draws the last one sees everybody's.  The fence
  // makes this chip's per-XCD L2 write its dirty lines back, which is slow: one wavefront per block (the one that
  // wrote the partials) runs it, and the grid is bounded (LOSS_MAX_BLOCKS) whatever the batch size.
  if (threadIdx.x < 64) {
    __threadfence();
    if (threadIdx.x == 0) s_last = atomicAdd(a.ticket, 1u) == (unsigned int)a.nblocks - 1u;
  }
  __syncthreads();
  if (!s_last) return;                            // block-uniform
  if (threadIdx.x < 64) __threadfence();
  __syncthreads();

  double tot[LOSS_NSUM + 1] = {0, 0, 0, 0, 0, 0};
  for (int i = threadIdx.x; i < a.nblocks; i += LOSS_THREADS)
#pragma unroll
    for (int q = 0; q < LOSS_NSUM; ++q)           // device-scope loads: other CUs wrote these during this launch
      tot[q] += __hip_atomic_load(a.partials + (int64_t)i * LOSS_NSUM + q, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  for (int64_t b = threadIdx.x; b < a.B; b += LOSS_THREADS) tot[LOSS_NSUM] += (double)a.seq_bad[b];
#pragma unroll
  for (int q = 0; q <= LOSS_NSUM; ++q) {
    const double v = wave_sum(tot[q]);
    if ((threadIdx.x & 63) == 0) s_sum[q][threadIdx.x >> 6] = v;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    double t[LOSS_NSUM + 1];
    for (int q = 0; q <= LOSS_NSUM; ++q) {
      t[q] = 0;
      for (int w = 0; w < LOSS_THREADS / 64; ++w) t[q] += s_sum[q][w];
    }
    const double den = t[4] > 0 ? t[4] : 1.0;
    a.loss[0] = (float)t[0];
    a.stats[0] = (float)t[4];
    a.stats[1] = (float)(t[1] / den);
    a.stats[2] = (float)(t[2] / den);
    a.stats[3] = (float)(t[3] / den);
    a.stats[4] = (float)t[5];
  }
}

// One wavefront per prompt: mean (and optionally population std) of its n rewards by shuffles, fp64 accumulation.
__global__ __launch_bounds__(256) void k_group_advantages(const float* rewards, int64_t P, int64_t n, int normalise_std,
                                                          float eps, float* adv) {
  const int64_t p = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (p >= P) return;
  const float* r = rewards + p * n;
  double s = 0.0;
  for (int64_t i = lane; i < n; i += 64) s += (double)r[i];
  const double mean = wave_sum(s) / (double)n;
  double scale = 1.0;
  if (normalise_std) {
    double q = 0.0;
    for (int64_t i = lane; i < n; i += 64) {
      const double dlt = (double)r[i] - mean;
      q += dlt * dlt;
    }
    scale = 1.0 / (sqrt(wave_sum(q) / (double)n) + (double)eps);
  }
  for (int64_t i = lane; i < n; i += 64) adv[p * n + i] = (float)(((double)r[i] - mean) * scale);
}

// One block per generation: masked sum of the per-token log-ratios log pi - log pi_base (fp64, fixed order), then
// shaped = reward - lambda * sum.  Masking is a select, so NaN at masked positions never enters the sum.
__global__ __launch_bounds__(LOSS_THREADS) void k_kl_shaped_rewards(const float* rewards, const float* logp,
                                                                    const float* base_logp, const uint8_t* mask,
                                                                    int64_t T, float lambda_kl, float* shaped,
                                                                    float* kl) {
  __shared__ double s_w[LOSS_THREADS / 64];
  const int64_t b = blockIdx.x;
  double acc = 0.0;
  for (int64_t t = threadIdx.x; t < T; t += LOSS_THREADS) {
    const int64_t i = b * T + t;
    const bool m = (mask == nullptr) || (mask[i] != 0);
    acc += m ? ((double)logp[i] - (double)base_logp[i]) : 0.0;
  }
  acc = wave_sum(acc);
  if ((threadIdx.x & 63) == 0) s_w[threadIdx.x >> 6] = acc;
  __syncthreads();
  if (threadIdx.x == 0) {
    double k = 0.0;
    for (int w = 0; w < LOSS_THREADS / 64; ++w) k += s_w[w];
    if (kl != nullptr) kl[b] = (float)k;
    shaped[b] = (float)((double)rewards[b] - (double)lambda_kl * k);
  }
}

}  // namespace llamarl
