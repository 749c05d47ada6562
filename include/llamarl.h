/*
 * llamarl.h -- C ABI of the MI355X (gfx950) library for the trainer-side hot
 * path of LlamaRL's asynchronous off-policy update ("AIPO", paper Sec. 6):
 *
 *   1. llamarl_token_logprobs      log pi(y_t | x, y_<t) of the sampled tokens
 *                                  under the learner, over the full vocabulary
 *   2. llamarl_offpolicy_loss_fwd  importance ratio pi/mu, one-sided clip at
 *                                  rho, advantage weighting, masked means
 *   3. llamarl_offpolicy_loss_bwd  gradients w.r.t. hidden states and LM head
 *
 * Conventions shared by every entry point
 * ---------------------------------------
 *  - All data pointers are DEVICE pointers (HIP global memory on the current
 *    device) unless a parameter says "host".  The caller owns every buffer,
 *    including the workspace; the library allocates nothing, keeps no state
 *    between calls, never synchronises and enqueues work only on `stream`
 *    (a hipStream_t passed as void*; NULL = the default stream).
 *  - Matrices are dense row-major: H [N,d], W [V,d], dH [N,d], dW [V,d].
 *    N = B*T token rows; row t belongs to generation b = t / T.
 *  - Every call validates its arguments on the host first.  If that fails it
 *    returns a non-zero status, launches nothing and leaves outputs untouched;
 *    llamarl_last_error() then returns a message (thread-local storage).
 *    LLAMARL_ERR_HIP (a launch the runtime refused) can come after earlier
 *    kernels of the same call were enqueued: outputs are then undefined.
 *  - Pointers must be 16-byte aligned (anything hipMalloc/torch returns is).
 *  - dtype LLAMARL_BF16 needs d % 8 == 0, LLAMARL_F32 needs d % 4 == 0
 *    (16-byte rows).  N, V are arbitrary (>= 1).  W may exceed 4 GiB; H must be
 *    smaller than 2 GiB (its rows are gathered with 32-bit offsets) and a
 *    256-row panel of any operand smaller than 2 GiB: LLAMARL_ERR_UNSUPPORTED
 *    otherwise (a larger batch is taken in several calls, dW accumulating).
 *  - Results are deterministic: the same inputs give the same bits, run to run
 *    (no floating-point atomics anywhere).
 */
#ifndef LLAMARL_H
#define LLAMARL_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  LLAMARL_OK = 0,
  LLAMARL_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, misaligned pointer, bad enum */
  LLAMARL_ERR_UNSUPPORTED = 2, /* shape the kernels cannot take (d not a multiple of the 16-byte row unit, ...) */
  LLAMARL_ERR_WORKSPACE = 3,   /* workspace null or smaller than llamarl_workspace_bytes() says */
  LLAMARL_ERR_HIP = 4          /* a HIP runtime call (launch, attribute) failed */
} llamarl_status;

typedef enum { LLAMARL_F32 = 0, LLAMARL_BF16 = 1 } llamarl_dtype;

/* How the importance ratio r = pi/mu is clipped.
 *  AIPO: w = min(r, rho), used as a constant weight on grad log pi
 *        (Sec. 6, display equation of the update; "clip ... from above").
 *  PPO : min(r A, clip(r, 1-eps_lo, 1+eps_hi) A), differentiated through r, so
 *        the gradient is zero on a clipped branch (App. A, display equation). */
typedef enum { LLAMARL_CLIP_AIPO = 0, LLAMARL_CLIP_PPO = 1 } llamarl_clip;

/* What the weighted token sum is divided by.  The paper writes the sum over
 * the tokens of one generation only (Sec. 6); batch aggregation is a choice. */
typedef enum {
  LLAMARL_NORM_TOKEN_MEAN = 0,  /* Z = number of valid tokens in the batch (at least 1)            */
  LLAMARL_NORM_SEQ_MEAN = 1,    /* Z_t = len(b(t)) * number of non-empty generations               */
  LLAMARL_NORM_SUM_T_MEAN_B = 2 /* Z = B: the paper's plain sum over t, averaged over generations  */
} llamarl_norm;

typedef struct {
  float rho;     /* AIPO clip constant; the paper reports rho in [2,10] works well; +inf = unclipped */
  int clip_mode; /* llamarl_clip */
  float eps_lo;  /* PPO mode only */
  float eps_hi;  /* PPO mode only */
  int norm_mode; /* llamarl_norm */
} llamarl_loss_params;

typedef enum { LLAMARL_PASS_LOGPROBS = 0, LLAMARL_PASS_LOSS_FWD = 1, LLAMARL_PASS_LOSS_BWD = 2 } llamarl_pass;

/* Bytes of device workspace the given entry point needs for these sizes
 * (for LLAMARL_PASS_LOSS_FWD pass N = B*T; d, V, dt are ignored).
 * Returns 0 for invalid sizes.  Host-only computation, no HIP call. */
size_t llamarl_workspace_bytes(int64_t N, int64_t d, int64_t V, llamarl_dtype dt, llamarl_pass pass);

/* Message for the last non-OK status returned on this thread ("" if none). */
const char* llamarl_last_error(void);

/* Library version string (static storage). */
const char* llamarl_version(void);

/*
 * Per-token log-probability of the sampled token under the learner policy
 * (Sec. 6: pi factorises token-wise; the head is z = H W^T, natural-log softmax
 * over all V entries, no bias, no scaling):
 *     lse[t]  = log sum_v exp(<H[t,:], W[v,:]>)
 *     logp[t] = <H[t,:], W[targets[t],:]> - lse[t]
 * The [N,V] logits exist only as MFMA accumulator tiles; they never reach HBM.
 *
 *   H, W      in  [N,d], [V,d] of type dt
 *   targets   in  int32 [N]
 *   mask      in  uint8 [N] or NULL (= all valid).  Rows with mask == 0, and
 *                 rows whose target is outside [0,V), get logp = lse = 0
 *                 whatever H holds there.
 *   logp,lse  out float [N]
 *   ws        scratch, >= llamarl_workspace_bytes(N,d,V,dt,LLAMARL_PASS_LOGPROBS)
 * Accumulation is fp32 for both dtypes.
 */
llamarl_status llamarl_token_logprobs(const void* H, const void* W, const int32_t* targets, const uint8_t* mask,
                                      int64_t N, int64_t d, int64_t V, llamarl_dtype dt, float* logp, float* lse,
                                      void* ws, size_t ws_bytes, void* stream);

/*
 * Importance-weighted clipped policy-gradient loss (Sec. 6 display equation;
 * App. A for the PPO mode).  With delta = logp - mu_logp, r = exp(delta):
 *     AIPO  coef[t] = -mask * min(r, rho) * A / Z_t          (= dloss/dlogp[t])
 *           loss    = sum_t coef[t] * logp[t]   (the weight is a constant:
 *                     descending this loss follows the paper's ascent update)
 *     PPO   loss    = -sum_t mask * min(r A, clip(r,1-eps_lo,1+eps_hi) A) / Z_t
 *           coef[t] = -mask * A * r / Z_t on the unclipped branch, else 0
 *
 *   logp, mu_logp  in  float [B*T]; mu_logp is the natural-log probability of
 *                      y_t under the generator, as shipped with the tokens
 *   adv            in  float [B] if adv_per_token == 0 (one advantage per
 *                      generation, broadcast over its tokens), else float [B*T]
 *   mask           in  uint8 [B*T] response mask (NULL = all valid).  Masking is
 *                      a select: NaN/Inf at masked positions never leak.
 *   targets, V     in  optional (targets may be NULL): an unmasked row whose
 *                      target is outside [0,V) is treated as masked and counted
 *   p              in  HOST pointer
 *   loss           out float [1]
 *   coef           out float [B*T]; exactly 0 at masked rows
 *   stats          out float [5]: valid tokens, mean r, clipped fraction
 *                      (r > rho strictly in AIPO mode), mean delta, bad targets
 *   ws             scratch, >= llamarl_workspace_bytes(B*T,0,0,0,LLAMARL_PASS_LOSS_FWD)
 */
llamarl_status llamarl_offpolicy_loss_fwd(const float* logp, const float* mu_logp, const float* adv,
                                          int adv_per_token, const uint8_t* mask, const int32_t* targets, int64_t V,
                                          int64_t B, int64_t T, const llamarl_loss_params* p, float* loss,
                                          float* coef, float* stats, void* ws, size_t ws_bytes, void* stream);

/*
 * llamarl_offpolicy_loss_fwd for callers that cannot allocate or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments without `ws`, same kernels, same
 * results bit for bit; the kernels' scratch (per-generation counters, per-block partial sums, a ticket: about
 * 0.5 MB) is a static device array inside the library, one copy per GPU, held until the process ends.
 *   - limits: B <= 65536 generations and B*T <= 4194304 tokens, LLAMARL_ERR_UNSUPPORTED beyond them;
 *   - allocates nothing (no hipMalloc / hipFree, no allocating library routine), clears what it needs with its
 *     own kernels (no memset node in a captured graph);
 *   - every call on a GPU shares that GPU's array: calls that overlap on one GPU (two streams, two threads) race.
 *     Calls on one stream, or ordered by events, are fine.  It works on the current device.
 *   - the first call on a device looks the array's address up (a host-side query, no stream work): make one call
 *     before capturing a graph.
 */
llamarl_status llamarl_offpolicy_loss_fwd_static(const float* logp, const float* mu_logp, const float* adv,
                                                 int adv_per_token, const uint8_t* mask, const int32_t* targets,
                                                 int64_t V, int64_t B, int64_t T, const llamarl_loss_params* p,
                                                 float* loss, float* coef, float* stats, void* stream);

/*
 * Backward of the loss through logp[t] = z[t,y_t] - lse[t] (chain rule on the
 * Sec. 6 update, which is a weighted sum of grad log pi(y_t|.)).  Logits are
 * recomputed tile by tile:
 *     dz[t,v] = grad_loss * coef[t] * (1[v == targets[t]] - exp(z[t,v] - lse[t]))
 *     dH = dz W          dW = dz^T H      (fp32 accumulation)
 * dz is staged in the workspace in type dt; the logits themselves are not.
 *
 *   H, W, targets  in  as in llamarl_token_logprobs
 *   lse            in  float [N] from llamarl_token_logprobs
 *   coef           in  float [N] from llamarl_offpolicy_loss_fwd; rows with
 *                      coef == 0 contribute nothing and get a zero dH row
 *                      whatever H, lse hold there
 *   grad_loss      in  upstream scalar dL/dloss (host value, usually 1)
 *   dH             out [N,d] of type dt
 *   dW             out [V,d] of type dW_dt (LLAMARL_F32 or dt); if
 *                      accumulate_dW != 0 the result is added to what dW holds
 *   ws             scratch, >= llamarl_workspace_bytes(N,d,V,dt,LLAMARL_PASS_LOSS_BWD)
 */
llamarl_status llamarl_offpolicy_loss_bwd(const void* H, const void* W, const int32_t* targets, const float* lse,
                                          const float* coef, float grad_loss, int64_t N, int64_t d, int64_t V,
                                          llamarl_dtype dt, void* dH, void* dW, llamarl_dtype dW_dt,
                                          int accumulate_dW, void* ws, size_t ws_bytes, void* stream);

/*
 * llamarl_offpolicy_loss_bwd with a bounded workspace.  The backward stages dz for the rows it works on; by default
 * that is every row of the batch (workspace ~ 2 * V * N bytes for bf16).  With max_rows_per_pass = R > 0 (rounded up
 * to a multiple of 256) it takes the active rows (coef != 0) R at a time: the workspace holds dz for R rows only,
 * each pass writes the dH rows of its tokens and adds its share to dW (the first pass stores, or adds if
 * accumulate_dW).  ceil(N / R) passes are enqueued whatever the number of active rows; passes past them find
 * nothing to do and cost microseconds.  A caller who knows that at most R rows are active bounds the workspace at
 * no cost; a smaller R trades it for one read-modify-write of dW per extra pass -- and, for a bf16 dW, one more
 * rounding to bf16 per pass (use dW_dt = LLAMARL_F32 when that matters).  max_rows_per_pass = 0 means N.
 * A dH row comes out of one pass only; it equals the one-pass result up to the order of its fp32 sums (where the
 * contraction's K range is cut depends on how many tiles the pass has), and is reproducible run to run like
 * everything else.
 *   ws >= llamarl_bwd_workspace_bytes(N, d, V, dt, max_rows_per_pass)   (returns 0 for invalid sizes)
 */
size_t llamarl_bwd_workspace_bytes(int64_t N, int64_t d, int64_t V, llamarl_dtype dt, int64_t max_rows_per_pass);
llamarl_status llamarl_offpolicy_loss_bwd_chunked(const void* H, const void* W, const int32_t* targets,
                                                  const float* lse, const float* coef, float grad_loss, int64_t N,
                                                  int64_t d, int64_t V, llamarl_dtype dt, void* dH, void* dW,
                                                  llamarl_dtype dW_dt, int accumulate_dW, int64_t max_rows_per_pass,
                                                  void* ws, size_t ws_bytes, void* stream);

/*
 * Vocabulary-sharded head (Sec. 8.2, Table 3: the trainer runs with model parallelism 8-32, i.e. every device
 * holds a slice of the head's vocabulary rows).  These three calls are one shard's share of the path; the exchange
 * between shards (an all-reduce of 12 bytes per token, a reduce-scatter of dH) is the caller's.  On one GPU the
 * shards can be run one after another.
 *
 * llamarl_token_logprobs_partial: W_slice holds rows [v0, v0 + V_slice) of a head with V_total rows; targets are
 * global vocabulary indices.  Per token, over the shard's logits z:
 *     m[t] = max_v z[t,v]     s[t] = sum_v exp(z[t,v] - m[t])     zt[t] = z[t, y_t] if v0 <= y_t < v0 + V_slice else 0
 * Rows with mask == 0 or a target outside [0, V_total) get (m, s, zt) = (-inf, 0, 0).
 *   m, s, zt  out float [N];  ws >= llamarl_workspace_bytes(N, d, V_slice, dt, LLAMARL_PASS_LOGPROBS)
 *
 * llamarl_merge_partials: what the all-reduce computes, for `shards` results stored shard-major ([shards][N]):
 *     M = max_p m_p    lse = M + log sum_p s_p exp(m_p - M)    logp = sum_p zt_p - lse
 * (rows dead in every shard: logp = lse = 0).  With shards = 1 it finishes a single partial call.
 *
 * llamarl_offpolicy_loss_bwd_slice: llamarl_offpolicy_loss_bwd for the shard.  lse is the GLOBAL log-sum-exp
 * (from llamarl_merge_partials), so dz[t,v] = grad_loss * coef[t] * (1[v0 + v == y_t] - exp(z[t,v] - lse[t]))
 * is the shard's slice of the full dz;  dW_slice [V_slice,d] = dz^T H is the shard's rows of dW, and
 * dH_partial [N,d] = dz W_slice is its summand of dH (the shards' partials add up to dH).
 *   ws >= llamarl_workspace_bytes(N, d, V_slice, dt, LLAMARL_PASS_LOSS_BWD)
 */
llamarl_status llamarl_token_logprobs_partial(const void* H, const void* W_slice, const int32_t* targets,
                                              const uint8_t* mask, int64_t N, int64_t d, int64_t V_slice, int64_t v0,
                                              int64_t V_total, llamarl_dtype dt, float* m, float* s, float* zt,
                                              void* ws, size_t ws_bytes, void* stream);
llamarl_status llamarl_merge_partials(const float* m, const float* s, const float* zt, int shards, int64_t N,
                                      float* logp, float* lse, void* stream);
llamarl_status llamarl_offpolicy_loss_bwd_slice(const void* H, const void* W_slice, const int32_t* targets,
                                                const float* lse, const float* coef, float grad_loss, int64_t N,
                                                int64_t d, int64_t V_slice, int64_t v0, llamarl_dtype dt,
                                                void* dH_partial, void* dW_slice, llamarl_dtype dW_dt,
                                                int accumulate_dW, void* ws, size_t ws_bytes, void* stream);

/*
 * MEASUREMENT AID, outside the method: llamarl_offpolicy_loss_bwd, which in addition records six caller-owned HIP events
 * (phase_events[0..5], HOST array of hipEvent_t passed as void*) on `stream`: [0] before the first kernel,
 * [1] after the set-up kernels (active-row list, zeroed dH rows, operand panels), [2] after the recompute + dz
 * kernel, [3] after the dH contraction (the reduction of its last round's split tiles included), [4] = [3],
 * [5] after the dW contraction.  Same results, same
 * kernels, same error behaviour (plus INVALID_ARG for a null event).  The backward's four stages are all in this
 * one call, so per-kernel rooflines of the backward can only be timed from inside it.
 */
llamarl_status llamarl_offpolicy_loss_bwd_phases(const void* H, const void* W, const int32_t* targets,
                                                 const float* lse, const float* coef, float grad_loss, int64_t N,
                                                 int64_t d, int64_t V, llamarl_dtype dt, void* dH, void* dW,
                                                 llamarl_dtype dW_dt, int accumulate_dW, void* ws, size_t ws_bytes,
                                                 void* stream, void* const* phase_events);

/*
 * MEASUREMENT AID, outside the method: runs v_mfma_f32_16x16x32_bf16 from registers only (no LDS, no memory
 * traffic) in the wave shape of the contraction kernels, one workgroup per CU, `iters` times two k-steps of 32
 * MFMAs per wavefront, and reports the flop it executed.  Timed by the caller, it gives the rate the matrix pipes of
 * this chip sustain under their own power draw: the ceiling a kernel that also moves operands can approach.
 *
 *   sink    device float [1], never written in practice
 *   flops   HOST pointer, out: floating-point operations of the launch
 */
llamarl_status llamarl_mfma_ceiling(int iters, float* sink, double* flops, void* stream);

/*
 * MEASUREMENT AID, outside the method: the loop of llamarl_mfma_ceiling in the slot order of the contraction
 * kernels' main loop, with that loop's operand traffic added back piece by piece and still without any barrier or
 * wait.  traffic bit 0: the twelve 16-byte fragment reads from LDS of every k-step; bit 1: the LDS-direct loads of
 * one 64 KB operand slab per two k-steps (from `panels`, which stays in L2).  What the rate loses against traffic = 0
 * is what that traffic costs: the chip is power-limited, so added traffic lowers the clock.
 *
 *   panels       device, 16-byte aligned, at least 4 MiB readable: two panels of 256 rows x 4096 bf16 whose values
 *                are the operands of the MFMAs (the power the matrix pipes draw depends on them)
 *   panel_bytes  bytes readable at panels (less than 4 MiB: LLAMARL_ERR_INVALID_ARG)
 *   sink, flops  as for llamarl_mfma_ceiling
 */
llamarl_status llamarl_mfma_ceiling_traffic(int traffic, int iters, const void* panels, size_t panel_bytes,
                                            float* sink, double* flops, void* stream);

/*
 * Group-mean baseline (Sec. 6: from one prompt, n generations are sampled and the baseline is the mean of their
 * rewards, constant over the tokens of a generation):
 *     adv[p,i] = r[p,i] - (1/n) sum_j r[p,j]
 * With normalise_std != 0 the result is also divided by (population std of the group + eps), the group
 * normalisation GRPO uses (the paper cites it; its own baseline is the plain mean).
 *
 *   rewards  in  float [P*n], generation i of prompt p at p*n + i
 *   adv      out float [P*n]  (may alias rewards)
 * The output is the `adv` argument of llamarl_offpolicy_loss_fwd when generations are stored prompt-major.
 */
llamarl_status llamarl_group_advantages(const float* rewards, int64_t P, int64_t n, int normalise_std, float eps,
                                        float* adv, void* stream);

/*
 * KL-regularised reward (Sec. 6: the reward of a generation is often combined with
 * lambda_KL * D_KL(pi(y|x), pi_base(y|x)) to penalise deviation from the reference policy).  The paper gives no
 * estimator; this one is the sampled-token estimate of the sequence KL, subtracted from the reward:
 *     kl[b]     = sum_t mask[b,t] * (logp[b,t] - base_logp[b,t])
 *     shaped[b] = rewards[b] - lambda_kl * kl[b]
 * base_logp is what a second llamarl_token_logprobs call returns with the reference model's hidden states and
 * head; `shaped` then feeds llamarl_group_advantages.
 *
 *   rewards         in  float [B]
 *   logp, base_logp in  float [B*T]
 *   mask            in  uint8 [B*T] or NULL (= all valid); masking is a select (NaN at masked rows is ignored)
 *   shaped          out float [B]  (may alias rewards)
 *   kl              out float [B] or NULL
 */
llamarl_status llamarl_kl_shaped_rewards(const float* rewards, const float* logp, const float* base_logp,
                                         const uint8_t* mask, int64_t B, int64_t T, float lambda_kl, float* shaped,
                                         float* kl, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LLAMARL_H */
