"""Plain fp64 CPU oracle for the trainer-side AIPO hot path (numpy only).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  It shares no code with the HIP library, and the
tests hand it inputs of the workload and its own earlier results only.

What it computes (all in float64, no blocking, no fusion, no reordering):

* token log-probabilities of the sampled tokens under the learner policy pi,
  which the paper defines token-wise and autoregressively (Sec. 6, first
  display of pi(y|x) as a product of per-token conditionals).  The LM head is
  a bias-free linear map followed by a natural-log softmax over the whole
  vocabulary: the paper never writes the head out, this is the reading taken.
* the importance ratio pi/mu per token, its one-sided clip from above by the
  constant rho, the advantage weighting and the sum over tokens (Sec. 6,
  unnumbered display equation of the AIPO update; "clip ... from above").
* the gradient of that update with respect to the hidden states and the head
  weight.  The paper states the update as a gradient, sum_t min(pi/mu, rho) *
  A * grad log pi: the clipped ratio is therefore a constant weight (no
  gradient flows through it), which is what separates AIPO from the PPO loss
  whose gradient vanishes outside the clip range (App. A, property (1)).

Conventions
-----------
N = B*T token rows, row t belongs to sequence b = t // T.
H [N,d] hidden states, W [V,d] head weight, targets [N] sampled tokens y_t,
mu_logp [N] natural-log probability of y_t under the generator mu,
adv [B] (one advantage per generation, Sec. 6 "single reward per generation")
or [B,T] (per-token advantage A(x, y_{1:t})), mask [B,T] response mask.

Floating-point inputs may be float64/float32 arrays or uint16 arrays holding
bfloat16 bit patterns; they are widened exactly to float64 first, so the
oracle reads the same numbers the device reads.

Every function is pinned by tests/test_oracle_pins.py against closed forms,
library routines (scipy log_softmax / logsumexp, torch autograd), brute-force
loops, finite differences and invariants.
"""
import numpy as np

# normalisation of the token sum (the paper gives only the sum over t of one
# generation; how generations are averaged is a reading of ours)
NORM_TOKEN_MEAN = 0   # divide by the number of valid tokens
NORM_SEQ_MEAN = 1     # mean over tokens inside a generation, then mean over generations
NORM_SUM_T_MEAN_B = 2  # paper-literal sum over t, mean over the B generations

CLIP_AIPO = 0  # w = min(ratio, rho), constant weight        (Sec. 6 display)
CLIP_PPO = 1   # min(r A, clip(r, 1-eps, 1+eps) A), differentiated (App. A display)


def widen(x):
    """Exact widening to float64.  uint16 arrays are bfloat16 bit patterns."""
    x = np.asarray(x)
    if x.dtype == np.uint16:
        return (x.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    if x.dtype in (np.float32, np.float64):
        return x.astype(np.float64, copy=False)
    raise TypeError("oracle inputs must be float64, float32 or uint16 (bf16 bits), got %s" % x.dtype)


def logits(H, W):
    """z[t,v] = <h_t, W_v>: bias-free LM head, no scaling (our reading; the
    paper only names pi(y_t | x, y_<t), Sec. 6)."""
    return widen(H) @ widen(W).T


def logsumexp_rows(Z):
    """lse_t = log sum_v exp(z[t,v]), the softmax normaliser, computed with the
    row maximum subtracted so that no exponential overflows."""
    m = Z.max(axis=1)
    return m + np.log(np.exp(Z - m[:, None]).sum(axis=1))


def token_logprobs(H, W, targets, mask=None):
    """log pi(y_t | x, y_<t) = z[t, y_t] - lse_t for every row (Sec. 6).

    Returns (logp [N], lse [N]).  Rows whose mask is 0 return logp = lse = 0
    whatever H holds there (a select, so NaNs in masked rows do not leak).
    A target outside [0, V) makes the row's logp = 0 and lse = 0 as well.
    """
    Hd, Wd = widen(H), widen(W)
    N, V = Hd.shape[0], Wd.shape[0]
    targets = np.asarray(targets).astype(np.int64).reshape(N)
    valid = np.ones(N, dtype=bool) if mask is None else (np.asarray(mask).reshape(N) != 0)
    valid = valid & (targets >= 0) & (targets < V)
    logp = np.zeros(N, dtype=np.float64)
    lse = np.zeros(N, dtype=np.float64)
    rows = np.nonzero(valid)[0]
    if rows.size:
        Z = Hd[rows] @ Wd.T
        l = logsumexp_rows(Z)
        lse[rows] = l
        logp[rows] = Z[np.arange(rows.size), targets[rows]] - l
    return logp, lse


def _normaliser(valid_bt, norm_mode):
    """Z_t [B,T]: what the weighted token sum is divided by."""
    B, T = valid_bt.shape
    if norm_mode == NORM_TOKEN_MEAN:
        return np.full((B, T), float(max(int(valid_bt.sum()), 1)))
    if norm_mode == NORM_SEQ_MEAN:
        lens = valid_bt.sum(axis=1).astype(np.float64)
        b_valid = float(max(int((lens > 0).sum()), 1))
        return np.repeat(np.maximum(lens, 1.0)[:, None] * b_valid, T, axis=1)
    if norm_mode == NORM_SUM_T_MEAN_B:
        return np.full((B, T), float(B))
    raise ValueError("unknown norm_mode %r" % (norm_mode,))


def offpolicy_loss_fwd(logp, mu_logp, adv, mask, rho, norm_mode=NORM_TOKEN_MEAN,
                       clip_mode=CLIP_AIPO, eps_lo=0.2, eps_hi=0.2, targets=None, V=None):
    """Importance-weighted, clipped policy-gradient loss (Sec. 6 display equation).

    delta_t = log pi_t - log mu_t,  r_t = exp(delta_t)          (importance ratio)
    AIPO:  w_t = min(r_t, rho)   -- clipped from above only, constant weight
           coef_t = -mask_t * w_t * A_t / Z_t   ( = dLoss/dlogp_t )
           loss   = sum_t coef_t * logp_t
      The sign makes gradient *descent* on `loss` follow the paper's ascent
      direction.  `surrogate` is a function of logp whose true derivative is
      coef (no stop-gradient needed), used for finite differences:
           -sum mask A g(delta)/Z,  g = e^delta below ln(rho), rho*(delta - ln rho + 1) above.
    PPO (App. A display): objective_t = min(r A, clip(r, 1-eps_lo, 1+eps_hi) A),
           loss = -sum mask * objective_t / Z, differentiated through r:
           coef_t = -mask * A * r / Z where the unclipped branch is active, else 0.

    adv is [B] (broadcast over the sequence) or [B,T].
    If `targets` and `V` are given, rows with a target outside [0,V) are treated
    as masked and counted in stats[4].
    Returns dict(loss, coef [B*T], stats [5], surrogate) with
    stats = (N_valid, mean ratio, fraction with r > rho (AIPO) or on a clipped
    branch (PPO), mean delta, bad-target count); means over valid tokens.
    """
    mask = np.asarray(mask)
    B, T = mask.shape
    logp = np.asarray(logp, dtype=np.float64).reshape(B, T)
    mu = np.asarray(mu_logp, dtype=np.float64).reshape(B, T)
    adv = np.asarray(adv, dtype=np.float64)
    if adv.size == B:
        A = np.repeat(adv.reshape(B, 1), T, axis=1)
    else:
        A = adv.reshape(B, T)
    valid = mask != 0
    n_bad = 0
    if targets is not None:
        tg = np.asarray(targets).astype(np.int64).reshape(B, T)
        bad = valid & ((tg < 0) | (tg >= int(V)))
        n_bad = int(bad.sum())
        valid = valid & ~bad
    Z = _normaliser(valid, norm_mode)

    with np.errstate(over="ignore", invalid="ignore"):
        delta = logp - mu
        r = np.exp(delta)
        if clip_mode == CLIP_AIPO:
            w = np.minimum(r, rho)
            coef = np.where(valid, -(w * A) / Z, 0.0)
            clipped = r > rho
            if np.isfinite(rho):
                lr = np.log(rho)
                g = np.where(delta <= lr, r, rho * (delta - lr + 1.0))
            else:
                g = r
            surrogate = float(np.where(valid, -(A * g) / Z, 0.0).sum())
            loss = float(np.where(valid, coef * logp, 0.0).sum())
        elif clip_mode == CLIP_PPO:
            rc = np.clip(r, 1.0 - eps_lo, 1.0 + eps_hi)
            obj = np.minimum(r * A, rc * A)
            active = (r * A) <= (rc * A)          # the unclipped term is the min
            coef = np.where(valid & active, -(A * r) / Z, 0.0)
            clipped = ~active
            loss = float(np.where(valid, -obj / Z, 0.0).sum())
            surrogate = loss
        else:
            raise ValueError("unknown clip_mode %r" % (clip_mode,))

    n_valid = int(valid.sum())
    den = float(max(n_valid, 1))
    stats = np.array([
        float(n_valid),
        float(np.where(valid, r, 0.0).sum()) / den,
        float((valid & clipped).sum()) / den,
        float(np.where(valid, delta, 0.0).sum()) / den,
        float(n_bad),
    ])
    return dict(loss=loss, coef=coef.reshape(B * T), stats=stats, surrogate=surrogate)


def offpolicy_loss_bwd(H, W, targets, lse, coef, grad_loss=1.0):
    """Gradient of the loss w.r.t. H and W by the chain rule through
    logp_t = z[t,y_t] - lse_t (Sec. 6: the update is a weighted sum of
    grad log pi(y_t|.)):

        dlogp_t = grad_loss * coef_t
        dz[t,v] = dlogp_t * (1[v = y_t] - exp(z[t,v] - lse_t))
        dH = dz @ W          dW = dz^T @ H

    Rows with coef_t == 0 contribute nothing (a select: their H, lse may hold
    anything).  Returns (dH [N,d], dW [V,d]).
    """
    Hd, Wd = widen(H), widen(W)
    N, d = Hd.shape
    V = Wd.shape[0]
    targets = np.asarray(targets).astype(np.int64).reshape(N)
    lse = np.asarray(lse, dtype=np.float64).reshape(N)
    dlogp = float(grad_loss) * np.asarray(coef, dtype=np.float64).reshape(N)
    dH = np.zeros((N, d), dtype=np.float64)
    dW = np.zeros((V, d), dtype=np.float64)
    rows = np.nonzero(dlogp != 0.0)[0]
    if rows.size:
        Hr = Hd[rows]
        Z = Hr @ Wd.T
        P = np.exp(Z - lse[rows][:, None])
        dZ = -P
        tg = targets[rows]
        ok = (tg >= 0) & (tg < V)
        dZ[np.nonzero(ok)[0], tg[ok]] += 1.0
        dZ *= dlogp[rows][:, None]
        dH[rows] = dZ @ Wd
        dW = dZ.T @ Hr
    return dH, dW


def token_logprobs_partial(H, W_slice, targets, v0, V_total, mask=None):
    """What one shard of a vocabulary-parallel head contributes (Sec. 8.2, Table 3: the trainer runs with model
    parallelism 8-32, so each device holds the rows [v0, v0 + V_slice) of the head weight): for every token the
    maximum m of its slice of the logits, s = sum over the slice of exp(z - m), and the target's logit zt if
    the target lies in the slice (0 otherwise).  Rows that are masked, or whose target is outside [0, V_total),
    return (m, s, zt) = (-inf, 0, 0).  Returns (m [N], s [N], zt [N])."""
    Hd, Wd = widen(H), widen(W_slice)
    N, Vs = Hd.shape[0], Wd.shape[0]
    targets = np.asarray(targets).astype(np.int64).reshape(N)
    valid = np.ones(N, dtype=bool) if mask is None else (np.asarray(mask).reshape(N) != 0)
    valid = valid & (targets >= 0) & (targets < int(V_total))
    m = np.full(N, -np.inf)
    s = np.zeros(N)
    zt = np.zeros(N)
    rows = np.nonzero(valid)[0]
    if rows.size:
        Z = Hd[rows] @ Wd.T
        mr = Z.max(axis=1)
        m[rows] = mr
        s[rows] = np.exp(Z - mr[:, None]).sum(axis=1)
        local = targets[rows] - int(v0)
        own = (local >= 0) & (local < Vs)
        zt[rows[own]] = Z[np.nonzero(own)[0], local[own]]
    return m, s, zt


def merge_partials(m_parts, s_parts, zt_parts):
    """Combine the shards' (m, s, zt) [p, N] into lse and logp: the quantities a vocabulary-parallel head would
    all-reduce (max for m, a rescaled sum for s, a plain sum for zt -- exactly one shard holds the target).
        M = max_p m_p,  lse = M + log sum_p s_p exp(m_p - M),  logp = sum_p zt_p - lse
    Rows whose every m_p is -inf (masked / bad target) return logp = lse = 0."""
    m = np.asarray(m_parts, dtype=np.float64)
    s = np.asarray(s_parts, dtype=np.float64)
    zt = np.asarray(zt_parts, dtype=np.float64)
    M = m.max(axis=0)
    live = np.isfinite(M)
    Ms = np.where(live, M, 0.0)
    with np.errstate(invalid="ignore"):
        S = np.where(np.isfinite(m), s * np.exp(m - Ms[None, :]), 0.0).sum(axis=0)
    lse = np.where(live, Ms + np.log(np.where(live, S, 1.0)), 0.0)
    logp = np.where(live, zt.sum(axis=0) - lse, 0.0)
    return logp, lse


def offpolicy_loss_bwd_slice(H, W_slice, targets, v0, lse, coef, grad_loss=1.0):
    """A shard's part of the backward: with the GLOBAL lse (from merge_partials) the slice of dz is
        dz[t,v] = grad_loss * coef_t * (1[v0 + v = y_t] - exp(z[t,v] - lse_t)),   v in the slice,
    its head-weight gradient is that shard's rows of dW, and dH_partial = dz @ W_slice is the shard's summand of
    dH (the shards' dH_partial add up to dH: the reduce-scatter of a vocabulary-parallel head).
    Returns (dH_partial [N,d], dW_slice [V_slice,d])."""
    Hd, Wd = widen(H), widen(W_slice)
    N, d = Hd.shape
    Vs = Wd.shape[0]
    targets = np.asarray(targets).astype(np.int64).reshape(N)
    lse = np.asarray(lse, dtype=np.float64).reshape(N)
    dlogp = float(grad_loss) * np.asarray(coef, dtype=np.float64).reshape(N)
    dH = np.zeros((N, d), dtype=np.float64)
    dW = np.zeros((Vs, d), dtype=np.float64)
    rows = np.nonzero(dlogp != 0.0)[0]
    if rows.size:
        Hr = Hd[rows]
        dZ = -np.exp(Hr @ Wd.T - lse[rows][:, None])
        local = targets[rows] - int(v0)
        own = (local >= 0) & (local < Vs)
        dZ[np.nonzero(own)[0], local[own]] += 1.0
        dZ *= dlogp[rows][:, None]
        dH[rows] = dZ @ Wd
        dW = dZ.T @ Hr
    return dH, dW


def group_advantages(rewards, n, normalise_std=False, eps=1e-6):
    """Group-mean baseline (Sec. 6): from one prompt n generations are sampled and the baseline is the mean of
    their rewards, constant over a generation's tokens: A_i = r_i - (1/n) sum_j r_j.  With normalise_std the
    result is divided by (population std of the group + eps) -- the GRPO normalisation the paper cites, not part
    of its own baseline.  rewards: [P*n] prompt-major.  Returns [P*n]."""
    r = np.asarray(rewards, dtype=np.float64).reshape(-1, n)
    a = r - r.mean(axis=1, keepdims=True)
    if normalise_std:
        a = a / (np.sqrt((a * a).mean(axis=1, keepdims=True)) + eps)
    return a.reshape(-1)


def kl_shaped_rewards(rewards, logp, base_logp, mask, lambda_kl):
    """KL-regularised reward (Sec. 6: the single reward per generation is combined with
    lambda_KL * D_KL(pi(y|x), pi_base(y|x)) to penalise deviation from the reference policy).  The paper gives
    no estimator; the reading taken: the sequence KL is E_{y~pi} sum_t [log pi(y_t|.) - log pi_base(y_t|.)], so
    the estimate on one sampled generation is the masked sum of the per-token log-ratios, and the penalty is
    subtracted:  kl_b = sum_t mask (logp - base_logp),  shaped_b = r_b - lambda_KL kl_b.
    logp, base_logp, mask: [B,T]; rewards: [B].  Returns (shaped [B], kl [B])."""
    m = np.asarray(mask).astype(bool)
    lr = np.where(m, np.asarray(logp, dtype=np.float64) - np.asarray(base_logp, dtype=np.float64), 0.0)
    kl = lr.sum(axis=1)
    return np.asarray(rewards, dtype=np.float64) - float(lambda_kl) * kl, kl


def aipo_step(H, W, targets, mu_logp, adv, mask, rho, norm_mode=NORM_TOKEN_MEAN, grad_loss=1.0,
              clip_mode=CLIP_AIPO, eps_lo=0.2, eps_hi=0.2):
    """The whole path in order: log-probs, loss, gradients."""
    mask = np.asarray(mask)
    B, T = mask.shape
    logp, lse = token_logprobs(H, W, targets, mask.reshape(B * T))
    V = np.asarray(W).shape[0]
    out = offpolicy_loss_fwd(logp, mu_logp, adv, mask, rho, norm_mode, clip_mode, eps_lo, eps_hi,
                             targets=targets, V=V)
    dH, dW = offpolicy_loss_bwd(H, W, targets, lse, out["coef"], grad_loss)
    out.update(logp=logp, lse=lse, dH=dH, dW=dW)
    return out
