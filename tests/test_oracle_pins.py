"""Pins for the fp64 oracle: closed forms, library routines, brute force,
finite differences and invariants.  None of the expected values here comes
from the oracle itself or from the HIP library."""
import math
import os

import numpy as np
import pytest
import scipy.special
import torch

from oracle import aipo_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_problem(seed, B=3, T=5, d=7, V=11):
    rng = np.random.default_rng(seed)
    N = B * T
    H = rng.standard_normal((N, d))
    W = rng.standard_normal((V, d)) / math.sqrt(d)
    tg = rng.integers(0, V, N)
    mu = np.log(rng.uniform(0.02, 0.5, N))
    adv = rng.standard_normal(B)
    lens = rng.integers(1, T + 1, B)
    mask = (np.arange(T)[None, :] < lens[:, None]).astype(np.uint8)
    return H, W, tg, mu, adv, mask


# ---------------------------------------------------------------- widening
def test_widen_bf16_bits_match_torch_conversion():
    g = torch.Generator().manual_seed(3)
    x = (torch.randn(4096, generator=g) * 10).to(torch.bfloat16)
    bits = x.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.widen(bits), x.to(torch.float64).numpy())
    special = torch.tensor([0.0, -0.0, 1.0, float("inf"), -float("inf"), 3.3895e38, 1e-40]).to(torch.bfloat16)
    sb = special.view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(orc.widen(sb), special.to(torch.float64).numpy())


def test_widen_rejects_other_types():
    with pytest.raises(TypeError):
        orc.widen(np.zeros(3, dtype=np.int32))


# ---------------------------------------------------------------- log-probs
def test_golden_two_token_example():
    gold = {}
    for line in open(os.path.join(GOLDEN, "two_token_example.txt")):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            gold[k] = float(v)
    H = np.array([[1.0], [2.0]])
    W = np.array([[0.0], [math.log(3.0)]])
    y = np.array([1, 0])
    mu = np.array([math.log(0.5), math.log(1 / 40)])
    out = orc.aipo_step(H, W, y, mu, np.array([2.0]), np.ones((1, 2), np.uint8), rho=2.0)
    got = dict(lse0=out["lse"][0], lse1=out["lse"][1], logp0=out["logp"][0], logp1=out["logp"][1],
               coef0=out["coef"][0], coef1=out["coef"][1], loss=out["loss"],
               dH0=out["dH"][0, 0], dH1=out["dH"][1, 0], dW0=out["dW"][0, 0], dW1=out["dW"][1, 0],
               mean_ratio=out["stats"][1], clip_frac=out["stats"][2], mean_log_ratio=out["stats"][3])
    for k, v in gold.items():
        assert got[k] == pytest.approx(v, rel=1e-12, abs=1e-13), k
    assert out["stats"][0] == 2 and out["stats"][4] == 0


def test_logp_matches_scipy_log_softmax_on_loop_logits():
    H, W, tg, *_ = _rand_problem(0)
    N, d = H.shape
    V = W.shape[0]
    Z = np.zeros((N, V))
    for t in range(N):            # brute-force triple loop, k ascending
        for v in range(V):
            acc = 0.0
            for k in range(d):
                acc += H[t, k] * W[v, k]
            Z[t, v] = acc
    ref = scipy.special.log_softmax(Z, axis=1)
    logp, lse = orc.token_logprobs(H, W, tg)
    assert np.allclose(logp, ref[np.arange(N), tg], rtol=0, atol=1e-13)
    assert np.allclose(lse, scipy.special.logsumexp(Z, axis=1), rtol=0, atol=1e-13)
    assert np.allclose(orc.logits(H, W), Z, rtol=0, atol=1e-13)


def test_logits_orientation_non_square():
    # a transposed operand cannot even produce this shape / these values
    H = np.array([[1.0, 2.0, 3.0]])
    W = np.array([[1.0, 0.0, 0.0], [0.0, 1.0, 0.0], [0.0, 0.0, 1.0], [1.0, 1.0, 1.0]])
    assert np.array_equal(orc.logits(H, W), np.array([[1.0, 2.0, 3.0, 6.0]]))


def test_zero_weight_gives_uniform_policy():
    for V in (2, 7, 1024):
        H = np.random.default_rng(V).standard_normal((5, 3))
        logp, lse = orc.token_logprobs(H, np.zeros((V, 3)), np.arange(5) % V)
        assert np.allclose(logp, -math.log(V), rtol=0, atol=1e-15)
        assert np.allclose(lse, math.log(V), rtol=0, atol=1e-15)


def test_two_class_head_is_log_sigmoid():
    rng = np.random.default_rng(5)
    H = rng.standard_normal((9, 4))
    W = rng.standard_normal((2, 4))
    y = rng.integers(0, 2, 9)
    z = H @ W.T
    margin = z[np.arange(9), y] - z[np.arange(9), 1 - y]
    expect = -np.logaddexp(0.0, -margin)          # log sigmoid(margin)
    logp, _ = orc.token_logprobs(H, W, y)
    assert np.allclose(logp, expect, rtol=0, atol=1e-14)


@pytest.mark.parametrize("kappa", [50.0, -50.0, 700.0])
def test_shift_invariance_via_ones_column(kappa):
    H, W, tg, *_ = _rand_problem(1)
    H = np.concatenate([H, np.ones((H.shape[0], 1))], axis=1)     # column k0 of ones
    W0 = np.concatenate([W, np.zeros((W.shape[0], 1))], axis=1)
    W1 = W0.copy()
    W1[:, -1] += kappa                                             # every logit + kappa
    lp0, lse0 = orc.token_logprobs(H, W0, tg)
    lp1, lse1 = orc.token_logprobs(H, W1, tg)
    assert np.allclose(lp0, lp1, rtol=0, atol=1e-11)
    assert np.allclose(lse1 - lse0, kappa, rtol=0, atol=1e-11)
    assert np.all(np.isfinite(lse1))


def test_probabilities_sum_to_one_over_vocab():
    H, W, *_ = _rand_problem(2, V=13)
    N, V = H.shape[0], W.shape[0]
    tot = np.zeros(N)
    for v in range(V):
        lp, _ = orc.token_logprobs(H, W, np.full(N, v))
        tot += np.exp(lp)
    assert np.allclose(tot, 1.0, rtol=0, atol=1e-13)


def test_masked_and_bad_target_rows_are_zero_even_with_nan():
    H, W, tg, *_ = _rand_problem(3)
    N = H.shape[0]
    m = np.ones(N, np.uint8)
    m[[1, 4]] = 0
    Hn = H.copy()
    Hn[1] = np.nan
    tg2 = tg.copy()
    tg2[6] = W.shape[0]      # out of range
    tg2[7] = -1
    lp, lse = orc.token_logprobs(Hn, W, tg2, m)
    ref, ref_lse = orc.token_logprobs(H, W, tg)
    keep = np.ones(N, bool)
    keep[[1, 4, 6, 7]] = False
    assert np.array_equal(lp[keep], ref[keep]) and np.array_equal(lse[keep], ref_lse[keep])
    assert np.all(lp[~keep] == 0) and np.all(lse[~keep] == 0)


def test_synthetic_logit_statistics():
    # iid N(0,1) logits: lse ~ ln V + 1/2 (log of the mean of a log-normal)
    rng = np.random.default_rng(7)
    d, V, N = 256, 4096, 64
    H = rng.standard_normal((N, d))
    W = rng.standard_normal((V, d)) / math.sqrt(d)
    _, lse = orc.token_logprobs(H, W, np.zeros(N, int))
    assert abs(lse.mean() - (math.log(V) + 0.5)) < 0.08


# ---------------------------------------------------------------- loss: ratio, clip, mask, norm
def _brute_loss(logp, mu, adv, mask, rho, norm_mode):
    B, T = mask.shape
    n_valid = sum(int(mask[b, t] != 0) for b in range(B) for t in range(T))
    lens = [sum(int(mask[b, t] != 0) for t in range(T)) for b in range(B)]
    b_valid = sum(1 for l in lens if l > 0)
    loss, coef = 0.0, [0.0] * (B * T)
    for b in range(B):
        for t in range(T):
            if mask[b, t] == 0:
                continue
            ratio = math.exp(logp[b * T + t] - mu[b * T + t])
            w = ratio if ratio < rho else rho
            if norm_mode == orc.NORM_TOKEN_MEAN:
                Z = max(n_valid, 1)
            elif norm_mode == orc.NORM_SEQ_MEAN:
                Z = max(b_valid, 1) * lens[b]
            else:
                Z = B
            coef[b * T + t] = -w * adv[b] / Z
            loss += coef[b * T + t] * logp[b * T + t]
    return loss, coef


@pytest.mark.parametrize("norm_mode", [orc.NORM_TOKEN_MEAN, orc.NORM_SEQ_MEAN, orc.NORM_SUM_T_MEAN_B])
@pytest.mark.parametrize("rho", [1.0, 2.0, 10.0])
def test_loss_against_python_loop(norm_mode, rho):
    H, W, tg, mu, adv, mask = _rand_problem(11)
    mask[2, :] = 0                       # one empty generation
    logp, _ = orc.token_logprobs(H, W, tg, mask.reshape(-1))
    mu = logp + np.random.default_rng(1).normal(0, 0.8, logp.shape)
    out = orc.offpolicy_loss_fwd(logp, mu, adv, mask, rho, norm_mode)
    loss, coef = _brute_loss(logp, mu, adv, mask, rho, norm_mode)
    assert out["loss"] == pytest.approx(loss, rel=1e-12, abs=1e-14)
    assert np.allclose(out["coef"], coef, rtol=1e-13, atol=0)
    assert (out["stats"][2] > 0) or rho >= 10.0


def test_on_policy_reduces_to_vanilla_policy_gradient():
    # the paper's on-policy baseline is the same estimator without the IS correction (Sec. 8.3)
    H, W, tg, mu, adv, mask = _rand_problem(12)
    logp, _ = orc.token_logprobs(H, W, tg)
    out = orc.offpolicy_loss_fwd(logp, logp.copy(), adv, mask, rho=2.0)
    B, T = mask.shape
    nv = mask.sum()
    A = np.repeat(adv, T)
    m = mask.reshape(-1).astype(float)
    assert np.allclose(out["coef"], -m * A / nv, rtol=1e-15, atol=0)
    assert out["loss"] == pytest.approx(float(-(m * A * logp).sum() / nv), rel=1e-13)
    assert out["stats"][1] == pytest.approx(1.0) and out["stats"][2] == 0 and out["stats"][3] == 0


def test_clip_engages_exactly_at_rho_and_never_from_below():
    rho, h = 3.0, 1e-3
    delta = np.array([math.log(rho) - h, math.log(rho), math.log(rho) + h, 5.0, -20.0, 0.0])
    logp = np.full(6, -2.0)
    mu = logp - delta
    out = orc.offpolicy_loss_fwd(logp, mu, np.array([1.0]), np.ones((1, 6), np.uint8), rho,
                                 orc.NORM_SUM_T_MEAN_B)
    w = -out["coef"]                   # A = 1, Z = B = 1
    expect = [rho * math.exp(-h), rho, rho, rho, math.exp(-20.0), 1.0]
    assert np.allclose(w, expect, rtol=1e-13, atol=0)
    # two tokens are strictly above rho; exp(ln rho) itself may round to either side of rho
    assert out["stats"][2] in (pytest.approx(2 / 6), pytest.approx(3 / 6))


def test_rho_infinite_is_plain_importance_sampling_and_mu_minus_inf_clips():
    logp = np.array([-1.0, -2.0, -3.0])
    mu = np.array([-3.0, -2.5, -np.inf])
    m = np.ones((1, 3), np.uint8)
    out = orc.offpolicy_loss_fwd(logp, mu, np.array([1.0]), m, np.inf, orc.NORM_SUM_T_MEAN_B)
    assert np.allclose(-out["coef"][:2], np.exp(logp[:2] - mu[:2]))
    out = orc.offpolicy_loss_fwd(logp, mu, np.array([1.0]), m, 4.0, orc.NORM_SUM_T_MEAN_B)
    assert -out["coef"][2] == 4.0


def test_masked_tokens_contribute_nothing_even_with_nan():
    H, W, tg, mu, adv, mask = _rand_problem(13)
    logp, _ = orc.token_logprobs(H, W, tg)
    ref = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0)
    lp2, mu2 = logp.copy(), mu.copy()
    dead = mask.reshape(-1) == 0
    assert dead.any()
    lp2[dead] = np.nan
    mu2[dead] = np.inf
    out = orc.offpolicy_loss_fwd(lp2, mu2, adv, mask, 2.0)
    assert out["loss"] == ref["loss"] and np.array_equal(out["coef"], ref["coef"])
    assert np.all(out["coef"][dead] == 0) and np.array_equal(out["stats"], ref["stats"])


def test_appending_a_fully_masked_generation_changes_nothing_in_token_mean():
    H, W, tg, mu, adv, mask = _rand_problem(14)
    logp, _ = orc.token_logprobs(H, W, tg)
    ref = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0)
    T = mask.shape[1]
    out = orc.offpolicy_loss_fwd(np.concatenate([logp, np.zeros(T)]), np.concatenate([mu, np.zeros(T)]),
                                 np.concatenate([adv, [7.0]]), np.concatenate([mask, np.zeros((1, T), np.uint8)]),
                                 2.0)
    assert out["loss"] == pytest.approx(ref["loss"], rel=1e-14)
    assert np.array_equal(out["coef"][: logp.size], ref["coef"]) and not out["coef"][logp.size:].any()
    out_s = orc.offpolicy_loss_fwd(np.concatenate([logp, np.zeros(T)]), np.concatenate([mu, np.zeros(T)]),
                                   np.concatenate([adv, [7.0]]), np.concatenate([mask, np.zeros((1, T), np.uint8)]),
                                   2.0, orc.NORM_SEQ_MEAN)
    ref_s = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, orc.NORM_SEQ_MEAN)
    assert out_s["loss"] == pytest.approx(ref_s["loss"], rel=1e-14)


def test_norm_mode_identities_when_all_lengths_equal():
    H, W, tg, mu, adv, mask = _rand_problem(15)
    mask[:] = 1
    T = mask.shape[1]
    logp, _ = orc.token_logprobs(H, W, tg)
    a = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, orc.NORM_TOKEN_MEAN)
    b = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, orc.NORM_SEQ_MEAN)
    c = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, orc.NORM_SUM_T_MEAN_B)
    assert b["loss"] == pytest.approx(a["loss"], rel=1e-14)
    assert c["loss"] == pytest.approx(T * a["loss"], rel=1e-14)


def test_all_masked_batch_is_zero_without_division_by_zero():
    H, W, tg, mu, adv, mask = _rand_problem(16)
    mask[:] = 0
    for mode in (0, 1, 2):
        out = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0, mode)
        assert out["loss"] == 0 and not out["coef"].any() and not out["dH"].any() and not out["dW"].any()
        assert out["stats"][0] == 0 and np.all(np.isfinite(out["stats"]))


def test_per_token_advantage_and_bad_targets():
    H, W, tg, mu, adv, mask = _rand_problem(17)
    B, T = mask.shape
    logp, _ = orc.token_logprobs(H, W, tg)
    A_bt = np.repeat(adv[:, None], T, axis=1)
    a = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0)
    b = orc.offpolicy_loss_fwd(logp, mu, A_bt, mask, 2.0)
    assert a["loss"] == b["loss"]
    A_bt[0, 0] += 1.0
    c = orc.offpolicy_loss_fwd(logp, mu, A_bt, mask, 2.0)
    assert c["coef"][0] != a["coef"][0] and np.array_equal(c["coef"][1:], a["coef"][1:])
    tg2 = tg.copy()
    tg2[0] = W.shape[0] + 3
    e = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, targets=tg2, V=W.shape[0])
    m2 = mask.copy()
    m2[0, 0] = 0
    f = orc.offpolicy_loss_fwd(logp, mu, adv, m2, 2.0)
    assert e["stats"][4] == 1 and e["loss"] == f["loss"] and np.array_equal(e["coef"], f["coef"])


# ---------------------------------------------------------------- gradients
def _torch_loss(H, W, tg, mu, adv, mask, rho, norm_mode, clip_mode=orc.CLIP_AIPO, eps=(0.2, 0.2)):
    """Independent reference: torch CPU float64 autograd of the loss written
    with torch's own log_softmax; the AIPO weight is detached."""
    B, T = mask.shape
    Ht = torch.tensor(H, dtype=torch.float64, requires_grad=True)
    Wt = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    lp = torch.log_softmax(Ht @ Wt.T, dim=1).gather(1, torch.tensor(tg)[:, None])[:, 0]
    m = torch.tensor(mask.reshape(-1) != 0)
    A = torch.tensor(np.repeat(adv, T))
    ratio = torch.exp(lp - torch.tensor(mu))
    lens = torch.tensor(mask.sum(1).astype(np.float64))
    if norm_mode == orc.NORM_TOKEN_MEAN:
        Z = torch.full((B * T,), float(max(int(mask.sum()), 1)), dtype=torch.float64)
    elif norm_mode == orc.NORM_SEQ_MEAN:
        Z = (lens.clamp(min=1) * max(int((lens > 0).sum()), 1)).repeat_interleave(T)
    else:
        Z = torch.full((B * T,), float(B), dtype=torch.float64)
    if clip_mode == orc.CLIP_AIPO:
        w = torch.clamp(ratio, max=rho).detach()
        per = -(w * A * lp) / Z
    else:
        per = -torch.minimum(ratio * A, torch.clamp(ratio, 1 - eps[0], 1 + eps[1]) * A) / Z
    loss = torch.where(m, per, torch.zeros_like(per)).sum()
    loss.backward()
    return loss.item(), Ht.grad.numpy(), Wt.grad.numpy()


@pytest.mark.parametrize("norm_mode", [0, 1, 2])
@pytest.mark.parametrize("rho", [1.0, 1.6])
def test_gradients_match_torch_autograd(norm_mode, rho):
    H, W, tg, mu, adv, mask = _rand_problem(21, B=4, T=6, d=5, V=9)
    lp, _ = orc.token_logprobs(H, W, tg)
    mu = lp + np.random.default_rng(2).normal(0, 1.0, lp.shape)    # straddle the clip bound
    out = orc.aipo_step(H, W, tg, mu, adv, mask, rho, norm_mode, grad_loss=1.0)
    loss, gH, gW = _torch_loss(H, W, tg, mu, adv, mask, rho, norm_mode)
    assert 0 < out["stats"][2] < 1
    assert out["loss"] == pytest.approx(loss, rel=1e-12)
    assert np.allclose(out["dH"], gH, rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], gW, rtol=1e-10, atol=1e-14)


def test_gradients_match_central_finite_differences_of_surrogate():
    H, W, tg, mu, adv, mask = _rand_problem(22, B=2, T=4, d=3, V=6)
    lp, _ = orc.token_logprobs(H, W, tg)
    mu = lp + np.random.default_rng(3).normal(0, 1.0, lp.shape)
    rho = 1.5

    def surrogate(Hx, Wx):
        l, _ = orc.token_logprobs(Hx, Wx, tg, mask.reshape(-1))
        return orc.offpolicy_loss_fwd(l, mu, adv, mask, rho)["surrogate"]

    out = orc.aipo_step(H, W, tg, mu, adv, mask, rho)
    assert 0 < out["stats"][2] < 1
    h = 1e-6
    for X, G, which in ((H, out["dH"], 0), (W, out["dW"], 1)):
        for idx in np.ndindex(*X.shape):
            Xp, Xm = X.copy(), X.copy()
            Xp[idx] += h
            Xm[idx] -= h
            fd = (surrogate(Xp, W) - surrogate(Xm, W)) / (2 * h) if which == 0 else \
                 (surrogate(H, Xp) - surrogate(H, Xm)) / (2 * h)
            assert G[idx] == pytest.approx(fd, rel=2e-6, abs=2e-9), (which, idx)


def test_surrogate_is_c1_at_the_clip_bound_and_equals_loss_gradient():
    # d surrogate / d logp == coef on both sides of ln(rho)
    rho = 2.0
    for delta in (math.log(rho) - 0.3, math.log(rho) + 0.3):
        logp = np.array([-1.0])
        mu = logp - delta
        one = np.ones((1, 1), np.uint8)
        f = lambda x: orc.offpolicy_loss_fwd(np.array([x]), mu, np.array([1.3]), one, rho)["surrogate"]
        fd = (f(-1.0 + 1e-6) - f(-1.0 - 1e-6)) / 2e-6
        coef = orc.offpolicy_loss_fwd(logp, mu, np.array([1.3]), one, rho)["coef"][0]
        assert coef == pytest.approx(fd, rel=1e-7)


def test_vocab_column_sums_of_dW_vanish_and_zero_weight_gives_zero_dH():
    H, W, tg, mu, adv, mask = _rand_problem(23)
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0)
    assert np.abs(out["dW"].sum(axis=0)).max() < 1e-14 * max(1.0, np.abs(out["dW"]).max()) * W.shape[0]
    out0 = orc.aipo_step(H, np.zeros_like(W), tg, mu, adv, mask, 2.0)
    assert np.abs(out0["dH"]).max() == 0.0
    assert np.abs(out0["dW"]).max() > 0


def test_gradients_linear_in_upstream_gradient_and_masked_rows_zero():
    H, W, tg, mu, adv, mask = _rand_problem(24)
    a = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0, grad_loss=1.0)
    b = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0, grad_loss=-2.5)
    assert np.allclose(b["dH"], -2.5 * a["dH"], rtol=1e-13) and np.allclose(b["dW"], -2.5 * a["dW"], rtol=1e-13)
    dead = mask.reshape(-1) == 0
    assert dead.any() and not a["dH"][dead].any()
    Hn = H.copy()
    Hn[dead] = np.nan
    c = orc.aipo_step(Hn, W, tg, mu, adv, mask, 2.0)
    assert np.array_equal(c["dW"], a["dW"]) and np.array_equal(c["dH"], a["dH"])


def test_bf16_inputs_are_read_exactly():
    g = torch.Generator().manual_seed(9)
    H = torch.randn(6, 8, generator=g).to(torch.bfloat16)
    W = (torch.randn(10, 8, generator=g) / 3).to(torch.bfloat16)
    tg = np.arange(6)
    hb = H.view(torch.int16).numpy().view(np.uint16)
    wb = W.view(torch.int16).numpy().view(np.uint16)
    a, _ = orc.token_logprobs(hb, wb, tg)
    b, _ = orc.token_logprobs(H.double().numpy(), W.double().numpy(), tg)
    assert np.array_equal(a, b)


# ---------------------------------------------------------------- PPO / GRPO double-sided clip (App. A)
@pytest.mark.parametrize("eps", [(0.2, 0.2), (0.1, 0.3)])
def test_ppo_mode_matches_torch_autograd_and_has_zero_gradient_outside_bounds(eps):
    H, W, tg, mu, adv, mask = _rand_problem(31, B=4, T=6, d=5, V=9)
    lp, _ = orc.token_logprobs(H, W, tg)
    mu = lp + np.random.default_rng(4).normal(0, 0.3, lp.shape)
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0, orc.NORM_TOKEN_MEAN, 1.0, orc.CLIP_PPO, eps[0], eps[1])
    loss, gH, gW = _torch_loss(H, W, tg, mu, adv, mask, 2.0, orc.NORM_TOKEN_MEAN, orc.CLIP_PPO, eps)
    assert 0 < out["stats"][2] < 1
    assert out["loss"] == pytest.approx(loss, rel=1e-12)
    assert np.allclose(out["dH"], gH, rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], gW, rtol=1e-10, atol=1e-14)
    # property (1) of App. A: ratio above 1+eps with A>0, or below 1-eps with A<0, gives zero gradient
    T = mask.shape[1]
    r = np.exp(lp - mu)
    A = np.repeat(adv, T)
    dead = ((r > 1 + eps[1]) & (A > 0)) | ((r < 1 - eps[0]) & (A < 0))
    assert dead.any() and not out["coef"][dead].any()
    live = ~dead & (mask.reshape(-1) != 0)
    assert np.all(out["coef"][live] != 0)


# ---------------------------------------------------------------- group-mean baseline (Sec. 6)
def _brute_ppo(logp, mu, adv, mask, eps_lo, eps_hi, norm_mode):
    """App. A display equation by case analysis on the sign of the advantage (no min / clip calls):
    A >= 0: the objective is A * min(r, 1 + eps_hi), so it follows r (gradient -A r / Z) up to the upper bound and
    is flat above it; A < 0: it is A * max(r, 1 - eps_lo), flat below the lower bound."""
    B, T = mask.shape
    lens = [sum(int(mask[b, t] != 0) for t in range(T)) for b in range(B)]
    n_valid, b_valid = sum(lens), sum(1 for l in lens if l > 0)
    loss, coef = 0.0, [0.0] * (B * T)
    sum_r = sum_d = 0.0
    n_flat = 0
    for b in range(B):
        for t in range(T):
            if mask[b, t] == 0:
                continue
            i = b * T + t
            delta = logp[i] - mu[i]
            r = math.exp(delta)
            Z = (max(n_valid, 1), max(b_valid, 1) * lens[b], B)[norm_mode]
            A = adv[b]
            if A >= 0:
                flat = r > 1.0 + eps_hi
                obj = A * (1.0 + eps_hi) if flat else A * r
            else:
                flat = r < 1.0 - eps_lo
                obj = A * (1.0 - eps_lo) if flat else A * r
            loss -= obj / Z
            coef[i] = 0.0 if flat else -A * r / Z
            n_flat += int(flat)
            sum_r += r
            sum_d += delta
    den = max(n_valid, 1)
    return loss, coef, [float(n_valid), sum_r / den, n_flat / den, sum_d / den, 0.0]


@pytest.mark.parametrize("norm_mode", [orc.NORM_TOKEN_MEAN, orc.NORM_SEQ_MEAN, orc.NORM_SUM_T_MEAN_B])
@pytest.mark.parametrize("eps", [(0.2, 0.2), (0.1, 0.3)])
def test_ppo_mode_loss_coef_and_stats_against_python_loop(norm_mode, eps):
    H, W, tg, mu, adv, mask = _rand_problem(33, B=5, T=7, d=5, V=9)
    mask[3, :] = 0
    logp, _ = orc.token_logprobs(H, W, tg, mask.reshape(-1))
    mu = logp + np.random.default_rng(6).normal(0, 0.3, logp.shape)
    out = orc.offpolicy_loss_fwd(logp, mu, adv, mask, 2.0, norm_mode, orc.CLIP_PPO, eps[0], eps[1])
    loss, coef, stats = _brute_ppo(logp, mu, adv, mask, eps[0], eps[1], norm_mode)
    assert 0.1 < stats[2] < 0.9
    assert out["loss"] == pytest.approx(loss, rel=1e-12, abs=1e-14)
    assert np.allclose(out["coef"], coef, rtol=1e-13, atol=0)
    assert np.allclose(out["stats"], stats, rtol=1e-13, atol=0)       # incl. the clipped-branch fraction, by value


@pytest.mark.parametrize("norm_mode", [orc.NORM_TOKEN_MEAN, orc.NORM_SEQ_MEAN, orc.NORM_SUM_T_MEAN_B])
def test_ppo_mode_gradients_match_torch_autograd_in_every_norm_mode(norm_mode):
    H, W, tg, mu, adv, mask = _rand_problem(35, B=4, T=6, d=5, V=9)
    lp, _ = orc.token_logprobs(H, W, tg)
    mu = lp + np.random.default_rng(8).normal(0, 0.3, lp.shape)
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0, norm_mode, 1.0, orc.CLIP_PPO, 0.15, 0.25)
    loss, gH, gW = _torch_loss(H, W, tg, mu, adv, mask, 2.0, norm_mode, orc.CLIP_PPO, (0.15, 0.25))
    assert out["loss"] == pytest.approx(loss, rel=1e-12)
    assert np.allclose(out["dH"], gH, rtol=1e-10, atol=1e-14)
    assert np.allclose(out["dW"], gW, rtol=1e-10, atol=1e-14)


def test_aipo_stats_against_python_loop():
    # mean ratio, clipped fraction (strict r > rho) and mean log-ratio over the valid tokens, by value
    H, W, tg, mu, adv, mask = _rand_problem(37, B=4, T=9)
    mask[1, :] = 0
    logp, _ = orc.token_logprobs(H, W, tg, mask.reshape(-1))
    mu = logp + np.random.default_rng(10).normal(0, 0.8, logp.shape)
    B, T = mask.shape
    for rho in (1.0, 2.0):
        out = orc.offpolicy_loss_fwd(logp, mu, adv, mask, rho)
        n = sr = sd = nc = 0
        for b in range(B):
            for t in range(T):
                if mask[b, t]:
                    dlt = logp[b * T + t] - mu[b * T + t]
                    n += 1
                    sr += math.exp(dlt)
                    sd += dlt
                    nc += 1 if math.exp(dlt) > rho else 0
        assert 0 < nc < n
        assert np.allclose(out["stats"], [n, sr / n, nc / n, sd / n, 0.0], rtol=1e-13, atol=0)


def test_group_advantages_closed_forms_and_loop():
    # hand example: rewards (1, 0, 0, 1 | 3, 3, 3, 3 | 2, 0, 0, 0), n = 4
    r = np.array([1, 0, 0, 1, 3, 3, 3, 3, 2, 0, 0, 0], dtype=np.float64)
    a = orc.group_advantages(r, 4)
    assert np.allclose(a, [0.5, -0.5, -0.5, 0.5, 0, 0, 0, 0, 1.5, -0.5, -0.5, -0.5], rtol=0, atol=1e-15)
    # normalised: group 0 has population std 1/2 -> +-1; a constant group stays 0 (eps keeps it finite)
    b = orc.group_advantages(r, 4, normalise_std=True, eps=1e-9)
    assert np.allclose(b[:4], [1, -1, -1, 1], rtol=1e-8) and np.all(b[4:8] == 0)
    assert np.allclose(b[8:], np.array([1.5, -0.5, -0.5, -0.5]) / math.sqrt(0.75), rtol=1e-8)
    # against a plain loop on random rewards; every group sums to zero
    rng = np.random.default_rng(3)
    r = rng.standard_normal(7 * 5)
    a = orc.group_advantages(r, 5)
    for p in range(7):
        g = r[5 * p:5 * p + 5]
        m = sum(g) / 5
        assert np.allclose(a[5 * p:5 * p + 5], [x - m for x in g], rtol=0, atol=1e-15)
        assert abs(a[5 * p:5 * p + 5].sum()) < 1e-14
    c = orc.group_advantages(r, 5, normalise_std=True, eps=0.0).reshape(7, 5)
    assert np.allclose((c * c).mean(axis=1), 1.0, rtol=1e-12)


# ---------------------------------------------------------------- KL-regularised reward (Sec. 6)
def test_kl_shaped_rewards_expectation_is_the_exact_sequence_kl():
    # Enumerate every sequence of a T=3, V=3 model with position-wise independent categoricals: under y ~ pi the
    # mean of the per-sequence estimate must be the exact KL(pi || base) = sum of the per-position KLs (scipy's
    # rel_entr), and the mean shaped reward E[r] - lambda * KL.  KL is not symmetric: swapped arguments fail.
    from itertools import product
    from scipy.special import rel_entr
    rng = np.random.default_rng(11)
    T, V, lam = 3, 3, 0.37
    pi = rng.dirichlet(np.ones(V), size=T)
    base = rng.dirichlet(np.ones(V), size=T)
    seqs = np.array(list(product(range(V), repeat=T)))                    # [27, T]
    logp = np.log(pi)[np.arange(T)[None, :], seqs]
    base_logp = np.log(base)[np.arange(T)[None, :], seqs]
    prob = np.exp(logp.sum(axis=1))
    assert abs(prob.sum() - 1.0) < 1e-14
    rewards = rng.standard_normal(len(seqs))
    shaped, kl = orc.kl_shaped_rewards(rewards, logp, base_logp, np.ones_like(seqs, dtype=np.uint8), lam)
    exact = rel_entr(pi, base).sum()
    assert abs((prob * kl).sum() - exact) < 1e-13
    assert abs((prob * shaped).sum() - ((prob * rewards).sum() - lam * exact)) < 1e-13
    assert abs((prob * kl).sum() - rel_entr(base, pi).sum()) > 1e-3


def test_kl_shaped_rewards_special_cases():
    rng = np.random.default_rng(12)
    B, T = 4, 9
    logp = -rng.random((B, T)) * 3
    base = -rng.random((B, T)) * 3
    mask = (rng.random((B, T)) < 0.6).astype(np.uint8)
    mask[2] = 0                                                           # an empty generation
    r = rng.standard_normal(B)
    # lambda = 0 and pi = base leave the reward alone
    assert np.array_equal(orc.kl_shaped_rewards(r, logp, base, mask, 0.0)[0], r)
    s, kl = orc.kl_shaped_rewards(r, logp, logp, mask, 5.0)
    assert np.array_equal(s, r) and np.all(kl == 0)
    # masked positions never count (NaN there is ignored); plain loops give the same numbers
    dirty = logp.copy()
    dirty[mask == 0] = np.nan
    s, kl = orc.kl_shaped_rewards(r, dirty, base, mask, 0.5)
    for b in range(B):
        k = sum(logp[b, t] - base[b, t] for t in range(T) if mask[b, t])
        assert abs(kl[b] - k) < 1e-14 and abs(s[b] - (r[b] - 0.5 * k)) < 1e-14
    assert kl[2] == 0 and s[2] == r[2]
    # a policy more confident than the base on its own samples is penalised (sign of the term)
    s, kl = orc.kl_shaped_rewards(np.zeros(1), np.full((1, 4), -0.1), np.full((1, 4), -2.0), np.ones((1, 4)), 1.0)
    assert kl[0] > 0 and s[0] < 0


# ---------------------------------------------------------------- vocabulary-sliced head (Sec. 8.2: trainer mp 8-32)
def _slices(V, p):
    edges = [round(i * V / p) for i in range(p + 1)]
    return [(edges[i], edges[i + 1]) for i in range(p) if edges[i + 1] > edges[i]]


@pytest.mark.parametrize("p", [1, 2, 3, 4])
def test_sliced_forward_merges_to_the_unsliced_log_probs(p):
    H, W, tg, mu, adv, mask = _rand_problem(41, B=3, T=6, d=7, V=13)
    H[:, 0] += 3.0                                   # uneven slice maxima
    tg[4] = 13                                       # out of range: the row is dead in every shard
    mflat = mask.reshape(-1)
    ref_logp, ref_lse = orc.token_logprobs(H, W, tg, mflat)
    parts = [orc.token_logprobs_partial(H, W[a:b], tg, a, W.shape[0], mflat) for a, b in _slices(W.shape[0], p)]
    m, s, zt = (np.stack([q[i] for q in parts]) for i in range(3))
    logp, lse = orc.merge_partials(m, s, zt)
    assert np.allclose(logp, ref_logp, rtol=1e-13, atol=1e-13) and np.allclose(lse, ref_lse, rtol=1e-13, atol=1e-13)
    dead = (mflat == 0) | (tg < 0) | (tg >= W.shape[0])
    assert dead.any() and not logp[dead].any() and not lse[dead].any()
    assert np.all(np.isneginf(m[:, dead])) and not s[:, dead].any() and not zt[:, dead].any()


def test_slice_partials_are_the_slice_logsumexp_and_the_target_logit():
    # each shard's (m, s) is its own logsumexp (library routine on loop logits), zt the one logit the shard owns
    H, W, tg, mu, adv, mask = _rand_problem(42, B=2, T=5, d=6, V=10)
    a, b = 3, 8
    m, s, zt = orc.token_logprobs_partial(H, W[a:b], tg, a, W.shape[0])
    for t in range(H.shape[0]):
        z = [sum(H[t, k] * W[v, k] for k in range(H.shape[1])) for v in range(a, b)]
        assert m[t] == pytest.approx(max(z), rel=1e-14)
        assert m[t] + math.log(s[t]) == pytest.approx(scipy.special.logsumexp(z), rel=1e-13)
        assert zt[t] == pytest.approx(z[tg[t] - a] if a <= tg[t] < b else 0.0, rel=1e-13, abs=0)
    # shifting every logit of a shard by kappa shifts its m by kappa and leaves s alone (ones column trick)
    H1 = np.concatenate([H, np.ones((H.shape[0], 1))], axis=1)
    W1 = np.concatenate([W, np.full((W.shape[0], 1), 40.0)], axis=1)
    m2, s2, _ = orc.token_logprobs_partial(H1, W1[a:b], tg, a, W.shape[0])
    assert np.allclose(m2, m + 40.0, rtol=1e-14) and np.allclose(s2, s, rtol=1e-12)


@pytest.mark.parametrize("p", [2, 4])
def test_sliced_backward_adds_up_to_the_unsliced_gradients(p):
    H, W, tg, mu, adv, mask = _rand_problem(43, B=3, T=5, d=6, V=11)
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 1.3, grad_loss=-0.7)
    dH = np.zeros_like(out["dH"])
    dW_rows = []
    for a, b in _slices(W.shape[0], p):
        gH, gW = orc.offpolicy_loss_bwd_slice(H, W[a:b], tg, a, out["lse"], out["coef"], -0.7)
        dH += gH
        dW_rows.append(gW)
    assert np.allclose(dH, out["dH"], rtol=1e-12, atol=1e-15)
    assert np.allclose(np.concatenate(dW_rows), out["dW"], rtol=1e-12, atol=1e-15)
    # the shard that does not own a token's target still gets -p * coef for it: its dW rows are not zero
    assert all(np.abs(g).max() > 0 for g in dW_rows)


def test_sliced_backward_matches_torch_autograd_of_the_full_loss_restricted_to_the_slice():
    # independent of the unsliced oracle backward: autograd of the detached-weight loss w.r.t. the FULL W, rows a:b
    H, W, tg, mu, adv, mask = _rand_problem(44, B=2, T=6, d=5, V=9)
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 1.5)
    loss, gH, gW = _torch_loss(H, W, tg, mu, adv, mask, 1.5, orc.NORM_TOKEN_MEAN)
    a, b = 2, 7
    _, gWs = orc.offpolicy_loss_bwd_slice(H, W[a:b], tg, a, out["lse"], out["coef"])
    assert np.allclose(gWs, gW[a:b], rtol=1e-10, atol=1e-14)
