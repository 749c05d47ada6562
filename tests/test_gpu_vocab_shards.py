"""GPU parity of the vocabulary-sharded entry points (one shard of a vocabulary-parallel head, paper Sec. 8.2,
Table 3: trainer model parallelism 8-32).  The shards run one after another on the one GPU; their partials are
merged by llamarl_merge_partials and everything is compared with the fp64 oracle of the FULL vocabulary and with
the oracle's own shard functions.  No collective and no second GPU is involved."""
import numpy as np
import pytest
import torch

import synth
from oracle import aipo_oracle as orc
from parity_util import check_grad, f64, oracle_forward_over_valid_rows, run_oracle, sample_rows

pytestmark = pytest.mark.gpu
W8 = synth.WORKLOADS["llama3_8b"]
W1 = synth.WORKLOADS["tiny_fp32"]


def _edges(V, p):
    return [round(i * V / p) for i in range(p + 1)]


def _sharded_forward(lib, x, V, p):
    mask = x["mask"].reshape(-1)
    e = _edges(V, p)
    parts = [lib.token_logprobs_partial(x["H"], x["W"][e[i]:e[i + 1]].contiguous(), x["targets"], e[i], V, mask)
             for i in range(p)]
    m, s, zt = (torch.stack([q[i] for q in parts]).contiguous() for i in range(3))
    logp, lse = lib.merge_partials(m, s, zt)
    return e, m, s, zt, logp, lse


@pytest.mark.parametrize("w,p", [
    (synth.scaled(W8, d=520, V=5003, B=3, T=347, len_lo=40, len_hi=347, seed=51), 4),
    (synth.scaled(W8, d=128, V=300, B=2, T=150, len_lo=20, len_hi=150, seed=52), 3),       # shards smaller than a tile
    (synth.scaled(W1, d=100, V=777, B=3, T=100, len_lo=10, len_hi=100, seed=53), 2),
], ids=["bf16_four_shards", "bf16_tiny_shards", "f32_two_shards"])
def test_shards_merge_to_the_full_vocabulary_result(lib, w, p):
    x = synth.make_inputs(w, "cuda")
    x["targets"][5] = w.V + 3                           # dead in every shard
    B, T = x["mask"].shape
    V, N = w.V, w.N
    tol = 1e-4 if w.dtype == "f32" else 2e-2
    ref = run_oracle(x, rho=1.1, grad_loss=0.5)         # the oracle of the unsharded path
    e, m, s, zt, logp, lse = _sharded_forward(lib, x, V, p)
    torch.cuda.synchronize()
    o = {k: synth.to_oracle(x[k]) for k in ("H", "W", "targets", "mask", "mu_logp", "adv")}
    mflat = o["mask"].reshape(-1)
    # every shard's partials against the oracle's shard function
    for i in range(p):
        om, os_, ozt = orc.token_logprobs_partial(o["H"], o["W"][e[i]:e[i + 1]], o["targets"], e[i], V, mflat)
        live = np.isfinite(om)
        assert np.array_equal(np.isfinite(f64(m[i])), live)
        assert np.abs(f64(m[i])[live] - om[live]).max() <= tol
        assert np.abs((f64(m[i])[live] + np.log(f64(s[i])[live])) - (om[live] + np.log(os_[live]))).max() <= tol
        assert np.abs(f64(zt[i]) - ozt).max() <= tol
        assert not f64(s[i])[~live].any() and not f64(zt[i])[~live].any()
    # merged result against the full-vocabulary oracle
    assert np.abs(f64(logp) - ref["logp"]).max() <= tol and np.abs(f64(lse) - ref["lse"]).max() <= tol
    assert not f64(logp)[ref["lse"] == 0].any()
    # the shards' backward with the merged (global) lse
    loss, coef, stats = lib.offpolicy_loss_fwd(logp, x["mu_logp"], x["adv"], x["mask"], B, T, rho=1.1,
                                               targets=x["targets"], V=V)
    dH = np.zeros((N, w.d))
    dW = []
    for i in range(p):
        gH, gW = lib.offpolicy_loss_bwd_slice(x["H"], x["W"][e[i]:e[i + 1]].contiguous(), x["targets"], e[i], lse, coef,
                                              grad_loss=0.5)
        torch.cuda.synchronize()
        oH, oW = orc.offpolicy_loss_bwd_slice(o["H"], o["W"][e[i]:e[i + 1]], o["targets"], e[i], ref["lse"],
                                              ref["coef"], 0.5)
        check_grad("dH_partial[%d]" % i, f64(gH), oH, w.dtype)
        check_grad("dW_slice[%d]" % i, f64(gW), oW, w.dtype)
        dH += f64(gH)
        dW.append(f64(gW))
    check_grad("sum of dH partials", dH, ref["dH"], w.dtype)
    check_grad("stacked dW slices", np.concatenate(dW), ref["dW"], w.dtype)


def test_one_shard_is_the_whole_head(lib):
    w = synth.scaled(W8, d=256, V=1500, B=2, T=200, len_lo=30, len_hi=200, seed=54)
    x = synth.make_inputs(w, "cuda")
    mask = x["mask"].reshape(-1)
    logp, lse = lib.token_logprobs(x["H"], x["W"], x["targets"], mask)
    m, s, zt = lib.token_logprobs_partial(x["H"], x["W"], x["targets"], 0, w.V, mask)
    lp2, lse2 = lib.merge_partials(m[None].contiguous(), s[None].contiguous(), zt[None].contiguous())
    torch.cuda.synchronize()
    assert torch.allclose(lse2, lse, rtol=0, atol=1e-5) and torch.allclose(lp2, logp, rtol=0, atol=1e-5)


def test_llama3_8b_shape_in_four_shards(lib):
    """d=4096, V=128256 in four shards of 32064 rows (what one of four tensor-parallel devices holds), all 16384
    token rows: merged log-probs of every valid row against one fp64 forward; the shards' dH summands of sampled
    rows and one shard's whole dW slice (gradient weight restricted to sampled rows) against the oracle."""
    w = W8
    x = synth.make_inputs(w, "cuda")
    B, T, N, V, p = w.B, w.T, w.N, w.V, 4
    e, m, s, zt, logp, lse = _sharded_forward(lib, x, V, p)
    torch.cuda.synchronize()
    Wd = orc.widen(synth.to_oracle(x["W"]))
    valid, o_logp, o_lse = oracle_forward_over_valid_rows(x, Wd)
    assert np.abs(f64(logp) - o_logp).max() <= 2e-2 and np.abs(f64(lse) - o_lse).max() <= 2e-2
    o_tg = synth.to_oracle(x["targets"])
    o = orc.offpolicy_loss_fwd(o_logp, synth.to_oracle(x["mu_logp"]), synth.to_oracle(x["adv"]),
                               synth.to_oracle(x["mask"]), 2.0, targets=o_tg, V=V)
    loss, coef, stats = lib.offpolicy_loss_fwd(logp, x["mu_logp"], x["adv"], x["mask"], B, T, rho=2.0,
                                               targets=x["targets"], V=V)
    rng = np.random.default_rng(7)
    rows = sample_rows(x, 96, rng)
    ridx = torch.as_tensor(rows, device="cuda")
    coef_s = torch.zeros_like(coef)
    coef_s[ridx] = coef[ridx]
    Hs = synth.to_oracle(x["H"][ridx])
    dH_sum = np.zeros((rows.size, w.d))
    for i in range(p):
        Wi = x["W"][e[i]:e[i + 1]].contiguous()
        gH, gW = lib.offpolicy_loss_bwd_slice(x["H"], Wi, x["targets"], e[i], lse, coef_s, dW_dtype=torch.float32)
        torch.cuda.synchronize()
        oH, oW = orc.offpolicy_loss_bwd_slice(Hs, Wd[e[i]:e[i + 1]], o_tg[rows], e[i], o_lse[rows], o["coef"][rows])
        check_grad("dH_partial[%d][sampled rows]" % i, f64(gH[ridx]), oH, "bf16")
        dH_sum += f64(gH[ridx])
        if i == 2:
            ref = torch.as_tensor(oW, device="cuda")
            err = gW.double() - ref
            assert float(err.norm() / ref.norm()) <= 1e-2 and float(err.abs().max() / ref.abs().max()) <= 1e-2
        keep = torch.zeros(N, dtype=torch.bool, device="cuda")
        keep[ridx] = True
        assert not bool(gH[~keep].any())
        print("shard", i, "done", flush=True)
    o_dH, _ = orc.offpolicy_loss_bwd(Hs, Wd, o_tg[rows], o_lse[rows], o["coef"][rows])
    check_grad("sum of dH partials [sampled rows]", dH_sum, o_dH, "bf16")
