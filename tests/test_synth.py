"""The seeded input synthesiser: shapes, determinism and the stated distributions."""
import math

import numpy as np
import torch

import synth


def test_five_named_workloads_have_the_stated_shapes():
    w = synth.WORKLOADS
    assert list(w) == ["tiny_fp32", "llama3_8b", "llama3_70b", "long_reasoning", "llama3_405b_head"]
    assert (w["tiny_fp32"].d, w["tiny_fp32"].V, w["tiny_fp32"].N, w["tiny_fp32"].dtype) == (256, 1024, 256, "f32")
    assert (w["llama3_8b"].d, w["llama3_8b"].V, w["llama3_8b"].B, w["llama3_8b"].T) == (4096, 128256, 8, 2048)
    assert (w["llama3_70b"].d, w["llama3_70b"].N) == (8192, 16384)
    assert (w["long_reasoning"].T, w["long_reasoning"].N) == (16384, 32768)
    assert (w["llama3_405b_head"].d, w["llama3_405b_head"].N) == (16384, 8192)


def test_tiny_workload_is_deterministic_and_well_formed():
    w = synth.WORKLOADS["tiny_fp32"]
    a, b = synth.make_inputs(w), synth.make_inputs(w)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    assert a["H"].dtype == torch.float32 and a["H"].shape == (256, 256) and a["W"].shape == (1024, 256)
    assert a["targets"].dtype == torch.int32 and int(a["targets"].min()) >= 0 and int(a["targets"].max()) < 1024
    assert a["mask"].dtype == torch.uint8 and a["mask"].shape == (4, 64)
    ln = a["lengths"]
    assert torch.equal(a["mask"].sum(1).to(torch.int64), ln) and int(ln.min()) >= 16 and int(ln.max()) <= 64
    # prefix mask
    assert all(bool((a["mask"][b, : ln[b]] == 1).all()) and bool((a["mask"][b, ln[b]:] == 0).all()) for b in range(4))
    assert abs(float(a["W"].std()) - 1 / 16) < 0.002 and abs(float(a["H"].std()) - 1.0) < 0.02
    assert bool((a["mu_logp"] < 0).all())
    # uniform targets under a near-uniform-ish policy: mu_logp ~ -(ln V + 1/2) on average
    assert abs(float(a["mu_logp"].mean()) + math.log(1024) + 0.5) < 0.25


def test_bf16_variant_softmax_targets_and_group_normalised_advantages():
    w = synth.scaled(synth.WORKLOADS["llama3_8b"], d=128, V=777, B=6, T=50, len_lo=5, len_hi=50)
    x = synth.make_inputs(w)
    assert x["H"].dtype == torch.bfloat16 and x["W"].dtype == torch.bfloat16
    assert abs(float(x["adv"].mean())) < 1e-5 and abs(float(x["adv"].std(unbiased=False)) - 1) < 1e-3
    # tokens sampled from the policy are more likely than uniform ones: mean logp ~ 1 - lse
    assert float(x["mu_logp"].mean()) > -(math.log(777) + 0.5) + 0.5
    bits = synth.to_oracle(x["H"])
    assert bits.dtype == np.uint16 and bits.shape == (300, 128)


def test_long_reasoning_variant_lengths_and_binary_advantages():
    w = synth.scaled(synth.WORKLOADS["long_reasoning"], d=64, V=300, B=12, T=256, len_lo=8, len_hi=256)
    x = synth.make_inputs(w)
    ln = x["lengths"]
    assert int(ln.min()) >= 8 and int(ln.max()) <= 256
    assert len(set(np.round(x["adv"].numpy(), 4).tolist())) <= 2       # +-1 rewards, normalised
    assert torch.equal(x["adv"][:4], x["adv"][8:12])                   # groups of 8 repeat
