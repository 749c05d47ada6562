"""GPU parity at mid-size odd shapes: tens of token tiles by hundreds of vocabulary tiles with ragged edges on every
side, so that the persistent tile schedule runs many patches, partial patches and a split tail -- between the small
sweep (a few tiles) and the five full-size workloads (all of which share V = 128256).  Every output against the fp64
oracle; the backward also in row passes."""
import pytest
import torch

import synth
from parity_util import check_all, check_grad, f64, run_hip, run_oracle, same_up_to_summation_order

pytestmark = pytest.mark.gpu
W8, W1 = synth.WORKLOADS["llama3_8b"], synth.WORKLOADS["tiny_fp32"]


@pytest.mark.parametrize("dt,d,V,B,T", [("bf16", 1032, 33001, 5, 1900), ("bf16", 264, 70001, 3, 1500),
                                        ("bf16", 4104, 9001, 6, 2500), ("f32", 516, 20011, 4, 1200),
                                        ("bf16", 520, 40003, 16, 700)])
def test_mid_shape(lib, dt, d, V, B, T):
    base = W8 if dt == "bf16" else W1
    w = synth.scaled(base, d=d, V=V, B=B, T=T, len_lo=T // 2, len_hi=T, seed=300 + d)
    x = synth.make_inputs(w, "cuda")
    got, ref = run_hip(lib, x, rho=1.0), run_oracle(x, rho=1.0)
    check_all(got, ref, dt, f32_loss_scaled=True)
    assert 0.0 < ref["stats"][2] < 1.0                                   # the clip is engaged
    dH, dW = lib.offpolicy_loss_bwd(x["H"], x["W"], x["targets"], got["lse"], got["coef"], max_rows_per_pass=1024,
                                    dW_dtype=torch.float32)
    torch.cuda.synchronize()
    assert same_up_to_summation_order(dH, got["dH"])
    check_grad("dW (row passes)", f64(dW), ref["dW"], dt, ref["floor_dW"])
