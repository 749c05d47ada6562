"""The autograd wrapper: `loss.backward()` through `aipo_loss` must give the gradients the fp64 oracle gives for the
same upstream factor, for both storage types."""
import pytest
import torch

import synth
from parity_util import check_grad, f64, run_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name,d,V,B,T", [("llama3_8b", 384, 2100, 3, 333), ("tiny_fp32", 256, 1024, 4, 64)])
def test_backward_through_the_wrapper_matches_the_oracle(lib, name, d, V, B, T):
    from paper_2505_24034_amd.autograd import aipo_loss
    base = synth.WORKLOADS[name]
    w = synth.scaled(base, d=d, V=V, B=B, T=T, len_lo=T // 4, len_hi=T, seed=77)
    x = synth.make_inputs(w, "cuda")
    H = x["H"].clone().requires_grad_(True)
    W = x["W"].clone().requires_grad_(True)
    loss, stats, logp = aipo_loss(H, W, x["targets"], x["mu_logp"], x["adv"], x["mask"], rho=1.1)
    assert loss.dim() == 0 and loss.requires_grad and not stats.requires_grad and not logp.requires_grad
    (3.0 * loss).backward()
    ref = run_oracle(x, rho=1.1, grad_loss=3.0)
    tol = 1e-4 if base.dtype == "f32" else 1e-2 * abs(ref["loss"]) + 1e-3
    assert abs(float(loss.detach()) - ref["loss"]) <= tol
    check_grad("H.grad", f64(H.grad), ref["dH"], base.dtype)
    check_grad("W.grad", f64(W.grad), ref["dW"], base.dtype)
    assert H.grad.dtype == H.dtype and W.grad.dtype == W.dtype
