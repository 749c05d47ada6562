"""llamarl_offpolicy_loss_fwd_static: the loss forward for callers that cannot allocate (its scratch is a static
device array inside the library).  Checked against llamarl_offpolicy_loss_fwd on the same inputs, bit for bit (they
run the same kernels), on two calls in a row -- the second with a smaller batch, so that what the first left in the
shared scratch must not matter -- and against the fp64 oracle."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import aipo_oracle as orc
from parity_util import f64

pytestmark = pytest.mark.gpu


def _batch(B, T, seed, V=5000):
    g = torch.Generator(device="cuda").manual_seed(seed)
    logp = -torch.rand(B * T, generator=g, device="cuda") * 12
    mu = logp + torch.randn(B * T, generator=g, device="cuda") * 0.5
    adv = torch.randn(B, generator=g, device="cuda")
    mask = (torch.rand(B, T, generator=g, device="cuda") < 0.6).to(torch.uint8)
    mask[B // 2] = 0                                            # one empty generation
    tg = torch.randint(0, V, (B * T,), generator=g, device="cuda", dtype=torch.int32)
    tg[3] = V + 7                                               # one out-of-range target at a (possibly) unmasked row
    return logp, mu, adv, mask, tg, V


def test_static_scratch_variant_matches_the_workspace_variant_twice_in_a_row(lib):
    for (B, T, seed, rho, mode) in ((37, 1300, 1, 1.2, 1), (5, 211, 2, 2.0, 0), (5, 211, 3, 1.05, 2)):
        logp, mu, adv, mask, tg, V = _batch(B, T, seed)
        ref_loss, ref_coef, ref_stats = lib.offpolicy_loss_fwd(logp, mu, adv, mask, B, T, rho=rho, norm_mode=mode,
                                                               targets=tg, V=V)
        loss = torch.full((1,), float("nan"), device="cuda")
        coef = torch.full((B * T,), float("nan"), device="cuda")
        stats = torch.full((5,), float("nan"), device="cuda")
        lib.offpolicy_loss_fwd_static(logp, mu, adv, mask, B, T, loss, coef, stats, rho=rho, norm_mode=mode,
                                      targets=tg, V=V)
        torch.cuda.synchronize()
        assert torch.equal(loss, ref_loss) and torch.equal(coef, ref_coef) and torch.equal(stats, ref_stats)
        o = orc.offpolicy_loss_fwd(f64(logp), f64(mu), f64(adv), mask.cpu().numpy(), rho, mode,
                                   targets=tg.cpu().numpy(), V=V)
        assert np.allclose(f64(coef), o["coef"], rtol=3e-6, atol=1e-12)
        assert float(loss) == pytest.approx(o["loss"], rel=1e-5, abs=1e-6)
        assert np.allclose(f64(stats), o["stats"], rtol=1e-5, atol=1e-6)
        assert 0.0 < o["stats"][2] < 1.0 and o["stats"][4] >= 0


def test_static_scratch_variant_rejects_batches_beyond_its_maximum(lib):
    # sizes are checked on the host before any pointer is used or any kernel is launched
    small = torch.zeros(16, device="cuda")
    loss, stats = torch.zeros(1, device="cuda"), torch.zeros(5, device="cuda")
    p = lib.LossParams(2.0, 0, 0.2, 0.2, 0)
    for B, T in ((2, (1 << 21) + 1), ((1 << 16) + 1, 1)):
        st = lib.load().llamarl_offpolicy_loss_fwd_static(lib._ptr(small), lib._ptr(small), lib._ptr(small), 0, None,
                                                          None, 0, B, T, ctypes.byref(p), lib._ptr(loss),
                                                          lib._ptr(small), lib._ptr(stats), None)
        assert st == lib.ERR_UNSUPPORTED
        assert "static scratch" in lib.load().llamarl_last_error().decode()
