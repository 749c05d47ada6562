"""Shared helpers of the GPU parity tests: run the HIP path, run the oracle on
the same inputs, compare with the tolerances of the benchmark definition."""
import numpy as np
import torch

from oracle import aipo_oracle as orc
import synth


def run_hip(lib, x, rho=2.0, norm_mode=0, grad_loss=1.0, clip_mode=0, eps=(0.2, 0.2), dW_dtype=None,
            pass_targets_to_loss=True):
    B, T = x["mask"].shape
    V = x["W"].shape[0]
    logp, lse = lib.token_logprobs(x["H"], x["W"], x["targets"], x["mask"].reshape(-1))
    loss, coef, stats = lib.offpolicy_loss_fwd(logp, x["mu_logp"], x["adv"], x["mask"], B, T, rho=rho,
                                               norm_mode=norm_mode, clip_mode=clip_mode, eps_lo=eps[0],
                                               eps_hi=eps[1], targets=x["targets"] if pass_targets_to_loss else None,
                                               V=V)
    dH, dW = lib.offpolicy_loss_bwd(x["H"], x["W"], x["targets"], lse, coef, grad_loss=grad_loss, dW_dtype=dW_dtype)
    torch.cuda.synchronize()
    return dict(logp=logp, lse=lse, loss=loss, coef=coef, stats=stats, dH=dH, dW=dW)


def run_oracle(x, rho=2.0, norm_mode=0, grad_loss=1.0, clip_mode=0, eps=(0.2, 0.2)):
    ref = _oracle_step(x, rho, norm_mode, grad_loss, clip_mode, eps)
    # natural magnitude of a gradient entry, from the inputs alone: |dz| <= |g coef|, and an entry of dH (dW) is a
    # sum of V (N_valid) such terms times an entry of W (H) with mixed signs.  Only used as the absolute floor of
    # comparisons whose reference is exactly zero (see check_grad).
    c = abs(grad_loss) * float(np.abs(ref["coef"]).max())
    ref["floor_dH"] = 1e-5 * c * float(x["W"].abs().max()) * np.sqrt(x["W"].shape[0])
    ref["floor_dW"] = 1e-5 * c * float(x["H"].abs().max()) * np.sqrt(max(1.0, float(ref["stats"][0])))
    return ref


def _oracle_step(x, rho, norm_mode, grad_loss, clip_mode, eps):
    return orc.aipo_step(synth.to_oracle(x["H"]), synth.to_oracle(x["W"]), synth.to_oracle(x["targets"]),
                         synth.to_oracle(x["mu_logp"]), synth.to_oracle(x["adv"]), synth.to_oracle(x["mask"]),
                         rho, norm_mode, grad_loss, clip_mode, eps[0], eps[1])


def f64(t):
    return t.detach().to(torch.float64).cpu().numpy()


def check_grad(name, got, ref, dtype, floor=0.0):
    """fp32 workload: |delta| <= 1e-4 everywhere.  bf16 workloads: relative Frobenius error <= 1e-2 and
    max |delta| <= 1e-2 * max |ref|.  floor: absolute slack per entry for references that are exactly zero in fp64
    (a one-entry vocabulary: softmax = 1, dz = 0) where fp32 leaves rounding-sized values and "relative" has no
    meaning; 1e-5 of the natural magnitude of an entry, far below 1e-2 of any non-degenerate reference."""
    got, ref = np.asarray(got, dtype=np.float64), np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, name
    assert np.all(np.isfinite(got)), name + " has non-finite entries"
    err = np.abs(got - ref).max() if got.size else 0.0
    if dtype == "f32":
        assert err <= 1e-4, "%s: max |delta| = %.3g" % (name, err)
        return
    scale = np.abs(ref).max()
    dn, rn = np.linalg.norm(got - ref), np.linalg.norm(ref)
    assert dn <= 1e-2 * rn + floor * np.sqrt(got.size), "%s: relative Frobenius error %.3g" % (name, dn / max(rn, 1e-300))
    assert err <= 1e-2 * scale + floor + 1e-30, "%s: max |delta| = %.3g vs max |ref| = %.3g" % (name, err, scale)


def same_up_to_summation_order(a, b):
    """Two results of the same contraction whose K range was cut into different parts (the plan that splits the
    last tiles of a store contraction depends on how many tiles there are): fp32 sums that differ by rounding, and
    for 16-bit outputs two roundings of such sums, at most one unit in the last place apart."""
    a32, b32 = a.to(torch.float32), b.to(torch.float32)
    scale = float(b32.abs().max())
    if a.dtype == torch.float32:
        return bool(((a32 - b32).abs() <= 4e-6 * scale).all())
    return bool(((a32 - b32).abs() <= 2.0 ** -7 * b32.abs() + 4e-6 * scale).all())


def check_all(got, ref, dtype, check_stats=True, f32_loss_scaled=False):
    tol_lp = 1e-4 if dtype == "f32" else 2e-2
    lp, lse = f64(got["logp"]), f64(got["lse"])
    assert np.abs(lp - ref["logp"]).max() <= tol_lp, "logp max |delta| = %.3g" % np.abs(lp - ref["logp"]).max()
    assert np.abs(lse - ref["lse"]).max() <= tol_lp, "lse max |delta| = %.3g" % np.abs(lse - ref["lse"]).max()
    coef = f64(got["coef"])
    # masked rows are exactly zero on both sides
    assert np.array_equal(coef == 0, ref["coef"] == 0)
    loss = float(got["loss"].item())
    if dtype == "f32":
        assert np.abs(coef - ref["coef"]).max() <= 1e-4
        # 1e-4 absolute is the bar of the tiny fp32 workload (token mean: the loss is O(1)).  A loss that is a SUM
        # over hundreds of tokens (paper-literal normalisation) carries fp32 rounding of each term: scale with it.
        tol = 1e-4 + (2e-6 * np.abs(ref["coef"] * ref["logp"]).sum() if f32_loss_scaled else 0.0)
        assert abs(loss - ref["loss"]) <= tol, (loss, ref["loss"], tol)
    else:
        cs = np.abs(ref["coef"]).max()
        assert np.abs(coef - ref["coef"]).max() <= 2.5e-2 * cs + 1e-30      # coef ~ exp(logp): 2e-2 in logp
        # relative to the loss's own terms, plus fp32 rounding of log-probs that are exactly 0 in fp64 (V = 1)
        scale = np.abs(ref["coef"] * ref["logp"]).sum()
        assert abs(loss - ref["loss"]) <= 1e-2 * scale + 1e-5 * np.abs(ref["coef"]).sum() + 1e-30, \
            (loss, ref["loss"], scale)
    if check_stats:
        st = f64(got["stats"])
        assert st[0] == ref["stats"][0] and st[4] == ref["stats"][4]
        tol = 1e-4 if dtype == "f32" else 2.5e-2
        assert abs(st[1] - ref["stats"][1]) <= tol and abs(st[3] - ref["stats"][3]) <= tol
        # clip fraction: a ratio within fp32 rounding of the bound may be counted on either side; among thousands of
        # tokens one or two such ratios do occur
        assert abs(st[2] - ref["stats"][2]) <= tol + 2.0 / max(1.0, ref["stats"][0])
    check_grad("dH", f64(got["dH"]), ref["dH"], dtype, ref.get("floor_dH", 0.0))
    check_grad("dW", f64(got["dW"]), ref["dW"], dtype, ref.get("floor_dW", 0.0))


def sample_rows(x, n, rng):
    """Valid rows: first / last valid token of every generation, rows next to 256-row tile edges, random ones."""
    mask = x["mask"].cpu().numpy()
    B, T = mask.shape
    valid = np.nonzero(mask.reshape(-1))[0]
    picks = []
    for b in range(B):
        ln = int(mask[b].sum())
        if ln:
            picks += [b * T, b * T + ln - 1]
    vs = set(valid.tolist())
    for e in (255, 256, 257, 511, 512):
        picks += [r for r in (e, valid[-1] - e) if r in vs]
    extra = rng.choice(valid, size=max(0, n - len(set(picks))), replace=False)
    return np.array(sorted(set(picks) | set(extra.tolist())))[: max(n, len(set(picks)))]


def oracle_forward_over_valid_rows(x, Wd, chunk=1024):
    """fp64 oracle log-probs / lse of EVERY valid row, in row chunks (rows are independent).  Inputs only: nothing
    the HIP library produced is read here."""
    mask_flat = synth.to_oracle(x["mask"]).reshape(-1)
    N = mask_flat.size
    valid = np.nonzero(mask_flat)[0]
    o_logp, o_lse = np.zeros(N), np.zeros(N)
    for c0 in range(0, valid.size, chunk):
        r = valid[c0:c0 + chunk]
        ridx = torch.as_tensor(r, device="cuda")
        lp, ls = orc.token_logprobs(synth.to_oracle(x["H"][ridx]), Wd, synth.to_oracle(x["targets"][ridx]))
        o_logp[r], o_lse[r] = lp, ls
        print("oracle forward rows", c0 + r.size, "/", valid.size, flush=True)
    return valid, o_logp, o_lse
