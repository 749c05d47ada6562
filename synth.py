"""Seeded synthetic inputs for the AIPO hot path.

These tensors stand in for what a LlamaRL trainer holds when it reaches the
loss (Sec. 6 of the paper: hidden states of the learner, LM-head weight,
tokens y_t sampled by the generator, the generator's log mu(y_t|.), one
advantage per generation, a response mask).  The paper's own runs use
Llama-3.1 weights and MATH prompts; neither is available, so shapes and value
distributions are synthetic.

This module only *makes inputs*.  It serves both the HIP library's tests and
the fp64 oracle's tests and imports neither.  The logits it needs to sample
tokens and to produce the generator's log-probabilities are formed with
torch's own matmul / log_softmax; whatever they return is an input, never an
expected value.
"""
import math
from dataclasses import dataclass, replace

import torch


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str            # "f32" | "bf16": storage type of H, W (and dH, dW)
    d: int
    V: int
    B: int
    T: int
    seed: int
    sigma_mu: float       # std of the generator-weight perturbation
    target_mode: str      # "uniform" | "softmax"
    len_mode: str         # "uniform" | "loguniform" | "full"
    len_lo: int
    len_hi: int
    adv_mode: str         # "normal" | "normal_std" | "binary_group8"

    @property
    def N(self):
        return self.B * self.T


# the five workloads the benchmark definition names, in its order
WORKLOADS = {
    "tiny_fp32": Workload("tiny_fp32", "f32", 256, 1024, 4, 64, 0, 1e-2, "uniform", "uniform", 16, 64, "normal"),
    "llama3_8b": Workload("llama3_8b", "bf16", 4096, 128256, 8, 2048, 1, 1e-3, "softmax", "uniform", 256, 2048,
                          "normal_std"),
    "llama3_70b": Workload("llama3_70b", "bf16", 8192, 128256, 4, 4096, 2, 2e-3, "softmax", "uniform", 512, 4096,
                           "normal_std"),
    "long_reasoning": Workload("long_reasoning", "bf16", 4096, 128256, 2, 16384, 3, 1e-3, "softmax", "loguniform",
                               512, 16384, "binary_group8"),
    "llama3_405b_head": Workload("llama3_405b_head", "bf16", 16384, 128256, 2, 4096, 4, 1e-3, "softmax", "uniform",
                                 1024, 4096, "normal_std"),
}


def scaled(w, **kw):
    """A copy of a workload with some fields replaced (test-sized variants)."""
    return replace(w, **kw)


def _lengths(w, gen, device):
    if w.len_mode == "full":
        return torch.full((w.B,), w.T, dtype=torch.int64, device=device)
    u = torch.rand(w.B, generator=gen, device=device, dtype=torch.float64)
    if w.len_mode == "uniform":
        ln = w.len_lo + torch.floor(u * (w.len_hi - w.len_lo + 1)).to(torch.int64)
    elif w.len_mode == "loguniform":
        ln = torch.round(torch.exp(math.log(w.len_lo) + u * (math.log(w.len_hi) - math.log(w.len_lo)))).to(torch.int64)
    else:
        raise ValueError(w.len_mode)
    return ln.clamp_(min(w.len_lo, w.T), w.T)


def _advantages(w, gen, device):
    if w.adv_mode == "normal":
        return torch.randn(w.B, generator=gen, device=device, dtype=torch.float32)
    if w.adv_mode == "normal_std":
        a = torch.randn(w.B, generator=gen, device=device, dtype=torch.float32)
        return (a - a.mean()) / (a.std(unbiased=False) + 1e-6)
    if w.adv_mode == "binary_group8":
        # one prompt, 8 generations with reward +-1; the batch holds the first B of them
        r = torch.where(torch.rand(8, generator=gen, device=device) < 0.5, -1.0, 1.0).to(torch.float32)
        a = (r - r.mean()) / (r.std(unbiased=False) + 1e-6)
        reps = (w.B + 7) // 8
        return a.repeat(reps)[: w.B].contiguous()
    raise ValueError(w.adv_mode)


def make_inputs(w, device="cpu", row_chunk=1024):
    """Build one batch.  Returns a dict of torch tensors on `device`:

    H [N,d], W [V,d] in the workload's storage dtype; targets int32 [N];
    mu_logp float32 [N]; adv float32 [B]; mask uint8 [B,T]; lengths int64 [B].
    The random streams of the CPU and GPU generators differ, so a batch is
    defined by (workload, device type).
    """
    device = torch.device(device)
    gen = torch.Generator(device=device)
    gen.manual_seed(1000003 * w.seed + 12345)
    store = torch.float32 if w.dtype == "f32" else torch.bfloat16
    N, d, V = w.N, w.d, w.V

    H = torch.randn(N, d, generator=gen, device=device, dtype=torch.float32).to(store)
    W32 = torch.randn(V, d, generator=gen, device=device, dtype=torch.float32) * (d ** -0.5)
    W = W32.to(store)
    # generator policy mu: the same head with perturbed weights (a lagging / quantised copy)
    Wmu = W.to(torch.float32) + w.sigma_mu * torch.randn(V, d, generator=gen, device=device, dtype=torch.float32)
    del W32
    Wf = W.to(torch.float32)

    targets = torch.empty(N, dtype=torch.int64, device=device)
    mu_logp = torch.empty(N, dtype=torch.float32, device=device)
    for r0 in range(0, N, row_chunk):
        Hc = H[r0:r0 + row_chunk].to(torch.float32)
        if w.target_mode == "uniform":
            tg = torch.randint(0, V, (Hc.shape[0],), generator=gen, device=device)
        else:
            # y_t ~ softmax of the trainer's logits at temperature 1 (Gumbel-max)
            z = Hc @ Wf.T
            u = torch.rand(z.shape, generator=gen, device=device, dtype=torch.float32).clamp_(1e-12, 1.0 - 1e-7)
            tg = torch.argmax(z - torch.log(-torch.log(u)), dim=1)
            del z, u
        zmu = Hc @ Wmu.T
        lp = torch.log_softmax(zmu, dim=1).gather(1, tg[:, None])[:, 0]
        targets[r0:r0 + row_chunk] = tg
        mu_logp[r0:r0 + row_chunk] = lp
        del zmu
    del Wmu, Wf

    lengths = _lengths(w, gen, device)
    mask = (torch.arange(w.T, device=device)[None, :] < lengths[:, None]).to(torch.uint8)
    adv = _advantages(w, gen, device)
    return dict(H=H, W=W, targets=targets.to(torch.int32), mu_logp=mu_logp, adv=adv, mask=mask.contiguous(),
                lengths=lengths)


def to_oracle(t):
    """Hand a tensor to numpy without changing a bit: bf16 becomes its uint16
    bit pattern (numpy has no bfloat16), everything else its own dtype."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view("uint16")
    return t.numpy()
