"""The whole path (token log-probs, loss forward, backward) recorded into a HIP graph and replayed: every entry point
only enqueues kernels on the stream it is given -- no allocation, no synchronisation, no memset node -- so a caller
may capture it.  Each replay runs on fresh input contents, with eager work and synchronisations in between, and must
reproduce the eager call on the same inputs bit for bit (the kernels are the same and their reductions have a fixed
order); the first replay is also checked against the fp64 oracle."""
import pytest
import torch

import synth
from parity_util import check_all, run_oracle

pytestmark = pytest.mark.gpu


def _step(lib, x, w, ws, out, rho, mode):
    logp, lse = lib.token_logprobs(x["H"], x["W"], x["targets"], x["mask"].reshape(-1), ws=ws[0])
    loss, coef, stats = lib.offpolicy_loss_fwd(logp, x["mu_logp"], x["adv"], x["mask"], w.B, w.T, rho=rho,
                                               norm_mode=mode, targets=x["targets"], V=w.V, ws=ws[1])
    lib.offpolicy_loss_bwd(x["H"], x["W"], x["targets"], lse, coef, dH=out["dH"], dW=out["dW"], ws=ws[2])
    return dict(logp=logp, lse=lse, loss=loss, coef=coef, stats=stats, dH=out["dH"], dW=out["dW"])


@pytest.mark.parametrize("name,d,V,B,T", [("llama3_8b", 512, 3000, 3, 700), ("tiny_fp32", 256, 1024, 4, 64)])
def test_graph_replays_match_eager_calls(lib, name, d, V, B, T):
    base = synth.WORKLOADS[name]
    rho, mode = 1.1, 0
    ws = x = out = None
    variants = []
    for seed in (11, 12, 13):
        w = synth.scaled(base, d=d, V=V, B=B, T=T, len_lo=T // 3, len_hi=T, seed=seed)
        variants.append(synth.make_inputs(w, "cuda"))
    dt = lib.BF16 if base.dtype == "bf16" else lib.F32
    N = B * T
    ws = [torch.empty(lib.workspace_bytes(N, d, V, dt, p), dtype=torch.uint8, device="cuda")
          for p in (lib.PASS_LOGPROBS, lib.PASS_LOSS_FWD, lib.PASS_LOSS_BWD)]
    keys = ("H", "W", "targets", "mask", "mu_logp", "adv")
    x = {k: variants[0][k].clone() for k in keys}                      # the graph's fixed input buffers
    out = {"dH": torch.empty_like(x["H"]), "dW": torch.empty_like(x["W"])}

    # eager results for the three input sets (own output buffers, same workspaces)
    eager = []
    for v in variants:
        o = {"dH": torch.empty_like(x["H"]), "dW": torch.empty_like(x["W"])}
        r = _step(lib, {k: v[k] for k in keys}, w, ws, o, rho, mode)
        torch.cuda.synchronize()
        eager.append({k: t.clone() for k, t in r.items()})

    side = torch.cuda.Stream()                                           # default priority
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        _step(lib, x, w, ws, out, rho, mode)                             # warm-up on the capture stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        got = _step(lib, x, w, ws, out, rho, mode)
    torch.cuda.synchronize()

    for rep, idx in enumerate((1, 2, 0, 1)):
        for k in keys:
            x[k].copy_(variants[idx][k])
        for t in got.values():
            t.fill_(float("nan"))                                        # a replay must rewrite every output
        for b in ws:
            b.fill_(0xA5 if rep % 2 else 0x00)                           # and may not depend on workspace contents
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for k, t in got.items():
            assert torch.equal(t, eager[idx][k]), "replay %d: %s differs from the eager call" % (rep, k)
        if rep == 0:
            ref = run_oracle(variants[idx], rho=rho, norm_mode=mode)
            check_all({k: t for k, t in got.items()}, ref, base.dtype, f32_loss_scaled=True)
