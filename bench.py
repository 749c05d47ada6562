#!/usr/bin/env python3
"""Benchmark of the AIPO hot path on one MI355X.

One step = llamarl_token_logprobs -> llamarl_offpolicy_loss_fwd -> llamarl_offpolicy_loss_bwd on one batch of
synthetic Llama-3-8B-shaped input (d=4096, V=128256, B=8 x T=2048, bf16) that is already resident in HBM.
Prints ONE JSON line: whole-step tokens/s, the MFMA roofline of the dominant contraction kernel (timed live with
HIP events on the launch stream) and the fp64 oracle timed on the host cores over a bounded sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA, published
METRIC = "tokens/s fwd+bwd logprob+IS loss at Llama-3-8B shape; % bf16 MFMA peak"


def cpu_baseline(x, w, rows):
    """The fp64 oracle as it stands, on `rows` valid token rows of the same batch at full V and d."""
    import numpy as np
    from oracle import aipo_oracle as orc
    import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    import torch
    idx = torch.nonzero(x["mask"].reshape(-1))[:rows, 0]
    rows = int(idx.numel())
    H = synth.to_oracle(x["H"][idx])
    W = synth.to_oracle(x["W"])
    tg = synth.to_oracle(x["targets"][idx])
    mu = synth.to_oracle(x["mu_logp"][idx])
    adv = np.array([1.0])
    mask = np.ones((1, rows), dtype=np.uint8)
    t0 = time.perf_counter()
    out = orc.aipo_step(H, W, tg, mu, adv, mask, 2.0)
    dt = time.perf_counter() - t0
    assert np.isfinite(out["loss"])
    return {"value": rows / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": "first %d valid token rows of the batch, full V=%d and d=%d, oracle fwd+bwd once, "
                      "%.1f s; cost is linear in rows" % (rows, w.V, w.d, dt)}


def library_gemm(x, flops):
    """Context, not part of the path: the vendor library's plain bf16 GEMM (torch.matmul -> hipBLASLt) of the same
    contraction, logits = H_active W^T written to HBM, timed the same way on the same machine.  It shows what a
    tuned GEMM reaches here under the chip's power limit; the path's kernels fuse their epilogues and never
    write the logits."""
    import torch
    rows = x["mask"].reshape(-1).nonzero().squeeze(1)
    Hc = x["H"].index_select(0, rows).contiguous()
    Wt = x["W"].t()
    out = torch.empty(Hc.shape[0], Wt.shape[1], dtype=Hc.dtype, device=Hc.device)
    for _ in range(3):
        torch.matmul(Hc, Wt, out=out)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 10
    e0.record()
    for _ in range(reps):
        torch.matmul(Hc, Wt, out=out)
    e1.record()
    torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    return {"what": "torch.matmul bf16 (hipBLASLt), [n_valid,d] x [d,V] -> logits in HBM, same shape", "ms": ms,
            "achieved": flops / (ms * 1e-3) / 1e12, "unit": "TFLOP/s",
            "frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}


def measured_traffic(kernel):
    """Bytes per launch of `kernel` between L2 and the fabric (reads include Infinity-Cache hits), from the committed
    rocprofv3 FETCH_SIZE / WRITE_SIZE summary, already scaled by the plain-copy calibration.  None if absent."""
    path = os.path.join(ROOT, "profiles", "bench_llama3_8b_hbm_traffic_pmc.md")
    try:
        for line in open(path):
            cells = [c.strip() for c in line.split("|")]
            if len(cells) >= 6 and kernel in cells[1]:
                return (float(cells[4]) + float(cells[5])) * 2 ** 30
    except (OSError, ValueError):
        pass
    return None


class HipEvents:
    """Raw HIP events through the runtime torch already loaded: the backward's phase boundaries are recorded by
    the library itself (llamarl_offpolicy_loss_bwd_phases), which needs hipEvent_t handles."""

    def __init__(self):
        import ctypes
        self.ct = ctypes
        self.hip = ctypes.CDLL("libamdhip64.so")
        self.hip.hipEventCreate.argtypes = [ctypes.POINTER(ctypes.c_void_p)]
        self.hip.hipEventElapsedTime.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.c_void_p, ctypes.c_void_p]
        self.hip.hipEventDestroy.argtypes = [ctypes.c_void_p]

    def create(self, n):
        out = []
        for _ in range(n):
            e = self.ct.c_void_p()
            assert self.hip.hipEventCreate(self.ct.byref(e)) == 0
            out.append(e.value)
        return out

    def elapsed_ms(self, a, b):
        ms = self.ct.c_float()
        assert self.hip.hipEventElapsedTime(self.ct.byref(ms), self.ct.c_void_p(a), self.ct.c_void_p(b)) == 0
        return float(ms.value)

    def destroy(self, evs):
        for e in evs:
            self.hip.hipEventDestroy(self.ct.c_void_p(e))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--cpu-rows", type=int, default=3072, help="rows of the bounded oracle sample (0 = skip)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run three plain 1 GiB device copies and exit (scale for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.copy_calibration:
        import torch
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda:0").fill_(7)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_calibration_bytes": 1 << 30, "copies": 3}))
        return 0
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported"
              % args.gpus, file=sys.stderr)
        return 2

    import torch
    from paper_2505_24034_amd import binding as L
    import synth

    L.load()                                   # fails loudly if the HIP library is not built
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    w = synth.WORKLOADS[args.workload]
    x = synth.make_inputs(w, dev)
    B, T, N, d, V = w.B, w.T, w.N, w.d, w.V
    dt = L.BF16 if w.dtype == "bf16" else L.F32
    mask_flat = x["mask"].reshape(-1)
    n_valid = int(x["mask"].sum().item())

    ws_fwd = torch.empty(L.workspace_bytes(N, d, V, dt, L.PASS_LOGPROBS), dtype=torch.uint8, device=dev)
    ws_loss = torch.empty(L.workspace_bytes(N, 0, 0, 0, L.PASS_LOSS_FWD), dtype=torch.uint8, device=dev)
    ws_bwd = torch.empty(L.workspace_bytes(N, d, V, dt, L.PASS_LOSS_BWD), dtype=torch.uint8, device=dev)
    dH = torch.empty(N, d, dtype=x["H"].dtype, device=dev)
    dW = torch.empty(V, d, dtype=x["W"].dtype, device=dev)
    stream = torch.cuda.current_stream()

    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(4)] for _ in range(args.steps)]
    hipev = HipEvents()
    phase = [hipev.create(6) for _ in range(args.steps)]      # backward phase boundaries, recorded by the library

    def step(e=None, ph=None):
        if e:
            e[0].record(stream)
        logp, lse = L.token_logprobs(x["H"], x["W"], x["targets"], mask_flat, ws=ws_fwd, stream=stream)
        if e:
            e[1].record(stream)
        loss, coef, stats = L.offpolicy_loss_fwd(logp, x["mu_logp"], x["adv"], x["mask"], B, T, rho=2.0,
                                                 targets=x["targets"], V=V, ws=ws_loss, stream=stream)
        if e:
            e[2].record(stream)
        L.offpolicy_loss_bwd(x["H"], x["W"], x["targets"], lse, coef, dH=dH, dW=dW, ws=ws_bwd, stream=stream,
                             phase_events=ph)
        if e:
            e[3].record(stream)
        return loss, stats

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        loss, stats = step(ev[k], phase[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall / args.steps * 1e3
    t_lp = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps      # ms, token_logprobs (forward contraction)
    t_loss = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    t_bwd = sum(e[2].elapsed_time(e[3]) for e in ev) / args.steps
    # Masked rows are compacted away before every contraction, so the algorithmic work of one contraction is
    # 2 * n_valid * V * d flop (never the 2 * N * V * d of the padded batch).
    flops_gemm = 2.0 * n_valid * V * d
    fwd_tflops = flops_gemm / (t_lp * 1e-3) / 1e12
    t_dz = sum(hipev.elapsed_ms(p[1], p[2]) for p in phase) / args.steps      # k_bwd_dz alone
    t_dh = sum(hipev.elapsed_ms(p[2], p[3]) for p in phase) / args.steps      # dH contraction alone
    t_dw = sum(hipev.elapsed_ms(p[4], p[5]) for p in phase) / args.steps      # dW contraction alone
    for p in phase:
        hipev.destroy(p)
    kernels = [
        ("k_fwd_partials (LM-head contraction + online logsumexp; timed as llamarl_token_logprobs, i.e. with "
         "~0.1 ms of row compaction and partial merge)", t_lp),
        ("k_bwd_dz (logits recompute + dz)", t_dz),
        ("k_gemm_store<k-major> (dH = dz W, split-K partials)" if w.dtype == "bf16" else "k_gemm_store (dH)", t_dh),
        ("k_gemm_store (dW = dz^T H)", t_dw),
    ]
    per_kernel = [{"kernel": n, "ms": t, "achieved": flops_gemm / (t * 1e-3) / 1e12, "unit": "TFLOP/s",
                   "frac": flops_gemm / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS} for n, t in kernels]
    dom = max(per_kernel, key=lambda k: k["ms"])                             # the dominant (slowest) contraction
    out = {
        "metric": METRIC, "value": N / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "d": d, "V": V, "B": B, "T": T, "n_valid_tokens": n_valid, "rho": 2.0,
                   "note": "value counts all B*T positions; masked positions cost nothing (row compaction)"},
        "tokens_per_s_valid": n_valid / (ms_step * 1e-3),
        "mfma_peak_frac_method_8NVd": 4 * flops_gemm / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "mfma_peak_frac_model_6NVd": 3 * flops_gemm / (ms_step * 1e-3) / 1e12 / PEAK_BF16_TFLOPS,
        "ms_token_logprobs": t_lp, "ms_loss_fwd": t_loss, "ms_loss_bwd": t_bwd,
        "loss": float(loss.item()), "stats": [float(v) for v in stats.tolist()],
        # the dominant kernel = the slowest of the four contractions, each 2*n_valid*V*d flop per launch
        "roofline": {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["achieved"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac"],
                     "traffic": measured_traffic(dom["kernel"].split()[0].split("<")[0] +
                                                 ("<llamarl::BF16, true" if "k-major" in dom["kernel"] else ""))
                     if w.name == "llama3_8b" else None,
                     "traffic_note": "bytes per launch between L2 and fabric, rocprofv3 FETCH_SIZE x2.0 + WRITE_SIZE "
                                     "x1.0 (plain-copy calibration; includes Infinity-Cache hits)"},
        "roofline_per_kernel": per_kernel,
    }
    if w.dtype == "bf16":
        out["library_gemm"] = library_gemm(x, flops_gemm)
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(x, w, args.cpu_rows)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
