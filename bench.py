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


def cpu_baseline(x, w, rows, rows_one_thread):
    """The fp64 oracle as it stands, on `rows` valid token rows of the same batch at full V and d, with all host
    threads of the BLAS pool, and again on `rows_one_thread` rows with the pool limited to one thread."""
    import numpy as np
    import torch
    from threadpoolctl import threadpool_info, threadpool_limits
    from oracle import aipo_oracle as orc
    import synth
    cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    valid = torch.nonzero(x["mask"].reshape(-1))[:, 0]
    W = synth.to_oracle(x["W"])          # bf16 bits: the oracle widens them itself, inside the timed call

    def leg(n):
        idx = valid[:n]
        n = int(idx.numel())
        H = synth.to_oracle(x["H"][idx])
        tg = synth.to_oracle(x["targets"][idx])
        mu = synth.to_oracle(x["mu_logp"][idx])
        t0 = time.perf_counter()
        out = orc.aipo_step(H, W, tg, mu, np.array([1.0]), np.ones((1, n), dtype=np.uint8), 2.0)
        dt = time.perf_counter() - t0
        assert np.isfinite(out["loss"])
        return n, dt

    n_all, t_all = leg(rows)
    res = {"value": n_all / t_all, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
           "sample": "first %d valid token rows of the batch, full V=%d and d=%d, oracle fwd+bwd once, %.1f s; cost is "
                     "linear in rows" % (n_all, w.V, w.d, t_all)}
    if rows_one_thread > 0:
        with threadpool_limits(limits=1):
            n_one, t_one = leg(rows_one_thread)
        res["one_thread"] = {"value": n_one / t_one, "unit": "tokens/s", "cores": 1,
                             "sample": "first %d valid token rows, %.1f s" % (n_one, t_one)}
    return res


def library_gemm(x, flops):
    """Context, not part of the path: the vendor library's plain bf16 GEMMs (torch.matmul -> hipBLASLt) of the same
    three contraction shapes, timed the same way on the same machine -- logits = H_active W^T written to HBM, and
    the two gradient products with a stand-in dz of the right shape and layout (vocab-major, as the path stages it).
    They show what a tuned GEMM reaches here under the chip's power limit; the path's kernels fuse their epilogues
    and never write the logits."""
    import torch
    rows = x["mask"].reshape(-1).nonzero().squeeze(1)
    Hc = x["H"].index_select(0, rows).contiguous()
    W = x["W"]
    n, V, d = Hc.shape[0], W.shape[0], W.shape[1]
    g = torch.Generator(device=Hc.device).manual_seed(3)
    dzT = (torch.randn(V, n, generator=g, device=Hc.device, dtype=torch.float32) * 1e-5).to(Hc.dtype)   # [V, n]
    logits = torch.empty(n, V, dtype=Hc.dtype, device=Hc.device)
    dH = torch.empty(n, d, dtype=Hc.dtype, device=Hc.device)
    dW = torch.empty(V, d, dtype=Hc.dtype, device=Hc.device)

    def timed(f, reps=10):
        for _ in range(3):
            f()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            f()
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        return {"ms": ms, "achieved": flops / (ms * 1e-3) / 1e12, "frac": flops / (ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS}

    res = timed(lambda: torch.matmul(Hc, W.t(), out=logits))
    res.update({"what": "torch.matmul bf16 (hipBLASLt), [n_valid,d] x [d,V] -> logits in HBM, same shape",
                "unit": "TFLOP/s",
                "dH_shape": timed(lambda: torch.matmul(dzT.t(), W, out=dH)),      # dz [n,V] (stored vocab-major) x W [V,d]
                "dW_shape": timed(lambda: torch.matmul(dzT, Hc, out=dW))})         # dz^T [V,n] x H [n,d]
    return res


def streaming_epilogue(L, x, w, t_loss_ms, dev, stream):
    """The HBM-bound part of the path (ratio, clip, advantage weighting, masked means: llamarl_offpolicy_loss_fwd, two
    launches).  Algorithmic bytes per token: logp 4 + mu_logp 4 + mask 1 + targets 4 read, coef 4 written (twice the
    mask and targets: the per-generation length pass reads them too).  At the workload's own N the call is a few
    microseconds of launch latency; the same call on a batch of 4 Mi tokens shows what the kernels stream at."""
    import torch
    per_token = 4 + 4 + 2 * (1 + 4) + 4
    res = {"bytes_per_token": per_token,
           "at_workload": {"tokens": w.N, "ms": t_loss_ms, "GBps": w.N * per_token / (t_loss_ms * 1e-3) / 1e9}}
    Bb, Tb = 512, 8192
    n = Bb * Tb
    g = torch.Generator(device=dev).manual_seed(7)
    logp = -torch.rand(n, generator=g, device=dev) * 10
    mu = logp + 0.1 * torch.randn(n, generator=g, device=dev)
    adv = torch.randn(Bb, generator=g, device=dev)
    mask = (torch.rand(Bb, Tb, generator=g, device=dev) < 0.6).to(torch.uint8)
    tg = torch.randint(0, w.V, (n,), generator=g, device=dev, dtype=torch.int32)
    ws = torch.empty(L.workspace_bytes(n, 0, 0, 0, L.PASS_LOSS_FWD), dtype=torch.uint8, device=dev)
    for _ in range(3):
        L.offpolicy_loss_fwd(logp, mu, adv, mask, Bb, Tb, rho=2.0, targets=tg, V=w.V, ws=ws, stream=stream)
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(11)]
    for a, b in evs:
        a.record(stream)
        L.offpolicy_loss_fwd(logp, mu, adv, mask, Bb, Tb, rho=2.0, targets=tg, V=w.V, ws=ws, stream=stream)
        b.record(stream)
    torch.cuda.synchronize()
    ms = sorted(a.elapsed_time(b) for a, b in evs)[len(evs) // 2]
    res["at_4Mi_tokens"] = {"tokens": n, "ms": ms, "GBps": n * per_token / (ms * 1e-3) / 1e9,
                            "peak_GBps": 8000.0, "frac": n * per_token / (ms * 1e-3) / 1e9 / 8000.0}
    return res


def optional(leg):
    """An optional (context) leg of the line: its failure is reported in its place and never costs the headline."""
    try:
        return leg()
    except Exception as e:                                   # noqa: BLE001 - reported, not hidden
        return {"error": "%s: %s" % (type(e).__name__, e)}


def ceiling_with_traffic(L, x, w, iters, sink, stream, median):
    """The MFMA loop in the main loop's slot order, operands = values of this workload (rows of H and of W), with
    the main loop's LDS fragment reads and / or slab loads added back (no barrier, no wait)."""
    import torch
    dev = sink.device
    panels = torch.empty(2, 256, 4096, dtype=torch.bfloat16, device=dev)
    if w.dtype == "bf16" and w.d >= 4096 and w.N >= 256:
        panels[0].copy_(x["H"][:256, :4096])
        panels[1].copy_(x["W"][:256, :4096])
    else:
        panels[0].normal_()
        panels[1].normal_(std=0.02)
    res = {}
    for name, mode in (("schedule_only", 0), ("lds_reads", 1), ("slab_loads", 2), ("lds_reads_and_slab_loads", 3)):
        for _ in range(2):
            fl = L.mfma_ceiling_traffic(mode, iters, panels, sink, stream=stream)
        tev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
        for a, b in tev:
            a.record(stream)
            L.mfma_ceiling_traffic(mode, iters, panels, sink, stream=stream)
            b.record(stream)
        torch.cuda.synchronize()
        res[name] = fl / (median([a.elapsed_time(b) for a, b in tev]) * 1e-3) / 1e12
    return res


def graph_replay(step, reps, median):
    """The same step recorded once into a HIP graph and replayed: what a launch-bound (small) batch gains when the
    caller captures the path, which it may, since the entry points only enqueue kernels."""
    import torch
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(stream=side)
    torch.cuda.synchronize()
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
    graph.replay()
    for a, b in ev:
        a.record()
        graph.replay()
        b.record()
    torch.cuda.synchronize()
    return {"ms_per_step": median([a.elapsed_time(b) for a, b in ev]), "replays": reps,
            "what": "one hipGraphLaunch per step (token_logprobs + loss_fwd + loss_bwd captured once)"}


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
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="llama3_8b")
    ap.add_argument("--cpu-rows", type=int, default=3072, help="rows of the bounded oracle sample (0 = skip)")
    ap.add_argument("--cpu-rows-one-thread", type=int, default=192, help="rows of the single-thread oracle leg")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the MFMA-ceiling, streaming-epilogue and library-GEMM legs (profiling runs)")
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

    def step(e=None, ph=None, stream=stream):
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

    def median(v):
        v = sorted(v)
        return 0.5 * (v[(len(v) - 1) // 2] + v[len(v) // 2])

    # ---- headline: the three named entry points back to back, K timed steps
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        loss, stats = step(ev[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_step_wall = wall / args.steps * 1e3
    ms_step = median([e[0].elapsed_time(e[3]) for e in ev])                # median step, HIP events on the stream
    t_lp = median([e[0].elapsed_time(e[1]) for e in ev])                   # llamarl_token_logprobs
    t_loss = median([e[1].elapsed_time(e[2]) for e in ev])                 # llamarl_offpolicy_loss_fwd
    t_bwd = median([e[2].elapsed_time(e[3]) for e in ev])                  # llamarl_offpolicy_loss_bwd
    # Masked rows are compacted away before every contraction, so the algorithmic work of one contraction is
    # 2 * n_valid * V * d flop (never the 2 * N * V * d of the padded batch).
    flops_gemm = 2.0 * n_valid * V * d

    # ---- per-kernel times of the backward: a separate loop through the variant that records events between its
    # kernels (a measurement aid; the headline above times the plain entry point)
    hipev = HipEvents()
    n_ph = min(args.steps, 10)
    phase = [hipev.create(6) for _ in range(n_ph)]
    for k in range(n_ph):
        step(None, phase[k])
    torch.cuda.synchronize()
    t_dz = median([hipev.elapsed_ms(p[1], p[2]) for p in phase])           # k_bwd_dz alone
    t_dh = median([hipev.elapsed_ms(p[2], p[3]) for p in phase])           # dH contraction alone
    t_dw = median([hipev.elapsed_ms(p[4], p[5]) for p in phase])           # dW contraction alone
    t_setup = median([hipev.elapsed_ms(p[0], p[1]) for p in phase])
    for p in phase:
        hipev.destroy(p)
    kernels = [
        ("k_fwd_partials (LM-head contraction + online logsumexp; timed as llamarl_token_logprobs, i.e. with "
         "the row compaction and partial merge)", t_lp),
        ("k_bwd_dz (logits recompute + dz)", t_dz),
        ("k_gemm_store<k-major> (dH = dz W; with the reduction of its last round's split tiles)" if w.dtype == "bf16"
         else "k_gemm_store (dH)", t_dh),
        ("k_gemm_store (dW = dz^T H)", t_dw),
    ]
    per_kernel = [{"kernel": n, "ms": t, "achieved": flops_gemm / (t * 1e-3) / 1e12, "unit": "TFLOP/s",
                   "frac": flops_gemm / (t * 1e-3) / 1e12 / PEAK_BF16_TFLOPS} for n, t in kernels]
    dom = max(per_kernel, key=lambda k: k["ms"])                             # the dominant (slowest) contraction

    # ---- what the matrix pipes sustain on this machine with nothing else running (MFMA-only kernel, same
    # instruction and wave shape): the published peak assumes 2.4 GHz, which the chip does not hold under MFMA load
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    iters = 20 if args.no_extras else 20000                                  # ~10 ms per launch
    for _ in range(3):
        ceil_flops = L.mfma_ceiling(iters, sink, stream=stream)
    cev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(7)]
    for a, b in cev:
        a.record(stream)
        L.mfma_ceiling(iters, sink, stream=stream)
        b.record(stream)
    torch.cuda.synchronize()
    ceil_ms = median([a.elapsed_time(b) for a, b in cev])
    ceil_tflops = ceil_flops / (ceil_ms * 1e-3) / 1e12
    ceil_traffic = None
    if not args.no_extras:
        ceil_traffic = optional(lambda: ceiling_with_traffic(L, x, w, iters, sink, stream, median))
    step_tflops = 4 * flops_gemm / (ms_step * 1e-3) / 1e12

    out = {
        "metric": METRIC, "value": N / (ms_step * 1e-3), "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms_step, "ms_per_step_is": "median of the timed steps (HIP events)",
        "ms_per_step_mean_wall": ms_step_wall, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "d": d, "V": V, "B": B, "T": T, "n_valid_tokens": n_valid, "rho": 2.0,
                   "note": "value counts all B*T positions; masked positions cost nothing (row compaction)"},
        "tokens_per_s_valid": n_valid / (ms_step * 1e-3),
        "mfma_peak_frac_method_8NVd": step_tflops / PEAK_BF16_TFLOPS,
        "mfma_peak_frac_model_6NVd": 0.75 * step_tflops / PEAK_BF16_TFLOPS,
        "mfma_ceiling": {"what": "MFMA-only kernel (v_mfma_f32_16x16x32_bf16 from registers, 8 wavefronts x 8x4 "
                                 "blocks per CU, no LDS / memory traffic), %d x 2 k-steps per wavefront" % iters,
                         "ms": ceil_ms, "achieved": ceil_tflops, "unit": "TFLOP/s",
                         "frac_of_published_peak": ceil_tflops / PEAK_BF16_TFLOPS,
                         "with_operand_traffic_TFLOPs": ceil_traffic,
                         "with_operand_traffic_is": "the same MFMA loop in the main loop's slot order on this "
                                                    "workload's operand values, plus the main loop's LDS fragment "
                                                    "reads and / or L2->LDS slab loads; no barrier, no wait, "
                                                    "operands resident in L2"},
        "step_frac_of_measured_ceiling_8NVd": step_tflops / ceil_tflops,
        "ms_token_logprobs": t_lp, "ms_loss_fwd": t_loss, "ms_loss_bwd": t_bwd,
        "ms_bwd_setup_kernels": t_setup,
        "loss": float(loss.item()), "stats": [float(v) for v in stats.tolist()],
        # the dominant kernel = the slowest of the four contractions, each 2*n_valid*V*d flop per launch
        "roofline": {"bound": "mfma", "kernel": dom["kernel"], "achieved": dom["achieved"],
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": dom["frac"],
                     "measured_ceiling": ceil_tflops, "frac_of_measured_ceiling": dom["achieved"] / ceil_tflops,
                     "traffic": measured_traffic(dom["kernel"].split()[0].split("<")[0] +
                                                 ("<llamarl::BF16, true" if "k-major" in dom["kernel"] else ""))
                     if w.name == "llama3_8b" else None,
                     "traffic_note": "bytes per launch between L2 and fabric, rocprofv3 FETCH_SIZE x2.0 + WRITE_SIZE "
                                     "x1.0 (plain-copy calibration; includes Infinity-Cache hits); read from "
                                     "profiles/bench_llama3_8b_hbm_traffic_pmc.md, not measured in this run"},
        "roofline_per_kernel": per_kernel,
    }
    if not args.no_extras:
        out["streaming_epilogue"] = optional(lambda: streaming_epilogue(L, x, w, t_loss, dev, stream))
        out["graph_replay"] = optional(lambda: graph_replay(step, args.steps, median))
    if args.no_extras:
        del out["mfma_ceiling"], out["step_frac_of_measured_ceiling_8NVd"]
        del out["roofline"]["measured_ceiling"], out["roofline"]["frac_of_measured_ceiling"]
    if w.dtype == "bf16" and not args.no_extras:
        out["library_gemm"] = optional(lambda: library_gemm(x, flops_gemm))
    if args.cpu_rows > 0:
        out["cpu_baseline"] = cpu_baseline(x, w, args.cpu_rows, args.cpu_rows_one_thread)
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
