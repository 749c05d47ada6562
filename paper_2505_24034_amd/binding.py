"""ctypes binding of libllamarl.so: argument marshalling only.

Function names and argument order follow include/llamarl.h.  torch supplies
device memory (`.data_ptr()`) and the HIP stream handle; every step of the path
runs in the library's kernels.  There is no fallback: if the library is not
built, or a call returns a non-zero status, a LlamarlError is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libllamarl.so")

OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP = 0, 1, 2, 3, 4
F32, BF16 = 0, 1
CLIP_AIPO, CLIP_PPO = 0, 1
NORM_TOKEN_MEAN, NORM_SEQ_MEAN, NORM_SUM_T_MEAN_B = 0, 1, 2
PASS_LOGPROBS, PASS_LOSS_FWD, PASS_LOSS_BWD = 0, 1, 2

EXPORTS = ("llamarl_workspace_bytes", "llamarl_last_error", "llamarl_version", "llamarl_token_logprobs",
           "llamarl_offpolicy_loss_fwd", "llamarl_offpolicy_loss_bwd", "llamarl_offpolicy_loss_bwd_phases",
           "llamarl_group_advantages", "llamarl_kl_shaped_rewards", "llamarl_mfma_ceiling", "llamarl_mfma_ceiling_traffic",
           "llamarl_offpolicy_loss_fwd_static", "llamarl_token_logprobs_partial", "llamarl_merge_partials",
           "llamarl_offpolicy_loss_bwd_slice", "llamarl_bwd_workspace_bytes", "llamarl_offpolicy_loss_bwd_chunked")


class LlamarlError(RuntimeError):
    def __init__(self, status, message):
        super().__init__("llamarl status %d: %s" % (status, message))
        self.status = status


class LossParams(ctypes.Structure):
    _fields_ = [("rho", ctypes.c_float), ("clip_mode", ctypes.c_int), ("eps_lo", ctypes.c_float),
                ("eps_hi", ctypes.c_float), ("norm_mode", ctypes.c_int)]


_lib = None


def load():
    """Load the in-tree shared library (built by build.py); raises if it is missing."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise LlamarlError(-1, "%s not found: build it with `python -m paper_2505_24034_amd.build`" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i64, sz, ci, cf = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t, ctypes.c_int, ctypes.c_float
    lib.llamarl_workspace_bytes.restype = sz
    lib.llamarl_workspace_bytes.argtypes = [i64, i64, i64, ci, ci]
    lib.llamarl_last_error.restype = ctypes.c_char_p
    lib.llamarl_last_error.argtypes = []
    lib.llamarl_version.restype = ctypes.c_char_p
    lib.llamarl_version.argtypes = []
    lib.llamarl_token_logprobs.restype = ci
    lib.llamarl_token_logprobs.argtypes = [vp, vp, vp, vp, i64, i64, i64, ci, vp, vp, vp, sz, vp]
    lib.llamarl_offpolicy_loss_fwd.restype = ci
    lib.llamarl_offpolicy_loss_fwd.argtypes = [vp, vp, vp, ci, vp, vp, i64, i64, i64, ctypes.POINTER(LossParams),
                                               vp, vp, vp, vp, sz, vp]
    lib.llamarl_offpolicy_loss_fwd_static.restype = ci
    lib.llamarl_offpolicy_loss_fwd_static.argtypes = [vp, vp, vp, ci, vp, vp, i64, i64, i64,
                                                      ctypes.POINTER(LossParams), vp, vp, vp, vp]
    lib.llamarl_offpolicy_loss_bwd.restype = ci
    lib.llamarl_offpolicy_loss_bwd.argtypes = [vp, vp, vp, vp, vp, cf, i64, i64, i64, ci, vp, vp, ci, ci, vp, sz, vp]
    lib.llamarl_offpolicy_loss_bwd_phases.restype = ci
    lib.llamarl_offpolicy_loss_bwd_phases.argtypes = [vp, vp, vp, vp, vp, cf, i64, i64, i64, ci, vp, vp, ci, ci, vp, sz,
                                                      vp, ctypes.POINTER(vp)]
    lib.llamarl_group_advantages.restype = ci
    lib.llamarl_group_advantages.argtypes = [vp, i64, i64, ci, cf, vp, vp]
    lib.llamarl_kl_shaped_rewards.restype = ci
    lib.llamarl_kl_shaped_rewards.argtypes = [vp, vp, vp, vp, i64, i64, cf, vp, vp, vp]
    lib.llamarl_token_logprobs_partial.restype = ci
    lib.llamarl_token_logprobs_partial.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, ci, vp, vp, vp, vp, sz, vp]
    lib.llamarl_merge_partials.restype = ci
    lib.llamarl_merge_partials.argtypes = [vp, vp, vp, ci, i64, vp, vp, vp]
    lib.llamarl_offpolicy_loss_bwd_slice.restype = ci
    lib.llamarl_offpolicy_loss_bwd_slice.argtypes = [vp, vp, vp, vp, vp, cf, i64, i64, i64, i64, ci, vp, vp, ci, ci, vp,
                                                     sz, vp]
    lib.llamarl_bwd_workspace_bytes.restype = sz
    lib.llamarl_bwd_workspace_bytes.argtypes = [i64, i64, i64, ci, i64]
    lib.llamarl_offpolicy_loss_bwd_chunked.restype = ci
    lib.llamarl_offpolicy_loss_bwd_chunked.argtypes = [vp, vp, vp, vp, vp, cf, i64, i64, i64, ci, vp, vp, ci, ci, i64,
                                                       vp, sz, vp]
    lib.llamarl_mfma_ceiling.restype = ci
    lib.llamarl_mfma_ceiling.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_double), vp]
    lib.llamarl_mfma_ceiling_traffic.restype = ci
    lib.llamarl_mfma_ceiling_traffic.argtypes = [ci, ci, vp, ctypes.c_size_t, vp, ctypes.POINTER(ctypes.c_double), vp]
    _lib = lib
    return lib


def _check(status):
    if status != OK:
        raise LlamarlError(status, load().llamarl_last_error().decode())


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return BF16
    if t.dtype == torch.float32:
        return F32
    raise LlamarlError(ERR_INVALID_ARG, "unsupported tensor dtype %s" % t.dtype)


def _need(t, dtype, name):
    if t.dtype != dtype or not t.is_contiguous() or not t.is_cuda:
        raise LlamarlError(ERR_INVALID_ARG, "%s must be a contiguous device tensor of %s" % (name, dtype))


def workspace_bytes(N, d, V, dt, which):
    return int(load().llamarl_workspace_bytes(N, d, V, dt, which))


def _workspace(nbytes, device, ws):
    if ws is None:
        ws = torch.empty(max(nbytes, 16), dtype=torch.uint8, device=device)
    return ws


def token_logprobs(H, W, targets, mask=None, ws=None, stream=None):
    """llamarl_token_logprobs: returns (logp [N], lse [N]) float32 device tensors."""
    lib = load()
    dt = _dtype_code(H)
    _need(H, H.dtype, "H"); _need(W, H.dtype, "W"); _need(targets, torch.int32, "targets")
    N, d = H.shape
    V = W.shape[0]
    if W.shape[1] != d or targets.numel() != N:
        raise LlamarlError(ERR_INVALID_ARG, "shape mismatch between H, W, targets")
    if mask is not None:
        _need(mask, torch.uint8, "mask")
        if mask.numel() != N:
            raise LlamarlError(ERR_INVALID_ARG, "mask must have N entries")
    logp = torch.empty(N, dtype=torch.float32, device=H.device)
    lse = torch.empty(N, dtype=torch.float32, device=H.device)
    ws = _workspace(workspace_bytes(N, d, V, dt, PASS_LOGPROBS), H.device, ws)
    _check(lib.llamarl_token_logprobs(_ptr(H), _ptr(W), _ptr(targets), _ptr(mask), N, d, V, dt, _ptr(logp), _ptr(lse),
                                      _ptr(ws), ws.numel(), _stream(stream)))
    return logp, lse


def offpolicy_loss_fwd(logp, mu_logp, adv, mask, B, T, rho=2.0, norm_mode=NORM_TOKEN_MEAN, clip_mode=CLIP_AIPO,
                       eps_lo=0.2, eps_hi=0.2, targets=None, V=0, ws=None, stream=None):
    """llamarl_offpolicy_loss_fwd: returns (loss [1], coef [B*T], stats [5]) float32 device tensors."""
    lib = load()
    N = B * T
    _need(logp, torch.float32, "logp"); _need(mu_logp, torch.float32, "mu_logp"); _need(adv, torch.float32, "adv")
    if logp.numel() != N or mu_logp.numel() != N or adv.numel() not in (B, N):
        raise LlamarlError(ERR_INVALID_ARG, "shape mismatch between logp, mu_logp, adv and B*T")
    per_token = 1 if (adv.numel() == N and N != B) else 0
    if mask is not None:
        _need(mask, torch.uint8, "mask")
        if mask.numel() != N:
            raise LlamarlError(ERR_INVALID_ARG, "mask must have B*T entries")
    if targets is not None:
        _need(targets, torch.int32, "targets")
    dev = logp.device
    loss = torch.empty(1, dtype=torch.float32, device=dev)
    coef = torch.empty(N, dtype=torch.float32, device=dev)
    stats = torch.empty(5, dtype=torch.float32, device=dev)
    p = LossParams(float(rho), int(clip_mode), float(eps_lo), float(eps_hi), int(norm_mode))
    ws = _workspace(workspace_bytes(N, 0, 0, 0, PASS_LOSS_FWD), dev, ws)
    _check(lib.llamarl_offpolicy_loss_fwd(_ptr(logp), _ptr(mu_logp), _ptr(adv), per_token, _ptr(mask), _ptr(targets),
                                          int(V), B, T, ctypes.byref(p), _ptr(loss), _ptr(coef), _ptr(stats),
                                          _ptr(ws), ws.numel(), _stream(stream)))
    return loss, coef, stats


def offpolicy_loss_fwd_static(logp, mu_logp, adv, mask, B, T, loss, coef, stats, rho=2.0, norm_mode=NORM_TOKEN_MEAN,
                              clip_mode=CLIP_AIPO, eps_lo=0.2, eps_hi=0.2, targets=None, V=0, stream=None):
    """llamarl_offpolicy_loss_fwd_static: the caller passes every buffer (loss [1], coef [B*T], stats [5]); the
    call allocates nothing and uses the library's static device scratch."""
    lib = load()
    N = B * T
    for t, n, name in ((logp, N, "logp"), (mu_logp, N, "mu_logp"), (coef, N, "coef"), (loss, 1, "loss"),
                       (stats, 5, "stats")):
        _need(t, torch.float32, name)
        if t.numel() != n:
            raise LlamarlError(ERR_INVALID_ARG, "%s must have %d entries" % (name, n))
    _need(adv, torch.float32, "adv")
    if adv.numel() not in (B, N):
        raise LlamarlError(ERR_INVALID_ARG, "adv must have B or B*T entries")
    per_token = 1 if (adv.numel() == N and N != B) else 0
    if mask is not None:
        _need(mask, torch.uint8, "mask")
    if targets is not None:
        _need(targets, torch.int32, "targets")
    p = LossParams(float(rho), int(clip_mode), float(eps_lo), float(eps_hi), int(norm_mode))
    _check(lib.llamarl_offpolicy_loss_fwd_static(_ptr(logp), _ptr(mu_logp), _ptr(adv), per_token, _ptr(mask),
                                                 _ptr(targets), int(V), B, T, ctypes.byref(p), _ptr(loss),
                                                 _ptr(coef), _ptr(stats), _stream(stream)))
    return loss, coef, stats


def bwd_workspace_bytes(N, d, V, dt, max_rows_per_pass):
    return int(load().llamarl_bwd_workspace_bytes(N, d, V, dt, max_rows_per_pass))


def offpolicy_loss_bwd(H, W, targets, lse, coef, grad_loss=1.0, dW_dtype=None, dW=None, accumulate_dW=False,
                       dH=None, ws=None, stream=None, phase_events=None, max_rows_per_pass=None):
    """llamarl_offpolicy_loss_bwd: returns (dH [N,d] in H's dtype, dW [V,d] in dW_dtype).
    phase_events: six raw hipEvent_t handles (ints) -> llamarl_offpolicy_loss_bwd_phases is called instead.
    max_rows_per_pass: -> llamarl_offpolicy_loss_bwd_chunked (workspace for that many active rows at a time)."""
    lib = load()
    dt = _dtype_code(H)
    _need(H, H.dtype, "H"); _need(W, H.dtype, "W"); _need(targets, torch.int32, "targets")
    _need(lse, torch.float32, "lse"); _need(coef, torch.float32, "coef")
    N, d = H.shape
    V = W.shape[0]
    if dW is not None:
        dW_dtype = dW.dtype
    if dW_dtype is None:
        dW_dtype = H.dtype
    if dW is None:
        if accumulate_dW:
            raise LlamarlError(ERR_INVALID_ARG, "accumulate_dW needs an existing dW tensor")
        dW = torch.empty(V, d, dtype=dW_dtype, device=H.device)
    if dH is None:
        dH = torch.empty(N, d, dtype=H.dtype, device=H.device)
    _need(dW, dW_dtype, "dW"); _need(dH, H.dtype, "dH")
    if max_rows_per_pass is not None:
        ws = _workspace(bwd_workspace_bytes(N, d, V, dt, int(max_rows_per_pass)), H.device, ws)
        _check(lib.llamarl_offpolicy_loss_bwd_chunked(
            _ptr(H), _ptr(W), _ptr(targets), _ptr(lse), _ptr(coef), float(grad_loss), N, d, V, dt, _ptr(dH), _ptr(dW),
            _dtype_code(dW), int(bool(accumulate_dW)), int(max_rows_per_pass), _ptr(ws), ws.numel(), _stream(stream)))
        return dH, dW
    ws = _workspace(workspace_bytes(N, d, V, dt, PASS_LOSS_BWD), H.device, ws)
    args = (_ptr(H), _ptr(W), _ptr(targets), _ptr(lse), _ptr(coef), float(grad_loss), N, d, V, dt, _ptr(dH), _ptr(dW),
            _dtype_code(dW), int(bool(accumulate_dW)), _ptr(ws), ws.numel(), _stream(stream))
    if phase_events is None:
        _check(lib.llamarl_offpolicy_loss_bwd(*args))
    else:
        ev = (ctypes.c_void_p * 6)(*[ctypes.c_void_p(int(e)) for e in phase_events])
        _check(lib.llamarl_offpolicy_loss_bwd_phases(*args, ev))
    return dH, dW


def group_advantages(rewards, n, normalise_std=False, eps=1e-6, stream=None):
    """llamarl_group_advantages: rewards [P*n] (prompt-major) -> advantages [P*n]."""
    lib = load()
    _need(rewards, torch.float32, "rewards")
    if n <= 0 or rewards.numel() % n != 0:
        raise LlamarlError(ERR_INVALID_ARG, "rewards must hold P*n entries")
    P = rewards.numel() // n
    adv = torch.empty_like(rewards)
    _check(lib.llamarl_group_advantages(_ptr(rewards), P, n, int(bool(normalise_std)), float(eps), _ptr(adv),
                                        _stream(stream)))
    return adv


def kl_shaped_rewards(rewards, logp, base_logp, mask, lambda_kl, stream=None):
    """llamarl_kl_shaped_rewards: rewards [B], logp / base_logp / mask [B,T] -> (shaped [B], kl [B])."""
    lib = load()
    _need(rewards, torch.float32, "rewards")
    _need(logp, torch.float32, "logp")
    _need(base_logp, torch.float32, "base_logp")
    if mask is not None:
        _need(mask, torch.uint8, "mask")
    B = rewards.numel()
    if B <= 0 or logp.numel() % B != 0 or base_logp.numel() != logp.numel() or \
            (mask is not None and mask.numel() != logp.numel()):
        raise LlamarlError(ERR_INVALID_ARG, "logp, base_logp and mask must hold B*T entries")
    T = logp.numel() // B
    shaped = torch.empty_like(rewards)
    kl = torch.empty_like(rewards)
    _check(lib.llamarl_kl_shaped_rewards(_ptr(rewards), _ptr(logp), _ptr(base_logp), _ptr(mask), B, T,
                                         float(lambda_kl), _ptr(shaped), _ptr(kl), _stream(stream)))
    return shaped, kl


def mfma_ceiling(iters, sink, stream=None):
    """llamarl_mfma_ceiling (measurement aid): enqueues the MFMA-only kernel, returns the flop it executes."""
    lib = load()
    _need(sink, torch.float32, "sink")
    flops = ctypes.c_double()
    _check(lib.llamarl_mfma_ceiling(int(iters), _ptr(sink), ctypes.byref(flops), _stream(stream)))
    return float(flops.value)


def mfma_ceiling_traffic(traffic, iters, panels, sink, stream=None):
    """llamarl_mfma_ceiling_traffic (measurement aid): the MFMA loop plus the main loop's LDS reads (traffic bit 0)
    and slab loads (bit 1); returns the flop it executes.  panels: device tensor of at least 4 MiB."""
    lib = load()
    flops = ctypes.c_double(0.0)
    _check(lib.llamarl_mfma_ceiling_traffic(int(traffic), int(iters), _ptr(panels), panels.numel() * panels.element_size(),
                                            _ptr(sink), ctypes.byref(flops), _stream(stream)))
    return flops.value


def token_logprobs_partial(H, W_slice, targets, v0, V_total, mask=None, ws=None, stream=None):
    """llamarl_token_logprobs_partial: one vocabulary shard's (m [N], s [N], zt [N])."""
    lib = load()
    dt = _dtype_code(H)
    _need(H, H.dtype, "H"); _need(W_slice, H.dtype, "W_slice"); _need(targets, torch.int32, "targets")
    N, d = H.shape
    Vs = W_slice.shape[0]
    if W_slice.shape[1] != d or targets.numel() != N:
        raise LlamarlError(ERR_INVALID_ARG, "shape mismatch between H, W_slice, targets")
    if mask is not None:
        _need(mask, torch.uint8, "mask")
    m, s, zt = (torch.empty(N, dtype=torch.float32, device=H.device) for _ in range(3))
    ws = _workspace(workspace_bytes(N, d, Vs, dt, PASS_LOGPROBS), H.device, ws)
    _check(lib.llamarl_token_logprobs_partial(_ptr(H), _ptr(W_slice), _ptr(targets), _ptr(mask), N, d, Vs, int(v0),
                                              int(V_total), dt, _ptr(m), _ptr(s), _ptr(zt), _ptr(ws), ws.numel(),
                                              _stream(stream)))
    return m, s, zt


def merge_partials(m, s, zt, stream=None):
    """llamarl_merge_partials: m, s, zt [shards, N] -> (logp [N], lse [N])."""
    lib = load()
    for t, name in ((m, "m"), (s, "s"), (zt, "zt")):
        _need(t, torch.float32, name)
    if m.dim() != 2 or m.shape != s.shape or m.shape != zt.shape:
        raise LlamarlError(ERR_INVALID_ARG, "m, s, zt must be [shards, N]")
    shards, N = m.shape
    logp = torch.empty(N, dtype=torch.float32, device=m.device)
    lse = torch.empty(N, dtype=torch.float32, device=m.device)
    _check(lib.llamarl_merge_partials(_ptr(m), _ptr(s), _ptr(zt), shards, N, _ptr(logp), _ptr(lse), _stream(stream)))
    return logp, lse


def offpolicy_loss_bwd_slice(H, W_slice, targets, v0, lse, coef, grad_loss=1.0, dW_dtype=None, ws=None, stream=None):
    """llamarl_offpolicy_loss_bwd_slice: returns (dH_partial [N,d], dW_slice [V_slice,d])."""
    lib = load()
    dt = _dtype_code(H)
    _need(H, H.dtype, "H"); _need(W_slice, H.dtype, "W_slice"); _need(targets, torch.int32, "targets")
    _need(lse, torch.float32, "lse"); _need(coef, torch.float32, "coef")
    N, d = H.shape
    Vs = W_slice.shape[0]
    dW_dtype = dW_dtype or H.dtype
    dH = torch.empty(N, d, dtype=H.dtype, device=H.device)
    dW = torch.empty(Vs, d, dtype=dW_dtype, device=H.device)
    ws = _workspace(workspace_bytes(N, d, Vs, dt, PASS_LOSS_BWD), H.device, ws)
    _check(lib.llamarl_offpolicy_loss_bwd_slice(_ptr(H), _ptr(W_slice), _ptr(targets), _ptr(lse), _ptr(coef),
                                                float(grad_loss), N, d, Vs, int(v0), dt, _ptr(dH), _ptr(dW),
                                                _dtype_code(dW), 0, _ptr(ws), ws.numel(), _stream(stream)))
    return dH, dW
