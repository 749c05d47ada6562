"""The C-ABI library without a GPU: it loads, exports every symbol the header
declares, sizes workspaces, and rejects bad arguments before touching HIP."""
import ctypes
import os
import re

import pytest
import torch

from paper_2505_24034_amd import binding

# The rejection tests pass made-up addresses: they must never reach a kernel, so they only run where no GPU
# could be handed them.
no_gpu_only = pytest.mark.skipif(torch.cuda.device_count() > 0, reason="fake device pointers: CPU-only test")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def clib():
    return binding.load()


def test_library_exports_every_declared_symbol(clib):
    header = open(os.path.join(ROOT, "include", "llamarl.h")).read()
    declared = set(re.findall(r"\b(llamarl_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(clib, name) is not None
    assert b"gfx950" in clib.llamarl_version()


def test_workspace_sizes(clib):
    wb = binding.workspace_bytes
    assert wb(0, 8, 8, binding.BF16, binding.PASS_LOGPROBS) == 0
    assert wb(16, 8, 0, binding.BF16, binding.PASS_LOGPROBS) == 0
    assert wb(16, 8, 8, 7, binding.PASS_LOSS_BWD) == 0
    small = wb(256, 64, 256, binding.BF16, binding.PASS_LOGPROBS)
    assert small >= 3 * 256 * 4 and small % 256 == 0
    assert wb(16384, 4096, 128256, binding.BF16, binding.PASS_LOGPROBS) >= 2 * 501 * 16384 * 4
    b = wb(16384, 4096, 128256, binding.BF16, binding.PASS_LOSS_BWD)
    assert b >= 16384 * 128256 * 2 + 4096 * 16384 * 2          # dz^T and H^T panels at least
    assert wb(16384, 4096, 128256, binding.F32, binding.PASS_LOSS_BWD) >= 2 * 16384 * 128256 * 4
    assert wb(1000, 0, 0, 0, binding.PASS_LOSS_FWD) >= 8 * 1000


def _call_logprobs(clib, H=1 << 20, W=1 << 21, tg=1 << 22, N=16, d=8, V=8, dt=binding.BF16, logp=1 << 23,
                   lse=1 << 24, ws=1 << 25, ws_bytes=1 << 30):
    # fake non-null device addresses: validation must fail before anything is dereferenced or launched
    vp = ctypes.c_void_p
    return clib.llamarl_token_logprobs(vp(H), vp(W), vp(tg), None, N, d, V, dt, vp(logp), vp(lse), vp(ws), ws_bytes,
                                       None)


@no_gpu_only
def test_token_logprobs_rejects_bad_arguments(clib):
    assert _call_logprobs(clib, H=0) == binding.ERR_INVALID_ARG
    assert b"null" in clib.llamarl_last_error()
    assert _call_logprobs(clib, N=0) == binding.ERR_INVALID_ARG
    assert _call_logprobs(clib, V=-3) == binding.ERR_INVALID_ARG
    assert _call_logprobs(clib, dt=5) == binding.ERR_INVALID_ARG
    assert _call_logprobs(clib, d=12) == binding.ERR_UNSUPPORTED          # bf16 rows must be 16-byte multiples
    assert _call_logprobs(clib, H=(1 << 20) + 2) == binding.ERR_INVALID_ARG
    assert b"aligned" in clib.llamarl_last_error()
    assert _call_logprobs(clib, ws_bytes=8) == binding.ERR_WORKSPACE
    assert b"needed" in clib.llamarl_last_error()
    assert _call_logprobs(clib, ws=0) == binding.ERR_WORKSPACE
    assert _call_logprobs(clib, d=1 << 23, V=8) == binding.ERR_UNSUPPORTED  # a 256-row panel above 2 GiB


@no_gpu_only
def test_loss_fwd_rejects_bad_arguments(clib):
    vp = ctypes.c_void_p
    p = binding.LossParams(2.0, 0, 0.2, 0.2, 0)

    def call(pp=p, B=2, T=4, ws_bytes=1 << 20, logp=1 << 20, targets=None, V=0):
        return clib.llamarl_offpolicy_loss_fwd(vp(logp), vp(1 << 21), vp(1 << 22), 0, None, targets, V, B, T,
                                               ctypes.byref(pp), vp(1 << 23), vp(1 << 24), vp(1 << 25), vp(1 << 26),
                                               ws_bytes, None)

    assert call(logp=0) == binding.ERR_INVALID_ARG
    assert call(B=0) == binding.ERR_INVALID_ARG
    assert call(pp=binding.LossParams(-1.0, 0, 0.2, 0.2, 0)) == binding.ERR_INVALID_ARG
    assert call(pp=binding.LossParams(float("nan"), 0, 0.2, 0.2, 0)) == binding.ERR_INVALID_ARG
    assert call(pp=binding.LossParams(2.0, 3, 0.2, 0.2, 0)) == binding.ERR_INVALID_ARG
    assert call(pp=binding.LossParams(2.0, 0, 0.2, 0.2, 9)) == binding.ERR_INVALID_ARG
    assert call(pp=binding.LossParams(2.0, 1, 1.5, 0.2, 0)) == binding.ERR_INVALID_ARG
    assert call(ws_bytes=4) == binding.ERR_WORKSPACE
    assert call(targets=vp(1 << 27), V=0) == binding.ERR_INVALID_ARG


@no_gpu_only
def test_loss_bwd_rejects_bad_arguments(clib):
    vp = ctypes.c_void_p

    def call(N=16, d=8, V=8, dt=binding.BF16, dW_dt=binding.BF16, g=1.0, ws_bytes=1 << 30, dH=1 << 26):
        return clib.llamarl_offpolicy_loss_bwd(vp(1 << 20), vp(1 << 21), vp(1 << 22), vp(1 << 23), vp(1 << 24), g, N,
                                               d, V, dt, vp(dH), vp(1 << 27), dW_dt, 0, vp(1 << 28), ws_bytes, None)

    assert call(dH=0) == binding.ERR_INVALID_ARG
    assert call(d=4) == binding.ERR_UNSUPPORTED
    assert call(dt=binding.F32, dW_dt=binding.BF16) == binding.ERR_INVALID_ARG
    assert call(g=float("inf")) == binding.ERR_INVALID_ARG
    assert call(ws_bytes=100) == binding.ERR_WORKSPACE
    assert call(N=-1) == binding.ERR_INVALID_ARG


@no_gpu_only
def test_group_advantages_rejects_bad_arguments(clib):
    vp = ctypes.c_void_p
    assert clib.llamarl_group_advantages(None, 2, 2, 0, 0.0, vp(1 << 20), None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_group_advantages(vp(1 << 20), 0, 2, 0, 0.0, vp(1 << 21), None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_group_advantages(vp(1 << 20), 2, 2, 1, -1.0, vp(1 << 21), None) == binding.ERR_INVALID_ARG


@no_gpu_only
def test_kl_shaped_rewards_rejects_bad_arguments(clib):
    vp = ctypes.c_void_p
    a, b, c, o = vp(1 << 20), vp(1 << 21), vp(1 << 22), vp(1 << 23)
    assert clib.llamarl_kl_shaped_rewards(None, b, c, None, 2, 2, 0.1, o, None, None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_kl_shaped_rewards(a, b, c, None, 2, 2, 0.1, None, None, None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_kl_shaped_rewards(a, b, c, None, 0, 2, 0.1, o, None, None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_kl_shaped_rewards(a, b, c, None, 2, 2, float("nan"), o, None, None) == binding.ERR_INVALID_ARG


def test_binding_fails_loudly_without_library(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libllamarl.so")
    with pytest.raises(binding.LlamarlError):
        binding.load()


def test_bounded_backward_workspace_sizes(clib):
    bw = binding.bwd_workspace_bytes
    N, d, V = 16384, 4096, 128256
    whole = binding.workspace_bytes(N, d, V, binding.BF16, binding.PASS_LOSS_BWD)
    assert bw(N, d, V, binding.BF16, 0) == whole == bw(N, d, V, binding.BF16, N) == bw(N, d, V, binding.BF16, 10 ** 9)
    capped = bw(N, d, V, binding.BF16, 8704)
    assert V * 8704 * 2 <= capped <= whole - V * (N - 8704 - 128) * 2     # dz^T for 8704 rows instead of 16384
    assert bw(N, d, V, binding.BF16, 300) == bw(N, d, V, binding.BF16, 512)      # rounded up to whole 256-row tiles
    assert bw(N, d, V, binding.BF16, -1) == 0 and bw(0, d, V, binding.BF16, 256) == 0 and bw(N, d, V, 9, 256) == 0


@no_gpu_only
def test_new_entry_points_reject_bad_arguments(clib):
    vp = ctypes.c_void_p
    fake = lambda i: vp(1 << (20 + i))
    # vocabulary shard outside the head
    st = clib.llamarl_token_logprobs_partial(fake(0), fake(1), fake(2), None, 16, 8, 8, 4, 10, binding.BF16, fake(3),
                                             fake(4), fake(5), fake(6), 1 << 30, None)
    assert st == binding.ERR_INVALID_ARG and b"slice" in clib.llamarl_last_error()
    st = clib.llamarl_token_logprobs_partial(fake(0), fake(1), fake(2), None, 16, 8, 8, 0, 8, binding.BF16, fake(3),
                                             fake(4), None, fake(6), 1 << 30, None)
    assert st == binding.ERR_INVALID_ARG
    assert clib.llamarl_merge_partials(fake(0), fake(1), fake(2), 0, 16, fake(3), fake(4), None) == binding.ERR_INVALID_ARG
    assert clib.llamarl_merge_partials(fake(0), None, fake(2), 2, 16, fake(3), fake(4), None) == binding.ERR_INVALID_ARG
    st = clib.llamarl_offpolicy_loss_bwd_slice(fake(0), fake(1), fake(2), fake(3), fake(4), 1.0, 16, 8, 8, -1,
                                               binding.BF16, fake(5), fake(6), binding.BF16, 0, fake(7), 1 << 30, None)
    assert st == binding.ERR_INVALID_ARG
    st = clib.llamarl_offpolicy_loss_bwd_chunked(fake(0), fake(1), fake(2), fake(3), fake(4), 1.0, 16, 8, 8,
                                                 binding.BF16, fake(5), fake(6), binding.BF16, 0, -5, fake(7), 1 << 30,
                                                 None)
    assert st == binding.ERR_INVALID_ARG and b"max_rows_per_pass" in clib.llamarl_last_error()
    st = clib.llamarl_offpolicy_loss_bwd_chunked(fake(0), fake(1), fake(2), fake(3), fake(4), 1.0, 1024, 64, 512,
                                                 binding.BF16, fake(5), fake(6), binding.BF16, 0, 256, fake(7), 1000, None)
    assert st == binding.ERR_WORKSPACE
    # the static-scratch loss: size limits and misaligned inputs are refused before any HIP call
    p = binding.LossParams(2.0, 0, 0.2, 0.2, 0)
    st = clib.llamarl_offpolicy_loss_fwd_static(fake(0), fake(1), fake(2), 0, None, None, 0, 2, (1 << 21) + 1,
                                                ctypes.byref(p), fake(3), fake(4), fake(5), None)
    assert st == binding.ERR_UNSUPPORTED and b"static scratch" in clib.llamarl_last_error()
    st = clib.llamarl_offpolicy_loss_fwd_static(vp((1 << 20) + 4), fake(1), fake(2), 0, None, None, 0, 2, 8,
                                                ctypes.byref(p), fake(3), fake(4), fake(5), None)
    assert st == binding.ERR_INVALID_ARG and b"aligned" in clib.llamarl_last_error()
    flops = ctypes.c_double()
    assert clib.llamarl_mfma_ceiling(0, fake(0), ctypes.byref(flops), None) == binding.ERR_INVALID_ARG
    # the traffic variant: mode, iteration count and the size of the operand panels are checked on the host
    assert clib.llamarl_mfma_ceiling_traffic(4, 10, fake(1), 1 << 22, fake(0), ctypes.byref(flops), None) == \
        binding.ERR_INVALID_ARG
    assert clib.llamarl_mfma_ceiling_traffic(3, 0, fake(1), 1 << 22, fake(0), ctypes.byref(flops), None) == \
        binding.ERR_INVALID_ARG
    assert clib.llamarl_mfma_ceiling_traffic(3, 10, fake(1), (1 << 22) - 1, fake(0), ctypes.byref(flops), None) == \
        binding.ERR_INVALID_ARG and b"panels" in clib.llamarl_last_error()
