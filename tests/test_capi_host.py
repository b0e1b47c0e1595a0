"""Host-only checks of the C-ABI boundary: the library loads, exports every
symbol the header declares, sizes its workspace sanely, and rejects bad
arguments before touching any device (so these run without a GPU)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

api = pytest.importorskip("paper_2509_14279_amd.api", reason="libfdl.so not built")

P = 0x10000  # a non-null, 256-byte aligned fake address; never dereferenced by a rejected call


def test_header_symbols_are_exported():
    text = open(os.path.join(ROOT, "include", "fdl.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(fdl_[a-z_]+)\s*\(", text))
    assert declared == set(api.EXPORTS)
    for name in declared:
        assert hasattr(api._lib, name), name


def test_nothing_but_the_declared_entry_points_is_exported():
    """The library is built with hidden visibility: its dynamic symbol table defines the C entry points and nothing
    of its internals (the compiler's own per-translation-unit markers aside)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", api.LIB_PATH], capture_output=True, text=True, check=True).stdout
    names = {ln.split()[-1] for ln in out.splitlines() if ln.strip()}
    names = {n for n in names if not n.startswith("__hip_cuid_")}
    assert names == set(api.EXPORTS), names ^ set(api.EXPORTS)


def test_status_strings():
    names = ["FDL_OK", "FDL_ERR_NULL", "FDL_ERR_SHAPE", "FDL_ERR_DTYPE", "FDL_ERR_EPS", "FDL_ERR_WORKSPACE",
             "FDL_ERR_ALIGN", "FDL_ERR_LAUNCH"]
    for code, n in enumerate(names):
        assert api.fdl_status_string(code).startswith(n)
    assert "unknown" in api.fdl_status_string(99)


def test_workspace_bytes():
    assert api.fdl_workspace_bytes(7, 8, 8, 8) == 0            # bad dtype
    assert api.fdl_workspace_bytes("f32", 8, 0, 8) == 0        # K < 1
    assert api.fdl_workspace_bytes("f32", 8, 8, 0) == 0
    assert api.fdl_workspace_bytes("f32", -1, 8, 8) == 0
    assert api.fdl_workspace_bytes("bf16", 1 << 25, 8, 8) == 0  # beyond the supported range
    small = api.fdl_workspace_bytes("bf16", 256, 256, 256)
    big = api.fdl_workspace_bytes("bf16", 65536, 2048, 8192)
    assert 0 < small < big
    assert big >= 65536 * 8192 * 2                              # holds dZ
    assert big < 3 * 65536 * 8192 * 2                           # and not wildly more
    assert api.fdl_workspace_bytes("f32", 3001, 771, 1537) >= 3001 * 1537 * 4
    assert api.fdl_workspace_bytes("f32", 0, 4, 4) > 0          # empty batch is a valid call


def _fwd(dt="f32", M=4, K=4, N=4, eps=1e-5, ws=P, ws_bytes=1 << 30, **over):
    a = dict(X=P, W=P, b=P, gamma=P, beta=P, Y=P, Zsave=P, mean=P, rstd=P)
    a.update(over)
    return api.fdl_forward_raw(dt, M, K, N, a["X"], a["W"], a["b"], a["gamma"], a["beta"], eps, a["Y"], a["Zsave"],
                               a["mean"], a["rstd"], ws, ws_bytes, None)


def _bwd(dt="f32", M=4, K=4, N=4, ws=P, ws_bytes=1 << 30, **over):
    a = dict(dY=P, X=P, W=P, gamma=P, Zsave=P, mean=P, rstd=P, dX=P, dW=P, db=P, dgamma=P, dbeta=P)
    a.update(over)
    return api.fdl_backward_raw(dt, M, K, N, a["dY"], a["X"], a["W"], a["gamma"], a["Zsave"], a["mean"], a["rstd"],
                                a["dX"], a["dW"], a["db"], a["dgamma"], a["dbeta"], ws, ws_bytes, None)


def test_forward_rejects_bad_arguments_before_any_launch():
    for name in ("X", "W", "b", "gamma", "beta", "Y", "Zsave", "mean", "rstd"):
        assert _fwd(**{name: 0}) == api.FDL_ERR_NULL, name
    assert _fwd(dt=5) == api.FDL_ERR_DTYPE
    for bad in (dict(M=-1), dict(K=0), dict(N=0), dict(M=(1 << 24) + 1)):
        assert _fwd(**bad) == api.FDL_ERR_SHAPE, bad
    for eps in (-1e-5, float("nan"), float("inf")):
        assert _fwd(eps=eps) == api.FDL_ERR_EPS
    assert _fwd(ws=0) == api.FDL_ERR_WORKSPACE
    assert _fwd(ws_bytes=api.fdl_workspace_bytes("f32", 4, 4, 4) - 1) == api.FDL_ERR_WORKSPACE
    assert _fwd(ws=P + 16) == api.FDL_ERR_ALIGN
    assert _fwd(X=P + 4) == api.FDL_ERR_ALIGN
    assert _fwd(Y=P + 8) == api.FDL_ERR_ALIGN
    assert _fwd(b=P + 2) == api.FDL_ERR_ALIGN
    # an empty batch is accepted and launches nothing
    assert _fwd(M=0) == api.FDL_OK


def _fwd_static(dt="f32", M=4, K=4, N=4, eps=1e-5, **over):
    a = dict(X=P, W=P, b=P, gamma=P, beta=P, Y=P, Zsave=P, mean=P, rstd=P)
    a.update(over)
    return api.fdl_forward_static_raw(dt, M, K, N, a["X"], a["W"], a["b"], a["gamma"], a["beta"], eps, a["Y"],
                                      a["Zsave"], a["mean"], a["rstd"], None)


def test_forward_static_rejects_bad_arguments_and_oversized_problems_before_any_device_call():
    for name in ("X", "W", "b", "gamma", "beta", "Y", "Zsave", "mean", "rstd"):
        assert _fwd_static(**{name: 0}) == api.FDL_ERR_NULL, name
    assert _fwd_static(dt=5) == api.FDL_ERR_DTYPE
    assert _fwd_static(K=0) == api.FDL_ERR_SHAPE
    assert _fwd_static(eps=float("nan")) == api.FDL_ERR_EPS
    assert _fwd_static(X=P + 4) == api.FDL_ERR_ALIGN
    assert _fwd_static(M=0) == api.FDL_OK
    # partial row statistics of 8 bytes per (row, 64-column tile): 65536 rows x 128 tiles = 64 MiB > the 16 MiB array
    assert _fwd_static(dt="f32", M=65536, K=64, N=8192) == api.FDL_ERR_WORKSPACE
    # the headline shape normalises without partials and needs no scratch at all: accepted up to the launch, which
    # this host-only test must not reach, so only its size is checked here
    assert api.FDL_STATIC_SCRATCH_BYTES == 16 * 1024 * 1024


def test_backward_rejects_bad_arguments_before_any_launch():
    for name in ("dY", "X", "W", "gamma", "Zsave", "mean", "rstd", "dX", "dW", "db", "dgamma", "dbeta"):
        assert _bwd(**{name: 0}) == api.FDL_ERR_NULL, name
    assert _bwd(dt=-1) == api.FDL_ERR_DTYPE
    for bad in (dict(M=-1), dict(K=0), dict(N=0), dict(N=(1 << 24) + 1)):
        assert _bwd(**bad) == api.FDL_ERR_SHAPE, bad
    assert _bwd(ws=0) == api.FDL_ERR_WORKSPACE
    assert _bwd(ws_bytes=16) == api.FDL_ERR_WORKSPACE
    assert _bwd(ws=P + 128) == api.FDL_ERR_ALIGN
    assert _bwd(dW=P + 4) == api.FDL_ERR_ALIGN
    assert _bwd(dbeta=P + 1) == api.FDL_ERR_ALIGN


def test_one_hip_runtime_in_the_process():
    """torch ships its own HIP runtime; the library must bind to that copy, whatever the import order of the
    test modules, or launches on torch buffers fail with device errors."""
    loaded = {ln.split()[-1] for ln in open("/proc/self/maps") if "libamdhip64" in ln}
    assert len(loaded) == 1, loaded
    import torch
    assert os.path.dirname(torch.__file__) in next(iter(loaded))


def test_sibling_entry_points_reject_bad_arguments_before_any_launch():
    big = 1 << 30
    # forward for inference
    # row statistics and (from 16384 rows on) the transposed weights: nothing of size M x N
    assert api.fdl_forward_inference_workspace_bytes("bf16", 65536, 2048, 8192) < (1 << 22) + 2 * 2048 * 8192
    assert api.fdl_forward_inference_workspace_bytes("bf16", 8192, 2048, 8192) < 1 << 22
    assert api.fdl_forward_inference_workspace_bytes(9, 8, 8, 8) == 0
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, 0, P, P, P, P, 1e-5, P, P, big, None) == api.FDL_ERR_NULL
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, P, P, P, P, P, 1e-5, 0, P, big, None) == api.FDL_ERR_NULL
    assert api.fdl_forward_inference_raw(3, 4, 4, 4, P, P, P, P, P, 1e-5, P, P, big, None) == api.FDL_ERR_DTYPE
    assert api.fdl_forward_inference_raw("f32", 4, 0, 4, P, P, P, P, P, 1e-5, P, P, big, None) == api.FDL_ERR_SHAPE
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, P, P, P, P, P, -1.0, P, P, big, None) == api.FDL_ERR_EPS
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, P, P, P, P, P, 1e-5, P, P, 8, None) == api.FDL_ERR_WORKSPACE
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, P, P, P, P, P, 1e-5, P, P + 16, big, None) == api.FDL_ERR_ALIGN
    assert api.fdl_forward_inference_raw("f32", 4, 4, 4, P + 4, P, P, P, P, 1e-5, P, P, big, None) == api.FDL_ERR_ALIGN
    assert api.fdl_forward_inference_raw("f32", 0, 4, 4, P, P, P, P, P, 1e-5, P, P, big, None) == api.FDL_OK
    # Linear + ReLU
    assert api.fdl_linear_relu_workspace_bytes("bf16", 4096, 512, 1024) >= 4096 * 1024 * 2
    assert api.fdl_linear_relu_workspace_bytes("f32", 8, 0, 8) == 0
    assert api.fdl_linear_relu_forward_raw("f32", 4, 4, 4, P, 0, P, P, P, big, None) == api.FDL_ERR_NULL
    assert api.fdl_linear_relu_forward_raw(7, 4, 4, 4, P, P, P, P, P, big, None) == api.FDL_ERR_DTYPE
    assert api.fdl_linear_relu_forward_raw("f32", -1, 4, 4, P, P, P, P, P, big, None) == api.FDL_ERR_SHAPE
    assert api.fdl_linear_relu_forward_raw("f32", 4, 4, 4, P, P, P, P, 0, big, None) == api.FDL_ERR_WORKSPACE
    assert api.fdl_linear_relu_forward_raw("f32", 4, 4, 4, P, P, P, P + 2, P, big, None) == api.FDL_ERR_ALIGN
    assert api.fdl_linear_relu_backward_raw("f32", 4, 4, 4, P, P, P, P, P, P, 0, P, big, None) == api.FDL_ERR_NULL
    assert api.fdl_linear_relu_backward_raw("f32", 4, 4, 4, P, P, P, P, P, P, P, P, 8, None) == api.FDL_ERR_WORKSPACE
    assert api.fdl_linear_relu_backward_raw("f32", 4, 4, 0, P, P, P, P, P, P, P, P, big, None) == api.FDL_ERR_SHAPE
    assert api.fdl_linear_relu_backward_raw("f32", 4, 4, 4, P, P, P, P, P + 8, P, P, P, big, None) == api.FDL_ERR_ALIGN
    # norms
    assert api.fdl_layernorm_forward_raw("f32", 4, 4, P, P, P, 1e-5, P, P, 0, None) == api.FDL_ERR_NULL
    assert api.fdl_layernorm_forward_raw("f32", 4, 0, P, P, P, 1e-5, P, P, P, None) == api.FDL_ERR_SHAPE
    assert api.fdl_layernorm_forward_raw("f32", 4, 4, P, P, P, float("nan"), P, P, P, None) == api.FDL_ERR_EPS
    assert api.fdl_layernorm_forward_raw(2, 4, 4, P, P, P, 1e-5, P, P, P, None) == api.FDL_ERR_DTYPE
    assert api.fdl_layernorm_forward_raw("f32", 4, 4, P, P + 4, P, 1e-5, P, P, P, None) == api.FDL_ERR_ALIGN
    assert api.fdl_rmsnorm_forward_raw("f32", 4, 4, P, 0, 1e-5, P, None) == api.FDL_ERR_NULL
    assert api.fdl_rmsnorm_forward_raw("f32", 1 << 25, 4, P, P, 1e-5, P, None) == api.FDL_ERR_SHAPE
    assert api.fdl_rmsnorm_forward_raw("f32", 4, 4, P, P, -1.0, P, None) == api.FDL_ERR_EPS
    assert api.fdl_rmsnorm_forward_raw("f32", 0, 4, P, P, 1e-5, P, None) == api.FDL_OK
    # Llama feed-forward
    assert api.fdl_llama_ffn_workspace_bytes("bf16", 1024, 512, 2048) >= 1024 * 2048 * 2          # fused gate: one M x H buffer
    assert api.fdl_llama_ffn_workspace_bytes("f32", 1024, 512, 2048) >= 2 * 1024 * 2048 * 4
    assert api.fdl_llama_ffn_workspace_bytes("bf16", 1024, 0, 2048) == 0
    assert api.fdl_llama_ffn_forward_raw("f32", 4, 4, 4, P, P, 0, P, P, P, big, None) == api.FDL_ERR_NULL
    assert api.fdl_llama_ffn_forward_raw("f32", 4, 4, 0, P, P, P, P, P, P, big, None) == api.FDL_ERR_SHAPE
    assert api.fdl_llama_ffn_forward_raw("f32", 4, 4, 4, P, P, P, P, P, P, 8, None) == api.FDL_ERR_WORKSPACE
    assert api.fdl_llama_ffn_forward_raw("f32", 4, 4, 4, P, P, P, P + 4, P, P, big, None) == api.FDL_ERR_ALIGN
    assert api.fdl_llama_ffn_forward_raw(-1, 4, 4, 4, P, P, P, P, P, P, big, None) == api.FDL_ERR_DTYPE
