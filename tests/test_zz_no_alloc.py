"""The entry point for callers that cannot allocate: fused_gemm_epilogue_static keeps the row
statistics of split rows (and K-slice partial products) in the library's static device array
instead of a caller workspace.  Its output must equal fused_gemm_epilogue's - same kernels, same
plan - on calls in a row that share the array, the second on a smaller problem."""
import numpy as np
import pytest
import torch

from paper_2512_23424_amd import binding as B
from paper_2512_23424_amd import inputs as I
from tests import _harness as H

DIST = {"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 0.1), "b": ("uniform", -0.5, 0.5),
        "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)}


def _wl(name, M, K, N, dt, act, norm):
    return I.Workload(name=name, M=M, K=K, N=N, in_dtype=dt, out_dtype=dt, act=act, norm=norm, alpha=0.5,
                      post_scale=1.5, eps=1e-5, dist=DIST)


def _both(w):
    """(existing entry point's out, aux), (static entry point's out, aux), oracle's (out, aux)"""
    t = I.generate(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    res = []
    for static in (False, True):
        out = torch.full((w.M, w.N), float("nan"), dtype=H.tdtype(w.out_dtype), device="cuda")
        aux = torch.full((w.M,), float("nan"), device="cuda") if w.norm == I.NORM_LOGSUMEXP else None
        p = B.make_params(d["X"], d["W"], out, alpha=w.alpha, post_scale=w.post_scale, eps=w.eps,
                          gamma=d["gamma"], beta=d["beta"], aux_out=aux)
        if static:
            B.fused_gemm_epilogue_static(d["X"], d["W"], d["b"], w.act, w.norm, p, out)
        else:
            n = B.fge_workspace_bytes(True, w.act, w.norm, p)
            assert n <= B.fge_static_scratch_bytes()
            ws = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
            p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel()
            B.fused_gemm_epilogue(d["X"], d["W"], d["b"], w.act, w.norm, p, out)
        torch.cuda.synchronize()
        res.append((H.to_host_f64(out), None if aux is None else H.to_host_f64(aux)))
    return res[0], res[1], H.oracle_chain(w, t)


@pytest.mark.gpu
def test_static_scratch_matches_the_workspace_entry_point():
    B.fge_static_scratch_init()
    cases = [
        _wl("static_coop", 4100, 136, 4000, I.BF16, I.ACT_SILU, I.NORM_RMSNORM),       # 256x256 tiles finish their rows themselves
        _wl("static_smaller", 300, 256, 1024, I.F32, I.ACT_GELU_TANH, I.NORM_LAYERNORM),  # smaller: statistics + second pass
        _wl("static_lse", 2050, 200, 2040, I.BF16, I.ACT_CLAMP, I.NORM_LOGSUMEXP),
        _wl("static_slices", 16, 4096, 1024, I.BF16, I.ACT_SILU, I.NORM_SOFTMAX),      # K slices: partial products in the array
        _wl("static_odd", 61, 37, 133, I.F32, I.ACT_RELU, I.NORM_SOFTMAX),             # element-granular kernels' fp32 intermediate
    ]
    for rep in range(2):                     # the second round meets the array as the first left it
        for w in cases:
            print(f"static scratch: {w.name} M={w.M} K={w.K} N={w.N} rep {rep}", flush=True)
            (eo, ea), (so, sa), (ref, raux) = _both(w)
            assert np.isfinite(so).all()
            assert np.array_equal(so, eo), f"{w.name}: static and workspace entry points differ"
            if ea is not None:
                assert np.array_equal(sa, ea)
            H.check(w, so, sa, ref, raux, f"static {w.name}")
