"""GPU parity of the gated form, out = rowop(act(X.W1^T + b1) * (X.W2^T + b2)), against the
float64 oracle: the gated tile kernel (bf16 / fp16 operands), its cooperative and two-pass
forms, and the unfused sequence that also serves fp32 operands and odd extents."""
import numpy as np
import pytest
import torch

from paper_2512_23424_amd import binding as B
from paper_2512_23424_amd import inputs as I
from oracle import oracle as O
from tests import _harness as H

pytestmark = pytest.mark.gpu
NORMS = [I.NORM_NONE, I.NORM_SOFTMAX, I.NORM_LAYERNORM, I.NORM_RMSNORM, I.NORM_LOGSUMEXP]


def _workload(dt, M, K, N, act, norm, odt=None):
    return I.Workload(name=f"gated{act}{norm}", M=M, K=K, N=N, in_dtype=dt, out_dtype=dt if odt is None else odt,
                      act=act, norm=norm, alpha=0.5, post_scale=1.5, clamp_lo=-1.0, clamp_hi=2.0, eps=1e-5,
                      dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 0.1), "b": ("uniform", -0.5, 0.5),
                            "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)})


def _oracle(w, t):
    f = {k: I.as_f64(v) for k, v in t.items()}
    return O.gated_chain(f["X"], f["W"], f["W2"], f["b"], f["b2"], f["gamma"], f["beta"], alpha=w.alpha,
                         post_scale=w.post_scale, act=w.act, clamp_lo=w.clamp_lo, clamp_hi=w.clamp_hi,
                         norm=w.norm, eps=w.eps)


def _run(w, d, path, flags=0):
    out = torch.full((w.M, w.N), float("nan"), dtype=H.tdtype(w.out_dtype), device="cuda")
    aux = torch.full((w.M,), float("nan"), device="cuda") if w.norm == I.NORM_LOGSUMEXP else None
    p = B.make_params(d["X"], d["W"], out, alpha=w.alpha, post_scale=w.post_scale, clamp_lo=w.clamp_lo,
                      clamp_hi=w.clamp_hi, eps=w.eps, gamma=d["gamma"], beta=d["beta"], aux_out=aux, flags=flags)
    n = B.fge_gated_workspace_bytes(path == "fused", w.act, w.norm, p)
    ws = torch.full((max(n, 16) // 4 + 1,), float("nan"), device="cuda")
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel() * 4
    fn = B.fused_gated_gemm_epilogue if path == "fused" else B.unfused_gated_gemm_epilogue
    fn(d["X"], d["W"], d["W2"], d["b"], d["b2"], w.act, w.norm, p, out)
    torch.cuda.synchronize()
    return H.to_host_f64(out), None if aux is None else H.to_host_f64(aux), B.fge_gated_tile_name(w.act, w.norm, p)


def _case(w, paths=("fused", "unfused"), flags=(0,), expect=None):
    t = I.generate_gated(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    ref, raux = _oracle(w, t)
    for path in paths:
        for fl in flags:
            got, gaux, name = _run(w, d, path, fl)
            if expect is not None:
                assert name == expect, name
            if name == "unfused_sequence" or path == "unfused":
                # the sequence keeps both products and the gated value in the output type: with
                # 16-bit storage the exponentials of a softmax see 2^-9 (2^-11) relative error of
                # values of magnitude up to ~8, hence the wider gate for that combination only
                wide = w.out_dtype != I.F32 and w.norm in (I.NORM_SOFTMAX, I.NORM_LOGSUMEXP)
                err = H.C.max_rel_err(got, ref)
                print(f"gated sequence {path} {name} {w.name}: {err:.3e}", flush=True)
                assert np.isfinite(got).all() and err <= (8e-2 if wide else H.TOL[w.in_dtype])
            else:
                H.check(w, got, gaux, ref, raux, f"gated {path} flags={fl} {name}")


@pytest.mark.parametrize("dt", [I.BF16, I.F16])
@pytest.mark.parametrize("norm", NORMS)
def test_gated_tile_kernel_all_row_ops(dt, norm):
    """Ragged M / N / K on the gated tile kernel, SiLU-and-Mul and GELU-and-Mul."""
    for act in (I.ACT_SILU, I.ACT_GELU_ERF):
        _case(_workload(dt, 300, 136, 1032, act, norm), expect="gated256x128_w2x4")
    _case(_workload(dt, 77, 72, 40, I.ACT_RELU, norm), expect="gated256x128_w2x4")


@pytest.mark.parametrize("norm", [I.NORM_SOFTMAX, I.NORM_LAYERNORM, I.NORM_RMSNORM, I.NORM_LOGSUMEXP])
def test_gated_split_rows_both_forms(norm):
    """Large enough for the one-kernel form (32 row blocks x 17 column tiles), with a partial
    last round; the two-pass form of the same call as well."""
    _case(_workload(I.BF16, 8100, 72, 2104, I.ACT_SILU, norm), paths=("fused",),
          flags=(0, B.FLAG_TWO_PASS), expect="gated256x128_w2x4")


def test_gated_fp32_and_odd_extents_take_the_sequence():
    for (dt, M, K, N) in [(I.F32, 130, 72, 264), (I.F32, 33, 17, 65), (I.BF16, 100, 101, 250), (I.F16, 3, 5, 7)]:
        for norm in (I.NORM_NONE, I.NORM_RMSNORM, I.NORM_SOFTMAX):
            _case(_workload(dt, M, K, N, I.ACT_SILU, norm), expect="unfused_sequence")


def test_gated_exact_integers_and_fp32_result():
    """Small integers: both products are exact, so with no activation the gate's product must
    match the oracle bit for bit (fp32 result of bf16 operands) - on the fused kernel and on the
    unfused sequence, whose intermediates are fp32 here and therefore exact as well."""
    w = I.Workload(name="gint", M=260, K=72, N=136, in_dtype=I.BF16, out_dtype=I.F32,
                   dist={"X": ("int", -2, 2), "W": ("int", -2, 2), "b": ("int", -3, 3)})
    t = I.generate_gated(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    ref, _ = _oracle(w, t)
    for path in ("fused", "unfused"):
        got, _, _ = _run(w, d, path)
        assert np.array_equal(got, ref), path


def test_gated_fp32_keeps_the_fp32_gate():
    """The gate multiplies two products and their errors: with fp32 operands both products run on
    the fp32 matrix instruction, which keeps the chain inside 1e-4 (two split-bf16 products left
    it on this shape)."""
    w = I.Workload(name="g32", M=583, K=84, N=316, in_dtype=I.F32, out_dtype=I.F32, act=I.ACT_GELU_ERF,
                   norm=I.NORM_LAYERNORM, alpha=0.9, post_scale=1.3, eps=1e-5,
                   dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 0.6 / 84 ** 0.5), "b": ("uniform", -0.5, 0.5),
                         "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)})
    t = I.generate_gated(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    ref, _ = _oracle(w, t)
    for path in ("fused", "unfused"):
        got, _, _ = _run(w, d, path)
        err = H.C.max_rel_err(got, ref)
        print(f"gated fp32 {path}: {err:.3e}", flush=True)
        assert err <= 2e-5


@pytest.mark.parametrize("dt", [I.BF16, I.F16, I.F8E4M3])
@pytest.mark.parametrize("norm", NORMS)
def test_gated_small_problems_with_a_long_k(dt, norm):
    """A handful of 256-row tiles and a long K: both products run as fp32 partial products (K cut
    into slices where that pays), then one kernel adds, activates and gates in fp32 and the row
    op follows - the same gates as the gated tile kernel, which the same call with too small a
    workspace still takes."""
    for (M, K, N, act) in [(24, 4096, 1032, I.ACT_SILU), (300, 1152, 520, I.ACT_GELU_ERF)]:
        if dt == I.F8E4M3:
            w = I.Workload(name=f"gsmall{norm}", M=M, K=K, N=N, in_dtype=dt, out_dtype=I.BF16, act=act, norm=norm,
                           alpha=1.0 / K ** 0.5, post_scale=1.5, clamp_lo=-1.0, clamp_hi=2.0, eps=1e-5,
                           dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0), "b": ("uniform", -0.5, 0.5),
                                 "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)})
        else:
            w = _workload(dt, M, K, N, act, norm)
            w = I.scaled(w, dist=dict(w.dist, W=("normal", 0.0, 1.0 / K ** 0.5)))
        _case(w, paths=("fused",), expect="partial_products_then_gate")
    # without the room for the partial products the gated tile kernel runs the same call
    t = I.generate_gated(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    out = torch.full((w.M, w.N), float("nan"), dtype=H.tdtype(w.out_dtype), device="cuda")
    aux = torch.full((w.M,), float("nan"), device="cuda") if norm == I.NORM_LOGSUMEXP else None
    p = B.make_params(d["X"], d["W"], out, alpha=w.alpha, post_scale=w.post_scale, clamp_lo=w.clamp_lo,
                      clamp_hi=w.clamp_hi, eps=w.eps, gamma=d["gamma"], beta=d["beta"], aux_out=aux)
    need = B.fge_gated_workspace_bytes(True, w.act, norm, p)
    assert need >= 2 * w.M * w.N * 4
    ws = torch.empty(1 << 16, dtype=torch.uint8, device="cuda")           # enough for the tile kernel's row statistics
    p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel()
    B.fused_gated_gemm_epilogue(d["X"], d["W"], d["W2"], d["b"], d["b2"], w.act, norm, p, out)
    torch.cuda.synchronize()
    ref, raux = _oracle(w, t)
    H.check(w, H.to_host_f64(out), None if aux is None else H.to_host_f64(aux), ref, raux, "gated tile kernel, small workspace")
