"""GPU parity for 8-bit E4M3 operands (fp32 accumulate, fp32 or bf16 output): the HIP path
through the C ABI against the float64 oracle on the same stored bits.  The operands are exact,
so the tolerance is that of the output type: 2e-2 with bf16 stores; with fp32 stores the same
gate is kept and the measured error (about 2e-4, the matrix instruction's own accumulation) is
printed.  Integer-valued problems must match bit for bit."""
import numpy as np
import pytest
import torch

from paper_2512_23424_amd import binding as B
from paper_2512_23424_amd import inputs as I
from tests import _harness as H

pytestmark = pytest.mark.gpu
F8 = I.F8E4M3
DIST = {"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0), "b": ("uniform", -0.5, 0.5),
        "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)}
ACTS = [I.ACT_NONE, I.ACT_RELU, I.ACT_GELU_TANH, I.ACT_GELU_ERF, I.ACT_SILU, I.ACT_CLAMP]
NORMS = [I.NORM_NONE, I.NORM_SOFTMAX, I.NORM_LAYERNORM, I.NORM_RMSNORM, I.NORM_LOGSUMEXP]


def _wl(M, K, N, act, norm, out_dtype, **kw):
    return I.Workload(name=f"f8a{act}n{norm}", M=M, K=K, N=N, in_dtype=F8, out_dtype=out_dtype, act=act,
                      norm=norm, alpha=1.0 / np.sqrt(K), post_scale=0.75, clamp_lo=-1.0, clamp_hi=2.0, eps=1e-5,
                      dist=DIST, **kw)


def _tile(w, t=None, flags=0):
    d = {k: H.to_device(v) for k, v in (t or I.generate(w)).items()}
    p = B.make_params(d["X"], d["W"], torch.empty(w.rows, w.N, dtype=H.tdtype(w.out_dtype), device="cuda"), flags=flags)
    return B.fge_tile_name(True, w.act, w.norm, p), B.fge_fault_word_offset(w.act, w.norm, p) is None and B.fge_fused_needs_finish(w.act, w.norm, p)


@pytest.mark.parametrize("shape", [(64, 64, 64), (96, 128, 160), (200, 80, 328), (300, 1024, 520)])
def test_exact_integer_gemm(shape):
    M, K, N = shape
    w = I.Workload(name="int8", M=M, K=K, N=N, in_dtype=F8, out_dtype=I.F32,
                   dist={"X": ("int", -2, 2), "W": ("int", -2, 2), "b": ("int", -3, 3)})
    t = I.generate(w)
    ref, _ = H.oracle_chain(w, t)
    for path in ("fused", "unfused"):
        got, _ = H.run_gpu(w, t, path)
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"{path} {shape}: {len(bad)} mismatches, first at {bad[:5].tolist()}"


def test_every_bit_pattern_is_read_as_e4m3():
    """All 254 finite patterns (largest 448, smallest 2^-9) as operands of a product with an
    identity-like W: the matrix instruction and the element-granular kernel must read each
    pattern as the value the format defines (the oracle decodes the same bytes by table)."""
    codes = np.array([c for c in range(256) if (c & 0x7F) != 0x7F], dtype=np.uint8)       # without the two NaNs
    K = 256
    X = np.zeros((len(codes), K), dtype=np.uint8)
    X[np.arange(len(codes)), np.arange(len(codes))] = codes                               # row i holds pattern i at k = i
    W = np.zeros((K, K), dtype=np.uint8)
    W[np.arange(K), np.arange(K)] = 0x38                                                  # 1.0 on the diagonal
    ref = I.as_f64(X) @ I.as_f64(W).T
    for Kc in (K, K - 3):                                                                 # fast path / element-granular
        Xd, Wd = H.to_device(np.ascontiguousarray(X[:, :Kc])), H.to_device(np.ascontiguousarray(W[:, :Kc]))
        out = torch.full((len(codes), K), float("nan"), device="cuda")
        p = B.make_params(Xd, Wd, out)
        B.fused_gemm_epilogue(Xd, Wd, None, I.ACT_NONE, I.NORM_NONE, p, out)
        torch.cuda.synchronize()
        r = I.as_f64(X[:, :Kc]) @ I.as_f64(W[:, :Kc]).T
        assert np.array_equal(out.double().cpu().numpy(), r), B.fge_tile_name(True, 0, 0, p)
    assert ref[0x7E, 0x7E] == 448.0 and ref[1, 1] == 2.0 ** -9


@pytest.mark.parametrize("out_dtype", [I.BF16, I.F32])
@pytest.mark.parametrize("norm", NORMS)
@pytest.mark.parametrize("N", [40, 328, 1032])          # whole-row 64, whole-row 512, split
def test_all_chains(out_dtype, norm, N):
    for act in ACTS:
        w = _wl(77, 144, N, act, norm, out_dtype)
        t = I.generate(w)
        ref, raux = H.oracle_chain(w, t)
        for path in ("fused", "unfused"):
            got, gaux = H.run_gpu(w, t, path)
            H.check(w, got, gaux, ref, raux, f"f8 {path} act{act} norm{norm}")


@pytest.mark.parametrize("norm", [I.NORM_SOFTMAX, I.NORM_LAYERNORM, I.NORM_RMSNORM, I.NORM_LOGSUMEXP])
@pytest.mark.parametrize("case", [(4100, 144, 4000, "256x256_w2x4"), (2050, 208, 2040, "128x128_w2x2")])
def test_split_rows_one_kernel_and_two_pass(norm, case):
    """Rows split over column tiles with a ragged last K tile (K < 128 bytes left) and a partial
    last round of the persistent grid: the one-kernel form and the two-pass form of the same
    call against the oracle."""
    M, K, N, tile = case
    w = _wl(M, K, N, I.ACT_SILU, norm, I.BF16)
    t = I.generate(w)
    assert _tile(w, t) == (tile, False)
    assert _tile(w, t, B.FLAG_TWO_PASS) == (tile, True)
    d = {k: H.to_device(v) for k, v in t.items()}
    ref, raux = H.oracle_chain(w, t)
    for flags in (0, B.FLAG_TWO_PASS):
        got, gaux = H.run_gpu(w, t, "fused", dev=d, flags=flags)
        H.check(w, got, gaux, ref, raux, f"f8 split flags={flags}")


@pytest.mark.parametrize("tile", ["64x64", "64x512", "128x128", "256x256", "128x256", "256x128"])
def test_every_tile_configuration(tile):
    from paper_2512_23424_amd import tune as T
    w = _wl(520, 400, 1040, I.ACT_GELU_ERF, I.NORM_SOFTMAX, I.F32)
    t = I.generate(w)
    flags = T.flag_tile(T.TILES[tile])
    assert _tile(w, t, flags)[0].startswith(tile)
    ref, raux = H.oracle_chain(w, t)
    got, gaux = H.run_gpu(w, t, "fused", flags=flags)
    H.check(w, got, gaux, ref, raux, f"f8 tile {tile}")


@pytest.mark.parametrize("shape", [(3, 5, 7), (33, 17, 65), (100, 101, 250), (70, 72, 1001)])
def test_any_shape_takes_the_element_granular_kernels(shape):
    M, K, N = shape
    for norm in NORMS:
        w = _wl(M, K, N, I.ACT_GELU_TANH, norm, I.F32)
        t = I.generate(w)
        assert _tile(w, t)[0] == "generic32x32_scalar"
        ref, raux = H.oracle_chain(w, t)
        for path in ("fused", "unfused"):
            got, gaux = H.run_gpu(w, t, path)
            H.check(w, got, gaux, ref, raux, f"f8 any-shape {path} {shape} norm{norm}")


def test_unsupported_pairs():
    X = torch.zeros(64, 64, device="cuda").to(torch.float8_e4m3fn)
    with pytest.raises(B.FgeError) as e:                   # fp8 operands go with fp32 or bf16 output
        p = B.make_params(X, X, torch.empty(64, 64, dtype=torch.float16, device="cuda"))
        B.fused_gemm_epilogue(X, X, None, 0, 0, p, torch.empty(64, 64, dtype=torch.float16, device="cuda"))
    assert e.value.status == 4


@pytest.mark.parametrize("norm", [I.NORM_NONE, I.NORM_RMSNORM, I.NORM_SOFTMAX])
@pytest.mark.parametrize("shape", [(300, 400, 520), (2050, 144, 2040), (70, 100, 90)])
def test_gated_form(norm, shape):
    """act(X.W1^T + b1) * (X.W2^T + b2) with 8-bit operands: the gated tile kernel (whole rows
    and split rows, ragged last K tile), the element-granular fallback for odd extents, and the
    unfused sequence, against the oracle."""
    from oracle import oracle as O
    M, K, N = shape
    w = _wl(M, K, N, I.ACT_SILU, norm, I.BF16)
    t = I.generate_gated(w)
    d = {k: H.to_device(v) for k, v in t.items()}
    f = {k: I.as_f64(v) for k, v in t.items()}
    ref, _ = O.gated_chain(f["X"], f["W"], f["W2"], f["b"], f["b2"], f["gamma"], f["beta"], alpha=w.alpha,
                           post_scale=w.post_scale, act=w.act, norm=norm, eps=w.eps)
    for fused in (True, False):
        out = torch.full((M, N), float("nan"), dtype=torch.bfloat16, device="cuda")
        p = B.make_params(d["X"], d["W"], out, alpha=w.alpha, post_scale=w.post_scale, eps=w.eps,
                          gamma=d["gamma"], beta=d["beta"])
        assert B.fge_gated_tile_name(w.act, norm, p) == ("gated256x128_w2x4" if K % 16 == 0 else "unfused_sequence")
        n = B.fge_gated_workspace_bytes(fused, w.act, norm, p)
        ws = torch.empty(max(n, 16), dtype=torch.uint8, device="cuda")
        p.workspace, p.workspace_bytes = ws.data_ptr(), n
        fn = B.fused_gated_gemm_epilogue if fused else B.unfused_gated_gemm_epilogue
        fn(d["X"], d["W"], d["W2"], d["b"], d["b2"], w.act, norm, p, out)
        torch.cuda.synchronize()
        got = H.to_host_f64(out)
        assert np.isfinite(got).all()
        err = H.C.max_rel_err(got, ref)
        print(f"f8 gated fused={fused} {shape} norm{norm}: {err:.3e}", flush=True)
        # the sequence rounds both products and the gated values to bf16 before the row op: the
        # exponentials of a softmax then see 2^-9 relative error of their arguments, hence the
        # wider gate for that combination only
        seq = not fused or K % 16 != 0
        assert err <= (8e-2 if seq and norm == I.NORM_SOFTMAX else 4e-2 if seq else 2e-2)


def test_headline_shape_sampled_rows():
    """cfg3's shape with E4M3 operands in the launch configuration the benchmark times; the
    oracle evaluates sampled complete rows."""
    w = I.EXTRA_WORKLOADS["cfg3_f8"]
    rng = np.random.default_rng(7)
    rows = np.unique(np.concatenate([[0, w.rows - 1], rng.integers(0, w.rows, 24)]))
    t = I.generate(w)
    assert _tile(w, t) == ("256x256_w2x4", False)
    d = {k: H.to_device(v) for k, v in t.items()}
    sub = dict(t, X=np.ascontiguousarray(t["X"][rows]))
    ref, raux = H.oracle_chain(w, sub)
    for path in ("fused", "unfused"):
        got, gaux = H.run_gpu(w, t, path, dev=d)
        assert np.isfinite(got).all()
        H.check(w, got[rows], None, ref, raux, f"f8 full {path}")
        g = t["gamma"].astype(np.float64)
        assert np.abs(((got / g) ** 2).mean(axis=1) - 1.0).max() < 2e-2
