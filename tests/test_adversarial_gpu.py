"""Rows chosen to break a row operation that quietly assumes tame inputs (the paper's benchmark
section names hidden input assumptions as the typical failure of generated kernels): activations
of large magnitude with one dominant element, constant rows, maxima tied across column tiles, and
rows whose common offset dwarfs their spread.  Every case runs the fused path in both forms of
split rows and the unfused sequence, on shapes that span several column tiles, against the oracle."""
import numpy as np
import pytest
import torch

from paper_2512_23424_amd import binding as B
from paper_2512_23424_amd import inputs as I
from tests import _harness as H

pytestmark = pytest.mark.gpu

DIST = {"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 0.05), "b": ("uniform", -0.5, 0.5),
        "gamma": ("normal", 1.0, 0.1), "beta": ("normal", 0.0, 0.1)}
# (dtype, M, K, N): whole rows in one tile; rows split over column tiles, small (second pass) and
# large enough for the one-kernel form
SHAPES = [(I.F32, 130, 64, 328), (I.F32, 300, 64, 1024), (I.BF16, 2050, 72, 2040), (I.F32, 2060, 100, 2040)]


def _wl(dt, M, K, N, norm, act=I.ACT_NONE, **kw):
    return I.Workload(name=f"adv{norm}", M=M, K=K, N=N, in_dtype=dt, out_dtype=dt, act=act, norm=norm, eps=1e-5,
                      dist=DIST, **kw)


def _all_paths(w, t, label):
    """Fused (both forms of split rows) and unfused against the oracle, on the primary gate: the
    row-floored max rel err at the storage type's tolerance (the unfused sequence rounds Y and A
    to a 16-bit storage type on the way: 8e-2 there).  The paper's fraction-of-elements rule is
    not applied to these rows: it switches to ABSOLUTE error below the row's mean magnitude, which
    for rows spanning -80 .. 80 would ask for an absolute 2e-2 of 16-bit values of size 30."""
    ref, raux = H.oracle_chain(w, t)
    d = {k: H.to_device(v) for k, v in t.items()}
    for path, flags in (("fused", 0), ("fused", B.FLAG_TWO_PASS), ("unfused", 0)):
        got, gaux = H.run_gpu(w, t, path, dev=d, flags=flags)
        bound = 8e-2 if (path == "unfused" and w.out_dtype != I.F32) else H.TOL[w.in_dtype]
        assert np.isfinite(got).all(), (label, path, flags)
        e = H.C.max_rel_err(got, ref)
        print(f"{label} {w.name} {path} flags={flags}: max rel err {e:.3e} (bound {bound:.1e})", flush=True)
        assert e <= bound, (label, path, flags, e)
        if w.norm == I.NORM_LOGSUMEXP:
            assert np.isfinite(gaux).all()
            e2 = H.C.max_rel_err_vec(gaux, raux)
            assert e2 <= bound, (label, path, flags, "lse", e2)
    return ref, raux, None


@pytest.mark.parametrize("norm", [I.NORM_SOFTMAX, I.NORM_LOGSUMEXP])
@pytest.mark.parametrize("shape", SHAPES)
def test_large_magnitudes_and_one_dominant_element(norm, shape):
    """|a| up to 80: exp(a) itself would overflow fp32; one column holds nearly all the mass, the
    others underflow to zero relative to it.  The result must still be finite and correct."""
    w = _wl(*shape, norm)
    t = I.adversarial(w, "dominant")
    ref, raux, _ = _all_paths(w, t, "dominant")
    if norm == I.NORM_SOFTMAX:
        assert ref.max() > 0.99 and ref.min() < 1e-30          # the case is what it claims to be
    else:
        assert raux.max() > 75.0


@pytest.mark.parametrize("norm", [I.NORM_SOFTMAX, I.NORM_LAYERNORM, I.NORM_RMSNORM, I.NORM_LOGSUMEXP])
@pytest.mark.parametrize("shape", SHAPES)
def test_constant_rows(norm, shape):
    """Every element of a row equal (3.25): softmax is exactly uniform, RMSNorm leaves gamma,
    logsumexp is the value plus ln N, LayerNorm leaves beta.  The LayerNorm case has zero variance:
    what any fp32 implementation returns besides beta is the rounding noise of the row mean (a few
    2^-24 of 3.25) times rsqrt(eps) times gamma.  It runs once with eps = 1e-2, where that noise
    stays inside the gate, and once with eps = 1e-5 against that bound as an absolute error."""
    w = _wl(*shape, norm)
    t = I.adversarial(w, "constant")
    if norm == I.NORM_LAYERNORM:
        import dataclasses
        ref, _, _ = _all_paths(dataclasses.replace(w, eps=1e-2), t, "constant eps=1e-2")
        assert np.allclose(ref, I.as_f64(t["beta"])[None, :], atol=1e-9)
        ref, _ = H.oracle_chain(w, t)
        bound = 8 * 3.25 * 2.0 ** -24 / np.sqrt(w.eps) * 1.5 + (2.0 ** -8 if shape[0] != I.F32 else 0.0)
        for path, flags in (("fused", 0), ("fused", B.FLAG_TWO_PASS), ("unfused", 0)):
            got, _ = H.run_gpu(w, t, path, flags=flags)
            assert np.isfinite(got).all() and np.abs(got - ref).max() <= bound, (path, flags, np.abs(got - ref).max(), bound)
        return
    ref, raux, _ = _all_paths(w, t, "constant")
    if norm == I.NORM_SOFTMAX:
        assert np.allclose(ref, 1.0 / w.N, rtol=1e-12)


@pytest.mark.parametrize("norm", [I.NORM_SOFTMAX, I.NORM_LOGSUMEXP])
@pytest.mark.parametrize("shape", SHAPES)
def test_maxima_tied_across_column_tiles(norm, shape):
    """The row maximum recurs every 64 columns, so every wave strip and every column tile reports
    exactly the same maximum: the merge of the partial (maximum, sum) pairs must not depend on
    which of the equal maxima it meets first."""
    w = _wl(*shape, norm)
    t = I.adversarial(w, "tied")
    _all_paths(w, t, "tied")


@pytest.mark.parametrize("shape", [(130, 64, 328), (300, 256, 1024), (2060, 100, 2040)])
def test_layernorm_of_rows_whose_offset_dwarfs_their_spread(shape):
    """A common offset of about 1000 under a spread of order one, carried by the PRODUCT (so it is
    subject to the product's rounding): LayerNorm cancels the offset and amplifies every absolute
    error of it by offset / spread.  Bounds on the row-floored max rel err (mean |out| is about
    0.8, the spread 0.4 to 0.8):

      * fp32 matrix instruction (FGE_FLAG_IEEE_FP32): products exact, but every fp32 addition into
        a partial sum near 1000 rounds to 6e-5; over K/2 additions that is a few 1e-4 absolute at the
        worst element, a few 1e-3 after the amplification - no fp32 accumulation does better.
        Held to 5e-3.
      * split-bf16 product (the default for fp32 operands): the offset term itself carries up to
        3 * 2^-18 of its size, 1.1e-2 absolute, which the cancellation turns into an error of the
        order of a percent of the spread - far outside the 1e-4 of well-conditioned rows, as
        declared for the default (data like this wants the flag).  Held to 5e-2."""
    M, K, N = shape
    w = _wl(I.F32, M, K, N, I.NORM_LAYERNORM)
    t = I.adversarial(w, "offset")
    ref, _ = H.oracle_chain(w, t)
    pre = I.as_f64(t["X"]) @ I.as_f64(t["W"]).T
    assert 900.0 < pre.mean() < 1100.0 and pre.std(axis=1).max() < 3.0      # the case is what it claims to be
    d = {k: H.to_device(v) for k, v in t.items()}
    got_i, _ = H.run_gpu(w, t, "fused", dev=d, flags=B.FLAG_IEEE_FP32)
    got_s, _ = H.run_gpu(w, t, "fused", dev=d)
    e_i, e_s = H.C.max_rel_err(got_i, ref), H.C.max_rel_err(got_s, ref)
    print(f"offset rows {shape}: fp32 instruction {e_i:.3e}, split product {e_s:.3e}", flush=True)
    assert np.isfinite(got_i).all() and np.isfinite(got_s).all()
    assert e_i <= 5e-3
    assert e_s <= 5e-2


def test_rmsnorm_and_softmax_of_offset_rows_stay_inside_the_gate():
    """Without a cancellation the same rows are harmless: RMSNorm divides by the offset, and the
    default product stays inside the fp32 gate."""
    w = _wl(I.F32, 300, 256, 1024, I.NORM_RMSNORM)
    t = I.adversarial(w, "offset")
    _all_paths(w, t, "offset rmsnorm")
