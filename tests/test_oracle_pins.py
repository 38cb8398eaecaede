"""Pins of the float64 oracle against things other than itself: hand-derived closed forms
(tests/golden/closed_forms.json), brute force in another loop order, invariants, and library
routines (numpy matmul, scipy.special, torch float64 CPU ops).  The paper prints no worked
numeric example for any operator, so no printed value exists to compare with."""
import json
import math
import os

import numpy as np
import pytest
import scipy.special as sp
import torch

from oracle import compare as C
from oracle import oracle as O
from paper_2512_23424_amd import inputs as I

GOLD = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "closed_forms.json")))


def _ev(v):
    if isinstance(v, str):
        return eval(v, {"log": math.log, "sqrt": math.sqrt, "exp": math.exp})
    return float(v)


def _row(vs):
    return np.array([[_ev(v) for v in vs]], dtype=np.float64)


RNG = np.random.default_rng(1234)

# ----------------------------------------------------------------- step 1: contraction

def test_gemm_bruteforce_other_loop_order_exact_integers():
    for (M, N, K) in [(1, 1, 1), (3, 5, 2), (8, 3, 7), (2, 8, 8), (5, 4, 1)]:
        X = RNG.integers(-2, 3, size=(M, K))
        W = RNG.integers(-2, 3, size=(N, K))
        ref = [[0] * N for _ in range(M)]
        for j in range(N):               # j-k-i order, python ints: exact
            for k in range(K):
                for i in range(M):
                    ref[i][j] += int(X[i, k]) * int(W[j, k])
        G = O.gemm(X.astype(np.float64), W.astype(np.float64))
        assert G.shape == (M, N)
        assert np.array_equal(G, np.array(ref, dtype=np.float64))


def test_gemm_structural_cases():
    K = 6
    X = RNG.standard_normal((4, K))
    assert np.array_equal(O.gemm(X, np.eye(K)), X)                    # W = I  ->  G = X
    W = RNG.standard_normal((5, K))
    E = np.zeros((4, K)); E[2, 3] = 1.0                               # X = e_p e_q^T
    G = O.gemm(E, W)
    assert np.array_equal(G[2], W[:, 3]) and not G[[0, 1, 3]].any()
    x = RNG.standard_normal((4, 1)); w = RNG.standard_normal((3, 1))  # K = 1: outer product
    assert np.array_equal(O.gemm(x, w), x * w.T)
    assert not O.gemm(np.zeros((4, K)), W).any()


def test_gemm_matches_numpy_nonsquare():
    X = RNG.standard_normal((37, 129)); W = RNG.standard_normal((53, 129))
    np.testing.assert_allclose(O.gemm(X, W), X @ W.T, rtol=0, atol=1e-12)
    # a transposed-operand mistake would change the shape or the values
    assert O.gemm(X, W).shape == (37, 53)


# ----------------------------------------------------------------- step 2: scale and bias

def test_scale_bias_order():
    b = RNG.standard_normal(5)
    Z = np.zeros((3, 5))
    for alpha in (0.25, 7.0):
        Y = O.scale_bias(Z, b, alpha, 2.0)                             # W = 0: Y = post_scale*b
        assert np.array_equal(Y, np.broadcast_to(2.0 * b, (3, 5)))
    G = RNG.standard_normal((3, 5))
    assert np.array_equal(O.scale_bias(G, None, 0.5, 4.0), 4.0 * (0.5 * G))
    assert np.array_equal(O.scale_bias(G, b, 1.0, 1.0), G + b)


# ----------------------------------------------------------------- step 3: activations

def test_relu_clamp_exact():
    y = np.array([[-3.0, -0.0, 0.0, 1e-300, 2.5, 7.0, -7.0, 5.0, -5.0]])
    r = O.act(y, I.ACT_RELU)
    assert np.array_equal(r, np.maximum(y, 0.0)) and (r >= 0).all()
    c = O.act(y, I.ACT_CLAMP, -5.0, 5.0)
    assert np.array_equal(c, np.clip(y, -5.0, 5.0))
    assert c.max() == 5.0 and c.min() == -5.0
    assert np.array_equal(O.act(y, I.ACT_NONE), y)


@pytest.mark.parametrize("kind", [I.ACT_GELU_TANH, I.ACT_GELU_ERF, I.ACT_SILU])
def test_smooth_activation_identities(kind):
    y = np.linspace(-9, 9, 721)[None, :]
    f = O.act(y, kind)
    fm = O.act(-y, kind)
    np.testing.assert_allclose(f - fm, y, rtol=0, atol=1e-14)         # f(y) - f(-y) = y
    assert O.act(np.zeros((1, 1)), kind)[0, 0] == 0.0
    big = O.act(np.array([[40.0, -40.0]]), kind)
    assert abs(big[0, 0] - 40.0) < 1e-12 and abs(big[0, 1]) < 1e-12 and big[0, 1] <= 0.0


def test_gelu_silu_closed_forms_and_libraries():
    g = GOLD["silu_ln3"]
    y = _row(g["y"])
    np.testing.assert_allclose(O.act(y, I.ACT_SILU)[0] / math.log(3), g["out_over_ln3"], rtol=1e-15)
    g = GOLD["gelu_erf_phi"]
    np.testing.assert_allclose(O.act(_row(g["y"]), I.ACT_GELU_ERF)[0], g["out"], rtol=1e-14)
    y = np.linspace(-7, 7, 1401)[None, :]
    erf_form = O.act(y, I.ACT_GELU_ERF)
    np.testing.assert_allclose(erf_form, 0.5 * y * sp.erfc(-y / math.sqrt(2.0)), rtol=0, atol=1e-15)
    t = torch.from_numpy(y)
    F = torch.nn.functional
    np.testing.assert_allclose(erf_form, F.gelu(t).numpy(), rtol=0, atol=1e-14)
    tanh_form = O.act(y, I.ACT_GELU_TANH)
    np.testing.assert_allclose(tanh_form, F.gelu(t, approximate="tanh").numpy(), rtol=0, atol=1e-14)
    np.testing.assert_allclose(O.act(y, I.ACT_SILU), F.silu(t).numpy(), rtol=0, atol=1e-14)
    # the two GELU forms are close but not equal
    d = np.abs(tanh_form - erf_form).max()
    assert 1e-5 < d < 1e-3


# ----------------------------------------------------------------- step 4: row operations

def test_softmax_and_logsumexp_closed_form():
    g = GOLD["softmax_logs"]
    a = _row(g["row"])
    p, _ = O.rowop(a, I.NORM_SOFTMAX)
    np.testing.assert_allclose(p[0], g["softmax"], rtol=1e-15)
    z, lse = O.rowop(a, I.NORM_LOGSUMEXP)
    assert np.array_equal(z, a)                                       # Z is passed through
    assert abs(lse[0] - _ev(g["logsumexp"])) < 1e-15


def test_softmax_invariants():
    A = RNG.standard_normal((16, 100)) * 4
    P, _ = O.rowop(A, I.NORM_SOFTMAX)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, rtol=0, atol=1e-12)
    assert (P > 0).all() and (P <= 1).all()
    P2, _ = O.rowop(A + 123.456, I.NORM_SOFTMAX)                      # shift invariance
    np.testing.assert_allclose(P2, P, rtol=1e-11)
    Pc, _ = O.rowop(np.full((2, 64), 3.25), I.NORM_SOFTMAX)
    assert np.array_equal(Pc, np.full((2, 64), 1.0 / 64))
    assert np.array_equal(np.argsort(A, axis=1, kind="stable"), np.argsort(P, axis=1, kind="stable"))
    np.testing.assert_allclose(P, sp.softmax(A, axis=1), rtol=1e-13)
    # rows are independent and the reduction runs along N (not M)
    P3, _ = O.rowop(A[:3], I.NORM_SOFTMAX)
    assert np.array_equal(P3, P[:3])
    big, _ = O.rowop(np.array([[1000.0, 1000.0, -1000.0]]), I.NORM_SOFTMAX)   # no overflow
    np.testing.assert_allclose(big[0], [0.5, 0.5, 0.0], atol=1e-300)


def test_logsumexp_bounds_and_consistency():
    N = 512
    Z = np.clip(RNG.standard_normal((32, N)) * 3, -5, 5)
    out, lse = O.rowop(Z, I.NORM_LOGSUMEXP)
    assert np.array_equal(out, Z)
    m = Z.max(axis=1)
    assert (lse >= m).all() and (lse <= m + math.log(N) + 1e-12).all()
    assert (lse >= -5 + math.log(N) - 1e-12).all() and (lse <= 5 + math.log(N) + 1e-12).all()
    np.testing.assert_allclose(np.exp(Z - lse[:, None]).sum(axis=1), 1.0, atol=1e-12)
    np.testing.assert_allclose(lse, sp.logsumexp(Z, axis=1), rtol=1e-14)
    P, _ = O.rowop(Z, I.NORM_SOFTMAX)                                 # ties LSE to softmax
    np.testing.assert_allclose(np.exp(Z - lse[:, None]), P, rtol=1e-12)


def test_layernorm_closed_forms_and_invariants():
    g = GOLD["layernorm_1to5"]
    o, _ = O.rowop(_row(g["row"]), I.NORM_LAYERNORM, 0.0)
    np.testing.assert_allclose(o[0] * math.sqrt(2.0), g["out_times_sqrt2"], atol=1e-15)
    g = GOLD["layernorm_eps"]
    o, _ = O.rowop(_row(g["row"]), I.NORM_LAYERNORM, g["eps"], np.array(g["gamma"], float),
                   np.array(g["beta"], float))
    np.testing.assert_allclose(o[0], g["out"], atol=1e-15)

    A = RNG.standard_normal((8, 96)) * 2 + 5
    eps = 1e-5
    o, _ = O.rowop(A, I.NORM_LAYERNORM, eps)
    var = A.var(axis=1)
    np.testing.assert_allclose(o.mean(axis=1), 0.0, atol=1e-13)
    np.testing.assert_allclose(o.var(axis=1), var / (var + eps), rtol=1e-12)   # biased variance
    beta = RNG.standard_normal(96)
    oc, _ = O.rowop(np.full((2, 96), 7.5), I.NORM_LAYERNORM, eps, None, beta)
    assert np.array_equal(oc, np.broadcast_to(beta, (2, 96)))                  # constant row
    o0, _ = O.rowop(A, I.NORM_LAYERNORM, 0.0)
    o1, _ = O.rowop(3.0 * A - 11.0, I.NORM_LAYERNORM, 0.0)                     # affine invariance
    np.testing.assert_allclose(o1, o0, atol=1e-12)
    gamma = RNG.standard_normal(96)
    ot, _ = O.rowop(A, I.NORM_LAYERNORM, eps, gamma, beta)
    ref = torch.nn.functional.layer_norm(torch.from_numpy(A), (96,), torch.from_numpy(gamma),
                                         torch.from_numpy(beta), eps).numpy()
    np.testing.assert_allclose(ot, ref, rtol=0, atol=1e-12)


def test_rmsnorm_sketch_steps_and_invariants():
    g = GOLD["rmsnorm_3_4"]
    o, _ = O.rowop(_row(g["row"]), I.NORM_RMSNORM, g["eps"], np.array(g["gamma"], float))
    np.testing.assert_allclose(o[0] * math.sqrt(2.0), g["out_times_sqrt2"], rtol=1e-15)

    A = RNG.standard_normal((8, 80)) * 3 + 1          # not centred: RMSNorm must not centre
    eps = 1e-6
    o, _ = O.rowop(A, I.NORM_RMSNORM, eps)
    ms = (A * A).mean(axis=1)
    np.testing.assert_allclose((o * o).mean(axis=1), ms / (ms + eps), rtol=1e-12)
    o0, _ = O.rowop(A, I.NORM_RMSNORM, 0.0)
    o1, _ = O.rowop(17.0 * A, I.NORM_RMSNORM, 0.0)                             # scale invariance
    np.testing.assert_allclose(o1, o0, rtol=1e-12)
    oz, _ = O.rowop(np.zeros((1, 80)), I.NORM_RMSNORM, eps)
    assert not oz.any()
    gamma = RNG.standard_normal(80)
    og, _ = O.rowop(A, I.NORM_RMSNORM, eps, gamma)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(A), (80,), torch.from_numpy(gamma), eps).numpy()
    np.testing.assert_allclose(og, ref, rtol=0, atol=1e-12)


def test_split_merge_equals_single_pass():
    """Per-tile (max, sum-exp) pairs and (count, mean, M2) triples merged in any grouping give
    the single-pass row statistics: the algebra the split-N GPU path relies on."""
    N = 360
    a = RNG.standard_normal(N) * 3
    _, lse = O.rowop(a[None, :], I.NORM_LOGSUMEXP)
    cuts = np.sort(RNG.choice(np.arange(1, N), size=7, replace=False))
    parts = np.split(a, cuts)
    ms = [(p.max(), np.exp(p - p.max()).sum()) for p in parts]
    order = RNG.permutation(len(ms))
    m, s = ms[order[0]]
    for t in order[1:]:
        m2, s2 = ms[t]
        mn = max(m, m2)
        s = s * math.exp(m - mn) + s2 * math.exp(m2 - mn)
        m = mn
    assert abs(m + math.log(s) - lse[0]) < 1e-12
    n, mean, M2 = 0, 0.0, 0.0
    for t in order:
        p = parts[t]
        nb, mb, M2b = len(p), p.mean(), ((p - p.mean()) ** 2).sum()
        d = mb - mean
        M2 = M2 + M2b + d * d * n * nb / (n + nb)
        mean = mean + d * nb / (n + nb)
        n += nb
    o, _ = O.rowop(a[None, :], I.NORM_LAYERNORM, 0.0)
    np.testing.assert_allclose((a - mean) / math.sqrt(M2 / n), o[0], atol=1e-12)


# ----------------------------------------------------------------- the whole chain

def test_chain_tiny_by_hand():
    g = GOLD["chain_tiny"]
    X = np.array(g["X"], float); W = np.array(g["W"], float); b = np.array(g["b"], float)
    Y = np.array(g["Y"], float)
    y, _ = O.chain(X, W, b, alpha=g["alpha"], post_scale=g["post_scale"])
    assert np.array_equal(y, Y)
    p, _ = O.chain(X, W, b, alpha=g["alpha"], post_scale=g["post_scale"], act=I.ACT_RELU,
                   norm=I.NORM_SOFTMAX)
    e1, e2 = math.exp(-1.0), math.exp(-2.0)
    np.testing.assert_allclose(p[0], np.array([1.0, e1, e2]) / (1 + e1 + e2), rtol=1e-15)
    np.testing.assert_allclose(p[1], np.array([1.0, e1, 1.0]) / (2 + e1), rtol=1e-15)


def _torch_chain(w: I.Workload, t):
    F = torch.nn.functional
    X, W = torch.from_numpy(t["X"]), torch.from_numpy(t["W"])
    y = w.alpha * (X @ W.T)
    if t["b"] is not None:
        y = y + torch.from_numpy(t["b"])
    y = w.post_scale * y
    a = {I.ACT_NONE: lambda v: v, I.ACT_RELU: F.relu,
         I.ACT_GELU_TANH: lambda v: F.gelu(v, approximate="tanh"), I.ACT_GELU_ERF: F.gelu,
         I.ACT_SILU: F.silu, I.ACT_CLAMP: lambda v: torch.clamp(v, w.clamp_lo, w.clamp_hi)}[w.act](y)
    g = None if t["gamma"] is None else torch.from_numpy(t["gamma"])
    be = None if t["beta"] is None else torch.from_numpy(t["beta"])
    aux = None
    if w.norm == I.NORM_SOFTMAX:
        o = torch.softmax(a, dim=-1)
    elif w.norm == I.NORM_LAYERNORM:
        o = F.layer_norm(a, (w.N,), g, be, w.eps)
    elif w.norm == I.NORM_RMSNORM:
        o = F.rms_norm(a, (w.N,), g, w.eps)
    elif w.norm == I.NORM_LOGSUMEXP:
        o, aux = a, torch.logsumexp(a, dim=-1)
    else:
        o = a
    return o.numpy(), None if aux is None else aux.numpy()


@pytest.mark.parametrize("name", ["cfg1", "cfg2", "cfg3", "cfg4", "cfg5"])
def test_chain_matches_library_composition(name):
    """Each workload's chain at a reduced, non-square shape against torch float64 CPU ops."""
    w = I.scaled(I.WORKLOADS[name], M=23, K=40, N=56, batch=2 if name == "cfg4" else 1)
    t = {k: I.as_f64(v) for k, v in I.generate(w).items()}
    out, aux = O.chain(t["X"], t["W"], t["b"], t["gamma"], t["beta"], alpha=w.alpha,
                       post_scale=w.post_scale, act=w.act, clamp_lo=w.clamp_lo,
                       clamp_hi=w.clamp_hi, norm=w.norm, eps=w.eps)
    ro, ra = _torch_chain(w, t)
    assert out.shape == (w.rows, w.N)
    np.testing.assert_allclose(out, ro, rtol=0, atol=1e-12)
    if ra is not None:
        np.testing.assert_allclose(aux, ra, rtol=1e-13)


def test_gated_chain_by_hand_and_special_cases():
    """The gated variant (act(G) * U, the SiLU-and-Mul / GELU-and-Mul operators of the paper's
    Section 3.6): a hand-computed case, reductions to the plain chain, and the scaling of each
    product - a swapped operand, a gate applied to the wrong factor or a bias added to the wrong
    product fails one of these."""
    X = np.array([[1.0, 2.0], [0.0, -1.0]])
    W1 = np.array([[1.0, 0.0], [0.0, 1.0], [1.0, 1.0]])          # G = [[1,2,3],[0,-1,-1]]
    W2 = np.array([[2.0, 0.0], [0.0, 0.5], [1.0, -1.0]])         # U = [[2,1,-1],[0,-0.5,1]]
    b1 = np.array([0.0, 1.0, -4.0]); b2 = np.array([1.0, 0.0, 0.0])
    # G + b1 = [[1,3,-1],[0,0,-5]], U + b2 = [[3,1,-1],[1,-0.5,1]]; relu(G+b1) * (U+b2):
    out, _ = O.gated_chain(X, W1, W2, b1, b2, act=I.ACT_RELU)
    assert np.array_equal(out, np.array([[3.0, 3.0, 0.0], [0.0, -0.0, 0.0]]))
    # alpha scales both products (not the biases), post_scale both biased sums
    out, _ = O.gated_chain(X, W1, W2, b1, b2, alpha=2.0, post_scale=0.5, act=I.ACT_NONE)
    G = 0.5 * (2.0 * X @ W1.T + b1); U = 0.5 * (2.0 * X @ W2.T + b2)
    assert np.array_equal(out, G * U)
    rng = np.random.default_rng(5)
    X = rng.normal(size=(7, 11)); W1 = rng.normal(size=(13, 11)); W2 = rng.normal(size=(13, 11))
    b1 = rng.normal(size=13); g = rng.normal(size=13) + 1.0; be = rng.normal(size=13)
    # U == 1 (W2 = 0, b2 = 1): the gated chain is the plain chain, for every activation and row op
    for act in range(6):
        for norm in range(5):
            a, ax = O.gated_chain(X, W1, np.zeros_like(W2), b1, np.ones(13), g, be, alpha=0.7, act=act,
                                  clamp_lo=-1.0, clamp_hi=0.5, norm=norm, eps=1e-5)
            r, rx = O.chain(X, W1, b1, g, be, alpha=0.7, act=act, clamp_lo=-1.0, clamp_hi=0.5, norm=norm, eps=1e-5)
            assert np.array_equal(a, r) and np.array_equal(ax, rx, equal_nan=True)
    # SiLU-and-Mul and GELU-and-Mul against scipy / numpy on the same products
    G = X @ W1.T + b1; U = X @ W2.T
    np.testing.assert_allclose(O.gated_chain(X, W1, W2, b1, None, act=I.ACT_SILU)[0], G * sp.expit(G) * U, rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(O.gated_chain(X, W1, W2, b1, None, act=I.ACT_GELU_ERF)[0],
                               G * sp.ndtr(G) * U, rtol=1e-12, atol=1e-15)
    # the gate is not symmetric: swapping W1 and W2 changes the result (unless act is none)
    assert not np.allclose(O.gated_chain(X, W1, W2, act=I.ACT_SILU)[0], O.gated_chain(X, W2, W1, act=I.ACT_SILU)[0])
    assert np.array_equal(O.gated_chain(X, W1, W2, act=I.ACT_NONE)[0], O.gated_chain(X, W2, W1, act=I.ACT_NONE)[0])
    # row op after the gate: torch float64 composition
    out, _ = O.gated_chain(X, W1, W2, b1, None, g, None, act=I.ACT_SILU, norm=I.NORM_RMSNORM, eps=1e-6)
    a = torch.from_numpy(G * sp.expit(G) * U)
    np.testing.assert_allclose(out, torch.nn.functional.rms_norm(a, (13,), torch.from_numpy(g), 1e-6).numpy(), rtol=0, atol=1e-12)
    np.testing.assert_array_equal(O.gate(G, U, I.ACT_RELU), np.maximum(G, 0.0) * U)
    with pytest.raises(ValueError):
        O.gated_chain(X, W1, W2, act=9)


def test_chain_rejects_unknown_codes():
    X = np.ones((2, 2)); W = np.ones((2, 2))
    with pytest.raises(ValueError):
        O.chain(X, W, act=17)
    with pytest.raises(ValueError):
        O.chain(X, W, norm=-1)


def test_workload_value_ranges():
    """Structure the workloads promise: cfg5's clamp is exercised and its lse range holds;
    cfg1 rows are valid softmaxes."""
    w = I.scaled(I.WORKLOADS["cfg5"], M=512)
    t = {k: I.as_f64(v) for k, v in I.generate(w).items()}
    Z, lse = O.chain(t["X"], t["W"], t["b"], alpha=w.alpha, post_scale=w.post_scale, act=w.act,
                     clamp_lo=w.clamp_lo, clamp_hi=w.clamp_hi, norm=w.norm)
    assert Z.min() == -5.0 or Z.max() == 5.0
    frac = np.mean(np.abs(Z) == 5.0)
    assert 0 < frac < 0.05
    assert (lse > -5 + math.log(512) - 1e-9).all() and (lse < 5 + math.log(512) + 1e-9).all()
    w = I.WORKLOADS["cfg1"]
    t = {k: I.as_f64(v) for k, v in I.generate(w).items()}
    P, _ = O.chain(t["X"], t["W"], t["b"], act=w.act, norm=w.norm)
    np.testing.assert_allclose(P.sum(axis=1), 1.0, atol=1e-12)


# ----------------------------------------------------------------- error metrics

def test_metrics_by_hand():
    ref = np.array([[1.0, -1.0, 0.0, 2.0]])            # row floor = mean|r| = 1
    got = ref + np.array([[1e-3, 0.0, 1e-3, 2e-3]])
    assert abs(C.max_rel_err(got, ref) - 1e-3) < 1e-15  # 1e-3/1, 1e-3/floor 1, 2e-3/2
    assert C.verifier_fraction(got, ref, 5e-4) == 0.75
    assert C.verifier_fraction(got, ref, 2e-3) == 0.0
    assert abs(C.max_rel_err_vec(np.array([2.02]), np.array([2.0])) - 0.01) < 1e-12


def test_metrics_count_a_missing_value_as_a_failure():
    """An element that is NaN has no error below any threshold: both gates must fail on it
    (the pass rule of the paper's Section 3.2.3 counts the elements that do NOT meet tau)."""
    ref = np.array([[1.0, -1.0, 0.0, 2.0]])
    got = ref.copy()
    got[0, 2] = np.nan
    assert not (C.max_rel_err(got, ref) <= 1e-4)
    assert C.verifier_fraction(got, ref, 1e-3) == 0.25
