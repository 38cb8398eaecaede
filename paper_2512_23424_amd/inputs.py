"""Seeded, synthetic inputs for the fused chain  out = norm_N(act(post_scale*(alpha*X.W^T + b))).

This module only *draws numbers*: it holds no arithmetic of the chain itself, so both the
CPU float64 oracle and the HIP path can be fed from it without sharing any of the method's
code.  The paper evaluates on operator suites (matmul / activation / softmax / LayerNorm /
RMSNorm families, Section 3.6 "benchmark" paragraph); the five workloads below stand in for
those families with fixed shapes and value distributions.

Generator (counter based, order independent, reproducible on any host):

    mix(z)   : the 64-bit finaliser of splitmix64 (xor-shift 30, multiply, xor-shift 27,
               multiply, xor-shift 31)
    key      = mix(mix(seed) ^ tensor_id)
    u(i)     = (mix(key + i) >> 11) * 2^-53                      in [0, 1)
    uniform  : a + (b - a) * u(i)
    normal   : mean + std * sqrt(-2 ln(1 - u(2i))) * cos(2 pi u(2i + 1))   (Box-Muller, cos branch)

Values are produced in float64 and rounded once (round-to-nearest-even) to the storage type
(fp32, bf16, fp16 or 8-bit E4M3).  bf16 tensors are returned as uint16 bit patterns, fp16
tensors as numpy float16 arrays, E4M3 tensors as uint8 bit patterns.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

# activation / row-op / dtype codes: the same integers as the C header's enums.
ACT_NONE, ACT_RELU, ACT_GELU_TANH, ACT_GELU_ERF, ACT_SILU, ACT_CLAMP = range(6)
NORM_NONE, NORM_SOFTMAX, NORM_LAYERNORM, NORM_RMSNORM, NORM_LOGSUMEXP = range(5)
F32, BF16, F16, F8E4M3 = 0, 1, 2, 3

TENSOR_ID = {"X": 0, "W": 1, "b": 2, "gamma": 3, "beta": 4, "W2": 5, "b2": 6}   # W2, b2: gated form

_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)
_MASK64 = (1 << 64) - 1


def _mix_int(z: int) -> int:
    z &= _MASK64
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & _MASK64
    return z ^ (z >> 31)


def _mix_vec(z: np.ndarray) -> np.ndarray:
    z = (z ^ (z >> np.uint64(30))) * _M1
    z = (z ^ (z >> np.uint64(27))) * _M2
    return z ^ (z >> np.uint64(31))


def stream_key(seed: int, tensor_id: int) -> int:
    return _mix_int(_mix_int(seed) ^ tensor_id)


def unit_uniform(key: int, start: int, count: int) -> np.ndarray:
    """u(start) .. u(start+count-1) as float64 in [0,1)."""
    idx = np.arange(start, start + count, dtype=np.uint64) + np.uint64(key)
    return (_mix_vec(idx) >> np.uint64(11)).astype(np.float64) * (2.0 ** -53)


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float64 -> bf16 bit pattern with ONE round-to-nearest-even step (going through fp32
    first could round twice).  Works on the float64 bit pattern: keep sign, exponent and the
    top 7 mantissa bits, round on the 45 dropped bits, then re-bias the exponent from 1023 to
    127.  Magnitudes below the bf16 normal range give signed zero; the workloads here stay
    far inside the normal range."""
    u = np.ascontiguousarray(x, dtype=np.float64).view(np.uint64)
    sign = (u >> np.uint64(63)).astype(np.uint64)
    mag = u & np.uint64(0x7FFFFFFFFFFFFFFF)
    mag = (mag + np.uint64((1 << 44) - 1) + ((mag >> np.uint64(45)) & np.uint64(1))) >> np.uint64(45)
    e11 = mag >> np.uint64(7)                      # biased-1023 exponent after rounding carry
    small = e11 < np.uint64(897)                   # below 2^-126 (or zero)
    mag8 = np.where(small, np.uint64(0), mag - np.uint64(896 << 7))
    return ((sign << np.uint64(15)) | mag8).astype(np.uint16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit pattern, round-to-nearest-even (finite inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = u + np.uint64(0x7FFF) + ((u >> np.uint64(16)) & np.uint64(1))
    return (u >> np.uint64(16)).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f64_to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """float64 -> 8-bit E4M3 pattern (sign, 4 exponent bits with bias 7, 3 mantissa bits; no
    infinities, largest finite value 448) with one round-to-nearest-even step.  Values are
    rounded on the grid of their binade - spacing 2^(e-3) for 2^e <= |x| < 2^(e+1), 2^-9 below
    the smallest normal 2^-6 - and magnitudes that round beyond 448 saturate to 448."""
    x = np.asarray(x, dtype=np.float64)
    a = np.abs(x)
    e = np.floor(np.log2(np.maximum(a, 2.0 ** -20)))
    e = np.clip(e, -6.0, 8.0)
    q = np.exp2(e - 3.0)                            # grid spacing (exact powers of two)
    r = np.minimum(np.rint(a / q) * q, 448.0)       # rint rounds halves to even
    e2 = np.clip(np.floor(np.log2(np.maximum(r, 2.0 ** -20))), -6.0, 8.0)   # rounding may reach the next binade
    normal = r >= 2.0 ** -6
    expo = np.where(normal, e2 + 7.0, 0.0)
    mant = np.where(normal, (r / np.exp2(e2) - 1.0) * 8.0, r * 512.0)
    bits = (expo.astype(np.uint8) << np.uint8(3)) | mant.astype(np.uint8)
    return (bits | (np.signbit(x).astype(np.uint8) << np.uint8(7))).astype(np.uint8)


def e4m3_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """Value of each 8-bit E4M3 pattern (NaN for 0x7F / 0xFF), through a 256-entry table."""
    codes = np.arange(256)
    expo, mant = (codes >> 3) & 15, codes & 7
    mag = np.where(expo == 0, mant * 2.0 ** -9, (1.0 + mant / 8.0) * np.exp2(expo.astype(np.float64) - 7.0))
    mag = np.where((expo == 15) & (mant == 7), np.nan, mag)
    table = np.where(codes >= 128, -mag, mag)
    return table[np.asarray(bits, dtype=np.uint8)]


def _store(v64: np.ndarray, dtype: int) -> np.ndarray:
    """One rounding (to nearest even) from float64 to the storage type; fp16 tensors are numpy
    float16 arrays (numpy converts double to half directly, without an fp32 step)."""
    if dtype == BF16:
        return f64_to_bf16_bits(v64)
    if dtype == F8E4M3:
        return f64_to_e4m3_bits(v64)
    return v64.astype(np.float16 if dtype == F16 else np.float32)


_CHUNK = 1 << 22


def draw(seed: int, tensor: str, shape: Tuple[int, ...], dist: Tuple, dtype: int = F32) -> np.ndarray:
    """Draw one tensor.  dist = ("normal", mean, std) | ("uniform", a, b) | ("int", lo, hi)
    ("int" draws integers lo..hi inclusive, exactly representable in bf16 and fp32)."""
    key = stream_key(seed, TENSOR_ID[tensor])
    n = int(np.prod(shape))
    out = np.empty(n, dtype={BF16: np.uint16, F16: np.float16, F8E4M3: np.uint8}.get(dtype, np.float32))
    for s in range(0, n, _CHUNK):
        c = min(_CHUNK, n - s)
        if dist[0] == "normal":
            u = unit_uniform(key, 2 * s, 2 * c)
            r = np.sqrt(-2.0 * np.log(1.0 - u[0::2]))
            v = dist[1] + dist[2] * (r * np.cos((2.0 * math.pi) * u[1::2]))
        elif dist[0] == "uniform":
            v = dist[1] + (dist[2] - dist[1]) * unit_uniform(key, s, c)
        elif dist[0] == "int":
            span = dist[2] - dist[1] + 1
            v = dist[1] + np.floor(unit_uniform(key, s, c) * span)
        else:
            raise ValueError(dist)
        out[s:s + c] = _store(v, dtype)
    return out.reshape(shape)


@dataclass(frozen=True)
class Workload:
    """Shape, storage types, chain parameters and value distributions of one workload."""
    name: str
    M: int
    K: int
    N: int
    batch: int = 1
    in_dtype: int = F32
    out_dtype: int = F32
    act: int = ACT_NONE
    norm: int = NORM_NONE
    alpha: float = 1.0
    post_scale: float = 1.0
    clamp_lo: float = 0.0
    clamp_hi: float = 0.0
    eps: float = 0.0
    dist: Dict[str, Optional[Tuple]] = field(default_factory=dict)
    seed: int = 0

    @property
    def rows(self) -> int:
        return self.M * self.batch

    @property
    def flops(self) -> float:
        return 2.0 * self.rows * self.N * self.K

    @property
    def algorithmic_bytes(self) -> int:
        """Every operand and result moved exactly once."""
        isz = {F32: 4, F8E4M3: 1}.get(self.in_dtype, 2)
        osz = 4 if self.out_dtype == F32 else 2
        vecs = sum(1 for t in ("b", "gamma", "beta") if self.dist.get(t) is not None)
        aux = self.rows * 4 if self.norm == NORM_LOGSUMEXP else 0
        return (self.rows * self.K * isz + self.N * self.K * isz + vecs * self.N * 4
                + self.rows * self.N * osz + aux)


def _wl(name, M, K, N, **kw) -> Workload:
    return Workload(name=name, M=M, K=K, N=N, **kw)


WORKLOADS: Dict[str, Workload] = {
    # fp32 64^3, ReLU, row softmax
    "cfg1": _wl("cfg1", 64, 64, 64, act=ACT_RELU, norm=NORM_SOFTMAX,
                dist={"X": ("normal", 0.0, 1.0 / 8.0), "W": ("normal", 0.0, 1.0 / 8.0),
                      "b": ("uniform", -0.1, 0.1)}),
    # fp32 4096x1024x1024, GELU(tanh), LayerNorm with affine
    "cfg2": _wl("cfg2", 4096, 1024, 1024, act=ACT_GELU_TANH, norm=NORM_LAYERNORM, eps=1e-5,
                dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0 / 32.0),
                      "b": ("uniform", -0.1, 0.1), "gamma": ("normal", 1.0, 0.1),
                      "beta": ("normal", 0.0, 0.1)}),
    # bf16 in / fp32 accumulate / bf16 out, 8192x4096x4096, SiLU, RMSNorm with gamma, no bias
    "cfg3": _wl("cfg3", 8192, 4096, 4096, in_dtype=BF16, out_dtype=BF16, act=ACT_SILU,
                norm=NORM_RMSNORM, eps=1e-6,
                dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0 / 64.0),
                      "gamma": ("normal", 1.0, 0.1)}),
    # batched bf16: 16 x (2048x512x2048), W and b shared, alpha = 1/sqrt(K), GELU(erf), softmax
    "cfg4": _wl("cfg4", 2048, 512, 2048, batch=16, in_dtype=BF16, out_dtype=BF16,
                act=ACT_GELU_ERF, norm=NORM_SOFTMAX, alpha=1.0 / math.sqrt(512.0),
                dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0 / math.sqrt(512.0)),
                      "b": ("uniform", -0.1, 0.1)}),
    # fp32 narrow-K: 262144x64x512, Z = clamp(2*(X.W^T+b), -5, 5), outputs Z and row logsumexp
    "cfg5": _wl("cfg5", 262144, 64, 512, act=ACT_CLAMP, norm=NORM_LOGSUMEXP, post_scale=2.0,
                clamp_lo=-5.0, clamp_hi=5.0,
                dist={"X": ("uniform", -1.0, 1.0), "W": ("normal", 0.0, 1.0 / 8.0),
                      "b": ("normal", 0.0, 0.5)}),
}


# Beyond the five: the headline shape with 8-bit E4M3 operands.  Unit-variance X and W are
# stored as they are (E4M3 keeps 3 mantissa bits at any magnitude within its range) and the
# per-tensor scale 1/sqrt(K) goes into alpha, as 8-bit pipelines do.
EXTRA_WORKLOADS: Dict[str, Workload] = {
    "cfg3_f8": _wl("cfg3_f8", 8192, 4096, 4096, in_dtype=F8E4M3, out_dtype=BF16, act=ACT_SILU,
                   norm=NORM_RMSNORM, eps=1e-6, alpha=1.0 / 64.0,
                   dist={"X": ("normal", 0.0, 1.0), "W": ("normal", 0.0, 1.0),
                         "gamma": ("normal", 1.0, 0.1)}),
}


def scaled(w: Workload, **kw) -> Workload:
    """Same chain and distributions at another shape (parity-test sizes)."""
    d = dict(w.__dict__)
    d.update(kw)
    return Workload(**d)


def generate(w: Workload, rows: Optional[np.ndarray] = None) -> Dict[str, Optional[np.ndarray]]:
    """All tensors of a workload.  X is (batch*M, K); W is (N, K); vectors are fp32 length N.
    If `rows` is given only those rows of X are kept (the draw itself is unchanged)."""
    out: Dict[str, Optional[np.ndarray]] = {}
    X = draw(w.seed, "X", (w.rows, w.K), w.dist["X"], w.in_dtype)
    out["X"] = X if rows is None else np.ascontiguousarray(X[rows])
    out["W"] = draw(w.seed, "W", (w.N, w.K), w.dist["W"], w.in_dtype)
    for t in ("b", "gamma", "beta"):
        d = w.dist.get(t)
        out[t] = None if d is None else draw(w.seed, t, (w.N,), d, F32)
    return out


def as_f64(a: Optional[np.ndarray]) -> Optional[np.ndarray]:
    """Exact float64 value of stored bits (uint16 arrays are bf16 patterns, uint8 arrays E4M3)."""
    if a is None:
        return None
    if a.dtype == np.uint16:
        return bf16_bits_to_f32(a).astype(np.float64)
    if a.dtype == np.uint8:
        return e4m3_bits_to_f64(a)
    return a.astype(np.float64)


def generate_gated(w: Workload) -> Dict[str, Optional[np.ndarray]]:
    """Tensors of the gated form of a workload: those of generate() with W, b as the first
    product's, plus W2 (drawn like W) and b2 (drawn like b) from streams of their own."""
    out = generate(w)
    out["W2"] = draw(w.seed, "W2", (w.N, w.K), w.dist["W"], w.in_dtype)
    d = w.dist.get("b")
    out["b2"] = None if d is None else draw(w.seed, "b2", (w.N,), d, F32)
    return out


def adversarial(w: Workload, kind: str) -> Dict[str, Optional[np.ndarray]]:
    """The tensors of generate(w) reshaped into rows that stress a row operation (the paper's
    benchmark section names hidden assumptions about the inputs as the typical failure of
    generated kernels).  Only stored values are chosen here; nothing of the chain is computed.

      "dominant" : the bias carries one dominant column (+80) over a spread of -80 .. 0, so the
                   activations of a row (with act = none) reach |a| = 80 and one element holds
                   almost all of a softmax's mass;
      "constant" : W = 0 and a constant bias - every row is constant;
      "tied"     : W = 0 and a bias whose maximum recurs every 64 columns, so that all column
                   tiles (and wave strips) of a row report exactly the same maximum;
      "offset"   : the first contraction index carries x = 1.2345678, w = 810.0123 for every row
                   and column: the product puts a common offset of about 1000 under every row,
                   against a spread of order one from the remaining random terms."""
    t = generate(w)
    n = np.arange(w.N)
    if kind == "dominant":
        b = -80.0 * ((n * 37) % 101) / 100.0
        b[(w.N * 5) // 7] = 80.0
        t["b"] = b.astype(np.float32)
    elif kind == "constant":
        t["W"] = _store(np.zeros((w.N, w.K)), w.in_dtype)
        t["b"] = np.full(w.N, 3.25, dtype=np.float32)
    elif kind == "tied":
        t["W"] = _store(np.zeros((w.N, w.K)), w.in_dtype)
        b = -1.0 - ((n * 13) % 17) / 4.0
        b[n % 64 == 5] = 5.0
        t["b"] = b.astype(np.float32)
    elif kind == "offset":
        X, W = as_f64(t["X"]).copy(), as_f64(t["W"]).copy()
        X[:, 0] = 1.2345678
        W[:, 0] = 810.0123
        t["X"], t["W"] = _store(X, w.in_dtype), _store(W, w.in_dtype)
    else:
        raise ValueError(kind)
    return t
