"""Search over the library's launch configurations for one problem.

The paper's optimisation loop (its evolutionary search, Section 3.5) proposes kernel variants,
has the Verifier accept or reject each one, times the accepted ones and keeps the fastest.  The
configuration space of this library is small and discrete - tile configuration x how split rows
are finished x (fp32 operands) which matrix instruction multiplies - so the search here visits
all of it instead of evolving a population: every configuration the library accepts for the
problem is run, checked against the automatic configuration's result (the Verifier's element
rule with the tolerance of the storage type), timed, and the table is returned fastest first.

    python -m paper_2512_23424_amd.tune cfg2            # one of the built-in workloads

The search only uses the public entry points; FGE_FLAG_TILE and FGE_FLAG_TWO_PASS select the
configuration.  It is a tool around the library, not part of a call's hot path."""
from __future__ import annotations

import sys
from typing import Callable, Dict, List, Optional

import torch

from . import binding as B
from . import inputs as I

TILES = {"64x64": 0, "64x512": 1, "128x128": 2, "256x256": 3, "narrow_k": 4, "64x128": 5}
_TOL = {I.F32: 1e-4, I.BF16: 2e-2, I.F16: 4e-3, I.F8E4M3: 2e-2}


def flag_tile(tile: int) -> int:
    return (tile + 1) << 8


def candidates(make_params: Callable[[int], B.FgeParams], act, norm) -> List[Dict]:
    """Distinct configurations the library accepts: (label, flags) with the kernel name each runs."""
    seen, out = set(), []
    base = make_params(0)
    extra = [0, B.FLAG_IEEE_FP32] if base.in_dtype == I.F32 else [0]
    for tname, tid in [("auto", None)] + list(TILES.items()):
        for two_pass in (0, B.FLAG_TWO_PASS):
            for ex in extra:
                flags = (0 if tid is None else flag_tile(tid)) | two_pass | ex
                p = make_params(flags)
                try:
                    kernel = B.fge_tile_name(True, act, norm, p)
                    finish = B.fge_fused_needs_finish(act, norm, p)
                except B.FgeError:
                    continue
                key = (kernel, finish)
                if key in seen:
                    continue
                seen.add(key)
                out.append({"label": f"{tname}{'+two_pass' if finish else ''}{'+ieee' if ex else ''}",
                            "flags": flags, "kernel": kernel, "kernels": 2 if finish else 1, "auto": tid is None})
    return out


def _deviation(got: torch.Tensor, ref: torch.Tensor) -> float:
    g, r = got.double(), ref.double()
    floor = r.abs().mean(dim=-1, keepdim=True)
    return float(((g - r).abs() / torch.maximum(r.abs(), floor)).max())


def tune(X, W, b, act, norm, out: torch.Tensor, *, steps: int = 20, warmup: int = 5, **params) -> List[Dict]:
    """Run, check and time every configuration for fused_gemm_epilogue(X, W, b, act, norm) -> out.
    `params` are the keyword arguments of binding.make_params (alpha, eps, gamma, ...)."""
    def make_params(flags: int) -> B.FgeParams:
        return B.make_params(X, W, out, flags=flags, **params)
    ref: Optional[torch.Tensor] = None
    table = []
    for c in candidates(make_params, act, norm):
        p = make_params(c["flags"])
        ws = torch.empty(max(B.fge_workspace_bytes(True, act, norm, p), 16), dtype=torch.uint8, device=out.device)
        p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel()
        out.fill_(float("nan"))
        B.fused_gemm_epilogue(X, W, b, act, norm, p, out)
        torch.cuda.synchronize()
        if ref is None:                     # the automatic configuration comes first
            ref = out.clone()
        dev = _deviation(out, ref)
        ok = bool(torch.isfinite(out).all()) and dev <= 2.0 * _TOL[p.out_dtype if p.out_dtype != I.F32 else p.in_dtype]
        for _ in range(warmup):
            B.fused_gemm_epilogue(X, W, b, act, norm, p, out)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(steps):
            B.fused_gemm_epilogue(X, W, b, act, norm, p, out)
        e1.record()
        torch.cuda.synchronize()
        table.append(dict(c, ms=e0.elapsed_time(e1) / steps, deviation=dev, accepted=ok))
    return sorted(table, key=lambda r: (not r["accepted"], r["ms"]))


def _upload(a):
    import numpy as np
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint8:
        return torch.from_numpy(a).cuda().view(torch.float8_e4m3fn)
    return torch.from_numpy(a).cuda()


def main(argv: List[str]) -> int:
    name = argv[1] if len(argv) > 1 else "cfg2"
    w = I.WORKLOADS[name] if name in I.WORKLOADS else I.EXTRA_WORKLOADS[name]
    t = {k: _upload(v) for k, v in I.generate(w).items()}
    X = t["X"].view(w.batch, w.M, w.K) if w.batch > 1 else t["X"]
    dt = {I.BF16: torch.bfloat16, I.F16: torch.float16}.get(w.out_dtype, torch.float32)
    out = torch.empty((w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N), dtype=dt, device="cuda")
    aux = torch.empty(w.rows, device="cuda") if w.norm == I.NORM_LOGSUMEXP else None
    table = tune(X, t["W"], t["b"], w.act, w.norm, out, alpha=w.alpha, post_scale=w.post_scale,
                 clamp_lo=w.clamp_lo, clamp_hi=w.clamp_hi, eps=w.eps, gamma=t["gamma"], beta=t["beta"], aux_out=aux)
    print(f"{name}: {len(table)} configurations")
    for r in table:
        print(f"  {r['ms']:9.4f} ms  {'ok ' if r['accepted'] else 'REJ'} dev {r['deviation']:.1e}  "
              f"{r['label']:24s} {r['kernel']}{' (automatic choice)' if r['auto'] else ''}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
