"""Search over the library's launch configurations for one problem.

The paper's optimisation loop (its evolutionary search, Section 3.5) proposes kernel variants,
has the Verifier accept or reject each one, times the accepted ones and keeps the fastest.  The
configuration space of this library is small and discrete - tile configuration x how split rows
are finished x (fp32 operands) which matrix instruction multiplies x whether a long K is cut
into slices - so the search here visits
all of it instead of evolving a population: every configuration the library accepts for the
problem is run, checked against the automatic configuration's result (the Verifier's element
rule with the tolerance of the storage type), timed, and the table is returned fastest first.

    python -m paper_2512_23424_amd.tune cfg2            # one of the built-in workloads

    python -m paper_2512_23424_amd.tune cfg2 --evolve   # the paper's loop instead of the full visit

`evolve` is that loop itself (Section 3.5, its algorithm "Iterative Search-Based Optimization")
with the language model taken out: K islands, R rounds, P candidates per island and round; the
parents of a round are a stratified sample of the island's population (its fastest and its
slowest members); a candidate is designed from an elite member by changing the choices on
which the fast parents differ from the slow ones (else an untried choice); the Verifier admits
it to the population only if its result passes; every M rounds each island receives the elite
of its neighbour; the answer is the fastest member of any island.  Here it reaches the same
configuration as the full visit with fewer kernel runs only when the space grows; it is kept
as the search driver for larger configuration spaces and is tested on synthetic ones.

The search only uses the public entry points; FGE_FLAG_TILE, FGE_FLAG_TWO_PASS, FGE_FLAG_IEEE_FP32
and FGE_FLAG_NO_SPLIT_K select the configuration.  It is a tool around the library, not part of a call's hot path."""
from __future__ import annotations

import random
import sys
from typing import Callable, Dict, List, Optional, Sequence, Tuple

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
                for whole_k in (0, B.FLAG_NO_SPLIT_K):
                    flags = (0 if tid is None else flag_tile(tid)) | two_pass | ex | whole_k
                    p = make_params(flags)
                    try:
                        kernel = B.fge_tile_name(True, act, norm, p)
                        slices = B.fge_fused_k_slices(act, norm, p)
                        finish = slices == 1 and B.fge_fused_needs_finish(act, norm, p)
                    except B.FgeError:
                        continue
                    if slices > 1:                      # partial products, their sum, (row op)
                        kernel += f" k/{slices}"
                    key = (kernel, finish)
                    if key in seen:
                        continue
                    seen.add(key)
                    out.append({"label": f"{tname}{'+two_pass' if finish else ''}{'+ieee' if ex else ''}"
                                         f"{'+whole_k' if whole_k else ''}",
                                "flags": flags, "kernel": kernel, "auto": tid is None and not whole_k,
                                "kernels": (2 if norm == I.NORM_NONE else 3) if slices > 1 else 2 if finish else 1})
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


# ---------------------------------------------------------------- the paper's search loop
Config = Tuple                      # one value per gene, in the order of the gene list


class Island:
    def __init__(self) -> None:
        self.population: List[Tuple[Config, float]] = []     # verified candidates with their time
        self.tried: set = set()                                # everything evaluated here, valid or not
        self.elite: List[Tuple[Config, float]] = []
        self.received: List[Tuple[Config, float]] = []         # what migration brought in

    def add(self, c: Config, ms: float) -> None:
        if all(c != q for q, _ in self.population):
            self.population.append((c, ms))

    def update_elite(self, n: int) -> None:
        self.elite = sorted(self.population, key=lambda e: e[1])[:n]


def stratified_sample(population: Sequence[Tuple[Config, float]], n: int = 2):
    """The n fastest and the n slowest members (disjoint; fewer if the population is small)."""
    ranked = sorted(population, key=lambda e: e[1])
    top = ranked[:n]
    bottom = [e for e in ranked[::-1][:n] if e not in top]
    return top, bottom


def design(genes: Sequence[Sequence], base: Optional[Config], top, bottom, tried: set, rng: random.Random) -> Config:
    """A new candidate.  Without a base (empty island): a random one.  Otherwise the base with the
    genes changed on which fast and slow parents disagree - towards the fast parents' choice - and,
    where that yields nothing new, one random gene set to a value not tried with this base."""
    if base is None:
        return tuple(rng.choice(list(v)) for v in genes)
    cand = list(base)
    for g in range(len(genes)):
        fast = {c[g] for c, _ in top}
        slow = {c[g] for c, _ in bottom}
        only_fast = sorted(fast - slow, key=str)
        if only_fast and cand[g] not in only_fast:
            cand[g] = rng.choice(only_fast)
    if tuple(cand) not in tried:
        return tuple(cand)
    for _ in range(8 * len(genes)):                    # explore around the base
        m = list(base)
        g = rng.randrange(len(genes))
        m[g] = rng.choice(list(genes[g]))
        if rng.random() < 0.3:
            g2 = rng.randrange(len(genes))
            m[g2] = rng.choice(list(genes[g2]))
        if tuple(m) not in tried:
            return tuple(m)
    return tuple(rng.choice(list(v)) for v in genes)


def evolve(evaluate: Callable[[Config], Tuple[bool, float]], genes: Sequence[Sequence], *, rounds: int = 3,
           parallel: int = 4, islands: int = 2, migrate_every: int = 1, elite: int = 2, seed: int = 0):
    """The loop of the paper's Section 3.5 over a discrete configuration space.  evaluate(config)
    is the Verifier: (valid, time).  Defaults are the paper's settings (R = 3, P = 4, K = 2,
    Section 4.1).  Returns (best config, its time, the islands)."""
    rng = random.Random(seed)
    isl = [Island() for _ in range(islands)]
    for r in range(1, rounds + 1):
        for k in isl:
            top, bottom = stratified_sample(k.population)
            for _ in range(parallel):
                pool = k.elite or top
                base = rng.choice(pool)[0] if pool else None
                c = design(genes, base, top, bottom, k.tried, rng)
                if c in k.tried:
                    continue                              # nothing new around here
                k.tried.add(c)
                valid, ms = evaluate(c)
                if valid:
                    k.add(c, ms)
            k.update_elite(elite)
        if r % migrate_every == 0 and islands > 1:
            incoming = [list(isl[i - 1].elite) for i in range(islands)]      # ring: i receives from i-1
            for i, k in enumerate(isl):
                for c, ms in incoming[i]:
                    k.add(c, ms)
                    k.tried.add(c)
                    k.received.append((c, ms))
                k.update_elite(elite)
    members = [e for k in isl for e in k.population]
    if not members:
        return None, float("inf"), isl
    best = min(members, key=lambda e: e[1])
    return best[0], best[1], isl


def evolve_library(X, W, b, act, norm, out: torch.Tensor, *, steps: int = 20, warmup: int = 5, seed: int = 0,
                   **params):
    """evolve() over the library's launch configurations for one problem: genes are the tile
    configuration (None = the automatic choice), the split-row form and, for fp32 operands, the
    matrix instruction.  The Verifier runs the candidate, compares with the automatic
    configuration's result (element rule, tolerance of the storage type) and times it; a
    configuration the library refuses is invalid."""
    base = B.make_params(X, W, out, flags=0, **params)
    genes = [[None] + list(TILES), [0, B.FLAG_TWO_PASS], [0, B.FLAG_IEEE_FP32] if base.in_dtype == I.F32 else [0],
             [0, B.FLAG_NO_SPLIT_K]]
    ref: List[Optional[torch.Tensor]] = [None]
    seen: Dict[Config, Dict] = {}

    def run(flags):
        p = B.make_params(X, W, out, flags=flags, **params)
        ws = torch.empty(max(B.fge_workspace_bytes(True, act, norm, p), 16), dtype=torch.uint8, device=out.device)
        p.workspace, p.workspace_bytes = ws.data_ptr(), ws.numel()
        return p, ws

    def evaluate(c: Config):
        if c in seen:                               # another island has run it already
            return seen[c]["accepted"], seen[c]["ms"]
        tname, two_pass, ieee, whole_k = c
        flags = (0 if tname is None else flag_tile(TILES[tname])) | two_pass | ieee | whole_k
        try:
            p, ws = run(flags)
            kernel = B.fge_tile_name(True, act, norm, p)
        except B.FgeError:
            return False, float("inf")
        if ref[0] is None:
            p0, ws0 = run(0)
            out.fill_(float("nan"))
            B.fused_gemm_epilogue(X, W, b, act, norm, p0, out)
            torch.cuda.synchronize()
            ref[0] = out.clone()
        out.fill_(float("nan"))
        B.fused_gemm_epilogue(X, W, b, act, norm, p, out)
        torch.cuda.synchronize()
        dev = _deviation(out, ref[0])
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
        ms = e0.elapsed_time(e1) / steps
        seen[c] = {"kernel": kernel, "ms": ms, "accepted": ok, "deviation": dev}
        return ok, ms
    best, ms, isl = evolve(evaluate, genes, seed=seed)
    return best, ms, seen


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
    import argparse
    known = sorted(I.WORKLOADS) + sorted(I.EXTRA_WORKLOADS)
    ap = argparse.ArgumentParser(prog="python -m paper_2512_23424_amd.tune",
                                 description="Time every configuration the library accepts for a workload.")
    ap.add_argument("workload", nargs="?", default="cfg2", choices=known)
    ap.add_argument("--evolve", action="store_true", help="island search instead of the exhaustive visit")
    args = ap.parse_args(argv[1:])
    name = args.workload
    w = I.WORKLOADS[name] if name in I.WORKLOADS else I.EXTRA_WORKLOADS[name]
    t = {k: _upload(v) for k, v in I.generate(w).items()}
    X = t["X"].view(w.batch, w.M, w.K) if w.batch > 1 else t["X"]
    dt = {I.BF16: torch.bfloat16, I.F16: torch.float16}.get(w.out_dtype, torch.float32)
    out = torch.empty((w.batch, w.M, w.N) if w.batch > 1 else (w.M, w.N), dtype=dt, device="cuda")
    aux = torch.empty(w.rows, device="cuda") if w.norm == I.NORM_LOGSUMEXP else None
    kw = dict(alpha=w.alpha, post_scale=w.post_scale, clamp_lo=w.clamp_lo, clamp_hi=w.clamp_hi, eps=w.eps,
              gamma=t["gamma"], beta=t["beta"], aux_out=aux)
    if args.evolve:
        best, ms, seen = evolve_library(X, t["W"], t["b"], w.act, w.norm, out, **kw)
        print(f"{name}: {len(seen)} configurations evaluated by the island search")
        for c, r in sorted(seen.items(), key=lambda e: e[1]["ms"]):
            print(f"  {r['ms']:9.4f} ms  {'ok ' if r['accepted'] else 'REJ'} dev {r['deviation']:.1e}  {str(c):40s} {r['kernel']}")
        print(f"  best: {best} at {ms:.4f} ms")
        return 0
    table = tune(X, t["W"], t["b"], w.act, w.norm, out, **kw)
    print(f"{name}: {len(table)} configurations")
    for r in table:
        print(f"  {r['ms']:9.4f} ms  {'ok ' if r['accepted'] else 'REJ'} dev {r['deviation']:.1e}  "
              f"{r['label']:24s} {r['kernel']}{' (automatic choice)' if r['auto'] else ''}")
    return 0


if __name__ == "__main__":
    sys.exit(main(sys.argv))
