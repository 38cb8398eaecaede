"""Shared plumbing of the GPU parity tests: upload seeded inputs, call the C ABI through the
binding, download, and evaluate the oracle on the same bits."""
from typing import Dict, Optional, Tuple

import numpy as np
import torch

from oracle import compare as C
from oracle import oracle as O
from paper_2512_23424_amd import binding as B
from paper_2512_23424_amd import inputs as I

# max rel err: fp32 / bf16-in fp32-accumulate / fp16-in fp32-accumulate (one fp16 rounding of the
# output is 2^-11 = 4.9e-4; the gate is the paper's float16 threshold)
TOL = {I.F32: 1e-4, I.BF16: 2e-2, I.F16: 4e-3, I.F8E4M3: 2e-2}
# the paper's pass rule (fp32 and float16 values from its setup section, Section 4.1)
TAU = {I.F32: 1e-3, I.BF16: 2e-2, I.F16: 4e-3, I.F8E4M3: 2e-2}


def to_device(a: Optional[np.ndarray]) -> Optional[torch.Tensor]:
    if a is None:
        return None
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint8:                     # 8-bit E4M3 bit patterns
        return torch.from_numpy(a).cuda().view(torch.float8_e4m3fn)
    return torch.from_numpy(a).cuda()


def to_host_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def tdtype(code: int):
    return {I.BF16: torch.bfloat16, I.F16: torch.float16}.get(code, torch.float32)


def oracle_chain(w: I.Workload, t: Dict[str, Optional[np.ndarray]]):
    f = {k: I.as_f64(v) for k, v in t.items()}
    return O.chain(f["X"], f["W"], f["b"], f["gamma"], f["beta"], alpha=w.alpha,
                   post_scale=w.post_scale, act=w.act, clamp_lo=w.clamp_lo, clamp_hi=w.clamp_hi,
                   norm=w.norm, eps=w.eps)


def run_gpu(w: I.Workload, t: Dict[str, Optional[np.ndarray]], path: str = "fused",
            dev: Optional[Dict[str, torch.Tensor]] = None, batched_call: bool = True,
            flags: int = 0, expect_fault: bool = False) -> Tuple[np.ndarray, Optional[np.ndarray]]:
    """One call of the fused or unfused path on freshly NaN-poisoned outputs."""
    d = dev if dev is not None else {k: to_device(v) for k, v in t.items()}
    X = d["X"]
    rows = X.shape[0]
    if w.batch > 1 and batched_call and rows == w.rows:
        X = X.view(w.batch, w.M, w.K)
        out = torch.full((w.batch, w.M, w.N), float("nan"), dtype=tdtype(w.out_dtype), device="cuda")
    else:
        out = torch.full((rows, w.N), float("nan"), dtype=tdtype(w.out_dtype), device="cuda")
    aux = (torch.full((rows,), float("nan"), dtype=torch.float32, device="cuda")
           if w.norm == I.NORM_LOGSUMEXP else None)
    p = B.make_params(X, d["W"], out, alpha=w.alpha, post_scale=w.post_scale, clamp_lo=w.clamp_lo,
                      clamp_hi=w.clamp_hi, eps=w.eps, gamma=d["gamma"], beta=d["beta"], aux_out=aux, flags=flags)
    nbytes = B.fge_workspace_bytes(path == "fused", w.act, w.norm, p)
    # the workspace is told to be exactly the size asked for, with a canary behind it: nothing may
    # be written past the end of what the call was given
    CANARY = 1024
    ws_bytes = (max(nbytes, 16) + 255) // 256 * 256
    raw = torch.full((ws_bytes + CANARY,), 0xA5, dtype=torch.uint8, device="cuda")
    ws = raw[:ws_bytes].view(torch.float32)
    ws.fill_(float("nan"))
    p.workspace, p.workspace_bytes = ws.data_ptr(), nbytes
    fn = B.fused_gemm_epilogue if path == "fused" else B.unfused_gemm_epilogue
    # one-kernel form of split rows: clear the word that reports a wait that ran out, check it after
    off = B.fge_fault_word_offset(w.act, w.norm, p) if path == "fused" else None
    fault = ws.view(torch.int32)[off // 4: off // 4 + 1] if off is not None and off + 4 <= nbytes else None
    if fault is not None:
        fault.zero_()
    fn(X, d["W"], d["b"], w.act, w.norm, p, out)
    torch.cuda.synchronize()
    assert bool((raw[ws_bytes:] == 0xA5).all()), "the call wrote past the end of its workspace"
    if fault is not None and not expect_fault:
        assert int(fault.item()) == 0, "a tile's wait for its row block ran out"
    if expect_fault:
        assert fault is not None and int(fault.item()) == 1, "the fault word was not set"
    o = to_host_f64(out).reshape(rows, w.N)
    return o, None if aux is None else to_host_f64(aux)


def check(w: I.Workload, got, got_aux, ref, ref_aux, label: str = ""):
    assert np.isfinite(got).all(), f"{label}: non-finite output (unwritten or overflow)"
    err = C.max_rel_err(got, ref)
    frac = C.verifier_fraction(got, ref, TAU[w.in_dtype])
    msg = f"{label} {w.name} M={w.rows} K={w.K} N={w.N}: max rel err {err:.3e}, frac>{TAU[w.in_dtype]} = {frac:.3e}"
    print(msg, flush=True)
    assert err <= TOL[w.in_dtype], msg
    assert frac <= TAU[w.in_dtype], msg
    if w.norm == I.NORM_LOGSUMEXP:
        assert np.isfinite(got_aux).all()
        e2 = C.max_rel_err_vec(got_aux, ref_aux)
        print(f"{label} {w.name}: lse max rel err {e2:.3e}", flush=True)
        assert e2 <= TOL[w.in_dtype], f"{label} lse err {e2:.3e}"
    return err
