"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function
the header declares, and rejects bad arguments with the documented status before any launch."""
import ctypes
import os
import re

import pytest

from paper_2512_23424_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = open(os.path.join(ROOT, "include", "fge.h")).read()


def declared_functions():
    body = re.sub(r"/\*.*?\*/", "", HEADER, flags=re.S)
    return sorted(set(re.findall(r"\b(\w+)\s*\([^;{}]*\)\s*;", body)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert {"fused_gemm_epilogue", "unfused_gemm_epilogue", "fge_workspace_bytes", "fge_fused_tiles",
            "fge_fused_finish", "fge_gemm_bias", "fge_activation", "fge_row_op",
            "fge_status_string", "fge_last_hip_error", "fge_tile_name",
            "fge_fused_needs_finish", "fge_fused_k_slices"} <= set(names)
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n


def test_struct_layout_matches_header():
    assert ctypes.sizeof(B.FgeParams) == 128
    assert B.FgeParams.ldx.offset == 16 and B.FgeParams.in_dtype.offset == 56
    assert B.FgeParams.gamma.offset == 88 and B.FgeParams.workspace_bytes.offset == 120


def _params(**kw):
    p = B.FgeParams()
    p.M, p.N, p.K, p.batch = 128, 256, 64, 1
    p.ldx, p.ldw, p.ldo = 64, 64, 256
    p.in_dtype = p.out_dtype = 0
    p.alpha = p.post_scale = 1.0
    for k, v in kw.items():
        setattr(p, k, v)
    return p


FAKE = 0x10000          # 16-byte aligned non-null address; never dereferenced on these paths


def _call(p, act=1, norm=1, X=FAKE, W=FAKE, out=FAKE, b=None):
    return B.lib().fused_gemm_epilogue(X, W, b, act, norm, ctypes.byref(p), out, None)


def test_argument_errors_are_reported_before_any_launch():
    assert B.lib().fused_gemm_epilogue(FAKE, FAKE, None, 1, 1, None, FAKE, None) == 1      # NULL params
    assert _call(_params(), X=None) == 1
    assert _call(_params(), out=None) == 1
    assert _call(_params(), act=6) == 2 and _call(_params(), act=-1) == 2
    assert _call(_params(), norm=5) == 2
    assert _call(_params(in_dtype=4)) == 2 and _call(_params(out_dtype=-1)) == 2
    assert _call(_params(in_dtype=3, out_dtype=3)) == 4       # E4M3 is an operand type only
    assert _call(_params(in_dtype=3, out_dtype=2)) == 4       # ... that goes with fp32 or bf16 results
    assert _call(_params(in_dtype=2, out_dtype=1)) == 4       # fp16 operands with a bf16 result
    assert _call(_params(in_dtype=1, out_dtype=2)) == 4
    assert _call(_params(M=0)) == 3 and _call(_params(K=-8)) == 3 and _call(_params(batch=0)) == 3
    assert _call(_params(ldo=128)) == 3                       # stride smaller than the row
    assert _call(_params(ldx=32)) == 3
    assert _call(_params(), X=FAKE + 4) == 5                  # misaligned base pointer
    # extents / strides that are not multiples of 16 bytes are valid: they take the element-granular kernels, which need a workspace for
    # the fp32 intermediate of a row op (so these calls stop at the missing workspace)
    for q in (_params(N=250, ldo=250), _params(K=62, ldx=64, ldw=64), _params(ldo=258)):
        assert B.fge_tile_name(True, 1, 1, q) == "generic32x32_scalar"
        assert B.lib().fge_workspace_bytes(1, 1, 1, ctypes.byref(q)) == q.M * q.N * 4
        assert B.fge_fused_needs_finish(1, 1, q) is False
        assert _call(q) == 6
    assert B.lib().fge_workspace_bytes(1, 1, 0, ctypes.byref(_params(N=250, ldo=250))) == 0
    # the fused tile kernels split rows of any width over column tiles (the row kernels on their
    # own stop at 8192 columns); only beyond 8192 column strips per row the generic kernels take over
    wide = _params(N=16384, ldo=16384)
    assert B.fge_tile_name(True, 1, 1, wide) == "64x64_w2x2_splitbf16" and B.fge_fused_needs_finish(1, 1, wide)
    assert B.lib().fge_workspace_bytes(1, 1, 1, ctypes.byref(wide)) == 128 * (256 * 2) * 8 and _call(wide) == 6
    assert B.fge_tile_name(True, 1, 1, _params(N=1 << 21, ldo=1 << 21)) == "generic32x32_scalar"
    assert _call(_params(), norm=4) == 1                      # logsumexp without aux_out
    # split rows need a workspace
    p = _params(M=4096, N=1024, K=1024, ldx=1024, ldw=1024, ldo=1024)
    need = B.lib().fge_workspace_bytes(1, 2, 2, ctypes.byref(p))
    # enough for both forms of split rows.  One-kernel form: a pair per (row, column tile), an
    # arrival mark per tile, a flag line; two-pass form: 8 column tiles x 4 waves across (one
    # 128x128 tile per CU: the eight-wave form) = 32 strips per row
    assert B.fge_tile_name(True, 2, 2, p) == "128x128_w2x4_splitbf16"
    assert 4096 * 8 * 8 + 64 * 8 * 4 + 256 < need == 4096 * (8 * 4) * 8
    p.flags = B.FLAG_TWO_PASS
    assert B.lib().fge_workspace_bytes(1, 2, 2, ctypes.byref(p)) == 4096 * (8 * 4) * 8
    p.flags = 0x10
    assert _call(p, act=2, norm=2) == 2        # unknown flag bit
    p.flags = 0
    assert _call(p, act=2, norm=2) == 6
    p.workspace, p.workspace_bytes = FAKE, need - 1
    assert _call(p, act=2, norm=2) == 6
    # unfused path: workspace for two intermediates
    assert B.lib().fge_workspace_bytes(0, 2, 2, ctypes.byref(p)) == 2 * 4096 * 1024 * 4
    assert B.lib().unfused_gemm_epilogue(FAKE, FAKE, None, 2, 2, ctypes.byref(p), FAKE, None) == 6
    assert B.lib().fge_workspace_bytes(1, 9, 2, ctypes.byref(p)) == ctypes.c_size_t(-1).value


def test_status_strings_and_tile_names():
    L = B.lib()
    seen = {L.fge_status_string(i) for i in range(8)}
    assert len(seen) == 8 and all(seen)
    assert L.fge_status_string(99) == b"unknown status"
    assert L.fge_last_hip_error() == 0
    # fp32 operands run the split-bf16 product unless the caller asks for the fp32 instruction
    assert B.fge_tile_name(True, 1, 1, _params(N=64, ldo=64)) == "64x64_w2x2_splitbf16"
    assert B.fge_tile_name(True, 1, 1, _params(N=64, ldo=64, flags=B.FLAG_IEEE_FP32)) == "64x64_w2x2"
    assert B.fge_tile_name(True, 5, 4, _params(M=262144, N=512, ldo=512, flags=B.FLAG_IEEE_FP32)) == "64x128_w2x2"
    assert B.fge_tile_name(True, 5, 4, _params(M=262144, N=512, ldo=512)) == "panel64x512_w1x8_splitbf16"
    assert B.fge_tile_name(True, 5, 4, _params(M=1000, N=512, ldo=512)) == "64x64_w2x2_splitbf16"     # few tiles
    assert B.fge_tile_name(True, 5, 4, _params(M=262144, N=256, ldo=256)) == "128x128_w2x2_splitbf16"  # row too narrow for it
    assert B.fge_tile_name(True, 5, 4, _params(M=8192, N=256, ldo=256)) == "64x64_w2x2_splitbf16"      # fewer 128x128 tiles than CUs
    huge = _params(M=4096, N=4096, K=4096, ldx=4096, ldw=4096, ldo=4096)
    assert B.fge_tile_name(True, 2, 2, huge) == "128x128_w2x2_splitbf16"
    huge.flags = B.FLAG_IEEE_FP32
    assert B.fge_tile_name(True, 2, 2, huge) == "64x512_w1x4"
    big = _params(M=8192, N=4096, K=4096, ldx=4096, ldw=4096, ldo=4096, in_dtype=1, out_dtype=1)
    assert B.fge_tile_name(True, 4, 3, big) == "256x256_w2x4"
    # the one-call entry point lets the tiles of this problem finish their rows themselves (it has a
    # fault word); the stage entry points always take two passes, whatever the flags
    assert B.fge_fault_word_offset(4, 3, big) is not None
    assert B.fge_fused_needs_finish(4, 3, big) is True
    big.flags = B.FLAG_TWO_PASS
    assert B.fge_fault_word_offset(4, 3, big) is None
    assert B.fge_fused_needs_finish(4, 3, big) is True
    small = _params(M=300, N=1024, K=256, ldx=256, ldw=256, ldo=1024)
    assert B.fge_fused_needs_finish(2, 2, small) is True     # small problems keep the second pass
    assert B.fge_fused_needs_finish(1, 1, _params(N=64, ldo=64)) is False
    with pytest.raises(B.FgeError):
        B.fge_fused_needs_finish(1, 1, _params(M=0))


def test_forced_tile_configurations():
    """FGE_FLAG_TILE picks the tile configuration; one without kernels for the operand type is
    refused before anything is launched."""
    def tile(t):
        return (t + 1) << 8
    f32 = dict(M=512, N=1024, K=256, ldx=256, ldw=256, ldo=1024)
    assert B.fge_tile_name(True, 2, 2, _params(**f32, flags=tile(0))) == "64x64_w2x2_splitbf16"
    assert B.fge_tile_name(True, 2, 2, _params(**f32, flags=tile(1))) == "64x512_w1x4_splitbf16"
    assert B.fge_tile_name(True, 2, 2, _params(**f32, flags=tile(5) | B.FLAG_IEEE_FP32)) == "64x128_w2x2"
    assert B.fge_tile_name(True, 2, 2, _params(**f32, flags=tile(2))) == "128x128_w2x2_splitbf16"
    assert _call(_params(**f32, flags=tile(2) | B.FLAG_IEEE_FP32)) == 4   # 128x128 with fp32 operands: split product only
    assert _call(_params(**f32, flags=tile(3))) == 4           # 256x256: 16-bit and 8-bit operands only
    assert _call(_params(**f32, flags=tile(4))) == 4           # narrow-K kernel needs K <= 64, N <= 512
    assert _call(_params(**f32, flags=tile(6))) == 4 and _call(_params(**f32, flags=tile(14))) == 4
    b16 = dict(f32, in_dtype=1, out_dtype=1)
    assert B.fge_tile_name(True, 2, 2, _params(**b16, flags=tile(3))) == "256x256_w2x4"
    assert B.fge_tile_name(True, 2, 2, _params(**b16, flags=tile(2))) == "128x128_w2x4_s3"    # 32 tiles, at most one per CU: eight waves, three stage buffers
    big16 = dict(b16, M=8192)
    assert B.fge_tile_name(True, 2, 2, _params(**big16, flags=tile(2))) == "128x128_w2x2"      # 512 tiles: two four-wave workgroups per CU
    assert B.fge_tile_name(True, 2, 2, _params(**big16, flags=tile(10))) == "128x128_w2x4_s3"
    assert _call(_params(**b16, flags=tile(5))) == 4           # 64x128: fp32 operands only
    nk = _params(M=100, N=328, K=40, ldx=40, ldw=40, ldo=328, flags=tile(4))
    assert B.fge_tile_name(True, 5, 4, nk) == "panel64x512_w1x8_splitbf16"
    # a forced tile changes the split-row bookkeeping accordingly
    p = _params(**b16, flags=tile(0))
    assert B.lib().fge_workspace_bytes(1, 2, 2, ctypes.byref(p)) == 512 * (16 * 2) * 8


def test_k_split_planning():
    """Few tiles and a long K: the one-call fused entry point cuts K into slices, and the workspace
    query asks for the partial products (plus the fp32 rows a row op reads)."""
    def prm(M, N, K, dt=1, **kw):
        return _params(M=M, N=N, K=K, ldx=K, ldw=K, ldo=N, in_dtype=dt, out_dtype=dt, **kw)
    p = prm(64, 4096, 4096)                       # 64 tiles of 64x64: 8 slices fill 512 workgroup slots
    assert B.fge_fused_k_slices(4, 3, p) == 8
    one = 64 * 4096 * 4
    assert B.lib().fge_workspace_bytes(1, 4, 3, ctypes.byref(p)) == 9 * one      # 8 partial products + the fp32 rows the row op reads
    assert B.lib().fge_workspace_bytes(1, 4, 0, ctypes.byref(p)) == 8 * one
    assert B.fge_fused_needs_finish(4, 3, p) is True                             # the stage entry points never slice
    p.flags = B.FLAG_NO_SPLIT_K
    assert B.fge_fused_k_slices(4, 3, p) == 1
    assert B.lib().fge_workspace_bytes(1, 4, 0, ctypes.byref(p)) == 0
    assert B.fge_fused_k_slices(4, 3, prm(256, 1024, 8192)) == 8                 # 64 tiles; 16 slices would pass two per CU
    assert B.fge_fused_k_slices(4, 3, prm(16, 1024, 8192)) == 16                 # 16 tiles, slices of 512
    assert B.fge_fused_k_slices(4, 3, prm(64, 4096, 2048)) == 1                  # K too short to pay ...
    assert B.fge_fused_k_slices(4, 3, prm(64, 4096, 2048, dt=0)) == 4            # ... but not for the split product
    assert B.fge_fused_k_slices(4, 3, prm(256, 4096, 4096)) == 1                 # 256 tiles: only from K = 8192 on
    assert B.fge_fused_k_slices(4, 3, prm(256, 4096, 8192)) == 2
    assert B.fge_fused_k_slices(4, 3, prm(64, 4096, 4096 + 64)) == 1             # slices would not be whole K tiles
    assert B.fge_fused_k_slices(4, 3, prm(1024, 4096, 4096)) == 1                # enough tiles as it is
    assert B.fge_fused_k_slices(4, 3, prm(64, 4096, 4096, dt=0)) == 8            # fp32 operands too
    assert B.fge_fused_k_slices(4, 3, prm(61, 4090, 4096, dt=0)) == 1            # odd extents: element-granular kernels
    with pytest.raises(B.FgeError):
        B.fge_fused_k_slices(1, 1, _params(M=0))


def test_gated_small_problem_planning():
    """A handful of gated tiles and a long K: fp32 partial products of both GEMMs, then the gate."""
    def prm(M, N, K):
        return _params(M=M, N=N, K=K, ldx=K, ldw=K, ldo=N, in_dtype=1, out_dtype=1)
    L = B.lib()
    p = prm(16, 4096, 4096)
    assert L.fge_gated_tile_name(4, 3, ctypes.byref(p)) == b"partial_products_then_gate"
    one = 16 * 4096 * 4
    assert L.fge_gated_workspace_bytes(1, 4, 3, ctypes.byref(p)) == (2 * 8 + 1) * one    # 8 slices per product + fp32 rows
    assert L.fge_gated_workspace_bytes(1, 4, 0, ctypes.byref(p)) == 2 * 8 * one
    assert L.fge_gated_tile_name(4, 3, ctypes.byref(prm(16, 4096, 512))) == b"gated256x128_w2x4"      # short K
    assert L.fge_gated_tile_name(4, 3, ctypes.byref(prm(2048, 4096, 4096))) == b"gated256x128_w2x4"   # 256 gated tiles
    assert L.fge_gated_tile_name(4, 0, ctypes.byref(prm(256, 11008, 4096))) == b"gated256x128_w2x4"   # too many 64x64 tiles
    q = prm(300, 520, 1152)                                                                           # not worth slicing
    assert L.fge_gated_tile_name(4, 3, ctypes.byref(q)) == b"partial_products_then_gate"
    assert L.fge_gated_workspace_bytes(1, 4, 3, ctypes.byref(q)) == 3 * ((300 * 520 * 4 + 255) // 256 * 256)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    """fused_gemm_epilogue_static checks its arguments, and the problem against the size of the
    library's scratch array, before the device is touched."""
    L = B.lib()
    assert L.fge_static_scratch_bytes() == 16 << 20
    fn = L.fused_gemm_epilogue_static
    assert fn(FAKE, FAKE, None, 1, 1, None, FAKE, None) == 1
    assert fn(FAKE, FAKE, None, 9, 1, ctypes.byref(_params()), FAKE, None) == 2
    assert fn(FAKE + 4, FAKE, None, 1, 1, ctypes.byref(_params()), FAKE, None) == 5
    # statistics of 65536 rows x 16 column tiles x 4 strips in the two-pass form: 32 MiB
    big = _params(M=65536, N=4096, K=64, ldx=64, ldw=64, ldo=4096, in_dtype=1, out_dtype=1, flags=B.FLAG_TWO_PASS)
    assert L.fge_workspace_bytes(1, 4, 3, ctypes.byref(big)) == 65536 * 64 * 8
    assert fn(FAKE, FAKE, None, 4, 3, ctypes.byref(big), FAKE, None) == 6
    # element-granular kernels: the fp32 intermediate of 3000 x 3001 rows does not fit either
    odd = _params(M=3000, N=3001, K=17, ldx=17, ldw=17, ldo=3001)
    assert fn(FAKE, FAKE, None, 1, 1, ctypes.byref(odd), FAKE, None) == 6


def test_tile_choice_reads_the_search_table_and_respects_its_limits():
    """16-bit operands: at a sweep point where the configuration search's find beat the rule, the
    choice is the table's entry - unless the caller asks for the rule alone, the problem needs
    another number of rounds of the chip than the entry's shape did (same tile, a few more rows), or
    few tiles and a long K call for the K slices."""
    import re
    def prm(M, N, K, **kw):
        return _params(M=M, N=N, K=K, ldx=K, ldw=K, ldo=N, in_dtype=1, out_dtype=1, **kw)
    names = {0: "64x64_w2x2", 1: "64x512_w1x4", 2: "128x128_w2x2", 3: "256x256_w2x4", 7: "128x256_w2x4", 8: "256x128_w4x2"}
    table = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2512_23424_amd", "csrc", "fge_tile_table.h")
    finds = 0
    for line in open(table):
        m = re.match(r"\s*\{0, 1, (\d+), (\d+), (\d+), (\d+), 0\},.*\(rule", line)      # 16-bit, row op, one-kernel form, a confirmed find
        if not m:
            continue
        mt, nt, K, tile = (int(v) for v in m.groups())
        if mt * nt < 64:             # (small problems: the K slices have a rule of their own)
            continue
        p = prm(mt * 256, nt * 256, K)
        assert B.fge_tile_name(True, 4, 3, p) == names[tile], line
        assert B.fge_tile_name(True, 4, 3, prm(mt * 256, nt * 256, K, flags=B.FLAG_NO_TABLE)) != names[tile], line
        finds += 1
    assert finds >= 5
    # same neighbourhood of the table, another number of rounds: the rule decides
    assert B.fge_tile_name(True, 4, 3, prm(6144, 4096, 4096)) == "128x256_w2x4"
    assert B.fge_tile_name(True, 4, 3, prm(6400, 4096, 4096)) == B.fge_tile_name(True, 4, 3, prm(6400, 4096, 4096, flags=B.FLAG_NO_TABLE)) == "256x256_w2x4"
    assert B.fge_tile_name(True, 4, 3, prm(64, 4096, 4096)) == "64x64_w2x2" and B.fge_fused_k_slices(4, 3, prm(64, 4096, 4096)) == 8
    # fp32 operands are not in the table
    f32 = _params(M=2048, N=4096, K=4096, ldx=4096, ldw=4096, ldo=4096)
    assert B.fge_tile_name(True, 4, 3, f32) == B.fge_tile_name(True, 4, 3, _params(M=2048, N=4096, K=4096, ldx=4096, ldw=4096, ldo=4096, flags=B.FLAG_NO_TABLE))


def test_rows_far_apart_leave_the_tile_kernels():
    """The tile kernels address an operand row by a 32-bit byte offset from its tile's first row:
    rows of X or W 8 MiB apart or more are repacked (large problems) or go to the element-granular
    kernels (small ones); just below the limit the tile kernels still take them."""
    def name(M, ld):
        return B.fge_tile_name(True, 4, 3, _params(M=M, N=1024 if M > 64 else 64, K=1024 if M > 64 else 64, ldx=ld,
                                                   ldw=1024 if M > 64 else 64, ldo=1024 if M > 64 else 64, in_dtype=1, out_dtype=1))
    assert name(512, (8 << 20) // 2 - 8) == "64x64_w2x2"
    assert name(512, (8 << 20) // 2) == "repacked_operands"
    assert name(64, (8 << 20) // 2) == "generic32x32_scalar"

