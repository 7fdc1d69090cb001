"""The C-ABI library loads, exports every symbol the header declares, and validates its arguments on the host
before anything is launched (so these checks need no GPU: every call below is rejected before a launch)."""
import ctypes
import re
from pathlib import Path

import pytest

ROOT = Path(__file__).resolve().parent.parent
LIB = ROOT / "paper_2509_23202_amd" / "libfp4mr.so"
HEADER = ROOT / "include" / "fp4mr.h"


@pytest.fixture(scope="module")
def lib():
    if not LIB.exists():
        from paper_2509_23202_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(str(LIB))


def declared_functions():
    txt = re.sub(r"/\*.*?\*/", "", HEADER.read_text(), flags=re.S)
    return sorted(set(re.findall(r"\b(fp4_[a-z0-9_]+)\s*\(", txt)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert {"fp4_rotate_quantize", "fp4_rotate_quantize_dense", "fp4_fused_linear", "fp4_w4a16_linear", "fp4_quantize_weights", "fp4_gptq_quantize_weights", "fp4_gptq_prepare", "fp4_gptq_accumulate_hessian", "fp4_gemm", "fp4_workspace_bytes",
            "fp4_packed_bytes", "fp4_status_string", "fp4_version", "fp4_set_option", "fp4_rotate_quantize_static"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    lib.fp4_version.restype = ctypes.c_int
    assert lib.fp4_version() >= 100


def test_binding_imports_and_matches_header():
    from paper_2509_23202_amd import binding
    for n in ("fp4_rotate_quantize", "fp4_rotate_quantize_dense", "fp4_quantize_weights", "fp4_gemm"):
        assert callable(getattr(binding, n))
    hdr = HEADER.read_text()
    for name in ("LAYOUT_GEMM", "INPUT_F32", "STATIC_TENSOR_SCALE", "A_LAYOUT_GEMM", "W_LAYOUT_GEMM", "OUT_F32", "SCALE_MSE",
                 "SCALE_ROUND43", "A_SCALE43", "W_SCALE43", "SCALE_FIT_TENSOR", "SCALE_FIT_RANGE"):
        m = re.search(rf"FP4MR_{name}\s*=\s*1u\s*<<\s*(\d+)", hdr)
        assert m and getattr(binding, name) == 1 << int(m.group(1)), name
    m = re.search(r"#define FP4MR_FIT_RANGE_FLOATS\s+(\d+)", hdr)
    assert m and binding.FIT_RANGE_FLOATS == int(m.group(1)) == 2 + 256


def test_sizes(lib):
    from paper_2509_23202_amd import binding as b
    assert b.packed_bytes(64, 4096, b.MXFP4) == (64 * 4096 // 2, 64 * 4096 // 32)        # 4.25 bits / element
    assert b.packed_bytes(64, 4096, b.NVFP4) == (64 * 4096 // 2, 64 * 4096 // 16)        # 4.5 bits / element
    c, s = b.packed_bytes(1, 4096, b.MXFP4, b.LAYOUT_GEMM)                               # rows padded to 16
    assert c == 16 * 4096 // 2 and s == 16 * 4096 // 32
    c, s = b.packed_bytes(17, 640, b.MXFP4, b.LAYOUT_GEMM)                               # K/128 = 5: scales padded to 1024
    assert c == 32 * 640 // 2 and s == 2 * 2 * 256
    assert b.workspace_bytes(b.OP_ROTATE_QUANTIZE, 64, 0, 4096, b.MXFP4) == 0
    assert b.workspace_bytes(b.OP_ROTATE_QUANTIZE, 64, 0, 4096, b.NVFP4) > 0
    assert b.workspace_bytes(b.OP_ROTATE_QUANTIZE, 64, 0, 4096, b.NVFP4, b.STATIC_TENSOR_SCALE) == 0
    # the tensor-scale fit adds two fp64 sums per wave of its reduction pass
    assert (b.workspace_bytes(b.OP_QUANTIZE_WEIGHTS, 64, 0, 4096, b.NVFP4, b.SCALE_MSE | b.SCALE_FIT_TENSOR)
            == b.workspace_bytes(b.OP_QUANTIZE_WEIGHTS, 64, 0, 4096, b.NVFP4, b.SCALE_MSE) + 4096 * 16)
    # the fitted scale range has a range pre-pass (two extremes per wave), unless alpha and beta are given
    assert b.workspace_bytes(b.OP_ROTATE_QUANTIZE, 64, 0, 4096, b.MXFP4, b.SCALE_FIT_RANGE) == 256 + 4096 * 4
    assert b.workspace_bytes(b.OP_ROTATE_QUANTIZE, 64, 0, 4096, b.MXFP4, b.SCALE_FIT_RANGE | b.STATIC_TENSOR_SCALE) == 0
    assert b.workspace_bytes(b.OP_GEMM, 64, 64, 4096, b.MXFP4, b.A_LAYOUT_GEMM | b.W_LAYOUT_GEMM) == 0
    assert b.workspace_bytes(b.OP_GEMM, 64, 64, 4096, b.MXFP4) > 0
    # optional split-K room: the minimum plus whole fp32 copies of the output where few tiles meet a long K, nothing else
    lay = b.A_LAYOUT_GEMM | b.W_LAYOUT_GEMM
    for fmt in (b.MXFP4, b.NVFP4):
        base = b.workspace_bytes(b.OP_GEMM, 128, 4096, 14336, fmt, lay)
        extra = b.workspace_bytes(b.OP_GEMM_SPLIT_K, 128, 4096, 14336, fmt, lay) - base
        assert extra > 0 and extra % (128 * 4096 * 4) <= 255 and 2 <= extra // (128 * 4096 * 4) <= 16
        assert b.workspace_bytes(b.OP_GEMM_SPLIT_K, 4096, 4096, 4096, fmt, lay) == b.workspace_bytes(b.OP_GEMM, 4096, 4096, 4096, fmt, lay)
        assert b.workspace_bytes(b.OP_GEMM_SPLIT_K, 16, 4096, 14336, fmt, lay) == b.workspace_bytes(b.OP_GEMM, 16, 4096, 14336, fmt, lay)
    # shapes that the few-token kernels take beyond 64 tokens need neither the split-K room nor (NVFP4) the fp16 copy of X
    for M, N, K in ((96, 4096, 4096), (256, 4096, 8192), (512, 2048, 4096)):
        assert b.workspace_bytes(b.OP_GEMM_SPLIT_K, M, N, K, b.MXFP4, lay) == 0
    for M, N, K in ((96, 4096, 4096), (256, 2048, 2048), (128, 8192, 1024)):
        assert b.workspace_bytes(b.OP_GEMM_SPLIT_K, M, N, K, b.NVFP4, lay) == 0
    assert b.workspace_bytes(b.OP_GEMM, 128, 16384, 4096, b.NVFP4, lay) >= 128 * 4096 * 2      # the many-token kernel's fp16 X


def test_argument_validation_happens_before_any_launch(lib):
    from paper_2509_23202_amd import binding as b
    L = b.lib
    fake = 0x10000            # non-NULL, 16-byte aligned, never dereferenced: every call below fails validation
    q = lambda **kw: L.fp4_rotate_quantize(kw.get("x", fake), kw.get("M", 4), kw.get("K", 128), kw.get("b", 32), kw.get("fmt", 0),
                                           kw.get("codes", fake), kw.get("scales", fake), kw.get("ts", None), kw.get("ws", None),
                                           kw.get("wsz", 0), kw.get("flags", 0), None)
    assert q(x=None) == 1                       # NULL
    assert q(codes=None) == 1
    assert q(M=0) == 2 and q(K=0) == 2 and q(K=48) == 2          # shape
    assert q(b=64, K=96) == 2                   # K % had_block
    assert q(K=160, flags=b.LAYOUT_GEMM) == 2   # GEMM layout wants K % 128
    assert q(b=8) == 3 and q(b=256) == 3 and q(b=0) == 3         # had_block
    assert q(b=32, flags=b.INPUT_F32) == 3      # fp32 input only without rotation
    assert q(fmt=2) == 4 and q(flags=1 << 9) == 4                # fmt / flags
    assert q(x=fake + 4) == 5 and q(codes=fake + 8) == 5         # alignment
    assert q(fmt=1) == 1                        # NVFP4 needs the tensor-scale pointer
    assert q(fmt=1, ts=fake, ws=fake, wsz=1 << 20, flags=b.SCALE_ROUND43) == 4   # the 4/3 rule is an MXFP4 rule
    assert q(flags=b.SCALE_ROUND43 | b.SCALE_MSE) == 4                           # one scale policy at a time
    FIT = b.SCALE_MSE | b.SCALE_FIT_TENSOR
    assert q(flags=FIT) == 4                                                     # the tensor-scale fit is an NVFP4 policy,
    assert q(fmt=1, ts=fake, ws=fake, wsz=1 << 20, flags=b.SCALE_FIT_TENSOR) == 4     # on top of the group search,
    assert q(fmt=1, ts=fake, ws=fake, wsz=1 << 20, flags=FIT | b.STATIC_TENSOR_SCALE) == 4   # with a fitted, not a given, s_T
    assert q(fmt=1, ts=fake, ws=fake, wsz=256 + 4096 * 4, flags=FIT) == 6        # and needs its larger workspace
    assert q(fmt=1, ts=fake) == 6               # ... and a workspace
    RNG = b.SCALE_FIT_RANGE
    assert q(fmt=1, ts=fake, ws=fake, wsz=1 << 20, flags=RNG) == 4               # the fitted scale range is an MXFP4 format
    assert q(flags=RNG | b.SCALE_MSE, ts=fake) == 4 and q(flags=RNG | b.SCALE_ROUND43, ts=fake) == 4   # and a policy of its own
    assert q(flags=RNG) == 1                                                     # needs the buffer for alpha, beta and the scale values
    assert q(flags=RNG, ts=fake) == 6 and q(flags=RNG, ts=fake, ws=fake, wsz=4096) == 6   # and the range pass's workspace
    assert q(fmt=1, ts=fake, ws=fake, wsz=8) == 6
    g = lambda **kw: L.fp4_gemm(kw.get("a", fake), fake, kw.get("ats", None), fake, fake, None, kw.get("M", 16), kw.get("N", 16),
                                kw.get("K", 128), kw.get("fmt", 0), kw.get("out", fake), kw.get("ws", None), kw.get("wsz", 0),
                                kw.get("flags", b.A_LAYOUT_GEMM | b.W_LAYOUT_GEMM), None)
    assert g(a=None) == 1 and g(out=None) == 1
    assert g(K=64) == 2 and g(M=0) == 2 and g(N=-1) == 2
    assert g(fmt=3) == 4 and g(flags=1 << 12) == 4
    assert g(out=fake + 2) == 5
    assert g(fmt=1) == 1                        # NVFP4 needs both tensor scales
    assert g(fmt=1, ats=fake, flags=b.A_LAYOUT_GEMM | b.W_LAYOUT_GEMM | b.W_SCALE43) in (1, 4)   # (w_ts NULL is caught first)
    assert g(flags=0) == 6                      # canonical operands need the repack workspace
    gq = lambda **kw: L.fp4_gptq_quantize_weights(fake, kw.get("N", 16), kw.get("K", 128), 32, kw.get("fmt", 0), kw.get("U", fake),
                                                  kw.get("perm", None), fake, fake, None, kw.get("ws", fake), kw.get("wsz", 1 << 30),
                                                  kw.get("flags", 0), None)
    assert gq(U=None) == 1 and gq(K=96) == 2 and gq(K=65536) == 2 and gq(flags=b.LAYOUT_GEMM) == 4
    assert gq(U=fake + 4) == 5 and gq(perm=fake + 4) == 5 and gq(ws=None) == 6 and gq(wsz=1024) == 6
    L.fp4_gptq_prepare.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_float, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                   ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    gp = lambda **kw: L.fp4_gptq_prepare(kw.get("H", fake), kw.get("K", 128), kw.get("damp", 0.01), 1, kw.get("perm", fake), kw.get("U", fake),
                                         kw.get("ws", fake), kw.get("wsz", 1 << 30), None)
    assert gp(H=None) == 1 and gp(perm=None) == 1 and gp(K=0) == 2 and gp(K=30000) == 2 and gp(damp=-1.0) == 2
    assert gp(U=fake + 8) == 5 and gp(ws=None) == 6 and gp(wsz=4096) == 6
    gh = lambda **kw: L.fp4_gptq_accumulate_hessian(kw.get("x", fake), kw.get("T", 64), kw.get("K", 128), kw.get("b", 32), kw.get("H", fake), 0,
                                                    kw.get("ws", fake), kw.get("wsz", 1 << 30), None)
    assert gh(x=None) == 1 and gh(H=None) == 1 and gh(T=0) == 2 and gh(K=100) == 2 and gh(b=8) == 3 and gh(ws=None) == 6 and gh(wsz=64) == 6
    assert b.workspace_bytes(b.OP_GPTQ_HESSIAN, 64, 0, 128, b.MXFP4) == 64 * 128 * 4
    assert b.workspace_bytes(b.OP_GPTQ_PREPARE, 0, 0, 256, b.MXFP4) >= 256 * 256 * 10
    assert b.workspace_bytes(b.OP_GPTQ, 128, 0, 256, b.MXFP4) >= 128 * 256 * 5 + 128 * 64 * 4 + 256 * 4
    # the allocation-free variant validates like the ordinary one, and has its own size limit
    qs = lambda **kw: L.fp4_rotate_quantize_static(kw.get("x", fake), kw.get("M", 4), kw.get("K", 128), kw.get("b", 32), kw.get("fmt", 0),
                                                   fake, fake, kw.get("ts", None), kw.get("flags", 0), None)
    assert qs(x=None) == 1 and qs(K=48) == 2 and qs(b=8) == 3 and qs(fmt=2) == 4 and qs(fmt=1) == 1
    assert qs(M=1 << 20, K=1 << 17) == 2        # above FP4MR_STATIC_MAX_ELEMENTS
    # few-token entry points: the quantizing one takes four tokens, the weight-only one sixteen
    fl = lambda fn, M: fn(fake, M, 128, 32, fake, fake, 16, 0, fake, b.W_LAYOUT_GEMM, None)
    assert fl(L.fp4_fused_linear, 5) == 2 and fl(L.fp4_fused_linear, 0) == 2 and fl(L.fp4_w4a16_linear, 17) == 2
    # options: unknown option / value out of range; a forced tile configuration that the format does not have
    assert L.fp4_set_option(99, 1) == 4 and L.fp4_set_option(b.OPT_GEMM_VARIANT, 19) == 4 and L.fp4_set_option(b.OPT_GEMM_GRID, -1) == 4
    assert L.fp4_set_option(b.OPT_GEMM_VARIANT, 9) == 0
    try:
        assert L.fp4_gemm(fake, fake, fake, fake, fake, fake, 16, 16, 128, 1, fake, None, 0, b.A_LAYOUT_GEMM | b.W_LAYOUT_GEMM, None) == 4
    finally:
        assert L.fp4_set_option(b.OPT_GEMM_VARIANT, 0) == 0
    assert L.fp4_status_string(2).decode().startswith("bad shape")
    for s in range(8):
        assert L.fp4_status_string(s)
