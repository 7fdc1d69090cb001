"""Thin ctypes binding of libfp4mr.so: argument marshalling only.

PyTorch supplies device memory (``torch.empty(..., device="cuda")``) and the current HIP stream; every step of
the path runs inside the library's HIP kernels.  There is no CPU fallback: importing this module raises if the
library has not been built (``python -m paper_2509_23202_amd.build``).
"""
from __future__ import annotations

import ctypes
from pathlib import Path

import torch

_LIB_PATH = Path(__file__).resolve().parent / "libfp4mr.so"
if not _LIB_PATH.exists():
    raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2509_23202_amd.build` "
                      "(there is no fallback path)")
lib = ctypes.CDLL(str(_LIB_PATH))

MXFP4, NVFP4 = 0, 1
GROUP = {MXFP4: 32, NVFP4: 16}

LAYOUT_GEMM = 1 << 0
INPUT_F32 = 1 << 1
STATIC_TENSOR_SCALE = 1 << 2
A_LAYOUT_GEMM = 1 << 3
W_LAYOUT_GEMM = 1 << 4
OUT_F32 = 1 << 5
SCALE_MSE = 1 << 6
SCALE_ROUND43 = 1 << 7
SCALE_FIT_TENSOR = 1 << 10
SCALE_FIT_RANGE = 1 << 11
FIT_RANGE_FLOATS = 258
A_SCALE43 = 1 << 8
W_SCALE43 = 1 << 9
OPT_GEMM_VARIANT, OPT_GEMM_GRID, OPT_SW_CODEC = 0, 1, 2
OP_ROTATE_QUANTIZE, OP_QUANTIZE_WEIGHTS, OP_GEMM, OP_GPTQ, OP_GPTQ_PREPARE, OP_GPTQ_HESSIAN, OP_GEMM_SPLIT_K = 0, 1, 2, 3, 4, 5, 6

_p, _i64, _i32, _u32, _sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_uint32, ctypes.c_size_t
_quant_sig = [_p, _i64, _i64, _i32, _i32, _p, _p, _p, _p, _sz, _u32, _p]
lib.fp4_rotate_quantize.argtypes = _quant_sig
lib.fp4_rotate_quantize.restype = _i32
lib.fp4_quantize_weights.argtypes = _quant_sig
lib.fp4_quantize_weights.restype = _i32
lib.fp4_rotate_quantize_static.argtypes = [_p, _i64, _i64, _i32, _i32, _p, _p, _p, _u32, _p]
lib.fp4_rotate_quantize_static.restype = _i32
lib.fp4_rotate_quantize_dense.argtypes = [_p, _i64, _i64, _i32, _p, _i32, _p, _p, _p, _p, _sz, _u32, _p]
lib.fp4_rotate_quantize_dense.restype = _i32
lib.fp4_fused_linear.argtypes = [_p, _i64, _i64, _i32, _p, _p, _i64, _i32, _p, _u32, _p]
lib.fp4_fused_linear.restype = _i32
lib.fp4_w4a16_linear.argtypes = lib.fp4_fused_linear.argtypes
lib.fp4_w4a16_linear.restype = _i32
lib.fp4_gptq_quantize_weights.argtypes = [_p, _i64, _i64, _i32, _i32, _p, _p, _p, _p, _p, _p, _sz, _u32, _p]
lib.fp4_gptq_quantize_weights.restype = _i32
lib.fp4_gptq_accumulate_hessian.argtypes = [_p, _i64, _i64, _i32, _p, _i32, _p, _sz, _p]
lib.fp4_gptq_accumulate_hessian.restype = _i32
lib.fp4_gptq_prepare.argtypes = [_p, _i64, ctypes.c_float, _i32, _p, _p, _p, _sz, _p]
lib.fp4_gptq_prepare.restype = _i32
lib.fp4_gemm.argtypes = [_p, _p, _p, _p, _p, _p, _i64, _i64, _i64, _i32, _p, _p, _sz, _u32, _p]
lib.fp4_gemm.restype = _i32
lib.fp4_workspace_bytes.argtypes = [_i32, _i64, _i64, _i64, _i32, _u32]
lib.fp4_workspace_bytes.restype = _sz
lib.fp4_packed_bytes.argtypes = [_i64, _i64, _i32, _u32, ctypes.POINTER(_sz), ctypes.POINTER(_sz)]
lib.fp4_packed_bytes.restype = _i32
lib.fp4_status_string.argtypes = [_i32]
lib.fp4_status_string.restype = ctypes.c_char_p
lib.fp4_version.restype = _i32
lib.fp4_probe.argtypes = [_i32, _p, _sz, _i32, _p]
lib.fp4_probe.restype = _i32
lib.fp4_dequantize.argtypes = [_p, _p, _p, _i64, _i64, _i32, _p, _u32, _p]
lib.fp4_dequantize.restype = _i32
lib.fp4_set_option.argtypes = [_i32, _i32]
lib.fp4_set_option.restype = _i32


class Fp4mrError(RuntimeError):
    def __init__(self, status: int):
        self.status = status
        super().__init__(f"fp4mr status {status}: {lib.fp4_status_string(status).decode()}")


def _check(status: int) -> None:
    if status != 0:
        raise Fp4mrError(status)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


def packed_bytes(rows: int, K: int, fmt: int, flags: int = 0):
    c, s = _sz(), _sz()
    _check(lib.fp4_packed_bytes(rows, K, fmt, flags, ctypes.byref(c), ctypes.byref(s)))
    return c.value, s.value


def workspace_bytes(op: int, M: int, N: int, K: int, fmt: int, flags: int = 0) -> int:
    return int(lib.fp4_workspace_bytes(op, M, N, K, fmt, flags))


def _quantize(fn, op, x, had_block, fmt, flags, tensor_scale, codes, scales, workspace, rot=None):
    assert x.is_cuda and x.dim() == 2 and x.is_contiguous()
    rows, K = x.shape
    if x.dtype == torch.float32:
        flags |= INPUT_F32
    elif x.dtype != torch.bfloat16:
        raise TypeError("x must be bfloat16 (or float32 with had_block=1)")
    if codes is None or scales is None:
        cb, sb = packed_bytes(rows, K, fmt, flags & LAYOUT_GEMM)
        codes = torch.empty(cb, dtype=torch.uint8, device=x.device)
        scales = torch.empty(sb, dtype=torch.uint8, device=x.device)
    ts = None
    if flags & SCALE_FIT_RANGE:
        # [alpha, beta, 256 scale values]; a caller-supplied tensor (its first two floats set) means: use that alpha, beta
        if tensor_scale is not None:
            assert tensor_scale.is_cuda and tensor_scale.dtype == torch.float32 and tensor_scale.numel() >= FIT_RANGE_FLOATS
            flags |= STATIC_TENSOR_SCALE
            ts = tensor_scale
        else:
            ts = torch.empty(FIT_RANGE_FLOATS, dtype=torch.float32, device=x.device)
    elif fmt == NVFP4:
        if tensor_scale is not None:
            flags |= STATIC_TENSOR_SCALE
            ts = tensor_scale
        else:
            ts = torch.empty(1, dtype=torch.float32, device=x.device)
    need = workspace_bytes(op, rows, 0, K, fmt, flags)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    wsz = 0 if workspace is None else workspace.numel()
    if rot is None:
        _check(fn(x.data_ptr(), rows, K, had_block, fmt, codes.data_ptr(), scales.data_ptr(), _ptr(ts), _ptr(workspace), wsz,
                  flags, _stream()))
    else:
        _check(fn(x.data_ptr(), rows, K, had_block, rot.data_ptr(), fmt, codes.data_ptr(), scales.data_ptr(), _ptr(ts),
                  _ptr(workspace), wsz, flags, _stream()))
    return codes, scales, ts


def fp4_rotate_quantize(x, had_block: int, fmt: int, *, flags: int = 0, tensor_scale=None, codes=None, scales=None,
                        workspace=None):
    """codes, scales, tensor_scale = Q(X H_b).  x: [M,K] bf16 cuda tensor (fp32 allowed with had_block=1).
    With flags=LAYOUT_GEMM the outputs are in the opaque GEMM layout; else canonical flat byte tensors
    (codes [M*K/2], scales [M*K/G])."""
    return _quantize(lib.fp4_rotate_quantize, OP_ROTATE_QUANTIZE, x, had_block, fmt, flags, tensor_scale, codes, scales, workspace)


def fp4_rotate_quantize_static(x, had_block: int, fmt: int, *, flags: int = 0, tensor_scale, codes, scales):
    """fp4_rotate_quantize without a workspace: the library's own static device scratch is used and nothing is allocated,
    here or in the library -- the caller passes every output (tensor_scale: a 1-element float32 cuda tensor for NVFP4,
    written unless flags has STATIC_TENSOR_SCALE; None for MXFP4)."""
    assert x.is_cuda and x.dim() == 2 and x.is_contiguous() and x.dtype == torch.bfloat16
    rows, K = x.shape
    _check(lib.fp4_rotate_quantize_static(x.data_ptr(), rows, K, had_block, fmt, codes.data_ptr(), scales.data_ptr(),
                                          _ptr(tensor_scale), flags, _stream()))
    return codes, scales, tensor_scale


def fp4_rotate_quantize_dense(x, rot, fmt: int, *, flags: int = 0, tensor_scale=None, codes=None, scales=None, workspace=None):
    """codes, scales, tensor_scale = Q(X R), R block-diagonal with the bf16 [k,k] cuda tensor `rot` on the diagonal
    (k in {16,32,64,128}); for weights pass W as x."""
    assert rot.is_cuda and rot.dtype == torch.bfloat16 and rot.dim() == 2 and rot.shape[0] == rot.shape[1] and rot.is_contiguous()
    return _quantize(lib.fp4_rotate_quantize_dense, OP_ROTATE_QUANTIZE, x, int(rot.shape[0]), fmt, flags, tensor_scale, codes,
                     scales, workspace, rot=rot)


def fp4_quantize_weights(w, had_block: int, fmt: int, *, flags: int = 0, tensor_scale=None, codes=None, scales=None,
                         workspace=None):
    """Offline RTN weight preparation, codes, scales, tensor_scale = Q(W H_b).  w: [N,K] bf16 cuda tensor."""
    return _quantize(lib.fp4_quantize_weights, OP_QUANTIZE_WEIGHTS, w, had_block, fmt, flags, tensor_scale, codes, scales, workspace)


def fp4_gptq_accumulate_hessian(x, had_block: int, hessian=None, *, workspace=None):
    """H (+)= (x H_b)^T (x H_b): x bf16 [T,K]; hessian fp32 [K,K] to add to, or None for a fresh one.  Returns hessian."""
    assert x.is_cuda and x.dim() == 2 and x.is_contiguous() and x.dtype == torch.bfloat16
    T, K = x.shape
    acc = hessian is not None
    if not acc:
        hessian = torch.empty((K, K), dtype=torch.float32, device=x.device)
    assert hessian.is_cuda and hessian.dtype == torch.float32 and hessian.is_contiguous() and tuple(hessian.shape) == (K, K)
    need = workspace_bytes(OP_GPTQ_HESSIAN, T, 0, K, MXFP4, 0)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    _check(lib.fp4_gptq_accumulate_hessian(x.data_ptr(), T, K, had_block, hessian.data_ptr(), 1 if acc else 0,
                                           workspace.data_ptr(), workspace.numel(), _stream()))
    return hessian


def fp4_gptq_prepare(hessian, damp: float = 1e-2, act_order: bool = True, *, workspace=None):
    """Hessian fp32 [K,K] -> (perm int32 [K], hinv_u fp32 [K,K]) for fp4_gptq_quantize_weights."""
    assert hessian.is_cuda and hessian.dtype == torch.float32 and hessian.is_contiguous() and hessian.dim() == 2
    K = hessian.shape[0]
    assert hessian.shape[1] == K
    perm = torch.empty(K, dtype=torch.int32, device=hessian.device)
    U = torch.empty((K, K), dtype=torch.float32, device=hessian.device)
    need = workspace_bytes(OP_GPTQ_PREPARE, 0, 0, K, MXFP4, 0)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=hessian.device)
    _check(lib.fp4_gptq_prepare(hessian.data_ptr(), K, float(damp), 1 if act_order else 0, perm.data_ptr(), U.data_ptr(),
                                workspace.data_ptr(), workspace.numel(), _stream()))
    return perm, U


def fp4_gptq_quantize_weights(w, had_block: int, fmt: int, hinv_u, perm=None, *, flags: int = 0, workspace=None):
    """MR-GPTQ sweep: w bf16 [N,K], hinv_u fp32 [K,K] (upper factor of the damped inverse Hessian in visiting order),
    perm int32 [K] or None.  Returns (codes, scales, tensor_scale) in canonical layout."""
    assert w.is_cuda and w.dim() == 2 and w.is_contiguous() and w.dtype == torch.bfloat16
    N, K = w.shape
    assert hinv_u.is_cuda and hinv_u.dtype == torch.float32 and hinv_u.is_contiguous() and tuple(hinv_u.shape) == (K, K)
    if perm is not None:
        assert perm.is_cuda and perm.dtype == torch.int32 and perm.is_contiguous() and perm.numel() == K
    cb, sb = packed_bytes(N, K, fmt, 0)
    codes = torch.empty(cb, dtype=torch.uint8, device=w.device)
    scales = torch.empty(sb, dtype=torch.uint8, device=w.device)
    ts = torch.empty(1, dtype=torch.float32, device=w.device) if fmt == NVFP4 else None
    if flags & SCALE_FIT_RANGE:
        ts = torch.empty(FIT_RANGE_FLOATS, dtype=torch.float32, device=w.device)
    need = workspace_bytes(OP_GPTQ, N, 0, K, fmt, flags)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=w.device)
    _check(lib.fp4_gptq_quantize_weights(w.data_ptr(), N, K, had_block, fmt, hinv_u.data_ptr(), _ptr(perm), codes.data_ptr(),
                                         scales.data_ptr(), _ptr(ts), workspace.data_ptr(), workspace.numel(), flags, _stream()))
    return codes, scales, ts


def fp4_gemm(a_codes, a_scales, a_tensor_scale, w_codes, w_scales, w_tensor_scale, M: int, N: int, K: int, fmt: int, *,
             flags: int = 0, out=None, workspace=None):
    """out[M,N] = Ahat @ What^T (bf16, or fp32 with OUT_F32).  Operand layouts per A_LAYOUT_GEMM / W_LAYOUT_GEMM."""
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32 if flags & OUT_F32 else torch.bfloat16, device=a_codes.device)
    need = workspace_bytes(OP_GEMM_SPLIT_K, M, N, K, fmt, flags)   # (what the call needs plus optional split-K room)
    if need and workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=a_codes.device)
    wsz = 0 if workspace is None else workspace.numel()
    _check(lib.fp4_gemm(a_codes.data_ptr(), a_scales.data_ptr(), _ptr(a_tensor_scale), w_codes.data_ptr(), w_scales.data_ptr(),
                        _ptr(w_tensor_scale), M, N, K, fmt, out.data_ptr(), _ptr(workspace), wsz, flags, _stream()))
    return out


def fp4_fused_linear(x, had_block: int, w_codes, w_scales, N: int, fmt: int = MXFP4, *, flags: int = 0, out=None):
    """out[M,N] = Q(X H_b) @ Q(W H_b)^T in one launch for M <= 4 tokens (MXFP4, W in GEMM layout)."""
    assert x.is_cuda and x.dim() == 2 and x.is_contiguous() and x.dtype == torch.bfloat16
    M, K = x.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32 if flags & OUT_F32 else torch.bfloat16, device=x.device)
    _check(lib.fp4_fused_linear(x.data_ptr(), M, K, had_block, w_codes.data_ptr(), w_scales.data_ptr(), N, fmt, out.data_ptr(),
                                flags | W_LAYOUT_GEMM, _stream()))
    return out


def fp4_w4a16_linear(x, had_block: int, w_codes, w_scales, N: int, fmt: int = MXFP4, *, flags: int = 0, out=None):
    """out[M,N] = bf16(X H_b) @ Q(W H_b)^T: weight-only variant of fp4_fused_linear (M <= 16, MXFP4, W in GEMM layout)."""
    assert x.is_cuda and x.dim() == 2 and x.is_contiguous() and x.dtype == torch.bfloat16
    M, K = x.shape
    if out is None:
        out = torch.empty((M, N), dtype=torch.float32 if flags & OUT_F32 else torch.bfloat16, device=x.device)
    _check(lib.fp4_w4a16_linear(x.data_ptr(), M, K, had_block, w_codes.data_ptr(), w_scales.data_ptr(), N, fmt, out.data_ptr(),
                                flags | W_LAYOUT_GEMM, _stream()))
    return out


PROBE_MFMA_FP4, PROBE_MFMA_F16, PROBE_COPY, PROBE_READ = 0, 1, 2, 3


def fp4_dequantize(codes, scales, tensor_scale, rows: int, K: int, fmt: int, *, flags: int = 0, out=None):
    """xhat [rows, K] = E2M1(code) * scale, bf16 (fp32 with OUT_F32), from canonical or (LAYOUT_GEMM) GEMM-layout operands.
    tensor_scale: the NVFP4 tensor scale, the FIT_RANGE_FLOATS buffer of a SCALE_FIT_RANGE call, else None."""
    assert codes.is_cuda and scales.is_cuda
    if out is None:
        out = torch.empty((rows, K), dtype=torch.float32 if flags & OUT_F32 else torch.bfloat16, device=codes.device)
    _check(lib.fp4_dequantize(codes.data_ptr(), scales.data_ptr(), _ptr(tensor_scale), rows, K, fmt, out.data_ptr(), flags, _stream()))
    return out


def fp4_probe(which: int, buf, iters: int = 1) -> None:
    """Launch one ceiling-measurement kernel on the current stream (see fp4_probe in the header); buf: cuda uint8 tensor."""
    assert buf.is_cuda and buf.is_contiguous()
    _check(lib.fp4_probe(int(which), buf.data_ptr(), buf.numel() * buf.element_size(), int(iters), _stream()))


def set_option(option: int, value: int) -> None:
    """Process-wide tuning / cross-check switch (OPT_GEMM_VARIANT, OPT_GEMM_GRID, OPT_SW_CODEC); 0 restores the default."""
    _check(lib.fp4_set_option(int(option), int(value)))


def version() -> int:
    return int(lib.fp4_version())
