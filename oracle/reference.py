"""NumPy front end of the plain-C oracle (``mrfp4_oracle.c``).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in the C file, written from the paper (arXiv 2509.23202, Sections 2, 3, 4.1,
4.2 and the proof of Lemma 1) and the OCP Microscaling rules; this module only compiles it with gcc,
loads it with ctypes and marshals NumPy arrays.  It shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "mrfp4_oracle.c"
_LIB = _HERE / "libmrfp4_oracle.so"

MXFP4 = 0
NVFP4 = 1
GROUP = {MXFP4: 32, NVFP4: 16}


def build(force: bool = False) -> Path:
    """Compile the C oracle (gcc, -O2, no contraction, no fast-math, OpenMP)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(".so.tmp%d" % os.getpid())
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared",
               "-fPIC", "-Wall", "-Wextra", "-o", str(tmp), str(_SRC), "-lm"]
        subprocess.run(cmd, check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(str(_LIB))
        i64, p, i32, dbl, u8 = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_uint8
        L.orc_max_threads.restype = i32
        L.orc_set_threads.argtypes = [i32]
        L.orc_hadamard.argtypes = [i32, p]
        L.orc_hadamard.restype = i32
        L.orc_rotate.argtypes = [p, i64, i64, i32, p]
        L.orc_rotate.restype = i32
        L.orc_rotate_dense.argtypes = [p, i64, i64, i32, p, p]
        L.orc_rotate_dense.restype = i32
        L.orc_rotate_f64.argtypes = [p, i64, i64, i32, p]
        L.orc_rotate_f64.restype = i32
        L.orc_e2m1_decode.argtypes = [u8]
        L.orc_e2m1_decode.restype = dbl
        L.orc_e2m1_encode.argtypes = [dbl]
        L.orc_e2m1_encode.restype = u8
        L.orc_e8m0_decode.argtypes = [u8]
        L.orc_e8m0_decode.restype = dbl
        L.orc_e8m0_from_amax.argtypes = [dbl]
        L.orc_e8m0_from_amax.restype = u8
        L.orc_e4m3_decode.argtypes = [u8]
        L.orc_e4m3_decode.restype = dbl
        L.orc_e4m3_encode.argtypes = [dbl]
        L.orc_e4m3_encode.restype = u8
        L.orc_quantize_mxfp4.argtypes = [p, i64, i64, p, p]
        L.orc_quantize_mxfp4.restype = i32
        L.orc_quantize_nvfp4.argtypes = [p, i64, i64, p, p, p, p]
        L.orc_quantize_nvfp4.restype = i32
        L.orc_quantize_mxfp4_mse.argtypes = [p, i64, i64, p, p]
        L.orc_quantize_mxfp4_mse.restype = i32
        L.orc_quantize_nvfp4_mse.argtypes = [p, i64, i64, p, p, p, p]
        L.orc_quantize_nvfp4_mse.restype = i32
        L.orc_quantize_nvfp4_mse_alt.argtypes = [p, i64, i64, i32, p, p, p, p]
        L.orc_quantize_nvfp4_mse_alt.restype = i32
        L.orc_quantize_mxfp4_round43.argtypes = [p, i64, i64, p, p]
        L.orc_quantize_mxfp4_round43.restype = i32
        L.orc_e8m0_round43_from_amax.argtypes = [ctypes.c_double]
        L.orc_e8m0_round43_from_amax.restype = ctypes.c_uint8
        L.orc_quantize_mxfp4_fit.argtypes = [p, i64, i64, p, p, p, p, p]
        L.orc_quantize_mxfp4_fit.restype = i32
        L.orc_quantize_given_scales.argtypes = [p, i64, i64, p, p, p]
        L.orc_quantize_given_scales.restype = i32
        L.orc_dequantize_table.argtypes = [p, p, p, i64, i64, p]
        L.orc_dequantize_table.restype = i32
        L.orc_dequantize.argtypes = [p, p, dbl, i32, i64, i64, p]
        L.orc_dequantize.restype = i32
        L.orc_matmul.argtypes = [p, p, i64, i64, i64, p, p]
        L.orc_matmul.restype = None
        _lib = L
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def max_threads() -> int:
    return int(_load().orc_max_threads())


def set_threads(n: int) -> None:
    _load().orc_set_threads(int(n))


# ---------------------------------------------------------------- scalar codecs
def e2m1_decode(code: int) -> float:
    return float(_load().orc_e2m1_decode(int(code) & 0xFF))


def e2m1_encode(v: float) -> int:
    return int(_load().orc_e2m1_encode(float(v)))


def e8m0_decode(byte: int) -> float:
    return float(_load().orc_e8m0_decode(int(byte)))


def e8m0_from_amax(amax: float) -> int:
    return int(_load().orc_e8m0_from_amax(float(amax)))


def e8m0_round43_from_amax(amax: float) -> int:
    return int(_load().orc_e8m0_round43_from_amax(float(amax)))


def e4m3_decode(byte: int) -> float:
    return float(_load().orc_e4m3_decode(int(byte)))


def e4m3_encode(t: float) -> int:
    return int(_load().orc_e4m3_encode(float(t)))


# ---------------------------------------------------------------- arrays
def hadamard(b: int) -> np.ndarray:
    H = np.zeros((b, b), dtype=np.int8)
    if _load().orc_hadamard(int(b), _ptr(H)) != 0:
        raise ValueError(f"hadamard: b={b} is not a power of two in [1,1024]")
    return H


def rotate(x_bf16_bits: np.ndarray, b: int) -> np.ndarray:
    """x: uint16 bf16 bit patterns [M,K] -> fp32 [M,K] = x @ blockdiag(H_b/sqrt(b))."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    M, K = x.shape
    y = np.empty((M, K), dtype=np.float32)
    if _load().orc_rotate(_ptr(x), M, K, int(b), _ptr(y)) != 0:
        raise ValueError(f"rotate: bad b={b} for K={K}")
    return y


def rotate_dense(x_bf16_bits: np.ndarray, rot_bf16_bits: np.ndarray) -> np.ndarray:
    """x: uint16 bf16 bit patterns [M,K], rot: uint16 bf16 bit patterns [b,b] -> fp32 [M,K] = x @ blockdiag(rot)."""
    x = np.ascontiguousarray(x_bf16_bits, dtype=np.uint16)
    R = np.ascontiguousarray(rot_bf16_bits, dtype=np.uint16)
    M, K = x.shape
    b = R.shape[0]
    if R.shape != (b, b):
        raise ValueError("rot must be square")
    y = np.empty((M, K), dtype=np.float32)
    if _load().orc_rotate_dense(_ptr(x), M, K, int(b), _ptr(R), _ptr(y)) != 0:
        raise ValueError(f"rotate_dense: bad b={b} for K={K}")
    return y


def rotate_f64(x: np.ndarray, b: int) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float64)
    M, K = x.shape
    y = np.empty((M, K), dtype=np.float64)
    if _load().orc_rotate_f64(_ptr(x), M, K, int(b), _ptr(y)) != 0:
        raise ValueError(f"rotate_f64: bad b={b} for K={K}")
    return y


def quantize(y_f32: np.ndarray, fmt: int, tensor_scale: float | None = None, policy: str = "absmax"):
    """fp32 [M,K] -> (codes u8 [M,K/2], scales u8 [M,K/G], s_T float32 scalar or None).
    policy: "absmax" (abs-max group scales), "mse" (group scale code chosen among the abs-max code and its two
    neighbours to minimise the group's squared error) or, MXFP4 only, "round43" (exponent round(log2(amax/6)), scale
    (4/3) 2^k; the returned s_T is then the tensor-level factor 4/3 in binary32)."""
    if policy not in ("absmax", "mse", "round43") or (policy == "round43" and fmt != MXFP4):
        raise ValueError(policy)
    y = np.ascontiguousarray(y_f32, dtype=np.float32)
    M, K = y.shape
    G = GROUP[fmt]
    if K % G:
        raise ValueError(f"quantize: K={K} not a multiple of {G}")
    codes = np.empty((M, K // 2), dtype=np.uint8)
    scales = np.empty((M, K // G), dtype=np.uint8)
    if fmt == MXFP4:
        fn = {"absmax": _load().orc_quantize_mxfp4, "mse": _load().orc_quantize_mxfp4_mse,
              "round43": _load().orc_quantize_mxfp4_round43}[policy]
        rc = fn(_ptr(y), M, K, _ptr(codes), _ptr(scales))
        s_T = np.float32(4.0 / 3.0) if policy == "round43" else None
    else:
        s_out = np.zeros(1, dtype=np.float32)
        s_in = None
        if tensor_scale is not None:
            s_in_arr = np.array([tensor_scale], dtype=np.float32)
            s_in = _ptr(s_in_arr)
        fn = _load().orc_quantize_nvfp4 if policy == "absmax" else _load().orc_quantize_nvfp4_mse
        rc = fn(_ptr(y), M, K, s_in, _ptr(codes), _ptr(scales), _ptr(s_out))
        s_T = np.float32(s_out[0])
    if rc != 0:
        raise ValueError("quantize failed")
    return codes, scales, s_T


def quantize_nvfp4_alternating(y_f32: np.ndarray, rounds: int = 3):
    """NVFP4 with the alternating optimisation of group scales and tensor scale (Section 4.1 "Ingredient 1").
    fp32 [M,K] -> (codes, scales, s_T float32, trace float32[rounds + 1] of the tensor scales)."""
    y = np.ascontiguousarray(y_f32, dtype=np.float32)
    M, K = y.shape
    if K % 16:
        raise ValueError(f"quantize: K={K} not a multiple of 16")
    codes = np.empty((M, K // 2), dtype=np.uint8)
    scales = np.empty((M, K // 16), dtype=np.uint8)
    s_out = np.zeros(1, dtype=np.float32)
    trace = np.zeros(rounds + 1, dtype=np.float32)
    if _load().orc_quantize_nvfp4_mse_alt(_ptr(y), M, K, int(rounds), _ptr(codes), _ptr(scales), _ptr(s_out), _ptr(trace)) != 0:
        raise ValueError("quantize failed")
    return codes, scales, np.float32(s_out[0]), trace


def quantize_mxfp4_fit(y_f32: np.ndarray, alpha_beta=None):
    """MXFP4 with the scale byte fitted to the tensor's range of scales (Appendix "MXFP scale fitting", s = 2^(alpha q + beta)).
    fp32 [M,K] -> (codes u8 [M,K/2], q u8 [M,K/32], (alpha, beta) fp64, table fp64[256] of the 256 scale values).
    alpha_beta: use these instead of fitting them (weights and activations of a layer sharing alpha)."""
    y = np.ascontiguousarray(y_f32, dtype=np.float32)
    M, K = y.shape
    if K % 32:
        raise ValueError(f"quantize: K={K} not a multiple of 32")
    codes = np.empty((M, K // 2), dtype=np.uint8)
    q = np.empty((M, K // 32), dtype=np.uint8)
    ab = np.zeros(2, dtype=np.float64)
    table = np.zeros(256, dtype=np.float64)
    ab_in = None
    if alpha_beta is not None:
        ab_arr = np.array(alpha_beta, dtype=np.float64)
        ab_in = _ptr(ab_arr)
    if _load().orc_quantize_mxfp4_fit(_ptr(y), M, K, ab_in, _ptr(codes), _ptr(q), _ptr(ab), _ptr(table)) != 0:
        raise ValueError("quantize failed")
    return codes, q, (float(ab[0]), float(ab[1])), table


def quantize_given_scales(y_f32: np.ndarray, q: np.ndarray, table_f32: np.ndarray) -> np.ndarray:
    """Elements of fp32 [M,K] against given scales (group g: binary32 table_f32[q[g]], binary32 arithmetic) -> codes."""
    y = np.ascontiguousarray(y_f32, dtype=np.float32)
    M, K = y.shape
    qq = np.ascontiguousarray(q, dtype=np.uint8)
    tab = np.ascontiguousarray(table_f32, dtype=np.float32)
    assert qq.size == M * (K // 32) and tab.size == 256
    codes = np.empty((M, K // 2), dtype=np.uint8)
    if _load().orc_quantize_given_scales(_ptr(y), M, K, _ptr(qq), _ptr(tab), _ptr(codes)) != 0:
        raise ValueError("quantize failed")
    return codes


def dequantize_table(codes: np.ndarray, q: np.ndarray, table: np.ndarray) -> np.ndarray:
    """codes [M,K/2], q [M,K/32], table[256] -> fp64 [M,K] = E2M1(code) * table[q]."""
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    qq = np.ascontiguousarray(q, dtype=np.uint8)
    tab = np.ascontiguousarray(table, dtype=np.float64)
    M, K2 = codes.shape
    out = np.empty((M, 2 * K2), dtype=np.float64)
    if _load().orc_dequantize_table(_ptr(codes), _ptr(qq), _ptr(tab), M, 2 * K2, _ptr(out)) != 0:
        raise ValueError("dequantize failed")
    return out


def dequantize(codes: np.ndarray, scales: np.ndarray, fmt: int, s_T=None) -> np.ndarray:
    codes = np.ascontiguousarray(codes, dtype=np.uint8)
    scales = np.ascontiguousarray(scales, dtype=np.uint8)
    M, K2 = codes.shape
    K = 2 * K2
    out = np.empty((M, K), dtype=np.float64)
    st = 1.0 if s_T is None else float(s_T)
    if _load().orc_dequantize(_ptr(codes), _ptr(scales), st, int(fmt), M, K, _ptr(out)) != 0:
        raise ValueError("dequantize failed")
    return out


def round_to_bf16(y_f32: np.ndarray) -> np.ndarray:
    """fp32 -> nearest bf16 (ties to even), returned as fp64 values.  Plain integer arithmetic on the bit patterns."""
    u = np.ascontiguousarray(y_f32, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7fff) + lsb) >> np.uint64(16)) << np.uint64(16)
    return r.astype(np.uint32).view(np.float32).astype(np.float64).reshape(np.shape(y_f32))


def linear_w4a16(x_bf16_bits: np.ndarray, w_bf16_bits: np.ndarray, b: int, fmt: int = MXFP4):
    """Weight-only micro-rotated layer (the paper's appendix on inference regimes): Y = bf16(X H_b) . Q(W H_b)^T with
    the rotated activations rounded to bf16 and only the weights quantized.  Returns (Y, S) like matmul."""
    ya = round_to_bf16(rotate(x_bf16_bits, b))
    wc, ws, wT = quantize(rotate(w_bf16_bits, b), fmt)
    return matmul(ya, dequantize(wc, ws, fmt, wT))


def matmul(A: np.ndarray, W: np.ndarray, want_abs: bool = True):
    """Y = A @ W.T and S = |A| @ |W|.T by plain fp64 loops."""
    A = np.ascontiguousarray(A, dtype=np.float64)
    W = np.ascontiguousarray(W, dtype=np.float64)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    Y = np.empty((M, N), dtype=np.float64)
    S = np.empty((M, N), dtype=np.float64) if want_abs else None
    _load().orc_matmul(_ptr(A), _ptr(W), M, N, K, _ptr(Y), _ptr(S) if want_abs else None)
    return Y, S


def rotate_quantize(x_bf16_bits: np.ndarray, b: int, fmt: int, tensor_scale=None):
    """The whole activation/weight encoding: rotate along K, then quantize."""
    y = rotate(x_bf16_bits, b)
    return quantize(y, fmt, tensor_scale) + (y,)


def linear(x_bits: np.ndarray, w_bits: np.ndarray, b: int, fmt: int):
    """Y = Q(X H_b) Q(W H_b)^T in fp64 plus the tolerance denominator S."""
    ac, asc, aT, _ = rotate_quantize(x_bits, b, fmt)
    wc, wsc, wT, _ = rotate_quantize(w_bits, b, fmt)
    A = dequantize(ac, asc, fmt, aT)
    W = dequantize(wc, wsc, fmt, wT)
    return matmul(A, W)
