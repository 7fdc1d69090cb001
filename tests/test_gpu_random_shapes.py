"""Seeded random shapes through the whole path (rotate+quantize both operands, GEMM) against the oracle: ragged M and N,
K any multiple of 128, every block size, both formats, both operand layouts, both output types."""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, compare_codes, gemm_layout_to_canonical, to_dev_bf16

pytestmark = pytest.mark.gpu


def say(msg):
    print("[case] " + msg, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def fp4():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2509_23202_amd import binding
    return binding


def np_(t):
    return t.detach().cpu().numpy()


def _cases():
    rng = np.random.default_rng(20250923)
    out = []
    for i in range(16):
        fmt = int(rng.integers(0, 2))
        b = int(rng.choice([1, 16, 32, 64, 128]))
        M = int(rng.choice([1, 3, 16, 17, 47, 64, 65, 130, 257, 300]))
        N = int(rng.choice([8, 24, 136, 256, 264, 520, 1032]))
        K = 128 * int(rng.integers(1, 20))
        out.append((i, fmt, b, M, N, K, bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return out


@pytest.mark.parametrize("case", _cases(), ids=lambda c: f"{c[0]}-fmt{c[1]}-b{c[2]}-M{c[3]}-N{c[4]}-K{c[5]}-{'gemm' if c[6] else 'canon'}-{'f32' if c[7] else 'bf16'}")
def test_random_shape_whole_path(fp4, oracle, case):
    import torch
    i, fmt, b, M, N, K, layout_gemm, out_f32 = case
    r = inputs.RECIPES[1 if fmt == MX else 4]
    xb, wb = r.x(M, K, salt=900 + i), r.w(N, K, salt=900 + i)
    say(f"random shape {case}")
    qflags = fp4.LAYOUT_GEMM if layout_gemm else 0
    qa = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, fmt, flags=qflags)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, fmt, flags=qflags)
    gflags = (fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM if layout_gemm else 0) | (fp4.OUT_F32 if out_f32 else 0)
    out = fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, N, K, fmt, flags=gflags)
    torch.cuda.synchronize()
    if layout_gemm:
        ac, asc = gemm_layout_to_canonical(np_(qa[0]), np_(qa[1]), M, K, fmt)
        wc, wsc = gemm_layout_to_canonical(np_(qw[0]), np_(qw[1]), N, K, fmt)
    else:
        G = 32 if fmt == MX else 16
        ac, asc = np_(qa[0]).reshape(M, K // 2), np_(qa[1]).reshape(M, K // G)
        wc, wsc = np_(qw[0]).reshape(N, K // 2), np_(qw[1]).reshape(N, K // G)
    ya, yw = oracle.rotate(xb, b), oracle.rotate(wb, b)
    aT = wT = None
    if fmt == NV:
        aT, wT = float(np_(qa[2])[0]), float(np_(qw[2])[0])
        for T, y in ((aT, ya), (wT, yw)):
            T_ref = np.float32(np.abs(y).max()) / np.float32(2688.0)
            assert abs(T - float(T_ref)) <= 2 * np.spacing(T_ref)
    rac, rasc, _ = oracle.quantize(ya, fmt, aT)
    rwc, rwsc, _ = oracle.quantize(yw, fmt, wT)
    compare_codes(ac, asc, rac, rasc, ya, fmt, max_frac=max(1e-4, 2.0 / ac.size / 2))
    compare_codes(wc, wsc, rwc, rwsc, yw, fmt, max_frac=max(1e-4, 2.0 / wc.size / 2))
    # the product is checked on the library's own codes (exactly what the GEMM consumed)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, fmt, aT), oracle.dequantize(wc, wsc, fmt, wT))
    got = np_(out.float()).astype(np.float64)
    tol = 1e-3 * S + (0 if out_f32 else np.abs(Y) * 2.0 ** -8)
    assert np.all(np.abs(got - Y) <= tol + 1e-300)
