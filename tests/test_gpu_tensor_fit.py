"""GPU parity for the alternating optimisation of NVFP4 group scales and tensor scale (FP4MR_SCALE_MSE |
FP4MR_SCALE_FIT_TENSOR; Section 4.1 "Ingredient 1") against the CPU oracle.

The tensor scale is a quotient of two fp64 sums; the kernel adds them in another (fixed) order than the oracle, and
its group search evaluates errors in fp32, so a handful of near-tie groups may carry another scale code into the
sums.  The bar: the returned tensor scale within 1e-5 relative of the oracle's (observed: equal or one binary32 step
away), and the returned codes and scales equal to the oracle's squared-error search run WITH the library's tensor scale,
under the rules of tests/test_gpu_mse_policy.py (bit-exact codes where the scale code agrees; scale codes differ only
in verified near-ties).
"""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import NV, to_dev, to_dev_bf16
from tests.test_gpu_mse_policy import check_against_oracle, np_

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


def sq_err(oracle, y, c, s, T):
    return float(((oracle.dequantize(c, s, NV, T) - y.astype(np.float64)) ** 2).sum())


@pytest.mark.parametrize("shape", [(131, 2304), (1, 256), (16, 4096)])
def test_tensor_fit_on_oracle_values(fp4, oracle, shape):
    import torch
    M, K = shape
    rng = np.random.default_rng(900 + M)
    y = (rng.standard_t(3, size=(M, K)) * np.exp(rng.uniform(-1, 1, (M, K)))).astype(np.float32)
    FL = fp4.SCALE_MSE | fp4.SCALE_FIT_TENSOR
    say(f"tensor fit on oracle values {shape}")
    c, s, T = fp4.fp4_rotate_quantize(to_dev(y), 1, NV, flags=FL)
    c1, s1, T1 = fp4.fp4_rotate_quantize(to_dev(y), 1, NV, flags=fp4.SCALE_MSE)
    torch.cuda.synchronize()
    Tg = np.float32(np_(T)[0])
    ref_c, ref_s, ref_T, trace = oracle.quantize_nvfp4_alternating(y, 3)
    ulps = abs(float(Tg) - float(ref_T)) / float(np.spacing(np.float32(ref_T)))
    say(f"   s_T: abs-max {float(np_(T1)[0]):.8g}, library {float(Tg):.8g}, oracle {float(ref_T):.8g} ({ulps:.0f} binary32 steps apart)")
    assert trace[0] == np_(T1)[0]
    assert abs(float(Tg) - float(ref_T)) <= 1e-5 * float(ref_T)
    c = np_(c).reshape(M, -1)
    s = np_(s).reshape(M, -1)
    rc, rs, _ = oracle.quantize(y, NV, tensor_scale=float(Tg), policy="mse")
    check_against_oracle(oracle, y, c, s, NV, float(Tg), rc, rs, exact_codes=True)
    # direction (the point of the procedure): not above the group search with the abs-max tensor scale
    e_fit = sq_err(oracle, y, c, s, float(Tg))
    e_mse = sq_err(oracle, y, np_(c1).reshape(M, -1), np_(s1).reshape(M, -1), float(np_(T1)[0]))
    say(f"   squared error {e_fit / e_mse:.5f} of the abs-max tensor scale's")
    assert e_fit <= e_mse * (1 + 1e-9)


@pytest.mark.parametrize("b", [1, 16, 128])
def test_tensor_fit_of_weights_end_to_end(fp4, oracle, b):
    """The offline use: bf16 weights through fp4_quantize_weights, with and without rotation, both layouts."""
    import torch
    from tests.gpu_util import gemm_layout_to_canonical
    N, K = 192, 2048
    wb = inputs.RECIPES[4].w(N, K, salt=40 + b)
    w = to_dev_bf16(wb)
    FL = fp4.SCALE_MSE | fp4.SCALE_FIT_TENSOR
    say(f"tensor fit of weights b={b}")
    c, s, T = fp4.fp4_quantize_weights(w, b, NV, flags=FL)
    cg, sg, Tgm = fp4.fp4_quantize_weights(w, b, NV, flags=FL | fp4.LAYOUT_GEMM)
    torch.cuda.synchronize()
    Tg = float(np_(T)[0])
    assert np_(Tgm)[0] == np_(T)[0]
    y = oracle.rotate(wb, b)
    _, _, ref_T, _ = oracle.quantize_nvfp4_alternating(y, 3)
    say(f"   s_T library {Tg:.8g}, oracle {float(ref_T):.8g}")
    assert abs(Tg - float(ref_T)) <= 1e-5 * float(ref_T)
    c = np_(c).reshape(N, -1)
    s = np_(s).reshape(N, -1)
    rc, rs, _ = oracle.quantize(y, NV, tensor_scale=Tg, policy="mse")
    check_against_oracle(oracle, y, c, s, NV, Tg, rc, rs, exact_codes=(b == 1), tie_rtol=1e-5 if b == 1 else 1e-3)
    rows = np.arange(N)
    cc, ss = gemm_layout_to_canonical(np_(cg), np_(sg), rows, K, NV)
    assert np.array_equal(cc, c) and np.array_equal(ss, s)


def test_tensor_fit_zero_tensor_and_repeatability(fp4, oracle):
    import torch
    FL = fp4.SCALE_MSE | fp4.SCALE_FIT_TENSOR
    z = torch.zeros((32, 512), dtype=torch.bfloat16, device="cuda")
    say("tensor fit: zero tensor")
    c, s, T = fp4.fp4_quantize_weights(z, 16, NV, flags=FL)
    torch.cuda.synchronize()
    assert float(np_(T)[0]) == 0.0 and not np_(c).any() and not np_(s).any()
    xb = inputs.RECIPES[4].x(300, 1024, salt=9)
    x = to_dev_bf16(xb)
    say("tensor fit: repeatability")
    outs = [fp4.fp4_quantize_weights(x, 16, NV, flags=FL) for _ in range(3)]
    torch.cuda.synchronize()
    for c2, s2, T2 in outs[1:]:
        assert torch.equal(c2, outs[0][0]) and torch.equal(s2, outs[0][1]) and torch.equal(T2, outs[0][2])
