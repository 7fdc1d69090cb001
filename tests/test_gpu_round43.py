"""GPU parity for the rounded-exponent scale rule with the 4/3 factor (FP4MR_SCALE_ROUND43, MXFP4 only) against the CPU
oracle: scale bytes and element codes are bit-exact when the kernel is fed the oracle's fp32 values (the exponent
decision is an exact mantissa comparison on both sides, the element rounding is correct rounding on both sides); with
the library's own rotation the end-to-end rule applies, a scale byte being allowed to differ only where the group's
abs-max sits within a few ulp of a decision boundary 6 * 2^(k + 1/2).  The products take the tensor-level 4/3 as a flag.
"""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, gemm_layout_to_canonical, grid_steps, to_dev, to_dev_bf16, unpack

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


def adversarial_rows():
    """Groups with abs-max 8 (exponent 0, scale 4/3) whose other elements are the binary32 neighbours of t / 0.75 for
    every tie point t of the E2M1 grid: 0.75 v is then within one rounding of a tie, the case in which rounding the
    product to binary32 first and to E2M1 second would return the wrong code."""
    ties = [0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    vals = []
    for t in ties:
        c = np.float32(t / 0.75)
        vals += [np.nextafter(c, np.float32(0)), c, np.nextafter(c, np.float32(np.inf))]
    vals = np.array(vals, dtype=np.float32)           # 21 values
    row = np.zeros(64, dtype=np.float32)
    row[0] = 8.0
    row[1:22] = vals
    row[32] = -8.0
    row[33:54] = -vals
    return row


@pytest.mark.parametrize("sw_codec", [False, True])
def test_round43_bit_exact_on_oracle_values(fp4, oracle, sw_codec, knobs):
    import torch
    knobs(sw_codec=sw_codec)
    rng = np.random.default_rng(700)
    M, K = 131, 2048 + 256
    y = (rng.laplace(size=(M, K)) * np.exp(rng.uniform(-2, 2, (M, K)))).astype(np.float32)
    y[1, 64:128] = 0.0
    y[3, :64] = adversarial_rows()
    y[4, :64] = adversarial_rows() * np.float32(2.0 ** -7)
    # abs-max values next to the exponent decision boundaries
    for i, k in enumerate(range(-4, 5)):
        t = np.float32(6.0 * 2.0 ** (k + 0.5))
        y[5, 32 * i:32 * (i + 1)] = 0.0
        y[5, 32 * i] = np.nextafter(t, np.float32(0))
        y[6, 32 * i:32 * (i + 1)] = 0.0
        y[6, 32 * i + 7] = -np.nextafter(t, np.float32(np.inf))
    ref_c, ref_s, ref_T = oracle.quantize(y, MX, policy="round43")
    abs_c, abs_s, _ = oracle.quantize(y, MX)
    say(f"round43 mode-i sw_codec={sw_codec}: {(ref_s != abs_s).mean():.1%} of the scale bytes differ from the floor rule")
    c, s, _ = fp4.fp4_rotate_quantize(to_dev(y), 1, MX, flags=fp4.SCALE_ROUND43)
    torch.cuda.synchronize()
    assert np.array_equal(np_(s).reshape(M, -1), ref_s)
    assert np.array_equal(np_(c).reshape(M, -1), ref_c)
    assert not np.array_equal(ref_s, abs_s)


def check_end_to_end(y, got_c, got_s, ref_c, ref_s):
    same = got_s == ref_s
    n_bad = int((~same).sum())
    if n_bad:
        assert n_bad <= max(1, int(2e-5 * same.size)), n_bad
        amax = np.abs(y.astype(np.float64)).reshape(y.shape[0], -1, 32).max(-1)[~same]
        bound = 6.0 * 2.0 ** (np.round(np.log2(amax / 6.0) - 0.5) + 0.5)
        assert np.all(np.abs(amax - bound) <= 8 * np.spacing(bound.astype(np.float32))), "scale differs away from a boundary"
        assert np.all(np.abs(got_s[~same].astype(int) - ref_s[~same].astype(int)) == 1)
    mask = np.repeat(same, 32, axis=1)
    steps = grid_steps(unpack(got_c), unpack(ref_c))
    assert steps[mask].max(initial=0) <= 1
    assert (steps[mask] != 0).mean() <= 1e-4
    return n_bad


@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_round43_end_to_end_with_rotation(fp4, oracle, b):
    import torch
    M, K = 90, 2048 + 512
    xb = inputs.RECIPES[6].x(M, K, salt=700 + b)
    y = oracle.rotate(xb, b)
    say(f"round43 e2e b={b}")
    c, s, _ = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, MX, flags=fp4.SCALE_ROUND43)
    torch.cuda.synchronize()
    ref_c, ref_s, _ = oracle.quantize(y, MX, policy="round43")
    check_end_to_end(y, np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s)


def test_round43_big_call_gemm_layout_equals_canonical(fp4, oracle):
    """[2048, 8192] goes through the fragment-order kernel; its bytes un-shuffle to the canonical kernel's, and 32
    sampled rows match the oracle."""
    import torch
    M, K, b = 2048, 8192, 32
    xb = inputs.RECIPES[1].x(M, K, salt=23)
    x = to_dev_bf16(xb)
    say("round43 big")
    c0, s0, _ = fp4.fp4_rotate_quantize(x, b, MX, flags=fp4.SCALE_ROUND43)
    c1, s1, _ = fp4.fp4_rotate_quantize(x, b, MX, flags=fp4.SCALE_ROUND43 | fp4.LAYOUT_GEMM)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(3).choice(M, 32, replace=False))
    cc, ss = gemm_layout_to_canonical(np_(c1), np_(s1), rows, K, MX)
    assert np.array_equal(cc, np_(c0).reshape(M, -1)[rows]) and np.array_equal(ss, np_(s0).reshape(M, -1)[rows])
    y = oracle.rotate(xb[rows], b)
    ref_c, ref_s, _ = oracle.quantize(y, MX, policy="round43")
    check_end_to_end(y, cc, ss, ref_c, ref_s)


def test_round43_dense_rotation_and_weights_entry_point(fp4, oracle):
    import torch
    M, K, b = 48, 1024, 32
    xb = inputs.RECIPES[6].x(M, K, salt=77)
    n_ = np.arange(b)[:, None]
    k_ = np.arange(b)[None, :]
    R = np.cos(np.pi * (2 * n_ + 1) * k_ / (2 * b)) * np.sqrt(2.0 / b)
    R[:, 0] = 1.0 / np.sqrt(b)
    Rb = inputs.f32_to_bf16_bits(R.astype(np.float32))
    say("round43 dense rotation / weights")
    c, s, _ = fp4.fp4_rotate_quantize_dense(to_dev_bf16(xb), to_dev_bf16(Rb), MX, flags=fp4.SCALE_ROUND43)
    cw, sw, _ = fp4.fp4_quantize_weights(to_dev_bf16(xb), b, MX, flags=fp4.SCALE_ROUND43)
    torch.cuda.synchronize()
    y = oracle.rotate_dense(xb, Rb)
    ref_c, ref_s, _ = oracle.quantize(y, MX, policy="round43")
    check_end_to_end(y, np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s)
    y = oracle.rotate(xb, b)
    ref_c, ref_s, _ = oracle.quantize(y, MX, policy="round43")
    check_end_to_end(y, np_(cw).reshape(M, -1), np_(sw).reshape(M, -1), ref_c, ref_s)


@pytest.mark.parametrize("M,a43,w43", [(8, True, True), (8, False, True), (48, True, False), (272, True, True), (272, False, True)])
def test_products_apply_the_tensor_level_factor(fp4, oracle, M, a43, w43):
    """Operands quantized by the oracle (either rule), multiplied by the library with the matching flags: the result
    is the oracle's product of the dequantized operands (4/3 applied per flagged operand) within the GEMM tolerance.
    M = 8 and 48 take the weight-streaming kernel, M = 272 the tile kernel."""
    import torch
    N, K, b = 528, 1280, 32
    r = inputs.RECIPES[1]
    xb, wb = r.x(M, K, salt=1), r.w(N, K, salt=2)
    ac, asc, aT = oracle.quantize(oracle.rotate(xb, b), MX, policy="round43" if a43 else "absmax")
    wc, wsc, wT = oracle.quantize(oracle.rotate(wb, b), MX, policy="round43" if w43 else "absmax")
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX, aT), oracle.dequantize(wc, wsc, MX, wT))
    say(f"round43 product M={M} a43={a43} w43={w43}")
    flags = fp4.OUT_F32 | (fp4.A_SCALE43 if a43 else 0) | (fp4.W_SCALE43 if w43 else 0)
    out = fp4.fp4_gemm(to_dev(ac.reshape(-1)), to_dev(asc.reshape(-1)), None, to_dev(wc.reshape(-1)), to_dev(wsc.reshape(-1)),
                       None, M, N, K, MX, flags=flags)
    torch.cuda.synchronize()
    got = np_(out).astype(np.float64)
    assert np.all(np.abs(got - Y) <= 1e-3 * S + 1e-30)
    # the factor really is there: without the flags the result is smaller by (4/3)^n
    plain = fp4.fp4_gemm(to_dev(ac.reshape(-1)), to_dev(asc.reshape(-1)), None, to_dev(wc.reshape(-1)), to_dev(wsc.reshape(-1)),
                         None, M, N, K, MX, flags=fp4.OUT_F32)
    torch.cuda.synchronize()
    f = (4.0 / 3.0) ** (int(a43) + int(w43))
    assert np.allclose(got, np_(plain).astype(np.float64) * f, rtol=1e-6, atol=1e-30)


@pytest.mark.parametrize("weight_only", [False, True])
def test_few_token_entry_points_take_round43_weights(fp4, oracle, weight_only):
    import torch
    M, N, K, b = 4, 272, 1024, 32
    r = inputs.RECIPES[1]
    xb, wb = r.x(M, K, salt=5), r.w(N, K, salt=6)
    wq = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.LAYOUT_GEMM | fp4.SCALE_ROUND43)
    fn = fp4.fp4_w4a16_linear if weight_only else fp4.fp4_fused_linear
    say(f"round43 few-token weight_only={weight_only}")
    out = fn(to_dev_bf16(xb), b, wq[0], wq[1], N, MX, flags=fp4.OUT_F32 | fp4.W_SCALE43)
    torch.cuda.synchronize()
    wc, wsc, wT = oracle.quantize(oracle.rotate(wb, b), MX, policy="round43")
    What = oracle.dequantize(wc, wsc, MX, wT)
    ya = oracle.rotate(xb, b)
    if weight_only:
        A = oracle.round_to_bf16(ya)
    else:
        ac, asc, _ = oracle.quantize(ya, MX)
        A = oracle.dequantize(ac, asc, MX)
    Y, S = oracle.matmul(A, What)
    assert np.all(np.abs(np_(out).astype(np.float64) - Y) <= 1e-3 * S + 1e-30)


def test_round43_is_rejected_for_nvfp4_and_with_mse(fp4):
    import torch
    x = torch.zeros((16, 128), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(Exception):
        fp4.fp4_rotate_quantize(x, 32, NV, flags=fp4.SCALE_ROUND43)
    with pytest.raises(Exception):
        fp4.fp4_rotate_quantize(x, 32, MX, flags=fp4.SCALE_ROUND43 | fp4.SCALE_MSE)


@pytest.mark.parametrize("variant", [11, 13, 14])
def test_tensor_level_factor_in_the_persistent_and_wide_tile_kernels(fp4, oracle, variant, knobs):
    """The factor is applied per tile before the epilogue: persistent workgroups walking several tiles (variants 11, 14)
    and the 256 x 192 tile (13, 14), bf16 output through the staged epilogue."""
    import torch
    knobs(variant=variant)
    knobs(grid=2)
    M, N, K, b = 272, 528, 1280, 32
    r = inputs.RECIPES[1]
    xb, wb = r.x(M, K, salt=11), r.w(N, K, salt=12)
    ac, asc, aT = oracle.quantize(oracle.rotate(xb, b), MX, policy="round43")
    wc, wsc, wT = oracle.quantize(oracle.rotate(wb, b), MX, policy="round43")
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX, aT), oracle.dequantize(wc, wsc, MX, wT))
    say(f"round43 product, variant {variant}")
    out = fp4.fp4_gemm(to_dev(ac.reshape(-1)), to_dev(asc.reshape(-1)), None, to_dev(wc.reshape(-1)), to_dev(wsc.reshape(-1)),
                       None, M, N, K, MX, flags=fp4.A_SCALE43 | fp4.W_SCALE43)
    torch.cuda.synchronize()
    got = np_(out.float()).astype(np.float64)
    # bf16 output: half an ulp of bf16 on top of the GEMM tolerance
    assert np.all(np.abs(got - Y) <= 1e-3 * S + 2.0 ** -8 * np.abs(Y) + 1e-30)
