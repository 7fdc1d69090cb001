"""GPU parity for the one-launch few-token path (fp4_fused_linear): against the two-launch path (bit-identical for
Hadamard blocks up to 32, where both use the same operand) and against the oracle (end-to-end rule on the product)."""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, compare_codes, to_dev_bf16

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


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("M,N,K,b", [(1, 256, 512, 32), (1, 4096, 4096, 32), (3, 520, 1152, 16), (4, 264, 128 * 9, 32),
                                     (2, 136, 128 * 37, 32), (4, 1032, 4096, 16), (3, 24, 128, 32)])
def test_fused_equals_two_launch_path(fp4, M, N, K, b, out_f32):
    import torch
    r = inputs.RECIPES[2]
    x, w = to_dev_bf16(r.x(M, K, salt=M + N)), to_dev_bf16(r.w(N, K, salt=M + N))
    qw = fp4.fp4_quantize_weights(w, b, MX, flags=fp4.LAYOUT_GEMM)
    flags = fp4.OUT_F32 if out_f32 else 0
    say(f"fused vs two launches M={M} N={N} K={K} b={b} f32={out_f32}")
    qa = fp4.fp4_rotate_quantize(x, b, MX, flags=fp4.LAYOUT_GEMM)
    ref = fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, M, N, K, MX, flags=flags | fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
    got = fp4.fp4_fused_linear(x, b, qw[0], qw[1], N, MX, flags=flags)
    torch.cuda.synchronize()
    assert torch.equal(got, ref)


@pytest.mark.parametrize("b", [16, 32, 64, 128])
@pytest.mark.parametrize("M", [1, 4])
def test_fused_against_oracle(fp4, oracle, M, b):
    """The one-launch result against the oracle's fp64 product of the codes the library itself produces for the same
    inputs (stand-alone quantizer, canonical order), to the bare accumulation bound; those codes are in turn held to
    the end-to-end rule against the oracle's.  One differing code can therefore neither hide in a widened product
    tolerance nor break it."""
    import torch
    N, K = 272, 2048 + 384
    r = inputs.RECIPES[2]
    xb, wb = r.x(M, K, salt=70 + b), r.w(N, K, salt=70 + b)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.LAYOUT_GEMM)
    say(f"fused vs oracle M={M} b={b}")
    got = fp4.fp4_fused_linear(to_dev_bf16(xb), b, qw[0], qw[1], N, MX, flags=fp4.OUT_F32)
    qa_c = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, MX)
    qw_c = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX)
    torch.cuda.synchronize()
    ac, asc = np_(qa_c[0]).reshape(M, -1), np_(qa_c[1]).reshape(M, -1)
    wc, wsc = np_(qw_c[0]).reshape(N, -1), np_(qw_c[1]).reshape(N, -1)
    rac, rasc, _, ya = oracle.rotate_quantize(xb, b, MX)
    rwc, rwsc, _, yw = oracle.rotate_quantize(wb, b, MX)
    compare_codes(ac, asc, rac, rasc, ya, MX)
    compare_codes(wc, wsc, rwc, rwsc, yw, MX)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    err = np.abs(np_(got).astype(np.float64) - Y)
    # the in-GEMM quantizer runs the same rotation (32-wide operand, butterfly levels for wider blocks) and the same
    # group quantizer as the stand-alone canonical-order kernel: same codes, so the bare accumulation bound applies
    assert np.all(err <= 1e-3 * S)


def test_fused_full_size_decode_layers(fp4, oracle):
    """Llama-3-8B decode shapes, M = 1: against the two-launch path (bit-identical)."""
    import torch
    for i, L in enumerate(inputs.LLAMA3_8B_LAYERS):
        r = inputs.RECIPES[2]
        x, w = to_dev_bf16(r.x(1, L.K, salt=i)), to_dev_bf16(r.w(L.N, L.K, salt=i))
        qw = fp4.fp4_quantize_weights(w, 32, MX, flags=fp4.LAYOUT_GEMM)
        qa = fp4.fp4_rotate_quantize(x, 32, MX, flags=fp4.LAYOUT_GEMM)
        say(f"fused full-size {L.name}")
        ref = fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, 1, L.N, L.K, MX, flags=fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
        got = fp4.fp4_fused_linear(x, 32, qw[0], qw[1], L.N, MX)
        torch.cuda.synchronize()
        assert torch.equal(got, ref)
        del w, qw


def test_fused_rejects_what_it_cannot_do(fp4):
    import torch
    x = torch.zeros((17, 256), dtype=torch.bfloat16, device="cuda")
    w = torch.zeros(16 * 128, dtype=torch.uint8, device="cuda")
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x, 32, w, w, 16, MX)
    assert e.value.status == 2            # more than four tokens
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x[:5].contiguous(), 32, w, w, 16, MX)
    assert e.value.status == 2 and "1..4 tokens" in str(e.value)
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_w4a16_linear(x, 32, w, w, 16, MX)
    assert e.value.status == 2            # the weight-only variant takes up to 16
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x[:4].contiguous(), 32, w, w, 16, NV)
    assert e.value.status == 4            # NVFP4 is not a one-pass operation
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x[:4].contiguous(), 1, w, w, 16, MX)
    assert e.value.status == 3


# ---------------------------------------------------------------- weight-only variant (W4A16)
def _w4a16_case(fp4, oracle, M, N, K, b, out_f32, salt):
    import torch
    r = inputs.RECIPES[2]
    xb, wb = r.x(M, K, salt=salt), r.w(N, K, salt=salt)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.LAYOUT_GEMM)
    say(f"w4a16 M={M} N={N} K={K} b={b} f32={out_f32}")
    got = fp4.fp4_w4a16_linear(to_dev_bf16(xb), b, qw[0], qw[1], N, MX, flags=fp4.OUT_F32 if out_f32 else 0)
    torch.cuda.synchronize()
    Y, S = oracle.linear_w4a16(xb, wb, b)
    err = np.abs(np_(got.float()).astype(np.float64) - Y)
    # The library's rotated activations differ from the oracle's by fp32 rounding before the bf16 rounding: an element
    # whose value sits next to a bf16 rounding boundary moves by one bf16 ulp (2^-8 relative) in a few cases per row;
    # weights likewise by one grid step in <= 1e-4 of the cases.  Budget: the accumulation bound plus 2^-8 of the
    # largest term times a handful of such events; most outputs must meet the bare bound.
    ya = np.abs(oracle.round_to_bf16(oracle.rotate(xb, b))).max()
    wmax = np.abs(oracle.rotate(wb, b)).max()
    tol = 1e-3 * S + (0 if out_f32 else np.abs(Y) * 2.0 ** -8)
    assert (err > tol).mean() <= 0.02
    assert np.all(err <= tol + 8 * 2.0 ** -8 * ya * wmax)
    return got


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("M,N,K,b", [(1, 256, 512, 32), (1, 1032, 4096, 32), (3, 520, 1152, 16), (4, 264, 128 * 9, 64),
                                     (16, 136, 128 * 37, 32), (2, 24, 128, 128), (9, 272, 2048, 128)])
def test_w4a16_against_oracle(fp4, oracle, M, N, K, b, out_f32):
    _w4a16_case(fp4, oracle, M, N, K, b, out_f32, salt=M + N + b)


def test_w4a16_exact_when_everything_is_representable(fp4, oracle):
    """Activations whose rotation is exact in bf16 (one non-zero per 32-block: the rotation gives +-x/sqrt(32)... not
    exact) -- so use had_block 16 (1/4 exact) with small-integer inputs: rotated values are multiples of 1/4 below 2^8,
    exact in bf16; weights on the grid after rotation.  Then every product and partial sum is exact in fp32 and the
    result must equal the oracle bit for bit."""
    import torch
    rng = np.random.default_rng(5)
    b, M, N, K = 16, 2, 48, 256
    x = rng.integers(-3, 4, (M, K)).astype(np.float32)                 # |sum of 16| <= 48, times 1/4: multiples of 0.25
    xb = inputs.f32_to_bf16_bits(x)
    H = oracle.hadamard(b).astype(np.float64)
    grid = np.array([0, .5, 1, 1.5, 2, 3, 4, 6])
    Wr = rng.choice(np.concatenate([-grid[1:], grid]), size=(N, K))
    Wr[:, ::32] = 6.0                                                  # abs-max 6 in every group: scale 2^0
    W = (Wr.reshape(N, K // b, b) @ H / 4.0).reshape(N, K)             # rotation is its own inverse: W H/4 = Wr
    wb = inputs.f32_to_bf16_bits(W.astype(np.float32))
    assert np.array_equal(inputs.bf16_bits_to_f32(wb).astype(np.float64), W)   # W itself is exact in bf16
    assert np.array_equal(oracle.rotate(wb, b).astype(np.float64), Wr)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.LAYOUT_GEMM)
    got = fp4.fp4_w4a16_linear(to_dev_bf16(xb), b, qw[0], qw[1], N, MX, flags=fp4.OUT_F32)
    torch.cuda.synchronize()
    Y, _ = oracle.linear_w4a16(xb, wb, b)
    assert np.array_equal(np_(got).astype(np.float64), Y)


def test_w4a16_full_size_decode_layers(fp4, oracle):
    for i, L in enumerate(inputs.LLAMA3_8B_LAYERS[:2] + inputs.LLAMA3_8B_LAYERS[3:]):
        N = min(L.N, 4096)
        _w4a16_case(fp4, oracle, 1, N, L.K, 32, False, salt=300 + i)
