"""GPU parity for the one-launch few-token path (fp4_fused_linear): against the two-launch path (bit-identical for
Hadamard blocks up to 32, where both use the same operand) and against the oracle (end-to-end rule on the product)."""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, to_dev_bf16

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
@pytest.mark.parametrize("M,N,K,b", [(1, 256, 512, 32), (1, 4096, 4096, 32), (3, 520, 1152, 16), (16, 264, 128 * 9, 32),
                                     (7, 136, 128 * 37, 32), (16, 1032, 4096, 16), (5, 24, 128, 32)])
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
@pytest.mark.parametrize("M", [1, 16])
def test_fused_against_oracle(fp4, oracle, M, b):
    import torch
    N, K = 272, 2048 + 384
    r = inputs.RECIPES[2]
    xb, wb = r.x(M, K, salt=70 + b), r.w(N, K, salt=70 + b)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.LAYOUT_GEMM)
    say(f"fused vs oracle M={M} b={b}")
    got = fp4.fp4_fused_linear(to_dev_bf16(xb), b, qw[0], qw[1], N, MX, flags=fp4.OUT_F32)
    torch.cuda.synchronize()
    ac, asc, _, _ = oracle.rotate_quantize(xb, b, MX)
    wc, wsc, _, _ = oracle.rotate_quantize(wb, b, MX)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    err = np.abs(np_(got).astype(np.float64) - Y)
    # codes may differ from the oracle's on <= 1e-4 of the elements by one grid step (end-to-end rule): allow for a
    # handful of such steps per output on top of the accumulation tolerance
    step = 2.0 * np.abs(oracle.dequantize(wc, wsc, MX)).max() * np.abs(oracle.dequantize(ac, asc, MX)).max()
    bad = err > 1e-3 * S
    assert bad.mean() <= 0.02, bad.mean()
    assert np.all(err <= 1e-3 * S + 4 * step)


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
    assert e.value.status == 2            # more than 16 tokens
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x[:4].contiguous(), 32, w, w, 16, NV)
    assert e.value.status == 4            # NVFP4 is not a one-pass operation
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_fused_linear(x[:4].contiguous(), 1, w, w, 16, MX)
    assert e.value.status == 3
