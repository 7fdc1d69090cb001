"""GPU parity for the caller-supplied dense block rotation (fp4_rotate_quantize_dense) against the CPU oracle.

Bars: identical to the Hadamard path's end-to-end rule (scales equal, <= 1e-4 of the codes differ, each by one grid
step) because the GPU accumulates the b products in fp32 while the oracle rounds once from fp64; bit-identical where
the arithmetic is exact (matrices with power-of-two entries).
"""
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


def bits(a):
    return inputs.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def dct_matrix(b):
    n = np.arange(b)[:, None]
    k = np.arange(b)[None, :]
    R = np.cos(np.pi * (2 * n + 1) * k / (2 * b)) * np.sqrt(2.0 / b)
    R[:, 0] = 1.0 / np.sqrt(b)
    return R


@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("b", [16, 64])
def test_dense_with_exact_hadamard_equals_hadamard_path(fp4, oracle, fmt, b):
    """H_b / sqrt(b) is exact in bf16 for b = 16, 64: products and sums scale by a power of two, so the dense
    kernel path and the built-in Hadamard path must agree bit for bit, in both output layouts."""
    import torch
    r = inputs.RECIPES[1 if fmt == MX else 4]
    M, K = 83, 2048 + 256
    xb = r.x(M, K, salt=200 + b)
    Rb = bits(oracle.hadamard(b).astype(np.float64) / np.sqrt(b))
    x, R = to_dev_bf16(xb), to_dev_bf16(Rb)
    for flags in (0, fp4.LAYOUT_GEMM):
        say(f"dense==hadamard fmt={fmt} b={b} flags={flags}")
        # zero-filled outputs: the GEMM layout pads rows to 16 and MXFP4 scales to 512 K, and padding is never written
        cb, sb = fp4.packed_bytes(M, K, fmt, flags)
        z = lambda n: torch.zeros(n, dtype=torch.uint8, device="cuda")
        c0, s0, T0 = fp4.fp4_rotate_quantize(x, b, fmt, flags=flags, codes=z(cb), scales=z(sb))
        c1, s1, T1 = fp4.fp4_rotate_quantize_dense(x, R, fmt, flags=flags, codes=z(cb), scales=z(sb))
        torch.cuda.synchronize()
        assert torch.equal(c0, c1) and torch.equal(s0, s1)
        if fmt == NV:
            assert np_(T0)[0] == np_(T1)[0]


@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_dense_dct_against_oracle(fp4, oracle, fmt, b):
    import torch
    r = inputs.RECIPES[1 if fmt == MX else 4]
    M, K = 77, 2048 + 512
    xb = r.x(M, K, salt=300 + b)
    Rb = bits(dct_matrix(b))
    y = oracle.rotate_dense(xb, Rb)
    ref_c, ref_s, ref_T = oracle.quantize(y, fmt)
    say(f"dense dct e2e fmt={fmt} b={b}")
    c, s, T = fp4.fp4_rotate_quantize_dense(to_dev_bf16(xb), to_dev_bf16(Rb), fmt)
    torch.cuda.synchronize()
    if fmt == NV:
        assert abs(float(np_(T)[0]) - float(ref_T)) <= 2 * np.spacing(np.float32(ref_T))
        if np_(T)[0] != ref_T:
            # same codes rule with the library's own tensor scale handed to the oracle
            ref_c, ref_s, _ = oracle.quantize(y, fmt, tensor_scale=float(np_(T)[0]))
    frac, flips = compare_codes(np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s, y, fmt)
    say(f"   differing codes: {frac:.2e}, scale flips: {flips}")


def test_dense_asymmetric_matrix_gemm_layout(fp4, oracle):
    """A non-symmetric matrix pins the orientation (x . R), and the GEMM layout un-shuffles to the same bytes."""
    import torch
    rng = np.random.default_rng(5)
    b, M, K = 32, 50, 1024 + 128
    Rb = bits(dct_matrix(b) + 0.05 * rng.standard_normal((b, b)))
    xb = inputs.RECIPES[1].x(M, K, salt=77)
    y = oracle.rotate_dense(xb, Rb)
    ref_c, ref_s, _ = oracle.quantize(y, MX)
    x, R = to_dev_bf16(xb), to_dev_bf16(Rb)
    say("dense asymmetric, both layouts")
    c0, s0, _ = fp4.fp4_rotate_quantize_dense(x, R, MX)
    c1, s1, _ = fp4.fp4_rotate_quantize_dense(x, R, MX, flags=fp4.LAYOUT_GEMM)
    torch.cuda.synchronize()
    compare_codes(np_(c0).reshape(M, -1), np_(s0).reshape(M, -1), ref_c, ref_s, y, MX)
    cc, ss = gemm_layout_to_canonical(np_(c1), np_(s1), M, K, MX)
    assert np.array_equal(cc, np_(c0).reshape(M, -1)) and np.array_equal(ss, np_(s0).reshape(M, -1))


def test_dense_identity_equals_no_rotation(fp4):
    import torch
    b, M, K = 32, 40, 1024
    x = to_dev_bf16(inputs.RECIPES[1].x(M, K, salt=9))
    R = to_dev_bf16(bits(np.eye(b)))
    say("dense identity")
    a = fp4.fp4_rotate_quantize(x, 1, MX)
    d = fp4.fp4_rotate_quantize_dense(x, R, MX)
    torch.cuda.synchronize()
    assert torch.equal(a[0], d[0]) and torch.equal(a[1], d[1])


def test_dense_large_tensor_sampled_rows(fp4, oracle):
    """[4096, 4096] with a DCT block: a large grid with several items per wave; 48 sampled rows against the oracle."""
    import torch
    b, M, K = 64, 4096, 4096
    r = inputs.RECIPES[1]
    xb = r.x(M, K, salt=11)
    Rb = bits(dct_matrix(b))
    say("dense large")
    c, s, _ = fp4.fp4_rotate_quantize_dense(to_dev_bf16(xb), to_dev_bf16(Rb), MX)
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(1).choice(M, 48, replace=False))
    y = oracle.rotate_dense(xb[rows], Rb)
    ref_c, ref_s, _ = oracle.quantize(y, MX)
    compare_codes(np_(c).reshape(M, -1)[rows], np_(s).reshape(M, -1)[rows], ref_c, ref_s, y, MX)


def test_dense_rejects_bad_arguments(fp4):
    import torch
    x = torch.zeros((16, 256), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_rotate_quantize_dense(x, torch.zeros((24, 24), dtype=torch.bfloat16, device="cuda"), MX)
    assert e.value.status == 3            # block not in {16, 32, 64, 128}
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_rotate_quantize_dense(x[:, :192].contiguous(), torch.zeros((128, 128), dtype=torch.bfloat16, device="cuda"), MX)
    assert e.value.status == 2            # K not a multiple of the block
