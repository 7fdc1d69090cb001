"""GPU parity of the fitted scale range (FP4MR_SCALE_FIT_RANGE; appendix on MXFP scale fitting, s = 2^(alpha q + beta))
against the CPU oracle.

log2 and exp2 are transcendental: the library evaluates them with the GPU's binary32 instructions, the oracle in fp64, so
(alpha, beta), the 256 scale values and the byte are compared within what binary32 log2 / exp2 can differ by, and the
byte as "the nearest table entry in the log domain".  The element codes are then compared BIT-EXACTLY (oracle-rotated fp32
input) or under the end-to-end rule (library's own rotation) against the oracle's quantizer run on the library's own
bytes and scale values.
"""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, gemm_layout_to_canonical, grid_steps, to_dev, to_dev_bf16, unpack

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


def spread_bits(seed, M, K, spread=1.0):
    rng = np.random.default_rng(seed)
    x = rng.laplace(size=(M, K)) * np.exp(rng.normal(size=(M, 1)) * spread) * np.exp(rng.normal(size=(1, K // 32)).repeat(32, axis=1) * 0.5)
    return inputs.f32_to_bf16_bits(x.astype(np.float32))


def check_fit(oracle, y, q_gpu, ts_gpu, given=None):
    """(alpha, beta), table and bytes of the library against the oracle's fp64 fit of the fp32 tensor y."""
    M, K = y.shape
    alpha, beta, table = float(ts_gpu[0]), float(ts_gpu[1]), ts_gpu[2:258].astype(np.float64)
    c_o, q_o, (a_o, b_o), t_o = oracle.quantize_mxfp4_fit(y, alpha_beta=given)
    if given is None:
        assert abs(alpha - a_o) <= 2e-6 * max(a_o, 1e-3) + 1e-9, (alpha, a_o)
        assert abs(beta - b_o) <= 8e-6, (beta, b_o)
    else:
        assert alpha == np.float32(given[0]) and beta == np.float32(given[1])
    # the published scale values are 2^(alpha q + beta) of the library's own binary32 alpha, beta
    want = np.exp2(alpha * np.arange(256) + beta)
    assert np.all(np.abs(table / want - 1.0) <= 3e-6), float(np.abs(table / want - 1.0).max())
    # the byte: nearest table entry in the log domain, up to binary32 log2 accuracy
    amax = np.abs(y.astype(np.float64)).reshape(M, -1, 32).max(axis=2)
    nz = amax > 0
    assert not q_gpu[~nz].any()
    ls = np.log2(amax[nz] / 6.0)
    lt = np.log2(table)[q_gpu[nz]]
    inside = (q_gpu[nz] > 0) & (q_gpu[nz] < 255)
    assert np.all(np.abs(lt - ls)[inside] <= alpha / 2 + 1.2e-5), float(np.abs(lt - ls)[inside].max())
    # clamped ends: the ideal scale lies beyond the end of the table (or within half a step of it)
    assert np.all((ls - lt)[q_gpu[nz] == 255] >= -alpha / 2 - 1.2e-5) and np.all((ls - lt)[q_gpu[nz] == 0] <= alpha / 2 + 1.2e-5)
    dq = np.abs(q_gpu.astype(int) - q_o.astype(int))
    assert dq.max() <= 1 and (dq != 0).mean() <= 5e-3, (int(dq.max()), float((dq != 0).mean()))
    return float((dq != 0).mean())


@pytest.mark.parametrize("layout_gemm", [False, True])
def test_fit_range_bit_exact_codes_on_oracle_rotation(fp4, oracle, layout_gemm):
    """fp32 input (the oracle's rotated values, no rotation in the library): the fit within binary32 accuracy, the codes
    bit-exact against the oracle's element chain on the library's bytes and scale values."""
    import torch
    M, K = 67, 1536
    y = oracle.rotate(spread_bits(1, M, K), 32)
    y[0, :8] = [4.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    y[1, 32:96] = 0.0                                     # two all-zero groups
    flags = fp4.SCALE_FIT_RANGE | (fp4.LAYOUT_GEMM if layout_gemm else 0)
    say(f"fit range mode-i layout_gemm={layout_gemm}")
    c, q, ts = fp4.fp4_rotate_quantize(to_dev(y), 1, MX, flags=flags)
    torch.cuda.synchronize()
    assert ts.numel() == fp4.FIT_RANGE_FLOATS
    c, q, ts = np_(c), np_(q), np_(ts)
    if layout_gemm:
        c, q = gemm_layout_to_canonical(c, q, M, K, MX)
    c, q = c.reshape(M, -1), q.reshape(M, -1)
    frac = check_fit(oracle, y, q, ts)
    say(f"   bytes off by one against the fp64 fit: {frac:.2e}")
    ref_c = oracle.quantize_given_scales(y, q, ts[2:258])
    assert np.array_equal(c, ref_c)
    assert not c[1, 16:48].any()


@pytest.mark.parametrize("layout_gemm", [False, True])
@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_fit_range_end_to_end(fp4, oracle, b, layout_gemm):
    """bf16 input through the library's own rotation, every Hadamard block size, both layouts (GEMM layout at this size
    runs the fragment-shaped kernel): codes under the end-to-end rule."""
    import torch
    M, K = 272, 4096                                       # 17 row-blocks x 8 items: the big-call kernel in GEMM layout
    xb = spread_bits(10 + b, M, K)
    y = oracle.rotate(xb, b)
    flags = fp4.SCALE_FIT_RANGE | (fp4.LAYOUT_GEMM if layout_gemm else 0)
    say(f"fit range e2e b={b} layout_gemm={layout_gemm}")
    c, q, ts = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, MX, flags=flags)
    torch.cuda.synchronize()
    c, q, ts = np_(c), np_(q), np_(ts)
    if layout_gemm:
        c, q = gemm_layout_to_canonical(c, q, M, K, MX)
    c, q = c.reshape(M, -1), q.reshape(M, -1)
    check_fit(oracle, y, q, ts)
    ref_c = oracle.quantize_given_scales(y, q, ts[2:258])
    steps = grid_steps(unpack(c), unpack(ref_c))
    assert steps.max() <= 1 and (steps != 0).mean() <= 1e-4, (int(steps.max()), float((steps != 0).mean()))
    # and what it is for: less squared error than the E8M0 floor rule on the same rotated values
    y64 = y.astype(np.float64)
    back = oracle.dequantize_table(c, q, ts[2:258].astype(np.float64))
    c0, s0, _ = oracle.quantize(y, MX)
    assert ((back - y64) ** 2).sum() < 0.85 * ((oracle.dequantize(c0, s0, MX) - y64) ** 2).sum()


def test_fit_range_few_tokens_and_weights_entry_point(fp4, oracle):
    """One token (a grid of one workgroup in both passes) and the weight-preparation entry point."""
    import torch
    for name, fn, M, K in (("one token", fp4.fp4_rotate_quantize, 1, 2048), ("weights", fp4.fp4_quantize_weights, 200, 1024)):
        xb = spread_bits(77 + M, M, K)
        y = oracle.rotate(xb, 32)
        say(f"fit range {name}")
        c, q, ts = fn(to_dev_bf16(xb), 32, MX, flags=fp4.SCALE_FIT_RANGE)
        torch.cuda.synchronize()
        c, q, ts = np_(c).reshape(M, -1), np_(q).reshape(M, -1), np_(ts)
        check_fit(oracle, y, q, ts)
        steps = grid_steps(unpack(c), unpack(oracle.quantize_given_scales(y, q, ts[2:258])))
        assert steps.max() <= 1 and (steps != 0).mean() <= 2e-4


def test_fit_range_given_alpha_beta_clamps(fp4, oracle):
    """Caller-supplied (alpha, beta) narrower than the data: bytes clamp at both ends, overshooting groups saturate."""
    import torch
    M, K = 40, 1024
    y = oracle.rotate(spread_bits(5, M, K, spread=2.0), 32)
    _, _, (a_fit, b_fit), _ = oracle.quantize_mxfp4_fit(y)
    given = (float(np.float32(a_fit * 0.5)), float(np.float32(b_fit + 0.25 * 255 * a_fit)))   # the middle half of the range
    ts = torch.zeros(fp4.FIT_RANGE_FLOATS, dtype=torch.float32, device="cuda")
    ts[0], ts[1] = given
    say("fit range static alpha, beta")
    c, q, ts_out = fp4.fp4_rotate_quantize(to_dev(y), 1, MX, flags=fp4.SCALE_FIT_RANGE, tensor_scale=ts)
    torch.cuda.synchronize()
    c, q, tsn = np_(c).reshape(M, -1), np_(q).reshape(M, -1), np_(ts_out)
    check_fit(oracle, y, q, tsn, given=given)
    assert (q == 0).sum() > 10 and (q == 255).sum() > 10
    assert np.array_equal(c, oracle.quantize_given_scales(y, q, tsn[2:258]))


def test_fit_range_degenerate_tensors(fp4, oracle):
    import torch
    z = torch.zeros((16, 256), dtype=torch.bfloat16, device="cuda")
    c, q, ts = fp4.fp4_rotate_quantize(z, 32, MX, flags=fp4.SCALE_FIT_RANGE)
    torch.cuda.synchronize()
    ts = np_(ts)
    assert ts[0] == 0 and ts[1] == 0 and np.all(ts[2:] == 1.0) and not np_(c).any() and not np_(q).any()
    one = torch.zeros((16, 256), dtype=torch.float32, device="cuda")
    one[3, 40] = -3.0
    c, q, ts = fp4.fp4_rotate_quantize(one, 1, MX, flags=fp4.SCALE_FIT_RANGE)
    torch.cuda.synchronize()
    ts, c, q = np_(ts), np_(c).reshape(16, -1), np_(q).reshape(16, -1)
    assert ts[0] == 0 and abs(ts[1] + 1.0) <= 1e-6 and not q.any()
    back = oracle.dequantize_table(c, q, ts[2:258].astype(np.float64))
    assert abs(back[3, 40] + 3.0) <= 1e-5 and np.count_nonzero(back) == 1


def test_fit_range_through_the_allocation_free_entry_point(fp4):
    """The entry point without a workspace runs the same kernels on the library's own scratch: bit-identical outputs."""
    import torch
    x = to_dev_bf16(spread_bits(31, 50, 1024))
    c0, q0, t0 = fp4.fp4_rotate_quantize(x, 64, MX, flags=fp4.SCALE_FIT_RANGE)
    c1, q1, t1 = torch.empty_like(c0), torch.empty_like(q0), torch.empty_like(t0)
    fp4.fp4_rotate_quantize_static(x, 64, MX, flags=fp4.SCALE_FIT_RANGE, tensor_scale=t1, codes=c1, scales=q1)
    torch.cuda.synchronize()
    assert torch.equal(c0, c1) and torch.equal(q0, q1) and torch.equal(t0, t1)


def test_fit_range_validation(fp4):
    import torch
    x = torch.zeros((16, 256), dtype=torch.bfloat16, device="cuda")
    for bad in (fp4.SCALE_MSE, fp4.SCALE_ROUND43):
        with pytest.raises(fp4.Fp4mrError) as e:
            fp4.fp4_rotate_quantize(x, 32, MX, flags=fp4.SCALE_FIT_RANGE | bad)
        assert e.value.status == 4
    with pytest.raises(fp4.Fp4mrError) as e:
        fp4.fp4_rotate_quantize(x, 16, fp4.NVFP4, flags=fp4.SCALE_FIT_RANGE)
    assert e.value.status == 4
