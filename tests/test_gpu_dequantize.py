"""GPU parity of fp4_dequantize (the decoding side of the formats) against the oracle's dequantizers: every scale policy's
output, both layouts, both output types.  The library's binary32 value must equal the oracle's fp64 value rounded once to
binary32 (the exact product has at most 30 significant bits); bf16 output is that value rounded to nearest even."""
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


def _case(fp4, oracle, policy, layout_gemm, out_f32, M=70, K=1152):
    import torch
    r = inputs.RECIPES[4 if policy == "nv" else 1]
    xb = r.x(M, K, salt=len(policy))
    zr = min(3, M - 1)
    xb[zr, 64:128] = 0
    fmt = NV if policy == "nv" else MX
    qflags = {"mx": 0, "nv": 0, "round43": fp4.SCALE_ROUND43, "fit": fp4.SCALE_FIT_RANGE}[policy] | (fp4.LAYOUT_GEMM if layout_gemm else 0)
    say(f"dequantize policy={policy} layout_gemm={layout_gemm} out_f32={out_f32}")
    c, s, ts = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 32 if fmt == MX else 16, fmt, flags=qflags)
    dflags = (qflags & (fp4.SCALE_ROUND43 | fp4.SCALE_FIT_RANGE | fp4.LAYOUT_GEMM)) | (fp4.OUT_F32 if out_f32 else 0)
    got = fp4.fp4_dequantize(c, s, ts, M, K, fmt, flags=dflags)
    # the oracle decodes the canonical form of the same bytes (the canonical call writes the same codes: tested elsewhere)
    cc, sc, tsc = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 32 if fmt == MX else 16, fmt, flags=qflags & ~fp4.LAYOUT_GEMM)
    torch.cuda.synchronize()
    cc, sc = np_(cc).reshape(M, -1), np_(sc).reshape(M, -1)
    if policy == "fit":
        assert torch.equal(ts, tsc)
        want = oracle.dequantize_table(cc, sc, np_(ts)[2:258].astype(np.float64))
    elif policy == "nv":
        assert torch.equal(ts, tsc)
        want = oracle.dequantize(cc, sc, NV, float(np_(ts)[0]))
    elif policy == "round43":
        want = oracle.dequantize(cc, sc, MX, float(np.float32(4.0 / 3.0)))
    else:
        want = oracle.dequantize(cc, sc, MX)
    want32 = want.astype(np.float32)
    if out_f32:
        assert got.dtype == torch.float32
        assert np.array_equal(np_(got), want32)
    else:
        assert got.dtype == torch.bfloat16
        assert np.array_equal(np_(got.view(torch.int16)).view(np.uint16), inputs.f32_to_bf16_bits(want32))
    assert not np_(got.float())[zr, 64:128].any()


@pytest.mark.parametrize("out_f32", [True, False])
@pytest.mark.parametrize("layout_gemm", [False, True])
@pytest.mark.parametrize("policy", ["mx", "nv", "round43", "fit"])
def test_dequantize_against_oracle(fp4, oracle, policy, layout_gemm, out_f32):
    _case(fp4, oracle, policy, layout_gemm, out_f32)


def test_dequantize_one_row_and_validation(fp4, oracle):
    import torch
    _case(fp4, oracle, "mx", True, True, M=1, K=128)
    z = torch.zeros(64, dtype=torch.uint8, device="cuda")
    for kw, status in ((dict(fmt=NV), 1), (dict(fmt=MX, flags=fp4.SCALE_FIT_RANGE), 1), (dict(fmt=NV, flags=fp4.SCALE_ROUND43, ts=True), 4),
                       (dict(fmt=MX, flags=fp4.SCALE_MSE), 4), (dict(fmt=MX, K=48), 2), (dict(fmt=MX, K=64, flags=fp4.LAYOUT_GEMM), 2)):
        ts = torch.zeros(258, dtype=torch.float32, device="cuda") if kw.get("ts") else None
        with pytest.raises(fp4.Fp4mrError) as e:
            fp4.fp4_dequantize(z, z, ts, 1, kw.get("K", 64), kw["fmt"], flags=kw.get("flags", 0))
        assert e.value.status == status, kw
