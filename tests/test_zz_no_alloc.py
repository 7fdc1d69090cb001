"""The allocation-free entry point (fp4_rotate_quantize_static: scratch in a device array inside the library) against
the ordinary one (fp4_rotate_quantize: scratch in a caller-supplied workspace), through the C ABI, bit for bit.

Two calls in a row on one GPU, the second with a smaller input, so that the second call finds the first call's
contents in the shared array: a big NVFP4 call (more than 256 per-wave partial maxima: the reducing kernel runs) and
then a few-token call (a handful of partials that the quantizing pass reduces itself), in both output layouts, then the
same pair again.  Every output is pre-allocated by the test: the binding of the new entry point marshals pointers only.
"""
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


def _pair(fp4, x, b, fmt, flags):
    """(ordinary entry point, allocation-free entry point) on the same input, outputs pre-filled with different bytes"""
    import torch
    rows, K = x.shape
    cb, sb = fp4.packed_bytes(rows, K, fmt, flags & fp4.LAYOUT_GEMM)
    outs = []
    for fill, static in ((0x11, False), (0xEE, True)):
        codes = torch.full((cb,), fill, dtype=torch.uint8, device="cuda")
        scales = torch.full((sb,), fill, dtype=torch.uint8, device="cuda")
        ts = torch.full((1,), -1.0, dtype=torch.float32, device="cuda") if fmt == NV else None
        if static:
            fp4.fp4_rotate_quantize_static(x, b, fmt, flags=flags, tensor_scale=ts, codes=codes, scales=scales)
        else:
            ws = torch.zeros(fp4.workspace_bytes(fp4.OP_ROTATE_QUANTIZE, rows, 0, K, fmt, flags) or 16, dtype=torch.uint8, device="cuda")
            st = fp4.lib.fp4_rotate_quantize(x.data_ptr(), rows, K, b, fmt, codes.data_ptr(), scales.data_ptr(),
                                             None if ts is None else ts.data_ptr(), ws.data_ptr(), ws.numel(), flags,
                                             torch.cuda.current_stream().cuda_stream)
            assert st == 0
        outs.append((codes, scales, ts))
    torch.cuda.synchronize()
    return outs


def test_static_scratch_entry_point_equals_the_workspace_one_on_two_calls_in_a_row(fp4):
    import torch
    r = inputs.RECIPES[4]
    big = to_dev_bf16(r.x(1200, 4096, salt=1))        # 300 abs-max workgroups: 1200 partials, reduced by the finalize kernel
    small = to_dev_bf16(r.x(8, 1024, salt=2))         # 8 fragments: 8 partials, reduced inside the quantize pass
    # the small input is louder than the big one: a tensor scale left over from the first call would show
    small = (small.float() * 16.0).to(torch.bfloat16)
    for rep in range(2):
        for name, x, flags in (("big, GEMM layout", big, fp4.LAYOUT_GEMM), ("small, canonical", small, 0),
                               ("small, GEMM layout", small, fp4.LAYOUT_GEMM), ("big, canonical", big, 0)):
            say(f"static scratch vs workspace: {name}, NVFP4 b=16, round {rep}")
            (c0, s0, t0), (c1, s1, t1) = _pair(fp4, x, 16, NV, flags)
            assert float(t0[0]) > 0 and torch.equal(t0, t1)
            assert torch.equal(s0, s1) and torch.equal(c0, c1)
    # formats and modes that need no scratch go through the same entry point
    (c0, s0, _), (c1, s1, _) = _pair(fp4, big, 32, MX, fp4.LAYOUT_GEMM)
    assert torch.equal(s0, s1) and torch.equal(c0, c1)
    ts = torch.tensor([2.0 ** -7], dtype=torch.float32, device="cuda")
    cb, sb = fp4.packed_bytes(8, 1024, NV, 0)
    ca, sa = torch.empty(cb, dtype=torch.uint8, device="cuda"), torch.empty(sb, dtype=torch.uint8, device="cuda")
    fp4.fp4_rotate_quantize_static(small, 16, NV, flags=fp4.STATIC_TENSOR_SCALE, tensor_scale=ts, codes=ca, scales=sa)
    cr, sr, _ = fp4.fp4_rotate_quantize(small, 16, NV, tensor_scale=ts)
    torch.cuda.synchronize()
    assert torch.equal(ca, cr) and torch.equal(sa, sr) and float(ts[0]) == 2.0 ** -7


def test_static_scratch_entry_point_rejects_what_is_too_big_before_any_launch(fp4):
    fake = 0x10000   # non-NULL, aligned, never dereferenced: the call is rejected on the host
    L = fp4.lib
    assert L.fp4_rotate_quantize_static(fake, 1 << 20, 1 << 17, 16, NV, fake, fake, fake, 0, None) == 2     # 2^37 elements
    assert L.fp4_rotate_quantize_static(fake, 16, 48, 32, MX, fake, fake, None, 0, None) == 2               # K % 32
    assert L.fp4_rotate_quantize_static(None, 16, 128, 32, MX, fake, fake, None, 0, None) == 1
    assert L.fp4_rotate_quantize_static(fake, 16, 128, 16, NV, fake, fake, None, 0, None) == 1              # NVFP4 needs the tensor-scale pointer
