"""The hot path under HIP-graph capture: rotate+quantize and the product recorded once and replayed on new activations must
give, on every replay, exactly what the same calls give eagerly.  (The library records kernel launches only -- no memset or
copy nodes -- and keeps no state between calls beyond what the caller's workspace holds within one call.)"""
import sys

import pytest

from tests.gpu_util import MX, NV

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


@pytest.mark.parametrize("fmt,M,N,K", [(MX, 16, 1040, 4096), (MX, 128, 528, 4096), (MX, 128, 272, 14336), (MX, 300, 784, 1024),
                                       (MX, 1024, 1040, 512), (NV, 16, 528, 8192), (NV, 40, 1040, 1152), (NV, 16, 272, 14336),
                                       (NV, 256, 528, 8320)])
def test_graph_replays_equal_the_eager_calls(fp4, fmt, M, N, K):
    """Persistent few-token kernels (one set, several sets, fp16-resident NVFP4), the tile kernels with and without the
    split-K workspace, the NVFP4 many-token kernel with its fp16 pre-pass and split, and the NVFP4 quantizer's two passes
    (tensor scale through the workspace): three different activation tensors, two rounds of replays, eager work and
    synchronisation between the replays, every output compared bit for bit."""
    import torch
    b = 32 if fmt == MX else 16
    GL = fp4.LAYOUT_GEMM
    gfl = fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM
    gen = torch.Generator(device="cuda").manual_seed(1000 + M + K)
    w = (torch.randn(N, K, device="cuda", generator=gen) * 0.02).to(torch.bfloat16)
    wc, wsc, wts = fp4.fp4_quantize_weights(w, b, fmt, flags=GL)
    xs = [(torch.randn(M, K, device="cuda", generator=gen) * (0.5 + i)).to(torch.bfloat16) for i in range(3)]
    x = torch.empty_like(xs[0])
    cb, sb = fp4.packed_bytes(M, K, fmt, GL)
    codes = torch.empty(cb, dtype=torch.uint8, device="cuda")
    scales = torch.empty(sb, dtype=torch.uint8, device="cuda")
    ts = torch.empty(1, dtype=torch.float32, device="cuda") if fmt == NV else None
    wsq = torch.empty(max(fp4.workspace_bytes(fp4.OP_ROTATE_QUANTIZE, M, 0, K, fmt, GL), 16), dtype=torch.uint8, device="cuda")
    wsg = torch.empty(max(fp4.workspace_bytes(fp4.OP_GEMM_SPLIT_K, M, N, K, fmt, gfl), 16), dtype=torch.uint8, device="cuda")
    out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
    say(f"graph fmt={fmt} M={M} N={N} K={K}")

    def step():
        st = torch.cuda.current_stream().cuda_stream
        rc = fp4.lib.fp4_rotate_quantize(x.data_ptr(), M, K, b, fmt, codes.data_ptr(), scales.data_ptr(), 0 if ts is None else ts.data_ptr(),
                                         wsq.data_ptr(), wsq.numel(), GL, st)
        assert rc == 0
        fp4.fp4_gemm(codes, scales, ts, wc, wsc, wts, M, N, K, fmt, flags=gfl, out=out, workspace=wsg)

    ref = []
    for xi in xs:
        x.copy_(xi)
        step()
        torch.cuda.synchronize()
        ref.append(out.clone())
    assert not torch.equal(ref[0], ref[1])

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        x.copy_(xs[0])
        step()
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step()
    torch.cuda.synchronize()
    for rnd in range(2):
        for i, xi in enumerate(xs):
            x.copy_(xi)
            out.zero_()
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref[i]), (rnd, i)
            # eager work of the program's own between the replays
            assert float(out.float().abs().sum().item()) > 0.0
