"""Shape sweep of fp4_gemm against the bf16 library GEMM (a tuning aid: where does which kernel family pay?).

    python -m paper_2509_23202_amd.sweep [--fmt mxfp4|nvfp4|both] [--shapes N,K ...] [--tokens M ...]

For every (format, N, K, M): time of fp4_gemm alone (operands already quantized, GEMM layout, the optional split-K workspace
given) and of torch.matmul on bf16 operands of the same shape.  Both are timed as HIP-graph replays whose calls cycle through
several identical copies of the weights (at least 400 MB in all), so every call streams its weights from HBM rather than
from the 256 MB last-level cache.  One line per (format, N, K): `M:ours_us/bf16_us=ratio`.
"""
import argparse

import torch

from . import binding as fp4


def graph_us(fn, n, reps=4):
    """Average time of one call in a replayed graph of fn(0) .. fn(n - 1), in microseconds."""
    st = torch.cuda.Stream()
    with torch.cuda.stream(st):
        for i in range(2):
            fn(i)
        st.synchronize()
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr, stream=st):
            for i in range(n):
                fn(i)
        for _ in range(2):
            gr.replay()
        st.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        for _ in range(reps):
            gr.replay()
        e1.record(st)
        st.synchronize()
    return e0.elapsed_time(e1) / (reps * n) * 1e3


DEFAULT_SHAPES = [(4096, 4096), (6144, 4096), (8192, 8192), (14336, 4096), (28672, 4096), (4096, 14336), (2048, 2048), (8192, 1024),
                  (10240, 8192), (8192, 28672), (16384, 6144), (57344, 8192)]
DEFAULT_TOKENS = [1, 16, 32, 64, 80, 96, 128, 192, 256, 384, 512, 1024, 2048]


def main():
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--fmt", default="both", choices=["mxfp4", "nvfp4", "both"])
    ap.add_argument("--shapes", nargs="*", default=None, help="N,K pairs")
    ap.add_argument("--tokens", nargs="*", type=int, default=None)
    args = ap.parse_args()
    shapes = DEFAULT_SHAPES if not args.shapes else [tuple(int(v) for v in s.split(",")) for s in args.shapes]
    tokens = args.tokens or DEFAULT_TOKENS
    fmts = [(fp4.MXFP4, 32, "mxfp4"), (fp4.NVFP4, 16, "nvfp4")]
    if args.fmt != "both":
        fmts = [f for f in fmts if f[2] == args.fmt]
    GL = fp4.LAYOUT_GEMM
    gfl = fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM
    print("format N K  M:fp4_gemm_us/bf16_gemm_us=ratio ...", flush=True)
    for fmt, b, name in fmts:
        for N, K in shapes:
            w = (torch.randn(N, K, device="cuda") * 0.02).to(torch.bfloat16)
            qw = fp4.fp4_quantize_weights(w, b, fmt, flags=GL)
            nc = max(2, min(24, int(400e6 / (N * K * 0.55)) + 1))
            copies = [(qw[0].clone(), qw[1].clone()) for _ in range(nc)]
            wts = [w] + [w.clone() for _ in range(max(2, min(8, int(400e6 / (N * K * 2)) + 1)) - 1)]
            row = []
            for M in tokens:
                x = torch.randn(M, K, device="cuda").to(torch.bfloat16)
                qa = fp4.fp4_rotate_quantize(x, b, fmt, flags=GL)
                out = torch.empty((M, N), dtype=torch.bfloat16, device="cuda")
                ws = torch.empty(max(fp4.workspace_bytes(fp4.OP_GEMM_SPLIT_K, M, N, K, fmt, gfl), 16), dtype=torch.uint8, device="cuda")
                n = max(12, nc) if M < 1024 else max(6, min(nc, 8))
                t = graph_us(lambda i: fp4.fp4_gemm(qa[0], qa[1], qa[2], copies[i % nc][0], copies[i % nc][1], qw[2], M, N, K, fmt,
                                                    flags=gfl, out=out, workspace=ws), n)
                tb = graph_us(lambda i: torch.matmul(x, wts[i % len(wts)].t(), out=out), n)
                row.append(f"{M}:{t:.1f}/{tb:.1f}={tb / t:.2f}")
            print(name, N, K, " ".join(row), flush=True)
            del w, qw, copies, wts


if __name__ == "__main__":
    main()
