"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (GEMM-layout operands, default
tile selection), on samples the oracle can compute row by row: MXFP4 rows are quantized independently, so a sample
of rows of X and W is re-encoded by the oracle and the corresponding sub-block of Y recomputed in fp64.
NVFP4 needs the tensor abs-max: the oracle rotates the whole tensor for it (cheap) and encodes the sampled rows."""
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
    assert torch.cuda.is_available()
    from paper_2509_23202_amd import binding
    return binding


def np_(t):
    return t.detach().cpu().numpy()


def sample_rows(n, count, rng):
    """first / last rows, tile boundaries and random ones"""
    fixed = [0, 1, 15, 16, 255, 256, n - 257, n - 17, n - 16, n - 1]
    fixed = [v for v in fixed if 0 <= v < n]
    extra = rng.choice(n, size=max(0, count - len(fixed)), replace=False) if n > count else np.arange(n)
    return np.unique(np.concatenate([np.array(fixed, dtype=np.int64), extra.astype(np.int64)]))[:max(count, len(fixed))]


def oracle_rows(oracle, bits_rows, b, fmt, tensor_scale=None):
    y = oracle.rotate(bits_rows, b)
    c, s, T = oracle.quantize(y, fmt, tensor_scale)
    return c, s, T, y


def check_stripes(fp4, oracle, qa, qw, out, M, K, N, fmt, aT, wT):
    """Whole stripes of the output -- every column of 32 rows and every row of 32 columns -- against the oracle's fp64
    product of the library's own codes.  Rows 248..263 and columns 248..263 cross a 256-tile boundary; rows
    M/2 + 120 .. M/2 + 135 cross a wave-tile boundary inside a tile; columns 184..199 cross the 192-wide tile's boundary
    (and a 64-column wave-tile boundary of the square tile).  A defect confined to one wave-tile position anywhere
    along a tile row or column shows up here."""
    import torch
    rows = np.concatenate([np.arange(248, 264), np.arange(M // 2 + 120, M // 2 + 136)])
    cols = np.concatenate([np.arange(184, 200), np.arange(248, 264)])
    rows, cols = np.unique(rows[rows < M]), np.unique(cols[cols < N])
    a_codes, a_scales, w_codes, w_scales = np_(qa[0]), np_(qa[1]), np_(qw[0]), np_(qw[1])
    bad = 0
    ac, asc = gemm_layout_to_canonical(a_codes, a_scales, rows, K, fmt)
    A = oracle.dequantize(ac, asc, fmt, aT)
    got = np_(out[torch.from_numpy(rows).cuda()].float()).astype(np.float64)
    for n0 in range(0, N, 4096):          # all N weight rows, in slabs that keep the fp64 copy small
        n1 = min(N, n0 + 4096)
        wc, wsc = gemm_layout_to_canonical(w_codes, w_scales, np.arange(n0, n1), K, fmt)
        Y, S = oracle.matmul(A, oracle.dequantize(wc, wsc, fmt, wT))
        bad += int((np.abs(got[:, n0:n1] - Y) > 1e-3 * S + np.abs(Y) * 2.0 ** -8).sum())
    say(f"   {len(rows)} whole rows: {bad} outputs outside the bound")
    wc, wsc = gemm_layout_to_canonical(w_codes, w_scales, cols, K, fmt)
    W = oracle.dequantize(wc, wsc, fmt, wT)
    got = np_(out[:, torch.from_numpy(cols).cuda()].float()).astype(np.float64)
    for m0 in range(0, M, 4096):
        m1 = min(M, m0 + 4096)
        ac, asc = gemm_layout_to_canonical(a_codes, a_scales, np.arange(m0, m1), K, fmt)
        Y, S = oracle.matmul(oracle.dequantize(ac, asc, fmt, aT), W)
        bad += int((np.abs(got[m0:m1] - Y) > 1e-3 * S + np.abs(Y) * 2.0 ** -8).sum())
    say(f"   ... and {len(cols)} whole columns: {bad} outputs outside the bound in all")
    assert bad == 0


def check_layer(fp4, oracle, recipe, M, K, N, fmt, b, n_m=40, n_n=56, salt=0, stripes=False, extra_n=()):
    import torch
    rng = np.random.default_rng(K + N + M)
    xb, wb = recipe.x(M, K, salt=salt), recipe.w(N, K, salt=salt)
    say(f"full-size layer fmt={fmt} b={b} M={M} K={K} N={N}")
    qa = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, fmt, flags=fp4.LAYOUT_GEMM)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, fmt, flags=fp4.LAYOUT_GEMM)
    out = fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, N, K, fmt, flags=fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
    torch.cuda.synchronize()
    mi, ni = sample_rows(M, n_m, rng), sample_rows(N, n_n, rng)
    if len(extra_n):
        ni = np.unique(np.concatenate([ni, np.asarray([v for v in extra_n if 0 <= v < N], dtype=np.int64)]))
    ac, asc = gemm_layout_to_canonical(np_(qa[0]), np_(qa[1]), mi, K, fmt)
    wc, wsc = gemm_layout_to_canonical(np_(qw[0]), np_(qw[1]), ni, K, fmt)
    aT = wT = None
    if fmt == NV:
        # tensor scales from the oracle's own rotation of the whole tensors
        aT_ref = np.float32(np.abs(oracle.rotate(xb, b)).max()) / np.float32(2688.0)
        wT_ref = np.float32(np.abs(oracle.rotate(wb, b)).max()) / np.float32(2688.0)
        aT, wT = np_(qa[2])[0], np_(qw[2])[0]
        assert abs(float(aT) - float(aT_ref)) <= 2 * np.spacing(aT_ref)
        assert abs(float(wT) - float(wT_ref)) <= 2 * np.spacing(wT_ref)
        rac, rasc, _, ya = oracle_rows(oracle, xb[mi], b, fmt, float(aT))
        rwc, rwsc, _, yw = oracle_rows(oracle, wb[ni], b, fmt, float(wT))
    else:
        rac, rasc, _, ya = oracle_rows(oracle, xb[mi], b, fmt)
        rwc, rwsc, _, yw = oracle_rows(oracle, wb[ni], b, fmt)
    fa, _ = compare_codes(ac, asc, rac, rasc, ya, fmt)
    fw, _ = compare_codes(wc, wsc, rwc, rwsc, yw, fmt)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, fmt, aT), oracle.dequantize(wc, wsc, fmt, wT))
    got = np_(out[torch.from_numpy(mi).cuda()][:, torch.from_numpy(ni).cuda()].float()).astype(np.float64)
    err = np.abs(got - Y)
    tol = 1e-3 * S + np.abs(Y) * 2.0 ** -8
    say(f"   code mismatch X {fa:.1e} W {fw:.1e}; max err/(1e-3 S) = {float((err / (1e-3 * S)).max()):.3f}")
    assert np.all(err <= tol)
    if stripes:
        check_stripes(fp4, oracle, qa, qw, out, M, K, N, fmt, aT, wT)


@pytest.mark.parametrize("layer", [1, 3, 0, 2])
def test_prefill_layers_mxfp4(fp4, oracle, layer):
    """The four layers of the benchmark's step at M = 4096 in the launch configuration it times (layer 2 = gate_up:
    persistent 256 x 256 tiles, seven 32-step tiles per workgroup), sampled outputs plus whole stripes."""
    L = inputs.LLAMA3_8B_LAYERS[layer]
    check_layer(fp4, oracle, inputs.RECIPES[3], 4096, L.K, L.N, MX, 32, salt=layer, stripes=True)


@pytest.mark.parametrize("M", [1, 16])
@pytest.mark.parametrize("layer", [0, 1, 2, 3])
def test_decode_layers_mxfp4(fp4, oracle, layer, M):
    L = inputs.LLAMA3_8B_LAYERS[layer]
    check_layer(fp4, oracle, inputs.RECIPES[2], M, L.K, L.N, MX, 32, n_m=M, salt=layer)


@pytest.mark.parametrize("M", [17, 64])
def test_few_tokens_wide_layer_mxfp4(fp4, oracle, M):
    """More than one 16-token block on the widest layer (gate_up, N = 28672): the 64 x 256 tile kernel's territory."""
    L = inputs.LLAMA3_8B_LAYERS[2]
    check_layer(fp4, oracle, inputs.RECIPES[2], M, L.K, L.N, MX, 32, n_m=M, salt=40 + M)


def test_config1_whole_output(fp4, oracle):
    """configs[0]: M=64, K=N=4096, every output element."""
    check_layer(fp4, oracle, inputs.RECIPES[1], 64, 4096, 4096, MX, 32, n_m=64, n_n=4096)


@pytest.mark.parametrize("M", [16, 4096])
def test_nvfp4_70b_qkv_layer(fp4, oracle, M):
    L = inputs.LLAMA3_70B_LAYERS[0]
    check_layer(fp4, oracle, inputs.RECIPES[4], M, L.K, L.N, NV, 16, n_m=min(M, 32), n_n=48, stripes=M == 4096)


@pytest.mark.parametrize("li,M", [(1, 16), (1, 4096), (2, 16), (2, 4096)])
def test_nvfp4_70b_wide_and_deep_layers(fp4, oracle, li, M):
    """The other two layers of the NVFP4 configuration: gate_up (N = 57344) through the weight-streaming kernel, down
    (K = 28672) through both kernels."""
    L = inputs.LLAMA3_70B_LAYERS[li]
    check_layer(fp4, oracle, inputs.RECIPES[4], M, L.K, L.N, NV, 16, n_m=min(M, 32), n_n=48)


@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_block_sweep_2048_8192(fp4, oracle, b):
    check_layer(fp4, oracle, inputs.RECIPES[5], 2048, 8192, 8192, MX, b, n_m=24, n_n=32, salt=b)


def test_standalone_rotate_quantize_16384_8192(fp4, oracle):
    import torch
    r = inputs.RECIPES[6]
    M, K = 16384, 8192
    xb = r.x(M, K)
    say("standalone rotate+quantize 16384 x 8192 (Laplace, outlier channels)")
    for flags in (fp4.LAYOUT_GEMM, 0):
        c, s, _ = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 32, MX, flags=flags)
        torch.cuda.synchronize()
        mi = sample_rows(M, 64, np.random.default_rng(1))
        if flags:
            gc, gs = gemm_layout_to_canonical(np_(c), np_(s), mi, K, MX)
        else:
            gc, gs = np_(c).reshape(M, -1)[mi], np_(s).reshape(M, -1)[mi]
        rc, rs, _, y = oracle_rows(oracle, xb[mi], 32, MX)
        compare_codes(gc, gs, rc, rs, y, MX)


@pytest.mark.parametrize("fmt", [MX, NV])
def test_rotate_quantize_more_than_32768_row_blocks_and_short_k(fp4, oracle, fmt):
    """540000 tokens x K = 384: the fragment-order kernel's grid needs a second slice of row-blocks (33750 > 32768)
    and a work item (1024 K-elements) reaches past the end of K; ragged last row-block (540000 = 33750 * 16 exactly,
    so one more case with 540007 rows)."""
    import torch
    rng = np.random.default_rng(9)
    K = 384
    for M in (540000, 540007):
        x = (rng.standard_normal((M, K), dtype=np.float32) * np.exp(rng.uniform(-2, 2, (M, 1))).astype(np.float32))
        xb = inputs.f32_to_bf16_bits(x)
        del x
        say(f"tall tensor fmt={fmt} M={M} K={K}")
        c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 32, fmt, flags=fp4.LAYOUT_GEMM)
        torch.cuda.synchronize()
        mi = np.unique(np.concatenate([sample_rows(M, 48, rng), np.array([32768 * 16 - 1, 32768 * 16, 32768 * 16 + 17, M - 2])]))
        gc, gs = gemm_layout_to_canonical(np_(c), np_(s), mi, K, fmt)
        Tg = None if fmt == MX else float(np_(T)[0])
        if fmt == NV:
            T_ref = np.float32(np.abs(oracle.rotate(xb, 32)).max()) / np.float32(2688.0)
            assert abs(Tg - float(T_ref)) <= 2 * np.spacing(T_ref)
        rc, rs, _, y = oracle_rows(oracle, xb[mi], 32, fmt, Tg)
        compare_codes(gc, gs, rc, rs, y, fmt)
        del c, s


def test_persistent_gemm_with_edge_tiles_at_scale(fp4, oracle):
    """425 tiles of 256 x 256 on 256 workgroups, the last tile row and column ragged (M = 4113, N = 6152): interior
    tiles (stores draining under the next tile) and edge tiles (full wait) alternate inside one workgroup."""
    check_layer(fp4, oracle, inputs.RECIPES[3], 4113, 512, 6152, MX, 32, n_m=48, n_n=64, salt=77)


@pytest.mark.parametrize("M,N", [(2048, 8192), (4099, 14344)])
def test_short_k_layers_take_the_two_workgroups_per_unit_tiles(fp4, oracle, M, N):
    """K = 1024 with more 256 x 256 tiles than one round of compute units: the shape rule picks 128 x 256 tiles, two
    workgroups per unit -- one round for the first shape, persistent workgroups with ragged edge tiles for the second."""
    check_layer(fp4, oracle, inputs.RECIPES[3], M, 1024, N, MX, 32, n_m=48, n_n=64, salt=M)


@pytest.mark.parametrize("M,N", [(2048, 10240), (2053, 10248), (4000, 10200)])
def test_nvfp4_two_launch_split_of_the_tile_grid(fp4, oracle, M, N):
    """More 256 x 256 tiles than one round of compute units and a partial round left over: the shape rule runs the tile
    columns that fill whole rounds as 256 x 256 tiles and the remaining columns as 128 x 128 tiles in a second launch
    (ragged last tile row and column in the second and third case).  Columns either side of every multiple of 256
    that can be the seam between the two launches are sampled on purpose."""
    seams = [c * 256 + d for c in range(1, (N + 255) // 256) for d in (-1, 0)]
    check_layer(fp4, oracle, inputs.RECIPES[4], M, 512, N, NV, 16, n_m=48, n_n=96, salt=M, extra_n=seams)


@pytest.mark.parametrize("M,N", [(1024, 10240), (1000, 10200), (512, 8192)])
def test_nvfp4_narrow_tiles_when_wide_ones_are_about_one_round(fp4, oracle, M, N):
    """Between one 128 x 256 tile per compute unit and a round and a quarter of them the whole product runs as
    128 x 128 tiles (640, 640 with ragged edges, and 256 of them here); columns either side of every multiple of 128
    near the middle and the end of N are sampled on purpose."""
    seams = [c * 128 + d for c in (1, 2, N // 256, N // 128 - 1, (N - 1) // 128) for d in (-1, 0) if 0 <= c * 128 + d < N]
    check_layer(fp4, oracle, inputs.RECIPES[4], M, 512, N, NV, 16, n_m=48, n_n=96, salt=M + 5, extra_n=seams)
