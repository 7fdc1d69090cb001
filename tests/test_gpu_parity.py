"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element.

Bars (from the benchmark spec):
  * quantizer fed the oracle's fp32 rotated values: codes, scales and tensor scale BIT-EXACT;
  * end to end (library's own rotation): <= 1e-4 of codes differ, each by <= 1 grid step;
  * GEMM: |gpu - oracle| <= 1e-3 * sum_k |a*w| per element (plus half a bf16 ulp of the value for bf16 output;
    the fp32-output runs check the bare bound).
"""
import os
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, compare_codes, gemm_layout_to_canonical, to_dev, to_dev_bf16, unpack

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


def rand_bits(rng, shape, spread=3.0):
    x = rng.standard_normal(shape) * np.exp(rng.uniform(-spread, spread, shape))
    return inputs.f32_to_bf16_bits(x.astype(np.float32))


# ---------------------------------------------------------------- quantizer, mode (i): bit-exact
@pytest.mark.parametrize("sw_codec", [False, True])
@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("b", [1, 16, 32, 64, 128])
def test_quantizer_bit_exact_on_oracle_rotation(fp4, oracle, fmt, b, sw_codec, knobs):
    import torch
    knobs(sw_codec=sw_codec)
    rng = np.random.default_rng(100 * b + fmt)
    M, K = 67, 1536                       # 100k elements: many work items, ragged last item
    xb = rand_bits(rng, (M, K))
    y = oracle.rotate(xb, b)
    # plant exact midpoints, zeros and a saturating value so that ties and edge codes are exercised
    y[0, :8] = [4.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0]
    y[1, 32:64] = 0.0
    y[2, 5] = -0.0
    ref_c, ref_s, ref_T = oracle.quantize(y, fmt)
    say(f"quantizer mode-i fmt={fmt} b={b} sw={sw_codec} M={M} K={K}")
    c, s, T = fp4.fp4_rotate_quantize(to_dev(y), 1, fmt)
    torch.cuda.synchronize()
    assert np.array_equal(np_(s).reshape(M, -1), ref_s)
    assert np.array_equal(np_(c).reshape(M, -1), ref_c)
    if fmt == NV:
        assert np_(T)[0] == ref_T


@pytest.mark.parametrize("fmt", [MX, NV])
def test_quantizer_bit_exact_bf16_no_rotation(fp4, oracle, fmt):
    """had_block = 1 on bf16 input is exact end to end (no irrational factor): bit-exact."""
    import torch
    rng = np.random.default_rng(7 + fmt)
    M, K = 33, 4096 + 512
    xb = rand_bits(rng, (M, K), 2.0)
    xb[3, 100:164] = 0
    ref_c, ref_s, ref_T, _ = oracle.rotate_quantize(xb, 1, fmt)
    say(f"quantizer b=1 bf16 fmt={fmt}")
    c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 1, fmt)
    torch.cuda.synchronize()
    assert np.array_equal(np_(s).reshape(M, -1), ref_s)
    assert np.array_equal(np_(c).reshape(M, -1), ref_c)
    if fmt == NV:
        assert np_(T)[0] == ref_T


# ---------------------------------------------------------------- quantizer, mode (ii): end to end
@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("b", [16, 32, 64, 128])
def test_rotate_quantize_end_to_end(fp4, oracle, fmt, b):
    import torch
    r = inputs.RECIPES[1 if fmt == MX else 4]
    M, K = 77, 2048 + 512
    xb = r.x(M, K, salt=b)
    ref_c, ref_s, ref_T, y = oracle.rotate_quantize(xb, b, fmt)
    say(f"rotate_quantize e2e fmt={fmt} b={b}")
    c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, fmt)
    torch.cuda.synchronize()
    if fmt == NV:
        assert abs(float(np_(T)[0]) - float(ref_T)) <= 2 * np.spacing(np.float32(ref_T))
        if np_(T)[0] != ref_T:
            # the library's fp32 rotation moved the tensor abs-max by an ulp: the oracle re-encodes its own rotated
            # values with the library's tensor scale and the comparison goes ahead
            ref_c, ref_s, _ = oracle.quantize(y, fmt, tensor_scale=float(np_(T)[0]))
    frac, flips = compare_codes(np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s, y, fmt)
    say(f"   differing codes: {frac:.2e}, scale flips: {flips}")


@pytest.mark.parametrize("b", [16, 64])
def test_rotate_quantize_nvfp4_static_tensor_scale(fp4, oracle, b):
    import torch
    r = inputs.RECIPES[4]
    M, K = 40, 1024
    xb = r.x(M, K, salt=3)
    sT = np.float32(2.0 ** -8)
    y = oracle.rotate(xb, b)
    ref_c, ref_s, ref_T = oracle.quantize(y, NV, tensor_scale=float(sT))
    say(f"nvfp4 static scale b={b}")
    ts = torch.tensor([sT], dtype=torch.float32, device="cuda")
    c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, NV, tensor_scale=ts)
    torch.cuda.synchronize()
    assert np_(T)[0] == sT
    compare_codes(np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s, y, NV)


@pytest.mark.parametrize("static", [False, True])
@pytest.mark.parametrize("M,K", [(1, 48), (3, 176), (5, 16), (7, 48), (2, 48)])
def test_nvfp4_block16_tensor_ending_in_half_a_32_vector(fp4, oracle, M, K, static):
    """NVFP4 with 16-element blocks accepts K = 16 * odd; with an odd row count the tensor then ends in half of the
    32-element vector the rotation kernel works in.  Every code and scale byte must be written (the outputs are
    pre-filled with a pattern no valid result holds everywhere) and the tail must count in the tensor abs-max: the
    largest element of the tensor is planted in the last 16 elements."""
    import torch
    rng = np.random.default_rng(1000 * M + K)
    xb = rand_bits(rng, (M, K), 1.0)
    x = inputs.bf16_bits_to_f32(xb)
    x[M - 1, K - 3] = 64.0 * np.abs(x).max()
    xb = inputs.f32_to_bf16_bits(x)
    y = oracle.rotate(xb, 16)
    say(f"nvfp4 b=16 half-vector tail M={M} K={K} static={static}")
    codes = torch.full((M * K // 2,), 0xEE, dtype=torch.uint8, device="cuda")
    scales = torch.full((M * K // 16,), 0xEE, dtype=torch.uint8, device="cuda")
    if static:
        sT = np.float32(2.0 ** -6)
        ref_c, ref_s, _ = oracle.quantize(y, NV, tensor_scale=float(sT))
        ts = torch.tensor([sT], dtype=torch.float32, device="cuda")
        c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 16, NV, tensor_scale=ts, codes=codes, scales=scales)
    else:
        ref_c, ref_s, ref_T = oracle.quantize(y, NV)
        c, s, T = fp4.fp4_rotate_quantize(to_dev_bf16(xb), 16, NV, codes=codes, scales=scales)
    torch.cuda.synchronize()
    if not static:
        # 1/sqrt(16) is exact and a 16-term sum of bf16 values with fp32 accumulation is within an ulp
        assert abs(float(np_(T)[0]) - float(ref_T)) <= 2 * np.spacing(np.float32(ref_T))
        if np_(T)[0] != ref_T:
            ref_c, ref_s, _ = oracle.quantize(y, NV, tensor_scale=float(np_(T)[0]))
    compare_codes(np_(c).reshape(M, -1), np_(s).reshape(M, -1), ref_c, ref_s, y, NV, max_frac=max(1e-4, 1.01 / (M * K)))   # (at most one code of a tiny tensor)
    assert np.array_equal(np_(s).reshape(M, -1), ref_s)


@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("b", [1, 16, 32, 64, 128])
def test_gemm_layout_is_a_permutation_of_canonical(fp4, fmt, b):
    """Same kernel, two output orders: un-shuffling the GEMM layout on the host gives the canonical bytes."""
    import torch
    r = inputs.RECIPES[1]
    M, K = 45, 1024 + 128                 # ragged row block (45 = 2*16 + 13), K/128 = 9 (not a multiple of 4)
    x = to_dev_bf16(r.x(M, K, salt=50 + b))
    say(f"gemm layout vs canonical fmt={fmt} b={b}")
    c0, s0, T0 = fp4.fp4_rotate_quantize(x, b, fmt)
    c1, s1, T1 = fp4.fp4_rotate_quantize(x, b, fmt, flags=fp4.LAYOUT_GEMM)
    torch.cuda.synchronize()
    cc, ss = gemm_layout_to_canonical(np_(c1), np_(s1), M, K, fmt)
    assert np.array_equal(cc, np_(c0).reshape(M, -1))
    assert np.array_equal(ss, np_(s0).reshape(M, -1))
    if fmt == NV:
        assert np_(T0)[0] == np_(T1)[0]


def test_quantize_weights_matches_rotate_quantize(fp4):
    import torch
    w = to_dev_bf16(inputs.RECIPES[1].w(96, 512))
    a = fp4.fp4_quantize_weights(w, 32, MX)
    b = fp4.fp4_rotate_quantize(w, 32, MX)
    torch.cuda.synchronize()
    assert torch.equal(a[0], b[0]) and torch.equal(a[1], b[1])


# ---------------------------------------------------------------- GEMM
def _gemm_case(fp4, oracle, fmt, M, N, K, seed, out_f32, layout_gemm):
    """Operands are the ORACLE's codes and scales; the product is checked against the oracle's fp64 product."""
    import torch
    rng = np.random.default_rng(seed)
    r = inputs.RECIPES[1 if fmt == MX else 4]
    b = 32 if fmt == MX else 16
    xb, wb = r.x(M, K, salt=seed), r.w(N, K, salt=seed)
    ac, asc, aT, _ = oracle.rotate_quantize(xb, b, fmt)
    wc, wsc, wT, _ = oracle.rotate_quantize(wb, b, fmt)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, fmt, aT), oracle.dequantize(wc, wsc, fmt, wT))
    say(f"gemm fmt={fmt} M={M} N={N} K={K} out_f32={out_f32} layout_gemm={layout_gemm}")
    flags = fp4.OUT_F32 if out_f32 else 0
    d = lambda a: to_dev(a.reshape(-1))
    ts = lambda v: None if v is None else torch.tensor([v], dtype=torch.float32, device="cuda")
    if layout_gemm:
        # let the library's quantizer produce GEMM-layout operands from the oracle's fp32 rotated values: they
        # are bit-identical to the oracle's codes (mode-i test), so the reference product is unchanged
        ya, yw = oracle.rotate(xb, b), oracle.rotate(wb, b)
        qa = fp4.fp4_rotate_quantize(to_dev(ya), 1, fmt, flags=fp4.LAYOUT_GEMM)
        qw = fp4.fp4_quantize_weights(to_dev(yw), 1, fmt, flags=fp4.LAYOUT_GEMM)
        out = fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, N, K, fmt,
                           flags=flags | fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
    else:
        out = fp4.fp4_gemm(d(ac), d(asc), ts(aT), d(wc), d(wsc), ts(wT), M, N, K, fmt, flags=flags)
    torch.cuda.synchronize()
    got = np_(out.float()).astype(np.float64)
    tol = 1e-3 * S
    if not out_f32:
        tol = tol + np.abs(Y) * 2.0 ** -8          # bf16 output rounding (half an ulp <= 2^-9 |y|), generous
    err = np.abs(got - Y)
    worst = float((err / (1e-3 * S + 1e-300)).max())
    say(f"   max err / (1e-3 S) = {worst:.3e}")
    assert np.all(err <= tol), f"worst ratio {worst}"
    return worst


@pytest.mark.parametrize("fmt", [MX, NV])
@pytest.mark.parametrize("M,N,K", [(64, 256, 512), (150, 328, 1152), (1, 4096, 4096), (16, 512, 2048), (300, 136, 128)])
def test_gemm_against_oracle_fp32_out(fp4, oracle, fmt, M, N, K):
    _gemm_case(fp4, oracle, fmt, M, N, K, seed=M + N + K, out_f32=True, layout_gemm=False)


@pytest.mark.parametrize("fmt", [MX, NV])
def test_gemm_gemm_layout_operands_bf16_out(fp4, oracle, fmt):
    _gemm_case(fp4, oracle, fmt, 200, 520, 1024 + 384, seed=5, out_f32=False, layout_gemm=True)


@pytest.mark.parametrize("variant", [1, 2, 3, 4, 5, 6, 7, 8, 9, 10, 11, 12, 13, 14, 15, 16, 17, 18])
def test_gemm_mxfp4_every_tile_variant(fp4, oracle, variant, knobs):
    knobs(variant=variant)
    _gemm_case(fp4, oracle, MX, 272, 528, 1280, seed=variant, out_f32=True, layout_gemm=True)


@pytest.mark.parametrize("out_f32", [False, True])
@pytest.mark.parametrize("variant", [1, 2, 3])
def test_gemm_nvfp4_every_tile_variant(fp4, oracle, variant, out_f32, knobs):
    """128 x 128, 16 x 256 and 256 x 256 tiles of the dequantizing NVFP4 kernel on a ragged tile grid (last tile row and
    column partly outside: clamped row-blocks, masked stores), K not a multiple of 512."""
    knobs(variant=variant)
    _gemm_case(fp4, oracle, NV, 272, 528, 1280, seed=30 + variant, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("variant", [2, 5, 10, 13, 15, 17, 18])
def test_gemm_mxfp4_tile_variants_bf16_output_through_the_staged_epilogue(fp4, oracle, variant, knobs):
    """bf16 output goes through the LDS transpose of the epilogue, whose chunk swizzle depends on the wave tile's width
    (64, 96 and 128 columns here); ragged last tile row and column."""
    knobs(variant=variant)
    _gemm_case(fp4, oracle, MX, 272, 528, 1280, seed=80 + variant, out_f32=False, layout_gemm=True)


@pytest.mark.parametrize("variant", [17, 18])
@pytest.mark.parametrize("K", [128, 512, 896, 1024, 1152, 2048, 2176, 4224])
def test_gemm_mxfp4_eight_stage_ring_with_two_scale_buffers(fp4, oracle, K, variant, knobs):
    """The 128x128 tile with an eight-stage operand ring (for launches with fewer tiles than compute units): the scale
    batches alternate between two buffers and are requested eight steps ahead.  K / 128 = 1, 4, 7 (shorter than the ring),
    8, 9 (one batch and the first step of the second), 16, 17, 33; scales that differ per row-block and K-step.  Variant 17:
    four waves of 64 x 64; variant 18: eight waves of 32 x 64."""
    import torch
    knobs(variant=variant)
    M, N = 272, 400
    rng = np.random.default_rng(8000 + K)

    def operand(rows):
        v = rng.standard_normal((rows, K))
        v *= 2.0 ** ((np.arange(rows)[:, None] // 16 * 5) % 11 - 5)
        v *= 2.0 ** ((np.arange(K)[None, :] // 128 * 3) % 7 - 3)
        return v.astype(np.float32)

    ya, yw = operand(M), operand(N)
    ac, asc, _ = oracle.quantize(ya, MX)
    wc, wsc, _ = oracle.quantize(yw, MX)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    say(f"gemm eight-stage ring K={K}")
    qa = fp4.fp4_rotate_quantize(to_dev(ya), 1, MX, flags=fp4.LAYOUT_GEMM | fp4.INPUT_F32)
    qw = fp4.fp4_quantize_weights(to_dev(yw), 1, MX, flags=fp4.LAYOUT_GEMM | fp4.INPUT_F32)
    for fl in (fp4.OUT_F32, 0):
        out = fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, M, N, K, MX, flags=fl | fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
        torch.cuda.synchronize()
        err = np.abs(np_(out.float()).astype(np.float64) - Y)
        tol = 1e-3 * S + (0 if fl else np.abs(Y) * 2.0 ** -8)
        assert np.all(err <= tol), float((err / (1e-3 * S + 1e-300)).max())


@pytest.mark.parametrize("grid", [1, 2, 4])
@pytest.mark.parametrize("out_f32", [False, True])
def test_gemm_mxfp4_persistent_workgroups_walk_several_tiles(fp4, oracle, grid, out_f32, knobs):
    """Six 256x256 tiles on 1, 2 or 4 workgroups: every workgroup computes a sequence of tiles (uneven for 4), with
    the next tile's first stages loaded while the previous tile's results are stored."""
    knobs(variant=11)
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, 272, 528, 1280, seed=40 + grid, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("variant", [11, 12, 14, 16])
@pytest.mark.parametrize("K", [128, 256, 384, 1024, 1152, 3072])
@pytest.mark.parametrize("grid", [1, 2])
def test_gemm_mxfp4_persistent_interior_tiles_overlap_their_stores(fp4, oracle, grid, K, variant, knobs):
    """All tiles interior (M, N multiples of the tile): every follow-on tile starts its main loop while the previous
    tile's stores are still draining; K = 128 ... 384 are the cases with fewer K-steps than the drain window."""
    knobs(variant=variant)
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, 512, 768, K, seed=60 + grid + K, out_f32=False, layout_gemm=True)


@pytest.mark.parametrize("variant", [11, 12, 14, 16])
@pytest.mark.parametrize("grid", [1, 3])
@pytest.mark.parametrize("out_f32", [False, True])
def test_gemm_mxfp4_persistent_variants_across_ragged_tiles(fp4, oracle, grid, out_f32, variant, knobs):
    """Every persistent tile shape on 1 and 3 workgroups over a ragged tile grid (K = 3072): uneven tile counts per
    workgroup, interior tiles followed by edge tiles (full wait) and the other way round, bf16 (staged) and fp32 (direct)
    epilogues."""
    knobs(variant=variant)
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, 528, 784, 3072, seed=90 + grid + variant, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("variant", [10, 11, 13, 3, 15, 17, 18])
@pytest.mark.parametrize("K", [640, 1152, 2176])
def test_gemm_mxfp4_scales_that_differ_per_row_block_and_k_block(fp4, oracle, variant, K, knobs):
    """The tile kernels fetch scale bytes in batches (eight K-steps of two row-blocks per copy with four stages, four
    K-steps of one row-block with three): every 16-row block and every 128-wide K-block gets its own magnitude, so a byte
    taken from the wrong row-block, K-step or batch changes a product by a power of two.  K / 128 = 5, 9, 17: batches that
    end inside the last scale dword, ragged M and N."""
    import torch
    M, N = 272, 400
    rng = np.random.default_rng(7000 + K + variant)

    def operand(rows):
        v = rng.standard_normal((rows, K))
        v *= 2.0 ** ((np.arange(rows)[:, None] // 16 * 5) % 11 - 5)          # per row-block
        v *= 2.0 ** ((np.arange(K)[None, :] // 128 * 3) % 7 - 3)             # per K-step
        return v.astype(np.float32)

    ya, yw = operand(M), operand(N)
    ac, asc, _ = oracle.quantize(ya, MX)
    wc, wsc, _ = oracle.quantize(yw, MX)
    assert len(np.unique(asc)) >= 12
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    knobs(variant=variant)
    say(f"gemm scale batches variant={variant} K={K}")
    qa = fp4.fp4_rotate_quantize(to_dev(ya), 1, MX, flags=fp4.LAYOUT_GEMM | fp4.INPUT_F32)
    qw = fp4.fp4_quantize_weights(to_dev(yw), 1, MX, flags=fp4.LAYOUT_GEMM | fp4.INPUT_F32)
    out = fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, M, N, K, MX, flags=fp4.OUT_F32 | fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
    torch.cuda.synchronize()
    err = np.abs(np_(out).astype(np.float64) - Y)
    assert np.all(err <= 1e-3 * S), float((err / (1e-3 * S + 1e-300)).max())


@pytest.mark.parametrize("grid", [1, 3])
@pytest.mark.parametrize("M,N,K,out_f32", [(1, 400, 512, True), (16, 784, 2176, False), (9, 1040, 4096, False), (16, 272, 640, True),
                                           (3, 200, 128, False), (17, 400, 512, False), (40, 784, 2176, True), (64, 1040, 4096, False),
                                           (33, 200, 128, True), (56, 1000, 384, False)])
def test_gemm_mxfp4_persistent_weight_streaming_kernel(fp4, oracle, grid, M, N, K, out_f32, knobs):
    """Up to 16 tokens on MXFP4 go to the persistent weight-streaming kernel when there are more 16-column blocks than
    resident workgroups (or several batches of K per wave); a grid cap of 1 or 3 workgroups makes every workgroup walk
    many row-blocks with the next batch's loads in flight across the reduction: K / 128 = 1, 4, 5, 17, 32 covers waves
    without a K share, one batch and several batches per row-block (X resident in registers / travelling with W), odd
    batch counts (the two register buffers swap roles between row-blocks), ragged N.  With 17 to 64 tokens and K <= 4096 the
    same kernel keeps two to four 16-token blocks of X resident (ragged M: a token block past the end re-reads the last one;
    waves whose rows or columns lie outside the matrix issue no store, which the in-flight count must know)."""
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, M, N, K, seed=300 + grid + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("grid", [0, 2])
@pytest.mark.parametrize("M,N,K,out_f32", [(16, 336, 5120, False), (7, 200, 8192, True), (16, 176, 4736, False), (12, 208, 9344, False),
                                           (16, 240, 14336, True), (1, 160, 16384, False), (16, 144, 16512, False), (20, 336, 5120, True),
                                           (32, 176, 8192, False), (25, 208, 12288, False), (32, 144, 12416, True), (40, 336, 6272, False),
                                           (48, 176, 8192, True), (33, 144, 8320, False), (64, 208, 4224, False), (32, 144, 16384, False),
                                           (17, 160, 16512, False), (64, 208, 8192, True), (50, 176, 8320, False), (31, 192, 14336, False),
                                           (48, 176, 14336, False), (64, 144, 12288, True), (60, 160, 16384, False)])
def test_gemm_mxfp4_persistent_kernel_with_several_batches_of_resident_activations(fp4, oracle, grid, M, N, K, out_f32, knobs):
    """K above 4096: a wave's share of K is two to four batches of four fragments, and the activations of up to 32 / 64
    tokens stay in registers for K up to 16384 / 8192 (every batch index static: the loop body is batches x buffers
    steps).  K / 128 = 33, 37, 40, 49, 64, 73, 96, 97, 112, 128: shares that end inside a batch, waves with fewer batches than
    the others or none; one step past each limit: K = 8320 with three and four token blocks, and K = 8192 < K <= 16384 with
    33 to 64 tokens, run as two sets of workgroups with two token blocks each; K = 16512 takes the kernels that do not
    keep X resident.  Grid cap 2: every workgroup walks many row-blocks, so batches of the next row-block are
    requested while the current one is multiplied and reduced."""
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, M, N, K, seed=700 + M + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("grid,M,N,K,out_f32", [(0, 65, 400, 4096, False), (0, 128, 1000, 4096, True), (16, 96, 2056, 2048, False),
                                                (16, 100, 1160, 1152, True), (1, 81, 520, 3072, False), (0, 113, 6144, 4096, False),
                                                (16, 128, 4104, 1536, True), (0, 72, 12288, 3200, False), (0, 96, 272, 8192, False),
                                                (16, 128, 400, 6144, True), (0, 70, 144, 5120, False), (16, 81, 528, 8192, True),
                                                (0, 200, 1000, 4096, False), (24, 256, 528, 8192, True), (0, 300, 272, 5120, False),
                                                (32, 512, 400, 4096, False), (0, 130, 8192, 4096, False)])
def test_gemm_mxfp4_65_to_512_tokens_on_sets_of_persistent_workgroups(fp4, oracle, grid, M, N, K, out_f32, knobs):
    """65 to 512 tokens on a narrow MXFP4 layer with 1024 < K <= 8192 (sets x N <= 32768): the persistent weight-streaming
    kernel runs as two to eight sets of workgroups, each with three or four 16-token blocks of X in registers (the last
    set's last blocks can lie past the end of M and are then neither loaded nor stored); a grid cap makes 8 walkers per
    set take many row-blocks each; ragged N, waves without a K share (K / 128 = 9, 12), fp32 and bf16 output."""
    knobs(grid=grid)
    _gemm_case(fp4, oracle, MX, M, N, K, seed=500 + M + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("grid", [0, 1, 3])
@pytest.mark.parametrize("M,N,K,out_f32", [(1, 400, 128, True), (16, 784, 384, False), (9, 1040, 1024, False), (16, 272, 1152, True),
                                           (3, 200, 2176, False), (16, 336, 4224, False), (12, 528, 8192, True), (16, 144, 8320, False),
                                           (16, 4112, 2048, False), (20, 1040, 1152, False), (40, 528, 8192, True), (64, 400, 4224, False),
                                           (33, 4112, 512, True), (100, 528, 4096, False), (128, 400, 1152, True), (200, 272, 2048, False),
                                           (256, 144, 8192, False), (65, 1040, 512, True), (400, 272, 2048, False), (512, 144, 1152, True)])
def test_gemm_nvfp4_persistent_kernel_with_fp16_resident_activations(fp4, oracle, grid, M, N, K, out_f32, knobs):
    """Up to 16 tokens on NVFP4 with K <= 8192: one workgroup per compute unit walks the row-blocks of W, its waves' shares
    of the activations dequantized once to fp16 and kept in registers, W in batches of two fragments with two batches in
    flight.  K / 128 = 1, 3, 8, 9, 17, 33, 64: one to four batches per row-block, shares that end inside a batch, waves
    without a share; K = 8320 is one step past the limit (the one-shot kernels); a grid of 1 or 3 workgroups makes each
    walk many row-blocks; ragged N, fp32 and bf16 output.  17 to 64 tokens on a narrow layer (N <= 12288): one set of such
    workgroups per 16-token block (two to four sets, the last block ragged); 65 to 512 tokens on a small layer: five to
    thirty-two sets."""
    knobs(grid=grid)
    _gemm_case(fp4, oracle, NV, M, N, K, seed=900 + grid + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("M,N,K,out_f32", [(1, 5000, 512, True), (16, 4944, 1152, False), (9, 5136, 128, False), (16, 8200, 640, True),
                                           (17, 5000, 512, False), (32, 4944, 1152, True), (40, 5136, 384, False), (64, 5000, 640, False),
                                           (50, 8200, 128, True), (16, 5000, 8320, False), (40, 5136, 8320, False), (17, 6160, 9216, True),
                                           (64, 400, 8448, False)])
def test_gemm_nvfp4_few_tokens_two_row_blocks_per_workgroup(fp4, oracle, M, N, K, out_f32):
    """Up to 64 tokens on NVFP4 with at least 0.6 workgroups per compute unit go to the kernel whose workgroups own two
    16-column blocks of the output (one dequantized X fragment per two W fragments): odd block counts (the last workgroup
    re-reads the last block and stores it once), ragged N, K / 128 = 1, 3, 4, 5, 9 (waves without a K share, ragged tails of
    the load batches), one to four 16-token blocks with ragged M (a token block past the end re-reads the last one).
    K / 128 = 65, 66, 72 with at most one workgroup per compute unit: the instantiations that request the next batch of
    fragments before they multiply the current one (two row-blocks per workgroup for N = 5000 ... 6160, one for N = 400)."""
    _gemm_case(fp4, oracle, NV, M, N, K, seed=4100 + N + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("M,N,K,out_f32", [(33, 5000, 512, False), (48, 4944, 1152, True), (64, 5136, 384, False), (50, 8200, 128, True)])
def test_gemm_mxfp4_three_and_four_token_blocks_two_row_blocks_per_workgroup(fp4, oracle, M, N, K, out_f32):
    """33 to 64 tokens on MXFP4 with at least 0.6 workgroups per compute unit (and N < 16384): the kernel whose workgroups
    own two 16-column blocks, so that every X fragment read from L2 serves two W fragments.  Ragged M, N, odd block counts,
    K / 128 = 1, 3, 4, 9."""
    _gemm_case(fp4, oracle, MX, M, N, K, seed=5100 + N + K, out_f32=out_f32, layout_gemm=True)


@pytest.mark.parametrize("M,N,K,out_f32", [(129, 400, 8320, True), (128, 1024, 14336, False), (200, 1000, 12416, False), (300, 272, 16512, True),
                                           (512, 520, 9088, False)])
def test_gemm_mxfp4_split_k(fp4, oracle, M, N, K, out_f32):
    """More than 64 tokens against a narrow layer with a long K: with the optional workspace the tiles' K ranges are
    shared by several workgroups (fp32 partials, added in split order).  Ragged M and N, K / 128 = 65, 71, 97, 112, 129
    (a last split of one K-step; splits that end inside a scale batch of eight steps), both output types; the same call
    with the minimum workspace runs unsplit and must meet the same bound."""
    import torch
    r = inputs.RECIPES[1]
    xb, wb = r.x(M, K, salt=M + K), r.w(N, K, salt=M + K)
    ya, yw = oracle.rotate(xb, 32), oracle.rotate(wb, 32)
    ac, asc, _ = oracle.quantize(ya, MX)
    wc, wsc, _ = oracle.quantize(yw, MX)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    qa = fp4.fp4_rotate_quantize(to_dev(ya), 1, MX, flags=fp4.LAYOUT_GEMM)
    qw = fp4.fp4_quantize_weights(to_dev(yw), 1, MX, flags=fp4.LAYOUT_GEMM)
    gfl = fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM | (fp4.OUT_F32 if out_f32 else 0)
    full = fp4.workspace_bytes(fp4.OP_GEMM_SPLIT_K, M, N, K, MX, gfl)
    assert fp4.workspace_bytes(fp4.OP_GEMM, M, N, K, MX, gfl) == 0 and full >= 2 * M * N * 4   # these shapes do split
    say(f"gemm split-K M={M} N={N} K={K} out_f32={out_f32}: {full // (M * N * 4)} splits")
    tol = 1e-3 * S + (0 if out_f32 else np.abs(Y) * 2.0 ** -8)
    for name, ws in (("split", None), ("unsplit", torch.empty(16, dtype=torch.uint8, device="cuda"))):
        out = fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, M, N, K, MX, flags=gfl, workspace=ws)
        torch.cuda.synchronize()
        err = np.abs(np_(out.float()).astype(np.float64) - Y)
        assert np.all(err <= tol), (name, float((err / (1e-3 * S + 1e-300)).max()))


@pytest.mark.parametrize("M,N,K,out_f32", [(65, 400, 8320, True), (128, 1024, 14336, False), (200, 1000, 10368, False), (300, 528, 16512, True),
                                           (520, 1040, 4096, False), (600, 520, 2048, True)])
def test_gemm_nvfp4_split_k(fp4, oracle, M, N, K, out_f32):
    """The NVFP4 many-token kernel with its K range shared by several workgroups (optional workspace): ragged M and N,
    K / 64 = 32, 64, 130, 162, 224, 258 (a last split of two K-steps of 64, i.e. one fragment; ragged last splits; short K in
    parts of eight steps on 128 x 128 tiles), both output types; the same call with the minimum workspace runs unsplit and must meet the same bound."""
    import torch
    r = inputs.RECIPES[4]
    xb, wb = r.x(M, K, salt=M + K), r.w(N, K, salt=M + K)
    ya, yw = oracle.rotate(xb, 16), oracle.rotate(wb, 16)
    ac, asc, aT = oracle.quantize(ya, NV)
    wc, wsc, wT = oracle.quantize(yw, NV)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, NV, aT), oracle.dequantize(wc, wsc, NV, wT))
    qa = fp4.fp4_rotate_quantize(to_dev(ya), 1, NV, flags=fp4.LAYOUT_GEMM)
    qw = fp4.fp4_quantize_weights(to_dev(yw), 1, NV, flags=fp4.LAYOUT_GEMM)
    assert np_(qa[2])[0] == aT and np_(qw[2])[0] == wT
    gfl = fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM | (fp4.OUT_F32 if out_f32 else 0)
    base = fp4.workspace_bytes(fp4.OP_GEMM, M, N, K, NV, gfl)
    full = fp4.workspace_bytes(fp4.OP_GEMM_SPLIT_K, M, N, K, NV, gfl)
    assert full - base >= 2 * M * N * 4                      # these shapes do split
    say(f"nvfp4 gemm split-K M={M} N={N} K={K} out_f32={out_f32}: {(full - base) // (M * N * 4)} splits")
    tol = 1e-3 * S + (0 if out_f32 else np.abs(Y) * 2.0 ** -8)
    for name, nbytes in (("split", full), ("unsplit", base)):
        ws = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
        out = fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, N, K, NV, flags=gfl, workspace=ws)
        torch.cuda.synchronize()
        err = np.abs(np_(out.float()).astype(np.float64) - Y)
        assert np.all(err <= tol), (name, float((err / (1e-3 * S + 1e-300)).max()))


def test_gemm_mxfp4_exact_on_small_integers(fp4, oracle):
    """With scale bytes chosen freely and on-grid codes, 4*a*w are small integers: the fp32 accumulator must be
    EXACT (any summation order), and distinct scales per K-group pin the scale-to-group wiring."""
    import torch
    rng = np.random.default_rng(99)
    M, N, K = 48, 80, 1024
    ac = rng.integers(0, 256, (M, K // 2), dtype=np.uint8)
    wc = rng.integers(0, 256, (N, K // 2), dtype=np.uint8)
    asc = rng.integers(126, 129, (M, K // 32)).astype(np.uint8)
    wsc = rng.integers(126, 130, (N, K // 32)).astype(np.uint8)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, MX), oracle.dequantize(wc, wsc, MX))
    assert np.abs(S).max() * 16 < 2.0 ** 24      # every term is a multiple of 2^-4: all partial sums are exact in fp32
    say("gemm exact integers")
    out = fp4.fp4_gemm(to_dev(ac.reshape(-1)), to_dev(asc.reshape(-1)), None, to_dev(wc.reshape(-1)), to_dev(wsc.reshape(-1)),
                       None, M, N, K, MX, flags=fp4.OUT_F32)
    torch.cuda.synchronize()
    assert np.array_equal(np_(out).astype(np.float64), Y)


def test_gemm_selector_weights_return_decoded_activations(fp4, oracle):
    """W rows with a single 1.0 pick single columns of the decoded A: pins row/column roles and K order."""
    import torch
    rng = np.random.default_rng(5)
    M, N, K = 32, 64, 256
    ac = rng.integers(0, 256, (M, K // 2), dtype=np.uint8)
    asc = rng.integers(124, 130, (M, K // 32)).astype(np.uint8)
    wc = np.zeros((N, K // 2), dtype=np.uint8)
    picks = rng.integers(0, K, N)
    for n, k in enumerate(picks):
        wc[n, k // 2] = 2 << (4 * (k & 1))         # code 2 = 1.0
    wsc = np.full((N, K // 32), 127, dtype=np.uint8)
    A = oracle.dequantize(ac, asc, MX)
    say("gemm selector")
    out = fp4.fp4_gemm(to_dev(ac.reshape(-1)), to_dev(asc.reshape(-1)), None, to_dev(wc.reshape(-1)), to_dev(wsc.reshape(-1)),
                       None, M, N, K, MX, flags=fp4.OUT_F32)
    torch.cuda.synchronize()
    assert np.array_equal(np_(out).astype(np.float64), A[:, picks])


# ---------------------------------------------------------------- whole path
@pytest.mark.parametrize("fmt,b", [(MX, 32), (NV, 16), (MX, 128), (MX, 64), (MX, 16)])
def test_linear_layer_whole_path(fp4, oracle, fmt, b):
    """bf16 X, W -> rotate+quantize (GEMM layout) -> FP4 GEMM -> bf16, all on the GPU, against the oracle run on
    the same bits.  The library's own codes are checked against the oracle's by the end-to-end rule; the product
    is checked against the oracle's product of the LIBRARY's codes (so one differing code cannot hide in the
    GEMM tolerance, nor break it)."""
    import torch
    r = inputs.RECIPES[1 if fmt == MX else 4]
    M, N, K = 64, 384, 4096
    xb, wb = r.x(M, K), r.w(N, K)
    say(f"whole path fmt={fmt} b={b}")
    qa = fp4.fp4_rotate_quantize(to_dev_bf16(xb), b, fmt, flags=fp4.LAYOUT_GEMM)
    qw = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, fmt, flags=fp4.LAYOUT_GEMM)
    out = fp4.fp4_gemm(qa[0], qa[1], qa[2], qw[0], qw[1], qw[2], M, N, K, fmt, flags=fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM)
    torch.cuda.synchronize()
    ac, asc = gemm_layout_to_canonical(np_(qa[0]), np_(qa[1]), M, K, fmt)
    wc, wsc = gemm_layout_to_canonical(np_(qw[0]), np_(qw[1]), N, K, fmt)
    rac, rasc, raT, ya = oracle.rotate_quantize(xb, b, fmt)
    rwc, rwsc, rwT, yw = oracle.rotate_quantize(wb, b, fmt)
    aT = None if fmt == MX else np_(qa[2])[0]
    wT = None if fmt == MX else np_(qw[2])[0]
    if fmt == NV:
        assert abs(float(aT) - float(raT)) <= 2 * np.spacing(raT) and abs(float(wT) - float(rwT)) <= 2 * np.spacing(rwT)
    if fmt == MX or (aT == raT and wT == rwT):
        compare_codes(ac, asc, rac, rasc, ya, fmt)
        compare_codes(wc, wsc, rwc, rwsc, yw, fmt)
    Y, S = oracle.matmul(oracle.dequantize(ac, asc, fmt, aT), oracle.dequantize(wc, wsc, fmt, wT))
    got = np_(out.float()).astype(np.float64)
    assert np.all(np.abs(got - Y) <= 1e-3 * S + np.abs(Y) * 2.0 ** -8)
    # and the oracle's own end result is within the same bound of the GPU's (codes differ in <= 1e-4 of places)
    Y0, S0 = oracle.linear(xb, wb, b, fmt)
    assert np.mean(np.abs(got - Y0) <= 1e-3 * S0 + np.abs(Y0) * 2.0 ** -8) > 0.999


# ---------------------------------------------------------------- edge cases
def test_zero_input_and_extreme_magnitudes(fp4, oracle):
    import torch
    M, K = 16, 256
    x = np.zeros((M, K), dtype=np.float32)
    x[1] = 3.0e38
    x[2] = 1e-40
    x[3, ::2] = -1e-38
    x[4, 7] = 2.0 ** -126
    for fmt in (MX,):
        ref_c, ref_s, _ = oracle.quantize(x, fmt)
        say(f"extremes fmt={fmt}")
        c, s, _ = fp4.fp4_rotate_quantize(to_dev(x), 1, fmt)
        torch.cuda.synchronize()
        assert np.array_equal(np_(s).reshape(M, -1), ref_s)
        assert np.array_equal(np_(c).reshape(M, -1), ref_c)
    z = np.zeros((M, K), dtype=np.float32)
    c, s, T = fp4.fp4_rotate_quantize(to_dev(z), 1, NV)
    torch.cuda.synchronize()
    assert np_(T)[0] == 0 and not np_(c).any() and not np_(s).any()


def test_results_are_deterministic(fp4):
    import torch
    r = inputs.RECIPES[1]
    x = to_dev_bf16(r.x(128, 1024))
    w = to_dev_bf16(r.w(256, 1024))
    outs = []
    for _ in range(2):
        qa = fp4.fp4_rotate_quantize(x, 32, MX, flags=fp4.LAYOUT_GEMM)
        qw = fp4.fp4_quantize_weights(w, 32, MX, flags=fp4.LAYOUT_GEMM)
        outs.append(fp4.fp4_gemm(qa[0], qa[1], None, qw[0], qw[1], None, 128, 256, 1024, MX,
                                 flags=fp4.A_LAYOUT_GEMM | fp4.W_LAYOUT_GEMM).clone())
    torch.cuda.synchronize()
    assert torch.equal(outs[0].view(torch.int16), outs[1].view(torch.int16))


def _few_token_cases():
    # (FP4MR_FUZZ_SEED / FP4MR_FUZZ_CASES: other seeds and more cases for a longer run by hand)
    rng = np.random.default_rng(int(os.environ.get("FP4MR_FUZZ_SEED", "20251128")))
    out = []
    for i in range(int(os.environ.get("FP4MR_FUZZ_CASES", "48"))):
        fmt = MX if i % 3 else NV
        M = int(rng.choice([1, 5, 16, 17, 31, 32, 33, 47, 48, 50, 64, 65, 80, 97, 128, 129, 200, 256, 300, 400, 512]))
        N = int(rng.choice([16, 40, 136, 264, 520, 1032, 2056, 4104]))
        K = 128 * int(rng.choice([1, 2, 3, 4, 7, 8, 9, 16, 24, 31, 32, 33, 40, 56, 63, 64, 65, 72, 96, 112, 128, 130]))
        if M * N * K > 6.0e9:
            N = 264
        out.append((i, fmt, M, N, K, bool(rng.integers(0, 2)), int(rng.choice([0, 0, 1, 5, 24]))))
    return out


@pytest.mark.parametrize("case", _few_token_cases(), ids=lambda c: f"{c[0]}-fmt{c[1]}-M{c[2]}-N{c[3]}-K{c[4]}-{'f32' if c[5] else 'bf16'}-grid{c[6]}")
def test_gemm_few_token_dispatch_on_seeded_random_shapes(fp4, oracle, case, knobs):
    """Seeded random shapes across the few-token dispatch: one to 512 tokens, K / 128 from 1 to 130, both formats, ragged N,
    with and without a cap on the persistent grid -- one-shot kernels (with and without the prefetching register set), the
    persistent kernels with one to four resident token blocks and one to four batches per row-block, two to eight sets of
    them, the NVFP4 kernels with fp16-resident activations, the kernel whose X fragments travel with W, and the tile kernels
    where none of them takes the shape."""
    i, fmt, M, N, K, out_f32, grid = case
    knobs(grid=grid)
    _gemm_case(fp4, oracle, fmt, M, N, K, seed=6000 + i, out_f32=out_f32, layout_gemm=True)
