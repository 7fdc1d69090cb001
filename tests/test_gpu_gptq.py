"""GPU parity of the MR-GPTQ sweep (fp4_gptq_quantize_weights) against the NumPy oracle (oracle/gptq.py).

The sweep rounds a running value that carries the accumulated updates of every earlier column; the kernel keeps it in
fp32, the oracle in fp64.  Where all the arithmetic is exact in both (dyadic weights and factor entries, errors pushed
one step only) the codes must be bit-exact.  On realistic inputs a rounding may flip where the running value sits
within fp32 noise of a grid midpoint, and a flip changes what later columns of that row see -- so the bar there is: the
scale bytes are the round-to-nearest ones bit for bit, nearly all codes equal the oracle's, and the quantity GPTQ
minimises, the layer's output error tr(dW H dW^T), is the oracle's within 1e-3 relative.
"""
import sys

import numpy as np
import pytest

from paper_2509_23202_amd import inputs
from tests.gpu_util import MX, NV, to_dev, to_dev_bf16, unpack

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


@pytest.fixture(scope="module")
def gptq():
    from oracle import gptq
    return gptq


def np_(t):
    return t.detach().cpu().numpy()


@pytest.mark.parametrize("N,K", [(5, 64), (70, 256), (150, 1088)])
def test_sweep_is_bit_exact_where_the_arithmetic_is_exact(fp4, oracle, gptq, N, K):
    """Weights on a 2^-6 lattice, no rotation, unit diagonal, and every even column (in visiting order) pushing its error
    onto a few later odd columns with factors +-2^-3, +-2^-4 (odd columns push nothing): every product and sum is exact
    in fp32, so the codes must equal the oracle's everywhere -- across the 64-column block boundaries and (K = 1088)
    the 512-column outer blocks of the update kernel, through a random visiting order, with ragged row groups."""
    import torch
    rng = np.random.default_rng(K)
    w = (rng.integers(-200, 201, (N, K)) / 64.0).astype(np.float32)
    wb = inputs.f32_to_bf16_bits(w)
    assert np.array_equal(inputs.bf16_bits_to_f32(wb), w)      # the lattice values are bf16 numbers
    perm = rng.permutation(K).astype(np.int32)
    U = np.eye(K, dtype=np.float32)
    for j in range(0, K, 2):
        for d, mag in ((1, 0.125), (3, 0.0625), (65, 0.125), (131, 0.0625), (513, 0.125), (701, 0.0625)):
            if j + d < K:
                U[j, j + d] = mag * rng.choice([-1.0, 1.0])
    y = oracle.rotate(wb, 1)
    _, scales, _ = oracle.quantize(y, MX)
    want, _ = gptq.sweep(y, scales, MX, None, U, perm)
    rtn, _, _ = oracle.quantize(y, MX)
    say(f"gptq exact lattice case N={N} K={K}")
    c, s, _ = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), 1, MX, to_dev(U), to_dev(perm))
    torch.cuda.synchronize()
    assert np.array_equal(np_(s).reshape(N, -1), scales)
    assert np.array_equal(np_(c).reshape(N, -1), want)
    assert (want != rtn).mean() > 0.02          # the pushed errors did change codes


@pytest.mark.parametrize("fmt", [MX, NV])
def test_diagonal_factor_gives_round_to_nearest(fp4, oracle, fmt):
    import torch
    N, K, b = 33, 512, 32
    wb = inputs.RECIPES[6].w(N, K, salt=9)
    U = np.diag(np.random.default_rng(1).uniform(0.5, 2.0, K)).astype(np.float32)
    say(f"gptq diagonal fmt={fmt}")
    c, s, T = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, fmt, to_dev(U), None)
    c0, s0, T0 = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, fmt)
    torch.cuda.synchronize()
    assert np.array_equal(np_(s), np_(s0))
    if fmt == NV:
        assert np_(T)[0] == np_(T0)[0]
    diff = unpack(np_(c).reshape(N, -1)) != unpack(np_(c0).reshape(N, -1))
    # MXFP4: w / s is exact both ways.  NVFP4: the quantizer multiplies by a rounded reciprocal, the sweep divides
    assert diff.mean() <= (0.0 if fmt == MX else 1e-4)


@pytest.mark.parametrize("fmt,policy,b", [(MX, "absmax", 32), (MX, "mse", 128), (MX, "round43", 32), (NV, "absmax", 16), (NV, "mse", 32),
                                          (NV, "mse_alt", 16), (NV, "mse_alt", 1)])
def test_sweep_matches_the_oracle_on_synthetic_hessians(fp4, oracle, gptq, fmt, policy, b):
    import torch
    N, K, T = 100, 512, 1024
    r = inputs.RECIPES[6]
    wb, xb = r.w(N, K, salt=40), r.x(T, K, salt=41)
    X = oracle.rotate(xb, b).astype(np.float64)
    H = X.T @ X
    perm = gptq.act_order(H).astype(np.int32)
    U = gptq.inverse_factor(H, perm, damp=1e-2).astype(np.float32)
    y = oracle.rotate(wb, b)
    if policy == "mse_alt":   # the grid of Ingredient 1 in full: group scales and tensor scale by alternating optimisation
        c_rtn, scales, sT, _ = oracle.quantize_nvfp4_alternating(y, 3)
    else:
        c_rtn, scales, sT = oracle.quantize(y, fmt, policy=policy)
    want, _ = gptq.sweep(y, scales, fmt, sT, U, perm)
    flags = {"absmax": 0, "mse": fp4.SCALE_MSE, "round43": fp4.SCALE_ROUND43, "mse_alt": fp4.SCALE_MSE | fp4.SCALE_FIT_TENSOR}[policy]
    say(f"gptq synthetic fmt={fmt} policy={policy} b={b}")
    c, s, Tg = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, fmt, to_dev(U), to_dev(perm), flags=flags)
    torch.cuda.synchronize()
    got_c, got_s = np_(c).reshape(N, -1), np_(s).reshape(N, -1)
    assert (got_s != scales).mean() <= 1e-3
    if fmt == NV:
        assert abs(float(np_(Tg)[0]) - float(sT)) <= 2 * np.spacing(np.float32(sT))
    rows_ok = (got_s == scales).all(axis=1)
    diff = unpack(got_c) != unpack(want)
    e_got = gptq.layer_error(y[rows_ok], got_c[rows_ok], scales[rows_ok], fmt, sT, H)
    e_ref = gptq.layer_error(y[rows_ok], want[rows_ok], scales[rows_ok], fmt, sT, H)
    e_rtn = gptq.layer_error(y[rows_ok], c_rtn[rows_ok], scales[rows_ok], fmt, sT, H)
    say(f"   codes differing from the oracle: {diff[rows_ok].mean():.2e}; layer error {e_got:.6e} vs oracle {e_ref:.6e} (round-to-nearest {e_rtn:.4e})")
    assert diff[rows_ok].mean() <= 1e-3
    assert abs(e_got - e_ref) <= 1e-3 * e_ref
    assert e_got < 0.8 * e_rtn


def test_gptq_on_the_fitted_scale_range(fp4, oracle, gptq):
    """MR-GPTQ with the scale byte fitted to the tensor's range as the fixed grid (appendix on MXFP scale fitting, table:
    MR-GPTQ on MXFP4-dagger): the grid is the library's own (bytes and the 256 scale values it publishes; its parity
    with the oracle's fit is tested with the quantizer), the sweep is compared with the oracle's sweep on that grid."""
    import torch
    b, N, K, T = 32, 100, 512, 1024
    r = inputs.RECIPES[6]
    wb, xb = r.w(N, K, salt=60), r.x(T, K, salt=61)
    X = oracle.rotate(xb, b).astype(np.float64)
    H = X.T @ X
    perm = gptq.act_order(H).astype(np.int32)
    U = gptq.inverse_factor(H, perm, damp=1e-2).astype(np.float32)
    y = oracle.rotate(wb, b)
    say("gptq on the fitted scale range")
    c, s, ts = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, MX, to_dev(U), to_dev(perm), flags=fp4.SCALE_FIT_RANGE)
    c0, s0, ts0 = fp4.fp4_quantize_weights(to_dev_bf16(wb), b, MX, flags=fp4.SCALE_FIT_RANGE)
    torch.cuda.synchronize()
    assert torch.equal(s, s0) and torch.equal(ts, ts0)          # the grid is the round-to-nearest call's, bit for bit
    got_c, q, table = np_(c).reshape(N, -1), np_(s).reshape(N, -1), np_(ts)[2:258].astype(np.float64)
    want, _ = gptq.sweep(y, q, MX, None, U, perm, table=table)
    diff = unpack(got_c) != unpack(want)
    e_got = gptq.layer_error(y, got_c, q, MX, None, H, table=table)
    e_ref = gptq.layer_error(y, want, q, MX, None, H, table=table)
    e_rtn = gptq.layer_error(y, np_(c0).reshape(N, -1), q, MX, None, H, table=table)
    say(f"   codes differing from the oracle: {diff.mean():.2e}; layer error {e_got:.6e} vs oracle {e_ref:.6e} (round-to-nearest {e_rtn:.4e})")
    assert diff.mean() <= 1e-3
    assert abs(e_got - e_ref) <= 1e-3 * e_ref
    assert e_got < 0.8 * e_rtn


def test_gptq_argument_validation(fp4):
    import torch
    w = torch.zeros((16, 128), dtype=torch.bfloat16, device="cuda")
    U = torch.eye(128, dtype=torch.float32, device="cuda")
    with pytest.raises(Exception):
        fp4.fp4_gptq_quantize_weights(w, 32, MX, U, None, flags=fp4.LAYOUT_GEMM)
    w96 = torch.zeros((16, 96), dtype=torch.bfloat16, device="cuda")
    U96 = torch.eye(96, dtype=torch.float32, device="cuda")
    with pytest.raises(Exception):
        fp4.fp4_gptq_quantize_weights(w96, 32, MX, U96, None)
    with pytest.raises(Exception):
        fp4.fp4_gptq_quantize_weights(w, 32, MX, U, None, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))


def synthetic_hessian(oracle, K, T, b, salt):
    xb = inputs.RECIPES[6].x(T, K, salt=salt)
    X = oracle.rotate(xb, b).astype(np.float64)
    return X.T @ X


@pytest.mark.parametrize("K", [64, 200, 320, 512, 1088])
def test_prepare_matches_the_oracle_order_and_factor(fp4, oracle, gptq, K):
    """Order: the same permutation as a stable descending sort of the diagonal.  Factor: fp32 blocked Cholesky and
    triangular inversion against NumPy in fp64 -- compared as matrices and through the identity U^T U A = I that
    defines it.  K = 200 and 320 have a ragged last block / an odd number of blocks (the doubling levels' tails)."""
    import torch
    b = 8 if K == 200 else 32
    H = synthetic_hessian(oracle, K, 2 * K + 100, b, salt=50 + K)
    H32 = H.astype(np.float32)
    say(f"gptq prepare K={K}")
    perm, U = fp4.fp4_gptq_prepare(to_dev(H32), 1e-2, True)
    torch.cuda.synchronize()
    perm, U = np_(perm), np_(U).astype(np.float64)
    want_perm = gptq.act_order(H32.astype(np.float64))
    assert np.array_equal(perm, want_perm)
    want_U = gptq.inverse_factor(H32.astype(np.float64), want_perm, damp=1e-2)
    assert np.all(np.tril(U, -1) == 0)
    rel = np.linalg.norm(U - want_U) / np.linalg.norm(want_U)
    A = H32.astype(np.float64)[np.ix_(want_perm, want_perm)]
    A[np.diag_indices(K)] += 1e-2 * np.mean(np.diag(A))
    resid = np.abs(U.T @ U @ A - np.eye(K)).max()
    say(f"   relative error of U {rel:.2e}; max |U^T U A - I| {resid:.2e}")
    assert rel <= 5e-4 and resid <= 2e-3
    # no re-ordering on request
    perm0, U0 = fp4.fp4_gptq_prepare(to_dev(H32), 1e-2, False)
    torch.cuda.synchronize()
    assert np.array_equal(np_(perm0), np.arange(K))
    want_U0 = gptq.inverse_factor(H32.astype(np.float64), np.arange(K), damp=1e-2)
    assert np.linalg.norm(np_(U0) - want_U0) / np.linalg.norm(want_U0) <= 5e-4


def test_prepare_orders_equal_diagonal_entries_by_index(fp4, gptq):
    import torch
    K = 128
    d = np.repeat(np.array([3.0, 1.0, 2.0, 3.0], dtype=np.float32), K // 4)
    H = np.diag(d).astype(np.float32)
    perm, U = fp4.fp4_gptq_prepare(to_dev(H), 1e-2, True)
    torch.cuda.synchronize()
    assert np.array_equal(np_(perm), gptq.act_order(H.astype(np.float64)))
    lam = 1e-2 * d.mean()
    assert np.allclose(np.diag(np_(U)), 1.0 / np.sqrt(d[np_(perm)] + lam), rtol=1e-6)


@pytest.mark.parametrize("fmt,policy", [(MX, "mse"), (NV, "absmax")])
def test_hessian_to_codes_entirely_on_the_gpu(fp4, oracle, gptq, fmt, policy):
    """H -> fp4_gptq_prepare -> fp4_gptq_quantize_weights against the oracle's whole quantizer (fp64 factor): same
    order, layer error within 1% of the oracle's and far below round-to-nearest."""
    import torch
    N, K, b = 96, 768, 32
    wb = inputs.RECIPES[6].w(N, K, salt=70)
    H = synthetic_hessian(oracle, K, 2048, b, salt=71).astype(np.float32)
    say(f"gptq whole path fmt={fmt} policy={policy}")
    perm, U = fp4.fp4_gptq_prepare(to_dev(H), 1e-2, True)
    flags = {"absmax": 0, "mse": fp4.SCALE_MSE}[policy]
    c, s, T = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, fmt, U, perm, flags=flags)
    torch.cuda.synchronize()
    H64 = H.astype(np.float64)
    want_c, want_s, sT, want_perm, _ = gptq.mr_gptq(wb, H64, b, fmt, policy=policy)
    assert np.array_equal(np_(perm), want_perm)
    got_c, got_s = np_(c).reshape(N, -1), np_(s).reshape(N, -1)
    ok = (got_s == want_s).all(axis=1)
    assert ok.mean() >= 0.98
    y = oracle.rotate(wb, b)
    c_rtn, _, _ = oracle.quantize(y, fmt, policy=policy)
    e_got = gptq.layer_error(y[ok], got_c[ok], want_s[ok], fmt, sT, H64)
    e_ref = gptq.layer_error(y[ok], want_c[ok], want_s[ok], fmt, sT, H64)
    e_rtn = gptq.layer_error(y[ok], c_rtn[ok], want_s[ok], fmt, sT, H64)
    diff = (unpack(got_c) != unpack(want_c))[ok].mean()
    say(f"   codes differing from the oracle: {diff:.2e}; layer error {e_got:.5e} vs oracle {e_ref:.5e} (round-to-nearest {e_rtn:.3e})")
    assert abs(e_got - e_ref) <= 1e-2 * e_ref
    assert e_got < 0.8 * e_rtn


@pytest.mark.parametrize("b", [1, 32, 128])
def test_hessian_accumulation_matches_the_fp64_product(fp4, oracle, b):
    """H = (X H_b)^T (X H_b) in fp32 against the oracle's rotation and a NumPy fp64 product; every entry within
    2e-5 of sqrt(H_ii H_jj) (its Cauchy-Schwarz scale; 700 terms of fp32 rounding each), symmetric, and two batches of
    rows accumulate to the same matrix."""
    import torch
    T, K = 700, 384
    xb = inputs.RECIPES[6].x(T, K, salt=90 + b)
    X = oracle.rotate(xb, b).astype(np.float64)
    want = X.T @ X
    say(f"gptq hessian b={b}")
    H = fp4.fp4_gptq_accumulate_hessian(to_dev_bf16(xb), b)
    H2 = fp4.fp4_gptq_accumulate_hessian(to_dev_bf16(xb[:300]), b)
    H2 = fp4.fp4_gptq_accumulate_hessian(to_dev_bf16(xb[300:]), b, H2)
    torch.cuda.synchronize()
    scale = np.sqrt(np.outer(np.diag(want), np.diag(want)))
    for got in (np_(H).astype(np.float64), np_(H2).astype(np.float64)):
        assert np.all(np.abs(got - want) <= 2e-5 * scale)
        assert np.array_equal(got, got.T)


def test_calibration_rows_to_codes_entirely_on_the_gpu(fp4, oracle, gptq):
    import torch
    N, K, T, b = 64, 512, 1536, 32
    r = inputs.RECIPES[6]
    wb, xb = r.w(N, K, salt=95), r.x(T, K, salt=96)
    say("gptq calibration rows -> codes")
    H = fp4.fp4_gptq_accumulate_hessian(to_dev_bf16(xb), b)
    perm, U = fp4.fp4_gptq_prepare(H, 1e-2, True)
    c, s, _ = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, MX, U, perm)
    torch.cuda.synchronize()
    X = oracle.rotate(xb, b).astype(np.float64)
    H64 = X.T @ X
    want_c, want_s, sT, want_perm, _ = gptq.mr_gptq(wb, H64, b, MX)
    assert np.array_equal(np_(perm), want_perm)
    got_c, got_s = np_(c).reshape(N, -1), np_(s).reshape(N, -1)
    assert np.array_equal(got_s, want_s)
    y = oracle.rotate(wb, b)
    c_rtn, _, _ = oracle.quantize(y, MX)
    e_got = gptq.layer_error(y, got_c, want_s, MX, sT, H64)
    e_ref = gptq.layer_error(y, want_c, want_s, MX, sT, H64)
    e_rtn = gptq.layer_error(y, c_rtn, want_s, MX, sT, H64)
    say(f"   codes differing: {(unpack(got_c) != unpack(want_c)).mean():.2e}; layer error {e_got:.5e} vs oracle {e_ref:.5e} (round-to-nearest {e_rtn:.3e})")
    assert abs(e_got - e_ref) <= 1e-2 * e_ref and e_got < 0.8 * e_rtn


def test_sweep_at_layer_size_on_sampled_rows(fp4, oracle, gptq):
    """A whole [4096, 4096] layer through the library (the benchmark's shape: 64 blocks, 8 outer blocks), checked against the
    oracle on 32 sampled rows -- rows never interact, so the oracle sweeps just those rows with the same factor."""
    import torch
    N, K, T, b = 4096, 4096, 4608, 32
    r = inputs.RECIPES[6]
    wb = r.w(N, K, salt=120)
    H = synthetic_hessian(oracle, K, T, b, salt=121)
    perm = gptq.act_order(H).astype(np.int32)
    U = gptq.inverse_factor(H, perm, damp=1e-2).astype(np.float32)
    say("gptq layer size: N = K = 4096")
    c, s, _ = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, MX, to_dev(U), to_dev(perm))
    torch.cuda.synchronize()
    rows = np.sort(np.random.default_rng(5).choice(N, 32, replace=False))
    y = oracle.rotate(wb[rows], b)
    c_rtn, scales, _ = oracle.quantize(y, MX)
    want, _ = gptq.sweep(y, scales, MX, None, U, perm)
    got_c, got_s = np_(c).reshape(N, -1)[rows], np_(s).reshape(N, -1)[rows]
    ok = (got_s == scales).all(axis=1)
    assert ok.mean() >= 0.9
    diff = (unpack(got_c) != unpack(want))[ok].mean()
    e_got = gptq.layer_error(y[ok], got_c[ok], scales[ok], MX, None, H)
    e_ref = gptq.layer_error(y[ok], want[ok], scales[ok], MX, None, H)
    e_rtn = gptq.layer_error(y[ok], c_rtn[ok], scales[ok], MX, None, H)
    say(f"   codes differing from the oracle: {diff:.2e}; layer error {e_got:.5e} vs oracle {e_ref:.5e} (round-to-nearest {e_rtn:.3e})")
    assert diff <= 1e-3 and abs(e_got - e_ref) <= 2e-3 * e_ref and e_got < 0.8 * e_rtn


def test_prepare_at_layer_size(fp4, oracle, gptq):
    """K = 4096 (64 diagonal blocks, six doubling levels of the triangular inversion) against the fp64 factor, and the
    defining identity on 64 sampled columns."""
    import torch
    K = 4096
    H32 = synthetic_hessian(oracle, K, 4608, 32, salt=121).astype(np.float32)
    say("gptq prepare K=4096")
    perm, U = fp4.fp4_gptq_prepare(to_dev(H32), 1e-2, True)
    torch.cuda.synchronize()
    perm, U = np_(perm), np_(U).astype(np.float64)
    H64 = H32.astype(np.float64)
    want_perm = gptq.act_order(H64)
    assert np.array_equal(perm, want_perm)
    want_U = gptq.inverse_factor(H64, want_perm, damp=1e-2)
    rel = np.linalg.norm(U - want_U) / np.linalg.norm(want_U)
    A = H64[np.ix_(want_perm, want_perm)]
    A[np.diag_indices(K)] += 1e-2 * np.mean(np.diag(A))
    cols = np.sort(np.random.default_rng(6).choice(K, 64, replace=False))
    resid = np.abs(U.T @ (U @ A[:, cols]) - np.eye(K)[:, cols]).max()
    say(f"   relative error of U {rel:.2e}; max |U^T U A - I| on 64 columns {resid:.2e}")
    assert rel <= 1e-3 and resid <= 5e-3


def test_widest_layer_of_the_benchmark_model(fp4, oracle, gptq):
    """K = 14336 (the down projection: 224 diagonal blocks, eight doubling levels, an 822 MB factor): the order against
    the oracle's, the factor through the identity that defines it, U^T U (H_perm + lambda I) = I, on sampled columns
    (an fp64 inverse of this size is minutes of CPU), and the sweep of 48 rows with that factor against the oracle's
    sweep of 12 of them.  The Hessian is a rank-96 Gram matrix plus a positive diagonal, built directly."""
    import torch
    K, N, b = 14336, 48, 32
    rng = np.random.default_rng(140)
    V = rng.standard_normal((K, 96)) * rng.uniform(0.3, 2.0, (K, 1))
    H64 = V @ V.T / 96.0
    H64[np.diag_indices(K)] += rng.uniform(0.5, 2.0, K)
    H32 = H64.astype(np.float32)
    H64 = H32.astype(np.float64)
    say("gptq prepare K=14336")
    perm_d, U_d = fp4.fp4_gptq_prepare(to_dev(H32), 1e-2, True)
    torch.cuda.synchronize()
    perm = np_(perm_d)
    want_perm = gptq.act_order(H64)
    assert np.array_equal(perm, want_perm)
    U = np_(U_d).astype(np.float64)
    assert np.all(np.diag(U) > 0)
    cols = np.sort(rng.choice(K, 16, replace=False))
    A_cols = H64[np.ix_(want_perm, want_perm[cols])]
    A_cols[cols, np.arange(16)] += 1e-2 * np.mean(np.diag(H64))
    E = np.zeros((K, 16))
    E[cols, np.arange(16)] = 1.0
    resid = np.abs(U.T @ (U @ A_cols) - E).max()
    below = max(np.abs(U[r, :r]).max() for r in (1, K // 2, K - 1))
    say(f"   max |U^T U A - I| on 16 columns {resid:.2e}")
    assert resid <= 5e-3 and below == 0.0

    wb = inputs.RECIPES[6].w(N, K, salt=141)
    say("gptq sweep N=48 K=14336")
    c, s, _ = fp4.fp4_gptq_quantize_weights(to_dev_bf16(wb), b, MX, U_d, perm_d)
    torch.cuda.synchronize()
    rows = np.arange(0, N, 4)
    y = oracle.rotate(wb[rows], b)
    c_rtn, scales, _ = oracle.quantize(y, MX)
    want, _ = gptq.sweep(y, scales, MX, None, U, perm)
    got_c, got_s = np_(c).reshape(N, -1)[rows], np_(s).reshape(N, -1)[rows]
    ok = (got_s == scales).all(axis=1)
    assert ok.mean() >= 0.9
    diff = (unpack(got_c) != unpack(want))[ok].mean()
    e_got = gptq.layer_error(y[ok], got_c[ok], scales[ok], MX, None, H64)
    e_ref = gptq.layer_error(y[ok], want[ok], scales[ok], MX, None, H64)
    e_rtn = gptq.layer_error(y[ok], c_rtn[ok], scales[ok], MX, None, H64)
    say(f"   codes differing from the oracle: {diff:.2e}; layer error {e_got:.5e} vs oracle {e_ref:.5e} (round-to-nearest {e_rtn:.3e})")
    assert diff <= 1e-3 and abs(e_got - e_ref) <= 2e-3 * e_ref and e_got < 0.9 * e_rtn
