"""Pins for the oracle's element and scale codecs (E2M1, E8M0, E4M3) and the Hadamard matrix.

Each check compares the C oracle with something it does not compute itself: values the paper prints
(tests/golden/paper_constants.txt), closed forms, exact rational brute force written here, or a library
routine (scipy.linalg.hadamard, torch's float8_e4m3fn cast).
"""
from fractions import Fraction
from pathlib import Path

import numpy as np
import pytest

GOLDEN = Path(__file__).parent / "golden" / "paper_constants.txt"


def golden():
    out = {}
    for line in GOLDEN.read_text().splitlines():
        line = line.split("#")[0].strip()
        if "=" in line:
            k, v = line.split("=")
            out[k.strip()] = v.split()
    return out


# ---------------------------------------------------------------- Hadamard
@pytest.mark.parametrize("b", [1, 2, 4, 8, 16, 32, 64, 128])
def test_hadamard_orthogonal_and_sylvester(oracle, b):
    import scipy.linalg
    H = oracle.hadamard(b).astype(np.int64)
    assert set(np.unique(H)) <= {-1, 1}
    assert np.array_equal(H @ H.T, b * np.eye(b, dtype=np.int64))          # H H^T = b I (Lemma 1 proof: U orthogonal)
    assert np.array_equal(H, scipy.linalg.hadamard(b).astype(np.int64))    # textbook Sylvester matrix
    i, j = np.meshgrid(np.arange(b), np.arange(b), indexing="ij")
    pop = np.vectorize(lambda v: bin(v).count("1"))(i & j)
    assert np.array_equal(H, 1 - 2 * (pop & 1))                             # closed form (-1)^popcount(i&j)
    assert np.array_equal(H, H.T)


def test_hadamard_rejects_non_power_of_two(oracle):
    for b in (0, 3, 12, 48, 2048):
        with pytest.raises(ValueError):
            oracle.hadamard(b)


# ---------------------------------------------------------------- E2M1
def test_e2m1_decode_table_matches_paper(oracle):
    want = [float(v) for v in golden()["e2m1_positive_values"]]
    got = [oracle.e2m1_decode(c) for c in range(1, 8)]
    assert got == want
    assert oracle.e2m1_decode(0) == 0.0
    for c in range(8):
        assert oracle.e2m1_decode(c | 8) == -oracle.e2m1_decode(c)
    # bit layout: s e1 e0 m  ->  (-1)^s * 2^(e-1) * (1 + m/2) for e>0, m/2 for e=0
    for c in range(16):
        s, e, m = c >> 3, (c >> 1) & 3, c & 1
        v = (m / 2.0) if e == 0 else 2.0 ** (e - 1) * (1 + m / 2.0)
        assert oracle.e2m1_decode(c) == (-v if s else v)


def test_e2m1_grid_values_round_trip(oracle):
    for c in range(16):
        assert oracle.e2m1_encode(oracle.e2m1_decode(c)) == c or (c == 8 and oracle.e2m1_encode(-0.0) == 8)
    assert oracle.e2m1_encode(0.0) == 0
    assert oracle.e2m1_encode(-0.0) == 8


def test_e2m1_midpoints_go_to_even_mantissa(oracle):
    # midpoint -> neighbour with mantissa bit 0
    cases = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for v, want in cases.items():
        assert oracle.e2m1_decode(oracle.e2m1_encode(v)) == want
        assert oracle.e2m1_decode(oracle.e2m1_encode(-v)) == -want
        # one float32 ulp either side resolves the tie the obvious way
        lo = float(np.nextafter(np.float32(v), np.float32(0)))
        hi = float(np.nextafter(np.float32(v), np.float32(10)))
        grid = [0, .5, 1, 1.5, 2, 3, 4, 6]
        below = max(g for g in grid if g < v)
        above = min(g for g in grid if g > v)
        assert oracle.e2m1_decode(oracle.e2m1_encode(lo)) == below
        assert oracle.e2m1_decode(oracle.e2m1_encode(hi)) == above


def test_e2m1_saturates_never_wraps(oracle):
    for v in (6.0, 6.5, 7.0, 7.999, 8.0, 100.0, 3.0e38, 1e300):
        assert oracle.e2m1_encode(v) == 7
        assert oracle.e2m1_encode(-v) == 15
    # dead zone (Section 3, remark "Quantization Dead-zone"): |u| < q_min/2 -> 0
    assert oracle.e2m1_encode(0.2499) == 0 and oracle.e2m1_encode(-0.2499) == 8


def _brute_e2m1(v: float) -> int:
    """Exact rational nearest-neighbour with explicit even-mantissa tie rule."""
    grid = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4), Fraction(6)]
    a = abs(Fraction(v))
    d = [abs(a - g) for g in grid]
    dmin = min(d)
    cands = [c for c in range(8) if d[c] == dmin]
    if len(cands) == 2:
        c = [k for k in cands if k % 2 == 0][0]
    else:
        (c,) = cands
    sign = 8 if np.signbit(v) else 0
    return sign | c


def test_e2m1_exhaustive_over_bf16(oracle):
    """Every finite bf16 bit pattern: C oracle == exact rational argmin (the grid is coarse, so bf16
    covers every decision boundary and both sides of it)."""
    bits = np.arange(1 << 16, dtype=np.uint32)
    vals = (bits << 16).view(np.float32)
    finite = np.isfinite(vals)
    # vectorised independent rule: thresholds at the midpoints, ties resolved to even code
    a = np.abs(vals[finite].astype(np.float64))
    mids = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    tie_up = np.array([False, True, False, True, False, True, False])  # midpoint k goes up iff code k+1 is even
    code = np.zeros(a.shape, dtype=np.int64)
    for k, (mid, up) in enumerate(zip(mids, tie_up)):
        code += (a > mid) | ((a == mid) & up)
    code |= np.where(np.signbit(vals[finite]), 8, 0)
    got = np.array([oracle.e2m1_encode(float(v)) for v in vals[finite]])
    assert np.array_equal(got, code)
    # and the rational brute force on a thinned subset (slow in pure Python)
    sub = vals[finite][::97]
    assert [oracle.e2m1_encode(float(v)) for v in sub] == [_brute_e2m1(float(v)) for v in sub]


# ---------------------------------------------------------------- E8M0
def test_e8m0_decode_all_bytes(oracle):
    for e in range(255):
        assert oracle.e8m0_decode(e) == 2.0 ** (e - 127)


def test_e8m0_floor_rule(oracle):
    # amax = 2^k (1 + eps) anywhere in the octave -> shared exponent k-2, i.e. amax/scale in [4, 8)
    for k in range(-126, 128):
        for frac in (1.0, 1.0 + 2.0 ** -23, 1.25, 1.5, 1.999, 2.0 - 2.0 ** -22):
            amax = frac * 2.0 ** k
            if amax > 3.4028234e38:
                continue
            byte = oracle.e8m0_from_amax(amax)
            want = min(max(k - 2 + 127, 0), 254)
            assert byte == want, (k, frac)
            if 0 < want < 254 or k - 2 + 127 == want:
                r = amax / oracle.e8m0_decode(byte)
                assert 4.0 <= r < 8.0
    assert oracle.e8m0_from_amax(0.0) == 0
    assert oracle.e8m0_from_amax(1e-45) == 0          # far below 2^-125: clamps to the smallest scale
    assert oracle.e8m0_from_amax(6.0) == 127           # 6 = largest E2M1 value -> scale 1
    assert oracle.e8m0_from_amax(4.0) == 127
    assert oracle.e8m0_from_amax(3.999) == 126
    assert oracle.e8m0_from_amax(7.999) == 127         # (6,8): same scale, the element saturates
    assert oracle.e8m0_from_amax(8.0) == 128


# ---------------------------------------------------------------- E4M3
def test_e4m3_decode_table(oracle):
    import torch
    codes = torch.arange(0, 0x7F, dtype=torch.uint8)
    want = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()      # library decode of every finite code
    got = np.array([oracle.e4m3_decode(int(c)) for c in range(0x7F)])
    assert np.array_equal(got, want)
    assert got.max() == float(golden()["e4m3_max"][0]) == 448.0
    assert got[1] == 2.0 ** -9 and got[8] == 2.0 ** -6
    assert np.all(np.diff(got) > 0)                                        # monotone in the code


def test_e4m3_round_trip_and_saturation(oracle):
    for c in range(0x7F):
        assert oracle.e4m3_encode(oracle.e4m3_decode(c)) == c
    assert oracle.e4m3_encode(448.0) == 0x7E
    assert oracle.e4m3_encode(449.0) == 0x7E
    assert oracle.e4m3_encode(1e9) == 0x7E and oracle.e4m3_encode(3e38) == 0x7E and oracle.e4m3_encode(1e300) == 0x7E
    assert oracle.e4m3_encode(0.0) == 0
    assert oracle.e4m3_encode(2.0 ** -10) == 0            # tie between 0 and 2^-9 -> even code 0
    assert oracle.e4m3_encode(3 * 2.0 ** -10) == 2        # tie between codes 1 and 2 -> 2


def test_e4m3_encode_matches_library_cast_in_range(oracle):
    """torch's CPU cast float32 -> float8_e4m3fn is round-to-nearest-even with subnormals for |t| <= 448."""
    import torch
    rng = np.random.default_rng(7)
    t = np.concatenate([
        np.exp(rng.uniform(np.log(2.0 ** -12), np.log(448.0), 20000)),
        np.linspace(0, 448, 4481),
        np.array([(oracle.e4m3_decode(c) + oracle.e4m3_decode(c + 1)) / 2 for c in range(0x7E)]),  # every midpoint
    ]).astype(np.float32)
    t = t[t <= 448.0]
    want = torch.from_numpy(t).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.e4m3_encode(float(v)) for v in t], dtype=np.uint8)
    assert np.array_equal(got, want)


def test_e4m3_brute_force_rational(oracle):
    vals = [Fraction(oracle.e4m3_decode(c)) for c in range(0x7F)]
    rng = np.random.default_rng(11)
    for t in np.exp(rng.uniform(np.log(2.0 ** -11), np.log(600.0), 300)).astype(np.float32):
        ft = Fraction(float(t))
        d = [abs(ft - v) for v in vals]
        dmin = min(d)
        c = [k for k in range(0x7F) if d[k] == dmin]
        want = c[0] if len(c) == 1 else [k for k in c if k % 2 == 0][0]
        assert oracle.e4m3_encode(float(t)) == want
