"""MR-GPTQ weight quantizer, CPU oracle in NumPy fp64.  TEST INFRASTRUCTURE ONLY (shares nothing with the HIP library).

What it follows (paper = arXiv 2509.23202, Section 4 "An FP4-Focused Variant of the GPTQ Algorithm"):

  * "Standard GPTQ": all rows are quantized in the same fixed column order; after a column is rounded, the columns not
    yet quantized are updated with second-order information so that the layer's output error ||X What - X W||^2 stays
    as small as it can.  The update is the one of Optimal Brain Quantization; in the form used here the inverse Hessian
    is factored once, Hinv = U^T U with U upper triangular, and quantizing column j moves the remaining columns by
    -(w_j - q_j) / U[j,j] * U[j, j+1:].
  * Section 4.1, Ingredient 3: the weights are rotated by the block Hadamard first (W H_k) and the Hessian is the one of
    the rotated inputs.
  * Section 4.1, Ingredient 1: the grid (the scales) is fixed BEFORE the sweep, from the rotated weights in their
    original column order ("absmax", or the squared-error scale search "mse").
  * Section 4.1, Ingredient 2: static activation re-ordering -- with grid and scales fixed, the columns are visited in
    descending order of the Hessian diagonal, and the codes land back at their original positions, so the group
    structure of the stored tensor is the original one.
  * Section 5 "Algorithms": Hessian dampening lambda = 1e-2 (times the mean of the diagonal, the usual convention).

Readings: the dampening is relative to the mean diagonal; the act-order sort is stable (equal diagonal entries keep
their original order); a group whose scale is zero quantizes to zero codes and propagates its (whole) value as error.
"""
from __future__ import annotations

import numpy as np

from . import reference as ref

E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0])
# midpoints between neighbouring grid values; at an exact midpoint the code with an even mantissa bit wins,
# i.e. the lower code at 0.25, 1.25, 2.5, 5.0 and the upper one at 0.75, 1.75, 3.5
_MID = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
_UPPER_WINS_TIE = np.array([False, True, False, True, False, True, False])


def e2m1_encode(v: np.ndarray) -> np.ndarray:
    """Nearest E2M1 code of every element (ties to the even code, saturating at 6), sign in bit 3."""
    a = np.abs(v)[..., None]
    above = np.where(_UPPER_WINS_TIE, a >= _MID, a > _MID)
    mag = above.sum(-1).astype(np.uint8)
    return (mag | (np.signbit(v).astype(np.uint8) << 3)).astype(np.uint8)


def e2m1_decode(c: np.ndarray) -> np.ndarray:
    return np.where(c & 8, -1.0, 1.0) * E2M1_GRID[c & 7]


def act_order(H: np.ndarray) -> np.ndarray:
    """Static activation order: column indices by descending Hessian diagonal (stable)."""
    return np.argsort(-np.diag(np.asarray(H, dtype=np.float64)), kind="stable")


def inverse_factor(H: np.ndarray, perm: np.ndarray, damp: float = 1e-2) -> np.ndarray:
    """Upper-triangular U with U^T U = (H_perm + damp * mean(diag H) * I)^-1, H_perm = H[perm][:, perm]."""
    Hp = np.asarray(H, dtype=np.float64)[np.ix_(perm, perm)].copy()
    Hp[np.diag_indices_from(Hp)] += damp * np.mean(np.diag(Hp))
    Hinv = np.linalg.inv(Hp)
    Hinv = 0.5 * (Hinv + Hinv.T)
    return np.linalg.cholesky(Hinv).T.copy()


def column_scales(scales: np.ndarray, fmt: int, s_T) -> np.ndarray:
    """Decoded scale of every (row, group): E8M0 or E4M3 byte times the tensor-level factor."""
    N = scales.shape[0]
    ones = np.tile(np.uint8(0x22), (N, scales.shape[1] * ref.GROUP[fmt] // 2))  # code 2 = 1.0 in both nibbles
    return ref.dequantize(ones, scales, fmt, s_T)[:, ::ref.GROUP[fmt]]


def sweep(w_rot: np.ndarray, scales: np.ndarray, fmt: int, s_T, U: np.ndarray, perm: np.ndarray, stop: int | None = None,
          table: np.ndarray | None = None):
    """The GPTQ sweep on fixed scales.  w_rot [N,K] rotated weights, scales [N,K/G] bytes (original column order),
    U [K,K] upper factor in act-order coordinates, perm [K].  Visits the columns perm[0], perm[1], ...:

        q = Q(w / s) ;  e = (w - q s) / U[j,j] ;  w[later columns] -= e * U[j, later]

    Returns (codes [N,K/2] packed in original order, work [N,K] = the working weights in act-order coordinates after
    `stop` columns (all of them by default): quantized values in the visited columns, updated weights in the rest).
    table: 256 scale values; a group's scale is then table[byte] (the scale byte fitted to the tensor's range of scales,
    appendix on MXFP scale fitting) instead of the decoded E8M0 / E4M3 byte."""
    G = ref.GROUP[fmt]
    W = np.asarray(w_rot, dtype=np.float64)[:, perm].copy()
    N, K = W.shape
    S_groups = column_scales(scales, fmt, s_T) if table is None else np.asarray(table, dtype=np.float64)[np.asarray(scales)]
    S = S_groups[:, np.asarray(perm) // G]      # scale of every visited column
    U = np.asarray(U, dtype=np.float64)
    Q = np.zeros((N, K), dtype=np.uint8)
    n_cols = K if stop is None else stop
    for j in range(n_cols):
        s = S[:, j]
        w = W[:, j].copy()
        ok = s > 0
        c = np.zeros(N, dtype=np.uint8)
        c[ok] = e2m1_encode(w[ok] / s[ok])
        dq = e2m1_decode(c) * s
        e = (w - dq) / U[j, j]
        W[:, j:] -= np.outer(e, U[j, j:])
        W[:, j] = dq                      # (what the line above leaves there, without the rounding of w - (w - dq))
        Q[:, j] = c
    codes = np.zeros((N, K), dtype=np.uint8)
    codes[:, perm] = Q
    packed = (codes[:, 0::2] | (codes[:, 1::2] << 4)).astype(np.uint8)
    return packed, W


def mr_gptq(w_bf16_bits: np.ndarray, H: np.ndarray, b: int, fmt: int, policy: str = "absmax", damp: float = 1e-2,
            order: bool = True):
    """Whole weight quantizer: rotate, fix the scales, order, factor, sweep.  H is the Hessian X'^T X' of the ROTATED
    calibration inputs [K,K].  Returns (codes, scales, s_T, perm, U)."""
    y = ref.rotate(w_bf16_bits, b)
    table = None
    if policy == "mse_alt":      # NVFP4: group scales and tensor scale by the alternating optimisation (Section 4.1 Ingredient 1)
        _, scales, s_T, _ = ref.quantize_nvfp4_alternating(y, 3)
    elif policy == "fit_range":  # MXFP4 with the scale byte fitted to the range of scales: s_T is then the table of 256 scale values
        _, scales, _, table = ref.quantize_mxfp4_fit(y)
        s_T = table
    else:
        _, scales, s_T = ref.quantize(y, fmt, policy=policy)
    K = y.shape[1]
    perm = act_order(H) if order else np.arange(K)
    U = inverse_factor(H, perm, damp)
    codes, _ = sweep(y, scales, fmt, None if table is not None else s_T, U, perm, table=table)
    return codes, scales, s_T, perm, U


def layer_error(w_rot: np.ndarray, codes: np.ndarray, scales: np.ndarray, fmt: int, s_T, H: np.ndarray, table=None) -> float:
    """tr((What - W) H (What - W)^T) = ||X' What^T - X' W^T||^2 for the rotated weights and inputs (table: see sweep)."""
    What = ref.dequantize(codes, scales, fmt, s_T) if table is None else ref.dequantize_table(codes, scales, table)
    D = What - np.asarray(w_rot, dtype=np.float64)
    return float(np.einsum("nk,kl,nl->", D, np.asarray(H, dtype=np.float64), D))
