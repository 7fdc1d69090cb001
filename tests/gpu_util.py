"""Helpers for the GPU parity tests (host side only; no arithmetic of the method)."""
import numpy as np

MX, NV = 0, 1
GRID = np.array([0, .5, 1, 1.5, 2, 3, 4, 6], dtype=np.float64)


def to_dev_bf16(bits: np.ndarray):
    import torch
    return torch.from_numpy(bits.view(np.int16).copy()).cuda().view(torch.bfloat16)


def to_dev(a: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def unpack(codes2d: np.ndarray) -> np.ndarray:
    lo = codes2d & 15
    hi = codes2d >> 4
    return np.stack([lo, hi], axis=-1).reshape(codes2d.shape[0], -1)


def grid_steps(ca: np.ndarray, cb: np.ndarray) -> np.ndarray:
    """Distance in grid steps between two arrays of 4-bit codes on the signed 15-point E2M1 grid
    (+0 and -0 are the same point)."""
    def pos(c):
        mag = (c & 7).astype(np.int64)
        return np.where((c & 8) != 0, -mag, mag)
    return np.abs(pos(ca) - pos(cb))


def gemm_layout_to_canonical(codes_g: np.ndarray, scales_g: np.ndarray, rows, K: int, fmt: int):
    """Undo the GEMM layout as documented in include/fp4mr.h / csrc/layout.hpp.  `rows` is a row count (all rows)
    or an array of row indices (a sample).  Returns canonical codes [len(rows),K/2] and scales [len(rows),K/G]."""
    KC = K // 128
    r = (np.arange(rows) if np.isscalar(rows) else np.asarray(rows, dtype=np.int64))[:, None]
    kb = np.arange(K // 2)[None, :]          # byte index along the row; element k = 2*kb
    k = 2 * kb
    off = ((r // 16) * KC + k // 128) * 1024 + (((k % 128) // 32) * 16 + r % 16) * 16 + (k % 32) // 2
    codes = codes_g[off]
    if fmt == MX:
        KS = (K + 511) // 512
        kg = np.arange(K // 32)[None, :]
        soff = (((r // 16) * KS + kg // 16) * 64 + ((kg % 4) * 16 + r % 16)) * 4 + (kg // 4) % 4
    else:
        g16 = np.arange(K // 16)[None, :]
        soff = (((r // 16) * KC + g16 // 8) * 64 + (((g16 % 8) // 2) * 16 + r % 16)) * 2 + g16 % 2
    return codes, scales_g[soff]


def compare_codes(got_codes, got_scales, ref_codes, ref_scales, y_ref, fmt, max_frac=1e-4):
    """End-to-end rule: scales equal except for groups whose abs-max sits within a few ulp of a scale decision
    boundary; among groups with equal scales at most max_frac of the codes differ, each by one grid step."""
    G = 32 if fmt == MX else 16
    gc, rc = unpack(got_codes), unpack(ref_codes)
    same_scale = got_scales == ref_scales
    n_bad_groups = int((~same_scale).sum())
    mask = np.repeat(same_scale, G, axis=1)
    steps = grid_steps(gc, rc)
    diff = (steps != 0) & mask
    frac = diff.sum() / max(1, mask.sum())
    assert steps[mask].max(initial=0) <= 1, "a code differs by more than one grid step"
    assert frac <= max_frac, f"fraction of differing codes {frac:.3e} > {max_frac}"
    if n_bad_groups:
        # a scale may only flip when the group's abs-max is within 8 ulp of the value where the scale changes
        assert n_bad_groups <= max(1, int(2e-5 * same_scale.size)), n_bad_groups
        assert fmt == MX, "NVFP4 scale flips need a per-case look"
        amax = np.abs(y_ref.astype(np.float64)).reshape(y_ref.shape[0], -1, G).max(-1)[~same_scale]
        p2 = 2.0 ** np.round(np.log2(amax))
        assert np.all(np.abs(amax - p2) <= 8 * np.spacing(p2.astype(np.float32))), "scale differs away from a boundary"
        assert np.all(np.abs(got_scales[~same_scale].astype(int) - ref_scales[~same_scale].astype(int)) == 1)
    return frac, n_bad_groups
