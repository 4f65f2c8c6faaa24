"""Comparators used by the parity tests (host logic only, no GPU, no product code).

``compare_store`` classifies every stored vector of a cache produced by the HIP
path against the oracle's cache for the same inputs:

* scale must agree within ``1e-3`` relative;
* codes must be bit-identical, except
  - elements whose fp64 pre-rounding value ``v = y/s`` lies within
    ``1e-6 * max(1, |v|)`` of a rounding boundary (``frac(v) = 1/2``): counted
    as ``near_boundary`` and exempt;
  - vectors whose zero-point differs by exactly one because ``-min/s`` itself
    lies that close to a boundary: every code then shifts by the same amount
    while ``c - z`` is unchanged away from the clip; counted as ``zero_flip``
    vectors and checked in that form.
  Anything else is a hard mismatch.
"""
from __future__ import annotations

import numpy as np

BOUNDARY_REL = 1e-6
SCALE_REL = 1e-3


def unpack(p: np.ndarray) -> np.ndarray:
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), np.int16)
    out[..., 0::2] = p & 0x0F
    out[..., 1::2] = p >> 4
    return out


def _near_boundary(v: np.ndarray) -> np.ndarray:
    frac = v - np.floor(v)
    return np.abs(frac - 0.5) <= BOUNDARY_REL * np.maximum(1.0, np.abs(v))


def compare_vectors(codes_gpu, meta_gpu, codes_ref, meta_ref, y, s64, z64) -> dict:
    """All arrays are per-vector: codes ``[n][d/2]`` u8, meta ``[n][2]`` f32, ``y [n][d]`` f64, ``s64, z64 [n]``."""
    cg = unpack(np.asarray(codes_gpu))
    cr = unpack(np.asarray(codes_ref))
    sg = np.asarray(meta_gpu, np.float64)[:, 0]
    zg = np.asarray(meta_gpu, np.float64)[:, 1]
    sr = np.asarray(meta_ref, np.float64)[:, 0]
    zr = np.asarray(meta_ref, np.float64)[:, 1]
    n, d = cg.shape
    scale_rel = np.abs(sg - sr) / np.maximum(np.abs(sr), 1e-300)
    res = {"vectors": n, "elements": n * d, "scale_max_rel": float(scale_rel.max(initial=0.0)),
           "scale_bad": int((scale_rel > SCALE_REL).sum())}

    v = y / s64[:, None]
    near = _near_boundary(v)
    zdiff = zg - zr
    zsame = zdiff == 0
    # zero-point flips: |dz| == 1 and -min/s near a boundary
    zpre = -y.min(axis=1) / s64
    zflip = (np.abs(zdiff) == 1) & _near_boundary(zpre)
    zbad = ~zsame & ~zflip
    res["zero_flip_vectors"] = int(zflip.sum())
    res["zero_bad_vectors"] = int(zbad.sum())

    diff = cg != cr
    # ordinary vectors
    ord_diff = diff & zsame[:, None]
    res["near_boundary_mismatch"] = int((ord_diff & near).sum())
    hard = ord_diff & ~near
    # zero-flip vectors: (c - z) must agree away from the clip and away from boundaries
    if zflip.any():
        rel_g = cg[zflip] - zg[zflip, None]
        rel_r = cr[zflip] - zr[zflip, None]
        clip = (cg[zflip] == 0) | (cg[zflip] == 15) | (cr[zflip] == 0) | (cr[zflip] == 15)
        bad = (rel_g != rel_r) & ~clip & ~near[zflip]
        res["zero_flip_bad_elements"] = int(bad.sum())
    else:
        res["zero_flip_bad_elements"] = 0
    res["hard_mismatch"] = int(hard.sum()) + int(diff[zbad].sum())
    res["near_boundary_elements"] = int(near.sum())
    res["first_hard"] = [tuple(map(int, ij)) for ij in np.argwhere(hard)[:5]]
    return res


def assert_store_ok(res: dict):
    assert res["scale_bad"] == 0, res
    assert res["zero_bad_vectors"] == 0, res
    assert res["zero_flip_bad_elements"] == 0, res
    assert res["hard_mismatch"] == 0, res


def attn_error(o_gpu: np.ndarray, o_ref: np.ndarray) -> float:
    """Max-abs error relative to the largest reference magnitude (the 2e-3 criterion)."""
    o_ref = np.asarray(o_ref, np.float64)
    den = np.abs(o_ref).max()
    return float(np.abs(np.asarray(o_gpu, np.float64) - o_ref).max() / (den if den > 0 else 1.0))
