"""The comparators themselves, exercised on the CPU with mistakes planted in a copy of the oracle's output."""
import numpy as np
import torch

import parity
from oracle import saw_oracle as O

RNG = np.random.default_rng(77)


def _case(n=4000, d=128, h=64):
    x = (RNG.standard_normal((n, d)) * np.abs(RNG.standard_t(3, size=d))).astype(np.float32)
    x = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    y = O.rotate(x, h)
    c, s, z = O.quantize(y)
    return y, O.pack_nibbles(c), np.stack([s, z], 1).astype(np.float32), s, z


def test_identical_is_clean():
    y, p, m, s, z = _case()
    r = parity.compare_vectors(p, m, p, m, y, s, z)
    assert r["hard_mismatch"] == 0 and r["scale_bad"] == 0 and r["zero_flip_vectors"] == 0
    parity.assert_store_ok(r)


def test_planted_code_error_is_hard():
    y, p, m, s, z = _case()
    v = y / s[:, None]
    frac = np.abs(v - np.floor(v) - 0.5)
    i, j = np.unravel_index(np.argmax(frac), frac.shape)           # far from any boundary
    bad = p.copy()
    bad[i, j // 2] ^= (1 << (4 * (j & 1)))
    r = parity.compare_vectors(bad, m, p, m, y, s, z)
    assert r["hard_mismatch"] == 1 and r["first_hard"] == [(int(i), int(j))]


def test_planted_scale_and_zero_errors():
    y, p, m, s, z = _case()
    m2 = m.copy()
    m2[3, 0] *= 1.01
    assert parity.compare_vectors(p, m2, p, m, y, s, z)["scale_bad"] == 1
    m3 = m.copy()
    m3[5, 1] += 1                                                   # a zero-point change with nothing near a boundary
    r = parity.compare_vectors(p, m3, p, m, y, s, z)
    assert r["zero_bad_vectors"] == 1


def test_fp32_pipeline_differences_are_classified_not_failed():
    # An fp32 re-computation (un-normalised butterfly, reciprocal multiply) differs from the fp64
    # oracle only at elements the 1e-6 boundary rule exempts or by whole zero-point flips.
    n, d, h = 20000, 128, 128
    x = (RNG.standard_normal((n, d)) * np.abs(RNG.standard_t(3, size=d))).astype(np.float32)
    x = torch.from_numpy(x).to(torch.bfloat16).float().numpy()
    y64 = O.rotate(x, h)
    c, s, z = O.quantize(y64)
    y = x.copy()
    st = 1
    while st < h:
        yy = y.reshape(n, d // (2 * st), 2, st)
        y = np.stack([yy[:, :, 0] + yy[:, :, 1], yy[:, :, 0] - yy[:, :, 1]], 2).reshape(n, d).astype(np.float32)
        st *= 2
    mn, mx = y.min(1), y.max(1)
    r32 = (mx - mn).astype(np.float32)
    inv = (np.float32(15) / r32).astype(np.float32)
    sg = (r32 * np.float32(1.0 / (15.0 * np.sqrt(h)))).astype(np.float32)
    zg = np.rint((-mn * inv).astype(np.float32))
    cg = np.clip(np.rint((y * inv[:, None]).astype(np.float32)) + zg[:, None], 0, 15).astype(np.uint8)
    r = parity.compare_vectors(O.pack_nibbles(cg), np.stack([sg, zg], 1), O.pack_nibbles(c),
                               np.stack([s, z], 1).astype(np.float32), y64, s, z)
    parity.assert_store_ok(r)
    assert r["scale_max_rel"] < 1e-6


def test_attn_error_norm():
    ref = np.array([[1.0, -4.0], [0.5, 2.0]])
    assert parity.attn_error(ref, ref) == 0.0
    assert abs(parity.attn_error(ref + np.array([[0.0, 0.0], [0.008, 0.0]]), ref) - 0.002) < 1e-12
