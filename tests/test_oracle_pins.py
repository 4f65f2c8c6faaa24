"""Pins for the CPU oracle: everything here checks ``oracle/`` against something that
is NOT the oracle -- closed forms, identities the paper states, hand-worked values,
brute force written separately, and library routines.  No GPU, no product code.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg
import torch

from oracle import saw_oracle as O

RNG = np.random.default_rng(1234)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "quant_worked_examples.txt")


# ---------------------------------------------------------------- rotation
@pytest.mark.parametrize("h", [1, 2, 4, 8, 16, 32, 64, 128])
def test_hadamard_closed_form_symmetry_orthogonality(h):
    H = O.hadamard(h)
    # closed form of the Sylvester construction: (-1)^popcount(i & j) / sqrt(h)
    ref = np.array([[(-1.0) ** bin(i & j).count("1") for j in range(h)] for i in range(h)]) / math.sqrt(h)
    assert np.array_equal(H, ref)
    assert np.array_equal(H, H.T)                                   # App. A.4: H = H^T
    assert np.allclose(H @ H.T, np.eye(h), atol=1e-14)              # App. A.4: H H^T = I
    assert np.allclose(H * math.sqrt(h), scipy.linalg.hadamard(h))  # library constructor


@pytest.mark.parametrize("d,h", [(128, 16), (128, 32), (128, 64), (128, 128), (64, 16), (64, 64)])
def test_block_structure(d, h):
    Hb = O.block_hadamard(d, h)
    for i in range(d // h):
        for j in range(d // h):
            blk = Hb[i * h:(i + 1) * h, j * h:(j + 1) * h]
            if i == j:
                assert np.array_equal(blk, O.hadamard(h))
            else:
                assert not blk.any()
    # one-hot a*e_j spreads to |a|/sqrt(h) over its own block only (Sec. 3 eq. 2-3)
    j = h + 3 if d > h else 3
    x = np.zeros(d)
    x[j] = -2.5
    y = O.rotate(x, h)
    b0 = (j // h) * h
    assert np.allclose(np.abs(y[b0:b0 + h]), 2.5 / math.sqrt(h), atol=1e-15)
    assert not np.delete(y, np.s_[b0:b0 + h]).any()
    # a constant block collapses onto the block's first coefficient
    x = np.zeros(d)
    x[b0:b0 + h] = 0.75
    y = O.rotate(x, h)
    assert abs(y[b0] - 0.75 * math.sqrt(h)) < 1e-13
    assert np.abs(np.delete(y, b0)).max() < 1e-13


@pytest.mark.parametrize("d,h", [(128, 16), (128, 64), (128, 128), (64, 32)])
def test_norm_and_inner_product_preserved(d, h):
    x = RNG.standard_normal((50, d)) * RNG.standard_t(3, size=d)
    q = RNG.standard_normal((7, d))
    xr, qr = O.rotate(x, h), O.rotate(q, h)
    assert np.allclose(np.linalg.norm(xr, axis=1), np.linalg.norm(x, axis=1), rtol=1e-13)  # Sec. 3
    assert np.allclose(qr @ xr.T, q @ x.T, rtol=0, atol=1e-11)      # App. A.4: (qH)(KH)^T = qK^T
    assert np.allclose(O.rotate(xr, h), x, atol=1e-12)              # H is its own inverse


def test_rotate_acts_on_row_vectors_blockwise():
    # x H_blk with x a row vector: chunk i of the result is (chunk i of x) H_h  (App. A.4)
    d, h = 64, 16
    x = RNG.standard_normal(d)
    y = O.rotate(x, h)
    for i in range(d // h):
        manual = np.array([sum(x[i * h + r] * (-1.0) ** bin(r & c).count("1") for r in range(h))
                           for c in range(h)]) / math.sqrt(h)
        assert np.allclose(y[i * h:(i + 1) * h], manual, atol=1e-13)


# ---------------------------------------------------------------- quantiser
def _golden_rows():
    rows = []
    with open(GOLDEN) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, h, x, s, z, codes, packed, xhat = [t.strip() for t in line.split("|")]
            rows.append((name, int(h), np.array(x.split(), float), float(s), float(z),
                         np.array(codes.split(), int), bytes.fromhex(packed.replace(" ", "")),
                         np.array(xhat.split(), float)))
    return rows


@pytest.mark.parametrize("row", _golden_rows(), ids=lambda r: r[0])
def test_hand_worked_examples(row):
    name, h, x, s_ref, z_ref, codes_ref, packed_ref, xhat_ref = row
    y = O.rotate(x, h)
    codes, s, z = O.quantize(y)
    assert abs(s - s_ref) <= 1e-12 * abs(s_ref)
    assert z == z_ref
    assert codes.tolist() == codes_ref.tolist()
    assert bytes(O.pack_nibbles(codes)) == packed_ref
    assert np.allclose(O.dequantize(codes, s, z), xhat_ref, rtol=0, atol=1e-12)
    # and through the paged store: one token, one head
    d = x.shape[0]
    cache = O.new_cache(3, 1, 16, d)
    pt = np.array([[2, 0, 1]], np.int32)
    O.rotate_quant_store(cache, x[None, None, :], x[None, None, :], pt, np.array([[0, 21]], np.int32), h)
    assert bytes(cache["k_codes"][0, 0, 5]) == packed_ref        # position 21 -> page_table[0][1] = 0, slot 5
    assert bytes(cache["v_codes"][0, 0, 5]) == packed_ref
    assert cache["k_meta"][0, 0, 5, 0] == np.float32(s) and cache["k_meta"][0, 0, 5, 1] == np.float32(z_ref)
    assert not cache["k_codes"][1:].any() and not cache["k_codes"][0, 0, :5].any()


def test_quantiser_invariants_random():
    y = RNG.standard_normal((2000, 128)) * np.abs(RNG.standard_t(3, size=128)) + RNG.standard_normal((2000, 1))
    codes, s, z = O.quantize(y)
    assert codes.min() >= 0 and codes.max() <= 15
    xh = O.dequantize(codes, s, z)
    assert (np.abs(xh - y) <= 0.5 * s[:, None] * (1 + 1e-9) + 1e-12).all()       # round-trip error <= s/2
    r = np.arange(len(y))
    assert (codes[r, y.argmin(1)] == 0).all() and (codes[r, y.argmax(1)] == 15).all()
    assert np.allclose(s, (y.max(1) - y.min(1)) / 15.0, rtol=1e-15)
    assert np.array_equal(z, np.round(z)) and np.abs(z + y.min(1) / s).max() <= 0.5
    # exact power-of-two rescaling leaves codes and z untouched, scales s
    c2, s2, z2 = O.quantize(y * 8.0)
    assert np.array_equal(c2, codes) and np.array_equal(z2, z) and np.array_equal(s2, s * 8.0)
    # one shared (s, z) per vector: permuting channels permutes codes
    perm = RNG.permutation(128)
    c3, s3, z3 = O.quantize(y[:, perm])
    assert np.array_equal(c3, codes[:, perm]) and np.array_equal(s3, s) and np.array_equal(z3, z)


def test_quantiser_range_without_zero_and_degenerate():
    y = 100.0 + RNG.random((64, 32))
    codes, s, z = O.quantize(y)
    assert (z < -15).all()                                         # zero-point is not clamped to [0, 15]
    assert (np.abs(O.dequantize(codes, s, z) - y) <= 0.5 * s[:, None] * (1 + 1e-9)).all()
    for val in (0.0, 3.25, -7.5):
        c, s, z = O.quantize(np.full((1, 16), val))
        assert not c.any()
        assert np.array_equal(O.dequantize(c, s, z), np.full((1, 16), val))


def test_pack_unpack_and_footprint():
    codes = RNG.integers(0, 16, size=(9, 128)).astype(np.uint8)
    p = O.pack_nibbles(codes)
    assert p.shape == (9, 64)                                      # 4 bits per value: 4x below 16-bit storage
    assert np.array_equal(p & 15, codes[:, 0::2]) and np.array_equal(p >> 4, codes[:, 1::2])
    assert np.array_equal(O.unpack_nibbles(p), codes)


def test_h1_equals_plain_and_mask_selects_rotation():
    T, Hkv, d, P = 20, 2, 64, 16
    K = RNG.standard_normal((T, Hkv, d))
    V = RNG.standard_normal((T, Hkv, d))
    pt = np.array([[1, 0]], np.int32)
    sl = np.stack([np.zeros(T, np.int32), np.arange(T, dtype=np.int32)], 1)
    a, b, c = (O.new_cache(2, Hkv, P, d) for _ in range(3))
    O.rotate_quant_store(a, K, V, pt, sl, 1, 3)
    O.rotate_quant_store(b, K, V, pt, sl, 32, 0)
    assert all(np.array_equal(a[k], b[k]) for k in ("k_codes", "v_codes", "k_meta", "v_meta"))
    O.rotate_quant_store(c, K, V, pt, sl, 32, O.ROT_K)            # K rotated, V plain
    assert np.array_equal(c["v_codes"], a["v_codes"]) and not np.array_equal(c["k_codes"], a["k_codes"])
    k_un, v_un = O.dequant_pages(c, pt, 0, 0, T, 32, O.ROT_K, unrotate=True)
    assert np.abs(k_un - K).max() < 0.5 and np.abs(v_un - V).max() < 0.5


def test_token_wise_independence_and_page_placement():
    w_T, Hkv, d, P = 37, 2, 128, 16
    K = RNG.standard_normal((w_T, Hkv, d))
    V = RNG.standard_normal((w_T, Hkv, d))
    pt1 = np.array([[4, 2, 0]], np.int32)
    pt2 = np.array([[1, 3, 5]], np.int32)
    sl = np.stack([np.zeros(w_T, np.int32), np.arange(w_T, dtype=np.int32)], 1)
    c1, c2, c3 = (O.new_cache(6, Hkv, P, d) for _ in range(3))
    O.rotate_quant_store(c1, K, V, pt1, sl, 64)
    O.rotate_quant_store(c2, K, V, pt2, sl, 64)
    for t in RNG.permutation(w_T):                                  # one token at a time, any order
        O.rotate_quant_store(c3, K[t:t + 1], V[t:t + 1], pt1, sl[t:t + 1], 64)
    for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
        assert np.array_equal(c1[k], c3[k])
    # physical placement: position p -> page_table[p // P], slot p % P, and nowhere else
    assert np.array_equal(c1["k_codes"][4], c2["k_codes"][1]) and np.array_equal(c1["k_codes"][0, :, :5], c2["k_codes"][5, :, :5])
    assert not c1["k_codes"][[1, 3, 5]].any() and not c1["k_codes"][0, :, 5:].any()
    a = O.dequant_pages(c1, pt1, 0, 0, w_T, 64)
    b = O.dequant_pages(c2, pt2, 0, 0, w_T, 64)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    q = RNG.standard_normal((1, 4, d))
    o1 = O.paged_decode_attn(c1, q, pt1, np.array([w_T]), 64)
    o2 = O.paged_decode_attn(c2, q, pt2, np.array([w_T]), 64)
    assert np.array_equal(o1, o2)


def test_rotation_reduces_error_on_outlier_channels():
    d = 128
    x = RNG.standard_normal((4000, d))
    x[:, [5, 40, 77, 120]] *= 20.0                                  # channel-wise range heterogeneity (Sec. 3)
    mse = {}
    for h in (1, 16, 64, 128):
        y = O.rotate(x, h)
        c, s, z = O.quantize(y)
        mse[h] = float(((O.rotate(O.dequantize(c, s, z), h) - x) ** 2).mean())
    assert mse[16] < mse[1] and mse[64] < mse[16] and mse[128] < 1.25 * mse[64] and mse[128] < mse[16]


# ---------------------------------------------------------------- attention
def _tiny_case(h, mask, Hq=4, Hkv=2, d=16, L=(5, 19, 0), P=16, dtype=np.float16):
    B = len(L)
    pt = RNG.permutation(2 * B + 1)[:2 * B].reshape(B, 2).astype(np.int32)
    cache = O.new_cache(2 * B + 1, Hkv, P, d)
    for b in range(B):
        if L[b]:
            K = (RNG.standard_normal((L[b], Hkv, d)) * 1.5).astype(dtype)
            V = RNG.standard_normal((L[b], Hkv, d)).astype(dtype)
            sl = np.stack([np.full(L[b], b, np.int32), np.arange(L[b], dtype=np.int32)], 1)
            O.rotate_quant_store(cache, K, V, pt, sl, h, mask)
    q = RNG.standard_normal((B, Hq, d)).astype(dtype)
    return cache, q, pt, np.array(L, np.int32)


def _brute_force(cache, q, pt, L, h, mask):
    """Scalar loops over the stored bytes: own indexing, own nibble extraction, own Hadamard entries,
    softmax without max subtraction (magnitudes are small)."""
    B, Hq, d = q.shape
    Hkv, P = cache["n_kv_heads"], cache["page_size"]
    G = Hq // Hkv

    def had(i, j):
        if i // h != j // h:
            return 0.0
        return (-1.0) ** bin((i % h) & (j % h)).count("1") / math.sqrt(h)

    def val(which, page, g, slot, ch):
        byte = int(cache[which + "_codes"][page, g, slot, ch // 2])
        code = (byte >> 4) if (ch & 1) else (byte & 15)
        s = float(cache[which + "_meta"][page, g, slot, 0])
        z = float(cache[which + "_meta"][page, g, slot, 1])
        return s * (code - z)

    out = np.zeros((B, Hq, d))
    for b in range(B):
        for j in range(Hq):
            if L[b] == 0:
                continue
            g = j // G
            qf = [float(x) for x in q[b, j]]
            if (mask & 1) and h > 1:
                qf = [sum(qf[i] * had(i, c) for i in range(d)) for c in range(d)]
            e = []
            for t in range(L[b]):
                page, slot = int(pt[b, t // P]), t % P
                e.append(math.exp(sum(qf[c] * val("k", page, g, slot, c) for c in range(d)) / math.sqrt(d)))
            den = sum(e)
            o = [0.0] * d
            for t in range(L[b]):
                page, slot = int(pt[b, t // P]), t % P
                for c in range(d):
                    o[c] += e[t] / den * val("v", page, g, slot, c)
            if (mask & 2) and h > 1:
                o = [sum(o[i] * had(i, c) for i in range(d)) for c in range(d)]
            out[b, j] = o
    return out


@pytest.mark.parametrize("h,mask", [(16, 3), (8, 3), (4, 1), (16, 2), (1, 3), (16, 0)])
def test_decode_attention_vs_brute_force(h, mask):
    cache, q, pt, L = _tiny_case(h, mask)
    o = O.paged_decode_attn(cache, q, pt, L, h, mask)
    ref = _brute_force(cache, q, pt, L, h, mask)
    assert np.allclose(o, ref, rtol=0, atol=1e-12)
    assert not o[2].any()                                           # empty sequence -> zero row


@pytest.mark.parametrize("h", [16, 64, 128])
def test_decode_attention_vs_library_sdpa_on_unrotated_cache(h):
    Hq, Hkv, d = 8, 2, 128
    cache, q, pt, L = _tiny_case(h, 3, Hq=Hq, Hkv=Hkv, d=d, L=(31, 7))
    o = O.paged_decode_attn(cache, q, pt, L, h, 3)
    for b in range(2):
        k_un, v_un = O.dequant_pages(cache, pt, b, 0, int(L[b]), h, 3, unrotate=True)
        kt = torch.from_numpy(k_un).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)  # [Hq][L][d]
        vt = torch.from_numpy(v_un).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
        qt = torch.from_numpy(q[b].astype(np.float64))[:, None, :]
        ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt)[:, 0, :].numpy()
        assert np.allclose(o[b], ref, rtol=0, atol=1e-11)
        # the same thing through the plain textbook routine of the oracle
        assert np.allclose(O.attention_plain(q[b], k_un, v_un), ref, rtol=0, atol=1e-11)


def test_rotated_space_attention_is_exact_without_quantisation():
    # Sec. 3 / App. A.4: attention computed in the rotated space carries no extra error.
    Hq, Hkv, d, L, h = 8, 2, 128, 40, 32
    q = RNG.standard_normal((Hq, d))
    K = RNG.standard_normal((L, Hkv, d)) * np.abs(RNG.standard_t(3, size=d))
    V = RNG.standard_normal((L, Hkv, d))
    plain = O.attention_plain(q, K, V)
    rot = O.rotate(O.attention_plain(O.rotate(q, h), O.rotate(K, h), O.rotate(V, h)), h)
    assert np.allclose(rot, plain, rtol=0, atol=1e-12)
    qt = torch.from_numpy(q)[:, None, :]
    kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(Hq // Hkv, 0)
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt)[:, 0, :].numpy()
    assert np.allclose(plain, ref, rtol=0, atol=1e-12)


def test_special_cases_single_token_and_zero_query():
    Hq, Hkv, d, h = 4, 2, 64, 64
    cache, q, pt, L = _tiny_case(h, 3, Hq=Hq, Hkv=Hkv, d=d, L=(1, 23))
    o = O.paged_decode_attn(cache, q, pt, L, h, 3)
    k_un, v_un = O.dequant_pages(cache, pt, 0, 0, 1, h, 3, unrotate=True)
    for j in range(Hq):                                             # L = 1: o = dequant(V_0) H
        assert np.allclose(o[0, j], v_un[0, j // (Hq // Hkv)], atol=1e-13)
    o0 = O.paged_decode_attn(cache, np.zeros_like(q), pt, L, h, 3)
    _, v_un = O.dequant_pages(cache, pt, 1, 0, 23, h, 3, unrotate=True)
    for j in range(Hq):                                             # q = 0: uniform weights -> mean of V^
        assert np.allclose(o0[1, j], v_un[:, j // (Hq // Hkv)].mean(0), atol=1e-13)


def test_sm_scale_and_gqa_mapping():
    Hq, Hkv, d, h = 8, 2, 16, 16
    cache, q, pt, L = _tiny_case(h, 3, Hq=Hq, Hkv=Hkv, d=d, L=(9, 12))
    a = O.paged_decode_attn(cache, q, pt, L, h, 3, sm_scale=0.0)
    b = O.paged_decode_attn(cache, q, pt, L, h, 3, sm_scale=1.0 / math.sqrt(d))
    assert np.array_equal(a, b)                                     # default scale is 1/sqrt(head_dim), not 1/sqrt(h)
    c = O.paged_decode_attn(cache, q, pt, L, h, 3, sm_scale=0.5)
    assert not np.allclose(a, c)
    # query heads 0..3 read kv head 0, 4..7 read kv head 1: identical queries in a group give identical rows
    q2 = q.copy()
    q2[:, 1] = q2[:, 0]
    q2[:, 4] = q2[:, 0]
    o = O.paged_decode_attn(cache, q2, pt, L, h, 3)
    assert np.array_equal(o[:, 1], o[:, 0]) and not np.allclose(o[:, 4], o[:, 0])


def test_kv16_baseline_matches_plain_attention():
    Hq, Hkv, d, P, L = 4, 2, 64, 16, 21
    K = RNG.standard_normal((L, Hkv, d)).astype(np.float16)
    V = RNG.standard_normal((L, Hkv, d)).astype(np.float16)
    q = RNG.standard_normal((1, Hq, d)).astype(np.float16)
    pt = np.array([[2, 0]], np.int32)
    kp = np.zeros((3, Hkv, P, d), np.float16)
    vp = np.zeros_like(kp)
    for t in range(L):
        kp[pt[0, t // P], :, t % P] = K[t]
        vp[pt[0, t // P], :, t % P] = V[t]
    o = O.kv16_paged_decode_attn(kp, vp, q, pt, np.array([L]))
    assert np.allclose(o[0], O.attention_plain(q[0], K, V), atol=1e-13)


# ---------------------------------------------------------------- randomised Hadamard (sign diagonal)
def _signs(d, seed):
    return np.where(np.random.default_rng(seed).random(d) < 0.5, -1.0, 1.0)


@pytest.mark.parametrize("d,h", [(16, 4), (64, 16), (128, 32), (128, 128)])
def test_signed_rotation_is_orthonormal_and_entrywise_closed_form(d, h):
    sg = _signs(d, 7 + h)
    R = O.rotation_matrix(d, h, sg)
    assert np.allclose(R @ R.T, np.eye(d), atol=1e-12) and np.allclose(R.T @ R, np.eye(d), atol=1e-12)
    # entry (i, j): sigma_i (-1)^popcount(i & j within the block) / sqrt(h) inside a block, 0 outside
    for i in range(0, d, max(1, d // 8)):
        for j in range(d):
            want = 0.0 if i // h != j // h else sg[i] * (-1.0) ** bin((i % h) & (j % h)).count("1") / math.sqrt(h)
            assert R[i, j] == pytest.approx(want, abs=1e-15)
    x = RNG.standard_normal((5, d))
    y = RNG.standard_normal((5, d))
    assert np.allclose(O.rotate(x, h, sg) @ O.rotate(y, h, sg).T, x @ y.T, atol=1e-11)      # (qR)(kR)^T = q k^T
    assert np.allclose(O.unrotate(O.rotate(x, h, sg), h, sg), x, atol=1e-12)
    assert np.allclose(np.linalg.norm(O.rotate(x, h, sg), axis=-1), np.linalg.norm(x, axis=-1))
    # all +1 is the plain matrix; the transform is NOT symmetric any more once a sign differs
    assert np.array_equal(O.rotation_matrix(d, h, np.ones(d)), O.block_hadamard(d, h))
    if (sg < 0).any() and (sg > 0).any():
        assert not np.allclose(R, R.T)
    # a one-hot input picks out the signed Hadamard row
    e = np.zeros(d); e[3] = 2.0
    assert np.allclose(O.rotate(e, h, sg), 2.0 * sg[3] * O.block_hadamard(d, h)[3])


def test_signed_store_equals_plain_store_of_prerotated_input():
    """Storing x with (h, signs) must give the very bytes that a no-rotation store of x R gives,
    R built here as an explicit dense matrix (fp64 product rounded the same way: inputs are small
    integers over a power of two, so x R is exact in both routes)."""
    d, h, Hkv, T, P = 32, 16, 2, 20, 16
    sg = _signs(d, 99)
    R = np.diag(sg) @ scipy.linalg.block_diag(*[scipy.linalg.hadamard(h) / math.sqrt(h)] * (d // h))
    K = RNG.integers(-64, 64, size=(T, Hkv, d)).astype(np.float64) / 8.0
    V = RNG.integers(-64, 64, size=(T, Hkv, d)).astype(np.float64) / 8.0
    pt = np.array([[2, 0]], np.int32)
    sl = np.stack([np.zeros(T, np.int32), np.arange(T, dtype=np.int32)], 1)
    a = O.new_cache(3, Hkv, P, d)
    b = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(a, K, V, pt, sl, h, O.ROT_K | O.ROT_V, signs=sg)
    O.rotate_quant_store(b, K @ R, V @ R, pt, sl, 1)
    for key in ("k_codes", "v_codes", "k_meta", "v_meta"):
        assert np.array_equal(a[key], b[key]), key
    # and K-only rotation leaves V unsigned
    c = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(c, K, V, pt, sl, h, O.ROT_K, signs=sg)
    e = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(e, K, V, pt, sl, 1)
    assert np.array_equal(c["v_codes"], e["v_codes"]) and np.array_equal(c["k_codes"], a["k_codes"])
    # read-back with the inverse rotation returns to the input within the quantiser's bound
    kq, vq = O.dequant_pages(a, pt, 0, 0, T, h, unrotate=True, signs=sg)
    s_k = a["k_meta"][[2] * 16 + [0] * 4, :, list(range(16)) + list(range(4)), 0].astype(np.float64)   # [T][Hkv]
    err = np.linalg.norm(kq - K, axis=-1)
    assert np.all(err <= 0.5 * s_k * math.sqrt(d) * (1 + 1e-6))


@pytest.mark.parametrize("mask", [3, 1, 2])
def test_signed_decode_attention_vs_dense_matrix_route(mask):
    """Attention with (h, signs) over a cache stored with (h, signs) equals, to rounding, plain
    softmax attention over the cache read back through the explicit dense R^T, and the brute-force
    loop over a no-rotation cache of pre-rotated tokens gives the same rotated-space result."""
    d, h, Hq, Hkv, P = 16, 8, 4, 2, 16
    sg = _signs(d, 5)
    R = np.diag(sg) @ scipy.linalg.block_diag(*[scipy.linalg.hadamard(h) / math.sqrt(h)] * (d // h))
    L = np.array([7, 21], np.int32)
    pt = np.array([[3, 1], [0, 2]], np.int32)
    cache = O.new_cache(4, Hkv, P, d)
    plain = O.new_cache(4, Hkv, P, d)
    Ks, Vs = [], []
    for b in range(2):
        K = RNG.integers(-32, 32, size=(L[b], Hkv, d)).astype(np.float64) / 4.0
        V = RNG.integers(-32, 32, size=(L[b], Hkv, d)).astype(np.float64) / 4.0
        sl = np.stack([np.full(L[b], b, np.int32), np.arange(L[b], dtype=np.int32)], 1)
        O.rotate_quant_store(cache, K, V, pt, sl, h, mask, signs=sg)
        O.rotate_quant_store(plain, K @ R if mask & 1 else K, V @ R if mask & 2 else V, pt, sl, 1)
        Ks.append(K); Vs.append(V)
    q = RNG.standard_normal((2, Hq, d))
    o = O.paged_decode_attn(cache, q, pt, L, h, mask, signs=sg)
    # route 2: no-rotation cache of pre-rotated tokens, query rotated here, output rotated back here
    q2 = q @ R if mask & 1 else q
    o2 = _brute_force(plain, q2, pt, L, 1, 0)
    if mask & 2:
        o2 = o2 @ R.T
    assert np.allclose(o, o2, rtol=0, atol=1e-12)
    # route 3: library SDPA on the cache read back in the original space
    for b in range(2):
        kq, vq = O.dequant_pages(cache, pt, b, 0, int(L[b]), h, mask, unrotate=True, signs=sg)
        for j in range(Hq):
            g = j // (Hq // Hkv)
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(q[b, j][None, None]), torch.from_numpy(kq[:, g][None]),
                torch.from_numpy(vq[:, g][None])).numpy()[0, 0]
            assert np.allclose(o[b, j], ref, atol=1e-10)
    # all +1 signs reproduce the unsigned path bit for bit
    un = O.new_cache(4, Hkv, P, d)
    for b in range(2):
        sl = np.stack([np.full(L[b], b, np.int32), np.arange(L[b], dtype=np.int32)], 1)
        O.rotate_quant_store(un, Ks[b], Vs[b], pt, sl, h, mask, signs=np.ones(d))
    ref_un = O.new_cache(4, Hkv, P, d)
    for b in range(2):
        sl = np.stack([np.full(L[b], b, np.int32), np.arange(L[b], dtype=np.int32)], 1)
        O.rotate_quant_store(ref_un, Ks[b], Vs[b], pt, sl, h, mask)
    assert np.array_equal(un["k_codes"], ref_un["k_codes"]) and np.array_equal(un["v_meta"], ref_un["v_meta"])


# ---------------------------------------------------------------- learned per-layer rotation (App. A.3)
def _orthogonal(d, seed):
    """A seeded random orthogonal matrix (QR of a Gaussian matrix) standing in for a calibrated R_l."""
    Q, Rr = np.linalg.qr(np.random.default_rng(seed).standard_normal((d, d)))
    return Q * np.sign(np.diag(Rr))


@pytest.mark.parametrize("d,h", [(16, 4), (64, 16), (128, 64), (128, 1)])
def test_learned_rotation_composes_after_the_hadamard(d, h):
    Rl = _orthogonal(d, 11 + h)
    assert np.allclose(Rl @ Rl.T, np.eye(d), atol=1e-12)
    Hb = scipy.linalg.block_diag(*[scipy.linalg.hadamard(h) / math.sqrt(h)] * (d // h)) if h > 1 else np.eye(d)
    W = Hb @ Rl                                                   # q^ = (q H_b) R_l  =  q (H_b R_l)
    assert np.allclose(W @ W.T, np.eye(d), atol=1e-12)
    x = RNG.standard_normal((6, d))
    y = RNG.standard_normal((6, d))
    xr = O.rotate(x, h, None, Rl)
    assert np.allclose(xr, x @ W, atol=1e-12)
    if h > 1:
        assert not np.allclose(xr, x @ (Rl @ Hb), atol=1e-3)      # the other order is a different transform
        assert not np.allclose(xr, x @ (Hb @ Rl.T), atol=1e-3)    # and so is the transposed matrix
    assert np.allclose(xr @ O.rotate(y, h, None, Rl).T, x @ y.T, atol=1e-11)          # q^ . k^ = q . k (App. A.3)
    assert np.allclose(np.linalg.norm(xr, axis=-1), np.linalg.norm(x, axis=-1))
    assert np.allclose(O.unrotate(xr, h, None, Rl), x, atol=1e-12)
    # the identity as R_l is the Hadamard-only transform, bit for bit
    assert np.array_equal(O.rotate(x, h, None, np.eye(d)), O.rotate(x, h))
    # with signs: diag(sigma) H_b R_l
    sg = _signs(d, 3)
    if h > 1:
        assert np.allclose(O.rotate(x, h, sg, Rl), ((x * sg) @ Hb) @ Rl, atol=1e-12)
    else:                                                         # the signs belong to the Hadamard: none without it
        assert np.array_equal(O.rotate(x, h, sg, Rl), O.rotate(x, h, None, Rl))


def test_learned_rotation_permutation_moves_codes():
    """With a permutation matrix as R_l the stored codes are the Hadamard-only codes with their channels
    moved: y_j = (x H_b)_{pi(j)}.  The permutation is a cyclic shift (not its own inverse), so a
    transposed operand or a wrong multiplication order shows."""
    d, h, Hkv, T, P = 32, 16, 2, 20, 16
    shift = 5
    Pm = np.zeros((d, d))
    for j in range(d):
        Pm[(j + shift) % d, j] = 1.0                               # column j picks input channel j + shift
    K = RNG.integers(-64, 64, size=(T, Hkv, d)).astype(np.float64) / 8.0
    V = RNG.integers(-64, 64, size=(T, Hkv, d)).astype(np.float64) / 8.0
    pt = np.array([[2, 0]], np.int32)
    sl = np.stack([np.zeros(T, np.int32), np.arange(T, dtype=np.int32)], 1)
    a = O.new_cache(3, Hkv, P, d)
    b = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(a, K, V, pt, sl, h, O.ROT_K | O.ROT_V, dense=Pm)
    O.rotate_quant_store(b, K, V, pt, sl, h, O.ROT_K | O.ROT_V)
    for which in ("k", "v"):
        ca = O.unpack_nibbles(a[which + "_codes"])
        cb = O.unpack_nibbles(b[which + "_codes"])
        assert np.array_equal(ca, np.roll(cb, -shift, axis=-1)), which
        assert np.array_equal(a[which + "_meta"], b[which + "_meta"])          # same min, max: same (s, z)
    # K-only: V is stored without any rotation
    c = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(c, K, V, pt, sl, h, O.ROT_K, dense=Pm)
    e = O.new_cache(3, Hkv, P, d)
    O.rotate_quant_store(e, K, V, pt, sl, 1)
    assert np.array_equal(c["v_codes"], e["v_codes"]) and np.array_equal(c["k_codes"], a["k_codes"])


def test_learned_rotation_store_equals_plain_store_of_prerotated_input():
    d, h, Hkv, T, P = 32, 8, 2, 20, 16
    Rl = _orthogonal(d, 21)
    Hb = scipy.linalg.block_diag(*[scipy.linalg.hadamard(h) / math.sqrt(h)] * (d // h))
    K = RNG.standard_normal((T, Hkv, d))
    V = RNG.standard_normal((T, Hkv, d))
    pt = np.array([[1, 0]], np.int32)
    sl = np.stack([np.zeros(T, np.int32), np.arange(T, dtype=np.int32)], 1)
    a = O.new_cache(2, Hkv, P, d)
    b = O.new_cache(2, Hkv, P, d)
    O.rotate_quant_store(a, K, V, pt, sl, h, O.ROT_K | O.ROT_V, dense=Rl)
    O.rotate_quant_store(b, (K @ Hb) @ Rl, (V @ Hb) @ Rl, pt, sl, 1)
    for key in ("k_codes", "v_codes", "k_meta", "v_meta"):
        assert np.array_equal(a[key], b[key]), key
    # read-back through the inverse returns to the input within the quantiser's bound
    kq, _ = O.dequant_pages(a, pt, 0, 0, T, h, unrotate=True, dense=Rl)
    s_k = a["k_meta"][[1] * 16 + [0] * 4, :, list(range(16)) + list(range(4)), 0].astype(np.float64)
    assert np.all(np.linalg.norm(kq - K, axis=-1) <= 0.5 * s_k * math.sqrt(d) * (1 + 1e-6))


@pytest.mark.parametrize("mask,h", [(3, 8), (1, 8), (2, 8), (3, 1)])
def test_learned_rotation_decode_attention_three_routes(mask, h):
    """Attention with (h, R_l) over a cache stored with (h, R_l) against (2) the brute-force loop over a
    no-rotation cache of pre-rotated tokens with the query pre-rotated and the output multiplied by
    (H_b R_l)^T here, and (3) the library SDPA on the cache read back in the original space."""
    d, Hq, Hkv, P = 16, 4, 2, 16
    Rl = _orthogonal(d, 31)
    Hb = scipy.linalg.block_diag(*[scipy.linalg.hadamard(h) / math.sqrt(h)] * (d // h)) if h > 1 else np.eye(d)
    W = Hb @ Rl
    L = np.array([7, 21], np.int32)
    pt = np.array([[3, 1], [0, 2]], np.int32)
    cache = O.new_cache(4, Hkv, P, d)
    plain = O.new_cache(4, Hkv, P, d)
    for b in range(2):
        K = RNG.standard_normal((L[b], Hkv, d))
        V = RNG.standard_normal((L[b], Hkv, d))
        sl = np.stack([np.full(L[b], b, np.int32), np.arange(L[b], dtype=np.int32)], 1)
        O.rotate_quant_store(cache, K, V, pt, sl, h, mask, dense=Rl)
        O.rotate_quant_store(plain, (K @ Hb) @ Rl if mask & 1 else K, (V @ Hb) @ Rl if mask & 2 else V, pt, sl, 1)
    for key in ("k_codes", "v_codes", "k_meta", "v_meta"):
        assert np.array_equal(cache[key], plain[key]), key
    q = RNG.standard_normal((2, Hq, d))
    o = O.paged_decode_attn(cache, q, pt, L, h, mask, dense=Rl)
    o2 = _brute_force(plain, q @ W if mask & 1 else q, pt, L, 1, 0)
    if mask & 2:
        o2 = o2 @ W.T
    assert np.allclose(o, o2, rtol=0, atol=1e-12)
    for b in range(2):
        kq, vq = O.dequant_pages(cache, pt, b, 0, int(L[b]), h, mask, unrotate=True, dense=Rl)
        for j in range(Hq):
            g = j // (Hq // Hkv)
            ref = torch.nn.functional.scaled_dot_product_attention(
                torch.from_numpy(q[b, j][None, None]), torch.from_numpy(kq[:, g][None]),
                torch.from_numpy(vq[:, g][None])).numpy()[0, 0]
            assert np.allclose(o[b, j], ref, atol=1e-10)
