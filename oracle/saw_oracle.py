"""CPU oracle for the SAW-INT4 KV-cache hot path.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain, fp64 statement of what the hot path computes.
Only the tests, the smoke check and the bench's ``cpu_baseline`` leg may import
it; the product (the HIP library and its Python binding) never does, and the
two share no code, tables or helpers.

What it follows (paper sections / equations, restated in code):

* Token-wise asymmetric INT4 quantisation -- App. A.1, the two displayed
  equations: ``s = (max - min) / 15``, ``z = round(-min / s)``,
  ``c_i = clip(round(x_i / s) + z, 0, 15)``, ``x^_i = s (c_i - z)``; two
  neighbouring codes share one byte.
* Orthonormal rotation before quantisation -- Sec. 3 eq. (1) and App. A.4:
  ``K~ = quant(K H)``, ``V~ = quant(V H)`` with ``H = H^T``, ``H H^T = I``.
* Block-diagonal rotation BDR-h -- Sec. 3 eqs. (2)-(3) and App. A.4: the head
  vector is cut into ``d/h`` contiguous chunks and each chunk is multiplied by
  the order-``h`` Hadamard matrix, i.e. ``H_blk = diag(H_h, ..., H_h)``.
* Attention in the rotated space -- Sec. 4.1 and App. A.4:
  ``Score = softmax((q H) dequant(K~)^T / sqrt(d))`` and
  ``Output = Score dequant(V~) H``; Sec. 2 gives the decode step as
  ``o = softmax(q K^T / sqrt(d)) V``.
* Randomised Hadamard -- Sec. 3 says the transforms used in practice are
  randomised; the standard construction (a fixed +/-1 diagonal in front of the
  Hadamard matrix) is taken: ``R = diag(sigma) H_blk``, still orthonormal,
  ``R^-1 = R^T = H_blk diag(sigma)``.  ``signs=None`` is the plain matrix.
* Learned per-layer rotation -- Sec. 3 ("Hessian-Aware Quantization") and
  App. A.3, runtime application: a dense orthogonal ``d x d`` matrix ``R_l`` is
  composed AFTER the block Hadamard, ``q^ = (q H_b) R_l``, ``k^ = (k H_b) R_l``,
  and the same transform is applied to V; the output returns through the
  transpose, ``o = o~ R_l^T H_b``.  ``dense=None`` leaves it out.  How ``R_l``
  is calibrated (the damped eigendecomposition of App. A.3) is outside this
  path: the matrix is an input.
* Paged cache -- Sec. 2 ("Paged Memory Layouts"): fixed-size pages of one
  uniform type reached through a page table, token-wise metadata only.

Readings taken where the paper is silent (all listed again in the design
notes): Sylvester/natural-order Hadamard scaled by 1/sqrt(h); one (s, z) pair
per (token, head) over all d channels even when h < d; round = round half to
even; z is an unclamped integer; a constant vector gets s = |max| (or 1 when it
is all zero); even channel -> low nibble; (s, z) are kept as fp32; logits are
scaled by 1/sqrt(d) with d the head dimension; query head j reads kv head
j // (Hq / Hkv).  These conventions are "parity unpinned" by the paper: the
tests pin the arithmetic (equations, identities, brute force), not the
conventions.

Everything is numpy fp64 with explicit matrices: no butterflies, no online
softmax, no tiling.
"""
from __future__ import annotations

import numpy as np

__all__ = [
    "hadamard", "block_hadamard", "rotate", "quantize", "dequantize",
    "pack_nibbles", "unpack_nibbles", "new_cache", "rotation_matrix", "unrotate", "rotates", "rotate_quant_store",
    "dequant_pages", "paged_decode_attn", "kv16_paged_decode_attn",
    "attention_plain",
]

ROT_K = 1  # bit 0 of rotate_mask: K (and q) live in the rotated space
ROT_V = 2  # bit 1 of rotate_mask: V lives in the rotated space, o is rotated back


# --------------------------------------------------------------------------
# Rotation (Sec. 3 eqs. 1-3, App. A.4)
# --------------------------------------------------------------------------
def hadamard(h: int) -> np.ndarray:
    """Orthonormal order-``h`` Hadamard matrix by Sylvester doubling.

    ``H_1 = [1]``, ``H_2n = [[H_n, H_n], [H_n, -H_n]]``, then scaled by
    ``1/sqrt(h)`` so that ``H H^T = I`` holds exactly (App. A.4 states the
    identity "up to normalisation"; the normalised form is the one used).
    """
    if h < 1 or (h & (h - 1)) != 0:
        raise ValueError("Hadamard order must be a power of two")
    H = np.ones((1, 1), dtype=np.float64)
    while H.shape[0] < h:
        H = np.block([[H, H], [H, -H]])
    return H / np.sqrt(np.float64(h))


def block_hadamard(d: int, h: int) -> np.ndarray:
    """``H_blk = diag(H_h, ..., H_h)`` with ``d/h`` diagonal blocks (Sec. 3 eq. 3)."""
    if h < 1 or d % h != 0:
        raise ValueError("block size must divide the head dimension")
    Hh = hadamard(h)
    out = np.zeros((d, d), dtype=np.float64)
    for i in range(d // h):
        out[i * h:(i + 1) * h, i * h:(i + 1) * h] = Hh
    return out


def rotation_matrix(d: int, h: int, signs=None) -> np.ndarray:
    """``R = diag(sigma) H_blk`` (Sec. 3: randomised Hadamard; ``signs`` = sigma, d entries of +/-1;
    None = all +1, the plain block Hadamard)."""
    R = block_hadamard(d, h)
    if signs is not None:
        sg = np.asarray(signs, np.float64)
        if sg.shape != (d,) or not np.all(np.abs(sg) == 1.0):
            raise ValueError("signs must be d values of +1 or -1")
        R = np.diag(sg) @ R
    return R


def _dense(dense, d: int):
    Rl = np.asarray(dense, np.float64)
    if Rl.shape != (d, d):
        raise ValueError("the learned rotation must be a d x d matrix")
    return Rl


def rotates(h: int, dense=None) -> bool:
    """Whether a tensor whose rotate_mask bit is set is transformed at all: a Hadamard order above 1, or
    a learned rotation (which may also be used alone, with ``h == 1``)."""
    return h > 1 or dense is not None


def rotate(x: np.ndarray, h: int, signs=None, dense=None) -> np.ndarray:
    """``(x R) R_l`` along the last axis, dense mat-vecs in fp64, in the order App. A.3 prints: the
    (signed) block Hadamard first, the learned rotation ``dense`` = ``R_l`` after it.  ``h == 1``
    skips the Hadamard (signs ignored: they are part of it); ``dense=None`` skips ``R_l``."""
    x = np.asarray(x, dtype=np.float64)
    y = x.copy() if h == 1 else x @ rotation_matrix(x.shape[-1], h, signs)
    if dense is not None:
        y = y @ _dense(dense, x.shape[-1])
    return y


def unrotate(y: np.ndarray, h: int, signs=None, dense=None) -> np.ndarray:
    """The inverse of ``rotate``: ``(y R_l^T) R^T`` (App. A.4: the transpose undoes an orthonormal
    rotation; for the plain symmetric Hadamard alone this is the same matrix again)."""
    y = np.asarray(y, dtype=np.float64)
    x = y.copy() if dense is None else y @ _dense(dense, y.shape[-1]).T
    if h > 1:
        x = x @ rotation_matrix(y.shape[-1], h, signs).T
    return x


_inverse_rotation = unrotate      # (dequant_pages has a flag of the same name)


# --------------------------------------------------------------------------
# Token-wise asymmetric INT4 (App. A.1)
# --------------------------------------------------------------------------
def quantize(y: np.ndarray):
    """Quantise every vector along the last axis with one shared (s, z).

    Returns ``(codes uint8 [..., d], s float64 [...], z float64 [...])``.
    ``np.rint`` rounds half to even.  A constant vector would give ``s = 0``;
    it takes ``s = |max|`` (1 if the vector is all zero), which makes every
    code 0 and ``s (0 - z)`` reproduce the constant exactly.
    """
    y = np.asarray(y, dtype=np.float64)
    mn = y.min(axis=-1)
    mx = y.max(axis=-1)
    s = (mx - mn) / 15.0
    flat = s == 0.0
    s = np.where(flat, np.where(mx != 0.0, np.abs(mx), 1.0), s)
    z = np.rint(-mn / s)
    c = np.rint(y / s[..., None]) + z[..., None]
    c = np.clip(c, 0.0, 15.0)
    return c.astype(np.uint8), s, z


def dequantize(codes: np.ndarray, s: np.ndarray, z: np.ndarray) -> np.ndarray:
    """``x^ = s (c - z)`` (App. A.1, second equation)."""
    return (np.asarray(s, np.float64)[..., None]
            * (codes.astype(np.float64) - np.asarray(z, np.float64)[..., None]))


def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """Two neighbouring codes per byte: channel 2j -> low nibble, 2j+1 -> high nibble."""
    c = np.asarray(codes, dtype=np.uint8)
    return (c[..., 0::2] | (c[..., 1::2] << 4)).astype(np.uint8)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    p = np.asarray(packed, dtype=np.uint8)
    out = np.empty(p.shape[:-1] + (p.shape[-1] * 2,), dtype=np.uint8)
    out[..., 0::2] = p & 0x0F
    out[..., 1::2] = p >> 4
    return out


# --------------------------------------------------------------------------
# Paged cache (Sec. 2, "Paged Memory Layouts")
# --------------------------------------------------------------------------
def new_cache(num_pages: int, n_kv_heads: int, page_size: int, head_dim: int) -> dict:
    """Empty cache: codes ``[page][kv_head][slot][d/2]`` u8, meta ``[page][kv_head][slot][2]`` f32."""
    shape_c = (num_pages, n_kv_heads, page_size, head_dim // 2)
    shape_m = (num_pages, n_kv_heads, page_size, 2)
    return {
        "k_codes": np.zeros(shape_c, np.uint8), "v_codes": np.zeros(shape_c, np.uint8),
        "k_meta": np.zeros(shape_m, np.float32), "v_meta": np.zeros(shape_m, np.float32),
        "page_size": page_size, "head_dim": head_dim, "n_kv_heads": n_kv_heads,
    }


def _encode(x: np.ndarray, h: int, rot: bool, signs=None, dense=None):
    y = rotate(x, h, signs, dense) if rot else np.asarray(x, np.float64)
    codes, s, z = quantize(y)
    return pack_nibbles(codes), s, z, y


def rotate_quant_store(cache: dict, K: np.ndarray, V: np.ndarray, page_table: np.ndarray,
                       slots: np.ndarray, had_block: int, rotate_mask: int = ROT_K | ROT_V,
                       return_prerounding: bool = False, signs=None, dense=None):
    """Rotate, quantise and place ``T`` new tokens (Sec. 3 eq. 1-3 then App. A.1; with ``dense`` the
    learned rotation of App. A.3 follows the Hadamard for every tensor whose mask bit is set).

    ``K, V``: ``[T][Hkv][d]`` (any float dtype, widened exactly to fp64).
    ``slots[t] = (sequence, logical position)``; the token lands in physical
    page ``page_table[sequence][position // P]`` at slot ``position % P``.
    With ``return_prerounding`` the fp64 rotated values and the unrounded
    (s, z) are returned too, so a comparator can tell how close an element was
    to a rounding boundary.
    """
    P = cache["page_size"]
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    h = int(had_block)
    kp, ks, kz, ky = _encode(K, h, bool(rotate_mask & ROT_K) and rotates(h, dense), signs, dense)
    vp, vs, vz, vy = _encode(V, h, bool(rotate_mask & ROT_V) and rotates(h, dense), signs, dense)
    seq = slots[:, 0].astype(np.int64)
    pos = slots[:, 1].astype(np.int64)
    page = np.asarray(page_table)[seq, pos // P].astype(np.int64)
    slot = pos % P
    cache["k_codes"][page, :, slot, :] = kp
    cache["v_codes"][page, :, slot, :] = vp
    cache["k_meta"][page, :, slot, 0] = ks.astype(np.float32)
    cache["k_meta"][page, :, slot, 1] = kz.astype(np.float32)
    cache["v_meta"][page, :, slot, 0] = vs.astype(np.float32)
    cache["v_meta"][page, :, slot, 1] = vz.astype(np.float32)
    if return_prerounding:
        return {"k_y": ky, "k_s": ks, "k_z": kz, "v_y": vy, "v_s": vs, "v_z": vz,
                "page": page, "slot": slot}
    return None


def _gather(cache: dict, which: str, page_table_row: np.ndarray, pos_begin: int, pos_end: int):
    """Dequantised (still rotated) values ``[pos_end-pos_begin][Hkv][d]`` of one sequence, fp64."""
    P = cache["page_size"]
    pos = np.arange(pos_begin, pos_end, dtype=np.int64)
    page = np.asarray(page_table_row)[pos // P].astype(np.int64)
    slot = pos % P
    codes = unpack_nibbles(cache[which + "_codes"][page, :, slot, :])   # [n][Hkv][d]
    meta = cache[which + "_meta"][page, :, slot, :].astype(np.float64)  # [n][Hkv][2]
    return dequantize(codes, meta[..., 0], meta[..., 1])


def dequant_pages(cache: dict, page_table: np.ndarray, seq: int, pos_begin: int, pos_end: int,
                  had_block: int, rotate_mask: int = ROT_K | ROT_V, unrotate: bool = False, signs=None,
                  dense=None):
    """Read back positions ``[pos_begin, pos_end)`` of one sequence as fp64 ``(K^, V^)``.

    ``unrotate`` applies the inverse rotation (App. A.4; for the plain
    Hadamard, symmetric and orthonormal, that is the same matrix once more;
    with a learned rotation ``R_l^T`` first, then the Hadamard's transpose).
    """
    k = _gather(cache, "k", page_table[seq], pos_begin, pos_end)
    v = _gather(cache, "v", page_table[seq], pos_begin, pos_end)
    if unrotate and rotates(had_block, dense):
        if rotate_mask & ROT_K:
            k = _inverse_rotation(k, had_block, signs, dense)
        if rotate_mask & ROT_V:
            v = _inverse_rotation(v, had_block, signs, dense)
    return k, v


# --------------------------------------------------------------------------
# Decode attention (Sec. 2; Sec. 4.1; App. A.4)
# --------------------------------------------------------------------------
def _softmax_rows(logits: np.ndarray) -> np.ndarray:
    m = logits.max(axis=-1, keepdims=True)
    e = np.exp(logits - m)
    return e / e.sum(axis=-1, keepdims=True)


def paged_decode_attn(cache: dict, q: np.ndarray, page_table: np.ndarray, seq_lens: np.ndarray,
                      had_block: int, rotate_mask: int = ROT_K | ROT_V,
                      sm_scale: float | None = None, signs=None, dense=None) -> np.ndarray:
    """One decode step over the INT4 cache as stored: ``o = softmax(q~ K^^T / sqrt(d)) V^ [R^T]``.

    ``q``: ``[B][Hq][d]``.  ``q~ = q R`` when K is rotated, else ``q``; the
    result is multiplied by ``R^T`` when V is rotated (``R = diag(signs) H_blk``;
    without signs ``R^T = R = H_blk``; with a learned rotation ``dense`` = ``R_l``,
    App. A.3: ``q~ = (q R) R_l`` and the result is multiplied by ``R_l^T`` and then
    ``R^T``).  A sequence of length 0 gives a zero row.
    """
    q = np.asarray(q, np.float64)
    B, Hq, d = q.shape
    Hkv = cache["n_kv_heads"]
    G = Hq // Hkv
    h = int(had_block)
    scale = (1.0 / np.sqrt(np.float64(d))) if (sm_scale is None or sm_scale <= 0) else float(sm_scale)
    rot_k = bool(rotate_mask & ROT_K) and rotates(h, dense)
    rot_v = bool(rotate_mask & ROT_V) and rotates(h, dense)
    out = np.zeros((B, Hq, d), np.float64)
    for b in range(B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        khat = _gather(cache, "k", page_table[b], 0, L)   # [L][Hkv][d]
        vhat = _gather(cache, "v", page_table[b], 0, L)
        for g in range(Hkv):
            qg = q[b, g * G:(g + 1) * G, :]                # [G][d]
            qt = rotate(qg, h, signs, dense) if rot_k else qg
            logits = (qt @ khat[:, g, :].T) * scale        # [G][L]
            p = _softmax_rows(logits)
            o = p @ vhat[:, g, :]                          # [G][d]
            out[b, g * G:(g + 1) * G, :] = unrotate(o, h, signs, dense) if rot_v else o
    return out


def kv16_paged_decode_attn(k_pages: np.ndarray, v_pages: np.ndarray, q: np.ndarray,
                           page_table: np.ndarray, seq_lens: np.ndarray,
                           sm_scale: float | None = None) -> np.ndarray:
    """The unquantised comparison path: same decode step over 16-bit pages ``[page][kv_head][slot][d]``."""
    q = np.asarray(q, np.float64)
    B, Hq, d = q.shape
    Hkv, P = k_pages.shape[1], k_pages.shape[2]
    G = Hq // Hkv
    scale = (1.0 / np.sqrt(np.float64(d))) if (sm_scale is None or sm_scale <= 0) else float(sm_scale)
    out = np.zeros((B, Hq, d), np.float64)
    for b in range(B):
        L = int(seq_lens[b])
        if L == 0:
            continue
        pos = np.arange(L)
        page = np.asarray(page_table[b])[pos // P].astype(np.int64)
        slot = pos % P
        k = np.asarray(k_pages[page, :, slot, :], np.float64)
        v = np.asarray(v_pages[page, :, slot, :], np.float64)
        for g in range(Hkv):
            logits = (q[b, g * G:(g + 1) * G, :] @ k[:, g, :].T) * scale
            out[b, g * G:(g + 1) * G, :] = _softmax_rows(logits) @ v[:, g, :]
    return out


def attention_plain(q: np.ndarray, K: np.ndarray, V: np.ndarray, sm_scale: float | None = None):
    """Textbook ``softmax(q K^T / sqrt(d)) V`` for one sequence: ``q [Hq][d]``, ``K, V [L][Hkv][d]``."""
    q = np.asarray(q, np.float64)
    K = np.asarray(K, np.float64)
    V = np.asarray(V, np.float64)
    Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    scale = (1.0 / np.sqrt(np.float64(d))) if (sm_scale is None or sm_scale <= 0) else float(sm_scale)
    out = np.zeros((Hq, d), np.float64)
    for j in range(Hq):
        g = j // G
        out[j] = _softmax_rows(((K[:, g, :] @ q[j]) * scale)[None, :])[0] @ V[:, g, :]
    return out
