"""Seeded synthetic workloads shaped like the paper's GQA serving runs.

This module only draws random numbers and lays out page tables; it contains
none of the method's arithmetic (no rotation, no quantisation, no attention),
so the CPU oracle's tests and the HIP path can both be fed from it.

The five named workloads mirror the benchmark configurations: a tiny full-parity
case, a Llama-3-8B-shaped layer, a high-concurrency ragged batch, a long-context
small batch and a prefill-store sweep.  K/V are N(0,1) times a fixed per-(kv-head,
channel) scale that plants the channel-wise range heterogeneity the paper
attributes INT4's accuracy loss to (Sec. 3, "Token-Wise INT4 Quantization").
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np
import torch

BASE_SEED = 20260419


@dataclass
class Workload:
    name: str
    seed: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    page_size: int
    had_block: int
    dtype: torch.dtype
    seq_lens: np.ndarray            # [B] int32: tokens cached per sequence
    page_table: np.ndarray          # [B][max_pages_per_seq] int32, unused entries 0
    num_pages: int                  # pool size (>= pages referenced)
    k_chan_scale: np.ndarray        # [Hkv][d] float32
    v_chan_scale: np.ndarray        # [Hkv][d] float32
    rotate_mask: int = 3
    signs: np.ndarray | None = None     # [d] of +1 / -1: diagonal in front of the Hadamard matrix (None: plain)
    dense: np.ndarray | None = None     # [d][d] float64 holding float32 values: a learned rotation's stand-in (None: none)
    extra: dict = field(default_factory=dict)

    @property
    def batch(self) -> int:
        return int(self.seq_lens.shape[0])

    @property
    def max_pages_per_seq(self) -> int:
        return int(self.page_table.shape[1])

    @property
    def total_tokens(self) -> int:
        return int(self.seq_lens.astype(np.int64).sum())


def _chan_scale(rng: np.random.Generator, kind: str, Hkv: int, d: int) -> np.ndarray:
    s = np.ones((Hkv, d), np.float32)
    if kind == "none":
        pass
    elif kind.startswith("outlier4x"):          # 4 fixed channels per head, times a factor
        f = float(kind[len("outlier4x"):])
        for g in range(Hkv):
            s[g, rng.choice(d, size=4, replace=False)] = f
    elif kind.startswith("pct1x"):              # 1 % of all Hkv*d channels, times a factor
        f = float(kind[len("pct1x"):])
        n = max(1, round(0.01 * Hkv * d))
        idx = rng.choice(Hkv * d, size=n, replace=False)
        s.reshape(-1)[idx] = f
    elif kind == "student_t3":                  # heavy-tailed |t_3| scale per channel
        s = np.abs(rng.standard_t(3.0, size=(Hkv, d))).astype(np.float32)
        s = np.maximum(s, np.float32(1e-3))
    else:
        raise ValueError(kind)
    return s


def _page_table(rng: np.random.Generator, seq_lens: np.ndarray, P: int, extra_tokens: int,
                slack_pages: int, shuffle: bool = True):
    """Pool of pages in a seeded random order; each sequence owns enough for L + extra tokens."""
    need = [(int(L) + extra_tokens + P - 1) // P for L in seq_lens]
    total = int(sum(need))
    num_pages = total + slack_pages
    perm = rng.permutation(num_pages)          # always drawn, so later draws do not depend on `shuffle`
    if not shuffle:
        perm = np.arange(num_pages)
    width = max(1, max(need))
    pt = np.zeros((len(seq_lens), width), np.int32)
    o = 0
    for b, n in enumerate(need):
        pt[b, :n] = perm[o:o + n]
        o += n
    return pt, num_pages


def make_workload(name: str, rep: int = 0, **over) -> Workload:
    """Build one of: tiny, llama8b, highconc, longctx1, longctx4, prefill, prefill_mha.

    Keyword overrides (``batch``, ``ctx``, ``had_block``, ``dtype`` ...) shrink or
    vary a workload while keeping its recipe, so tests can run the same
    structure at sizes a CPU finishes in seconds.
    """
    table = {
        #  name        idx  B    ctx            Hq  Hkv d    h    dtype            scales
        "tiny":       (0,   4,   256,           32, 8,  128, 128, torch.float16,  "outlier4x20"),
        "llama8b":    (1,   16,  4096,          32, 8,  128, 128, torch.bfloat16, "pct1x10"),
        "highconc":   (2,   256, (512, 4096),   32, 8,  128, 64,  torch.bfloat16, "student_t3"),
        "longctx1":   (3,   1,   131072,        64, 8,  128, 128, torch.bfloat16, "outlier4x20"),
        "longctx4":   (3,   4,   131072,        64, 8,  128, 128, torch.bfloat16, "outlier4x20"),
        "prefill":    (4,   1,   32768,         32, 8,  128, 128, torch.bfloat16, "outlier4x20"),
        "prefill_mha": (4,  1,   32768,         32, 32, 64,  64,  torch.bfloat16, "outlier4x20"),
    }
    idx, B, ctx, Hq, Hkv, d, h, dtype, kind = table[name]
    B = over.get("batch", B)
    ctx = over.get("ctx", ctx)
    Hq = over.get("n_q_heads", Hq)
    Hkv = over.get("n_kv_heads", Hkv)
    d = over.get("head_dim", d)
    h = over.get("had_block", h)
    dtype = over.get("dtype", dtype)
    kind = over.get("scales", kind)
    P = over.get("page_size", 16)
    seed = BASE_SEED + 1000 * idx + rep
    rng = np.random.default_rng(seed)
    if isinstance(ctx, tuple):
        seq_lens = rng.integers(ctx[0], ctx[1] + 1, size=B).astype(np.int32)
    else:
        seq_lens = np.full(B, ctx, np.int32)
    if "seq_lens" in over:
        seq_lens = np.asarray(over["seq_lens"], np.int32)
    pt, num_pages = _page_table(rng, seq_lens, P, over.get("extra_tokens", 16),
                                over.get("slack_pages", 3), over.get("shuffle", True))
    if over.get("table_width", 0) > pt.shape[1]:
        # a page table wider than any sequence needs (a serving engine sizes it for the longest context it
        # admits); the extra entries are never used and stay 0
        pt = np.concatenate([pt, np.zeros((pt.shape[0], over["table_width"] - pt.shape[1]), np.int32)], axis=1)
    ks = _chan_scale(rng, kind, Hkv, d)
    vs = _chan_scale(rng, kind, Hkv, d)
    return Workload(name=name, seed=seed, n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, page_size=P,
                    had_block=h, dtype=dtype, seq_lens=seq_lens, page_table=pt, num_pages=num_pages,
                    k_chan_scale=ks, v_chan_scale=vs, rotate_mask=over.get("rotate_mask", 3),
                    signs=random_signs(d, over["sign_seed"]) if over.get("sign_seed") is not None else None,
                    dense=random_orthogonal(d, over["dense_seed"]) if over.get("dense_seed") is not None else None)


def random_signs(d: int, seed: int) -> np.ndarray:
    """d values of +1 / -1, half of them negative on average (the diagonal of a randomised Hadamard)."""
    return np.where(np.random.default_rng(int(seed)).random(d) < 0.5, -1.0, 1.0)


def random_orthogonal(d: int, seed: int) -> np.ndarray:
    """A seeded random orthogonal d x d matrix (QR of a Gaussian matrix, column signs fixed), rounded to
    float32 and returned as float64, so that a float32 copy on the device holds exactly these values.
    It stands in for a calibrated per-layer rotation, which this repository has no data to compute."""
    Q, Rr = np.linalg.qr(np.random.default_rng(int(seed)).standard_normal((d, d)))
    return (Q * np.sign(np.diag(Rr))).astype(np.float32).astype(np.float64)


def _gen(seed: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    return g


def gen_kv(w: Workload, seq: int, pos_begin: int, pos_end: int, device="cpu"):
    """K, V ``[n][Hkv][d]`` in the workload dtype for positions [pos_begin, pos_end) of one sequence.

    The draw depends only on (seed, seq, pos_begin, n), so any chunk can be
    regenerated later for a sampled comparison.
    """
    n = pos_end - pos_begin
    g = _gen(w.seed * 1000003 + seq * 7919 + pos_begin, device)
    shape = (n, w.n_kv_heads, w.head_dim)
    ks = torch.from_numpy(w.k_chan_scale).to(device)
    vs = torch.from_numpy(w.v_chan_scale).to(device)
    K = (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * ks).to(w.dtype)
    V = (torch.randn(shape, generator=g, device=device, dtype=torch.float32) * vs).to(w.dtype)
    return K, V


def gen_q(w: Workload, device="cpu", step: int = 0) -> torch.Tensor:
    g = _gen(w.seed * 1000003 + 999331 + step, device)
    return torch.randn((w.batch, w.n_q_heads, w.head_dim), generator=g, device=device,
                       dtype=torch.float32).to(w.dtype)


def slots_for(seq: int, pos_begin: int, pos_end: int) -> np.ndarray:
    """``[n][2]`` int32 rows of (sequence index, logical position)."""
    pos = np.arange(pos_begin, pos_end, dtype=np.int32)
    return np.stack([np.full_like(pos, seq), pos], axis=1)
