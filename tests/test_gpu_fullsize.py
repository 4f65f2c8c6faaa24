"""Parity at the benchmark's full sizes, in the launch configuration bench.py times (automatic split
choice, bf16 inputs, fp32 or bf16 output): the whole workload runs through the HIP path and EVERY sequence
is compared with the oracle, over cache bytes the oracle's store wrote (uploaded), so that both sides
attend over identical bytes.  The call bench.py times as its step, saw_append_decode_attn on the ragged
256-sequence batch, is compared the same way: every sequence's output and every appended token's codes.
Properties that hold at any size (finite output, a convex combination of cached vectors cannot be longer
than the longest of them, bit-identical repeats) are checked as well.
"""
import numpy as np
import pytest
import torch

import gpu_cases as gc
import parity
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2e-3


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _fill_device(w, saw, skip, chunk=8192):
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        if b in skip:
            continue
        L = int(w.seq_lens[b])
        for p0 in range(0, L, chunk):
            p1 = min(L, p0 + chunk)
            K, V = synth.gen_kv(w, b, p0, p1, device="cuda")
            saw.rotate_quant_store(cache, K, V, pt, torch.from_numpy(synth.slots_for(b, p0, p1)).cuda())
    torch.cuda.synchronize()
    return cache, pt


def _pages_of(w, seqs):
    P = w.page_size
    return np.concatenate([w.page_table[b, :(int(w.seq_lens[b]) + P - 1) // P] for b in seqs])


def _sample(w, n):
    order = np.argsort(w.seq_lens, kind="stable")
    picks = {int(order[0]), int(order[-1])}                       # shortest and longest always
    rng = np.random.default_rng(w.seed + 77)
    while len(picks) < min(n, w.batch):
        picks.add(int(rng.integers(0, w.batch)))
    return sorted(picks)


@pytest.mark.parametrize("name,n_sample,out_dtype,over", [
    ("highconc", None, torch.bfloat16, {}),  # the headline configuration: 256 ragged sequences, bf16 in and out
    ("highconc", None, torch.float32, {}),
    ("llama8b", None, torch.float32, {}),
    ("longctx4", None, torch.float32, {}),
    ("longctx1", None, torch.float32, {}),
    # the other figures bench.py reports: 1024 items (four-wavefront pair blocks), and head_dim 64 (pairs of
    # kv heads per block) with 8 and with 32 kv heads (the last one sampled: 4096 items, longest first)
    ("highconc", None, torch.float32, dict(n_q_heads=16, n_kv_heads=4)),
    ("highconc", None, torch.float32, dict(head_dim=64, had_block=64)),
    ("highconc", 6, torch.float32, dict(head_dim=64, had_block=64, n_kv_heads=32)),
])
def test_decode_full_size(saw, name, n_sample, out_dtype, over):
    """`n_sample` None: every sequence of the workload is compared with the oracle."""
    w = synth.make_workload(name, **over)
    seqs = list(range(w.batch)) if n_sample is None else _sample(w, n_sample)
    print(f"[{name}] B={w.batch} tokens={w.total_tokens} compared sequences: {len(seqs)} of {w.batch}", flush=True)
    ref = gc.oracle_fill(w, chunk=8192, seqs=seqs)
    cache, pt = _fill_device(w, saw, skip=set(seqs))
    gc.upload_cache(ref, w, saw, into=cache, pages=_pages_of(w, seqs))
    q = synth.gen_q(w)
    sl = torch.from_numpy(w.seq_lens).cuda()
    o = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=out_dtype, device="cuda")
    saw.paged_decode_attn(cache, q.cuda(), pt, sl, max_seq_len=int(w.seq_lens.max()), out=o)   # every row written
    torch.cuda.synchronize()
    # the path has no atomics and a fixed reduction order: repeated launches agree bit for bit
    for _ in range(3):
        again = saw.paged_decode_attn(cache, q.cuda(), pt, sl, max_seq_len=int(w.seq_lens.max()), out_dtype=out_dtype)
        assert torch.equal(o, again), f"{name}: repeated launches differ"
    o = o.float().cpu().numpy()
    assert np.isfinite(o).all()
    plan = saw.decode_plan(cache, w.batch, int(w.seq_lens.max()))
    # the compared sequences against the oracle, one by one (error relative to the sequence's own largest value)
    worst, worst_b = 0.0, -1
    for b in seqs:
        o_ref = O.paged_decode_attn(ref, q[b:b + 1].float().numpy(), w.page_table[b:b + 1], w.seq_lens[b:b + 1],
                                    w.had_block, w.rotate_mask)
        err = parity.attn_error(o[b:b + 1], o_ref)
        if err > worst:
            worst, worst_b = err, b
    print(f"  worst: seq {worst_b} len {int(w.seq_lens[worst_b])}: err={worst:.2e}", flush=True)
    tol = TOL if out_dtype == torch.float32 else TOL + 2.0 ** -8
    assert worst < tol, f"{name}: plan={plan} worst error {worst:.2e} (sequence {worst_b})"
    # every sequence: the output is a convex combination of dequantised V rows (un-rotated by an
    # orthonormal matrix), so its norm cannot exceed the largest row norm; sqrt(d) * max|s (c - z)| <=
    # sqrt(d) * 15 * max scale bounds that without dequantising the cache.
    vmax = float(cache.v_meta[..., 0].abs().max()) * 15.0 * np.sqrt(w.head_dim)
    assert np.linalg.norm(o, axis=-1).max() <= vmax * 1.01
    nonempty = w.seq_lens > 0
    assert (np.abs(o[nonempty]).max(axis=(1, 2)) > 0).all()


@pytest.mark.parametrize("name,over,hint", [("highconc", {}, True), ("highconc", {}, False), ("llama8b", {}, False),
                                            ("highconc", dict(head_dim=64, had_block=64), True)])
def test_append_decode_full_size(saw, name, over, hint):
    """The step bench.py times: saw_append_decode_attn on the whole workload in the bench's launch shape
    (bf16 K/V/q, fp32 output, the bound at the longest sequence).  Every sequence's output against the oracle
    (2e-3; a sequence whose new token took a code the boundary rule exempts: the loose composed bound), every
    appended token's codes and metadata under the store criterion, nothing else in the cache changed.
    `hint`: with the caller's longest-first order, as bench.py calls it (saw_append_decode_attn_hinted)."""
    import test_gpu_append as TA
    w = synth.make_workload(name, **over)
    print(f"[{name} {over}] B={w.batch} tokens={w.total_tokens}", flush=True)
    TA._case(saw, w, order=np.argsort(-w.seq_lens, kind="stable") if hint else None)


@pytest.mark.parametrize("name", ["prefill", "prefill_mha"])
def test_store_full_size(saw, name):
    """32k-token prefill store, every vector compared with the oracle (bit-exact codes up to the boundary rule)."""
    w = synth.make_workload(name)
    cache, ref, recs, _ = gc.fill_caches(w, saw, chunk=32768)
    res = gc.compare_store(gc.cache_to_numpy(cache, w), ref, recs)
    print(f"[{name}] {res}", flush=True)
    parity.assert_store_ok(res)


@pytest.mark.parametrize("name", ["prefill", "prefill_mha"])
def test_flatten_full_size_sampled(saw, name):
    """32k-token flatten in the launch shape the bench times (whole sequence, bf16 out, rotated back):
    sampled token ranges against the oracle's read-back of the oracle-written bytes (only the sampled
    pages are uploaded, the rest of the device cache is the HIP store's), every output row written,
    repeated launches identical."""
    import test_gpu_flatten as TF
    w = synth.make_workload(name)
    T = int(w.seq_lens[0])
    cache, _, _, pt = gc.fill_caches(w, saw, chunk=32768, with_ref=False)
    rng = np.random.default_rng(11)
    starts = sorted({0, T - 40, *[int(x) for x in rng.integers(0, T - 64, size=6)]})
    ranges = [(p0, min(T, p0 + 40)) for p0 in starts]
    # oracle bytes for the sampled positions: store those chunks with the oracle, upload their pages
    ref = O.new_cache(w.num_pages, w.n_kv_heads, w.page_size, w.head_dim)
    pages = set()
    for p0, p1 in ranges:
        a, b = (p0 // 16) * 16, min(T, ((p1 + 15) // 16) * 16)
        K, V = synth.gen_kv(w, 0, a, b)
        O.rotate_quant_store(ref, K.float().numpy(), V.float().numpy(), w.page_table, synth.slots_for(0, a, b),
                                w.had_block, w.rotate_mask)
        pages.update(int(w.page_table[0, p // 16]) for p in range(a, b, 16))
    gc.upload_cache(ref, w, saw, into=cache, pages=sorted(pages))
    k = torch.full((T, w.n_kv_heads, w.head_dim), float("nan"), dtype=torch.bfloat16, device="cuda")
    v = torch.full_like(k, float("nan"))
    saw.flatten_dequant(cache, pt, 0, 0, T, unrotate=True, k_out=k, v_out=v)
    torch.cuda.synchronize()
    assert torch.isfinite(k.float()).all() and torch.isfinite(v.float()).all()      # every row written
    for p0, p1 in ranges:
        kr, vr = O.dequant_pages(ref, w.page_table, 0, p0, p1, w.had_block, w.rotate_mask, unrotate=True)
        TF._check(k[p0:p1], kr, torch.bfloat16, f"[{name} full size [{p0},{p1})] K")
        TF._check(v[p0:p1], vr, torch.bfloat16, f"[{name} full size [{p0},{p1})] V")
    k2 = torch.empty_like(k)
    v2 = torch.empty_like(v)
    saw.flatten_dequant(cache, pt, 0, 0, T, unrotate=True, k_out=k2, v_out=v2)
    assert torch.equal(k, k2) and torch.equal(v, v2)
