"""Parity of saw_rotate_quant_store / saw_dequant_pages with the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import gpu_cases as gc
import parity
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _run(saw, w, **kw):
    cache, ref, recs, pt = gc.fill_caches(w, saw, **kw)
    got = gc.cache_to_numpy(cache, w)
    res = gc.compare_store(got, ref, recs)
    print(f"[{w.name} h={w.had_block} d={w.head_dim} mask={w.rotate_mask} {w.dtype}] {res}", flush=True)
    parity.assert_store_ok(res)
    assert res["untouched_ok"]
    return cache, ref, got, pt, res


def test_tiny_full_parity(saw):
    """Config 1 in full: every code, scale and zero-point of 4 x 256 tokens x 8 heads."""
    w = synth.make_workload("tiny")
    _, ref, got, _, res = _run(saw, w)
    assert res["vectors"] > 0
    # placement is exact: the byte arrays agree wherever no exemption applies
    frac = (got["k_codes"] != ref["k_codes"]).mean()
    assert frac < 1e-4


@pytest.mark.parametrize("h", [1, 16, 32, 64, 128])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_block_size_sweep_d128(saw, h, dtype):
    w = synth.make_workload("prefill", ctx=700, had_block=h, dtype=dtype)     # several blocks + a ragged tail
    _run(saw, w)


@pytest.mark.parametrize("h", [1, 16, 32, 64])
def test_block_size_sweep_mha_d64(saw, h):
    w = synth.make_workload("prefill_mha", ctx=333, had_block=h)
    _run(saw, w)


@pytest.mark.parametrize("mask", [0, 1, 2, 3])
def test_rotate_mask(saw, mask):
    w = synth.make_workload("llama8b", batch=3, ctx=97, rotate_mask=mask)
    _run(saw, w)


@pytest.mark.parametrize("Hkv", [1, 2, 3, 6])
@pytest.mark.parametrize("h,mask", [(64, 3), (16, 1), (32, 2), (1, 3)])
def test_d64_head_pairs_and_odd_head_counts(saw, Hkv, h, mask):
    """head_dim 64: an even head count takes the two-heads-per-wavefront path, an odd one the
    one-head path; whole pages, ragged ends and shuffled token order (per-token placement)."""
    w = synth.make_workload("prefill_mha", batch=2, seq_lens=[83, 16], n_kv_heads=Hkv, n_q_heads=Hkv,
                            had_block=h, rotate_mask=mask, sign_seed=3 if h == 32 else None)
    _run(saw, w)
    _run(saw, w, order_rng=np.random.default_rng(Hkv))


def test_heavy_tailed_ragged_batch(saw):
    w = synth.make_workload("highconc", batch=9, ctx=(1, 300))
    _run(saw, w, order_rng=np.random.default_rng(5))


def test_small_head_counts_and_single_token(saw):
    for Hkv in (1, 2, 3):
        w = synth.make_workload("tiny", batch=2, seq_lens=[1, 17], n_kv_heads=Hkv, n_q_heads=Hkv)
        _run(saw, w)


def test_degenerate_vectors_and_huge_offsets(saw):
    dev = "cuda"
    Hkv, d = 2, 128
    cache = saw.Cache(4, Hkv, d, 64, 3, device=dev)
    ref = O.new_cache(4, Hkv, 16, d)
    K = torch.zeros((6, Hkv, d), dtype=torch.float16)
    V = torch.zeros_like(K)
    K[1] = 3.25                                  # constant vectors: rotate to one DC coefficient per block
    K[2, 0, :64] = -7.5                          # constant inside one Hadamard block only
    V[3] = -2.0
    V[4, 1] = torch.linspace(1000.0, 1001.0, d).to(torch.float16)   # range far from zero: large |z|
    K[5, :, 5] = 60000.0                         # one huge channel
    pt = np.array([[2, 0]], np.int32)
    sl = synth.slots_for(0, 11, 17)              # straddles a page boundary
    saw.rotate_quant_store(cache, K.to(dev), V.to(dev), torch.from_numpy(pt).to(dev), torch.from_numpy(sl).to(dev))
    rec = O.rotate_quant_store(ref, K.float().numpy(), V.float().numpy(), pt, sl, 64, 3, return_prerounding=True)
    torch.cuda.synchronize()
    got = {k: getattr(cache, k).cpu().numpy() for k in ("k_codes", "v_codes", "k_meta", "v_meta")}
    res = gc.compare_store(got, ref, [rec])
    print(res, flush=True)
    parity.assert_store_ok(res)
    # the all-zero vector: s = 1, z = 0, codes 0
    assert got["k_meta"][2, 0, 11].tolist() == [1.0, 0.0] and not got["k_codes"][2, 0, 11].any()


def test_out_of_range_slots_are_skipped_and_strided_input(saw):
    dev = "cuda"
    Hkv, d = 2, 64
    cache = saw.Cache(3, Hkv, d, 32, 3, device=dev)
    g = torch.Generator().manual_seed(3)
    big = torch.randn((5, Hkv * d + 24), generator=g).to(torch.bfloat16)      # token stride > Hkv*d
    bigv = torch.randn((5, Hkv * d + 24), generator=g).to(torch.bfloat16)
    Kd, Vd = big.to(dev), bigv.to(dev)
    K = Kd[:, :Hkv * d].view(5, Hkv, d)
    V = Vd[:, :Hkv * d].view(5, Hkv, d)
    pt = np.array([[1, 7]], np.int32)                                          # page 7 does not exist
    sl = np.array([[0, 3], [0, 20], [1, 0], [0, -1], [0, 40]], np.int32)       # only the first is valid
    saw.rotate_quant_store(cache, K, V, torch.from_numpy(pt).to(dev), torch.from_numpy(sl).to(dev))
    torch.cuda.synchronize()
    ref = O.new_cache(3, Hkv, 16, d)
    O.rotate_quant_store(ref, big[:1, :Hkv * d].float().numpy().reshape(1, Hkv, d),
                         bigv[:1, :Hkv * d].float().numpy().reshape(1, Hkv, d), pt, sl[:1], 32, 3)
    assert np.array_equal(cache.k_codes.cpu().numpy(), ref["k_codes"])
    assert np.array_equal(cache.v_codes.cpu().numpy(), ref["v_codes"])
    assert np.allclose(cache.k_meta.cpu().numpy(), ref["k_meta"], rtol=1e-6)


@pytest.mark.parametrize("name,kw", [("tiny", dict(batch=2, ctx=90)),
                                     ("prefill_mha", dict(ctx=70, had_block=16)),
                                     ("llama8b", dict(batch=1, ctx=50, rotate_mask=1))])
@pytest.mark.parametrize("unrotate", [False, True])
def test_dequant_pages(saw, name, kw, unrotate):
    w = synth.make_workload(name, **kw)
    got = gc.oracle_fill(w)                               # both sides read the bytes the oracle's store wrote
    cache = gc.upload_cache(got, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        for (p0, p1) in [(0, L), (5, min(L, 37)), (L - 1, L)]:
            k, v = saw.dequant_pages(cache, pt, b, p0, p1, unrotate=unrotate)
            kr, vr = O.dequant_pages(got, w.page_table, b, p0, p1, w.had_block, w.rotate_mask, unrotate=unrotate,
                                     signs=w.signs, dense=w.dense)
            for a, r in ((k, kr), (v, vr)):
                a = a.cpu().numpy().astype(np.float64)
                assert np.abs(a - r).max() <= 2e-6 * np.abs(r).max()
    # with rotation undone the values are the inputs up to the quantisation step
    if unrotate:
        K, V = synth.gen_kv(w, 0, 0, int(w.seq_lens[0]))
        k, v = saw.dequant_pages(cache, pt, 0, 0, int(w.seq_lens[0]), unrotate=True)
        s = got["k_meta"][..., 0].max()
        assert (k.cpu() - K.float()).abs().max() <= 0.51 * s * (w.head_dim ** 0.5)


@pytest.mark.parametrize("n_layers,dense", [(3, False), (35, False), (2, True)])
def test_store_layers_in_one_launch(saw, n_layers, dense):
    """saw_rotate_quant_store_layers: every layer's cache holds exactly the bytes a per-layer call writes, and
    (first and last layer) the oracle's codes under the store criterion.  35 layers go out as two launches.
    With a learned rotation every layer has its own matrix."""
    w = synth.make_workload("tiny", batch=2, seq_lens=[37, 16], had_block=64)
    pt = torch.from_numpy(w.page_table).cuda()
    Rs = [synth.random_orthogonal(128, 50 + l) if dense else None for l in range(n_layers)]
    mk = lambda l: saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask, dense=Rs[l])
    multi = [mk(l) for l in range(n_layers)]
    single = [mk(l) for l in range(n_layers)]
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        sl = torch.from_numpy(synth.slots_for(b, 0, L)).cuda()
        KV = [synth.gen_kv(w, b + 100 * l, 0, L, device="cuda") for l in range(n_layers)]
        saw.rotate_quant_store_layers(multi, [k for k, _ in KV], [v for _, v in KV], pt, sl)
        for l in range(n_layers):
            saw.rotate_quant_store(single[l], KV[l][0], KV[l][1], pt, sl)
    torch.cuda.synchronize()
    for l in range(n_layers):
        for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
            assert torch.equal(getattr(multi[l], k), getattr(single[l], k)), (l, k)
    for l in (0, n_layers - 1):
        ref = O.new_cache(w.num_pages, w.n_kv_heads, w.page_size, w.head_dim)
        recs = []
        for b in range(w.batch):
            L = int(w.seq_lens[b])
            K, V = synth.gen_kv(w, b + 100 * l, 0, L, device="cuda")
            recs.append(O.rotate_quant_store(ref, K.float().cpu().numpy(), V.float().cpu().numpy(), w.page_table,
                                             synth.slots_for(b, 0, L), w.had_block, w.rotate_mask,
                                             return_prerounding=True, dense=Rs[l]))
        res = gc.compare_store(gc.cache_to_numpy(multi[l], w), ref, recs)
        parity.assert_store_ok(res)
        assert res["untouched_ok"]


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
def test_plain_store_on_the_vector_alu_matches_the_oracle(saw, dtype):
    """The lean plain INT4 store that bench.py uses as a comparator: no rotation whatever the descriptor says,
    codes under the store criterion, ragged token counts, tokens in arbitrary order."""
    w = synth.make_workload("tiny", batch=3, seq_lens=[37, 16, 100], had_block=64, dtype=dtype)
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask)
    ref = O.new_cache(w.num_pages, w.n_kv_heads, w.page_size, w.head_dim)
    pt = torch.from_numpy(w.page_table).cuda()
    recs = []
    rng = np.random.default_rng(3)
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        K, V = synth.gen_kv(w, b, 0, L)
        sl = synth.slots_for(b, 0, L)
        perm = rng.permutation(L)
        K, V, sl = K[perm].contiguous(), V[perm].contiguous(), sl[perm]
        saw.plain_quant_store_valu(cache, K.cuda(), V.cuda(), pt, torch.from_numpy(sl).cuda())
        recs.append(O.rotate_quant_store(ref, K.float().numpy(), V.float().numpy(), w.page_table, sl, 1, 0,
                                         return_prerounding=True))
    torch.cuda.synchronize()
    res = gc.compare_store(gc.cache_to_numpy(cache, w), ref, recs)
    parity.assert_store_ok(res)
    assert res["untouched_ok"]


def test_read_probe_reads_every_listed_tile_once(saw):
    """The read-only probe behind bench.py's streaming ceiling: the XOR of the words it hands back equals the
    XOR of every dword of the listed pages' K/V code tiles and (scale, zero) pairs (a multiple of four pages:
    nothing is read twice), whatever the page order."""
    w = synth.make_workload("tiny", batch=2, ctx=200)
    cache, _, _, _ = gc.fill_caches(w, saw, with_ref=False)
    pages = np.concatenate([w.page_table[b, :12] for b in range(2)]).astype(np.int32)      # 24 pages
    sink = torch.zeros(2048, dtype=torch.int32, device="cuda")
    n = saw.read_probe(cache, torch.from_numpy(pages).cuda(), sink)
    torch.cuda.synchronize()
    assert n == 24 * w.n_kv_heads * 2304
    want = 0
    for t in (cache.k_codes, cache.v_codes, cache.k_meta, cache.v_meta):
        a = t.cpu().numpy()[pages].reshape(-1).view(np.uint32)
        want ^= int(np.bitwise_xor.reduce(a))
    got = int(np.bitwise_xor.reduce(sink.cpu().numpy().view(np.uint32)))
    assert got == want
