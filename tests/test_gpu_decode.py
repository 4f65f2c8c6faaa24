"""Parity of saw_paged_decode_attn (and the 16-bit comparison path) with the fp64 oracle."""
import numpy as np
import pytest
import torch

import gpu_cases as gc
import parity
from oracle import saw_oracle as O
from paper_2604_19157_amd import synth

pytestmark = pytest.mark.gpu
TOL = 2e-3          # max-abs error relative to the largest reference magnitude


@pytest.fixture(scope="module")
def saw():
    from paper_2604_19157_amd import binding
    binding.lib()
    return binding


def _decode_case(saw, w, num_splits=0, out_dtype=torch.float32, sm_scale=0.0, q_dtype=None, end_to_end=True,
                 max_seq_len=None, order=None):
    """Criterion: both sides attend over the SAME bytes, the ones the oracle's store wrote (uploaded to
    the device cache), so the decode kernel is compared with the oracle independently of the store.
    `max_seq_len`: the host-side bound handed to the call (None: the longest sequence; 0: the call's
    default, the page table's capacity)."""
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    pt = torch.from_numpy(w.page_table).cuda()
    q = synth.gen_q(w)
    if q_dtype is not None:
        q = q.to(q_dtype)
    sl = torch.from_numpy(w.seq_lens).cuda()
    kw = dict(max_seq_len=int(w.seq_lens.max()) if max_seq_len is None else max_seq_len, sm_scale=sm_scale,
              out_dtype=out_dtype, num_splits=num_splits)
    if order is not None:               # the caller's longest-first order (saw_paged_decode_attn_hinted)
        kw["order"] = torch.from_numpy(np.asarray(order, np.int32)).cuda()
    # the output starts as NaN: a row the path never writes fails the comparison
    o = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=out_dtype, device="cuda")
    saw.paged_decode_attn(cache, q.cuda(), pt, sl, out=o, **kw)
    torch.cuda.synchronize()
    o = o.float().cpu().numpy()
    qn = q.float().numpy()
    o_ref = O.paged_decode_attn(ref, qn, w.page_table, w.seq_lens, w.had_block, w.rotate_mask,
                                sm_scale=sm_scale if sm_scale > 0 else None, signs=w.signs, dense=w.dense)
    err = parity.attn_error(o, o_ref)
    msg = f"[{w.name} B={w.batch} Hq={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim} h={w.had_block} mask={w.rotate_mask} splits={num_splits}] err={err:.2e}"
    if end_to_end:
        # HIP store + HIP decode against oracle store + oracle decode.  Not a 2e-3 criterion: a code the
        # boundary rule exempts (an element that sits on a rounding tie) moves one value by a whole
        # quantisation step, so this only guards against gross disagreement of the composed path.
        cache2, _, _, _ = gc.fill_caches(w, saw, with_ref=False)
        o2 = saw.paged_decode_attn(cache2, q.cuda(), pt, sl, **kw).float().cpu().numpy()
        e2 = parity.attn_error(o2, o_ref)
        msg += f" end-to-end err={e2:.2e}"
        assert e2 < 5e-2, msg
    print(msg, flush=True)
    tol = TOL if out_dtype == torch.float32 else TOL + 2.0 ** -8
    assert err < tol, msg
    assert np.isfinite(o).all()
    return o, o_ref


def test_tiny_config(saw):
    _decode_case(saw, synth.make_workload("tiny"))


@pytest.mark.parametrize("splits", [1, 2, 3, 0])
def test_split_kv(saw, splits):
    _decode_case(saw, synth.make_workload("tiny", batch=3, ctx=(130, 700)), num_splits=splits)


@pytest.mark.parametrize("h,mask", [(1, 3), (16, 3), (32, 3), (64, 3), (128, 3), (64, 1), (64, 2), (64, 0)])
def test_block_sizes_and_masks(saw, h, mask):
    _decode_case(saw, synth.make_workload("llama8b", batch=2, ctx=(40, 200), had_block=h, rotate_mask=mask))


@pytest.mark.parametrize("Hq,Hkv,d", [(8, 8, 128), (8, 4, 128), (16, 2, 128), (64, 8, 128),
                                      (4, 4, 64), (8, 4, 64), (8, 2, 64), (16, 2, 64)])
def test_group_sizes_and_head_dims(saw, Hq, Hkv, d):
    w = synth.make_workload("highconc", batch=3, ctx=(20, 150), n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d,
                            had_block=min(64, d))
    _decode_case(saw, w)


def test_ragged_lengths_with_empty_and_single(saw):
    w = synth.make_workload("highconc", batch=7, seq_lens=[0, 1, 15, 16, 17, 64, 333])
    o, _ = _decode_case(saw, w, num_splits=2)
    assert not o[0].any()                                           # empty sequence -> zero row


@pytest.mark.parametrize("B,Hkv", [(70, 8), (129, 4), (300, 2), (65, 8), (130, 8), (162, 8), (191, 8), (383, 4),
                                   (200, 8), (255, 8), (300, 8), (257, 8), (260, 8), (288, 8), (575, 4)])
def test_many_sequences_balanced_item_order(saw, B, Hkv):
    """More (sequence, kv head) items than compute units: the kernel pairs long with short sequences
    (everything resident at once: blocks of four wavefronts per pair from 576 to 1024 items, the first
    four cases, blocks of four over three sequences up to 1536 items, the next four, blocks of two up to
    2048 items, blocks of two over three sequences up to 2304 items, the last four) or, beyond that, takes
    them longest first.  Every sequence is
    compared, so an item served twice or never shows up; lengths include empty sequences and many ties."""
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 330, size=B)
    lens[rng.integers(0, B, size=B // 5)] = 64                      # ties
    lens[:3] = [0, 329, 1]
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv)
    _decode_case(saw, w, num_splits=1, end_to_end=False)
    _decode_case(saw, w, num_splits=0, end_to_end=False)


@pytest.mark.parametrize("lens,kw", [([0, 1, 63, 64, 65, 500], {}), ([2304] * 4 + [0, 7], {}), ([2500] * 30, {}),
                                     ([1000, 1024, 512, 3, 130, 129, 128, 127] * 4, {}),
                                     ([300, 0, 2000], dict(n_q_heads=64)),
                                     ([90, 0, 300, 64, 1], dict(n_q_heads=8, n_kv_heads=4, head_dim=64, had_block=64)),
                                     ([200, 40, 0], dict(dense_seed=3))])
def test_small_batch_blocks_of_eight(saw, lens, kw):
    """Small batches of short contexts: the plan takes one partition and one block of eight wavefronts per
    (sequence, kv head); the wavefronts fold their states in LDS and the call is a single launch."""
    w = synth.make_workload("tiny", batch=len(lens), seq_lens=lens, **kw)
    cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask)
    assert saw.decode_plan(cache, w.batch, max(lens))[0] == 1
    _decode_case(saw, w, end_to_end=False)
    _decode_case(saw, w, end_to_end=False, out_dtype=torch.bfloat16)


def test_batch_beyond_the_ranking_limit(saw):
    """More than 1024 sequences: the in-kernel length ranking is not used (one wavefront per item)."""
    rng = np.random.default_rng(7)
    lens = rng.integers(0, 40, size=1100)
    w = synth.make_workload("highconc", batch=1100, seq_lens=lens, n_q_heads=4, n_kv_heads=2)
    _decode_case(saw, w, end_to_end=False)


def test_long_context_many_splits(saw):
    w = synth.make_workload("longctx1", ctx=9000, n_q_heads=64)
    _decode_case(saw, w, num_splits=0, end_to_end=False)
    _decode_case(saw, w, num_splits=37, end_to_end=False)


@pytest.mark.parametrize("out_dtype", [torch.bfloat16, torch.float16])
def test_output_and_query_dtypes(saw, out_dtype):
    w = synth.make_workload("tiny", batch=2, ctx=75)
    _decode_case(saw, w, out_dtype=out_dtype, q_dtype=torch.float32, sm_scale=0.11)


def test_page_table_permutation_invariance(saw):
    w1 = synth.make_workload("tiny", batch=2, ctx=200)
    w2 = synth.make_workload("tiny", batch=2, ctx=200, shuffle=False)
    o1, _ = _decode_case(saw, w1, end_to_end=False)
    o2, _ = _decode_case(saw, w2, end_to_end=False)
    assert np.array_equal(o1, o2)


def test_large_magnitudes_stay_finite(saw):
    w = synth.make_workload("tiny", batch=1, ctx=100, scales="outlier4x2000")
    _decode_case(saw, w)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("Hq,Hkv,d", [(32, 8, 128), (64, 8, 128), (8, 8, 64), (8, 4, 128)])
def test_kv16_comparison_path(saw, dtype, Hq, Hkv, d):
    w = synth.make_workload("highconc", batch=4, ctx=(1, 400), n_q_heads=Hq, n_kv_heads=Hkv, head_dim=d, dtype=dtype)
    kc = saw.Kv16Cache(w.num_pages, Hkv, d, dtype)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        K, V = synth.gen_kv(w, b, 0, L)
        saw.kv16_store(kc, K.cuda(), V.cuda(), pt, torch.from_numpy(synth.slots_for(b, 0, L)).cuda())
    q = synth.gen_q(w)
    o_ref = O.kv16_paged_decode_attn(kc.k_pages.float().cpu().numpy(), kc.v_pages.float().cpu().numpy(),
                                     q.float().numpy(), w.page_table, w.seq_lens)
    for splits in (2, 1, 0):
        o = torch.full((w.batch, Hq, d), float("nan"), device="cuda")
        saw.kv16_paged_decode_attn(kc, q.cuda(), pt, torch.from_numpy(w.seq_lens).cuda(), num_splits=splits, out=o)
        torch.cuda.synchronize()
        err = parity.attn_error(o.cpu().numpy(), o_ref)
        print(f"[kv16 {dtype} Hq={Hq}/{Hkv} d={d} splits={splits}] err={err:.2e}", flush=True)
        assert err < TOL


@pytest.mark.parametrize("lens", [[0] * 64, [1] * 64, [0] * 40 + [1] * 24, [64] * 63 + [0], [65] * 32 + [63] * 32,
                                  [200] * 2 + [1] * 62, [129] * 33 + [0] * 32, [256] + [0] * 63,
                                  list(range(64)), [128] * 64, [64 * (i % 5) for i in range(64)]])
def test_pair_blocks_of_four_share_boundaries(saw, lens):
    """64 sequences x 8 kv heads = 512 items: blocks of four wavefronts over (long, short) pairs.  The
    lengths put the cuts between the wavefronts' shares everywhere: fewer batches than wavefronts,
    empty sequences, the pair's boundary on a cut, inside a share, and a short sequence that is
    itself shared between wavefronts."""
    w = synth.make_workload("highconc", batch=len(lens), seq_lens=lens)
    _decode_case(saw, w, end_to_end=False)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float16])
@pytest.mark.parametrize("B,Hq,Hkv", [(70, 32, 8), (129, 4, 4), (255, 16, 8)])
def test_kv16_comparison_path_pair_mode(saw, dtype, B, Hq, Hkv):
    """The 16-bit kernel's two-wavefront blocks over (long, short) sequence pairs (one partition, 257..2048
    items): every sequence compared, lengths with empty sequences and ties."""
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 200, size=B)
    lens[rng.integers(0, B, size=B // 5)] = 32
    lens[:4] = [0, 199, 1, 33]
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=Hq, n_kv_heads=Hkv, dtype=dtype)
    kc = saw.Kv16Cache(w.num_pages, Hkv, w.head_dim, dtype)
    pt = torch.from_numpy(w.page_table).cuda()
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        if L:
            K, V = synth.gen_kv(w, b, 0, L)
            saw.kv16_store(kc, K.cuda(), V.cuda(), pt, torch.from_numpy(synth.slots_for(b, 0, L)).cuda())
    q = synth.gen_q(w)
    o_ref = O.kv16_paged_decode_attn(kc.k_pages.float().cpu().numpy(), kc.v_pages.float().cpu().numpy(),
                                     q.float().numpy(), w.page_table, w.seq_lens)
    o = torch.full((w.batch, Hq, w.head_dim), float("nan"), device="cuda")
    saw.kv16_paged_decode_attn(kc, q.cuda(), pt, torch.from_numpy(w.seq_lens).cuda(), num_splits=1, out=o)
    torch.cuda.synchronize()
    err = parity.attn_error(o.cpu().numpy(), o_ref)
    print(f"[kv16 pair {dtype} B={B} Hq={Hq}/{Hkv}] err={err:.2e}", flush=True)
    assert err < TOL
    assert not o[0].any()


def _random_case(seed):
    """A seeded random decode shape: batch sizes that reach every way of handing out work (partitions with
    a merge pass, several wavefronts per item, pair blocks of two and of four, longest-first order), group
    sizes, both head dims, block orders, rotation masks, and lengths with empty sequences, ties and
    multiples of the 64-token batch."""
    rng = np.random.default_rng(1000 + seed)
    d = int(rng.choice([64, 128]))
    Hkv = int(rng.choice([1, 2, 3, 4, 8]))
    G = int(rng.choice([1, 2, 4, 8]))
    items_target = int(rng.choice([3, 40, 300, 600, 900, 1300, 1900, 2500]))
    per_seq = Hkv // 2 if (d == 64 and Hkv % 2 == 0) else Hkv
    B = int(min(1024, max(1, round(items_target / per_seq))))
    top = int(rng.choice([70, 200, 700])) if B <= 40 else int(rng.choice([40, 130]))
    lens = rng.integers(0, top + 1, size=B)
    lens[rng.random(B) < 0.15] = 0
    lens[rng.random(B) < 0.15] = 64 * int(rng.integers(0, max(1, top // 64) + 1))
    if lens.max() == 0:
        lens[0] = 1
    h = int(rng.choice([1, 16, 32, 64] + ([128] if d == 128 else [])))
    mask = int(rng.choice([3, 3, 1, 2]))
    kw = dict(batch=B, seq_lens=lens, n_q_heads=G * Hkv, n_kv_heads=Hkv, head_dim=d, had_block=h, rotate_mask=mask)
    if rng.random() < 0.3:
        kw["sign_seed"] = int(rng.integers(1, 100))
    splits = int(rng.choice([0, 0, 1, 3]))
    return kw, splits


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes(saw, seed):
    kw, splits = _random_case(seed)
    w = synth.make_workload("highconc", **kw)
    _decode_case(saw, w, num_splits=splits, end_to_end=False)


@pytest.mark.parametrize("B,Hkv", [(70, 8), (129, 4), (150, 8), (191, 8), (200, 8), (255, 8), (300, 8), (383, 4)])
def test_caller_supplied_order(saw, B, Hkv):
    """saw_paged_decode_attn_hinted: the longest-first order comes from the caller (a stable host sort of the
    lengths, empty sequences last) and the kernels skip their own ranking: pair blocks of two and of four,
    blocks over three sequences, and the longest-first single-wavefront order."""
    rng = np.random.default_rng(B + 1)
    lens = rng.integers(0, 330, size=B)
    lens[rng.integers(0, B, size=B // 5)] = 64
    lens[:3] = [0, 329, 1]
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv)
    order = np.argsort(-lens, kind="stable")
    o, _ = _decode_case(saw, w, num_splits=1, end_to_end=False, order=order)
    assert not o[lens == 0].any()
    # entries outside [0, B) are clamped: nothing out of bounds, whatever the rows hold
    cache = gc.upload_cache(gc.oracle_fill(w), w, saw)
    bad = torch.from_numpy(np.where(np.arange(B) % 7 == 0, 10 ** 6, order).astype(np.int32)).cuda()
    saw.paged_decode_attn(cache, synth.gen_q(w).cuda(), torch.from_numpy(w.page_table).cuda(),
                          torch.from_numpy(w.seq_lens).cuda(), max_seq_len=int(lens.max()), num_splits=1, order=bad)
    torch.cuda.synchronize()


def test_device_side_order_matches_a_stable_host_sort(saw):
    """saw_decode_order: exactly longest first (after clamping), ties by index, empty sequences last; and the
    hinted decode call accepts it as it is."""
    rng = np.random.default_rng(9)
    for B, top, bound in [(1, 5, 0), (7, 3, 0), (256, 4096, 0), (300, 100, 50), (1024, 70, 0)]:
        lens = rng.integers(0, top + 1, size=B).astype(np.int32)
        lens[rng.random(B) < 0.2] = 0
        got = saw.decode_order(torch.from_numpy(lens).cuda(), bound).cpu().numpy()
        eff = np.minimum(lens, bound) if bound > 0 else lens
        assert np.array_equal(got, np.argsort(-eff, kind="stable"))
    lens = rng.integers(0, 330, size=200)
    w = synth.make_workload("highconc", batch=200, seq_lens=lens)
    order = saw.decode_order(torch.from_numpy(w.seq_lens).cuda()).cpu().numpy()
    _decode_case(saw, w, num_splits=1, end_to_end=False, order=order)


LOOSE_WIDTH = 2048          # page-table columns of a table sized for 32768-token contexts


@pytest.mark.parametrize("bound", [0, 16 * LOOSE_WIDTH - 40])
@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_loose_bound(saw, seed, bound):
    """The same shapes as a serving engine calls them: a page table sized for long contexts and the host
    bound left at its default (the table's capacity) or set loosely - no host read of the lengths.  The
    length classes of the in-kernel ranking then have to come from the lengths themselves."""
    kw, splits = _random_case(seed)
    w = synth.make_workload("highconc", table_width=LOOSE_WIDTH, **kw)
    _decode_case(saw, w, num_splits=splits, end_to_end=False, max_seq_len=bound)


@pytest.mark.parametrize("lens,Hkv", [([0] + [256] * 255, 8), ([0] * 3 + [40] * 200 + [0] * 2 + [7] * 51, 8),
                                      ([0] + [300] * 127, 8), ([0] * 5 + [70] * 120 + [0] * 3, 8),
                                      ([0] * 50 + [300] * 100, 8), ([0, 65] * 90, 8), ([0] * 10 + [33] * 350, 8)])
def test_empty_sequences_under_a_loose_bound(saw, lens, Hkv):
    """Empty sequences that come first in index order, with a bound so loose that the caller's bound alone
    would put them in one length class with everything else: pair blocks of two and of four, blocks over
    three sequences, and the longest-first order."""
    w = synth.make_workload("highconc", batch=len(lens), seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv,
                            table_width=8192)
    o, _ = _decode_case(saw, w, end_to_end=False, max_seq_len=0)
    assert not o[np.asarray(lens) == 0].any()


@pytest.mark.parametrize("lens", [[0] * 260, [1] * 270, [64] * 200 + [0] * 60, [200] * 3 + [1] * 257, [300, 10, 5] * 90,
                                  [129] * 90 + [64] * 90 + [0] * 90, list(range(288)), [128] * 259,
                                  [64 * (i % 4) for i in range(277)], [257] * 130 + [3] * 130, [40, 200, 200] * 88])
def test_blocks_of_two_over_three_sequences(saw, lens):
    """2049..2304 items: a block of two wavefronts takes three sequences laid end to end; the one cut between
    the two shares falls in any of them (a wavefront that holds the head of a shared sequence and an earlier
    sequence after it leaves that record in the block's spare slot), in a gap, or nowhere (empty sequences)."""
    w = synth.make_workload("highconc", batch=len(lens), seq_lens=lens)
    _decode_case(saw, w, end_to_end=False)
    _decode_case(saw, w, end_to_end=False, order=np.argsort(-np.asarray(lens), kind="stable"))


@pytest.mark.parametrize("lens", [[0] * 150, [1] * 150, [64] * 100 + [0] * 50, [200] * 3 + [1] * 147,
                                  [129] * 50 + [64] * 50 + [0] * 50, [300, 10, 5] * 50, list(range(150)),
                                  [128] * 148, [64 * (i % 4) for i in range(191)], [257] * 75 + [3] * 75])
def test_blocks_of_four_over_three_sequences(saw, lens):
    """1152..1536 items: a block of four wavefronts takes three sequences laid end to end.  The lengths
    put the cuts everywhere: sequences that fit inside one share (three ranges for one wavefront), empty
    sequences, batches fewer than wavefronts, a batch size that leaves the last block with one or two
    sequences only."""
    w = synth.make_workload("highconc", batch=len(lens), seq_lens=lens)
    _decode_case(saw, w, end_to_end=False)


@pytest.mark.parametrize("seed", range(200, 230))
def test_schedules_agree(saw, seed):
    """Whatever launch shape the plan picks (blocks of eight wavefronts, partitions with a merge pass, pair
    blocks, longest-first order; ranking in the kernel or the caller's order) is only a schedule: on one cache
    the automatic call, the call forced into three partitions, the call with one partition and the hinted
    call agree to rounding (1e-4 of the largest output), under a tight and under the default bound."""
    kw, _ = _random_case(seed)
    w = synth.make_workload("highconc", **kw)
    cache, _, _, pt = gc.fill_caches(w, saw, with_ref=False)
    sl = torch.from_numpy(w.seq_lens).cuda()
    q = synth.gen_q(w).cuda()
    for bound in (int(w.seq_lens.max()), 0):
        ref = saw.paged_decode_attn(cache, q, pt, sl, max_seq_len=bound, num_splits=3)
        den = float(ref.abs().max()) or 1.0
        outs = {"auto": saw.paged_decode_attn(cache, q, pt, sl, max_seq_len=bound),
                "one partition": saw.paged_decode_attn(cache, q, pt, sl, max_seq_len=bound, num_splits=1)}
        if w.batch <= 1024:
            outs["caller's order"] = saw.paged_decode_attn(cache, q, pt, sl, max_seq_len=bound, order=saw.decode_order(sl, bound))
        for name, o in outs.items():
            assert torch.isfinite(o).all(), name
            assert float((o - ref).abs().max()) / den < 1e-4, (name, bound, kw["batch"])
