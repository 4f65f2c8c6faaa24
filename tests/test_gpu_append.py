"""Parity of saw_append_decode_attn (fused decode step: append the new token, attend over the cache
including it) with the oracle's store followed by the oracle's decode.

The cached tokens are bytes the oracle's store wrote (uploaded); the step's new K/V token is stored by
the HIP path inside the call, so its codes are checked against the oracle's under the store criterion
(bit-exact up to the rounding-boundary rule) and the attention output under the 2e-3 criterion - except
for a sequence whose new token took an exempt boundary code, which moves one value by a whole
quantisation step and is only held to the loose composed bound."""
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


def _new_tokens(w):
    ks, vs = [], []
    for b in range(w.batch):
        L = int(w.seq_lens[b])
        K, V = synth.gen_kv(w, b, L, L + 1)
        ks.append(K)
        vs.append(V)
    return torch.cat(ks).contiguous(), torch.cat(vs).contiguous()


def _case(saw, w, out_dtype=torch.float32, unmapped=(), max_seq_len=None, order=None):
    """`unmapped`: sequences whose new token's page is taken out of the page table (attended, not stored).
    `max_seq_len`: the host-side bound handed to the call (None: the longest sequence; 0: the default)."""
    B = w.batch
    ref = gc.oracle_fill(w)
    cache = gc.upload_cache(ref, w, saw)
    page_table = w.page_table.copy()
    for b in unmapped:
        page_table[b, int(w.seq_lens[b]) >> 4] = -1
    pt = torch.from_numpy(page_table).cuda()
    lens = torch.from_numpy(w.seq_lens).cuda()
    Kn, Vn = _new_tokens(w)
    q = synth.gen_q(w)
    out = torch.full((B, w.n_q_heads, w.head_dim), float("nan"), dtype=out_dtype, device="cuda")
    before = gc.cache_to_numpy(cache, w)
    saw.append_decode_attn(cache, Kn.cuda(), Vn.cuda(), q.cuda(), pt, lens,
                           max_seq_len=int(w.seq_lens.max()) if max_seq_len is None else max_seq_len, out=out,
                           order=None if order is None else torch.from_numpy(np.asarray(order, np.int32)).cuda())
    torch.cuda.synchronize()
    assert torch.equal(lens.cpu(), torch.from_numpy(w.seq_lens))              # lengths are the caller's to advance
    got = gc.cache_to_numpy(cache, w)

    # oracle: store the new tokens (into the mapped table: an unmapped token is still attended to), then decode
    slots = np.stack([np.arange(B, dtype=np.int32), w.seq_lens.astype(np.int32)], 1)
    rec = O.rotate_quant_store(ref, Kn.float().numpy(), Vn.float().numpy(), w.page_table, slots, w.had_block,
                               w.rotate_mask, return_prerounding=True, signs=w.signs, dense=w.dense)
    o_ref = O.paged_decode_attn(ref, q.float().numpy(), w.page_table, w.seq_lens + 1, w.had_block, w.rotate_mask,
                                signs=w.signs, dense=w.dense)

    # (1) the appended token's bytes
    page, slot = rec["page"], rec["slot"]
    exempt = np.zeros(B, bool)
    written = np.zeros(got["k_codes"].shape[:3], bool)
    for b in range(B):
        if b in unmapped:
            continue
        written[page[b], :, slot[b]] = True
        for which in ("k", "v"):
            n = w.n_kv_heads
            res = parity.compare_vectors(got[which + "_codes"][page[b], :, slot[b], :], got[which + "_meta"][page[b], :, slot[b], :],
                                         ref[which + "_codes"][page[b], :, slot[b], :], ref[which + "_meta"][page[b], :, slot[b], :],
                                         rec[which + "_y"][b].reshape(n, -1), rec[which + "_s"][b].reshape(n),
                                         rec[which + "_z"][b].reshape(n))
            parity.assert_store_ok(res)
            exempt[b] |= bool(res["near_boundary_mismatch"] or res["zero_flip_vectors"])
    # nothing else in the cache changed
    for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
        assert np.array_equal(got[k][~written], before[k][~written]), k

    # (2) the attention output
    o = out.float().cpu().numpy()
    assert np.isfinite(o).all()
    tol = TOL if out_dtype == torch.float32 else TOL + 2.0 ** -8
    worst = 0.0
    for b in range(B):
        err = parity.attn_error(o[b:b + 1], o_ref[b:b + 1])
        # (a code the boundary rule exempts moves one value by a whole quantisation step: up to 2/15 of the
        # largest magnitude when the new token is most of what the sequence holds)
        lim = (0.15 if int(w.seq_lens[b]) < 8 else 5e-2) if exempt[b] else tol
        assert err < lim, f"[{w.name} seq {b} len {int(w.seq_lens[b])} exempt={exempt[b]}] err={err:.2e}"
        worst = max(worst, err)
    print(f"[{w.name} B={B} Hq={w.n_q_heads}/{w.n_kv_heads} d={w.head_dim} h={w.had_block} mask={w.rotate_mask}] "
          f"worst err={worst:.2e} exempt sequences={int(exempt.sum())}", flush=True)


def test_small_batch_one_launch(saw):
    """Small batches of short contexts: one block of eight wavefronts per (sequence, kv head), the whole step
    in one launch: lengths that leave wavefronts of a block without a batch, empty sequences, ragged tails."""
    _case(saw, synth.make_workload("tiny"))
    for lens in ([0, 1, 63, 64, 65, 500], [2304] * 4 + [0, 7], [1000, 1024, 512, 3, 130, 129, 128, 127]):
        w = synth.make_workload("tiny", batch=len(lens), seq_lens=lens)
        cache = saw.Cache(w.num_pages, w.n_kv_heads, w.head_dim, w.had_block, w.rotate_mask)
        assert saw.decode_plan(cache, w.batch, max(lens) + 1)[0] == 1
        _case(saw, w)
    _case(saw, synth.make_workload("longctx1", batch=3, seq_lens=[300, 0, 2000], had_block=64))      # G = 8
    _case(saw, synth.make_workload("highconc", batch=5, seq_lens=[90, 0, 300, 64, 1], n_q_heads=8, n_kv_heads=4,
                                   head_dim=64, had_block=64))                                           # head pairs


@pytest.mark.parametrize("B,Hkv", [(70, 8), (129, 4), (150, 8), (191, 8), (200, 8), (300, 8), (260, 8), (288, 8)])
def test_large_ragged_batch_pair_mode(saw, B, Hkv):
    rng = np.random.default_rng(B)
    lens = rng.integers(0, 330, size=B)
    lens[:6] = [0, 329, 1, 16, 15, 64]                       # empty, page boundaries, batch boundary
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv)
    _case(saw, w)


@pytest.mark.parametrize("B,Hkv", [(70, 8), (150, 8), (200, 8), (300, 8)])
def test_caller_supplied_order(saw, B, Hkv):
    """saw_append_decode_attn_hinted: the same step with the longest-first order supplied by the caller."""
    rng = np.random.default_rng(B + 2)
    lens = rng.integers(0, 330, size=B)
    lens[:6] = [0, 329, 1, 16, 15, 64]
    w = synth.make_workload("highconc", batch=B, seq_lens=lens, n_q_heads=4 * Hkv, n_kv_heads=Hkv)
    _case(saw, w, order=np.argsort(-lens, kind="stable"))


@pytest.mark.parametrize("h,mask", [(1, 3), (16, 3), (32, 3), (64, 3), (128, 3), (64, 1), (64, 2)])
def test_block_sizes_and_masks(saw, h, mask):
    _case(saw, synth.make_workload("llama8b", batch=3, seq_lens=[0, 47, 200], had_block=h, rotate_mask=mask))


@pytest.mark.parametrize("Hq,Hkv", [(8, 8), (16, 8), (64, 8)])
def test_group_sizes(saw, Hq, Hkv):
    _case(saw, synth.make_workload("highconc", batch=3, ctx=(20, 150), n_q_heads=Hq, n_kv_heads=Hkv, dtype=torch.float16))


def test_split_kv_and_head_dim_64(saw):
    _case(saw, synth.make_workload("llama8b", batch=2, ctx=2000))                 # several partitions per sequence
    _case(saw, synth.make_workload("highconc", batch=3, ctx=(20, 150), n_q_heads=8, n_kv_heads=4, head_dim=64,
                                   had_block=64))


def test_unmapped_page_is_attended_but_not_stored(saw):
    w = synth.make_workload("tiny", batch=3, seq_lens=[16, 40, 95])
    _case(saw, w, unmapped=(0,))


def test_bf16_output(saw):
    _case(saw, synth.make_workload("tiny", batch=2, ctx=75), out_dtype=torch.bfloat16)


def test_several_partitions_with_lengths_on_partition_boundaries(saw):
    """The append inside the split-KV path: the partition that starts a sequence carries the new token
    and the merge takes exactly the partitions that ran -- also when the cached length is zero, sits
    exactly on a partition boundary, or one past it."""
    longest = 2700                       # (long enough that the plan takes partitions, not one block of eight wavefronts)
    w0 = synth.make_workload("tiny", batch=8, seq_lens=[0, 1, 192, 193, 384, 513, 700, longest])
    cache = saw.Cache(w0.num_pages, w0.n_kv_heads, w0.head_dim, w0.had_block, w0.rotate_mask)
    splits, chunk = saw.decode_plan(cache, w0.batch, longest + 1)
    assert splits > 1
    lens = [0, 1, chunk - 1, chunk, chunk + 1, 2 * chunk, 2 * chunk + 1, longest]
    w = synth.make_workload("tiny", batch=len(lens), seq_lens=lens)
    _case(saw, w)
    _case(saw, synth.make_workload("longctx1", batch=2, seq_lens=[700, 0], had_block=64))     # G = 8


def test_pair_blocks_of_four_with_empty_sequences(saw):
    """512 items: four-wavefront pair blocks; empty sequences still attend to (and store) their new token."""
    lens = [0] * 20 + [1] * 10 + [64] * 10 + [200] * 23 + [129]
    _case(saw, synth.make_workload("highconc", batch=len(lens), seq_lens=lens))


@pytest.mark.parametrize("seed", range(100, 112))
def test_random_shapes(saw, seed):
    """The decode test's seeded random shapes through the append entry point."""
    import test_gpu_decode as TD
    kw, _ = TD._random_case(seed)
    _case(saw, synth.make_workload("highconc", **kw))


@pytest.mark.parametrize("bound", [0, 32000])
@pytest.mark.parametrize("seed", range(100, 112))
def test_random_shapes_loose_bound(saw, seed, bound):
    """The same with a page table sized for 32768-token contexts and the bound at its default or loose."""
    import test_gpu_decode as TD
    kw, _ = TD._random_case(seed)
    _case(saw, synth.make_workload("highconc", table_width=TD.LOOSE_WIDTH, **kw), max_seq_len=bound)


@pytest.mark.parametrize("lens,width", [([0] + [256] * 255, 1024), ([0] + [2048] * 127, 8192),
                                        ([0] * 50 + [300] * 100, 8192), ([0, 65] * 90, 2048),
                                        ([0] * 3 + [40] * 200 + [0] * 2 + [7] * 51, 4096)])
def test_empty_sequence_first_under_a_loose_bound(saw, lens, width):
    """An empty sequence at a low index and a bound so loose that, ranked by the caller's bound, it would
    share a length class with the non-empty ones and rank ahead of them: blocks of two wavefronts (2048
    items), of four over pairs (1024 items) and of four over three sequences.  The ranking keeps empty
    sequences in a class of their own, so the block's first sequence is never the empty one."""
    _case(saw, synth.make_workload("highconc", batch=len(lens), seq_lens=lens, table_width=width), max_seq_len=0)


def test_length_beyond_the_bound_is_not_stored(saw):
    """seq_lens[b] > max_seq_len breaks the caller's promise: nothing is stored for that sequence (a store
    at the clamped position would overwrite a cached token), the other sequences are unaffected, and its
    own output row stays finite (the fused kernel attends over max_seq_len cached tokens plus the new one)."""
    for kw in (dict(), dict(n_q_heads=6, n_kv_heads=3, head_dim=64, had_block=64)):      # fused kernel; store + decode launches
        w = synth.make_workload("tiny", batch=3, seq_lens=[40, 100, 70], **kw)
        ref = gc.oracle_fill(w)
        cache = gc.upload_cache(ref, w, saw)
        before = gc.cache_to_numpy(cache, w)
        Kn, Vn = _new_tokens(w)
        q = synth.gen_q(w)
        bound = 70
        out = saw.append_decode_attn(cache, Kn.cuda(), Vn.cuda(), q.cuda(), torch.from_numpy(w.page_table).cuda(),
                                     torch.from_numpy(w.seq_lens).cuda(), max_seq_len=bound)
        torch.cuda.synchronize()
        got = gc.cache_to_numpy(cache, w)
        # sequence 1 is over the bound: its pages are untouched; the oracle sees it as `bound` cached tokens + the new one
        pages1 = w.page_table[1, :(100 + 16) // 16 + 1]
        for k in ("k_codes", "v_codes", "k_meta", "v_meta"):
            assert np.array_equal(got[k][pages1], before[k][pages1]), k
        lens_ref = np.minimum(w.seq_lens, bound)
        pt_ref = w.page_table.copy()
        slots = np.stack([np.arange(3, dtype=np.int32), lens_ref.astype(np.int32)], 1)
        O.rotate_quant_store(ref, Kn.float().numpy(), Vn.float().numpy(), pt_ref, slots, w.had_block, w.rotate_mask)
        o_ref = O.paged_decode_attn(ref, q.float().numpy(), pt_ref, lens_ref + 1, w.had_block, w.rotate_mask)
        assert torch.isfinite(out).all()
        for b in (0, 2) if kw else (0, 1, 2):          # (the two-launch path attends over the clamped cached range only)
            err = parity.attn_error(out[b:b + 1].cpu().numpy(), o_ref[b:b + 1])
            assert err < 5e-2, (b, err)
